"""Host-side checks that need no GPU: the library loads, exports what the header declares,
and its byte accounting matches the paper's Table 1."""
import os
import re

import pytest

from paper_2311_14898_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "hongtu.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(ht_[a-z0-9_]+)\s*\(", hdr))
    assert {"ht_partition", "ht_layer_fwd", "ht_layer_bwd", "ht_epoch"} <= names
    lib = B.load()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in hongtu.h but not exported"
    assert names == set(B.EXPORTS), "binding and header list different entry points"


def test_memory_model_matches_table1():
    with open(os.path.join(ROOT, "tests", "golden", "table1_memory.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    GB = float(1 << 30)
    for name, V, d0, d1, d2, d3, vtx, intr in rows:
        vb, ib = B.ht_memory_model(int(V), [int(d0), int(d1), int(d2), int(d3)])
        assert abs(vb / GB - float(vtx)) < 0.35, (name, vb / GB)
        assert abs(ib / GB - float(intr)) < 0.1, (name, ib / GB)


def test_chunk_rows_model():
    # (1 + alpha) |V| / (m n), Sec. 4.3
    assert B.ht_chunk_rows_model(1000, 10, 2.5) == pytest.approx(350.0)
    assert B.ht_strerror_text(B.HT_ESHAPE) != ""


def test_comm_cost_model():
    # Eq. 4 with the Sec. 5.1 example's printed counts (11 rows after sharing between GPUs, 8 after reuse)
    # and an arbitrary 14 rows without any dedup
    c = B.ht_comm_cost_model(14, 11, 8, 400, 25e9, 200e9, 1500e9)
    assert c == pytest.approx(8 * 400 / 25e9 + 3 * 400 / 200e9 + 3 * 400 / 1500e9, rel=1e-12)
    # one GPU: the inter-GPU term is void, its throughput is not looked at
    assert B.ht_comm_cost_model(14, 14, 8, 400, 25e9, 0.0, 1500e9) == pytest.approx(8 * 400 / 25e9 + 6 * 400 / 1500e9)
    assert B.ht_comm_cost_model(14, 11, 12, 400, 25e9, 200e9, 1500e9) == -1.0      # v_ru > v_p2p
    assert B.ht_comm_cost_model(14, 11, 8, 400, 0.0, 200e9, 1500e9) == -1.0        # a needed throughput is missing


C_CLIENT = r"""
#include <stdio.h>
#include <string.h>
#include "hongtu.h"
int main(void) {
  /* a plain C99 caller: the header alone, no C++ and no torch */
  int32_t dims[4] = {128, 256, 256, 172};
  double vb = 0.0, ib = 0.0;
  if (ht_memory_model(111000000LL, 3, dims, &vb, &ib) != HT_OK) return 1;
  printf("%.0f %.0f\n", vb, ib);
  printf("%.6f\n", ht_chunk_rows_model(1000, 10, 2.5));
  printf("%.9e\n", ht_comm_cost_model(19, 11, 8, 400, 25e9, 200e9, 1500e9));
  if (strlen(ht_strerror(HT_ENOMEM)) == 0 || strlen(ht_strerror(12345)) == 0) return 2;
  /* argument errors come back as codes, nothing is dereferenced */
  if (ht_ctx_set_hbm_budget(NULL, 1) != HT_EINVAL) return 3;
  if (ht_graph_destroy(NULL) == 12345) return 4;
  if (ht_ctx_graph_launches(NULL) != -1) return 5;
  ht_plan_opts p;
  memset(&p, 0, sizeof p);
  p.stats_detail = HT_STATS_AGG_FWD;
  printf("%d %d\n", (int)sizeof(ht_tensor), (int)sizeof p);
  return 0;
}
"""


def test_a_c99_program_links_against_the_library(tmp_path):
    import ctypes as C
    import subprocess
    B.load()
    libdir = os.path.join(ROOT, "paper_2311_14898_amd")
    src = tmp_path / "client.c"
    src.write_text(C_CLIENT)
    exe = tmp_path / "client"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-lhongtu", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    vb, ib = B.ht_memory_model(111_000_000, [128, 256, 256, 172])
    assert float(out[0]) == vb and float(out[1]) == ib
    assert float(out[2]) == pytest.approx(350.0)
    assert float(out[3]) == pytest.approx(8 * 400 / 25e9 + (19 - 11) * 400 / 200e9 + (11 - 8) * 400 / 1500e9, rel=1e-9)
    # the binding's ctypes mirrors have the C compiler's sizes
    assert int(out[4]) == C.sizeof(B.ht_tensor) and int(out[5]) == C.sizeof(B.ht_plan_opts)


def test_no_fallback_when_the_library_is_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libhongtu.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.load()
    with pytest.raises(RuntimeError):
        B.ht_memory_model(10, [4, 4])


def test_product_package_and_oracle_do_not_import_each_other():
    pkg = os.path.join(ROOT, "paper_2311_14898_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
                assert "gcn_oracle" not in text and "orc_" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".cpp", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "binding" not in text and "hongtu.h" not in text and "libhongtu" not in text, f


def test_without_a_gpu_a_context_is_refused():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.HongtuError):
        B.ht_ctx_create(0)
