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
