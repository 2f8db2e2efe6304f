"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This module holds no arithmetic of the training method: it only draws random
graphs, features, labels and initial weights.  Both sides consume the same
bytes.  The graphs stand in for the paper's evaluation datasets (Table 3 of
the paper): only their vertex/edge/feature/class counts and their power-law
shape are taken, nothing of their content.

Topology is R-MAT (a=0.57, b=c=0.19, d=0.05) drawn with an integer-only,
counter-based generator, so the same (seed, V, E) gives bit-identical edges on
any device torch runs on.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

# 32-bit quadrant thresholds for (a, a+b, a+b+c) = (0.57, 0.76, 0.95).
RMAT_T_A = int(0.57 * (1 << 32))
RMAT_T_AB = int(0.76 * (1 << 32))
RMAT_T_ABC = int(0.95 * (1 << 32))


def _s64(x: int) -> int:
    """Two's-complement view of a 64-bit constant, as torch int64 needs it."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on int64 lanes (wrap-around arithmetic)."""
    z = x
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def mix64_py(x: int) -> int:
    """The same function on a Python int; used to cross-check the tensor code."""
    z = x & _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def rmat_scale(V: int) -> int:
    return max(1, math.ceil(math.log2(V))) if V > 1 else 1


def _rmat_samples(seed: int, i0: int, count: int, scale: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """Endpoints of samples i0 .. i0+count-1 (before rejection)."""
    idx = torch.arange(i0, i0 + count, dtype=torch.int64, device=device)
    base = idx * 64 + _s64(seed * _GOLDEN)
    u = torch.zeros(count, dtype=torch.int64, device=device)
    v = torch.zeros(count, dtype=torch.int64, device=device)
    for k in range(scale):
        if k % 2 == 0:
            z = mix64(base + (k // 2))
            r = _lsr(z, 32)
        else:
            r = z & 0xFFFFFFFF
        ub = (r >= RMAT_T_AB).to(torch.int64)
        vb = (((r >= RMAT_T_A) & (r < RMAT_T_AB)) | (r >= RMAT_T_ABC)).to(torch.int64)
        sh = scale - 1 - k
        u |= ub << sh
        v |= vb << sh
    return u, v


def rmat_sample_py(seed: int, i: int, scale: int) -> Tuple[int, int]:
    """One sample with Python ints (slow; for tests of the tensor code)."""
    base = (i * 64 + seed * _GOLDEN) & _MASK64
    u = v = 0
    z = 0
    for k in range(scale):
        if k % 2 == 0:
            z = mix64_py((base + k // 2) & _MASK64)
            r = z >> 32
        else:
            r = z & 0xFFFFFFFF
        ub = 1 if r >= RMAT_T_AB else 0
        vb = 1 if ((RMAT_T_A <= r < RMAT_T_AB) or r >= RMAT_T_ABC) else 0
        u |= ub << (scale - 1 - k)
        v |= vb << (scale - 1 - k)
    return u, v


def rmat_edges(V: int, E: int, seed: int = 1, device="cpu", batch: int = 1 << 24) -> Tuple[torch.Tensor, torch.Tensor]:
    """First E accepted R-MAT samples, in sample-index order.

    A sample is rejected when an endpoint is >= V or when it is a self-loop.
    Duplicate edges are kept.  Returns (src, dst) as int32 tensors of length E.
    """
    scale = rmat_scale(V)
    srcs: List[torch.Tensor] = []
    dsts: List[torch.Tensor] = []
    have = 0
    i0 = 0
    while have < E:
        need = E - have
        count = min(batch, max(1024, int(need * 1.25) + 1024))
        u, v = _rmat_samples(seed, i0, count, scale, device)
        ok = (u < V) & (v < V) & (u != v)
        u = u[ok]
        v = v[ok]
        if u.numel() > need:
            u = u[:need]
            v = v[:need]
        srcs.append(u.to(torch.int32))
        dsts.append(v.to(torch.int32))
        have += u.numel()
        i0 += count
    return torch.cat(srcs), torch.cat(dsts)


def permute_ids(src: torch.Tensor, dst: torch.Tensor, V: int, seed: int = 7) -> Tuple[torch.Tensor, torch.Tensor]:
    """The same graph with its vertices relabelled by a seeded random permutation (R-MAT puts the hubs at the
    low ids; real datasets do not order their vertices that way).  Used for a sensitivity row only."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    perm = torch.randperm(V, generator=g).to(torch.int32).to(src.device)
    return perm[src.long()], perm[dst.long()]


def features(V: int, d: int, seed: int = 2) -> torch.Tensor:
    """N(0,1) fp32 features [V, d], generated on the CPU."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(V, d, generator=g, dtype=torch.float32)


def labels(V: int, C: int, seed: int = 3, labelled_one_in: int = 1) -> torch.Tensor:
    """Uniform class labels in [0, C); -1 marks an unlabelled vertex.

    With labelled_one_in = k > 1, vertex v keeps its label only when a seeded
    hash of v is divisible by k (about 1/k of the vertices).
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    y = torch.randint(0, C, (V,), generator=g, dtype=torch.int64).to(torch.int32)
    if labelled_one_in > 1:
        h = mix64(torch.arange(V, dtype=torch.int64) + _s64(seed * _GOLDEN))
        keep = (_lsr(h, 33) % labelled_one_in) == 0
        y = torch.where(keep, y, torch.full_like(y, -1))
    return y


def glorot_weights(dims: List[int], seed: int = 4) -> List[torch.Tensor]:
    """Glorot-uniform W^l of shape [dims[l], dims[l+1]], fp32, on the CPU."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    out = []
    for l in range(len(dims) - 1):
        b = math.sqrt(6.0 / (dims[l] + dims[l + 1]))
        w = (torch.rand(dims[l], dims[l + 1], generator=g, dtype=torch.float32) * 2.0 - 1.0) * b
        out.append(w.contiguous())
    return out


def attention_vectors(dims: List[int], seed: int = 5):
    """Per layer the two halves of the attention vector (destination half, source half), each
    [dims[l+1]], uniform in +-sqrt(6 / (2 dims[l+1] + 1)), fp32, on the CPU."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    a_dst, a_src = [], []
    for l in range(len(dims) - 1):
        b = math.sqrt(6.0 / (2 * dims[l + 1] + 1))
        a_dst.append(((torch.rand(dims[l + 1], generator=g, dtype=torch.float32) * 2.0 - 1.0) * b).contiguous())
        a_src.append(((torch.rand(dims[l + 1], generator=g, dtype=torch.float32) * 2.0 - 1.0) * b).contiguous())
    return a_dst, a_src


@dataclass
class Workload:
    """One configuration: graph shape, layer widths, chunk count, residency."""
    name: str
    V: int
    E: int
    dims: List[int]
    n_chunks: int
    residency: str = "hbm"          # "hbm" | "host" (h^l, grad h^l in pinned host memory) | "host_all" (a^l too)
    labelled_one_in: int = 1
    graph_seed: int = 1
    lr: float = 0.01
    note: str = ""

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1

    def scaled(self, s: float) -> "Workload":
        """Same average degree, widths and chunk count at s times the vertices."""
        if s >= 1.0:
            return self
        return Workload(f"{self.name}@s={s:g}", max(2, int(self.V * s)), max(1, int(self.E * s)),
                        list(self.dims), self.n_chunks, self.residency, self.labelled_one_in,
                        self.graph_seed, self.lr, f"scaled by {s:g}")


WORKLOADS = {
    "cfg1": Workload("cfg1", 10_000, 100_000, [64, 32, 8], 4, "hbm"),
    "cfg2": Workload("cfg2", 232_965, 114_600_000, [602, 256, 41], 8, "hbm"),
    "cfg3": Workload("cfg3", 2_450_000, 61_900_000, [100, 256, 256, 47], 16, "host"),
    "cfg4": Workload("cfg4", 111_000_000, 1_600_000_000, [128, 256, 256, 172], 64, "host_all", labelled_one_in=100),
    "cfg5": Workload("cfg5", 65_600_000, 3_600_000_000, [256, 256, 256, 64], 128, "host_all"),
}


def make_inputs(w: Workload, device="cpu"):
    """(src, dst, X, y, Ws) for a workload; X, y, Ws on the CPU, edges on `device`."""
    src, dst = rmat_edges(w.V, w.E, w.graph_seed, device=device)
    X = features(w.V, w.dims[0])
    y = labels(w.V, w.dims[-1], labelled_one_in=w.labelled_one_in)
    Ws = glorot_weights(w.dims)
    return src, dst, X, y, Ws
