"""The seeded generators: determinism, the tensor code against Python ints, shape."""
import numpy as np
import torch

from paper_2311_14898_amd import inputs


def test_mix64_matches_python_ints():
    xs = [0, 1, 2, 12345678901234567, (1 << 63) + 5, (1 << 64) - 1]
    t = torch.tensor([inputs._s64(x) for x in xs], dtype=torch.int64)
    got = inputs.mix64(t).tolist()
    for x, g in zip(xs, got):
        assert (g & ((1 << 64) - 1)) == inputs.mix64_py(x)


def test_rmat_samples_match_python_ints():
    scale = 14
    u, v = inputs._rmat_samples(1, 1000, 64, scale, "cpu")
    for k in range(64):
        pu, pv = inputs.rmat_sample_py(1, 1000 + k, scale)
        assert (int(u[k]), int(v[k])) == (pu, pv)


def test_rmat_edges_deterministic_and_valid():
    V, E = 10_000, 100_000
    s1, d1 = inputs.rmat_edges(V, E, seed=1)
    s2, d2 = inputs.rmat_edges(V, E, seed=1, batch=1 << 14)   # batching must not change the stream
    assert torch.equal(s1, s2) and torch.equal(d1, d2)
    assert s1.numel() == E and s1.dtype == torch.int32
    assert int(s1.max()) < V and int(d1.max()) < V and int(s1.min()) >= 0
    assert not bool((s1 == d1).any())
    s3, _ = inputs.rmat_edges(V, E, seed=2)
    assert not torch.equal(s1, s3)


def test_rmat_is_power_law_shaped():
    V, E = 10_000, 100_000
    s, d = inputs.rmat_edges(V, E, seed=1)
    deg = np.bincount(d.numpy(), minlength=V)
    top = np.sort(deg)[::-1]
    # heavy head: the top 1% of destinations hold far more than 1% of the edges
    assert top[: V // 100].sum() > 0.10 * E
    assert deg.max() > 20 * deg.mean()


def test_labels_and_weights():
    y = inputs.labels(1000, 8)
    assert y.min() >= 0 and y.max() < 8
    y2 = inputs.labels(100_000, 172, labelled_one_in=100)
    frac = float((y2 >= 0).float().mean())
    assert 0.005 < frac < 0.02
    Ws = inputs.glorot_weights([64, 32, 8])
    assert [tuple(w.shape) for w in Ws] == [(64, 32), (32, 8)]
    assert float(Ws[0].abs().max()) <= (6.0 / 96) ** 0.5 + 1e-6
    assert torch.equal(Ws[0], inputs.glorot_weights([64, 32, 8])[0])
