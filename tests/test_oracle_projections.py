"""Pins for the oracle's projections (CPU only): the head equation's W^i X_k written as loops,
the library's linear layer in float64, and identity weights."""
import numpy as np
import torch

from oracle import mate_oracle as orc
from paper_2109_04312_amd import synth

L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD


def _case(seed, B=2, N=9, H=3, m=4, E=10):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, N, E))
    w = rng.standard_normal((3 * H * m, E))
    bias = rng.standard_normal(3 * H * m)
    flags = rng.choice([L, G, P], size=(B, N)).astype(np.uint8)
    return x, w, bias, flags, H, m, E


def test_qkv_per_head_loops():
    x, w, bias, flags, H, m, E = _case(0)
    q, k, v = orc.project_qkv(x, w, bias, flags, H)
    for t, got in enumerate((q, k, v)):
        for b in range(x.shape[0]):
            for i in range(H):
                Wi = w[(t * H + i) * m:(t * H + i + 1) * m]          # W^i of the head equation, [m, E]
                bi = bias[(t * H + i) * m:(t * H + i + 1) * m]
                for kk in range(x.shape[1]):
                    want = [sum(Wi[d, e] * x[b, kk, e] for e in range(E)) + bi[d] for d in range(m)]
                    if flags[b, kk] == P:
                        want = [0.0] * m
                    assert np.allclose(got[b, i, kk], want, atol=1e-12)


def test_projections_vs_library_linear_and_identity():
    x, w, bias, flags, H, m, E = _case(1, N=17)
    q, k, v = orc.project_qkv(x, w, None, flags, H)
    y = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w)).numpy()
    y = y * (flags != P)[:, :, None]
    for t, got in enumerate((q, k, v)):
        for i in range(H):
            assert np.allclose(got[:, i], y[:, :, (t * H + i) * m:(t * H + i + 1) * m], atol=1e-12)
    # identity weights: head i of Q is the i-th slice of x
    E2 = H * m
    x2 = np.random.default_rng(2).standard_normal((2, 5, E2))
    w_id = np.concatenate([np.eye(E2)] * 3)
    fl = np.full((2, 5), L, np.uint8)
    q, k, v = orc.project_qkv(x2, w_id, None, fl, H)
    for got in (q, k, v):
        assert np.array_equal(got.transpose(0, 2, 1, 3).reshape(2, 5, E2), x2)
    # output projection: library linear over the concatenated heads; identity gives them back
    o = np.random.default_rng(3).standard_normal((2, H, 5, m))
    w_o = np.random.default_rng(4).standard_normal((7, E2))
    b_o = np.random.default_rng(5).standard_normal(7)
    fl[1, 3] = P
    cat = np.concatenate([o[:, i] for i in range(H)], axis=-1)
    want = torch.nn.functional.linear(torch.from_numpy(cat), torch.from_numpy(w_o), torch.from_numpy(b_o)).numpy()
    want[1, 3] = 0
    assert np.allclose(orc.project_out(o, w_o, b_o, fl), want, atol=1e-12)
    assert np.array_equal(orc.project_out(o, np.eye(E2), None, np.full((2, 5), G, np.uint8)), cat)
