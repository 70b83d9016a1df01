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


def _loss_qkv(x, w, bias, flags, H, cq, ck, cv):
    q, k, v = orc.project_qkv(x, w, bias, flags, H)
    return float((q * cq).sum() + (k * ck).sum() + (v * cv).sum())


def test_qkv_backward_vs_finite_differences_and_autograd():
    """dx, dw, dbias of the QKV projection: central differences of the oracle's own forward
    (float64, so 1e-7 relative is reachable), then torch.autograd through the library's linear
    layer with the pad rows masked the way the forward masks them."""
    x, w, bias, flags, H, m, E = _case(7, B=2, N=6, H=2, m=3, E=5)
    rng = np.random.default_rng(8)
    cq, ck, cv = (rng.standard_normal((2, H, 6, m)) for _ in range(3))     # dL/dq, dL/dk, dL/dv
    dx, dw, db = orc.project_qkv_backward(x, w, flags, cq, ck, cv, H)
    eps = 1e-6
    for arr, grad in ((x, dx), (w, dw), (bias, db)):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            keep = arr[idx]
            arr[idx] = keep + eps
            up = _loss_qkv(x, w, bias, flags, H, cq, ck, cv)
            arr[idx] = keep - eps
            dn = _loss_qkv(x, w, bias, flags, H, cq, ck, cv)
            arr[idx] = keep
            assert abs((up - dn) / (2 * eps) - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx])), idx
    assert np.all(dx[flags == P] == 0)
    tx, tw, tb = (torch.from_numpy(a.copy()).requires_grad_() for a in (x, w, bias))
    y = torch.nn.functional.linear(tx, tw, tb) * torch.from_numpy((flags != P)[:, :, None].astype(np.float64))
    g = np.concatenate([t.transpose(0, 2, 1, 3).reshape(2, 6, H * m) for t in (cq, ck, cv)], axis=-1)
    (y * torch.from_numpy(g)).sum().backward()
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-12)
    assert np.allclose(dw, tw.grad.numpy(), atol=1e-12)
    assert np.allclose(db, tb.grad.numpy(), atol=1e-12)


def test_out_backward_vs_autograd_and_loops():
    rng = np.random.default_rng(11)
    B, H, N, m, E = 2, 3, 5, 4, 7
    o = rng.standard_normal((B, H, N, m))
    w_o = rng.standard_normal((E, H * m))
    b_o = rng.standard_normal(E)
    flags = rng.choice([L, G, P], size=(B, N)).astype(np.uint8)
    flags[0, 2] = P
    dy = rng.standard_normal((B, N, E))
    d_o, dw, db = orc.project_out_backward(o, w_o, flags, dy)
    to, tw, tb = (torch.from_numpy(a.copy()).requires_grad_() for a in (o, w_o, b_o))
    cat = to.permute(0, 2, 1, 3).reshape(B, N, H * m)
    y = torch.nn.functional.linear(cat, tw, tb) * torch.from_numpy((flags != P)[:, :, None].astype(np.float64))
    (y * torch.from_numpy(dy)).sum().backward()
    assert np.allclose(d_o, to.grad.numpy(), atol=1e-12)
    assert np.allclose(dw, tw.grad.numpy(), atol=1e-12)
    assert np.allclose(db, tb.grad.numpy(), atol=1e-12)
    # and written out: d_o[b,i,k,d] = sum_e dy[b,k,e] w_o[e, i*m+d];  dw[e,j] = sum_{b,k} dy[b,k,e] o_cat[b,k,j]
    for b in range(B):
        for k in range(N):
            for i in range(H):
                for d in range(m):
                    want = 0.0 if flags[b, k] == P else sum(dy[b, k, e] * w_o[e, i * m + d] for e in range(E))
                    assert abs(d_o[b, i, k, d] - want) <= 1e-12
    e, j = 3, 2 * m + 1
    want = sum(dy[b, k, e] * o[b, 2, k, 1] for b in range(B) for k in range(N) if flags[b, k] != P)
    assert abs(dw[e, j] - want) <= 1e-12
    assert np.allclose(db, sum(dy[b, k] for b in range(B) for k in range(N) if flags[b, k] != P), atol=1e-12)
