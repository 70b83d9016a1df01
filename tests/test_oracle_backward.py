"""Pins for the oracle's backward pass and segment tables (CPU only)."""
import math

import numpy as np
import pytest
import torch

from oracle import mate_oracle as orc
from paper_2109_04312_amd import synth

L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD
ROW, COL = synth.HEAD_ROW, synth.HEAD_COL


def _problem(seed, N=40, D=6, H=2, **kw):
    rng = np.random.default_rng(seed)
    st = synth.random_structure(rng, 1, N, **kw)
    q, k, v, do = (rng.standard_normal((1, H, N, D)) for _ in range(4))
    hk = np.array([ROW, COL] * (H // 2), np.uint8)
    return rng, st, q, k, v, do, hk


@pytest.mark.parametrize("seed", range(3))
def test_backward_vs_central_finite_differences(seed):
    rng, st, q, k, v, do, hk = _problem(seed, scatter=seed == 1)
    sc = 0.6
    args = (st.row_ids, st.col_ids, st.flags, hk, sc)
    dq, dk, dv = orc.attn_backward(q, k, v, do, *args)
    nonpad = (st.flags != P)[:, None, :, None]

    def loss(q_, k_, v_):
        o, _ = orc.attn_forward(q_, k_, v_, *args)
        return float((o * do * nonpad).sum())

    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(25):
            idx = tuple(int(rng.integers(0, s)) for s in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            tri = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            trm = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            fd = (loss(*tri) - loss(*trm)) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(fd)), (name, idx, fd, g[idx])


@pytest.mark.parametrize("case", ["all_global", "one_row", "one_col"])
def test_backward_dense_cases_vs_library_autograd(case):
    rng = np.random.default_rng(17)
    N, D, H = 36, 8, 2
    flags = np.full(N, L, np.uint8)
    flags[-5:] = P
    flags[:3] = G
    row = rng.integers(0, 4, N).astype(np.int32)
    col = rng.integers(0, 4, N).astype(np.int32)
    if case == "all_global":
        flags[flags == L] = G
    elif case == "one_row":
        row[:] = 2
    else:
        col[:] = 5
    q, k, v, do = (rng.standard_normal((1, H, N, D)) for _ in range(4))
    hk = np.array([ROW, COL], np.uint8)
    sc = 1 / math.sqrt(D)
    dq, dk, dv = orc.attn_backward(q, k, v, do, row[None], col[None], flags[None], hk, sc)
    nonpad = flags != P
    heads = {"all_global": [0, 1], "one_row": [0], "one_col": [1]}[case]
    for h in heads:
        tq, tk, tv = (torch.tensor(x[0, h][nonpad], dtype=torch.float64, requires_grad=True)
                      for x in (q, k, v))
        o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], scale=sc)[0]
        (o * torch.tensor(do[0, h][nonpad])).sum().backward()
        for mine, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
            np.testing.assert_allclose(mine[0, h][nonpad], ref.numpy(), rtol=0, atol=1e-12)
            assert np.all(mine[0, h][~nonpad] == 0)


def test_backward_closed_forms_and_pad_isolation():
    rng, st, q, k, v, do, hk = _problem(4, N=64, H=4, scatter=True)
    sc = 0.35
    args = (st.row_ids, st.col_ids, st.flags, hk, sc)
    dq, dk, dv = orc.attn_backward(q, k, v, do, *args)
    nonpad = st.flags[0] != P
    # columns of P^T dO: sum_j dV_j = sum over non-pad k of dO_k (rows of P sum to one)
    np.testing.assert_allclose(dv.sum(axis=2), (do[:, :, nonpad]).sum(axis=2), atol=1e-11)
    # softmax Jacobian has zero row sums: K = const vector c  ->  dQ = scale * (sum_j dS) c = 0
    kc = np.broadcast_to(rng.standard_normal((1, 4, 1, q.shape[-1])), q.shape).copy()
    dq_c, _, _ = orc.attn_backward(q, kc, v, do, *args)
    np.testing.assert_allclose(dq_c, 0, atol=1e-12)
    # pads: zero gradient into pad rows, and dO / inputs at pad rows change nothing
    for g in (dq, dk, dv):
        assert np.all(g[:, :, ~nonpad] == 0)
    do2, q2, k2, v2 = do.copy(), q.copy(), k.copy(), v.copy()
    for t in (do2, q2, k2, v2):
        t[:, :, ~nonpad] = 1e5
    for a, b_ in zip(orc.attn_backward(q2, k2, v2, do2, *args), (dq, dk, dv)):
        np.testing.assert_array_equal(a, b_)


def test_backward_block_structure():
    # A table token's K/V gradient comes only from queries that can see it; with no globals
    # and dO non-zero only inside one row, a row head's gradients vanish outside that row.
    rng = np.random.default_rng(8)
    N, D = 48, 4
    row, col, flags = synth.flatten_table(N, 0, 4, 3, rng.integers(1, 4, 12))
    q, k, v, do = (rng.standard_normal((1, 1, N, D)) for _ in range(4))
    inside = (flags == L) & (row == 2)
    do[:, :, ~inside] = 0
    dq, dk, dv = orc.attn_backward(q, k, v, do, row[None], col[None], flags[None],
                                   np.array([ROW], np.uint8), 0.5)
    for g in (dq, dk, dv):
        assert np.all(g[:, :, ~inside] == 0)
        assert np.abs(g[:, :, inside]).min() > 0


# ---------------------------------------------------------------------------------------
# segment tables
# ---------------------------------------------------------------------------------------
def brute_rank(ids, flags):
    """slot of table token k = #{table j : id_j < id_k} + #{table j < k : id_j = id_k}."""
    N = len(ids)
    out = {}
    for kk in range(N):
        if flags[kk] != L:
            continue
        out[kk] = sum(1 for j in range(N) if flags[j] == L and
                      (ids[j] < ids[kk] or (ids[j] == ids[kk] and j < kk)))
    return out


@pytest.mark.parametrize("seed", range(5))
def test_segments_vs_brute_force_rank(seed):
    rng = np.random.default_rng(50 + seed)
    st = synth.random_structure(rng, 3, 80, max_rows=8, max_cols=6, scatter=seed % 2 == 0,
                                sparse_ids=seed % 2 == 1)
    seg = orc.build_segments(st.row_ids, st.col_ids, st.flags)
    B, N = st.flags.shape
    for b in range(B):
        f = st.flags[b]
        nG, nL = int((f == G).sum()), int((f == L).sum())
        assert seg["counts"][b, 0] == nG and seg["counts"][b, 1] == nL
        assert seg["global_idx"][b, :nG].tolist() == np.nonzero(f == G)[0].tolist()
        assert np.all(seg["global_idx"][b, nG:] == -1)
        for view, ids in enumerate((st.row_ids[b], st.col_ids[b])):
            perm = seg["perm"][view, b]
            rank = brute_rank(ids, f)
            for tok, slot in rank.items():
                assert perm[slot] == tok
            assert np.all(perm[nL:] == -1)
            S = seg["counts"][b, 2 + view]
            assert S == len(np.unique(ids[f == L]))
            off = seg["seg_off"][view, b]
            assert off[0] == (0 if nL else off[0]) and off[S] == nL and np.all(off[S + 1:] == -1)
            assert np.all(np.diff(off[: S + 1]) > 0)
            sorted_ids = ids[perm[:nL]]
            for i in range(S):
                run = sorted_ids[off[i]: off[i + 1]]
                assert np.all(run == run[0])
                if i:
                    assert sorted_ids[off[i] - 1] < run[0]
                assert np.all(seg["seg_of_tok"][view, b][perm[off[i]: off[i + 1]]] == i)
            assert np.all(seg["seg_of_tok"][view, b][f != L] == -1)


def test_segments_match_mask_blocks():
    # Two table tokens share a segment in a view iff the mask of that head kind lets them
    # attend to each other.
    rng = np.random.default_rng(77)
    st = synth.random_structure(rng, 2, 64, scatter=True, sparse_ids=True)
    seg = orc.build_segments(st.row_ids, st.col_ids, st.flags)
    for b in range(2):
        loc = st.flags[b] == L
        for view, kind in enumerate((ROW, COL)):
            m = orc.attention_mask(st.row_ids[b], st.col_ids[b], st.flags[b], kind).astype(bool)
            s = seg["seg_of_tok"][view, b]
            same = (s[:, None] == s[None, :]) & loc[:, None] & loc[None, :]
            assert np.array_equal(same, m & loc[:, None] & loc[None, :])


def test_segments_empty_and_degenerate():
    flags = np.array([[P] * 8, [G] * 8, [L] * 8], np.uint8)
    row = np.zeros((3, 8), np.int32)
    col = np.arange(8, dtype=np.int32)[None].repeat(3, 0)
    seg = orc.build_segments(row, col, flags)
    assert seg["counts"].tolist() == [[0, 0, 0, 0], [8, 0, 0, 0], [0, 8, 1, 8]]
    assert seg["seg_off"][0, 2, :2].tolist() == [0, 8]
    assert seg["seg_off"][1, 2, :9].tolist() == list(range(9))
    assert seg["seg_off"][0, 0, 0] == 0 and seg["seg_off"][0, 0, 1] == -1
