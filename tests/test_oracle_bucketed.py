"""Pins for the oracle's bucketed mode, the approximation of Section 3.1 (CPU only).

What the paper fixes, and what is checked against it here:
  * the claim at the end of Section 3.1: once G holds the question part and R holds the longest
    row / column, the bucketed pattern IS the mask-based pattern of Section 3;
  * the section's own description read token by token (the first G question tokens attend to
    and from everything; the rest of the head's order is cut into buckets of R; a token of
    bucket j attends to the global part and to the tokens of buckets j - 1, j, j + 1 that share
    its row / column), written out below as plain loops with explicit key lists and a softmax
    by hand, must give the oracle's outputs;
  * a hand-derived 8-token example and closed-form pair counts.
The readings the paper leaves open (how the global part is filled, no wrap-around between the
first and the last bucket) are shared by both sides of these tests: for them parity is
unpinned, as the oracle's header says.
"""
import numpy as np
import pytest

from oracle import mate_oracle as orc
from paper_2109_04312_amd import synth

L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD
ROW, COL = synth.HEAD_ROW, synth.HEAD_COL


def longest_segment(ids, flags):
    loc = np.asarray(flags) == L
    if not loc.any():
        return 1
    return int(np.unique(np.asarray(ids)[loc], return_counts=True)[1].max())


@pytest.mark.parametrize("seed", range(6))
def test_large_enough_G_and_R_give_the_mask_based_pattern(seed):
    rng = np.random.default_rng(seed)
    st = synth.random_structure(rng, 4, 90, max_rows=7, max_cols=5, max_global=9, max_cell=4,
                                scatter=seed % 2 == 1, sparse_ids=seed % 3 == 2)
    for b in range(st.B):
        row, col, fl = st.row_ids[b], st.col_ids[b], st.flags[b]
        n_q = int((fl == G).sum())
        for kind, ids in ((ROW, row), (COL, col)):
            want = orc.attention_mask(row, col, fl, kind)
            R = longest_segment(ids, fl)
            for g_len, radius in ((n_q, R), (n_q + 5, R), (n_q, R + 3), (1000, 1000)):
                got = orc.bucketed_attention_mask(row, col, fl, kind, g_len, radius)
                assert np.array_equal(got, want), (b, kind, g_len, radius)
            if R >= 3:      # and a radius that is too small does change the pattern
                got = orc.bucketed_attention_mask(row, col, fl, kind, n_q, 1)
                assert got.sum() < want.sum()
                assert not (got & ~want).any()


def test_hand_derived_example():
    """8 positions: three question tokens, four table tokens in rows 1,1,1,2, one pad; G = 2,
    R = 1, row head.  The third question token joins the long part with its id 0.  Sorted long
    part: positions 2 | 3 4 5 | 6 = slots 0..4 = buckets 0..4 (R = 1).  Position 3 (bucket 1)
    reaches buckets 0..2 but only 3 and 4 share its row; position 5 (bucket 3) reaches 4 and
    5; position 4 reaches all of its row."""
    flags = np.array([G, G, G, L, L, L, L, P], np.uint8)
    row = np.array([0, 0, 0, 1, 1, 1, 2, 0], np.int32)
    col = np.zeros(8, np.int32)
    want = np.array([
        [1, 1, 1, 1, 1, 1, 1, 0],
        [1, 1, 1, 1, 1, 1, 1, 0],
        [1, 1, 1, 0, 0, 0, 0, 0],
        [1, 1, 0, 1, 1, 0, 0, 0],
        [1, 1, 0, 1, 1, 1, 0, 0],
        [1, 1, 0, 0, 1, 1, 0, 0],
        [1, 1, 0, 0, 0, 0, 1, 0],
        [0, 0, 0, 0, 0, 0, 0, 0]], np.uint8)
    assert np.array_equal(orc.bucketed_attention_mask(row, col, flags, ROW, 2, 1), want)
    # R = 2: buckets {2,3} {4,5} {6}: the whole row 1 lies in two adjacent buckets
    want2 = want.copy()
    want2[3, 5] = want2[5, 3] = 1
    assert np.array_equal(orc.bucketed_attention_mask(row, col, flags, ROW, 2, 2), want2)
    assert np.array_equal(orc.bucketed_flags(flags, 2), [G, G, L, L, L, L, L, P])
    assert np.array_equal(orc.bucketed_flags(flags, 0), [L, L, L, L, L, L, L, P])
    assert np.array_equal(orc.bucketed_flags(flags, 3), flags)


@pytest.mark.parametrize("n_tok,radius", [(12, 3), (13, 3), (40, 7), (5, 9), (64, 1), (30, 30)])
def test_pair_count_closed_form_single_segment(n_tok, radius):
    """One segment of n tokens and nothing else: bucket sizes b_0 .. b_m (all R but the last);
    a token of bucket j sees b_{j-1} + b_j + b_{j+1} tokens."""
    flags = np.full(n_tok, L, np.uint8)
    ids = np.full(n_tok, 4, np.int32)
    sizes = [min(radius, n_tok - s) for s in range(0, n_tok, radius)]
    padded = [0] + sizes + [0]
    want = sum(padded[j] * (padded[j - 1] + padded[j] + padded[j + 1]) for j in range(1, len(sizes) + 1))
    assert orc.useful_pairs(ids, ids, flags, ROW, bucketed=(0, radius)) == want
    if n_tok % radius == 0 and n_tok // radius >= 2:
        assert want == (3 * (n_tok // radius) - 2) * radius * radius


# ---- Section 3.1 read as prose, token by token (no mask matrix) ----------------------------
def prose_forward(q, k, v, ids, flags, g_len, radius, scale):
    """One (sequence, head), written from the section's description alone: the input is ordered
    by the head's traversal; its first g_len question tokens form the global part, which attends
    to everything; the rest is cut into buckets of `radius` consecutive tokens of that order; a
    token of bucket j attends to the global part and to those tokens of buckets j - 1, j, j + 1
    that share its row / column.  Plain loops over buckets and tokens with explicit key lists and
    a softmax by hand.  Returns O [N, D] (zeros at pads)."""
    import math
    N, D = q.shape
    question = [p for p in range(N) if flags[p] == G]
    global_part = question[:g_len]
    rest = [p for p in range(N) if flags[p] == L] + question[g_len:]
    rest.sort(key=lambda p: (int(ids[p]), p))                 # the head's order of traversal
    buckets = [rest[s:s + radius] for s in range(0, len(rest), radius)]
    out = np.zeros((N, D))

    def attend(query, keys):
        scores = [scale * sum(q[query, d] * k[j, d] for d in range(D)) for j in keys]
        top = max(scores)
        weights = [math.exp(x - top) for x in scores]
        total = sum(weights)
        for j, wgt in zip(keys, weights):
            for d in range(D):
                out[query, d] += wgt / total * v[j, d]

    for query in global_part:
        attend(query, global_part + rest)
    for j, bucket in enumerate(buckets):
        nearby = []
        for jj in (j - 1, j, j + 1):
            if 0 <= jj < len(buckets):
                nearby += buckets[jj]
        for query in bucket:
            attend(query, global_part + [t for t in nearby if ids[t] == ids[query]])
    return out


@pytest.mark.parametrize("seed", range(5))
def test_forward_equals_the_section_read_token_by_token(seed):
    rng = np.random.default_rng(100 + seed)
    N, D = 70, 5
    st = synth.random_structure(rng, 3, N, max_rows=5, max_cols=4, max_global=8, max_cell=6,
                                scatter=seed % 2 == 0)
    q, k, v = (rng.standard_normal((3, 2, N, D)) for _ in range(3))
    hk = np.array([ROW, COL], np.uint8)
    for g_len, radius in ((3, 4), (100, 2), (0, 5), (5, 64)):
        o, _ = orc.attn_forward(q, k, v, st.row_ids, st.col_ids, st.flags, hk, 0.7, bucketed=(g_len, radius))
        for b in range(3):
            for h, ids in ((0, st.row_ids[b]), (1, st.col_ids[b])):
                want = prose_forward(q[b, h], k[b, h], v[b, h], ids, st.flags[b], g_len, radius, 0.7)
                assert np.abs(o[b, h] - want).max() < 1e-12, (g_len, radius, b, h)


@pytest.mark.parametrize("seed", range(4))
def test_window_table_lists_exactly_the_attended_table_tokens(seed):
    rng = np.random.default_rng(200 + seed)
    st = synth.random_structure(rng, 3, 80, max_rows=5, max_cols=4, max_global=7, max_cell=7, scatter=seed >= 2)
    for bucketed in (None, (4, 3), (0, 1), (2, 10)):
        tab = orc.build_segments(st.row_ids, st.col_ids, st.flags, bucketed=bucketed)
        for b in range(st.B):
            fl = st.flags[b] if bucketed is None else orc.bucketed_flags(st.flags[b], bucketed[0])
            assert tab["counts"][b, 0] == (fl == G).sum() and tab["counts"][b, 1] == (fl == L).sum()
            for view, kind in ((0, ROW), (1, COL)):
                if bucketed is None:
                    m = orc.attention_mask(st.row_ids[b], st.col_ids[b], st.flags[b], kind)
                else:
                    m = orc.bucketed_attention_mask(st.row_ids[b], st.col_ids[b], st.flags[b], kind, *bucketed)
                perm = tab["perm"][view, b]
                n_l = int(tab["counts"][b, 1])
                for s in range(n_l):
                    lo, hi = tab["window"][view, b, s]
                    seen = {int(j) for j in np.flatnonzero(m[perm[s]]) if fl[j] == L}
                    assert seen == {int(p) for p in perm[lo:hi]}, (bucketed, b, view, s)
                assert not tab["window"][view, b, n_l:].any()


def test_properties_subset_symmetry_self():
    rng = np.random.default_rng(7)
    st = synth.random_structure(rng, 5, 100, max_rows=4, max_cols=3, max_global=12, max_cell=9, scatter=True)
    for b in range(st.B):
        row, col, fl = st.row_ids[b], st.col_ids[b], st.flags[b]
        for kind in (ROW, COL):
            for g_len, radius in ((5, 2), (0, 4), (50, 6)):
                m = orc.bucketed_attention_mask(row, col, fl, kind, g_len, radius).astype(bool)
                cut = orc.bucketed_flags(fl, g_len)
                assert not (m & ~orc.attention_mask(row, col, cut, kind).astype(bool)).any()
                loc = cut == L
                ll = m[np.ix_(loc, loc)]
                assert np.array_equal(ll, ll.T)
                nonpad = cut != P
                assert m[np.arange(100), np.arange(100)][nonpad].all()
                assert not m[~nonpad].any() and not m[:, ~nonpad].any()
                assert (cut == G).sum() == min(g_len, (fl == G).sum())


def test_backward_vs_finite_differences_in_bucketed_mode():
    rng = np.random.default_rng(11)
    N, D = 24, 3
    st = synth.random_structure(rng, 1, N, max_rows=3, max_cols=2, max_global=5, max_cell=5)
    hk = np.array([ROW, COL], np.uint8)
    q, k, v, do = (rng.standard_normal((1, 2, N, D)) for _ in range(4))
    args = (st.row_ids, st.col_ids, st.flags, hk, 0.6)
    mode = (2, 3)
    dq, dk, dv = orc.attn_backward(q, k, v, do, *args, bucketed=mode)
    nonpad = (st.flags[0] != P)[None, None, :, None]
    loss = lambda q_, k_, v_: float((orc.attn_forward(q_, k_, v_, *args, bucketed=mode)[0] * do * nonpad).sum())
    eps = 1e-6
    for name, grad, idx in (("q", dq, 0), ("k", dk, 1), ("v", dv, 2)):
        for _ in range(12):
            pos = tuple(int(rng.integers(0, s)) for s in q.shape)
            xs = [q.copy(), k.copy(), v.copy()]
            xs[idx][pos] += eps
            up = loss(*xs)
            xs[idx][pos] -= 2 * eps
            fd = (up - loss(*xs)) / (2 * eps)
            assert abs(fd - grad[pos]) < 1e-6, (name, pos)

