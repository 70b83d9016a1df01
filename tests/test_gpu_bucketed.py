"""GPU parity of the bucketed mode (the approximation of Section 3.1) through the C ABI:
segment tables and windows bit-exact, attention forward and backward within the tolerances,
against the oracle's bucketed pattern on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2109_04312_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu
ROW, COL = synth.HEAD_ROW, synth.HEAD_COL
PAPER_MODE = (116, 42)   # G and R of the published models (appendix, fine-tuning set-up)


def _build(st, bucketed, zeroed=False):
    from paper_2109_04312_amd import mate
    r, c, f = hp.dev_structure(st)
    out = None
    if zeroed:   # the few alignment words between the tables are never written
        out = mate.Segments(torch.zeros(mate.mate_segments_bytes(st.B, st.N), dtype=torch.uint8, device="cuda"),
                            st.B, st.N)
    return mate.build_segments(r, c, f, out=out, bucketed=bucketed)


@pytest.mark.parametrize("mode", [(0, 1), (3, 2), (5, 7), (116, 42), (1, 64), (10 ** 6, 10 ** 6)])
@pytest.mark.parametrize("N", [1, 65, 700, 1025, 5000, 16384])
def test_bucketed_tables_scattered(N, mode):
    print(f"bucketed tables N={N} G,R={mode}", flush=True)
    rng = np.random.default_rng(N + mode[0])
    st = synth.random_structure(rng, 3, N, max_rows=max(1, min(300, N // 3)), max_cols=6,
                                max_global=min(N, 300), max_cell=9, scatter=N % 2 == 1, sparse_ids=N > 1000)
    hp.compare_segments(_build(st, mode), st, bucketed=mode)


@pytest.mark.parametrize("idx", [2, 4, 5, 6])
def test_bucketed_tables_benchmark_configs(idx):
    print(f"bucketed tables config {idx}", flush=True)
    w = synth.make_config(idx, tensors=False)
    hp.compare_segments(_build(w.structure, PAPER_MODE), w.structure, bucketed=PAPER_MODE)


def test_large_G_and_R_reproduce_the_plain_tables():
    """Last sentence of the section's description: with G >= the question part and R >= the
    longest row / column the efficient form equals the mask-based one.  Here: the whole table
    buffer is identical to mate_build_segments' but for the two header words holding G and R."""
    w = synth.make_config(3, tensors=False)
    plain = _build(w.structure, None, True).buf.view(torch.int32).clone()
    n_q = int((w.structure.flags == synth.TOK_GLOBAL).sum(axis=1).max())
    longest = 0
    for b in range(w.structure.B):
        loc = w.structure.flags[b] == synth.TOK_LOCAL
        for ids in (w.structure.row_ids[b], w.structure.col_ids[b]):
            longest = max(longest, int(np.unique(ids[loc], return_counts=True)[1].max()))
    for mode in ((n_q, longest), (10 ** 9, 10 ** 9)):
        got = _build(w.structure, mode, True).buf.view(torch.int32).clone()
        got[4:6] = plain[4:6]
        assert torch.equal(got, plain), mode
    tight = _build(w.structure, (n_q, longest // 2), True).buf.view(torch.int32)
    assert not torch.equal(tight[16:], plain[16:])


def check(w, mode, pairs=None, label=""):
    print(f"case {label or w.name} bucketed={mode} dtype={w.dtype} shape={w.shape}", flush=True)
    got, seg = hp.run_hip(w, True, bucketed=mode)
    hp.compare_segments(seg, w.structure, bucketed=mode)
    ref = hp.run_oracle(w, True, pairs, bucketed=mode)
    worst = hp.compare(got, ref, w, label or w.name)
    print(hp.report(worst), flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("seed,mode", [(0, (3, 2)), (1, (0, 5)), (2, (8, 1)), (3, (4, 11))])
def test_small_scattered_fwd_bwd(seed, mode, dtype):
    rng = np.random.default_rng(40 + seed)
    N = [200, 333, 130, 270][seed]
    st = synth.random_structure(rng, 2, N, max_rows=6, max_cols=4, max_global=20, max_cell=9,
                                scatter=seed != 0, sparse_ids=seed == 2)
    q, k, v, do = synth.draw_tensors(rng, 2, 4, N, 64, dtype, 4)
    hk = np.array([ROW, COL] * 2, np.uint8)
    check(synth.Workload(f"bucketed{seed}", dtype, st, hk, q, k, v, do, 0.125), mode)


def test_more_question_tokens_than_the_global_part():
    """200 question tokens, G = 116: 84 of them join the long part (id 0 in both views, so they
    share the first buckets with row 0 in the row view and form their own column segment)."""
    rng = np.random.default_rng(116)
    N, R, C = 2048, 60, 5
    row, col, flag = synth.flatten_table(N, 200, R, C, synth.geometric_lengths(rng, 5.0, 40, R * C))
    st = synth.Structure(row[None], col[None], flag[None])
    q, k, v, do = synth.draw_tensors(rng, 1, 2, N, 64, "bf16", 4)
    w = synth.Workload("bucketed_question_overflow", "bf16", st, np.array([ROW, COL], np.uint8), q, k, v, do, 0.125)
    check(w, PAPER_MODE)


def test_config2_paper_mode():
    check(synth.make_config(2), PAPER_MODE)


def test_config4_headline_paper_mode_sampled_heads():
    # columns of 1600 tokens are cut to windows of at most 126; rows (about 32 tokens) are not
    check(synth.make_config(4), PAPER_MODE, pairs=[(0, 0), (0, 15), (1, 7), (1, 8)])


def test_config6_long_cells_paper_mode_sampled_heads():
    check(synth.make_config(6), PAPER_MODE, pairs=[(0, 0), (0, 8), (5, 3), (7, 15)])


@pytest.mark.parametrize("idx", [4, 5])
def test_full_size_invariants_over_all_heads(idx):
    """Oracle-free invariants on EVERY (sequence, head) of the full-size configurations in the
    published models' mode (each softmax row sums to 1 whatever the window; rows of dS sum to 0)."""
    from paper_2109_04312_amd import mate
    w = synth.make_config(idx)
    r, c, f = hp.dev_structure(w.structure)
    seg = mate.build_segments(r, c, f, bucketed=PAPER_MODE)
    q, k, v, do = (hp.to_dev(x, "bf16") for x in (w.q, w.k, w.v, w.do))
    nonpad = (f != synth.TOK_PAD)[:, None, :, None]
    o1, _ = mate.attn_fwd(q, k, torch.ones_like(v), seg, w.head_kind, w.scale)
    assert float(((o1.float() - 1.0).abs() * nonpad).max()) <= 4e-3
    out, lse = mate.attn_fwd(q, k, v, seg, w.head_kind, w.scale)
    dq, dk, dv = mate.attn_bwd(q, k, v, out, lse, do, seg, w.head_kind, w.scale)
    torch.cuda.synchronize()
    n_tok = nonpad.sum(dim=2).clamp(min=1).float()
    sum_do = (do.float() * nonpad).sum(dim=2)
    assert float(((dv.float().sum(dim=2) - sum_do).abs() / n_tok.sqrt()).max()) <= 8e-3
    scale_k = dk.float().abs().sum(dim=2).clamp(min=1e-3)
    assert float((dk.float().sum(dim=2).abs() / scale_k).max()) <= 8e-3
    assert bool(torch.isfinite(dq.float()).all())


def test_bad_arguments():
    from paper_2109_04312_amd import mate
    w = synth.make_config(1, tensors=False)
    for mode in ((-1, 4), (4, 0), (4, -2)):
        with pytest.raises(mate.MateError) as e:
            _build(w.structure, mode)
        assert e.value.status == mate.MATE_ERR_UNSUPPORTED
