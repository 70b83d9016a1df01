"""GPU parity of the dense-mask entry points (short sequences, no segment tables) vs the float64
oracle, element by element, through the C ABI -- the same oracle and tolerances as the segment path."""
import numpy as np
import pytest
import torch

from paper_2109_04312_amd import synth
from tests import helpers as hp
from tests.test_gpu_attention import small_workload, ROW, COL

pytestmark = pytest.mark.gpu


def check_dense(w, label=""):
    print(f"dense case {label or w.name} shape={w.shape}", flush=True)
    got, _ = hp.run_hip(w, backward=True, dense=True)
    ref = hp.run_oracle(w, True, None)
    worst = hp.compare(got, ref, w, label or w.name)
    print(hp.report(worst), flush=True)


@pytest.mark.parametrize("seed,N", [(0, 64), (1, 200), (2, 333), (3, 512), (4, 1024)])
def test_dense_small_scattered(seed, N):
    # tokens of all three kinds interleaved at arbitrary positions, sparse ids (incl. table tokens
    # with id 0), lengths that are and are not multiples of the 64- and 128-row tiles
    w = small_workload(seed, "bf16", B=2, N=N, H=4, max_rows=12, max_cols=7, max_global=20,
                       max_cell=4, scatter=seed != 0, sparse_ids=seed >= 2)
    check_dense(w)


def test_dense_degenerate_structures():
    """All pad, all global (plain dense attention), no globals, one row, one column, single tokens."""
    L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD
    N = 150
    rng = np.random.default_rng(12)
    flags = np.full((7, N), L, np.uint8)
    row = rng.integers(0, 9, (7, N)).astype(np.int32)
    col = rng.integers(0, 4, (7, N)).astype(np.int32)
    flags[0] = P
    flags[1] = G
    flags[1, 100:] = P
    row[3] = 5
    col[4] = 1
    flags[4, :3] = G
    flags[5] = P
    flags[5, 77] = L
    flags[6] = P
    flags[6, 3] = G
    flags[6, 140] = L
    st = synth.Structure(row, col, flags)
    q, k, v, do = synth.draw_tensors(rng, 7, 2, N, 64, "bf16", 4)
    check_dense(synth.Workload("degenerate", "bf16", st, np.array([ROW, COL], np.uint8), q, k, v, do, 0.125))


def test_dense_config2_sampled_heads_and_agreement_with_segment_path():
    # configuration 2 (N = 512): the dense variant against the oracle on a sample of pairs, and
    # against the segment path on everything (two roundings of the same sums: a few bf16 ulps)
    w = synth.make_config(2)
    dense, _ = hp.run_hip(w, backward=True, dense=True)
    ref = hp.run_oracle(w, True, [(0, 0), (0, 11), (17, 5), (31, 6)])
    hp.compare(dense, ref, w, "cfg2 dense")
    seg, _ = hp.run_hip(w, backward=True, dense=False)
    for name in dense:
        d = np.abs(dense[name] - seg[name]) / hp.bound(name, seg[name], "bf16")
        assert d.max() <= 2.0, (name, d.max())


def test_dense_rejects_what_it_does_not_support():
    from paper_2109_04312_amd import mate
    w = small_workload(1, "f32", B=1, N=64, H=2, bwd=False)
    r, c, f = hp.dev_structure(w.structure)
    q32 = hp.to_dev(w.q, "f32")
    out = torch.full_like(q32, 7.0)
    lse = torch.full((1, 2, 64), 7.0, device="cuda")
    hk = np.array([0, 1], np.uint8)
    st = mate.mate_attn_fwd_dense(q32.data_ptr(), q32.data_ptr(), q32.data_ptr(), r.data_ptr(), c.data_ptr(),
                                  f.data_ptr(), hk.ctypes.data, 1, 2, 64, 64, mate.MATE_F32, 0.125,
                                  out.data_ptr(), lse.data_ptr(), None)
    assert st == mate.MATE_ERR_UNSUPPORTED               # f32
    st = mate.mate_attn_fwd_dense(q32.data_ptr(), q32.data_ptr(), q32.data_ptr(), r.data_ptr(), c.data_ptr(),
                                  f.data_ptr(), hk.ctypes.data, 1, 2, 2048, 64, mate.MATE_BF16, 0.125,
                                  out.data_ptr(), lse.data_ptr(), None)
    assert st == mate.MATE_ERR_UNSUPPORTED               # too long for the dense variant
    torch.cuda.synchronize()
    assert bool((out == 7).all()) and bool((lse == 7).all())
