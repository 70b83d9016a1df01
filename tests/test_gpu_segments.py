"""GPU parity: segment builder vs the oracle's stable sort, bit-exact, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2109_04312_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _build(st):
    from paper_2109_04312_amd import mate
    r, c, f = hp.dev_structure(st)
    return mate.build_segments(r, c, f)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6])
def test_segments_benchmark_configs(idx):
    print(f"segments config {idx}", flush=True)
    w = synth.make_config(idx, tensors=False)
    hp.compare_segments(_build(w.structure), w.structure)


@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 1000, 1024, 1025, 4097, 8192, 9000, 16384])
def test_segments_sizes_scattered_sparse_ids(N):
    print(f"segments N={N}", flush=True)
    rng = np.random.default_rng(N)
    st = synth.random_structure(rng, 3, N, max_rows=max(1, min(300, N // 3)), max_cols=12,
                                max_global=min(N, 40), max_cell=4, scatter=True, sparse_ids=True)
    hp.compare_segments(_build(st), st)


def test_segments_degenerate_sequences():
    N = 300
    L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD
    flags = np.stack([np.full(N, P), np.full(N, G), np.full(N, L), np.full(N, L), np.full(N, L)]).astype(np.uint8)
    row = np.zeros((5, N), np.int32)
    col = np.zeros((5, N), np.int32)
    row[3] = np.arange(N)[::-1]              # every token its own row, descending ids
    col[3] = 2**31 - 1                       # one column with the largest id
    row[4] = np.arange(N) % 7
    col[4] = (np.arange(N) * 2654435761 % 2**31).astype(np.int64) % 5
    st = synth.Structure(row, col, flags)
    hp.compare_segments(_build(st), st)


def test_segments_bad_ids_reported():
    from paper_2109_04312_amd import mate
    N = 70
    flags = np.zeros((2, N), np.uint8)
    row = np.ones((2, N), np.int32)
    col = np.ones((2, N), np.int32)
    st = synth.Structure(row, col, flags)
    seg = _build(st)
    mate.segments_export(seg, 0)             # clean input: no error
    row2 = row.copy()
    row2[1, 5] = -3
    with pytest.raises(mate.MateError) as e:
        mate.segments_export(_build(synth.Structure(row2, col, flags)), 0)
    assert e.value.status == mate.MATE_ERR_BAD_ID
    flags2 = flags.copy()
    flags2[0, 9] = 7
    with pytest.raises(mate.MateError) as e:
        mate.segments_export(_build(synth.Structure(row, col, flags2)), 1)
    assert e.value.status == mate.MATE_ERR_BAD_ID


def test_segments_many_sequences():
    """More sequences than the export and status calls copy per batch (64): tables of every
    sequence bit-exact, and an invalid id in a late sequence still reported."""
    from paper_2109_04312_amd import mate
    B, N = 150, 48
    rng = np.random.default_rng(150)
    st = synth.random_structure(rng, B, N, max_rows=6, max_cols=4, max_global=8, max_cell=3,
                                scatter=True, sparse_ids=False)
    seg = _build(st)
    hp.compare_segments(seg, st)
    assert mate.segments_status(seg) == mate.MATE_OK
    row = st.row_ids.copy()
    b = max(i for i in range(128, B) if (st.flags[i] == synth.TOK_LOCAL).any())
    k = int(np.nonzero(st.flags[b] == synth.TOK_LOCAL)[0][0])
    row[b, k] = -1
    seg = _build(synth.Structure(row, st.col_ids, st.flags))
    assert mate.segments_status(seg) == mate.MATE_ERR_BAD_ID


def test_segments_rebuild_is_deterministic_and_reusable():
    """The builder writes the valid part of every list only, so determinism is checked on
    zero-filled buffers, and reuse in place (stale entries of another batch behind the valid
    parts) through the exported tables and through the attention kernels' results."""
    from paper_2109_04312_amd import mate
    rng = np.random.default_rng(3)
    st1 = synth.random_structure(rng, 4, 777, max_rows=50, max_cols=9, scatter=True)
    st2 = synth.random_structure(rng, 4, 777, max_rows=20, max_cols=3)
    nbytes = mate.mate_segments_bytes(4, 777)
    zeroed = lambda: mate.Segments(torch.zeros(nbytes, dtype=torch.uint8, device="cuda"), 4, 777)
    r1, c1, f1 = hp.dev_structure(st1)
    a = mate.build_segments(r1, c1, f1, out=zeroed())
    b = mate.build_segments(r1, c1, f1, out=zeroed())
    torch.cuda.synchronize()
    assert torch.equal(a.buf, b.buf)
    q, k, v, _ = (hp.to_dev(x, "bf16") for x in synth.draw_tensors(rng, 4, 2, 777, 64, "bf16", 4))
    hk = np.array([synth.HEAD_ROW, synth.HEAD_COL], np.uint8)
    want = mate.attn_fwd(q, k, v, a, hk, 0.125)
    r2, c2, f2 = hp.dev_structure(st2)
    mate.build_segments(r2, c2, f2, out=a)     # overwrite in place with another batch
    hp.compare_segments(a, st2)
    mate.build_segments(r1, c1, f1, out=a)     # and back
    hp.compare_segments(a, st1)
    got = mate.attn_fwd(q, k, v, a, hk, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])


def _positions(st):
    from oracle import mate_oracle as orc
    from paper_2109_04312_amd import mate
    r, c, f = hp.dev_structure(st)
    out = torch.full(f.shape, -7, dtype=torch.int32, device="cuda")
    mate.cell_positions(r, c, f, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), orc.cell_positions(st.row_ids, st.col_ids, st.flags))


@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 1000, 1024, 1025, 4097, 8192, 9000, 16384])
def test_cell_positions_sizes(N):
    """Positional index restarting per cell, bit-exact: cells of 1..40 tokens crossing batch
    and wavefront boundaries, in table order and with positions shuffled."""
    print(f"cell positions N={N}", flush=True)
    rng = np.random.default_rng(N)
    for scatter in (False, True):
        st = synth.random_structure(rng, 3, N, max_rows=max(1, min(300, N // 3)), max_cols=12,
                                    max_global=min(N, 40), max_cell=40, scatter=scatter)
        _positions(st)


@pytest.mark.parametrize("idx", [1, 4, 5, 6])
def test_cell_positions_benchmark_configs(idx):
    _positions(synth.make_config(idx, tensors=False).structure)


def test_cell_positions_one_long_cell_and_all_kinds():
    N = 5000
    L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD
    flags = np.stack([np.full(N, L), np.full(N, G), np.full(N, P), np.full(N, L)]).astype(np.uint8)
    row = np.zeros((4, N), np.int32)
    col = np.zeros((4, N), np.int32)
    row[3] = np.arange(N)                    # every token its own cell
    _positions(synth.Structure(row, col, flags))   # sequence 0: one cell of 5000 tokens
