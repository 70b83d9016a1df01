"""GPU parity: forward and backward vs the float64 oracle, element by element, through the C ABI."""
import time

import numpy as np
import pytest
import torch

from paper_2109_04312_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu
ROW, COL = synth.HEAD_ROW, synth.HEAD_COL


def small_workload(seed, dtype, B=2, N=200, H=4, bwd=True, **kw):
    rng = np.random.default_rng(seed)
    st = synth.random_structure(rng, B, N, **kw)
    q, k, v, do = synth.draw_tensors(rng, B, H, N, 64, dtype, 4)
    hk = np.array([ROW, COL] * (H // 2), np.uint8)
    return synth.Workload(f"small{seed}", dtype, st, hk, q, k, v, do if bwd else None, 0.125)


def check_workload(w, backward, pairs=None, label=""):
    print(f"case {label or w.name} dtype={w.dtype} shape={w.shape} bwd={backward}", flush=True)
    got, seg = hp.run_hip(w, backward)
    hp.compare_segments(seg, w.structure)
    t0 = time.perf_counter()
    ref = hp.run_oracle(w, backward, pairs)
    print(f"   oracle: {len(ref)} (sequence, head) pairs in {time.perf_counter() - t0:.1f} s", flush=True)
    worst = hp.compare(got, ref, w, label or w.name)
    print(hp.report(worst), flush=True)


def test_config1_tiny_f32_forward():
    check_workload(synth.make_config(1), backward=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_small_scattered_fwd_bwd(seed, dtype):
    w = small_workload(seed, dtype, N=[200, 333, 130][seed], max_rows=12, max_cols=7, max_global=20,
                       max_cell=4, scatter=seed != 0, sparse_ids=seed == 2)
    check_workload(w, backward=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_structures(dtype):
    """All pad, all global (dense), no globals, one row, one column, single tokens."""
    L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD
    N = 150
    rng = np.random.default_rng(12)
    flags = np.full((7, N), L, np.uint8)
    row = rng.integers(0, 9, (7, N)).astype(np.int32)
    col = rng.integers(0, 4, (7, N)).astype(np.int32)
    flags[0] = P                                   # empty sequence
    flags[1] = G                                   # dense attention
    flags[1, 100:] = P
    row[3] = 5                                     # one row, no globals  (flags[2]: generic, no globals)
    col[4] = 1                                     # one column
    flags[4, :3] = G
    flags[5] = P                                   # a single table token
    flags[5, 77] = L
    flags[6] = P                                   # one global + one local
    flags[6, 3] = G
    flags[6, 140] = L
    st = synth.Structure(row, col, flags)
    q, k, v, do = synth.draw_tensors(rng, 7, 2, N, 64, dtype, 4)
    w = synth.Workload("degenerate", dtype, st, np.array([ROW, COL], np.uint8), q, k, v, do, 0.125)
    check_workload(w, backward=True)


@pytest.mark.parametrize("n_global,N", [(200, 2048), (700, 1500), (1024, 1024), (129, 4000)])
def test_many_question_tokens(n_global, N):
    """Question-token owners spanning several 128-row tiles, with and without chunked streams
    (the all-question case is plain dense attention)."""
    rng = np.random.default_rng(n_global)
    R, C = 60, 5
    row, col, flag = synth.flatten_table(N, n_global, R, C, synth.geometric_lengths(rng, 4.0, 12, R * C))
    st = synth.Structure(row[None], col[None], flag[None])
    q, k, v, do = synth.draw_tensors(rng, 1, 2, N, 64, "bf16", 4)
    w = synth.Workload(f"globals{n_global}", "bf16", st, np.array([ROW, COL], np.uint8), q, k, v, do, 0.125)
    check_workload(w, backward=True)


def test_maximum_sequence_length():
    """N = 16384, the largest length the library accepts (the segment builder's LDS limit): a
    full 128-tile owner grid, 9-bit and 10-bit ids, a sequence filled to the last position."""
    N = 16384
    rng = np.random.default_rng(16384)
    R, C = 700, 12
    row, col, flag = synth.flatten_table(N, 100, R, C, synth.geometric_lengths(rng, 2.0, 8, R * C))
    assert (flag != synth.TOK_PAD).all()      # the table is cut at N: no padding at all
    st = synth.Structure(row[None], col[None], flag[None])
    q, k, v, do = synth.draw_tensors(rng, 1, 2, N, 64, "bf16", 4)
    w = synth.Workload("max_length", "bf16", st, np.array([ROW, COL], np.uint8), q, k, v, do, 0.125)
    check_workload(w, backward=True)


def test_config2_bf16_fwd_bwd():
    check_workload(synth.make_config(2), backward=True)


def test_config3_bf16_fwd_bwd():
    # 64 of the 128 (sequence, head) pairs: every sequence, four row heads and four column heads
    w = synth.make_config(3)
    pairs = [(b, h) for b in range(8) for h in (0, 1, 6, 7, 8, 9, 14, 15)]
    check_workload(w, backward=True, pairs=pairs)


@pytest.mark.parametrize("b,kind", [(0, ROW), (0, COL), (1, ROW), (1, COL)])
def test_config4_headline_every_head(b, kind):
    # Full benchmark size, the launch configuration bench.py times: every one of the 32
    # (sequence, head) pairs is compared with the oracle element by element, eight per test (one
    # sequence's row heads or column heads; the oracle takes 1.5 - 6 s per pair at this length).
    w = synth.make_config(4)
    pairs = [(b, h) for h in range(16) if w.head_kind[h] == kind]
    assert len(pairs) == 8
    check_workload(w, backward=True, pairs=pairs, label=f"{w.name} b={b} kind={kind}")


def test_config5_ragged_sampled_heads():
    # every sequence with one row head and one column head (32 of the 256 pairs);
    # b=0: one-row table (row heads dense), b=1: one-column table (column heads dense)
    w = synth.make_config(5)
    pairs = [(b, h) for b in range(16) for h in (b % 8, 8 + (3 * b) % 8)]
    check_workload(w, backward=True, pairs=pairs)


def test_config6_long_cells_sampled_heads():
    # long expanded cells: both views have segments of hundreds of tokens; every sequence, two
    # row heads and two column heads (32 of the 128 pairs)
    w = synth.make_config(6)
    check_workload(w, backward=True, pairs=[(b, h) for b in range(8) for h in (0, 5, 8, 15)])


@pytest.mark.parametrize("idx", [4, 5])
def test_full_size_properties_over_all_heads(idx):
    """Invariants that need no oracle, checked on EVERY (sequence, head) of the full-size
    configurations (the oracle comparison above covers a sample of them):
      * V = 1 everywhere  =>  O = 1 at every non-pad position (each softmax row sums to 1);
      * sum_j dV_j = sum_k dO_k over non-pad tokens (same reason);
      * sum_j dK_j = 0 (every row of dS sums to 0)."""
    from paper_2109_04312_amd import mate
    w = synth.make_config(idx)
    r, c, f = hp.dev_structure(w.structure)
    seg = mate.build_segments(r, c, f)
    q, k, v, do = (hp.to_dev(x, "bf16") for x in (w.q, w.k, w.v, w.do))
    nonpad = (f != synth.TOK_PAD)[:, None, :, None]
    ones = torch.ones_like(v)
    o1, _ = mate.attn_fwd(q, k, ones, seg, w.head_kind, w.scale)
    assert float(((o1.float() - 1.0).abs() * nonpad).max()) <= 4e-3      # one bf16 ulp at 1
    out, lse = mate.attn_fwd(q, k, v, seg, w.head_kind, w.scale)
    dq, dk, dv = mate.attn_bwd(q, k, v, out, lse, do, seg, w.head_kind, w.scale)
    torch.cuda.synchronize()
    sum_do = (do.float() * nonpad).sum(dim=2)                 # [B, H, D]
    sum_dv = dv.float().sum(dim=2)
    n_tok = nonpad.sum(dim=2).clamp(min=1).float()            # rounding of n_tok bf16 values
    # bf16 rounding of n_tok values: observed 2e-3; one missing 128-row unit would give ~1e-1
    assert float(((sum_dv - sum_do).abs() / n_tok.sqrt()).max()) <= 8e-3
    sum_dk = dk.float().sum(dim=2)
    scale_k = dk.float().abs().sum(dim=2).clamp(min=1e-3)
    assert float((sum_dk.abs() / scale_k).max()) <= 8e-3      # observed 4e-4 .. 2e-3
    assert bool(torch.isfinite(dq.float()).all())


def test_backward_is_bit_reproducible():
    from paper_2109_04312_amd import mate
    w = small_workload(5, "bf16", B=2, N=700, H=4, max_rows=40, max_cols=6, max_global=70, max_cell=5)
    r, c, f = hp.dev_structure(w.structure)
    seg = mate.build_segments(r, c, f)
    q, k, v, do = (hp.to_dev(x, "bf16") for x in (w.q, w.k, w.v, w.do))
    out, lse = mate.attn_fwd(q, k, v, seg, w.head_kind, w.scale)
    a = mate.attn_bwd(q, k, v, out, lse, do, seg, w.head_kind, w.scale)
    b = mate.attn_bwd(q, k, v, out, lse, do, seg, w.head_kind, w.scale)
    out2, lse2 = mate.attn_fwd(q, k, v, seg, w.head_kind, w.scale)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert torch.equal(out, out2) and torch.equal(lse, lse2)


@pytest.mark.parametrize("id_step", [1, 1000])
def test_more_unit_cuts_than_records(id_step):
    """Every row is a segment of 129 slots and every column one of 258: cutting at each of them
    would need about twice as many unit records as a view has, so the builder falls back to a cut
    every 128 slots, and units straddle long segments again.  id_step = 1000 takes the ids past
    the counting sort's range (general sorting path)."""
    N, rows, cols = 4096, 30, 15
    L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD
    flags = np.full((1, N), P, np.uint8)
    row = np.zeros((1, N), np.int32)
    col = np.zeros((1, N), np.int32)
    flags[0, :20] = G
    n = rows * 129
    assert n == cols * 258 and 20 + n <= N
    flags[0, 20:20 + n] = L
    i = np.arange(n)
    row[0, 20:20 + n] = (1 + i // 129) * id_step
    col[0, 20:20 + n] = (1 + i % cols) * id_step
    st = synth.Structure(row, col, flags)
    rng = np.random.default_rng(129 + id_step)
    q, k, v, do = synth.draw_tensors(rng, 1, 2, N, 64, "bf16", 4)
    w = synth.Workload(f"cuts_step{id_step}", "bf16", st, np.array([ROW, COL], np.uint8), q, k, v, do, 0.125)
    check_workload(w, backward=True)


def test_head_kind_mix_and_order():
    # any assignment of kinds to heads, not only "first half rows"
    w = small_workload(8, "bf16", B=1, N=260, H=5, max_rows=10, max_cols=5, max_global=9)
    w.head_kind = np.array([COL, COL, ROW, COL, ROW], np.uint8)
    check_workload(w, backward=True)


@pytest.mark.parametrize("kinds", [(ROW, ROW, ROW), (COL, COL, COL), (ROW, COL, COL)])
def test_single_kind_and_odd_pair_counts(kinds):
    # only row heads / only column heads; B * H = 9 is not a multiple of the eight work queues
    w = small_workload(11, "bf16", B=3, N=300, H=3, max_rows=12, max_cols=5, max_global=20)
    w.head_kind = np.array(kinds, np.uint8)
    check_workload(w, backward=True, label=f"kinds{kinds}")


def test_argument_errors_leave_outputs_untouched():
    from paper_2109_04312_amd import mate
    w = small_workload(1, "f32", B=1, N=64, H=2, bwd=False)
    r, c, f = hp.dev_structure(w.structure)
    seg = mate.build_segments(r, c, f)
    q = hp.to_dev(w.q, "f32")
    out = torch.full_like(q, 7.0)
    lse = torch.full((1, 2, 64), 7.0, device="cuda")
    hk = np.array([0, 9], np.uint8)
    st = mate.mate_attn_fwd(q.data_ptr(), q.data_ptr(), q.data_ptr(), seg.buf.data_ptr(), hk.ctypes.data,
                            1, 2, 64, 64, 0, 0.125, out.data_ptr(), lse.data_ptr(), None, 0, None)
    assert st == mate.MATE_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((out == 7).all()) and bool((lse == 7).all())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tables_of_another_shape_leave_outputs_untouched(dtype):
    """The attention calls are asynchronous and cannot return what only the device sees: given a
    table buffer that was built for another (B, N), or never built, every workgroup leaves before
    using it, the outputs stay as they were, and mate_segments_status names the problem."""
    from paper_2109_04312_amd import mate
    w = small_workload(31, dtype, B=2, N=300, H=2, max_rows=9, max_cols=4, max_global=12)
    r, c, f = hp.dev_structure(w.structure)
    q, k, v, do = (hp.to_dev(x, dtype) for x in (w.q, w.k, w.v, w.do))
    B, H, N, D = q.shape
    code = mate.MATE_BF16 if dtype == "bf16" else mate.MATE_F32
    hk = np.ascontiguousarray(w.head_kind)
    nbytes = max(mate.mate_segments_bytes(B, N), mate.mate_segments_bytes(1, 200))
    other = mate.Segments(torch.zeros(nbytes, dtype=torch.uint8, device="cuda"), 1, 200)
    mate.build_segments(r[:1, :200].contiguous(), c[:1, :200].contiguous(), f[:1, :200].contiguous(), out=other)
    never = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device="cuda")
    good = mate.build_segments(r, c, f)
    assert mate.segments_status(good) == mate.MATE_OK
    assert mate.mate_segments_status(other.buf.data_ptr(), B, N, None) == mate.MATE_ERR_SHAPE
    assert mate.mate_segments_status(never.data_ptr(), B, N, None) == mate.MATE_ERR_SHAPE
    out_ref, lse_ref = mate.attn_fwd(q, k, v, good, hk, 0.125)
    ws_f = mate.workspace(B, H, N, D, code, False, "cuda")
    ws_b = mate.workspace(B, H, N, D, code, True, "cuda")
    for buf in (other.buf, never):
        out = torch.full_like(q, 7.0)
        lse = torch.full((B, H, N), 7.0, device="cuda")
        grads = [torch.full_like(q, 7.0) for _ in range(3)]
        st = mate.mate_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), buf.data_ptr(), hk.ctypes.data,
                                B, H, N, D, code, 0.125, out.data_ptr(), lse.data_ptr(),
                                ws_f.data_ptr(), ws_f.numel(), None)
        assert st == mate.MATE_OK          # nothing the host can see is wrong
        st = mate.mate_attn_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out_ref.data_ptr(), lse_ref.data_ptr(),
                                do.data_ptr(), buf.data_ptr(), hk.ctypes.data, B, H, N, D, code, 0.125,
                                *(g.data_ptr() for g in grads), ws_b.data_ptr(), ws_b.numel(), None)
        assert st == mate.MATE_OK
        torch.cuda.synchronize()
        for t in (out, lse, *grads):
            assert bool((t == 7).all())
    with pytest.raises(mate.MateError) as e:      # the binding knows the shape its tables were built for
        mate.attn_fwd(q, k, v, other, hk, 0.125)
    assert e.value.status == mate.MATE_ERR_SHAPE


def test_invalid_ids_are_reported_by_the_status_call():
    from paper_2109_04312_amd import mate
    w = small_workload(32, "bf16", B=3, N=150, H=2, max_rows=6, max_cols=4, max_global=5)
    st = w.structure
    table = np.flatnonzero(st.flags[1] == synth.TOK_LOCAL)
    st.row_ids[1, table[3]] = -4                     # a negative id on a table token of sequence 1
    r, c, f = hp.dev_structure(st)
    seg = mate.build_segments(r, c, f)
    assert mate.segments_status(seg) == mate.MATE_ERR_BAD_ID
    # the tables are still consistent, so the attention runs and writes every row
    q, k, v = (hp.to_dev(x, "bf16") for x in (w.q, w.k, w.v))
    out, lse = mate.attn_fwd(q, k, v, seg, w.head_kind, 0.125, out=torch.full_like(q, float("nan")))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    st.row_ids[1, table[3]] = 0
    st.flags[2, 5] = 9                               # a flag value above 2
    r, c, f = hp.dev_structure(st)
    assert mate.segments_status(mate.build_segments(r, c, f)) == mate.MATE_ERR_BAD_ID


def test_step_replays_identically_from_a_captured_graph():
    """The library allocates nothing, clears nothing with memsets and never synchronises inside
    build / forward / backward, so a whole step can be captured once and replayed: every replay
    (with eager work in between) must reproduce the eager result bit for bit."""
    from paper_2109_04312_amd import mate
    w = small_workload(21, "bf16", B=2, N=900, H=4, max_rows=30, max_cols=6, max_global=80, max_cell=6)
    r, c, f = hp.dev_structure(w.structure)
    q, k, v, do = (hp.to_dev(x, "bf16") for x in (w.q, w.k, w.v, w.do))
    B, H, N, D = q.shape
    code = mate.MATE_BF16

    def buffers():
        seg = mate.Segments(torch.zeros(mate.mate_segments_bytes(B, N), dtype=torch.uint8, device="cuda"), B, N)
        return dict(seg=seg, out=torch.empty_like(q), lse=torch.empty((B, H, N), dtype=torch.float32, device="cuda"),
                    dq=torch.empty_like(q), dk=torch.empty_like(q), dv=torch.empty_like(q),
                    ws_f=mate.workspace(B, H, N, D, code, False, "cuda"), ws_b=mate.workspace(B, H, N, D, code, True, "cuda"))

    def step(bf):
        mate.build_segments(r, c, f, out=bf["seg"])
        mate.attn_fwd(q, k, v, bf["seg"], w.head_kind, w.scale, out=bf["out"], lse=bf["lse"], ws=bf["ws_f"])
        mate.attn_bwd(q, k, v, bf["out"], bf["lse"], do, bf["seg"], w.head_kind, w.scale,
                      dq=bf["dq"], dk=bf["dk"], dv=bf["dv"], ws=bf["ws_b"])

    eager, graphed = buffers(), buffers()
    step(eager)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graphed)                                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(graphed)
    for replay in range(3):
        for name in ("out", "lse", "dq", "dk", "dv"):
            graphed[name].fill_(float("nan"))          # a replay must rewrite everything
        step(eager)                                     # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        for name in ("out", "lse", "dq", "dk", "dv"):
            assert torch.equal(graphed[name], eager[name]), (replay, name)
