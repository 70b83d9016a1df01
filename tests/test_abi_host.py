"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU (no compute calls here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mate.h")


@pytest.fixture(scope="module")
def mate():
    from paper_2109_04312_amd import mate as m
    return m


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mate_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(mate):
    names = declared_functions()
    assert set(names) == set(mate.EXPORTS)
    lib = C.CDLL(mate.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_size_queries(mate):
    assert mate.mate_segments_bytes(0, 128) == 0
    assert mate.mate_segments_bytes(1, 0) == 0
    assert mate.mate_segments_bytes(1, mate.MATE_MAX_N + 1) == 0
    small, big = mate.mate_segments_bytes(1, 128), mate.mate_segments_bytes(2, 8192)
    assert 0 < small < big and big % 4 == 0
    # ~14 int32 words per token (two views of perm, seg_off, seg_of_tok, slot range + two lists)
    assert big < 2 * 8192 * 4 * 16
    assert mate.mate_workspace_bytes(2, 16, 8192, 64, mate.MATE_BF16, 0) >= 0
    assert mate.mate_workspace_bytes(2, 16, 8192, 64, mate.MATE_BF16, 1) >= 2 * 16 * 8192 * 4
    assert mate.mate_workspace_bytes(2, 16, 8192, 32, mate.MATE_BF16, 1) == 0


def test_status_strings(mate):
    seen = {mate.mate_status_string(s) for s in range(0, -7, -1)}
    assert len(seen) == 7 and "ok" in seen
    assert mate.mate_status_string(-99) == "unknown status"


def test_argument_errors_are_caught_on_the_host(mate):
    hk = np.zeros(4, np.uint8)
    fake = 0x1000  # never dereferenced: every call below must fail validation first
    f = mate.mate_attn_fwd
    assert f(None, fake, fake, fake, hk.ctypes.data, 1, 4, 128, 64, 0, 1.0, fake, fake, None, 0, None) == mate.MATE_ERR_NULL
    assert f(fake, fake, fake, None, hk.ctypes.data, 1, 4, 128, 64, 0, 1.0, fake, fake, None, 0, None) == mate.MATE_ERR_NULL
    assert f(fake, fake, fake, fake, hk.ctypes.data, 1, 4, 128, 32, 0, 1.0, fake, fake, None, 0, None) == mate.MATE_ERR_UNSUPPORTED
    assert f(fake, fake, fake, fake, hk.ctypes.data, 1, 4, 128, 64, 5, 1.0, fake, fake, None, 0, None) == mate.MATE_ERR_UNSUPPORTED
    assert f(fake, fake, fake, fake, hk.ctypes.data, 0, 4, 128, 64, 0, 1.0, fake, fake, None, 0, None) == mate.MATE_ERR_SHAPE
    assert f(fake, fake, fake, fake, hk.ctypes.data, 1, 4, 1 << 20, 64, 0, 1.0, fake, fake, None, 0, None) == mate.MATE_ERR_SHAPE
    assert f(fake, fake, fake, fake, hk.ctypes.data, 1, 999, 128, 64, 0, 1.0, fake, fake, None, 0, None) == mate.MATE_ERR_SHAPE
    g = mate.mate_attn_bwd
    args = [fake] * 7 + [hk.ctypes.data, 1, 4, 128, 64, 1, 1.0, fake, fake, fake]
    assert g(*args, None, 0, None) == mate.MATE_ERR_WORKSPACE
    assert g(*args, fake, 16, None) == mate.MATE_ERR_WORKSPACE
    bad = list(args)
    bad[14] = None
    assert g(*bad, fake, 1 << 30, None) == mate.MATE_ERR_NULL
    b = mate.mate_build_segments
    assert b(None, fake, fake, 1, 128, fake, None) == mate.MATE_ERR_NULL
    assert b(fake, fake, fake, 1, 0, fake, None) == mate.MATE_ERR_SHAPE
    assert mate.mate_segments_export(None, 1, 128, 0, None, None, None, None, None, None) == mate.MATE_ERR_NULL
    assert mate.mate_segments_export(fake, 1, 128, 2, None, None, None, None, None, None) == mate.MATE_ERR_SHAPE


def test_argument_errors_of_the_later_entry_points(mate):
    fake = 0x1000  # never dereferenced
    bb = mate.mate_build_segments_bucketed
    assert bb(fake, fake, None, 1, 128, 116, 42, fake, None) == mate.MATE_ERR_NULL
    assert bb(fake, fake, fake, 1, 0, 116, 42, fake, None) == mate.MATE_ERR_SHAPE
    assert bb(fake, fake, fake, 1, 128, -1, 42, fake, None) == mate.MATE_ERR_UNSUPPORTED
    assert bb(fake, fake, fake, 1, 128, 116, 0, fake, None) == mate.MATE_ERR_UNSUPPORTED
    assert mate.mate_segments_export_windows(fake, 1, 128, 0, None, None) == mate.MATE_ERR_NULL
    assert mate.mate_segments_export_windows(fake, 1, 128, 3, fake, None) == mate.MATE_ERR_SHAPE
    cp = mate.mate_cell_positions
    assert cp(fake, fake, fake, 1, 128, None, None) == mate.MATE_ERR_NULL
    assert cp(fake, fake, fake, 1, mate.MATE_MAX_N + 1, fake, None) == mate.MATE_ERR_SHAPE
    qp = mate.mate_qkv_project
    ok = [fake, fake, None, fake, 2, 512, 12, 768, mate.MATE_BF16, fake, fake, fake, None]
    for pos, val, want in ((0, None, mate.MATE_ERR_NULL), (11, None, mate.MATE_ERR_NULL),
                           (6, 11, mate.MATE_ERR_UNSUPPORTED),      # odd number of heads
                           (7, 700, mate.MATE_ERR_UNSUPPORTED),     # width not a multiple of 128
                           (8, mate.MATE_F32, mate.MATE_ERR_UNSUPPORTED), (5, 0, mate.MATE_ERR_SHAPE)):
        args = list(ok)
        args[pos] = val
        assert qp(*args) == want, (pos, val)
    op = mate.mate_out_project
    ok = [fake, fake, None, fake, 2, 512, 12, 768, mate.MATE_BF16, fake, None]
    for pos, val, want in ((1, None, mate.MATE_ERR_NULL), (9, None, mate.MATE_ERR_NULL),
                           (7, 64, mate.MATE_ERR_UNSUPPORTED), (4, 0, mate.MATE_ERR_SHAPE)):
        args = list(ok)
        args[pos] = val
        assert op(*args) == want, (pos, val)


def test_argument_errors_of_the_projection_backward(mate):
    fake = 0x1000  # never dereferenced
    assert mate.mate_project_bwd_workspace_bytes(2, 512, 12, 768) > 3 * 12 * 64 * 768 * 2
    assert mate.mate_project_bwd_workspace_bytes(2, 512, 11, 768) == 0
    assert mate.mate_project_bwd_workspace_bytes(2, 512, 12, 700) == 0
    qb = mate.mate_qkv_project_bwd
    ok = [fake, fake, fake, fake, fake, fake, 2, 512, 12, 768, mate.MATE_BF16, fake, fake, fake, fake, 1 << 40, None]
    for pos, val, want in ((0, None, mate.MATE_ERR_NULL), (4, None, mate.MATE_ERR_NULL),
                           (8, 11, mate.MATE_ERR_UNSUPPORTED), (10, mate.MATE_F32, mate.MATE_ERR_UNSUPPORTED),
                           (7, 0, mate.MATE_ERR_SHAPE), (15, 16, mate.MATE_ERR_WORKSPACE),
                           (14, None, mate.MATE_ERR_WORKSPACE), (12, None, mate.MATE_ERR_NULL)):
        args = list(ok)
        args[pos] = val
        assert qb(*args) == want, (pos, val)
    ob = mate.mate_out_project_bwd
    ok = [fake, fake, fake, fake, 2, 512, 12, 768, mate.MATE_BF16, fake, fake, fake, fake, 1 << 40, None]
    for pos, val, want in ((3, None, mate.MATE_ERR_NULL), (7, 64, mate.MATE_ERR_UNSUPPORTED),
                           (13, 16, mate.MATE_ERR_WORKSPACE), (10, None, mate.MATE_ERR_NULL)):
        args = list(ok)
        args[pos] = val
        assert ob(*args) == want, (pos, val)


def test_choice_between_the_two_implementations(mate):
    """Section 3.1: the faster of the two equivalent implementations is used per case.  The
    library's choice is the measured break-even: bf16 up to MATE_DENSE_PREFERRED_MAX_N."""
    f = mate.mate_attn_prefers_dense
    edge = mate.MATE_DENSE_PREFERRED_MAX_N
    assert f(32, 12, 128, mate.MATE_BF16) == 1 and f(1, 1, edge, mate.MATE_BF16) == 1
    assert f(32, 12, edge + 1, mate.MATE_BF16) == 0 and f(2, 16, 8192, mate.MATE_BF16) == 0
    assert f(1, 4, 128, mate.MATE_F32) == 0          # the dense variant is bf16 only
    assert f(1, 4, 0, mate.MATE_BF16) == 0
    assert edge <= mate.MATE_DENSE_MAX_N


def test_status_call_argument_errors(mate):
    fake = 0x1000  # never dereferenced
    assert mate.mate_segments_status(None, 1, 128, None) == mate.MATE_ERR_NULL
    assert mate.mate_segments_status(fake, 0, 128, None) == mate.MATE_ERR_SHAPE
    assert mate.mate_segments_status(fake, 1, mate.MATE_MAX_N + 1, None) == mate.MATE_ERR_SHAPE


def test_bench_pair_count_matches_the_oracle():
    """bench.py counts useful (query, key) pairs with its own vectorised formula (it may not use
    the oracle outside its cpu_baseline leg); here that bookkeeping is held against the oracle's
    mask, in both modes."""
    import importlib.util
    from oracle import mate_oracle as orc
    from paper_2109_04312_amd import synth
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    rng = np.random.default_rng(21)
    for scatter in (False, True):
        st = synth.random_structure(rng, 4, 150, max_rows=6, max_cols=4, max_global=25, max_cell=9, scatter=scatter)
        for mode in (None, (7, 3), (0, 1), (100, 50)):
            got = bench.useful_pairs_per_view(st, mode)
            for b in range(st.B):
                for v, kind in enumerate((synth.HEAD_ROW, synth.HEAD_COL)):
                    want = orc.useful_pairs(st.row_ids[b], st.col_ids[b], st.flags[b], kind, bucketed=mode)
                    assert got[b, v] == want, (scatter, mode, b, v)


def test_bench_reads_the_tracked_traffic_summary(tmp_path):
    """roofline.traffic comes from the tracked counter summary of the workload: the summary parses,
    names the three attention kernels with plausible byte counts (at least the outputs each must
    write: 26.3 MB per tensor on the headline batch), and --summarize-pmc turns profiler csv
    files into the same lines."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module2", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    table, digest = bench.read_traffic("cfg4_B2_N8192_H16")
    assert digest and len(digest) == 16
    per_tensor = 128 * 12853 * 16
    for kernel, tensors_written in (("fwd_mfma_kernel", 1), ("bwd_dq_mfma_kernel", 1), ("bwd_dkv_mfma_kernel", 2)):
        assert table[kernel]["write_bytes"] >= tensors_written * per_tensor
        assert table[kernel]["fetch_bytes"] >= 3 * per_tensor
        assert table[kernel]["fetch_bytes"] + table[kernel]["write_bytes"] < 40 * per_tensor
    # the csv -> summary direction, on a two-dispatch file written here
    for name, counter, values in (("f", "FETCH_SIZE", (100.0, 300.0)), ("w", "WRITE_SIZE", (50.0, 70.0))):
        d = tmp_path / name
        d.mkdir()
        with open(d / "p_counter_collection.csv", "w") as fh:
            fh.write("Dispatch_Id,Kernel_Name,Counter_Name,Counter_Value\n")
            for i, v in enumerate(values):
                # a dispatch reports one row per shader engine / XCD: they add up
                fh.write(f"{i},mate::(anonymous namespace)::fwd_mfma_kernel(mate::AttnArgs),{counter},{v / 2}\n")
                fh.write(f"{i},mate::(anonymous namespace)::fwd_mfma_kernel(mate::AttnArgs),{counter},{v / 2}\n")
    import contextlib
    import io
    buf = io.StringIO()
    with contextlib.redirect_stdout(buf):
        bench.summarize_pmc(str(tmp_path / "f"), str(tmp_path / "w"))
    lines = buf.getvalue().split("\n")
    assert lines[0] == "sources " + bench.sources_digest()
    assert "counter fwd_mfma_kernel 200 60" in lines
