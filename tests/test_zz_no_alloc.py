"""mate_attn_bwd_dense_static -- the entry point for callers that cannot allocate -- against
mate_attn_bwd_dense through the C ABI: same kernels, so the gradients must agree bit for bit,
on two calls in a row that share the library's static scratch, the second on a smaller input.
(Collected last on purpose: the file name sorts after every other test file.)"""
import numpy as np
import pytest
import torch

from paper_2109_04312_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu
ROW, COL = synth.HEAD_ROW, synth.HEAD_COL


def _case(seed, B, N, H):
    rng = np.random.default_rng(seed)
    st = synth.random_structure(rng, B, N, max_rows=14, max_cols=6, max_global=24, max_cell=5,
                                scatter=seed % 2 == 1, sparse_ids=True)
    q, k, v, do = synth.draw_tensors(rng, B, H, N, 64, "bf16", 4)
    hk = np.array([ROW, COL] * (H // 2), np.uint8)
    return synth.Workload(f"static{seed}", "bf16", st, hk, q, k, v, do, 0.125)


def _both(w):
    """dQ, dK, dV from the workspace entry point and from the static-scratch one."""
    from paper_2109_04312_amd import mate
    r, c, f = hp.dev_structure(w.structure)
    q, k, v, do = (hp.to_dev(x, "bf16") for x in (w.q, w.k, w.v, w.do))
    B, H, N, D = q.shape
    hk = np.ascontiguousarray(w.head_kind)
    out, lse = mate.attn_fwd_dense(q, k, v, r, c, f, hk, w.scale)
    want = mate.attn_bwd_dense(q, k, v, out, lse, do, r, c, f, hk, w.scale)
    got = [torch.full_like(q, float("nan")) for _ in range(3)]
    st = mate.mate_attn_bwd_dense_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                         lse.data_ptr(), do.data_ptr(), r.data_ptr(), c.data_ptr(),
                                         f.data_ptr(), hk.ctypes.data, B, H, N, D, mate.MATE_BF16,
                                         float(w.scale), got[0].data_ptr(), got[1].data_ptr(),
                                         got[2].data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == mate.MATE_OK, mate.mate_status_string(st)
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_matches_the_workspace_entry_point_twice():
    big, small = _case(41, 4, 700, 4), _case(42, 2, 130, 2)
    for w in (big, small):          # the second call is smaller: stale scratch lies beyond it
        print(f"static scratch case {w.name} shape={w.shape}", flush=True)
        want, got = _both(w)
        for name, a, b in zip(("dq", "dk", "dv"), want, got):
            assert torch.equal(a, b), f"{w.name}: {name} differs from mate_attn_bwd_dense"
    # and the result is right, not merely equal: the second case against the oracle
    ref = hp.run_oracle(small, True, None)
    res = {n: t.float().cpu().numpy().astype(np.float64) for n, t in zip(("dq", "dk", "dv"), got)}
    hp.compare(res, {bh: {n: d[n] for n in res} for bh, d in ref.items()}, small, "static scratch")


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2109_04312_amd import mate
    fake = 0x1000  # never dereferenced: the size check comes before any launch
    hk = np.zeros(16, np.uint8)
    args = [fake] * 9 + [hk.ctypes.data]
    tail = [64, mate.MATE_BF16, 0.125, fake, fake, fake, None]
    f = mate.mate_attn_bwd_dense_static
    assert 2 * 33 * 16 * 1024 * 4 > mate.MATE_STATIC_SCRATCH_BYTES
    assert f(*args, 33, 16, 1024, *tail) == mate.MATE_ERR_WORKSPACE
    assert f(*args, 1, 16, 2048, *tail) == mate.MATE_ERR_UNSUPPORTED     # longer than the dense variant takes
    assert f(*([None] + args[1:]), 1, 16, 128, *tail) == mate.MATE_ERR_NULL
