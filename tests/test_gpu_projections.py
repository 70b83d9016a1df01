"""GPU parity of the projections either side of the attention (bf16 MFMA GEMMs with the head
split / head gather fused) against the float64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import mate_oracle as orc
from paper_2109_04312_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu
P = synth.TOK_PAD


def bf16(x):
    return synth.round_to_bf16(np.asarray(x, np.float32)).astype(np.float32)


def dev(x, dtype=torch.bfloat16):
    return torch.from_numpy(np.ascontiguousarray(x)).to(dtype).cuda()


def close(got, want, what):
    """bf16 output of an fp32-accumulated product: |err| <= 2e-2 + 2^-8 |ref| (a bf16 store alone
    costs |ref| 2^-9) and the bf16 path's mean-rel bound."""
    got = got.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - want)
    ratio = float((err / hp.bound("projection", want, "bf16")).max()) if err.size else 0.0
    mean_rel = float(err.mean() / (np.abs(want).mean() + 1e-3))
    print(f"   {what}: max-abs {float(err.max()):.2e} = {ratio:.2f} x bound, mean-rel {mean_rel:.2e}", flush=True)
    assert ratio <= 1.0 and mean_rel <= hp.TOL["bf16"]["mean_rel"], what


def make(seed, B, N, H, E, pad_tail=0, scattered_pads=True, bias=True):
    rng = np.random.default_rng(seed)
    x = bf16(rng.standard_normal((B, N, E)))
    w_qkv = bf16(rng.standard_normal((3 * H * 64, E)) / np.sqrt(E))
    w_o = bf16(rng.standard_normal((E, H * 64)) / np.sqrt(H * 64))
    b_qkv = rng.standard_normal(3 * H * 64).astype(np.float32) if bias else None
    b_o = rng.standard_normal(E).astype(np.float32) if bias else None
    flags = rng.choice([synth.TOK_LOCAL, synth.TOK_GLOBAL], size=(B, N)).astype(np.uint8)
    if scattered_pads:
        flags[rng.random((B, N)) < 0.1] = P
    if pad_tail:
        flags[:, N - pad_tail:] = P
    o = bf16(rng.standard_normal((B, H, N, 64)))
    return x, w_qkv, b_qkv, w_o, b_o, flags, o


def check(seed, B, N, H, E, **kw):
    from paper_2109_04312_amd import mate
    print(f"projections B={B} N={N} H={H} E={E} {kw}", flush=True)
    x, w_qkv, b_qkv, w_o, b_o, flags, o = make(seed, B, N, H, E, **kw)
    nan = lambda *shape: torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    fl = torch.from_numpy(flags).cuda()
    q, k, v = mate.qkv_project(dev(x), dev(w_qkv), None if b_qkv is None else dev(b_qkv, torch.float32), fl, H,
                               q=nan(B, H, N, 64), k=nan(B, H, N, 64), v=nan(B, H, N, 64))
    y = mate.out_project(dev(o), dev(w_o), None if b_o is None else dev(b_o, torch.float32), fl, y=nan(B, N, E))
    torch.cuda.synchronize()
    want = orc.project_qkv(x, w_qkv, b_qkv, flags, H)
    for name, g, r in zip("qkv", (q, k, v), want):
        close(g, r, name)
        assert bool((g.float().cpu().numpy()[np.broadcast_to((flags == P)[:, None, :, None], r.shape)] == 0).all())
    close(y, orc.project_out(o, w_o, b_o, flags), "y")
    assert bool((y.float().cpu().numpy()[flags == P] == 0).all())


@pytest.mark.parametrize("N", [1, 64, 127, 128, 129, 200, 333])
def test_small_ragged(N):
    check(N, 2, N, 2, 128)


def test_no_bias_and_tiles_of_padding_only():
    check(1, 3, 700, 4, 256, pad_tail=300, bias=False)
    check(2, 1, 512, 2, 128, pad_tail=512, scattered_pads=False)       # nothing but padding


def test_bert_base_shape():
    check(3, 4, 512, 12, 768, pad_tail=100)


def test_large_tiles_ragged_with_scattered_pads():
    # enough tiles for the 256 x 256 shape of the QKV kernel; N is not a multiple of 256
    check(5, 9, 1000, 12, 768, pad_tail=120)
    check(6, 3, 2500, 16, 1024, pad_tail=0)


def test_headline_shape():
    # configuration 4's layer: B=2, N=8192, 16 heads, model width 1024
    check(4, 2, 8192, 16, 1024, pad_tail=1700, scattered_pads=False)


def test_layer_forward_end_to_end():
    """x -> QKV projection -> segment build -> attention -> output projection, every step in the
    library, against the same chain in the oracle (which keeps float64 between the steps, so the
    bound is looser than a single step's: three roundings to bf16 on the way)."""
    from paper_2109_04312_amd import mate
    w = synth.make_config(2, tensors=False)
    st = w.structure
    B, N, H, E = st.B, st.N, 12, 768
    rng = np.random.default_rng(9)
    x = bf16(rng.standard_normal((B, N, E)))
    w_qkv = bf16(rng.standard_normal((3 * H * 64, E)) / np.sqrt(E))
    w_o = bf16(rng.standard_normal((E, H * 64)) / np.sqrt(H * 64))
    hk = synth.half_row_half_col(H)
    r, c, f = hp.dev_structure(st)
    q, k, v = mate.qkv_project(dev(x), dev(w_qkv), None, f, H)
    seg = mate.build_segments(r, c, f)
    o, _ = mate.attn_fwd(q, k, v, seg, hk, 0.125)
    y = mate.out_project(o, dev(w_o), None, f)
    torch.cuda.synchronize()
    for b in (0, 17):
        sl = slice(b, b + 1)
        qr, kr, vr = orc.project_qkv(x[sl], w_qkv, None, st.flags[sl], H)
        orf, _ = orc.attn_forward(qr, kr, vr, st.row_ids[sl], st.col_ids[sl], st.flags[sl], hk, 0.125)
        yr = orc.project_out(orf, w_o, None, st.flags[sl])
        got = y[sl].float().cpu().numpy().astype(np.float64)
        err = np.abs(got - yr)
        ratio = float((err / hp.bound("projection", yr, "bf16")).max())
        mean_rel = float(err.mean() / (np.abs(yr).mean() + 1e-3))
        print(f"   layer b={b}: max-abs {float(err.max()):.2e} = {ratio:.2f} x one step's bound, "
              f"mean-rel {mean_rel:.2e}", flush=True)
        assert ratio <= 1.5 and mean_rel <= 1.5e-2


def close_f32(got, want, what, k_len):
    """fp32 output of a bf16 x bf16 product accumulated in fp32 over k_len terms: the products are
    exact, so the only error is fp32 summation, bounded by k_len * 2^-24 * sum|terms|; held to
    1e-5 * (1 + |ref|) * sqrt(k_len), far above that and far below one bf16 ulp."""
    got = got.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - want)
    tol = 1e-5 * np.sqrt(k_len) * (1.0 + np.abs(want))
    print(f"   {what}: max-abs {float(err.max()):.2e} (|ref| up to {float(np.abs(want).max()):.1f}), "
          f"worst err/bound {float((err / tol).max()):.2f}", flush=True)
    assert (err <= tol).all(), what


def check_bwd(seed, B, N, H, E, **kw):
    from paper_2109_04312_amd import mate
    print(f"projection backward B={B} N={N} H={H} E={E} {kw}", flush=True)
    x, w_qkv, _, w_o, _, flags, o = make(seed, B, N, H, E, **kw)
    rng = np.random.default_rng(seed + 1000)
    dq, dk, dv = (bf16(rng.standard_normal((B, H, N, 64))) for _ in range(3))
    dy = bf16(rng.standard_normal((B, N, E)))
    fl = torch.from_numpy(flags).cuda()
    n_tok = max(1, int((flags != P).sum()))
    # --- QKV projection ---
    dx, dw, db = mate.qkv_project_bwd(dev(x), dev(w_qkv), fl, dev(dq), dev(dk), dev(dv))
    torch.cuda.synchronize()
    rx, rw, rb = orc.project_qkv_backward(x, w_qkv, flags, dq, dk, dv, H)
    close(dx, rx, "dx")
    assert bool((dx.float().cpu().numpy()[flags == P] == 0).all())
    close_f32(dw, rw, "dw_qkv", n_tok)
    close_f32(db, rb, "dbias_qkv", n_tok)
    # --- output projection ---
    d_o, dwo, dbo = mate.out_project_bwd(dev(o), dev(w_o), fl, dev(dy))
    torch.cuda.synchronize()
    ro, rwo, rbo = orc.project_out_backward(o, w_o, flags, dy)
    close(d_o, ro, "d_o")
    assert bool((d_o.float().cpu().numpy()[np.broadcast_to((flags == P)[:, None, :, None], ro.shape)] == 0).all())
    close_f32(dwo, rwo, "dw_o", n_tok)
    close_f32(dbo, rbo, "dbias_o", n_tok)


@pytest.mark.parametrize("N", [1, 63, 64, 65, 200, 333])
def test_backward_small_ragged(N):
    check_bwd(N, 2, N, 2, 128)


def test_backward_padding_only_blocks_and_scattered_pads():
    check_bwd(1, 3, 700, 4, 256, pad_tail=300)
    check_bwd(2, 1, 512, 2, 128, pad_tail=512, scattered_pads=False)       # nothing but padding: all zero


def test_backward_bert_base_and_large_shapes():
    check_bwd(3, 4, 512, 12, 768, pad_tail=100)
    check_bwd(5, 9, 1000, 12, 768, pad_tail=120)


def test_backward_headline_shape():
    check_bwd(4, 2, 8192, 16, 1024, pad_tail=1700, scattered_pads=False)


def test_backward_is_bit_reproducible_and_honours_null_outputs():
    from paper_2109_04312_amd import mate
    x, w_qkv, _, w_o, _, flags, o = make(7, 3, 900, 4, 256, pad_tail=77)
    rng = np.random.default_rng(77)
    dq, dk, dv = (dev(bf16(rng.standard_normal((3, 4, 900, 64)))) for _ in range(3))
    fl = torch.from_numpy(flags).cuda()
    a = mate.qkv_project_bwd(dev(x), dev(w_qkv), fl, dq, dk, dv)
    b = mate.qkv_project_bwd(dev(x), dev(w_qkv), fl, dq, dk, dv)
    only_dx = mate.qkv_project_bwd(dev(x), dev(w_qkv), fl, dq, dk, dv, want_dw=False, want_dbias=False)
    only_dw = mate.qkv_project_bwd(dev(x), dev(w_qkv), fl, dq, dk, dv, want_dx=False, want_dbias=False)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    assert torch.equal(only_dx[0], a[0]) and only_dx[1] is None and only_dx[2] is None
    assert only_dw[0] is None and torch.equal(only_dw[1], a[1])
    with pytest.raises(mate.MateError) as e:        # a bias gradient without the weight gradient
        mate.qkv_project_bwd(dev(x), dev(w_qkv), fl, dq, dk, dv, want_dw=False)
    assert e.value.status == mate.MATE_ERR_NULL


def test_layer_forward_backward_end_to_end():
    """x -> QKV projection -> attention -> output projection and all the way back (d y -> d o ->
    dq, dk, dv -> dx, plus the weight gradients), every step in the library, against the same
    chain in the oracle in float64.  Five bf16 roundings lie on the way to dx, so the bound is
    a multiple of a single step's."""
    from paper_2109_04312_amd import mate
    w = synth.make_config(2, tensors=False)
    st = w.structure
    B, N, H, E = st.B, st.N, 12, 768
    rng = np.random.default_rng(19)
    x = bf16(rng.standard_normal((B, N, E)))
    w_qkv = bf16(rng.standard_normal((3 * H * 64, E)) / np.sqrt(E))
    w_o = bf16(rng.standard_normal((E, H * 64)) / np.sqrt(H * 64))
    dy = bf16(rng.standard_normal((B, N, E)))
    hk = synth.half_row_half_col(H)
    r, c, f = hp.dev_structure(st)
    q, k, v = mate.qkv_project(dev(x), dev(w_qkv), None, f, H)
    seg = mate.build_segments(r, c, f)
    o, lse = mate.attn_fwd(q, k, v, seg, hk, 0.125)
    d_o, dwo, _ = mate.out_project_bwd(o, dev(w_o), f, dev(dy), want_dbias=False)
    dq, dk, dv = mate.attn_bwd(q, k, v, o, lse, d_o, seg, hk, 0.125)
    dx, dwq, _ = mate.qkv_project_bwd(dev(x), dev(w_qkv), f, dq, dk, dv, want_dbias=False)
    torch.cuda.synchronize()
    # the oracle chain on two sequences (weight gradients sum over the batch: compare dx per sequence,
    # and the weight gradients of a two-sequence batch computed separately below)
    for b in (0, 17):
        sl = slice(b, b + 1)
        qr, kr, vr = orc.project_qkv(x[sl], w_qkv, None, st.flags[sl], H)
        args = (st.row_ids[sl], st.col_ids[sl], st.flags[sl], hk, 0.125)
        orf, _ = orc.attn_forward(qr, kr, vr, *args)
        dor, _, _ = orc.project_out_backward(orf, w_o, st.flags[sl], dy[sl])
        dqr, dkr, dvr = orc.attn_backward(qr, kr, vr, dor, *args)
        dxr, _, _ = orc.project_qkv_backward(x[sl], w_qkv, st.flags[sl], dqr, dkr, dvr, H)
        got = dx[sl].float().cpu().numpy().astype(np.float64)
        err = np.abs(got - dxr)
        ratio = float((err / hp.bound("projection", dxr, "bf16")).max())
        mean_rel = float(err.mean() / (np.abs(dxr).mean() + 1e-3))
        print(f"   layer dx b={b}: max-abs {float(err.max()):.2e} = {ratio:.2f} x one step's bound, "
              f"mean-rel {mean_rel:.2e}", flush=True)
        assert ratio <= 2.0 and mean_rel <= 2e-2


def test_unsupported_arguments():
    from paper_2109_04312_amd import mate
    x, w_qkv, b_qkv, w_o, b_o, flags, o = make(0, 1, 64, 3, 128, bias=False)
    with pytest.raises(mate.MateError) as e:        # odd number of heads
        mate.qkv_project(dev(x), dev(w_qkv), None, torch.from_numpy(flags).cuda(), 3)
    assert e.value.status == mate.MATE_ERR_UNSUPPORTED
    x, w_qkv, b_qkv, w_o, b_o, flags, o = make(0, 1, 64, 2, 192, bias=False)
    with pytest.raises(mate.MateError) as e:        # width not a multiple of 128
        mate.out_project(dev(o), dev(w_o), None, torch.from_numpy(flags).cuda())
    assert e.value.status == mate.MATE_ERR_UNSUPPORTED
