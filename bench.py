#!/usr/bin/env python3
"""Benchmark of the MATE attention hot path on one MI355X.

A step is one pass of the whole path over the headline batch (B=2, N=8192, H=16: 8 row + 8
column heads, D=64, bf16, 64 question tokens, 400 x 8 table): segment build, forward,
backward, with all inputs already resident in HBM.  Prints ONE JSON line.

  value            tokens/s = B*N*steps / time of the timed region (build + fwd + bwd)
  useful_tflops    896 flop per useful (query, key) pair (fwd 4*D, bwd 10*D) / time
  roofline         dominant kernel vs the bf16 MFMA peak, from HIP-event timings taken in a
                   second pass of the same loop
  cpu_baseline     the float64 oracle on a sample of (sequence, head) pairs, scaled to the batch
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
D = 64
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0   # what a plain copy of known size reads on these counters
CSRC = os.path.join(ROOT, "paper_2109_04312_amd", "csrc")


def sources_digest():
    """sha256 over the kernel sources: a traffic figure measured on other sources is not
    reported as if it belonged to this build."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()[:16]


def traffic_summary_path(workload):
    return os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic_pmc.txt")


def read_traffic(workload):
    """HBM bytes per launch from the tracked rocprofv3 --pmc summary of this workload
    (lines `counter <kernel> <FETCH_SIZE KiB> <WRITE_SIZE KiB>` and `sources <digest>`).
    Returns ({kernel: {fetch_bytes, write_bytes}}, digest of the sources it was measured on)."""
    path = traffic_summary_path(workload)
    if not os.path.exists(path):
        return {}, None
    table, digest = {}, None
    for line in open(path):
        f = line.split()
        if len(f) == 2 and f[0] == "sources":
            digest = f[1]
        if len(f) == 4 and f[0] == "counter":
            table[f[1]] = {"fetch_bytes": int(float(f[2]) * 1024 * FETCH_SCALE),
                           "write_bytes": int(float(f[3]) * 1024 * WRITE_SCALE)}
    return table, digest


def summarize_pmc(fetch_dir, write_dir):
    """Prints the machine-readable part of profiles/<workload>_hbm_traffic_pmc.txt from the csv
    output of two `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --output-format csv` runs of this script."""
    import csv
    import glob

    def per_kernel(d, counter):
        acc = {}
        for path in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(path)):
                if row["Counter_Name"] == counter:
                    name = row["Kernel_Name"].replace("(anonymous namespace)::", "").replace("void ", "")
                    name = name.split("(")[0].replace("mate::", "")
                    acc.setdefault(name, {}).setdefault(row["Dispatch_Id"], 0.0)
                    acc[name][row["Dispatch_Id"]] += float(row["Counter_Value"])
        return {k: sum(v.values()) / len(v) for k, v in acc.items()}

    fetch, write = per_kernel(fetch_dir, "FETCH_SIZE"), per_kernel(write_dir, "WRITE_SIZE")
    print("sources", sources_digest())
    for k in sorted(fetch):
        if k.endswith("_kernel") or "_kernel<" in k:
            print("counter", k.replace(" ", ""), round(fetch[k]), round(write.get(k, 0.0)))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def useful_pairs_per_view(st, bucketed=None):
    """[B,2] useful (query,key) pairs per sequence for a row head / a column head:
    L*G + sum_i s_i^2 + G*T  (table->question, table->own segment, question->all).
    bucketed = (G, R): the question tokens past the first G count as table tokens and a table
    token meets only the part of its segment in its own and the two adjacent buckets of R
    sorted slots (Section 3.1)."""
    from paper_2109_04312_amd import synth
    out = np.zeros((st.B, 2), np.int64)
    for b in range(st.B):
        f = st.flags[b].copy()
        if bucketed is not None:
            quest = np.flatnonzero(f == synth.TOK_GLOBAL)
            f[quest[bucketed[0]:]] = synth.TOK_LOCAL
        G = int((f == synth.TOK_GLOBAL).sum())
        Lc = int((f == synth.TOK_LOCAL).sum())
        for v, ids in enumerate((st.row_ids[b], st.col_ids[b])):
            srt = np.sort(ids[f == synth.TOK_LOCAL].astype(np.int64), kind="stable")
            _, first, s = np.unique(srt, return_index=True, return_counts=True)
            lo, hi = np.repeat(first, s), np.repeat(first + s, s)     # segment range per sorted slot
            if bucketed is not None:
                j = np.arange(Lc) // bucketed[1]
                lo, hi = np.maximum(lo, (j - 1) * bucketed[1]), np.minimum(hi, (j + 2) * bucketed[1])
            out[b, v] = Lc * G + int((hi - lo).sum()) + G * (G + Lc)
    return out


def _oracle_fwd_bwd(w, pairs, bucketed=None):
    from oracle import mate_oracle as orc
    st = w.structure
    t0 = time.perf_counter()
    for b, h in pairs:
        sl = (slice(b, b + 1), slice(h, h + 1))
        args = (st.row_ids[b:b + 1], st.col_ids[b:b + 1], st.flags[b:b + 1], w.head_kind[h:h + 1], w.scale)
        orc.attn_forward(w.q[sl], w.k[sl], w.v[sl], *args, bucketed=bucketed)
        orc.attn_backward(w.q[sl], w.k[sl], w.v[sl], w.do[sl], *args, bucketed=bucketed)
    return time.perf_counter() - t0


def cpu_baseline(w, pairs, total_heads, bucketed=None):
    """Times the oracle (as it stands) on a few (b,h) pairs; scales to the whole batch.  Also the
    oracle on ONE thread on the short configuration 2 (one sequence, every head)."""
    from paper_2109_04312_amd import synth
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    dt = _oracle_fwd_bwd(w, pairs, bucketed)
    B, H, N, _ = w.shape
    est = dt * total_heads / len(pairs)
    res = dict(value=B * N / est, unit="tokens/s", cores=int(cores), kind="oracle", cpu_model=cpu_model(),
               sample=f"fwd+bwd of {len(pairs)} of {total_heads} (sequence, head) pairs "
                      f"{pairs} of the same batch in {dt:.1f} s, scaled by {total_heads}/{len(pairs)}; "
                      "segment tables not included")
    if threadpool_limits is not None:
        w2 = synth.make_config(2)
        B2, H2, N2, _ = w2.shape
        with threadpool_limits(limits=1):
            dt2 = _oracle_fwd_bwd(w2, [(0, h) for h in range(H2)])
        res["one_thread_config2"] = dict(value=B2 * N2 / (dt2 * B2), unit="tokens/s", cores=1,
                                         sample=f"{w2.name}: fwd+bwd of the {H2} heads of one of {B2} "
                                                f"sequences on one thread in {dt2:.2f} s, scaled by {B2}")
    return res


def settle(fn, seconds):
    """Untimed: repeats `fn` for a fixed wall time so that what follows is timed at settled clocks
    (the GPU ramps its clocks over tens of milliseconds).  Returns the number of calls."""
    import torch
    n, t_end = 0, time.perf_counter() + max(0.0, seconds)
    while time.perf_counter() < t_end:
        for _ in range(20):
            fn()
        n += 20
        torch.cuda.synchronize()
    return n


def breakeven(steps, warmup, lengths=(64, 128, 256, 384, 512, 768, 1024)):
    """Section 3.1 uses the faster of two equivalent implementations per sequence length: times
    both here on tables shaped like configuration 2 (B=32, H=12, 4 columns, short cells)."""
    import torch
    from paper_2109_04312_amd import mate, synth
    torch.cuda.set_device(0)
    B, H, rows = 32, 12, []
    for N in lengths:
        rng = np.random.default_rng(synth.BASE_SEED + N)
        G, C = max(4, N // 16), 4
        R = max(2, int((N - G) * 0.85 / (C * 2)))
        st = synth._stack([synth.flatten_table(N, G, R, C, synth.geometric_lengths(rng, 2.0, 8, R * C))
                           for _ in range(B)])
        q, k, v, do = (torch.from_numpy(x).to(torch.bfloat16).cuda()
                       for x in synth.draw_tensors(rng, B, H, N, D, "bf16", 4))
        r, c, f = (torch.from_numpy(x).cuda() for x in (st.row_ids, st.col_ids, st.flags))
        hk = synth.half_row_half_col(H)
        seg = mate.Segments(torch.empty(mate.mate_segments_bytes(B, N), dtype=torch.uint8, device="cuda"), B, N)
        out, lse = torch.empty_like(q), torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        ws_f = mate.workspace(B, H, N, D, mate.MATE_BF16, False, "cuda")
        ws_b = mate.workspace(B, H, N, D, mate.MATE_BF16, True, "cuda")
        ws_d = torch.empty(mate.mate_dense_workspace_bytes(B, H, N), dtype=torch.uint8, device="cuda")

        def seg_step():
            mate.build_segments(r, c, f, out=seg)
            mate.attn_fwd(q, k, v, seg, hk, 0.125, out=out, lse=lse, ws=ws_f)
            mate.attn_bwd(q, k, v, out, lse, do, seg, hk, 0.125, dq=dq, dk=dk, dv=dv, ws=ws_b)

        def dense_step():
            mate.attn_fwd_dense(q, k, v, r, c, f, hk, 0.125, out=out, lse=lse)
            mate.attn_bwd_dense(q, k, v, out, lse, do, r, c, f, hk, 0.125, dq=dq, dk=dk, dv=dv, ws=ws_d)

        t = {}
        if not rows:
            settle(seg_step, 0.3)
        for name, fn in (("segment", seg_step), ("dense", dense_step)):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            t[name] = (time.perf_counter() - t0) / steps * 1e6
        rows.append({"N": N, "segment_us": round(t["segment"], 1), "dense_us": round(t["dense"], 1),
                     "faster": min(t, key=t.get)})
    return {"breakeven": rows, "B": B, "H": H, "dtype": "bf16", "steps": steps,
            "step": "segment: build + fwd + bwd; dense: fwd + bwd"}


def projections(cfg, steps, warmup):
    """Times the projection kernels, forward and backward, on a configuration's layer shape (model
    width 64 * H) with HIP events recorded by the library around each launch."""
    import ctypes as C
    import torch
    from paper_2109_04312_amd import mate, synth
    torch.cuda.set_device(0)
    w = synth.make_config(cfg, tensors=False)
    st = w.structure
    B, N, H = st.B, st.N, len(w.head_kind)
    E = 64 * H
    g = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED)
    x = torch.randn((B, N, E), device="cuda", generator=g).to(torch.bfloat16)
    w_qkv = (torch.randn((3 * E, E), device="cuda", generator=g) / E ** 0.5).to(torch.bfloat16)
    w_o = (torch.randn((E, E), device="cuda", generator=g) / E ** 0.5).to(torch.bfloat16)
    b_qkv = torch.randn(3 * E, device="cuda", generator=g)
    b_o = torch.randn(E, device="cuda", generator=g)
    fl = torch.from_numpy(st.flags).cuda()
    q, k, v = (torch.empty((B, H, N, 64), dtype=torch.bfloat16, device="cuda") for _ in range(3))
    y = torch.empty((B, N, E), dtype=torch.bfloat16, device="cuda")
    dy = torch.randn((B, N, E), device="cuda", generator=g).to(torch.bfloat16)
    ws = mate.project_bwd_workspace(B, N, H, E, "cuda")
    hip = C.CDLL("libamdhip64.so")

    def new_event():
        ev = C.c_void_p()
        assert hip.hipEventCreate(C.byref(ev)) == 0
        return ev

    def step():
        mate.qkv_project(x, w_qkv, b_qkv, fl, H, q=q, k=k, v=v)
        mate.out_project(q, w_o, b_o, fl, y=y)

    def step_bwd():   # gradients of the same two calls (q, k, v stand in for dq, dk, dv and for o)
        mate.out_project_bwd(q, w_o, fl, dy, ws=ws)
        mate.qkv_project_bwd(x, w_qkv, fl, q, k, v, ws=ws)

    def wall(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    settle(step, 0.3)
    stream = C.c_void_p(mate._stream())
    both, both_bwd = wall(step), wall(step_bwd)
    res = {}
    for name, kid, fn in (("qkv_project", mate.MATE_KERNEL_QKV_PROJECT, step),
                          ("out_project", mate.MATE_KERNEL_OUT_PROJECT, step),
                          ("qkv_project_dgrad", mate.MATE_KERNEL_QKV_PROJECT_DGRAD, step_bwd),
                          ("qkv_project_wgrad", mate.MATE_KERNEL_QKV_PROJECT_WGRAD, step_bwd),
                          ("out_project_dgrad", mate.MATE_KERNEL_OUT_PROJECT_DGRAD, step_bwd),
                          ("out_project_wgrad", mate.MATE_KERNEL_OUT_PROJECT_WGRAD, step_bwd)):
        evs = [(new_event(), new_event()) for _ in range(steps)]
        empty = [(new_event(), new_event()) for _ in range(steps)]
        for (e0, e1), (a0, a1) in zip(evs, empty):
            assert mate.mate_profile_kernel(kid, e0, e1) == 0
            fn()
            # an event pair with nothing in it: what a bracket reads beyond the kernel (see main())
            assert hip.hipEventRecord(a0, stream) == 0 and hip.hipEventRecord(a1, stream) == 0
        torch.cuda.synchronize()

        def median_s(pairs):
            out = []
            for e0, e1 in pairs:
                ms = C.c_float()
                assert hip.hipEventElapsedTime(C.byref(ms), e0, e1) == 0
                out.append(ms.value * 1e-3)
            return sorted(out)[len(out) // 2]

        res[name] = median_s(evs) - median_s(empty)
    nonpad = int((st.flags != synth.TOK_PAD).sum())
    big, small = 2.0 * nonpad * E * 3 * E, 2.0 * nonpad * E * E
    flop = {"qkv_project": big, "out_project": small, "qkv_project_dgrad": big, "qkv_project_wgrad": big,
            "out_project_dgrad": small, "out_project_wgrad": small}
    out = {"projections": {n: {"median_us": t * 1e6, "algorithmic_flop": flop[n], "achieved_tflops": flop[n] / t / 1e12,
                               "frac_of_bf16_mfma_peak": flop[n] / t / 1e12 / PEAK_BF16_TFLOPS} for n, t in res.items()},
           "workload": w.name, "B": B, "N": N, "H": H, "E": E, "non_pad_tokens": nonpad, "dtype": "bf16",
           "us_forward_wall": both * 1e6, "us_backward_wall": both_bwd * 1e6, "steps": steps,
           "backward_wall_includes": "weight transposes and pad masks (preparation kernel), partial-sum finalize kernels",
           "flop_convention": "2 * non-pad tokens * K * F per product (pad rows are not algorithmic work)",
           "timing": "median of HIP event brackets recorded by the library around each launch, minus the median "
                     "of event pairs with nothing between their records"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-s", type=float, default=0.3,
                    help="seconds of untimed steps before the warm-up steps, so that a short run is timed at "
                         "the clocks of a long one (the GPU ramps its clocks over tens of milliseconds; 0 = none)")
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration (default: headline 4)")
    ap.add_argument("--bucketed", default=None, metavar="G,R",
                    help="bucketed mode of Section 3.1 (the published models use 116,42)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the short runs of the other modes (bucketed tables, projections, break-even) "
                         "that the default line carries under `extras`")
    ap.add_argument("--plain", action="store_true",
                    help="for profiler runs: the warm-up, the timed steps and the per-kernel event pass of the "
                         "chosen configuration, every launch the same shape (no per-head-kind runs, no peak "
                         "probes, no CPU baseline)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 256 MiB device copy three times (to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc) and exit")
    ap.add_argument("--breakeven", action="store_true",
                    help="only time the segment path (build + fwd + bwd) against the dense-mask "
                         "entry points (fwd + bwd) at short sequence lengths and exit")
    ap.add_argument("--summarize-pmc", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"), default=None,
                    help="print the machine-readable part of profiles/<workload>_hbm_traffic_pmc.txt from the "
                         "csv output directories of two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE); no GPU needed")
    ap.add_argument("--projections", action="store_true",
                    help="time the QKV and output projection kernels on the configuration's layer shape and exit")
    args = ap.parse_args()
    if args.summarize_pmc:
        summarize_pmc(*args.summarize_pmc)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2109_04312_amd import mate, synth

    if args.calibrate_copy:
        torch.cuda.set_device(0)
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_each_way": src.numel() * 4}))
        return

    if args.breakeven:
        print(json.dumps(breakeven(args.steps, args.warmup)))
        return

    if args.projections:
        print(json.dumps(projections(args.config, args.steps, args.warmup)))
        return

    w = synth.make_config(args.config)
    B, H, N, _ = w.shape
    st = w.structure
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    dev = "cuda:0"
    torch.cuda.set_device(0)
    q, k, v = (torch.from_numpy(x).to(dt).to(dev) for x in (w.q, w.k, w.v))
    do = torch.from_numpy(w.do if w.do is not None else w.q).to(dt).to(dev)
    row, col, flg = (torch.from_numpy(x).to(dev) for x in (st.row_ids, st.col_ids, st.flags))
    code = mate.MATE_BF16 if w.dtype == "bf16" else mate.MATE_F32
    seg = mate.Segments(torch.empty(mate.mate_segments_bytes(B, N), dtype=torch.uint8, device=dev), B, N)
    out, lse = torch.empty_like(q), torch.empty((B, H, N), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    ws_f = mate.workspace(B, H, N, D, code, False, dev)
    ws_b = mate.workspace(B, H, N, D, code, True, dev)
    hk = w.head_kind

    bucketed = tuple(int(x) for x in args.bucketed.split(",")) if args.bucketed else None

    def step():
        mate.build_segments(row, col, flg, out=seg, bucketed=bucketed)
        mate.attn_fwd(q, k, v, seg, hk, w.scale, out=out, lse=lse, ws=ws_f)
        mate.attn_bwd(q, k, v, out, lse, do, seg, hk, w.scale, dq=dq, dk=dk, dv=dv, ws=ws_b)

    # untimed: the same step repeated for a fixed wall time, until the clocks have settled (a run of
    # 20 steps lasts 5 ms, and without this it reads 15-20 % slower than a run of 200), then the
    # requested warm-up steps
    settle_steps = settle(step, args.settle_s)
    for _ in range(args.warmup):
        step()
    # the timed region: exactly `steps` steps between two synchronisations; an event every
    # `block` steps on the stream the kernels run on gives the spread inside it
    block = max(1, args.steps // 20)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps // block + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        if (i + 1) % block == 0:
            marks[(i + 1) // block].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    block_ms = sorted(marks[i].elapsed_time(marks[i + 1]) / block for i in range(len(marks) - 1))
    ms_median, ms_min = block_ms[len(block_ms) // 2], block_ms[0]

    # second pass of the same loop: HIP events recorded by the library around ONE kernel launch
    # per step (on the stream the kernels run on), cycling through the kernels
    import ctypes as C
    hip = C.CDLL("libamdhip64.so")
    def new_event():
        ev = C.c_void_p()
        assert hip.hipEventCreate(C.byref(ev)) == 0
        return ev
    kernels = {"build_segments": mate.MATE_KERNEL_BUILD, "attn_fwd": mate.MATE_KERNEL_FWD,
               "attn_bwd_dq": mate.MATE_KERNEL_BWD_DQ, "attn_bwd_dkv": mate.MATE_KERNEL_BWD_DKV}
    per_kernel = max(10, args.steps // len(kernels))
    pairs_ev = {name: [(new_event(), new_event()) for _ in range(per_kernel)] for name in kernels}
    # An event pair with NOTHING between its two records reads about 5 us on this hardware (what the
    # command processor spends on the two event packets), and a pair around a kernel reads the
    # kernel plus that.  One empty pair per profiled step, recorded on the same stream between two
    # steps, measures it; it is subtracted from every bracket.
    empty_ev = [(new_event(), new_event()) for _ in range(per_kernel * len(kernels))]
    stream = C.c_void_p(mate._stream())
    t1 = time.perf_counter()
    for i in range(per_kernel):
        for j, (name, kid) in enumerate(kernels.items()):
            e0, e1 = pairs_ev[name][i]
            assert mate.mate_profile_kernel(kid, e0, e1) == 0
            step()
            a0, a1 = empty_ev[i * len(kernels) + j]
            assert hip.hipEventRecord(a0, stream) == 0 and hip.hipEventRecord(a1, stream) == 0
    torch.cuda.synchronize()
    ms_per_step_pass2 = 1e3 * (time.perf_counter() - t1) / (per_kernel * len(kernels))

    def elapsed_s(e0, e1):
        ms = C.c_float()
        assert hip.hipEventElapsedTime(C.byref(ms), e0, e1) == 0
        return ms.value * 1e-3

    empties = sorted(elapsed_s(a0, a1) for a0, a1 in empty_ev)
    bracket_s = empties[len(empties) // 2]
    kernel_s, kernel_median_s, kernel_min_s, kernel_raw_s = {}, {}, {}, {}
    for name in kernels:
        samples = sorted(elapsed_s(e0, e1) for e0, e1 in pairs_ev[name])
        kernel_raw_s[name] = sum(samples) / len(samples)
        kernel_s[name] = kernel_raw_s[name] - bracket_s
        kernel_median_s[name] = samples[len(samples) // 2] - bracket_s
        kernel_min_s[name] = samples[0] - bracket_s
    if args.plain:
        print(json.dumps({"plain": True, "workload": w.name, "steps": args.steps, "settle_steps": settle_steps,
                          "ms_per_step": ms_per_step,
                          "ms_per_step_median": ms_median, "ms_per_step_min": ms_min,
                          "event_bracket_overhead_us": 1e6 * bracket_s,
                          "kernel_us_hip_events": {n: {"avg": 1e6 * kernel_s[n], "median": 1e6 * kernel_median_s[n],
                                                       "min": 1e6 * kernel_min_s[n],
                                                       "avg_before_subtracting_the_bracket": 1e6 * kernel_raw_s[n],
                                                       "launches": per_kernel}
                                                   for n in kernels}}))
        return
    t_build, t_fwd = kernel_s["build_segments"], kernel_s["attn_fwd"]
    t_dq, t_dkv = kernel_s["attn_bwd_dq"], kernel_s["attn_bwd_dkv"]

    pv = useful_pairs_per_view(st, bucketed)
    pairs = int(sum(pv[b, int(hk[h])] for b in range(B) for h in range(H)))
    tokens = B * N
    nonpad_b = (st.flags != synth.TOK_PAD).sum(axis=1)
    nonpad = int(nonpad_b.sum())
    value = tokens / (elapsed / args.steps)
    # algorithmic flop per useful pair: forward 4*D (QK^T, PV); backward 10*D, of which the dQ
    # kernel is credited S, dP and dQ (6*D) and the dK/dV kernel dV and dK (4*D) -- its own
    # recomputation of S and dP is not algorithmic work
    cand = {"fwd_mfma_kernel": (4 * D * pairs, t_fwd), "bwd_dq_mfma_kernel": (6 * D * pairs, t_dq),
            "bwd_dkv_mfma_kernel": (4 * D * pairs, t_dkv)}
    dom = max(cand, key=lambda n: cand[n][1])
    ach = cand[dom][0] / cand[dom][1] / 1e12
    # the same kernel against the HBM roof: tensor passes it would need as a stand-alone kernel
    # (128 B per non-pad token row per head per pass)
    passes = {"fwd_mfma_kernel": 4, "bwd_dq_mfma_kernel": 6, "bwd_dkv_mfma_kernel": 6}[dom]
    alg_bytes = passes * 128 * nonpad * H
    hbm_gbs = alg_bytes / cand[dom][1] / 1e9
    t_attn = ms_per_step * 1e-3 - t_build

    # HBM traffic of the dominant kernel: from the tracked rocprofv3 --pmc summary of this
    # workload, reported only if it was measured on the kernel sources this run was built from
    table, digest = ({}, None) if bucketed else read_traffic(w.name)
    fresh = digest is not None and digest == sources_digest()
    traffic_detail = None
    if dom in table:
        traffic_detail = dict(table[dom], unit="HBM bytes per launch", profiled_on_sources=digest,
                              matches_this_build=fresh,
                              source=os.path.relpath(traffic_summary_path(w.name), ROOT)
                                     + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy)")
    traffic = table[dom]["fetch_bytes"] + table[dom]["write_bytes"] if (dom in table and fresh) else None

    # ---- the box's own peaks, measured in this process -----------------------------------------
    sink = torch.empty(2048 * 256, dtype=torch.float32, device=dev)
    flop = C.c_double()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    mate.mate_probe_mfma(sink.data_ptr(), sink.numel() * 4, 2048, 100, C.byref(flop), mate._stream())  # warm-up
    ev[0].record()
    assert mate.mate_probe_mfma(sink.data_ptr(), sink.numel() * 4, 2048, 600, C.byref(flop), mate._stream()) == 0
    ev[1].record()
    src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev[2].record()
    for _ in range(5):
        dst.copy_(src)
    ev[3].record()
    torch.cuda.synchronize()
    mfma_tflops = flop.value / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e12
    copy_gbs = 5 * 2 * src.numel() * 4 / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e9
    del src, dst, sink
    peaks_measured = {"mfma_bf16_tflops": mfma_tflops, "mfma_frac_of_nominal": mfma_tflops / PEAK_BF16_TFLOPS,
                      "mfma_probe": "2048 workgroups x 4 wavefronts x 600 x 8 independent 32x32x16 bf16 MFMAs",
                      "copy_gbs": copy_gbs, "copy_frac_of_nominal": copy_gbs / PEAK_HBM_GBS,
                      "copy_probe": "256 MiB device-to-device copy x 5, read + write bytes"}

    # ---- combined roofline: every (sequence, head) against the roof that binds it ----------------
    # flop_h = 896 * useful pairs, bytes_h = 12 tensor passes * 128 B * non-pad tokens (+ 12 B of
    # LSE / delta per token);  t_bound = sum_h max(flop_h / peak, bytes_h / bandwidth)
    def t_bound(kinds, peak_tflops, bw_gbs):
        t = 0.0
        for b in range(B):
            for h in range(H):
                if int(hk[h]) in kinds:
                    fl = 14 * D * int(pv[b, int(hk[h])])
                    by = (12 * 128 + 12) * int(nonpad_b[b])
                    t += max(fl / (peak_tflops * 1e12), by / (bw_gbs * 1e9))
        return t

    # ---- per head kind: the same tensors restricted to the row heads / the column heads ----------
    per_kind = {}
    if w.do is not None and not bucketed:
        for kind, label in ((0, "row_heads"), (1, "col_heads")):
            sel = [h for h in range(H) if int(hk[h]) == kind]
            if not sel:
                continue
            qs, ks, vs, dos = (t[:, sel].contiguous() for t in (q, k, v, do))
            Hs = len(sel)
            hks = np.full(Hs, kind, np.uint8)
            outs, lses = torch.empty_like(qs), torch.empty((B, Hs, N), dtype=torch.float32, device=dev)
            g = [torch.empty_like(qs) for _ in range(3)]
            wf = mate.workspace(B, Hs, N, D, code, False, dev)
            wb = mate.workspace(B, Hs, N, D, code, True, dev)

            def kind_step():
                mate.attn_fwd(qs, ks, vs, seg, hks, w.scale, out=outs, lse=lses, ws=wf)
                mate.attn_bwd(qs, ks, vs, outs, lses, dos, seg, hks, w.scale, dq=g[0], dk=g[1], dv=g[2], ws=wb)

            n_k = max(10, args.steps // 4)
            for _ in range(5):
                kind_step()
            torch.cuda.synchronize()
            tk = time.perf_counter()
            for _ in range(n_k):
                kind_step()
            torch.cuda.synchronize()
            t_kind = (time.perf_counter() - tk) / n_k
            tb = t_bound({kind}, PEAK_BF16_TFLOPS, PEAK_HBM_GBS)
            kp = int(sum(pv[b, kind] for b in range(B)) * Hs)
            per_kind[label] = {"heads": Hs, "ms_fwd_bwd": t_kind * 1e3, "useful_pairs": kp,
                               "useful_tflops": 14 * D * kp / t_kind / 1e12,
                               "t_bound_us": tb * 1e6, "frac_of_bound": tb / t_kind,
                               "bound": "mfma" if 14 * D * kp / (PEAK_BF16_TFLOPS * 1e12) > (12 * 128 + 12) * nonpad * Hs / (PEAK_HBM_GBS * 1e9) else "hbm"}
            del qs, ks, vs, dos, outs, lses, g, wf, wb

    tb_nom = t_bound({0, 1}, PEAK_BF16_TFLOPS, PEAK_HBM_GBS)
    tb_meas = t_bound({0, 1}, mfma_tflops, copy_gbs)
    combined = {"t_bound_us": tb_nom * 1e6, "frac_of_attn_time": tb_nom / t_attn,
                "t_bound_us_measured_peaks": tb_meas * 1e6, "frac_of_attn_time_measured_peaks": tb_meas / t_attn,
                "definition": "sum over (sequence, head) of max(896 * useful pairs / MFMA peak, "
                              "1548 B * non-pad tokens / HBM bandwidth), over the time of forward + backward"}

    res = {
        "metric": "MATE attn fwd+bwd tokens/s & useful-pair TFLOP/s, seq 8192, 16 heads, 1 GPU",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + (f"_bucketed_G{bucketed[0]}_R{bucketed[1]}" if bucketed else ""), "B": B, "N": N, "H": H, "D": D, "row_heads": int((hk == 0).sum()),
                   "col_heads": int((hk == 1).sum()), "non_pad_tokens": nonpad, "useful_pairs": pairs,
                   "step": ("mate_build_segments_bucketed" if bucketed else "mate_build_segments")
                           + " + mate_attn_fwd + mate_attn_bwd"},
        "untimed_before_warmup": {"settle_s": args.settle_s, "steps": settle_steps,
                                  "why": "the same step repeated until the clocks have settled, so that a short "
                                         "run reads like a long one; not part of the timed region"},
        "ms_per_step_median": ms_median, "ms_per_step_min": ms_min,
        "ms_per_step_spread": f"median and min over blocks of {block} consecutive steps of the timed region (HIP events)",
        "non_pad_tokens_per_s": nonpad / (elapsed / args.steps),
        "useful_tflops": 14 * D * pairs / (elapsed / args.steps) / 1e12,
        "useful_tflops_attn_only": 14 * D * pairs / t_attn / 1e12,
        "tokens_per_s_attn_only": tokens / t_attn,
        "kernel_ms": {k: v * 1e3 for k, v in kernel_s.items()},
        "kernel_ms_events_before_subtracting_the_bracket": {k: v * 1e3 for k, v in kernel_raw_s.items()},
        "event_bracket_overhead_us": {"value": bracket_s * 1e6,
                                      "what": "median of event pairs with nothing between their two records, one "
                                              "per profiled step on the same stream; subtracted from every "
                                              "per-kernel bracket, so that kernel_ms is the kernel alone (what a "
                                              "kernel trace shows)"},
        "kernel_ms_median": {k: v * 1e3 for k, v in kernel_median_s.items()},
        "kernel_ms_min": {k: v * 1e3 for k, v in kernel_min_s.items()},
        "ms_per_step_event_pass": ms_per_step_pass2,
        "flop_convention": "fwd 4*D, bwd 10*D flop per useful (query,key) pair; exp not counted",
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_detail": traffic_detail,
                     "frac_of_measured_peak": ach / mfma_tflops,
                     "limiter": "the kernel is a dense contraction, so it is priced against the matrix peak; what "
                                "limits it today is SIMD issue time (vector ALU + matrix instructions taking turns) "
                                "and per-unit latency, see profiles/" + w.name + "_sq_counters_pmc.txt",
                     "algorithmic_flop_per_launch": cand[dom][0],
                     "avg_launch_us": cand[dom][1] * 1e6, "median_launch_us": kernel_median_s[{"fwd_mfma_kernel": "attn_fwd", "bwd_dq_mfma_kernel": "attn_bwd_dq", "bwd_dkv_mfma_kernel": "attn_bwd_dkv"}[dom]] * 1e6,
                     "hbm_view": {"algorithmic_bytes_per_launch": alg_bytes, "achieved": hbm_gbs,
                                  "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": hbm_gbs / PEAK_HBM_GBS}},
        "combined_roofline": combined,
        "per_kind": per_kind,
        "peaks_measured": peaks_measured,
        "segment_builder": {"us": t_build * 1e6, "keys_per_s": 2 * tokens / t_build,
                            "algorithmic_GBps": 30.0 * tokens / t_build / 1e9,
                            "frac_hbm": 30.0 * tokens / t_build / 1e9 / PEAK_HBM_GBS},
    }
    if not args.no_extras and not bucketed and args.config == 4:
        # the other measured modes in short form, so that one default run shows them all
        # (`--bucketed`, `--projections` and `--breakeven` give the full versions)
        def ms_of(fn, n=50):
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t0) / n

        def bucketed_step():
            mate.build_segments(row, col, flg, out=seg, bucketed=(116, 42))
            mate.attn_fwd(q, k, v, seg, hk, w.scale, out=out, lse=lse, ws=ws_f)
            mate.attn_bwd(q, k, v, out, lse, do, seg, hk, w.scale, dq=dq, dk=dk, dv=dv, ws=ws_b)

        pj = projections(args.config, 30, 5)
        res["extras"] = {
            "bucketed_G116_R42": {"ms_per_step": ms_of(bucketed_step),
                                  "useful_pairs": int(sum(useful_pairs_per_view(st, (116, 42))[b, int(hk[h])]
                                                          for b in range(B) for h in range(H))),
                                  "step": "mate_build_segments_bucketed + mate_attn_fwd + mate_attn_bwd, same batch"},
            "projections": {"us_and_frac_of_bf16_peak": {n: [round(v["median_us"], 1), round(v["frac_of_bf16_mfma_peak"], 3)]
                                                         for n, v in pj["projections"].items()},
                            "shape": f"{B * N} tokens ({pj['non_pad_tokens']} non-pad) x {pj['E']} -> 3 x {pj['E']} and "
                                     f"{pj['E']} -> {pj['E']}, flop counted on non-pad tokens"},
            "breakeven": breakeven(50, 10, lengths=(128, 256, 384, 512)),
        }
    if not args.no_cpu_baseline and w.do is not None:
        # equal numbers of row and column heads, every sequence: about 10-30 s of CPU work
        rows_h = [h for h in range(H) if hk[h] == 0][:2]
        cols_h = [h for h in range(H) if hk[h] == 1][:2]
        sample = [(b, h) for b in range(min(B, 2)) for h in rows_h + cols_h]
        res["cpu_baseline"] = cpu_baseline(w, sample, B * H, bucketed)
    print(json.dumps(res))

if __name__ == "__main__":
    main()
