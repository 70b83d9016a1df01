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


def useful_pairs_per_view(st):
    """[B,2] useful (query,key) pairs per sequence for a row head / a column head:
    L*G + sum_i s_i^2 + G*T  (table->question, table->own segment, question->all)."""
    from paper_2109_04312_amd import synth
    out = np.zeros((st.B, 2), np.int64)
    for b in range(st.B):
        f = st.flags[b]
        G = int((f == synth.TOK_GLOBAL).sum())
        Lc = int((f == synth.TOK_LOCAL).sum())
        for v, ids in enumerate((st.row_ids[b], st.col_ids[b])):
            _, s = np.unique(ids[f == synth.TOK_LOCAL], return_counts=True)
            out[b, v] = Lc * G + int((s.astype(np.int64) ** 2).sum()) + G * (G + Lc)
    return out


def cpu_baseline(w, pairs, total_heads):
    """Times the oracle (as it stands) on a few (b,h) pairs; scales to the whole batch."""
    from oracle import mate_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    st = w.structure
    t0 = time.perf_counter()
    for b, h in pairs:
        sl = (slice(b, b + 1), slice(h, h + 1))
        args = (st.row_ids[b:b + 1], st.col_ids[b:b + 1], st.flags[b:b + 1], w.head_kind[h:h + 1], w.scale)
        orc.attn_forward(w.q[sl], w.k[sl], w.v[sl], *args)
        orc.attn_backward(w.q[sl], w.k[sl], w.v[sl], w.do[sl], *args)
    dt = time.perf_counter() - t0
    B, H, N, _ = w.shape
    est = dt * total_heads / len(pairs)
    return dict(value=B * N / est, unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"fwd+bwd of {len(pairs)} of {total_heads} (sequence, head) pairs "
                       f"{pairs} of the same batch in {dt:.1f} s, scaled by {total_heads}/{len(pairs)}; "
                       "segment tables not included")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration (default: headline 4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2109_04312_amd import mate, synth

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

    def step(ev=None):
        if ev: ev[0].record()
        mate.build_segments(row, col, flg, out=seg)
        if ev: ev[1].record()
        mate.attn_fwd(q, k, v, seg, hk, w.scale, out=out, lse=lse, ws=ws_f)
        if ev: ev[2].record()
        mate.attn_bwd(q, k, v, out, lse, do, seg, hk, w.scale, dq=dq, dk=dk, dv=dv, ws=ws_b)
        if ev: ev[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    # second pass of the same loop with HIP events between the calls (current stream = the
    # stream the kernels run on): per-call device time
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for e in evs:
        step(e)
    torch.cuda.synchronize()
    t_build = float(np.mean([e[0].elapsed_time(e[1]) for e in evs])) * 1e-3
    t_fwd = float(np.mean([e[1].elapsed_time(e[2]) for e in evs])) * 1e-3
    t_bwd = float(np.mean([e[2].elapsed_time(e[3]) for e in evs])) * 1e-3

    pv = useful_pairs_per_view(st)
    pairs = int(sum(pv[b, int(hk[h])] for b in range(B) for h in range(H)))
    tokens = B * N
    nonpad = int((st.flags != synth.TOK_PAD).sum())
    value = tokens / (elapsed / args.steps)
    fl_fwd, fl_bwd = 4 * D * pairs, 10 * D * pairs
    cand = {"mate_attn_fwd": (fl_fwd, t_fwd), "mate_attn_bwd": (fl_bwd, t_bwd)}
    dom = max(cand, key=lambda n: cand[n][1])
    ach = cand[dom][0] / cand[dom][1] / 1e12

    res = {
        "metric": "MATE attn fwd+bwd tokens/s & useful-pair TFLOP/s, seq 8192, 16 heads, 1 GPU",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": B, "N": N, "H": H, "D": D, "row_heads": int((hk == 0).sum()),
                   "col_heads": int((hk == 1).sum()), "non_pad_tokens": nonpad, "useful_pairs": pairs,
                   "step": "mate_build_segments + mate_attn_fwd + mate_attn_bwd"},
        "useful_tflops": 14 * D * pairs / (elapsed / args.steps) / 1e12,
        "useful_tflops_attn_only": 14 * D * pairs / (t_fwd + t_bwd) / 1e12,
        "tokens_per_s_attn_only": tokens / (t_fwd + t_bwd),
        "device_ms": {"build_segments": t_build * 1e3, "attn_fwd": t_fwd * 1e3, "attn_bwd": t_bwd * 1e3},
        "flop_convention": "fwd 4*D, bwd 10*D flop per useful (query,key) pair; exp not counted",
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None},
        "segment_builder": {"us": t_build * 1e6, "keys_per_s": 2 * tokens / t_build,
                            "algorithmic_GBps": 30.0 * tokens / t_build / 1e9,
                            "frac_hbm": 30.0 * tokens / t_build / 1e9 / PEAK_HBM_GBS},
    }
    if not args.no_cpu_baseline and w.do is not None:
        sample = [(0, 0), (0, H - 1)]
        res["cpu_baseline"] = cpu_baseline(w, sample, B * H)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
