#!/usr/bin/env python3
"""Benchmark of the FCP rank-local attention hot path on one MI355X.

A "step" is one pass of the whole path for the reported rank of the workload:
  fcp_attn_fwd_step_direct (all ring steps) -> fcp_lse_merge_direct -> fcp_attn_bwd_delta ->
  fcp_attn_bwd_step_direct (all ring steps) -> fcp_grad_finalize_direct
(--forward partial: fcp_attn_fwd_step -> fcp_lse_merge;  --backward accumulate: zero grads -> fcp_attn_bwd_delta ->
fcp_attn_bwd_step -> fcp_grad_finalize x3),
with every input already resident in HBM.  The metric is causal-effective TFLOP/s:
14 * pairs * head_dim * hq / time (4 forward + 10 backward flops per visible pair, channel
and head; masked pairs are not counted).  --mask mixed times the same path through the
*_mixed entry points on the workload with synthetic image spans (not the headline number).

Prints ONE JSON line (see the keys below); `roofline` is for the dominant kernel (the
backward step), `cpu_baseline` times the fp64 CPU oracle on a bounded sample of the same
workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA: 256 CU x 4 SIMD x 1024 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0
# HBM bytes per fcp_attn_bwd_step(_direct) launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a plain 1 GiB copy (profiles/bench_packed32k_hbm_traffic.txt); known for the default workload only.
MEASURED_BWD_TRAFFIC_BYTES = {("packed32k_lognormal24_h32x8_D128", "accumulate"): 5.66e9,
                              ("packed32k_lognormal24_h32x8_D128", "direct"): 4.65e9}


def cpu_baseline(wl, q, k, v, do, rows, budget_rows=1 << 30, spans=None):
    """Times the oracle (as it stands) on a bounded sample: one KV-head group (hq/hkv query
    heads + 1 KV head) and every `stride`-th of the rank's rows; forward, dQ and the dK/dV
    partial of those rows.  Heads and rows are independent, so the rate carries over."""
    from oracle import attn as oattn
    from oracle import plan as oplan
    sid = None if spans is None else oplan.span_ids(wl.seq_lens, spans)
    G = wl.hq // wl.hkv
    stride = max(1, len(rows) // budget_rows)
    sample = np.ascontiguousarray(rows[::stride])
    qs, dos = np.ascontiguousarray(q[:, :G]), np.ascontiguousarray(do[:, :G])
    ks, vs = np.ascontiguousarray(k[:, :1]), np.ascontiguousarray(v[:, :1])
    cu = wl.cu_seqlens
    seq_of = np.searchsorted(cu, sample, side="right") - 1
    pairs = int((sample - cu[seq_of] + 1).sum())
    if sid is not None:     # plus the keys after the row inside its own span
        for n, (sk, st, ln) in enumerate(spans):
            in_span = sample[sid[sample] == n]
            pairs += int((cu[sk] + st + ln - 1 - in_span).sum())
    t0 = time.perf_counter()
    O, LSE = oattn.attn_fwd(qs, ks, vs, cu, wl.softmax_scale, sample, span_id=sid)
    oattn.attn_dq(qs, ks, vs, dos, cu, wl.softmax_scale, sample, O, LSE, span_id=sid)
    oattn.attn_dkv(qs, ks, vs, dos, cu, wl.softmax_scale, sample, O, LSE, span_id=sid)
    dt = time.perf_counter() - t0
    flops = 14.0 * pairs * wl.head_dim * G
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oattn.num_threads(), "kind": "oracle",
            "sample": f"{len(sample)} of the rank's {len(rows)} rows (every {stride}th), {G} query heads + 1 KV head, "
                      f"fwd + dQ + dK/dV partial, {pairs} pairs, {dt:.1f} s"}


def degree_sweep(steps, warmup):
    """One 32768-token sequence at CP degrees 1..8: what rank 0 does per layer (all ring steps of its two zigzag
    chunks, merge, backward), device-side random inputs."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    rows = []
    for d in range(1, 9):
        ra = RankAttention([32768], [d], 0, 32, 8, 128)
        ra.set_random_inputs(seed=d)
        pairs = ra.pairs()
        for _ in range(warmup):
            ra.forward(); ra.backward()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        tf, tm, tb = [], [], []
        for _ in range(steps):
            ev[0].record(); ra.forward_steps(); ev[1].record(); ra.merge(); ev[2].record()
            ra.zero_grads(); ra.backward_delta(); torch.cuda.synchronize()
            ev[0].synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); ra.backward_steps(); b.record(); torch.cuda.synchronize()
            tf.append(ev[0].elapsed_time(ev[1])); tm.append(ev[1].elapsed_time(ev[2])); tb.append(a.elapsed_time(b))
        f, m, b = float(np.median(tf)), float(np.median(tm)), float(np.median(tb))
        fl = pairs * 128.0 * 32.0
        rows.append({"degree": d, "rank": 0, "rank_rows": ra.tq, "pairs": pairs, "n_parts": ra.n_parts,
                     "fwd_step_ms": f, "merge_ms": m, "bwd_step_ms": b,
                     "fwd_tflops": 4.0 * fl / (f * 1e-3) / 1e12, "bwd_tflops": 10.0 * fl / (b * 1e-3) / 1e12,
                     "fwd_frac_mfma_peak": 4.0 * fl / (f * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "bwd_frac_mfma_peak": 10.0 * fl / (b * 1e-3) / 1e12 / PEAK_BF16_TFLOPS})
        del ra
        torch.cuda.empty_cache()
    return {"metric": "rank-local varlen causal attn TFLOP/s, CP degree sweep on one 32768-token sequence",
            "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "L32768_d1to8_h32x8_D128", "rank": 0}, "sweep": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=2, help="index into the five workloads (default: 32K packed)")
    ap.add_argument("--mask", choices=["causal", "mixed"], default="causal",
                    help="mixed: the same workload with synthetic image spans (576 tokens each, about 35 %% of a "
                         "sequence) that attend in full; pairs and flops then count the pairs visible under that mask")
    ap.add_argument("--forward", choices=["direct", "partial", "running"], default="direct",
                    help="direct (default): fcp_attn_fwd_step_direct + fcp_lse_merge_direct - rows fed by one work item "
                         "get their final O / LSE from the forward kernel, only the others are merged; partial: "
                         "fcp_attn_fwd_step + fcp_lse_merge for every row; running: one fcp_attn_fwd_step_running call "
                         "per ring step (no partial results, no merge), a comparison")
    ap.add_argument("--backward", choices=["direct", "accumulate"], default="direct",
                    help="direct (default): fcp_attn_bwd_step_direct + fcp_grad_finalize_direct - rows whose whole "
                         "gradient comes from one unit of work are written as bf16 by their kernel, nothing is cleared "
                         "beforehand; accumulate: clear the fp32 accumulators, fcp_attn_bwd_step, convert all of them")
    ap.add_argument("--degree-sweep", action="store_true",
                    help="secondary table instead of the benchmark line: one 32768-token sequence at CP degrees 1..8 "
                         "(rank 0's share, 32 / 8 heads, D = 128), forward and backward step times and rates")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy after the timed steps: the reference dispatch for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the ring steps of a CP group are simulated locally with all "
              "KV resident); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import fcp_synth as synth
    from paper_2602_21788_amd.rank import RankAttention

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.degree_sweep:
        print(json.dumps(degree_sweep(args.steps, args.warmup)))
        return
    wl = synth.make_workload(args.workload)
    q, k, v, do = synth.draw_qkvdo(wl)
    spans = synth.image_spans(wl.seq_lens, wl.seed) if args.mask == "mixed" else None
    ra = RankAttention(wl.seq_lens, wl.cp_degree, wl.rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale, spans=spans)
    ra.set_inputs(q, k, v, do)
    wl_name = wl.name + ("_img576" if spans is not None else "")
    pairs = ra.pairs()
    flops_fwd = 4.0 * pairs * wl.head_dim * wl.hq
    flops_bwd = 10.0 * pairs * wl.head_dim * wl.hq

    names = ["fwd_step", "merge", "zero", "delta", "bwd_step", "finalize"]

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        if args.forward == "running":
            mark(0); ra.forward_running()
            mark(1)
        elif args.forward == "direct":
            mark(0); ra.forward_steps_direct()
            mark(1); ra.merge_direct()
        else:
            mark(0); ra.forward_steps()
            mark(1); ra.merge()
        if args.backward == "direct":
            mark(2)
            mark(3); ra.backward_delta()
            mark(4); ra.backward_steps_direct()
            mark(5); ra.finalize_direct()
        else:
            mark(2); ra.zero_grads()
            mark(3); ra.backward_delta()
            mark(4); ra.backward_steps()
            mark(5); ra.finalize()
        mark(6)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    seg_ms = {n: float(np.mean([evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(args.steps)]))
              for i, n in enumerate(names)}

    import paper_2602_21788_amd as fcp
    assert fcp.fcp_scratch_status(ra.scratch_f)[1] == 0 and fcp.fcp_scratch_status(ra.scratch_b)[1] == 0

    value = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12
    bwd_tflops = flops_bwd / (seg_ms["bwd_step"] * 1e-3) / 1e12
    fwd_tflops = flops_fwd / (seg_ms["fwd_step"] * 1e-3) / 1e12
    merge_gbs = ra.merge_bytes(direct=args.forward == "direct") / (seg_ms["merge"] * 1e-3) / 1e9
    out = {
        "metric": "rank-local varlen causal attn TFLOP/s fwd+bwd, % of MFMA bf16 peak",
        "value": value, "unit": "TFLOP/s", "pct_of_mfma_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl_name, "mask": args.mask, "forward": args.forward, "backward": args.backward, "n_spans": 0 if spans is None else len(spans), "total_tokens": wl.total_tokens, "n_seqs": int(len(wl.seq_lens)),
                   "rank": wl.rank, "rank_rows": ra.tq, "pairs": pairs, "hq": wl.hq, "hkv": wl.hkv,
                   "head_dim": wl.head_dim, "n_parts": ra.n_parts, "max_cp_degree": int(wl.cp_degree.max()),
                   "seed": wl.seed},
        "roofline": {"bound": "mfma", "kernel": f"{'fcp_attn_bwd_step_direct' if args.backward == 'direct' else 'fcp_attn_bwd_step'} (dkv_kernel<{wl.head_dim}> + dq_kernel<{wl.head_dim}>)",
                     "achieved": bwd_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": bwd_tflops / PEAK_BF16_TFLOPS, "traffic": MEASURED_BWD_TRAFFIC_BYTES.get((wl_name, args.backward))},
        "kernels": {
            "fwd_step": {"ms": seg_ms["fwd_step"], "tflops": fwd_tflops, "frac_mfma_peak": fwd_tflops / PEAK_BF16_TFLOPS},
            "bwd_step": {"ms": seg_ms["bwd_step"], "tflops": bwd_tflops, "frac_mfma_peak": bwd_tflops / PEAK_BF16_TFLOPS},
            "merge": {"ms": seg_ms["merge"], "gbs": merge_gbs, "frac_hbm_peak": merge_gbs / PEAK_HBM_GBS},
            "delta": {"ms": seg_ms["delta"]}, "zero": {"ms": seg_ms["zero"]}, "finalize": {"ms": seg_ms["finalize"]},
        },
    }
    if args.copy_calibration:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, q, k, v, do, ra.rows, spans=spans)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
