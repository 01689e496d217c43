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

Prints ONE JSON line.  `value` / `ms_per_step` come from the wall clock around the K timed steps; every segment is
also timed per step with events on the stream the kernels run on and reported as mean, median and min.  `roofline`
is for the dominant launch (the backward step: its scheduling launch and the two attention kernels), `cpu_baseline`
times the fp64 CPU oracle on a bounded sample of the same workload, and `secondary` (default run only) holds the
other workloads, the CP-degree sweep and the merge on a bandwidth-sized input, a few steps each, device-side random
inputs.
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
# counters read for a plain 1 GiB copy (profiles/bench_packed32k_hbm_traffic.txt); known for the default workload and path only.
MEASURED_BWD_TRAFFIC_BYTES = {("packed32k_lognormal24_h32x8_D128", "direct"): 4.52e9}
SEGMENTS = ["fwd_step", "merge", "zero", "delta", "bwd_step", "finalize"]


# ---- bookkeeping of a rank's share (algorithmic work; none of it is on the timed path) -------------------------------
def rank_pairs(ra) -> int:
    """Visible (query, key) pairs of the rank: sum over its rows of (position + 1), or of (last visible key
    position + 1) under a mixed mask."""
    if ra.spans is not None:
        return int(ra.q_limit.astype(np.int64).sum()) + ra.tq
    tot = 0
    for c in ra.my_chunks:
        a, n = int(c["seq_start"]), int(c["len"])
        tot += n * a + n * (n + 1) // 2
    return tot


def merge_bytes(ra, direct: bool) -> int:
    """Algorithmic bytes of the merge: per row and head, each contributing slot is read once (D fp32 + its LSE),
    every slot's LSE is read, and O (bf16) + LSE are written.  direct: fcp_lse_merge_direct skips the rows that
    exactly one work item feeds (one state byte per row is read)."""
    parts_per_row = np.zeros(ra.tq, np.int64)
    for w in ra.work:
        parts_per_row[int(w["q_local_off"]):int(w["q_local_off"]) + int(w["q_len"])] += 1
    D = ra.D
    if direct:
        merged = parts_per_row != 1
        return int(ra.hq * (parts_per_row[merged].sum() * (D * 4) + merged.sum() * (ra.n_parts * 4 + D * 2 + 4)) + ra.tq * ra.hq)
    return int(ra.hq * (parts_per_row.sum() * (D * 4) + ra.tq * (ra.n_parts * 4 + D * 2 + 4)))


def stats(xs):
    xs = np.asarray(xs, np.float64)
    return {"mean": float(xs.mean()), "median": float(np.median(xs)), "min": float(xs.min())}


def timed_steps(ra, steps, warmup, forward="direct", backward="direct"):
    """W warm-up steps, then K timed ones.  Returns (wall ms per step, {segment: [ms per step]})."""
    import torch

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        if forward == "running":
            mark(0); ra.forward_running()
            mark(1)
        elif forward == "direct":
            mark(0); ra.forward_steps_direct()
            mark(1); ra.merge_direct()
        else:
            mark(0); ra.forward_steps()
            mark(1); ra.merge()
        if backward == "direct":
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

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        step(evs[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    seg = {n: [evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(steps)] for i, n in enumerate(SEGMENTS)}
    seg["step"] = [evs[s][0].elapsed_time(evs[s][6]) for s in range(steps)]
    import paper_2602_21788_amd as fcp
    assert fcp.fcp_scratch_status(ra.scratch_f)[1] == 0 and fcp.fcp_scratch_status(ra.scratch_b)[1] == 0
    return (t1 - t0) * 1e3 / steps, seg


def rates(ra, seg, pairs, forward, backward):
    """Per-segment times (mean / median / min over the timed steps) and the rates that follow from the medians."""
    fl = float(pairs) * ra.D * ra.hq
    st = {n: stats(seg[n]) for n in seg}
    f, b, m = st["fwd_step"]["median"], st["bwd_step"]["median"], st["merge"]["median"]
    whole_bwd = float(np.median(np.asarray(seg["zero"]) + np.asarray(seg["delta"]) + np.asarray(seg["bwd_step"]) +
                                np.asarray(seg["finalize"])))
    mb = merge_bytes(ra, forward == "direct")
    return {
        "fwd_step": {"ms": st["fwd_step"], "tflops": 4 * fl / f / 1e9, "frac_mfma_peak": 4 * fl / f / 1e9 / PEAK_BF16_TFLOPS},
        "bwd_step": {"ms": st["bwd_step"], "tflops": 10 * fl / b / 1e9, "frac_mfma_peak": 10 * fl / b / 1e9 / PEAK_BF16_TFLOPS},
        "bwd_whole": {"ms": whole_bwd, "tflops": 10 * fl / whole_bwd / 1e9, "frac_mfma_peak": 10 * fl / whole_bwd / 1e9 / PEAK_BF16_TFLOPS,
                      "covers": "zero + delta + bwd_step + finalize"},
        "merge": {"ms": st["merge"], "bytes": mb, "gbs": mb / m / 1e6, "frac_hbm_peak": mb / m / 1e6 / PEAK_HBM_GBS},
        "delta": {"ms": st["delta"]}, "zero": {"ms": st["zero"]}, "finalize": {"ms": st["finalize"]},
        "step": {"ms": st["step"], "tflops": 14 * fl / st["step"]["median"] / 1e9},
    }


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
    chunks, merge, backward) through the plain entry points, device-side random inputs; medians."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    rows = []
    for d in range(1, 9):
        ra = RankAttention([32768], [d], 0, 32, 8, 128)
        ra.set_random_inputs(seed=d)
        pairs = rank_pairs(ra)
        _, seg = timed_steps(ra, steps, warmup, "partial", "accumulate")
        r = rates(ra, seg, pairs, "partial", "accumulate")
        rows.append({"degree": d, "rank": 0, "rank_rows": ra.tq, "pairs": pairs, "n_parts": ra.n_parts,
                     "fwd_step_ms": r["fwd_step"]["ms"]["median"], "merge_ms": r["merge"]["ms"]["median"],
                     "bwd_step_ms": r["bwd_step"]["ms"]["median"],
                     "fwd_tflops": r["fwd_step"]["tflops"], "bwd_tflops": r["bwd_step"]["tflops"],
                     "fwd_frac_mfma_peak": r["fwd_step"]["frac_mfma_peak"], "bwd_frac_mfma_peak": r["bwd_step"]["frac_mfma_peak"],
                     "merge_gbs": r["merge"]["gbs"]})
        del ra
        torch.cuda.empty_cache()
    return rows


def secondary(steps, warmup):
    """The other workloads (rank of the workload table, direct entry points), the plain-path merge of the 131072-token
    workload (1.9 GB of partial results: the merge's bandwidth figure), and the degree sweep."""
    import torch
    import fcp_synth as synth
    from paper_2602_21788_amd.rank import RankAttention
    out = {"steps": steps, "warmup": warmup, "inputs": "device-side N(0,1) bf16", "timing": "median over the timed steps",
           "workloads": {}}
    for cfg in (1, 3, 4):
        wl = synth.make_workload(cfg)
        ra = RankAttention(wl.seq_lens, wl.cp_degree, wl.rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale)
        ra.set_random_inputs(seed=cfg)
        pairs = rank_pairs(ra)
        wall, seg = timed_steps(ra, steps, warmup)
        r = rates(ra, seg, pairs, "direct", "direct")
        entry = {"rank": wl.rank, "rank_rows": ra.tq, "pairs": pairs, "n_parts": ra.n_parts, "ms_per_step_wall": wall,
                 "tflops": 14.0 * pairs * wl.head_dim * wl.hq / (wall * 1e-3) / 1e12, "kernels": r}
        if cfg == 3:
            _, seg_p = timed_steps(ra, steps, warmup, "partial", "direct")
            rp = rates(ra, seg_p, pairs, "partial", "direct")
            entry["merge_plain"] = rp["merge"]
            entry["merge_plain"]["note"] = "fcp_lse_merge over every row of the rank: the merge's HBM figure"
            # the same launches on all-zero operands: what the chip's clock does when the matrix units' inputs do not
            # toggle (a diagnostic, not a throughput claim: the instruction streams are the same)
            for t in (ra.q, ra.k, ra.v, ra.d_o):
                t.zero_()
            _, seg_z = timed_steps(ra, max(3, steps // 2), 2)
            rz = rates(ra, seg_z, pairs, "direct", "direct")
            entry["zero_operands_diagnostic"] = {
                "note": "same launches, Q = K = V = dO = 0: same shader cycles, higher clock (the chip is power-limited "
                        "on N(0,1) operands); not a throughput claim",
                "fwd_step_ms": rz["fwd_step"]["ms"]["median"], "fwd_frac_mfma_peak": rz["fwd_step"]["frac_mfma_peak"],
                "bwd_step_ms": rz["bwd_step"]["ms"]["median"], "bwd_frac_mfma_peak": rz["bwd_step"]["frac_mfma_peak"]}
        out["workloads"][wl.name] = entry
        del ra
        torch.cuda.empty_cache()
    out["degree_sweep_L32768_h32x8_D128_rank0_plain_entry_points"] = degree_sweep(steps, warmup)
    return out


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
    ap.add_argument("--no-secondary", action="store_true",
                    help="leave out the secondary measurements (other workloads, merge at size, degree sweep)")
    ap.add_argument("--secondary-steps", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--operands", choices=["normal", "zero"], default="normal",
                    help="normal (default): the workload's N(0,1) inputs.  zero: the same launches on all-zero Q, K, V, dO - "
                         "a diagnostic of how far the chip's clock under matrix load depends on the operand data (the "
                         "instruction streams are the same); its line says so in `data` and is not a throughput claim")
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
    wl = synth.make_workload(args.workload)
    q, k, v, do = synth.draw_qkvdo(wl)
    spans = synth.image_spans(wl.seq_lens, wl.seed) if args.mask == "mixed" else None
    ra = RankAttention(wl.seq_lens, wl.cp_degree, wl.rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale, spans=spans)
    if args.operands == "zero":
        q, k, v, do = (np.zeros_like(x) for x in (q, k, v, do))
    ra.set_inputs(q, k, v, do)
    wl_name = wl.name + ("_img576" if spans is not None else "")
    pairs = rank_pairs(ra)
    flops = 14.0 * pairs * wl.head_dim * wl.hq

    ms_per_step, seg = timed_steps(ra, args.steps, args.warmup, args.forward, args.backward)
    kern = rates(ra, seg, pairs, args.forward, args.backward)
    value = flops / (ms_per_step * 1e-3) / 1e12
    # roofline of the dominant launch: algorithmic flops of one backward step over the AVERAGE duration of the launch
    bwd_mean_ms = kern["bwd_step"]["ms"]["mean"]
    bwd_tflops = 10.0 * pairs * wl.head_dim * wl.hq / (bwd_mean_ms * 1e-3) / 1e12
    default_line = (args.workload == 2 and args.mask == "causal" and args.forward == "direct" and args.backward == "direct"
                    and args.operands == "normal")
    out = {
        "metric": "rank-local varlen causal attn TFLOP/s fwd+bwd, % of MFMA bf16 peak",
        "value": value, "unit": "TFLOP/s", "pct_of_mfma_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": kern["step"]["ms"]["median"], "ms_per_step_min": kern["step"]["ms"]["min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic" if args.operands == "normal" else "all-zero operands (clock diagnostic, not a throughput claim)",
        "config": {"workload": wl_name, "mask": args.mask, "forward": args.forward, "backward": args.backward, "n_spans": 0 if spans is None else len(spans), "total_tokens": wl.total_tokens, "n_seqs": int(len(wl.seq_lens)),
                   "rank": wl.rank, "rank_rows": ra.tq, "pairs": pairs, "hq": wl.hq, "hkv": wl.hkv,
                   "head_dim": wl.head_dim, "n_parts": ra.n_parts, "max_cp_degree": int(wl.cp_degree.max()),
                   "seed": wl.seed},
        "roofline": {"bound": "mfma", "kernel": f"{'fcp_attn_bwd_step_direct' if args.backward == 'direct' else 'fcp_attn_bwd_step'} (scheduling launch + dkv_kernel<{wl.head_dim}> + dq_kernel<{wl.head_dim}>)",
                     "achieved": bwd_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": bwd_tflops / PEAK_BF16_TFLOPS, "traffic": MEASURED_BWD_TRAFFIC_BYTES.get((wl_name, args.backward)),
                     "frac_whole_backward": kern["bwd_whole"]["frac_mfma_peak"],
                     "frac_forward_step": kern["fwd_step"]["frac_mfma_peak"]},
        "kernels": kern,
    }
    if args.copy_calibration:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    rows = ra.rows
    del ra
    torch.cuda.empty_cache()
    if default_line and not args.no_secondary:
        out["secondary"] = secondary(args.secondary_steps, 3)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, q, k, v, do, rows, spans=spans)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
