#!/usr/bin/env python3
"""Per-step report of a denoising sequence: skip ratio, time, and the error against dense attention.

    python -m paper_2511_11062_amd.report --workload wan1.3b_sweep --steps 10 --thresholds -2 -3 -4

For every threshold it runs the sequence twice through the C ABI on cuda:0 -- once with the threshold and once with
the threshold disabled (the dense result O_t) -- and prints, per step, the fraction of tiles skipped on entry, the
attention-kernel time, and the paper's error measure eta_t = |O^s_t - O_t|_1 / |O_t|_1 (Accumulated-Error
Calibration section).  Inputs are the seeded synthetic workloads of `inputs.py`; PyTorch is used only to hold the
tensors and to take the L1 norms.
"""
import argparse
import json

import torch

from . import inputs
from . import lite_attn as la


# threshold sweep of the 12-head N=32760 sequence: found by a one-off sweep on the synthetic inputs, linear order;
# skipped fraction at step 9: 0.299, 0.452, 0.603, 0.707 (eta_9: 0.13, 0.30, 0.71, 1.17)
SWEEP_THRESHOLDS = {"wan1.3b_sweep": [-2.75, -1.5, -0.5, -0.1]}


def run_sequence(wl, data, thresholds, dense_out=None, diagonal_first=False, immediate=False):
    """thresholds: one value per step.  Returns (outputs or None, per-step dicts).  If dense_out is given, eta is
    computed against it; otherwise the outputs are returned (used to produce the dense reference)."""
    B, H, N = wl.batch, wl.heads, wl.seqlen
    steps = len(data)
    flags = ((la.LITE_ATTN_ORDER_DIAGONAL_FIRST if diagonal_first else 0) |
             (la.LITE_ATTN_PV_SKIP_IMMEDIATE if immediate else 0))
    h = la.lite_attn_init_mask(B, H, N, protect=wl.protect, max_steps=steps, flags=flags)
    la.lite_attn_set_stream(h, torch.cuda.current_stream().cuda_stream)
    la.lite_attn_profile(h, True)
    outs, rows = [], []
    try:
        for t, (q, k, v) in enumerate(data):
            out = torch.empty_like(q)
            la.lite_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), h, thresholds[t], t)
            torch.cuda.synchronize()
            st = la.lite_attn_skip_stats(h, t)
            prep_ms, attn_ms = la.lite_attn_kernel_times(h, t)
            row = {"step": t, "threshold": thresholds[t], "skip_ratio": st.tiles_skipped_in / st.tiles_total,
                   "newly_marked": st.tiles_newly_marked / st.tiles_total, "prep_ms": prep_ms, "attn_ms": attn_ms}
            if dense_out is not None:
                ref = dense_out[t].float()
                row["eta"] = float((out.float() - ref).abs().sum() / ref.abs().sum())
            else:
                outs.append(out)
            rows.append(row)
    finally:
        la.lite_attn_free_mask(h)
    return (outs if dense_out is None else None), rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="wan1.3b_sweep")
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--thresholds", type=float, nargs="+", default=None,
                    help="default: the workload's sweep (for wan1.3b_sweep the four values that leave about 30, 45, "
                         "60 and 70 %% of the tiles skipped at step 9)")
    ap.add_argument("--json", action="store_true", help="print one JSON document instead of a table")
    ap.add_argument("--diagonal-first", action="store_true",
                    help="visit the K/V tiles of Q tile i in the order i, i+1, ..., Tk-1, 0, ..., i-1")
    ap.add_argument("--immediate", action="store_true",
                    help="drop a fired tile in the call that marks it (Algorithm 2 literally) instead of from the next "
                         "call on")
    args = ap.parse_args()
    wl = inputs.WORKLOADS[args.workload]
    steps = args.steps or wl.steps
    seq = inputs.DriftSequence(wl, "cuda:0")
    data = [next(seq) for _ in range(steps)]
    thresholds = args.thresholds or SWEEP_THRESHOLDS.get(wl.name, [-4.0, -3.0, -2.0, -1.0])
    dense_out, dense_rows = run_sequence(wl, data, [-float("inf")] * steps)
    result = {"workload": wl.name, "steps": steps, "diagonal_first": args.diagonal_first, "immediate": args.immediate,
              "dense_ms": [r["attn_ms"] for r in dense_rows], "runs": []}
    for thr in thresholds:
        _, rows = run_sequence(wl, data, [thr] * steps, dense_out, args.diagonal_first, args.immediate)
        result["runs"].append({"threshold": thr, "per_step": rows})
    if args.json:
        print(json.dumps(result))
        return
    print("workload %s: B=%d H=%d N=%d, %d steps; dense attention %.2f ms/step" % (
        wl.name, wl.batch, wl.heads, wl.seqlen, steps, sum(result["dense_ms"]) / steps))
    for run in result["runs"]:
        print("threshold %.2f" % run["threshold"])
        print("  step  skipped  newly   attn ms  ms/dense  live frac   eta")
        for r, d in zip(run["per_step"], result["dense_ms"]):
            print("  %4d  %6.3f  %6.4f  %8.3f  %8.3f  %9.3f  %.4f" % (
                r["step"], r["skip_ratio"], r["newly_marked"], r["attn_ms"], r["attn_ms"] / d, 1 - r["skip_ratio"],
                r["eta"]))


if __name__ == "__main__":
    main()
