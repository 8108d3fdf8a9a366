#!/usr/bin/env python3
"""Per-timestep threshold schedule from error bounds (the paper's Accumulated-Error Calibration, on synthetic inputs).

The paper divides the timesteps evenly into three segments with error bounds xi - tau, xi, xi + tau and searches,
per timestep, the threshold that meets the bound on eta_t = |O^s_t - O_t|_1 / |O_t|_1.  The paper's calibrated values
need the real model's activations; this driver runs the same search on any sequence of (q, k, v) through the C ABI.

Because a tile marked at step t still contributes at step t (deferred mask update), the threshold of step t shows in
the output only once its mask is in force.  The error attributed to a candidate threshold at step t is therefore
that of step t's own inputs evaluated under the mask the candidate leaves behind: each trial runs the step with the
candidate (which extends the mask), then once more on the same inputs with marking disabled, and compares that
output with dense attention.  The search is a bisection on the threshold (eta grows monotonically as the threshold
approaches 0, since a larger threshold marks a superset of tiles).

    python -m paper_2511_11062_amd.calibrate --workload tiny --xi 0.075 --tau 0.01
"""
import argparse
import json

import numpy as np
import torch

from . import inputs
from . import lite_attn as la

NINF = -float("inf")


def _fwd(handle, q, k, v, out, thr, step):
    la.lite_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), handle, thr, step)


def calibrate(wl, data, xi=0.075, tau=0.01, lo=-12.0, hi=-0.05, iters=8, keep_masks=False):
    """data: list of (q,k,v) bf16 device tensors, one per timestep.  Returns a list of per-step dicts with the chosen
    threshold, its eta, the bound, and the skip ratio it leaves behind (keep_masks: also "mask_bits", the exported
    Skip-Mask words that the step's threshold leaves behind)."""
    B, H, N = wl.batch, wl.heads, wl.seqlen
    T = len(data)
    bounds = [xi - tau if 3 * t < T else (xi if 3 * t < 2 * T else xi + tau) for t in range(T)]
    dense = la.lite_attn_init_mask(B, H, N, protect=wl.protect, max_steps=2)
    work = la.lite_attn_init_mask(B, H, N, protect=wl.protect, max_steps=T + 2)
    stream = torch.cuda.current_stream().cuda_stream
    la.lite_attn_set_stream(dense, stream)
    la.lite_attn_set_stream(work, stream)
    schedule = []
    try:
        entry = None                                           # mask in force when step t starts (None = empty)
        for t, (q, k, v) in enumerate(data):
            ref = torch.empty_like(q)
            _fwd(dense, q, k, v, ref, NINF, 0)
            ref32 = ref.float()
            ref_l1 = ref32.abs().sum()
            out = torch.empty_like(q)

            def trial(thr):
                """eta of step t's inputs under the mask that `thr` leaves behind, and that mask."""
                if entry is None:
                    _fwd(work, q, k, v, out, thr, 0)           # step 0 clears the mask
                else:
                    la.lite_attn_mask_import(work, entry, t)
                    _fwd(work, q, k, v, out, thr, t)
                left = la.lite_attn_mask_export(work)
                _fwd(work, q, k, v, out, NINF, t + 1)          # same inputs, the new mask in force, no marking
                torch.cuda.synchronize()
                eta = float((out.float() - ref32).abs().sum() / ref_l1)
                return eta, left

            a, b = lo, hi                                      # invariant: eta(a) <= bound (or a == lo)
            best_thr, (best_eta, best_mask) = lo, trial(lo)
            if best_eta <= bounds[t]:
                for _ in range(iters):
                    mid = 0.5 * (a + b)
                    eta, left = trial(mid)
                    if eta <= bounds[t]:
                        a, best_thr, best_eta, best_mask = mid, mid, eta, left
                    else:
                        b = mid
            entry = best_mask
            skipped = int(np.unpackbits(best_mask.view(np.uint8)).sum())
            schedule.append({"step": t, "bound": bounds[t], "threshold": best_thr, "eta": best_eta,
                             "skipped_after": skipped / (B * H * (-(-N // 128)) ** 2), "met": best_eta <= bounds[t]})
            if keep_masks:
                schedule[-1]["mask_bits"] = best_mask.copy()
    finally:
        la.lite_attn_free_mask(dense)
        la.lite_attn_free_mask(work)
    return schedule


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="tiny")
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--xi", type=float, default=0.075)
    ap.add_argument("--tau", type=float, default=0.01)
    args = ap.parse_args()
    wl = inputs.WORKLOADS[args.workload]
    seq = inputs.DriftSequence(wl, "cuda:0")
    data = [next(seq) for _ in range(args.steps or wl.steps)]
    for row in calibrate(wl, data, args.xi, args.tau):
        print(json.dumps(row))


if __name__ == "__main__":
    main()
