#!/usr/bin/env python3
"""Benchmark of the LiteAttention hot path on one MI355X.

A "step" is one denoising timestep of one attention layer: one lite_attn_fwd call (Skip-List compaction, V^T pre-pass,
fused skip-aware attention) over one set of synthetic Q, K, V already resident in HBM.  The timed region is
the first K steps of a fresh trajectory (step 0 starts from an empty Skip-Mask, i.e. the dense path; later
steps skip what earlier steps marked).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload wan14b] [--threshold T]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

TILE_FLOP = 4.0 * 128 * 128 * 128          # QK^T + PV of one live 128x128 tile pair, d = 128
PEAK_BF16_TFLOPS = 2500.0                  # MI355X dense bf16 MFMA, published

# HBM/fabric bytes per launch of lite_attn_fwd_kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs (counters
# are not readable from inside the process, so these are constants taken from the committed summaries under profiles/,
# not something this run measures): FETCH_SIZE scaled x2 and WRITE_SIZE x1 by what a 1 GiB device copy reads on the same
# counters.  Keyed on (workload, threshold); per launch the read bytes depend on whether anything is skipped yet
# (dense_read: empty Skip-Mask; sparse_read: the mask this threshold leaves from step 1 on), so any --steps / --warmup
# gets a figure: the mean over its timed launches.  Other workloads or thresholds report null.
MEASURED_TRAFFIC = {
    ("wan14b", -3.0): {"dense_read_bytes": 44.7e9, "sparse_read_bytes": 94.2e9, "write_bytes": 0.78e9,
                       "algorithmic_min_bytes": 3.09e9, "source": "profiles/lite_attn_fwd_wan14b.txt"},
}

# skip threshold (natural-log units of S) used per workload when none is given
DEFAULT_THRESHOLD = {"tiny": -2.0, "wan1.3b_dense": -float("inf"), "wan1.3b_sweep": -3.0, "wan14b": -3.0,
                     "longvideo": -3.0}


def cpu_baseline(wl, q, k, v, threshold, budget_rows, heads_sampled=4):
    """Times the CPU oracle, as it stands, on a sample of Q-tile rows of step 0 (dense: empty mask) spread over a
    few heads."""
    import numpy as np
    from oracle import lite_attn_oracle as orc
    from paper_2511_11062_amd import inputs
    N, d = wl.seqlen, wl.head_dim
    Tq = -(-N // 128)
    cores = orc.threads()
    hs = sorted(set(int(x) for x in np.linspace(0, wl.heads - 1, min(heads_sampled, wl.heads))))
    per_head = max(1, min(budget_rows // len(hs), Tq))
    tiles = sorted(set(int(x) for x in np.linspace(0, Tq - 1, per_head)))
    qs, ks, vs = (inputs.bf16_bits(x[:1, hs]) for x in (q, k, v))               # [1, len(hs), N, d] on the host
    rows = [a * Tq + i for a in range(len(hs)) for i in tiles]
    mask = np.zeros((1, len(hs), Tq, Tq), dtype=np.uint8)
    orc.oracle_step(qs, ks, vs, mask, threshold, protect=wl.protect, rows=rows[:1])     # load + page in
    t0 = time.perf_counter()
    orc.oracle_step(qs, ks, vs, mask, threshold, protect=wl.protect, rows=rows)
    dt = time.perf_counter() - t0
    valid = sum(min(128, N - (r % Tq) * 128) for r in rows)
    flops = 4.0 * valid * N * d
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s (dense-equivalent)", "cores": cores, "kind": "oracle",
            "sample": "%d of %d Q-tile rows of step 0 (empty mask), %d rows of each of heads %s, over all %d K/V "
                      "tiles, %.1f s, extrapolated per row" % (len(rows), wl.batch * wl.heads * Tq, len(tiles), hs, Tq, dt),
            "ms_per_step_extrapolated": dt / len(rows) * wl.batch * wl.heads * Tq * 1e3}


_MFMA_LIB = None


def mfma_only_tflops(hip_stream, dev_operands, iters=3000):
    """Sustained TFLOP/s of a register-resident bf16 MFMA loop on operands read from `dev_operands` (>= 64 KiB):
    the benchmark-only microkernel in libla_bench_mfma.so (not part of the attention library)."""
    import ctypes
    global _MFMA_LIB
    if _MFMA_LIB is None:
        _MFMA_LIB = ctypes.CDLL(os.path.join(ROOT, "paper_2511_11062_amd", "libla_bench_mfma.so"))
        _MFMA_LIB.la_bench_mfma_peak.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                                 ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
    ms, fl = ctypes.c_float(), ctypes.c_double()
    rc = _MFMA_LIB.la_bench_mfma_peak(ctypes.c_void_p(int(hip_stream)), ctypes.c_void_p(int(dev_operands)), int(iters),
                                      ctypes.byref(ms), ctypes.byref(fl))
    if rc != 0:
        raise RuntimeError("la_bench_mfma_peak: hipError_t %d" % rc)
    return fl.value / (ms.value * 1e-3) / 1e12


def run_workload(la, torch, inputs, wl, thr, K, W, dev, after=None):
    """W warm-up steps of a throw-away trajectory, then steps 0..K-1 of a fresh one (step 0 starts from an empty
    Skip-Mask), timed as a whole.  `after(data)` runs before the inputs are released (diagnostics on the same data).
    -> dict(wall seconds, per-step records, live-tile flop, summed attention-kernel ms, what `after` returned)."""
    B, H, N = wl.batch, wl.heads, wl.seqlen
    Tk = -(-N // 128)
    seq = inputs.DriftSequence(wl, dev)
    data = [next(seq) for _ in range(K)]                    # K steps of bf16 (q,k,v), resident in HBM
    del seq
    out = torch.empty_like(data[0][0])
    handle = la.lite_attn_init_mask(B, H, N, protect=wl.protect, max_steps=max(K, W, 1))
    la.lite_attn_set_stream(handle, torch.cuda.current_stream().cuda_stream)
    la.lite_attn_profile(handle, True)

    def run(steps):
        for t in range(steps):
            q, k, v = data[t % K]
            la.lite_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), handle, thr, t)

    run(W)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # flop of one live tile pair, the ragged last tile row / column counted by their valid share (exact when nothing
    # is skipped; with skips it assumes that the skipped tiles hold their share of the ragged ones)
    tile_flop = TILE_FLOP * (N / (128.0 * Tk)) ** 2
    per_step, live_flop, fwd_ms_total = [], 0.0, 0.0
    for t in range(K):
        st = la.lite_attn_skip_stats(handle, t)
        cms, fms = la.lite_attn_kernel_times(handle, t)
        live = st.tiles_total - st.tiles_skipped_in
        live_flop += live * tile_flop
        fwd_ms_total += fms
        per_step.append({"step": t, "skip_ratio": round(st.tiles_skipped_in / st.tiles_total, 4),
                         "newly_marked": round(st.tiles_newly_marked / st.tiles_total, 4),
                         "prep_ms": round(cms, 4), "attn_ms": round(fms, 3),
                         "attn_tflops_live": round(live * tile_flop / fms / 1e9, 1)})
    la.lite_attn_free_mask(handle)
    extra = after(data) if after else None
    return {"wall": wall, "per_step": per_step, "live_flop": live_flop, "fwd_ms": fwd_ms_total, "after": extra}


# workloads run after the main one inside the same process (steps, warm-up, threshold or None for the workload's
# default), reported compactly in `other_workloads`: the dense check, the 10-step sequence at the four thresholds of
# the sweep (about 30, 45, 60 and 70 % of the tiles skipped at the end), the first steps of the long-video layer
OTHER_WORKLOADS = {"wan14b": [("wan1.3b_dense", 10, 1, None)] +
                             [("wan1.3b_sweep", 10, 1, t) for t in (-2.75, -1.5, -0.5, -0.1)] +
                             [("longvideo", 3, 1, None)]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="default: the workload's sequence length (wan14b: 50)")
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="wan14b")
    ap.add_argument("--threshold", type=float, default=None)
    ap.add_argument("--cpu-rows", type=int, default=None, help="Q-tile rows the oracle baseline runs (0 = skip)")
    ap.add_argument("--no-others", action="store_true", help="skip the other_workloads block")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (heads would shard across GPUs with no collective inside "
                 "attention); --gpus %d is not supported" % args.gpus)

    import torch
    from paper_2511_11062_amd import inputs
    from paper_2511_11062_amd import lite_attn as la
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    wl = inputs.WORKLOADS[args.workload]
    thr = DEFAULT_THRESHOLD[args.workload] if args.threshold is None else args.threshold
    # default: the workload's whole sequence; a single-step workload (dense check) runs 10 steps of its drift
    K, W = args.steps or (wl.steps if wl.steps > 1 else 10), args.warmup
    dev = torch.device("cuda:0")
    B, H, N, d = wl.batch, wl.heads, wl.seqlen, wl.head_dim
    Tq = -(-N // 128)
    stream = torch.cuda.current_stream().cuda_stream

    if args.copy_calibration:       # a copy kernel of known size: reads 1 GiB, writes 1 GiB
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def diagnostics(data):
        """Runs after the timed region, on the same inputs."""
        res = {}
        # practical matrix-core ceiling on this workload's own bit patterns (register-resident MFMA loop, ~5 ms);
        # operands: this workload's V, i.e. N(0,1) values; and K rows from the middle of the sequence
        res["mfma_v"] = mfma_only_tflops(stream, data[0][2].data_ptr())
        res["mfma_k"] = mfma_only_tflops(stream, data[0][1][0, 0, N // 2].data_ptr())
        # the same kernel on all-zero operands (dense, one launch after a warm-up): the instruction stream is
        # identical, only the power drawn by the matrix cores differs
        zeros = torch.zeros_like(data[0][0])
        zout = torch.empty_like(zeros)
        zh = la.lite_attn_init_mask(B, H, N, protect=wl.protect, max_steps=2)
        la.lite_attn_set_stream(zh, stream)
        la.lite_attn_profile(zh, True)
        for t in range(2):
            la.lite_attn_fwd(zeros.data_ptr(), zeros.data_ptr(), zeros.data_ptr(), zout.data_ptr(), zh,
                             -float("inf"), t)
        torch.cuda.synchronize()
        res["zero_ms"] = la.lite_attn_kernel_times(zh, 1)[1]
        la.lite_attn_free_mask(zh)
        del zeros, zout
        rows = args.cpu_rows
        if rows is None:
            from oracle import lite_attn_oracle as orc
            # about 10-30 s of oracle time: one row-step costs 4*128*N*d flop at roughly 6 GFLOP/s per core
            per_row_s = 4.0 * 128 * N * d / 6.0e9
            rows = max(1, min(Tq, int(20.0 / per_row_s * orc.threads())))
        if rows > 0:
            res["cpu"] = cpu_baseline(wl, data[0][0], data[0][1], data[0][2], thr, rows)
        return res

    r = run_workload(la, torch, inputs, wl, thr, K, W, dev, after=diagnostics)
    wall, per_step, diag = r["wall"], r["per_step"], r["after"]
    dense = wl.dense_flops()
    achieved = r["live_flop"] / (r["fwd_ms"] * 1e-3) / 1e12
    zero_ms = diag["zero_ms"]

    traffic = None
    t_ = MEASURED_TRAFFIC.get((wl.name, thr))
    if t_:
        n_dense = sum(1 for s_ in per_step if s_["skip_ratio"] == 0.0)
        read = (n_dense * t_["dense_read_bytes"] + (K - n_dense) * t_["sparse_read_bytes"]) / K
        traffic = dict(t_, read_bytes=read, dense_launches=n_dense, sparse_launches=K - n_dense,
                       note="constants from the committed rocprofv3 counter runs (not measured by this run): mean "
                            "over this run's launches of the dense-step / sparse-step read bytes, plus the write bytes")

    others = []
    if not args.no_others:
        for name, k2, w2, thr2 in OTHER_WORKLOADS.get(wl.name, []):
            wl2 = inputs.WORKLOADS[name]
            thr2 = DEFAULT_THRESHOLD[name] if thr2 is None else thr2
            torch.cuda.empty_cache()
            r2 = run_workload(la, torch, inputs, wl2, thr2, k2, w2, dev)
            ps = r2["per_step"]
            others.append({"workload": "%s: B=%d H=%d N=%d" % (name, wl2.batch, wl2.heads, wl2.seqlen),
                           "threshold": thr2 if thr2 > -1e30 else "-inf (disabled)",
                           "steps": k2, "warmup": w2,
                           "ms_per_step": round(r2["wall"] / k2 * 1e3, 3),
                           "value_tflops": round(k2 * wl2.dense_flops() / r2["wall"] / 1e12, 1),
                           "attn_ms": [s_["attn_ms"] for s_ in ps], "skip_ratio": [s_["skip_ratio"] for s_ in ps],
                           "roofline_frac": round(r2["live_flop"] / (r2["fwd_ms"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)})

    result = {
        "metric": "dense-equivalent attention TFLOP/s over a denoising sequence (4*B*H*N^2*d per step / time)",
        "value": round(K * dense / wall / 1e12, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(wall / K * 1e3, 3),
        "median_attn_ms": round(sorted(s_["attn_ms"] + s_["prep_ms"] for s_ in per_step)[K // 2], 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: B=%d H=%d N=%d d=%d, %dx%dx%d latent grid%s, steps 0..%d of a drift sequence" % (
            wl.name, B, H, N, d, wl.grid[0], wl.grid[1], wl.grid[2],
            " + %d protected text tokens" % wl.text_tokens if wl.text_tokens else "", K - 1),
            "threshold": thr if thr > -1e30 else "-inf (disabled)", "mask_tile": "128x128",
            "mean_skip_ratio": round(sum(s["skip_ratio"] for s in per_step) / K, 4)},
        "dense_step": {"ms": per_step[0]["attn_ms"], "tflops": per_step[0]["attn_tflops_live"],
                       "frac_of_bf16_peak": round(per_step[0]["attn_tflops_live"] / PEAK_BF16_TFLOPS, 4),
                       "frac_of_measured_mfma_only": round(per_step[0]["attn_tflops_live"] / diag["mfma_v"], 4)},
        "per_step": per_step,
        "roofline": {"bound": "mfma", "kernel": "lite_attn_fwd_kernel", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic["read_bytes"] + traffic["write_bytes"] if traffic else None,
                     "traffic_detail": traffic,
                     "measured_mfma_only_tflops": round(diag["mfma_v"], 1),
                     "measured_mfma_only_tflops_on_k": round(diag["mfma_k"], 1),
                     "frac_of_measured_mfma_only": round(achieved / diag["mfma_v"], 4),
                     "dense_step_on_zero_operands": {"ms": round(zero_ms, 3),
                                                     "tflops": round(dense / zero_ms / 1e9, 1),
                                                     "frac": round(dense / zero_ms / 1e9 / PEAK_BF16_TFLOPS, 4)},
                     "note": "achieved = 8.39 MFLOP x (N / (128 Tk))^2 (ragged last tiles by their valid share) x live "
                             "tiles of the K timed launches / their summed HIP-event durations"},
        "other_workloads": others,
    }
    if "cpu" in diag:
        result["cpu_baseline"] = diag["cpu"]
    print(json.dumps(result))


if __name__ == "__main__":
    main()
