"""Parity at the benchmark's full shapes, in the launch configuration bench.py times, on sampled Q-tile rows
(rows are independent, so the oracle computes exactly those rows over all K/V of their heads)."""
import numpy as np
import pytest
import torch

import parity
from paper_2511_11062_amd import inputs

pytestmark = pytest.mark.gpu
NINF = -float("inf")


def loud(capsys):
    """A print that reaches the terminal while pytest captures output: long tests report every step as they go."""
    def say(msg):
        with capsys.disabled():
            print("\n    " + msg, end="", flush=True)
    return say


def schedule_spread_rows(name, threshold, per_group=4, xcd_heads=8, xcd_rows=3):
    """Row ids chosen to cover the launch schedule of the fused kernel: the kernel ranks every head's Q-tile rows by
    Skip-List length and deals rank-chunks of 64 rows to the 8 XCDs, each chunk to the XCD with the least work so far
    (so the first rank-chunks of heads 0..7 open the eight XCDs).  A probe call of step 0 on the HIP path gives the mask
    from which steps 1.. are ranked; from it this picks, for the first and the last head, `per_group` rows of the
    first, the middle and the last rank-chunk, and `xcd_rows` rows of the first rank-chunk of each of `xcd_heads`
    consecutive heads (one head per XCD).  Only the
    CHOICE of rows comes from the probe: what the oracle computes for them does not."""
    from paper_2511_11062_amd import lite_attn as la
    wl = inputs.WORKLOADS[name]
    B, H, N = wl.batch, wl.heads, wl.seqlen
    Tq = -(-N // 128)
    q, k, v = next(inputs.DriftSequence(wl, "cuda:0"))
    out = torch.empty_like(q)
    h = la.lite_attn_init_mask(B, H, N, protect=wl.protect, max_steps=1)
    try:
        la.lite_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), h, threshold, 0)
        torch.cuda.synchronize()
        skipped = parity.unpack_mask(la.lite_attn_mask_export(h).reshape(B * H, Tq, -1), Tq).sum(axis=2)
    finally:
        la.lite_attn_free_mask(h)
    del q, k, v, out
    rows = set()
    chunks = -(-Tq // 64)
    for bh in (0, B * H - 1):
        ranked = np.argsort(skipped[bh], kind="stable")              # longest Skip-List (fewest skipped) first
        for c in (0, chunks // 2, chunks - 1):
            part = ranked[64 * c:64 * (c + 1)]
            rows |= {bh * Tq + int(i) for i in part[np.linspace(0, len(part) - 1, per_group).astype(int)]}
    for bh in range(min(xcd_heads, B * H)):
        ranked = np.argsort(skipped[bh], kind="stable")[:64]
        rows |= {bh * Tq + int(i) for i in ranked[np.linspace(0, len(ranked) - 1, xcd_rows).astype(int)]}
    return sorted(rows)


def test_wan13b_dense_equals_softmax_attention():
    """Config 2: B=1,H=12,N=32760, empty mask, threshold disabled."""
    reps = parity.run_sequence_check("wan1.3b_dense", steps=1, threshold=NINF, sample_rows=12, verbose=True)
    assert reps[0]["skipped_out"] == 0.0 and reps[0]["gpu_newly"] == 0.0


def test_wan13b_sweep_three_steps():
    """Config 3 shape, three steps with a fixed threshold."""
    reps = parity.run_sequence_check("wan1.3b_sweep", steps=3, threshold=-3.0, sample_rows=12, verbose=True)
    assert reps[-1]["skipped_out"] > 0.1


@pytest.mark.parametrize("threshold,expect", [(-2.75, 0.30), (-1.5, 0.45), (-0.5, 0.60), (-0.1, 0.70)])
def test_wan13b_sweep_ten_steps_four_thresholds(threshold, expect):
    """Config 3 in full: the 10-step sequence at each of the four thresholds of the sweep (about 30, 45, 60 and 70 %
    of the tiles skipped at the end), sampled rows, every step compared."""
    reps = parity.run_sequence_check("wan1.3b_sweep", steps=10, threshold=threshold, sample_rows=12, seed=3)
    assert abs(reps[-1]["gpu_skipped_in"] - expect) < 0.03


def test_wan14b_two_steps():
    """Config 4: B=1,H=40,N=75600 (tail tile of 80 columns)."""
    reps = parity.run_sequence_check("wan14b", steps=2, threshold=-3.0, sample_rows=10, verbose=True)
    assert reps[-1]["skipped_out"] > 0.1


def test_wan14b_six_steps_growing_mask():
    """Config 4 shape over six steps with a threshold that rises, so that the mask grows at several steps and the
    row schedule (rows ranked by Skip-List length) is exercised on masks of different shapes."""
    reps = parity.run_sequence_check("wan14b", steps=6, thresholds=[-4.0, -3.0, -3.0, -2.0, -2.0, -1.0], sample_rows=8,
                                     seed=11, verbose=True)
    frac = [r["skipped_out"] for r in reps]
    assert frac == sorted(frac) and frac[-1] > 0.4


def test_wan14b_diagonal_first_and_immediate():
    """Config 4 shape with both flags: diagonal-first visiting order and immediate PV-skip."""
    reps = parity.run_sequence_check("wan14b", steps=3, thresholds=[-3.0, -2.0, -1.0], sample_rows=6, seed=12,
                                     diagonal_first=True, immediate=True, verbose=True)
    assert reps[-1]["skipped_out"] > 0.4


def test_longvideo_with_text_tokens_two_steps():
    """Config 5: B=1,H=24,N=118800+256 text tokens (931x931 tiles, tail tile of 16 columns, protected range)."""
    reps = parity.run_sequence_check("longvideo", steps=2, threshold=-3.0, sample_rows=8, verbose=True)
    assert reps[-1]["skipped_out"] > 0.1


def test_longvideo_four_steps_growing_mask():
    """Config 5 shape over four steps with a rising threshold; the rows touching the text tokens are among the
    compared rows and must stay unmarked (the oracle's mask has them pinned)."""
    reps = parity.run_sequence_check("longvideo", steps=4, thresholds=[-3.0, -2.0, -1.5, -1.0], sample_rows=6, seed=13,
                                     verbose=True)
    frac = [r["skipped_out"] for r in reps]          # over the compared rows, several of which are pinned
    assert frac == sorted(frac) and frac[-1] > 0.3


def test_wan14b_bench_configuration_all_fifty_steps():
    """The sequence bench.py times by default (config 4: 50 steps, threshold -3), every step compared on sampled rows."""
    reps = parity.run_sequence_check("wan14b", steps=50, threshold=-3.0, sample_rows=4, seed=21)
    assert len(reps) == 50 and 0.25 < reps[-1]["gpu_skipped_in"] < 0.35
    assert max(r["max_dO"] / r["max_O"] for r in reps) <= parity.MAX_REL


def test_longvideo_all_thirty_steps():
    """Config 5 in full: 30 steps, threshold -3, sampled rows including those that touch the protected text tokens."""
    reps = parity.run_sequence_check("longvideo", steps=30, threshold=-3.0, sample_rows=3, seed=22)
    assert len(reps) == 30 and 0.25 < reps[-1]["gpu_skipped_in"] < 0.35


def test_maximum_sequence_length():
    """The longest sequence the library accepts (16383 K/V tiles per row is the limit): one head of N = 2 095 626
    tokens, 16 373 x 16 373 tiles with a 10-column tail, two steps, sampled rows.  One more tile row is refused."""
    from paper_2511_11062_amd import inputs, lite_attn as la
    wl = inputs.Workload("max_len", 1, 1, (13, 401, 402), steps=2, seed=31)
    assert -(-wl.seqlen // 128) == 16373
    reps = parity.run_sequence_check(wl, steps=2, threshold=-3.0, sample_rows=2, seed=31)
    assert reps[1]["gpu_skipped_in"] > 0.1
    with pytest.raises(la.LiteAttnError) as err:
        la.lite_attn_init_mask(1, 1, 128 * 16384)
    assert err.value.code == -3


def test_wan13b_every_row_marking_step_and_skipping_step(capsys):
    """Config 2/3 shape (B=1, H=12, N=32760: 256 x 256 tiles, 3072 Q-tile rows): EVERY row's output and mask row
    compared with the oracle, for the step that marks (empty mask on entry, dense path) and for the next step, which
    skips what was marked."""
    reps = parity.run_sequence_check("wan1.3b_sweep", steps=2, threshold=-3.0, sample_rows=None, verbose=True,
                                     say=loud(capsys))
    assert [r["rows"] for r in reps] == [3072, 3072]
    assert reps[0]["gpu_skipped_in"] == 0.0 and reps[0]["gpu_newly"] > 0.2
    assert abs(reps[1]["gpu_skipped_in"] - reps[0]["skipped_out"]) < 1e-3


def test_wan14b_three_steps_rows_across_the_schedule(capsys):
    """Config 4, three steps, more than 64 compared rows: the usual pinned ones (first, last, ragged tail), seeded
    random ones, and rows chosen to sit in the first, middle and last rank-chunk of two heads and on every XCD."""
    rows = schedule_spread_rows("wan14b", -3.0)
    reps = parity.run_sequence_check("wan14b", steps=3, threshold=-3.0, sample_rows=24, seed=41, extra_rows=rows,
                                     verbose=True, say=loud(capsys))
    assert all(r["rows"] >= 64 for r in reps) and reps[-1]["gpu_skipped_in"] > 0.25


def test_longvideo_three_steps_rows_across_the_schedule(capsys):
    """Config 5, three steps, more than 64 compared rows chosen as for config 4, plus the rows that touch the
    protected text tokens."""
    rows = schedule_spread_rows("longvideo", -3.0)
    reps = parity.run_sequence_check("longvideo", steps=3, threshold=-3.0, sample_rows=24, seed=42, extra_rows=rows,
                                     verbose=True, say=loud(capsys))
    assert all(r["rows"] >= 64 for r in reps) and reps[-1]["gpu_skipped_in"] > 0.25
