"""Parity at the benchmark's full shapes, in the launch configuration bench.py times, on sampled Q-tile rows
(rows are independent, so the oracle computes exactly those rows over all K/V of their heads)."""
import pytest

import parity

pytestmark = pytest.mark.gpu
NINF = -float("inf")


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
