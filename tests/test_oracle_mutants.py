"""Shows that the pins in test_oracle_pins.py have teeth: each plausible mistake, planted in a copy of the
oracle's C source and compiled on the CPU, makes at least one pin fail."""
import functools
import os
import subprocess

import pytest

import test_oracle_pins as pins
from oracle import lite_attn_oracle as orc

SRC = os.path.join(os.path.dirname(orc.__file__), "lite_attn_oracle.c")

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("no_scale", "s *= inv_sqrt_d;", ";"),
    ("predicate_sign", "real diff = mloc[r] - mnew[r];", "real diff = mnew[r] - mloc[r];"),
    ("predicate_direction", "(gval <= thr) && !pinned", "(gval >= thr) && !pinned"),
    ("predicate_strict", "(gval <= thr) && !pinned", "(gval < thr) && !pinned"),
    ("min_over_rows", "if (diff > gval) gval = diff;", "if (r == 0 || diff < gval) gval = diff;"),
    ("l_not_rescaled", "l[r] = a * l[r] + rowsum;", "l[r] = l[r] + rowsum;"),
    ("acc_not_rescaled", "for (int x = 0; x < d; ++x) accr[x] *= a;", ";"),
    ("mask_overwritten", "mask_row[j] |= newmask[j];", "mask_row[j] = newmask[j];"),
    ("running_max_starts_at_zero", "m[r] = -INFINITY; /* m_{i,-1} */", "m[r] = 0;"),
    ("fired_tile_always_dropped", "if (fire && sh->immediate) continue;", "if (fire) continue;"),
    ("fired_tile_never_dropped", "if (fire && sh->immediate) continue;", ";"),
    ("q_tile_not_pinned", "const int pinned = q_pinned ||", "const int pinned ="),
    ("k_tile_not_pinned", "q_pinned || intersects(c0, c0 + nc, sh->protect_start, sh->protect_len)", "q_pinned"),
    ("skipped_tile_computed", "if (mask_row[j]) {", "if (0) {"),
    ("v_columns_reversed", "accr[x] += p * vc[x];", "accr[x] += p * vc[d - 1 - x];"),
    ("running_max_not_updated", "m[r] = mnew[r];\n", ";\n"),
    ("tail_columns_ignored", "const int nc = (N - c0 < hk) ? (N - c0) : hk;", "const int nc = hk; if (c0 + nc > N) continue;"),
    ("stride_h_as_stride_b", "(int64_t)h * sh->stride_h;", "(int64_t)h * sh->stride_b;"),
    ("visiting_order_ignored", "const int j = visit ? visit[t] : t;", "const int j = t;"),
    ("visiting_order_of_row_zero", "visit ? visit + (int64_t)i * Tk : NULL", "visit"),
]

PINS = [
    lambda: pins.test_threshold_disabled_equals_dense_softmax_attention(200, 64, 64, 32, False),
    lambda: pins.test_threshold_disabled_equals_dense_softmax_attention(97, 16, 32, 48, True),
    pins.test_strided_bnhd_layout_matches_bhnd,
    lambda: pins.test_output_is_softmax_over_live_tiles(False),
    lambda: pins.test_output_is_softmax_over_live_tiles(True),
    lambda: pins.test_predicate_values_match_prefix_max_formula(256, 32, 64, 64),
    pins.test_fired_tiles_have_exponentially_small_weights,
    pins.test_two_tile_closed_form,
    pins.test_mask_evolution_invariants,
    pins.test_pinned_tiles_never_fire,
    pins.test_first_tile_never_fires_when_all_scores_are_negative,
    pins.test_visiting_order,
]


def _build_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site %r must occur exactly once in the oracle source" % old
    src = tmp_path / ("mutant_%s.c" % name)
    src.write_text(text.replace(old, new))
    libs = {}
    for f64 in (False, True):
        out = str(tmp_path / ("mutant_%s_%d.so" % (name, f64)))
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared"] + (["-DLA_ORACLE_F64"] if f64 else [])
        subprocess.run(cmd + [str(src), "-o", out, "-lm"], check=True)
        libs[f64] = orc.load_library(out, f64)
    return libs


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, monkeypatch, name, old, new):
    libs = _build_mutant(tmp_path, name, old, new)
    monkeypatch.setattr(pins, "oracle_step", functools.partial(orc.oracle_step, libs=libs))
    caught = []
    for pin in PINS:
        try:
            pin()
        except (AssertionError, ValueError):
            caught.append(pin)
    assert caught, "no pin noticed mutant %s" % name


def test_unmutated_source_passes_every_pin(tmp_path, monkeypatch):
    libs = _build_mutant(tmp_path, "identity", "s *= inv_sqrt_d;", "s *= inv_sqrt_d; ")
    monkeypatch.setattr(pins, "oracle_step", functools.partial(orc.oracle_step, libs=libs))
    for pin in PINS:
        pin()
