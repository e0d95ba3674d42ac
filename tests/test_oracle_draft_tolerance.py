"""The tolerances of the rd_draft parity tests are derived, not chosen: this test recomputes, on the
CPU, the deviation that a plain numpy fp32 evaluation of the draft model shows against the fp64
oracle -- over every small-model shape of the GPU parity test and on the Vicuna-7B-sized inputs --
and checks that the bounds the GPU tests use (tests/draft_tolerance.py: SAFETY x the stored
deviation, rounded up) follow from it."""
import numpy as np

import draft_tolerance as dt


def test_tolerances_follow_from_the_stored_deviations():
    s = dt.stored()
    assert dt.TOL == dt.round_up(dt.SAFETY * s["small"])
    assert dt.TOL_7B == dt.round_up(dt.SAFETY * max(s["vicuna7b"], s["vicuna13b"]))
    assert dt.round_up(0.0123) == 0.02 and dt.round_up(0.02) == 0.02 and abs(dt.round_up(9.6e-3) - 1e-2) < 1e-12
    assert 1e-3 < dt.TOL < 5e-2 and dt.TOL <= dt.TOL_7B < 1e-1        # log-probability units: far below what separates candidates


def test_small_models_fp32_deviation_is_what_the_bound_is_built_on():
    d = dt.small_deviation()
    stored = dt.stored()["small"]
    # the same computation as the stored figure (another BLAS may sum in another order and meet other
    # rounding boundaries: the same effect, another sample)
    assert d <= dt.TOL, (d, dt.TOL)
    assert stored / 4 <= d <= stored * 4, (d, stored)
    assert d > 1e-4                                    # the effect is real: far above fp32 accumulation error (~1e-6)


def test_vicuna7b_fp32_deviation_is_what_the_bound_is_built_on():
    d = dt.fp32_deviation(*dt.inputs_7b(), 8, 5)
    stored = dt.stored()["vicuna7b"]
    assert d <= dt.TOL_7B, (d, dt.TOL_7B)
    assert stored / 4 <= d <= stored * 4, (d, stored)
