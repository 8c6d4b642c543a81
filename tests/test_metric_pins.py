"""The error measures every parity assertion goes through, pinned on hand-made pairs (no GPU):
the tests' own relf / row_err / elem_err and the oracle's rel_frobenius."""
import math

import numpy as np
import pytest

from oracle import ffsplit_oracle as orc
import gpu_util as gu


A = np.array([[3.0, 4.0], [0.0, 0.0]])
B = np.array([[0.0, 0.0], [0.0, 5.0]])


@pytest.mark.parametrize("fn", [gu.relf, orc.rel_frobenius])
def test_relative_frobenius_on_hand_values(fn):
    # ||A - B||_F = sqrt(9 + 16 + 25), ||B||_F = 5
    assert fn(A, B) == pytest.approx(math.sqrt(50.0) / 5.0, rel=1e-15)
    assert fn(B, B) == 0.0
    # not symmetric: the second argument is the reference
    assert fn(B, A) == pytest.approx(math.sqrt(50.0) / 5.0, rel=1e-15)
    assert fn(2 * A, A) == pytest.approx(1.0, rel=1e-15)
    # a zero reference leaves the absolute norm
    assert fn(A, np.zeros_like(A)) == pytest.approx(5.0, rel=1e-15)
    # scale invariance and a single changed entry among many
    big = np.ones((100, 100))
    one = big.copy()
    one[7, 3] += 1.0
    assert fn(one, big) == pytest.approx(1.0 / 100.0, rel=1e-12)
    assert fn(1e6 * one, 1e6 * big) == pytest.approx(1.0 / 100.0, rel=1e-12)


def test_row_error_finds_the_one_bad_row():
    want = np.ones((1000, 64))
    got = want.copy()
    got[123] *= 1.5                       # one token off by 50 %: invisible to the whole-tensor figure
    assert gu.relf(got, want) == pytest.approx(0.5 / math.sqrt(1000.0), rel=1e-12)
    assert gu.relf(got, want) < 2e-2
    assert gu.row_err(got, want) == pytest.approx(0.5, rel=1e-12)
    # the floor: a row that is tiny in the reference is measured against half the rms row norm
    want2 = want.copy()
    want2[5] = 0.0
    got2 = want2.copy()
    got2[5, 0] = 0.04
    rms = math.sqrt((999 * 64) / 1000.0)
    assert gu.row_err(got2, want2) == pytest.approx(0.04 / (0.5 * rms), rel=1e-12)
    # a garbage row in place of a small one is still far above any bar
    got3 = want2.copy()
    got3[5] = 1.0
    assert gu.row_err(got3, want2) > 1.0
    assert gu.row_err(want, want) == 0.0


def test_element_error_of_score_vectors():
    want = np.array([1.0, 10.0, 1000.0, 0.0])
    got = np.array([1.1, 10.0, 1000.0, 0.5])
    # entry 0: 0.1 / 1 ; entry 3: 0.5 / (1e-3 * 1000)
    assert gu.elem_err(got, want) == pytest.approx(0.5, rel=1e-12)
    assert gu.elem_err(np.array([1.1, 10.0, 1000.0, 0.0]), want) == pytest.approx(0.1, rel=1e-9)


def test_assert_close_applies_both_bars():
    n_before = len(gu.OBSERVED)
    want = np.ones((1000, 64))
    got = want.copy()
    got[123] *= 1.5
    with pytest.raises(AssertionError):
        gu.assert_close(got, want, "bf16", "one bad row")
    gu.assert_close(want * (1 + 1e-3), want, "bf16", "uniform small error")
    with pytest.raises(AssertionError):
        gu.assert_close(want * (1 + 1.5e-2), want, "bf16", "uniform error above the bar")
    bad = want.copy()
    bad[0, 0] = np.nan
    with pytest.raises(AssertionError):
        gu.assert_close(bad, want, "bf16", "NaN")
    del gu.OBSERVED[n_before:]            # planted mistakes do not belong in the run's summary
