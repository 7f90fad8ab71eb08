"""The shared parity assertions on planted mistakes (CPU): a reference with bf16-sized noise
passes; the same array with one wrong token row, one wrong 32-row block, a wrong ragged tail or
one wrong element fails, although the plane norm alone would let most of them through."""
import numpy as np
import pytest

from oracle import reslim_oracle as O
from parity_checks import assert_parity, plane_row_element_errors


def _ref_and_noisy(shape, seed=0, sigma=4e-3):
    rng = np.random.default_rng(seed)
    ref = rng.standard_normal(shape)
    return ref, ref + sigma * rng.standard_normal(shape) * np.abs(ref).mean()


def test_noise_of_bf16_size_passes_and_fp32_size_passes():
    ref, got = _ref_and_noisy((2, 1300, 512))
    assert_parity(got, ref, 2e-2, "noise")
    ref, got = _ref_and_noisy((3, 200, 64), sigma=3e-7)
    assert_parity(got, ref, 1e-5, "fp32 noise")


@pytest.mark.parametrize("plant", ["row", "block32", "tail", "element", "scaled_row"])
def test_planted_mistakes_fail(plant):
    ref, got = _ref_and_noisy((2, 8000, 128) if plant == "row" else (2, 1300, 512), seed=1)
    rng = np.random.default_rng(7)
    if plant == "row":                       # one token row replaced by another's values
        got[1, 777] = ref[1, 3]
    elif plant == "block32":                 # one 32-row block of a matrix tile zeroed
        got[0, 640:672] = 0.0
    elif plant == "tail":                    # the ragged tail (last 20 rows of 1300) left unwritten
        got[1, 1280:] = rng.standard_normal((20, 512))
    elif plant == "element":                 # a single element off by a fifth of the scale
        got[0, 10, 10] += 0.2
    elif plant == "scaled_row":              # a row off by 5 %
        got[0, 5] = 1.05 * ref[0, 5]
    plane = O.rel_l2(got, ref)
    if plant in ("row", "element", "scaled_row"):
        assert plane <= 2e-2                 # the norm over the plane does not see it
    with pytest.raises(AssertionError):
        assert_parity(got, ref, 2e-2, plant)


def test_error_measures_on_hand_made_arrays():
    ref = np.zeros((1, 2, 4))
    ref[0, 0] = [2.0, 2.0, 2.0, 2.0]         # plane rms = sqrt(16 / 8) = sqrt 2; row 1 is zero
    got = ref.copy()
    got[0, 0, 0] += 0.4                      # row 0: 0.4 / 4 = 0.1
    got[0, 1, 3] += 0.3                      # row 1: floor rms * sqrt(4) = 2 sqrt 2 -> 0.3 / 2.828
    plane, row, elem = plane_row_element_errors(got, ref)
    assert plane == pytest.approx(0.5 / 4.0)
    assert row == pytest.approx(max(0.1, 0.3 / (2.0 * np.sqrt(2.0))))
    assert elem == pytest.approx(0.4 / np.sqrt(2.0))
