"""The three bounds every GPU-vs-oracle comparison applies (tests/util.py), checked on the CPU with
planted mistakes: errors that a per-tensor relative L2 lets through must trip the row or the element
bound, and honest rounding must pass all three."""
import numpy as np
import pytest

from paper_2204_12013_amd import synth
from util import TOL, assert_close, closeness, rel_l2


def _pair(shape=(4096, 1024), seed=0):
    rng = np.random.default_rng(seed)
    want = rng.standard_normal(shape)
    got = synth.round_to_storage(want.astype(np.float32), synth.DTYPE_BF16).astype(np.float64)   # honest bf16 rounding
    return want, got, rng


def test_honest_rounding_passes():
    want, got, _ = _pair()
    t, r, e = closeness(got, want, TOL[synth.DTYPE_BF16])
    assert t < 0.2 and r < 0.2 and e < 0.2
    assert_close(got, want, TOL[synth.DTYPE_BF16], "rounding")


def test_one_wrong_row_passes_the_norm_but_not_the_row_bound():
    want, got, rng = _pair()
    got[1234] = 0.0                                          # one of 4096 rows was never written
    assert rel_l2(got, want) <= TOL[synth.DTYPE_BF16]        # the tensor norm alone does not see it
    with pytest.raises(AssertionError, match="row"):
        assert_close(got, want, TOL[synth.DTYPE_BF16], "one bad row")


def test_sparse_wrong_elements_trip_the_element_bound():
    want, got, rng = _pair()
    ii = rng.integers(0, got.shape[0], 40)
    jj = rng.integers(0, got.shape[1], 40)
    got[ii, jj] += 1.0                                       # 40 elements off by one standard deviation
    assert rel_l2(got, want) <= TOL[synth.DTYPE_BF16]
    t, r, e = closeness(got, want, TOL[synth.DTYPE_BF16])
    assert t <= 1.0 and e > 1.0
    with pytest.raises(AssertionError):
        assert_close(got, want, TOL[synth.DTYPE_BF16], "sparse")


def test_a_wrong_32x32_tile_is_caught():
    want, got, rng = _pair()
    got[64:96, 128:160] = 0.0                                # a tile never written
    assert rel_l2(got, want) <= TOL[synth.DTYPE_BF16]
    with pytest.raises(AssertionError):
        assert_close(got, want, TOL[synth.DTYPE_BF16], "tile")


def test_vectors_and_nonfinite_values():
    want = np.linspace(-1, 1, 513)
    assert_close(want * (1 + 1e-5), want, 1e-4, "vector")
    bad = want.copy()
    bad[7] = np.nan
    with pytest.raises(AssertionError):
        assert_close(bad, want, 1e-4, "nan")
