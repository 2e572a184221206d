"""The comparison gate of the GPU parity tests, checked on the CPU with planted mistakes: rounding-level noise passes, a
single wrong 256 x 256 tile of a large tensor, a single wild element, or a uniformly scaled tensor fail."""
import numpy as np
import pytest

from gpu_util import assert_close
from paper_2506_03077_amd import synth


def reference(shape=(2048, 1536), seed=0):
    return np.random.default_rng(seed).standard_normal(shape)


def test_bf16_rounding_noise_passes():
    ref = reference()
    got = synth.round_bf16(ref).astype(np.float64)          # one bf16 rounding per element: ~2e-3 relative
    assert assert_close(got, ref, 2e-2, "rounded") < 5e-3


def test_one_wrong_tile_fails_although_the_tensor_norm_hardly_moves():
    ref = reference()
    got = ref.copy()
    got[512:768, 1024:1280] = 0.0                            # one output tile of 48 never written
    whole = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert whole > 2e-2                                      # at this size the whole-tensor norm still sees it ...
    big = reference((8192, 4096), 1)
    bad = big.copy()
    bad[256:512, 512:768] *= 0.5                             # ... at 512 tiles, a half-scaled tile moves it by 2.2e-2 * ...
    assert np.linalg.norm(bad - big) / np.linalg.norm(big) < 2.3e-2
    bad[256:512, 512:768] = big[256:512, 512:768] * 0.7      # 30 % off in one tile of 512: norm-wise 1.3e-2 < 2e-2
    assert np.linalg.norm(bad - big) / np.linalg.norm(big) < 2e-2
    with pytest.raises(AssertionError, match="tile|max-abs"):
        assert_close(bad, big, 2e-2, "one tile 30 % off")
    with pytest.raises(AssertionError):
        assert_close(got, ref, 2e-2, "one tile missing")


def test_one_wild_element_fails_the_max_abs_gate():
    ref = reference((4096, 4096), 2)
    got = ref.copy()
    got[4095, 4095] += 0.5 * np.abs(ref).max()               # last element of the last ragged-free tile
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 1e-3
    with pytest.raises(AssertionError, match="max-abs"):
        assert_close(got, ref, 2e-2, "wild element")


def test_scaled_or_transposed_result_fails():
    ref = reference((512, 512), 3)
    with pytest.raises(AssertionError):
        assert_close(ref * 1.05, ref, 2e-2, "5 % scale error")
    with pytest.raises(AssertionError):
        assert_close(ref.T.copy(), ref, 2e-2, "transposed")


def test_ragged_edges_vectors_and_zero_reference_tiles():
    ref = reference((300, 700), 4)
    ref[:, 512:] = 0.0                                       # tiles whose reference is exactly zero
    assert_close(ref.copy(), ref, 1e-4, "exact")
    got = ref.copy()
    got[299, 699] = 1.0                                      # garbage where the reference is zero, in the ragged corner tile
    with pytest.raises(AssertionError):
        assert_close(got, ref, 2e-2, "garbage in a zero region")
    v = reference((3584,), 5)
    assert_close(v * (1 + 1e-5), v, 1e-4, "vector")
    assert_close(np.zeros((4, 4)), np.zeros((4, 4)), 1e-4, "all zero")
