"""Host conversion of a K-cache to the banded layout, against the index formula the header states:
element (t, h, j) of a sequence sits at ((t // 32) * H + h) * 32 * d_k + (t % 32) * d_k + j."""
import numpy as np
import pytest

from paper_2503_05840_amd import binding


@pytest.mark.parametrize("B,ts,H,d_k,dtype", [(1, 32, 1, 8, np.uint16), (2, 96, 3, 16, np.uint16),
                                              (3, 64, 5, 24, np.float32), (1, 160, 32, 96, np.uint16)])
def test_band_kcache_follows_the_index_formula(B, ts, H, d_k, dtype):
    rng = np.random.default_rng(B * 1000 + ts)
    d = H * d_k
    K = rng.integers(0, 60000, size=(B, ts, d)).astype(dtype)
    got = binding.slim_band_kcache(K, H).reshape(B, ts * d)
    for _ in range(400):
        b, t, h, j = rng.integers(B), rng.integers(ts), rng.integers(H), rng.integers(d_k)
        assert got[b, ((t // 32) * H + h) * 32 * d_k + (t % 32) * d_k + j] == K[b, t, h * d_k + j]
    # a permutation: nothing lost, nothing duplicated
    assert np.array_equal(np.sort(got, axis=1), np.sort(K.reshape(B, ts * d), axis=1))


def test_band_kcache_wants_whole_bands():
    with pytest.raises(binding.SlimError) as ei:
        binding.slim_band_kcache(np.zeros((1, 33, 16), dtype=np.uint16), 2)
    assert ei.value.code == binding.SLIM_ERR_LAYOUT
