"""CPU pins of the oracle's E-step (section "Binary Codebook Compression": nearest centroid of a +-1 vector,
||b - c||^2 = 4 d_H(b, c), d_H = POPCNT(b xor c); a vector identical to a centroid goes to that centroid)."""
import numpy as np
import pytest

import btc_synth as S


def _popcount(a):
    a = a.astype(np.uint64)
    return np.array([bin(int(x)).count("1") for x in a.reshape(-1)], dtype=np.int64).reshape(a.shape)


@pytest.mark.parametrize("v,K,N", [(4, 5, 64), (10, 37, 300), (9, 512, 200), (16, 100, 150), (20, 64, 100), (32, 9, 80)])
def test_matches_xor_popcount_closed_form(oracle, v, K, N):
    """Squared Euclidean distance on +-1 vectors is four times the Hamming distance; the minimum over k and the
    first index that attains it are recomputed with XOR and a bit count in Python integers."""
    rng = np.random.default_rng(v * 1000 + K)
    mask = (1 << v) - 1
    vec = (rng.integers(0, 1 << 32, size=N, dtype=np.uint64) & mask).astype(np.uint32)
    cb = (rng.integers(0, 1 << 32, size=K, dtype=np.uint64) & mask).astype(np.uint32)
    z, d2 = oracle.assign(vec, v, cb)
    dh = _popcount(vec[:, None].astype(np.uint64) ^ cb[None, :].astype(np.uint64))
    assert np.array_equal(d2, 4 * dh.min(axis=1))
    assert np.array_equal(z, dh.argmin(axis=1))            # numpy returns the first minimum


def test_identical_vector_goes_to_its_centroid(oracle):
    rng = np.random.default_rng(1)
    cb = S.draw_codebook(rng, 10, 256)
    pick = rng.integers(0, 256, size=500)
    z, d2 = oracle.assign(cb[pick], 10, cb)
    assert np.array_equal(z, pick) and not d2.any()


def test_full_codebook_is_the_identity(oracle):
    cb = np.arange(1 << 9, dtype=np.uint32)
    vec = np.random.default_rng(2).integers(0, 1 << 9, size=400).astype(np.uint32)
    z, d2 = oracle.assign(vec, 9, cb)
    assert np.array_equal(z, vec.astype(np.int32)) and not d2.any()


def test_ties_go_to_the_lowest_index_and_duplicates_too(oracle):
    cb = np.array([0b0011, 0b0101, 0b0101, 0b1111], dtype=np.uint32)
    vec = np.array([0b0111, 0b0101, 0b0001, 0b1011], dtype=np.uint32)
    z, d2 = oracle.assign(vec, 4, cb)
    # 0111: distance 1 to 0011, 0101, 0101 and 1111 -> index 0; 0101: equal to entries 1 and 2 -> 1;
    # 0001: distance 1 to 0011 and 0101 -> 0; 1011: distance 1 to 0011 and 1111 -> 0
    assert z.tolist() == [0, 1, 0, 0] and d2.tolist() == [4, 0, 4, 4]


def test_bits_above_v_are_ignored(oracle):
    rng = np.random.default_rng(3)
    vec = rng.integers(0, 1 << 10, size=100).astype(np.uint32)
    cb = rng.integers(0, 1 << 10, size=40).astype(np.uint32)
    z0, d0 = oracle.assign(vec, 10, cb)
    z1, d1 = oracle.assign(vec | np.uint32(0xABC00000), 10, cb | np.uint32(0x12300000 & ~0x3FF))
    assert np.array_equal(z0, z1) and np.array_equal(d0, d1)


def test_brute_force_in_pure_python(oracle):
    rng = np.random.default_rng(4)
    v, K = 6, 7
    vec = rng.integers(0, 1 << v, size=30).astype(np.uint32)
    cb = rng.integers(0, 1 << v, size=K).astype(np.uint32)
    z, d2 = oracle.assign(vec, v, cb)
    for i, b in enumerate(vec):
        best = None
        for k, c in enumerate(cb):
            d = sum(((1 if (int(b) >> t) & 1 else -1) - (1 if (int(c) >> t) & 1 else -1)) ** 2 for t in range(v))
            if best is None or d < best[0]:
                best = (d, k)
        assert (d2[i], z[i]) == best
