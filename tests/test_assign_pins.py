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


# ---- M-step: c_k = sign(mean of the vectors assigned to k), sign(0) = +1, empty clusters unchanged

def test_update_majority_vote_against_numpy(oracle):
    rng = np.random.default_rng(10)
    for (v, K, N) in [(10, 16, 500), (9, 40, 300), (4, 3, 50), (20, 7, 200), (32, 5, 90)]:
        vec = rng.integers(0, 1 << 32, size=N, dtype=np.uint64).astype(np.uint32) & np.uint32((1 << v) - 1 if v < 32 else 0xFFFFFFFF)
        z = rng.integers(0, K, size=N).astype(np.int32)
        z[z == K - 1] = 0                                        # the last cluster stays empty
        old = rng.integers(0, 1 << min(v, 31), size=K).astype(np.uint32)
        new = oracle.update(vec, z, v, old)
        signs = np.where((vec[:, None] >> np.arange(v, dtype=np.uint32)[None, :]) & 1, 1, -1)   # N x v of +-1
        for k in range(K):
            member = signs[z == k]
            if len(member) == 0:
                assert new[k] == old[k]
                continue
            mean = member.mean(axis=0)
            want = sum(1 << t for t in range(v) if mean[t] >= 0)
            assert int(new[k]) == want


def test_update_ties_give_plus_one_and_single_member_is_copied(oracle):
    vec = np.array([0b0011, 0b0101, 0b1111, 0b1000], dtype=np.uint32)
    z = np.array([0, 0, 1, 2], dtype=np.int32)
    new = oracle.update(vec, z, 4, np.zeros(4, dtype=np.uint32) + 9)
    # cluster 0: elements (+,+) (+,-) (-,+) (-,-): sums 2, 0, 0, -2 -> 0111; clusters 1, 2: their only member; 3: empty
    assert new.tolist() == [0b0111, 0b1111, 0b1000, 9]


def test_update_is_a_fixed_point_after_assigning_exact_copies(oracle):
    rng = np.random.default_rng(11)
    cb = S.draw_codebook(rng, 10, 64)
    vec = cb[rng.integers(0, 64, size=1000)]
    z, d2 = oracle.assign(vec, 10, cb)
    assert not d2.any() and np.array_equal(oracle.update(vec, z, 10, cb), cb)


def test_update_never_increases_the_total_distance(oracle):
    """One E-step / M-step round of the clustering cannot raise the summed distance (each centroid moves to the
    per-dimension majority, which minimises the Hamming distance to its members)."""
    rng = np.random.default_rng(12)
    cb = S.draw_codebook(rng, 10, 32)
    vec = rng.integers(0, 1 << 10, size=4000).astype(np.uint32)
    z, d2 = oracle.assign(vec, 10, cb)
    new = oracle.update(vec, z, 10, cb)
    after = np.array([bin(int(a) ^ int(new[k])).count("1") for a, k in zip(vec, z)]) * 4
    assert after.sum() <= d2.sum()
    z2, d3 = oracle.assign(vec, 10, new)
    assert d3.sum() <= after.sum()


def test_update_rejects_assignments_out_of_range(oracle):
    with pytest.raises(ValueError):
        oracle.update(np.zeros(3, dtype=np.uint32), np.array([0, 5, 1], dtype=np.int32), 4, np.zeros(4, dtype=np.uint32))
