"""Pins of the oracle's storage variant with several (alpha, mu) groups per weight row (Table "Study of Number of
Split Points").  The group map is drawn here (2 bits per weight, packed LSB-first per row); the pins check the
routine against the single-group routine (pinned in test_oracle_pins.py) and against what the definition fixes."""
import numpy as np
import pytest

import btc_synth as S


def pack_groups(g):
    """int [out][in] in [0, 4) -> uint32 [out][ceil(2 in / 32)], weight k in bits [2k, 2k+2) of its row."""
    out, n = g.shape
    words = np.zeros((out, (2 * n + 31) // 32), dtype=np.uint64)
    for k in range(n):
        words[:, (2 * k) >> 5] |= g[:, k].astype(np.uint64) << np.uint64((2 * k) & 31)
    return words.astype(np.uint32)


def _case(seed, out, n_in, v, K, G):
    layer, x = S.make_case(seed, out, n_in, v, K, 3)
    rng = np.random.default_rng(seed + 1)
    g = rng.integers(0, G, size=(out, n_in))
    alpha = np.abs(rng.normal(0, 0.02, size=(out, G))).astype(np.float32)
    mu = rng.normal(0, 0.002, size=(out, G)).astype(np.float32)
    return layer, x, g, alpha, mu


def test_one_group_is_the_plain_layer(oracle):
    layer, x, g, alpha, mu = _case(1, 23, 205, 10, 256, 1)
    packed = oracle.pack(layer.idx, layer.K)
    W1 = oracle.materialise_groups(packed, layer.codebook, alpha, mu, pack_groups(g), 205, 10, 256)
    W0 = oracle.materialise(packed, layer.codebook, alpha[:, 0], mu[:, 0], 205, 10, 256)
    assert np.array_equal(W1, W0)


@pytest.mark.parametrize("G", [2, 3, 4])
def test_equal_parameters_in_every_group_give_the_plain_layer(oracle, G):
    layer, x, g, alpha, mu = _case(2, 17, 133, 9, 300, G)
    alpha[:] = alpha[:, :1]
    mu[:] = mu[:, :1]
    packed = oracle.pack(layer.idx, layer.K)
    W = oracle.materialise_groups(packed, layer.codebook, alpha, mu, pack_groups(g), 133, 9, 300)
    assert np.array_equal(W, oracle.materialise(packed, layer.codebook, alpha[:, 0], mu[:, 0], 133, 9, 300))


@pytest.mark.parametrize("G", [2, 3, 4])
def test_each_group_is_its_own_plain_layer(oracle, G):
    """W restricted to the weights of group g equals the plain layer with (alpha[:, g], mu[:, g]) there: the
    definition, evaluated through the separately pinned single-group routine; and relabelling the groups together
    with their parameters changes nothing."""
    layer, x, g, alpha, mu = _case(3, 31, 250, 10, 512, G)
    packed = oracle.pack(layer.idx, layer.K)
    W = oracle.materialise_groups(packed, layer.codebook, alpha, mu, pack_groups(g), 250, 10, 512)
    for gg in range(G):
        Wg = oracle.materialise(packed, layer.codebook, alpha[:, gg], mu[:, gg], 250, 10, 512)
        assert np.array_equal(W[g == gg], Wg[g == gg])
    perm = np.random.default_rng(9).permutation(G)           # new label of old group j is perm[j]
    a2, m2 = np.empty_like(alpha), np.empty_like(mu)
    a2[:, perm], m2[:, perm] = alpha, mu
    W2 = oracle.materialise_groups(packed, layer.codebook, a2, m2, pack_groups(perm[g]), 250, 10, 512)
    assert np.array_equal(W2, W)
    # a row subset in a given order
    rows = np.array([30, 0, 7])
    assert np.array_equal(oracle.materialise_groups(packed, layer.codebook, alpha, mu, pack_groups(g), 250, 10, 512,
                                                    rows=rows), W[rows])


def test_layer_is_the_sum_over_groups_of_masked_plain_layers(oracle):
    layer, x, g, alpha, mu = _case(4, 19, 170, 10, 128, 3)
    packed = oracle.pack(layer.idx, layer.K)
    y = oracle.linear_groups(packed, layer.codebook, alpha, mu, pack_groups(g), x, 170, 10, 128)
    X = oracle.widen(x, "f16")
    ref = np.zeros_like(y)
    for gg in range(3):
        Wg = oracle.materialise(packed, layer.codebook, alpha[:, gg], mu[:, gg], 170, 10, 128) * (g == gg)
        ref += X @ Wg.T
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
