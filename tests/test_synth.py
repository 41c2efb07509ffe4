"""The seeded input recipe: shapes, distributions and determinism."""
import numpy as np

import btc_synth as S


def test_determinism_and_draw_order():
    a, xa = S.make_case(0, 64, 205, 10, 512, 2)
    b, xb = S.make_case(0, 64, 205, 10, 512, 2)
    assert np.array_equal(a.codebook, b.codebook) and np.array_equal(a.idx, b.idx)
    assert np.array_equal(a.alpha, b.alpha) and np.array_equal(a.mu, b.mu) and np.array_equal(xa, xb)
    c, _ = S.make_case(1, 64, 205, 10, 512, 2)
    assert not np.array_equal(a.idx, c.idx)


def test_codebook_distinct_or_evenly_duplicated():
    rng = np.random.default_rng(0)
    cb = S.draw_codebook(rng, 10, 512)
    assert cb.dtype == np.uint32 and len(np.unique(cb)) == 512 and cb.max() < 1024
    cb = S.draw_codebook(rng, 9, 1024)
    vals, counts = np.unique(cb, return_counts=True)
    assert len(vals) == 512 and np.all(counts == 2)
    cb = S.draw_codebook(rng, 20, 64)
    assert len(np.unique(cb)) == 64 and cb.max() < (1 << 20)


def test_shapes_and_scales():
    L, x = S.make_case(0, 4096, 4096, 10, 512, 1)
    assert L.idx.shape == (4096, 410) and L.wpr == 116 and L.b == 9
    assert L.idx.min() >= 0 and L.idx.max() < 512
    assert np.all(L.alpha >= 0) and abs(L.alpha.mean() - 0.02 * np.sqrt(2 / np.pi)) < 1e-3
    assert abs(L.mu.std() - 0.002) < 2e-4
    xf = x.view(np.float16).astype(np.float64)
    assert x.shape == (1, 4096) and abs(xf.std() - 1.0) < 0.05


def test_bounded_zipf():
    rng = np.random.default_rng(0)
    idx = S.draw_indices(rng, 512, 512, 256, "zipf")
    assert idx.min() == 0 and idx.max() <= 255
    freq = np.bincount(idx.ravel(), minlength=256) / idx.size
    w = np.arange(1, 257) ** -1.1
    w /= w.sum()
    assert abs(freq[0] - w[0]) < 0.01 and abs(freq[1] - w[1]) < 0.01 and freq[255] > 0


def test_outlier_channels_shared_by_batch_rows():
    rng = np.random.default_rng(3)
    x = S.draw_x(rng, 4, 4096, "f16", outlier_frac=0.01)
    xf = np.abs(x.view(np.float16).astype(np.float64))
    big = (xf.mean(axis=0) > 8.0)
    assert 30 <= big.sum() <= 40            # floor(0.01 * 4096) = 40 channels, |N(0,1)|*20 mean ~ 16


def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 1.0 + 2.0 ** -8 + 2.0 ** -20], np.float32)
    bits = S.f32_to_bf16_bits(a)
    back = S.bf16_bits_to_f32(bits)
    assert list(back) == [1.0, 1.0, 1.0 + 2.0 ** -6, -2.5, 1.0 + 2.0 ** -7]


def test_config_tables():
    assert len(S.config_cases(0)) == 1 and len(S.config_cases(1)) == 9
    assert len(S.config_cases(2)) == 3 and len(S.config_cases(3)) == 6 and len(S.config_cases(4)) == 12
    assert all(c["seed"] == 0 for k in range(5) for c in S.config_cases(k))


def test_transform_pair_is_seeded_and_well_formed():
    bits, P1, P2 = S.draw_transform(3, 6, 10)
    bits2, Q1, Q2 = S.draw_transform(3, 6, 10)
    assert np.array_equal(bits, bits2) and np.array_equal(P1, Q1) and np.array_equal(P2, Q2)
    assert bits.dtype == np.uint32 and bits.shape == (2,) and (int(bits[1]) >> (60 - 32)) == 0   # tail bits zero
    assert P1.shape == (6, 6) and P2.shape == (10, 10) and P1.dtype == np.float32
    for P in (P1, P2):                                       # near-orthogonal, hence invertible and well conditioned
        assert np.linalg.cond(P.astype(np.float64)) < 2.0


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
