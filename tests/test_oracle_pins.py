"""Pins for the CPU oracle: each test fixes the oracle to something other than
itself -- brute force from a byte view of the stream, a dense sign matrix that
never touches the packing, popcount integers, algebraic invariants, the
paper's own two-stage table algorithm, numpy's fp16 decoding, and the
storage figures the paper states.  All inputs are integer- or dyadic-valued
where exact equality is asserted.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import btc_synth as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16_bits(a):
    return np.asarray(a, dtype=np.float16).view(np.uint16)


def small_int_x(rng, batch, n_in, lo=-8, hi=9):
    return f16_bits(rng.integers(lo, hi, size=(batch, n_in)).astype(np.float64))


# ---------------------------------------------------------------- P0 brute force
def brute_pack_words(idx_row, b, wpr):
    """One row as a big integer: index j occupies bits [j*b, (j+1)*b)."""
    big = 0
    for j, code in enumerate(idx_row):
        big |= int(code) << (j * b)
    return [(big >> (32 * w)) & 0xFFFFFFFF for w in range(wpr)]


def brute_linear(packed, codebook, alpha, mu, x, n_in, v, K):
    """Second, independently written evaluation: walks the stream as little-
    endian BYTES and does everything in exact rational arithmetic."""
    b = max(1, (K - 1).bit_length())
    out = packed.shape[0]
    nchunks = -(-n_in // v)
    raw = packed.astype("<u4").tobytes()
    row_bytes = packed.shape[1] * 4
    M = x.shape[0]
    y = [[Fraction(0)] * out for _ in range(M)]
    for i in range(out):
        base = i * row_bytes
        a = Fraction(float(alpha[i]))
        m = Fraction(float(mu[i]))
        for j in range(nchunks):
            code = 0
            for q in range(b):
                p = j * b + q
                code += ((raw[base + p // 8] >> (p % 8)) & 1) * (1 << q)
            pat = int(codebook[code])
            for t in range(v):
                k = j * v + t
                if k >= n_in:
                    continue
                s = 1 if (pat // (1 << t)) % 2 == 1 else -1
                w = a * s + m
                for mm in range(M):
                    y[mm][i] += w * Fraction(float(x[mm][k]))
    return np.array([[float(t) for t in row] for row in y])


@pytest.mark.parametrize("out,n_in,v,K", [
    (5, 40, 10, 16), (8, 37, 10, 13), (3, 29, 9, 16), (4, 31, 3, 8),
    (6, 18, 4, 9), (2, 33, 10, 512), (3, 17, 9, 1024), (7, 10, 10, 2),
])
def test_p0_brute_force(oracle, out, n_in, v, K):
    rng = np.random.default_rng(100 + out * 7 + n_in)
    nchunks = -(-n_in // v)
    if K <= (1 << v):
        codebook = rng.choice(1 << v, size=K, replace=False).astype(np.uint32)
    else:
        codebook = rng.permutation(np.tile(np.arange(1 << v), K // (1 << v))).astype(np.uint32)
    idx = rng.integers(0, K, size=(out, nchunks), dtype=np.int32)
    b = oracle.index_bits(K)
    assert b == max(1, (K - 1).bit_length())
    packed = oracle.pack(idx, K)
    wpr = packed.shape[1]
    assert wpr == -(-(nchunks * b) // 32)
    for i in range(out):
        assert list(packed[i]) == brute_pack_words(idx[i], b, wpr)
    assert np.array_equal(oracle.unpack(packed, nchunks, K), idx)
    # dyadic alpha/mu and small-integer x: every product and sum is exact in fp64
    alpha = (rng.integers(1, 64, size=out) / 32.0).astype(np.float32)
    mu = (rng.integers(-32, 32, size=out) / 64.0).astype(np.float32)
    x = small_int_x(rng, 2, n_in)
    y = oracle.linear(packed, codebook, alpha, mu, x, n_in, v, K)
    y_ref = brute_linear(packed, codebook, alpha, mu, x.view(np.float16).astype(np.float64), n_in, v, K)
    assert y.shape == (2, out)
    assert np.array_equal(y, y_ref)


def test_pack_rejects_out_of_range(oracle):
    idx = np.array([[0, 1, 5]], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.pack(idx, 5)
    with pytest.raises(ValueError):
        oracle.pack(np.array([[0, -1]], dtype=np.int32), 4)


def test_pack_tail_bits_are_zero(oracle):
    rng = np.random.default_rng(7)
    K, nchunks = 512, 410           # 3690 bits -> 116 words, 22 spare bits
    idx = np.full((3, nchunks), K - 1, dtype=np.int32)
    packed = oracle.pack(idx, K)
    assert packed.shape == (3, 116)
    assert np.all(packed[:, :115] == 0xFFFFFFFF)
    assert np.all(packed[:, 115] == (1 << (3690 - 115 * 32)) - 1)
    idx = rng.integers(0, K, size=(3, nchunks), dtype=np.int32)
    assert np.all(oracle.pack(idx, K)[:, 115] >> (3690 - 115 * 32) == 0)


# ------------------------------------------------- P1 full codebook = plain W1A16
@pytest.mark.parametrize("out,n_in,v", [(24, 70, 10), (16, 45, 9), (9, 64, 8), (5, 23, 10)])
def test_p1_full_codebook_is_dense_sign_matrix(oracle, out, n_in, v):
    """K = 2**v and codebook[k] = k: the index of a chunk IS its sign bits, so
    y = alpha * (sign(W) x) + mu * sum(x), computed here from the dense +-1
    matrix without any packing."""
    rng = np.random.default_rng(out * 1000 + n_in)
    K = 1 << v
    nchunks = -(-n_in // v)
    Wd = rng.normal(size=(out, n_in))
    Sg = np.where(Wd >= 0, 1.0, -1.0)                     # sign(0) = +1
    bits = np.zeros((out, nchunks * v), dtype=np.int64)
    bits[:, :n_in] = (Sg > 0)
    bits[:, n_in:] = rng.integers(0, 2, size=(out, nchunks * v - n_in))  # surplus: anything
    idx = (bits.reshape(out, nchunks, v) << np.arange(v)).sum(axis=2).astype(np.int32)
    codebook = np.arange(K, dtype=np.uint32)
    alpha = (rng.integers(1, 100, size=out) / 64.0).astype(np.float32)
    mu = (rng.integers(-50, 50, size=out) / 128.0).astype(np.float32)
    x = small_int_x(rng, 3, n_in)
    xd = x.view(np.float16).astype(np.float64)
    y = oracle.linear(oracle.pack(idx, K), codebook, alpha, mu, x, n_in, v, K)
    y_ref = (xd @ Sg.T) * alpha.astype(np.float64) + xd.sum(axis=1, keepdims=True) * mu.astype(np.float64)
    assert np.array_equal(y, y_ref)
    W = oracle.materialise(oracle.pack(idx, K), codebook, alpha, mu, n_in, v, K)
    assert W.shape == (out, n_in)
    assert np.array_equal(W, Sg * alpha[:, None].astype(np.float64) + mu[:, None].astype(np.float64))


# ------------------------------------------------------------- P2 ones vector
@pytest.mark.parametrize("out,n_in,v,K", [(12, 4096 // 8 + 3, 10, 512), (7, 100, 9, 1024), (5, 77, 10, 128)])
def test_p2_ones_vector_gives_popcount_integers(oracle, out, n_in, v, K):
    L, _ = S.make_case(3, out, n_in, v, K, 1)
    ones = f16_bits(np.ones((1, n_in)))
    y = oracle.linear(oracle.pack(L.idx, K), L.codebook, np.ones(out, np.float32),
                      np.zeros(out, np.float32), ones, n_in, v, K)
    nchunks = L.nchunks
    expect = np.zeros(out, dtype=np.int64)
    for j in range(nchunks):
        ln = min(v, n_in - j * v)
        mask = (1 << ln) - 1
        pc = np.array([bin(int(L.codebook[c]) & mask).count("1") for c in L.idx[:, j]])
        expect += 2 * pc - ln
    assert np.array_equal(y[0], expect.astype(np.float64))


# ------------------------------------------------------------- P3 linearity in x
def test_p3_linearity(oracle):
    L, _ = S.make_case(11, 33, 205, 10, 256, 1, dist="zipf")
    rng = np.random.default_rng(5)
    packed = oracle.pack(L.idx, L.K)
    x1 = rng.integers(-6, 7, size=(1, L.n_in)).astype(np.float64)
    x2 = rng.integers(-6, 7, size=(1, L.n_in)).astype(np.float64)
    a, b = 0.5, -2.0
    f = lambda xx: oracle.linear(packed, L.codebook, L.alpha, L.mu, f16_bits(xx), L.n_in, L.v, L.K)
    y12 = f(a * x1 + b * x2)                     # still exactly representable in fp16
    assert np.allclose(y12, a * f(x1) + b * f(x2), rtol=1e-13, atol=1e-13)
    assert np.array_equal(f(np.zeros((1, L.n_in))), np.zeros((1, L.out)))


# ------------------------------------------------------------- P4 affine split
def test_p4_affine_split_in_alpha_mu(oracle):
    L, x = S.make_case(12, 21, 333, 10, 512, 2)
    packed = oracle.pack(L.idx, L.K)
    one, zero = np.ones(L.out, np.float32), np.zeros(L.out, np.float32)
    y = oracle.linear(packed, L.codebook, L.alpha, L.mu, x, L.n_in, L.v, L.K)
    y10 = oracle.linear(packed, L.codebook, one, zero, x, L.n_in, L.v, L.K)
    sx = x.view(np.float16).astype(np.float64).sum(axis=1, keepdims=True)
    expect = y10 * L.alpha.astype(np.float64) + sx * L.mu.astype(np.float64)
    assert np.allclose(y, expect, rtol=1e-12, atol=1e-12)
    # and the pure-mean layer: alpha = 0 -> y = mu * sum(x) whatever the indices are
    y01 = oracle.linear(packed, L.codebook, zero, one, x, L.n_in, L.v, L.K)
    assert np.allclose(y01, np.broadcast_to(sx, y01.shape), rtol=1e-12, atol=1e-12)


# ------------------------------------------------ P5 XNOR-popcount closed form
@pytest.mark.parametrize("n_in,v,K", [(250, 10, 256), (83, 9, 1024), (64, 8, 100)])
def test_p5_xnor_popcount(oracle, n_in, v, K):
    """For x in {+-1}^in with bit pattern X_j per chunk,
    <x_j, C_k> = len_j - 2 * popcount((C_k xor X_j) & mask_j), from
    ||b - c||^2 = 4 d_H(b, c), d_H = popcount(b xor c) (Section 4.1, E-step)."""
    out = 19
    L, _ = S.make_case(21, out, n_in, v, K, 1)
    rng = np.random.default_rng(9)
    xb = rng.integers(0, 2, size=n_in)
    x = f16_bits((2.0 * xb - 1.0)[None, :])
    y = oracle.linear(oracle.pack(L.idx, K), L.codebook, np.ones(out, np.float32),
                      np.zeros(out, np.float32), x, n_in, v, K)
    expect = np.zeros(out, dtype=np.int64)
    for j in range(L.nchunks):
        ln = min(v, n_in - j * v)
        Xj = sum(int(xb[j * v + t]) << t for t in range(ln))
        mask = (1 << ln) - 1
        for i in range(out):
            expect[i] += ln - 2 * bin((int(L.codebook[L.idx[i, j]]) ^ Xj) & mask).count("1")
    assert np.array_equal(y[0], expect.astype(np.float64))


# ---------------------------------------------- P6 the paper's two-stage tables
def two_stage_lut_gemv(idx, codebook, xd, v, seg):
    """Appendix "Binary Codebook LUT-GEMM": Stage-I activation tables over
    segments of length `seg`, Stage-II codebook table through precomputed keys,
    then index-gather accumulation.  Needs seg | v and v | in."""
    out, nchunks = idx.shape
    P = v // seg
    K = codebook.shape[0]
    key = np.array([[(int(codebook[k]) >> (p * seg)) & ((1 << seg) - 1) for p in range(P)]
                    for k in range(K)])
    y = np.zeros(out)
    for j in range(nchunks):
        xj = xd[j * v:(j + 1) * v]
        lut = np.zeros((P, 1 << seg))
        for p in range(P):
            for s in range(1 << seg):
                lut[p, s] = sum((1.0 if (s >> t) & 1 else -1.0) * xj[p * seg + t] for t in range(seg))
        cblut = np.array([sum(lut[p, key[k, p]] for p in range(P)) for k in range(K)])
        y += cblut[idx[:, j]]
    return y


@pytest.mark.parametrize("v,seg,K", [(10, 5, 64), (8, 4, 32), (8, 8, 16)])
def test_p6_two_stage_lut_equals_definition(oracle, v, seg, K):
    out, n_in = 14, v * 6
    L, x = S.make_case(31, out, n_in, v, K, 1)
    xd = x.view(np.float16).astype(np.float64)[0]
    y = oracle.linear(oracle.pack(L.idx, K), L.codebook, np.ones(out, np.float32),
                      np.zeros(out, np.float32), x, n_in, v, K)
    y_lut = two_stage_lut_gemv(L.idx, L.codebook, xd, v, seg)
    assert np.allclose(y[0], y_lut, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------- relabelling / duplicates
def test_codebook_relabelling_and_duplicates(oracle):
    L, x = S.make_case(41, 17, 95, 9, 1024, 2)          # 1024 entries of length 9: duplicates
    assert len(np.unique(L.codebook)) == 512
    y = oracle.linear(oracle.pack(L.idx, L.K), L.codebook, L.alpha, L.mu, x, L.n_in, L.v, L.K)
    perm = np.random.default_rng(1).permutation(L.K)
    cb2 = np.empty_like(L.codebook)
    cb2[perm] = L.codebook                              # entry k moves to perm[k]
    idx2 = perm[L.idx].astype(np.int32)
    y2 = oracle.linear(oracle.pack(idx2, L.K), cb2, L.alpha, L.mu, x, L.n_in, L.v, L.K)
    assert np.array_equal(y, y2)
    # collapse duplicates to the 512-entry full codebook: same result
    first = {int(p): k for k, p in reversed(list(enumerate(L.codebook)))}
    idx3 = np.vectorize(lambda c: int(L.codebook[c]))(L.idx).astype(np.int32)
    y3 = oracle.linear(oracle.pack(idx3, 512), np.arange(512, dtype=np.uint32), L.alpha, L.mu, x,
                       L.n_in, L.v, 512)
    assert np.array_equal(y, y3) and len(first) == 512


def test_surplus_bits_of_last_chunk_do_not_matter(oracle):
    """in = 37, v = 10: the last chunk has 7 valid positions; flipping the 3
    surplus bits of every pattern must not change anything."""
    L, x = S.make_case(51, 9, 37, 10, 64, 1)
    packed = oracle.pack(L.idx, L.K)
    y = oracle.linear(packed, L.codebook, L.alpha, L.mu, x, L.n_in, L.v, L.K)
    W = oracle.materialise(packed, L.codebook, L.alpha, L.mu, L.n_in, L.v, L.K)
    assert W.shape == (9, 37)
    # patterns used ONLY in the last chunk column may have surplus bits flipped
    only_last = np.setdiff1d(L.idx[:, -1], L.idx[:, :-1])
    cb2 = L.codebook.copy()
    cb2[only_last] ^= np.uint32(0b111 << 7)
    y2 = oracle.linear(packed, cb2, L.alpha, L.mu, x, L.n_in, L.v, L.K)
    assert len(only_last) > 0 and np.array_equal(y, y2)


def test_row_subset_matches_full(oracle):
    L, x = S.make_case(61, 40, 123, 10, 128, 3)
    packed = oracle.pack(L.idx, L.K)
    y = oracle.linear(packed, L.codebook, L.alpha, L.mu, x, L.n_in, L.v, L.K)
    rows = np.array([39, 0, 7, 7, 21])
    ys = oracle.linear(packed, L.codebook, L.alpha, L.mu, x, L.n_in, L.v, L.K, rows=rows)
    assert np.array_equal(ys, y[:, rows])


def test_batch_rows_are_independent_and_layout_is_row_major(oracle):
    L, x = S.make_case(71, 13, 90, 10, 32, 4)
    packed = oracle.pack(L.idx, L.K)
    y = oracle.linear(packed, L.codebook, L.alpha, L.mu, x, L.n_in, L.v, L.K)
    assert y.shape == (4, 13)
    for m in range(4):
        ym = oracle.linear(packed, L.codebook, L.alpha, L.mu, x[m:m + 1], L.n_in, L.v, L.K)
        assert np.array_equal(ym[0], y[m])


# ----------------------------------------------------- fp16 / bf16 widening
def test_f16_widening_matches_numpy_for_every_pattern(oracle):
    bits = np.arange(1 << 16, dtype=np.uint16)
    ours = oracle.widen(bits, "f16")
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(ours), nan)
    assert np.array_equal(ours[~nan], ref[~nan])
    assert np.array_equal(np.signbit(ours[~nan]), np.signbit(ref[~nan]))
    assert oracle.f16_to_f64(0x3C00) == 1.0 and oracle.f16_to_f64(0xC000) == -2.0
    assert oracle.f16_to_f64(0x0001) == 2.0 ** -24 and oracle.f16_to_f64(0x7BFF) == 65504.0


def test_bf16_widening(oracle):
    bits = np.arange(1 << 16, dtype=np.uint16)
    ours = oracle.widen(bits, "bf16")
    ref = S.bf16_bits_to_f32(bits).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(ours[~nan], ref[~nan])
    assert oracle.bf16_to_f64(0x3F80) == 1.0 and oracle.bf16_to_f64(0xC040) == -3.0
    # 1 + 2^-7 is the next bf16 after 1
    assert oracle.bf16_to_f64(0x3F81) == 1.0 + 2.0 ** -7


# ----------------------------------------------------------- P7 accounting
def read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def test_p7_bit_rates_stated_by_the_paper(oracle):
    """ceil(log2 c) / v bits per weight (Compression Analysis) for the settings
    named 0.9 / 0.8 / 0.7 bit, and the 16 v / ceil(log2 c) compression ratio."""
    for v, c, bits, ratio in read_golden("bit_rates.txt"):
        v, c = int(v), int(c)
        b = oracle.index_bits(c)
        assert abs(b / v - float(bits)) < 1e-12
        assert abs(16.0 * v / b - float(ratio)) < 5e-3
        # large matrix with v | in: index bits dominate, codebook is v*c bits
        out, n_in = 4096, 4096 - 4096 % v
        total = oracle.storage_bits(out, n_in, v, c)
        assert total == v * c + b * out * n_in // v
        assert abs((total - v * c) / (out * n_in) - float(bits)) < 1e-12


def test_p7_row_padding_slack(oracle):
    """Stored bits per weight of the per-row uint32 stream at the benchmark widths."""
    for n_in, v, K, expect in [(4096, 10, 512, 0.9062), (5120, 10, 256, 0.8000),
                               (8192, 10, 128, 0.7031), (8192, 9, 1024, 1.1133)]:
        wpr = oracle.words_per_row(n_in, v, K)
        assert wpr == S.words_per_row(n_in, v, K)
        assert abs(wpr * 32 / n_in - expect) < 5e-5
    assert oracle.words_per_row(4096, 10, 512) == 116
    assert oracle.words_per_row(11008, 10, 512) == 310
    assert oracle.words_per_row(13824, 10, 256) == 346
    assert oracle.num_chunks(11008, 10) == 1101


def test_index_bits_non_power_of_two(oracle):
    # codebook sizes of the vector-length ablation (Table 3a) and their ceil(log2 c)
    for c, b in [(9, 4), (85, 7), (256, 8), (777, 10), (2353, 12), (7132, 13), (21619, 15), (65536, 16),
                 (2, 1), (3, 2), (512, 9), (513, 10)]:
        assert oracle.index_bits(c) == b == S.index_bits(c)
