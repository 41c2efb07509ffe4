"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer work (pack/unpack) must match bit for bit;
float outputs must satisfy  ||y-y*||_2/||y*||_2 <= 2e-3  and
max|y-y*| <= 1e-2 max|y*|  per call."""
import numpy as np
import pytest

import btc_synth as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_util
    return gpu_util


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ pack / unpack
PACK_SHAPES = [(64, 100, 10, 512), (33, 4096, 10, 512), (17, 11008, 10, 512), (40, 5120, 10, 256),
               (9, 8192, 9, 1024), (21, 8192, 10, 128), (5, 37, 3, 8), (12, 333, 4, 9), (3, 250, 20, 65536),
               (7, 64, 32, 2), (11, 130, 16, 7132), (1, 1, 1, 2)]


@pytest.mark.parametrize("out,n_in,v,K", PACK_SHAPES)
def test_pack_unpack_bit_exact(G, oracle, out, n_in, v, K):
    import torch
    B = G.B
    say(f"pack/unpack out={out} in={n_in} v={v} K={K}")
    rng = np.random.default_rng(out * 31 + n_in)
    s = B.btc_shape_init(out, n_in, v, K)
    idx = rng.integers(0, K, size=(out, s.nchunks), dtype=np.int32)
    idx[0, :] = K - 1
    idx[-1, -1] = K - 1
    ref = oracle.pack(idx, K)
    packed = G.GuardedOutput(out, s.words_per_row, torch.int32)
    ws = torch.zeros(16, dtype=torch.uint8, device="cuda")
    B.btc_pack(s, G.dev(idx), packed.payload, ws)
    packed.check_guards()
    got = packed.payload.cpu().numpy().view(np.uint32).reshape(out, s.words_per_row)
    assert np.array_equal(got, ref)
    back = G.GuardedOutput(out, s.nchunks, torch.int32)
    B.btc_unpack(s, G.dev(ref), back.payload)
    back.check_guards()
    assert np.array_equal(back.payload.cpu().numpy().reshape(out, s.nchunks), idx)
    assert np.array_equal(oracle.unpack(got, s.nchunks, K), idx)


def test_pack_rejects_out_of_range_index(G):
    import torch
    B = G.B
    s = B.btc_shape_init(8, 100, 10, 500)          # b = 9: 500..511 fit the field but are invalid
    ws = torch.zeros(16, dtype=torch.uint8, device="cuda")
    packed = torch.zeros(8 * s.words_per_row, dtype=torch.int32, device="cuda")
    for bad in (500, 511, 512, -1, 1 << 20):
        idx = np.zeros((8, s.nchunks), dtype=np.int32)
        idx[5, 7] = bad
        with pytest.raises(B.BtcError) as e:
            B.btc_pack(s, G.dev(idx), packed, ws)
        assert e.value.status == B.binding.BTC_ERR_INDEX_RANGE
    idx = np.full((8, s.nchunks), 499, dtype=np.int32)
    B.btc_pack(s, G.dev(idx), packed, ws)          # and the flag is cleared on the next call


# ------------------------------------------------------------------------- GEMV
GEMV_SMALL = [
    # out, in, v, K, batch, dist
    (300, 4096, 10, 512, 1, "uniform"), (260, 1101 * 10 - 2, 10, 512, 1, "uniform"),
    (129, 5120, 10, 256, 1, "zipf"), (70, 13824, 10, 256, 1, "zipf"),
    (200, 8192, 9, 1024, 1, "uniform"), (200, 8192, 10, 128, 1, "uniform"),
    (67, 1000, 10, 512, 2, "uniform"), (67, 1003, 10, 512, 3, "uniform"), (130, 2049, 10, 512, 4, "uniform"),
    (65, 777, 10, 256, 5, "uniform"), (96, 4096, 10, 512, 16, "uniform"),
    (50, 333, 4, 9, 1, "uniform"), (31, 260, 8, 85, 2, "uniform"), (20, 250, 20, 65536, 1, "uniform"),
    (9, 640, 32, 2, 1, "uniform"), (1, 10, 10, 512, 1, "uniform"), (5, 3, 10, 4, 1, "uniform"),
    (40, 330, 16, 7132, 4, "uniform"), (64, 96, 12, 777, 16, "uniform"),
    # 3..16 rows on the matrix-core engine (v = 10, 7..10 index bits; with 2 rows matrices this small
    # still take one pass per row): every index width, rows that are not 16-byte aligned, ragged last
    # chunk, out not a multiple of 4 / below one block of 16, several row and column tiles
    (300, 4096, 10, 128, 6, "uniform"), (131, 6408, 10, 256, 7, "zipf"), (77, 2570, 10, 1024, 16, "uniform"),
    (260, 1234, 10, 512, 3, "uniform"), (13, 648, 10, 256, 15, "uniform"), (1030, 10240, 10, 256, 4, "uniform"),
    (523, 5128, 10, 100, 9, "uniform"),
    # one row on wide matrices with 9 or 10 index bits: the single-kernel variant (ragged rows and columns,
    # rows of the stream that are not 16-byte aligned, chunk length 9)
    (70, 13824, 10, 512, 1, "uniform"), (130, 11006, 10, 512, 1, "zipf"), (200, 12006, 9, 1024, 1, "uniform"),
    (1, 10250, 10, 1024, 1, "uniform"),
    # the same engine at chunk length 9 (one tail value per chunk)
    (200, 8192, 9, 1024, 4, "uniform"), (77, 2700, 9, 512, 16, "uniform"), (130, 1000, 9, 256, 3, "zipf"),
    (300, 5770, 9, 128, 5, "uniform"),
]


@pytest.mark.parametrize("out,n_in,v,K,batch,dist", GEMV_SMALL)
@pytest.mark.parametrize("y_f32", [False, True])
def test_gemv_small_full_compare(G, oracle, out, n_in, v, K, batch, dist, y_f32):
    B = G.B
    say(f"gemv small out={out} in={n_in} v={v} K={K} batch={batch} {dist} f32={y_f32}")
    layer, x = S.make_case(7, out, n_in, v, K, batch, dist=dist, outlier_frac=0.01 if batch > 1 else 0.0)
    dl = G.DeviceLayer(layer, oracle)
    y = G.gemv(dl, x, B.BTC_F32 if y_f32 else B.BTC_F16)
    y_ref = oracle.linear(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, x, n_in, v, K)
    G.assert_close(y, y_ref, "gemv")
    y2 = G.gemv(dl, x, B.BTC_F32 if y_f32 else B.BTC_F16)
    assert np.array_equal(y, y2), "two runs differ"


def _full_size_gemv(G, oracle, case):
    """Every output of the call is compared with the oracle (no sampling)."""
    B = G.B
    say(f"gemv full {case}")
    layer, x = S.make_case(**case)
    dl = G.DeviceLayer(layer, oracle)
    y = G.gemv(dl, x, B.BTC_F16)
    G.assert_close(y, G.oracle_all_rows(oracle, dl, x), f"gemv {case}")


@pytest.mark.parametrize("case", S.config_cases(0) + S.config_cases(2), ids=lambda c: f"{c['out']}x{c['n_in']}")
def test_gemv_config_0_and_2_full_size(G, oracle, case):
    _full_size_gemv(G, oracle, case)


@pytest.mark.parametrize("case", S.config_cases(1), ids=lambda c: f"{c['out']}x{c['n_in']}b{c['batch']}")
def test_gemv_config_1_full_size(G, oracle, case):
    _full_size_gemv(G, oracle, case)


@pytest.mark.parametrize("case", S.config_cases(4),
                         ids=lambda c: f"{c['out']}x{c['n_in']}v{c['v']}K{c['K']}")
def test_gemv_config_4_full_size(G, oracle, case):
    _full_size_gemv(G, oracle, case)


def test_gemv_large_ragged_streaming(G, oracle):
    """A matrix large enough for the streaming kernel of the table engine (9-bit indices), with a
    ragged last row tile and a ragged last column block."""
    _full_size_gemv(G, oracle, dict(seed=3, out=28700, n_in=8190, v=10, K=512, batch=1))


def test_gemv_wide_single_row_on_matrix_cores(G, oracle):
    """A single activation row on a large, very wide matrix takes the matrix-core engine; here with
    ragged row tiles, a ragged last chunk and rows of the stream that are not 16-byte aligned."""
    _full_size_gemv(G, oracle, dict(seed=4, out=9001, n_in=28666, v=10, K=512, batch=1))


def test_gemv_calls_share_one_workspace(G, oracle):
    """One workspace, zero-filled once, serves calls of different shapes and batch sizes in a row:
    the table engine must find (and leave) its slots empty whatever ran before."""
    import torch
    B = G.B
    cases = [(700, 3008, 10, 64, 1), (700, 3008, 10, 64, 16), (300, 7008, 10, 64, 1), (9000, 4096, 10, 512, 16),
             (9000, 4096, 10, 512, 1), (700, 3008, 10, 64, 4), (300, 7008, 10, 64, 1)]
    layers = {}
    need = 16
    for (out, n_in, v, K, batch) in cases:
        if (out, n_in, K) not in layers:
            layer, _ = S.make_case(11, out, n_in, v, K, 1)
            layers[(out, n_in, K)] = (layer, G.DeviceLayer(layer, oracle))
        need = max(need, B.btc_workspace_bytes(layers[(out, n_in, K)][1].shape, batch, False))
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    rng = np.random.Generator(np.random.PCG64(5))
    for (out, n_in, v, K, batch) in cases:
        say(f"shared workspace: out={out} in={n_in} K={K} batch={batch}")
        layer, dl = layers[(out, n_in, K)]
        x = S.draw_x(rng, batch, n_in, "f16")
        y = G.GuardedOutput(batch, out, torch.float16)
        B.btc_gemv(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, G.dev(x), batch, y.payload, B.BTC_F16, ws)
        y.check_guards()
        assert int(ws.count_nonzero()) == 0, "btc_gemv did not hand the workspace back zero-filled"
        G.assert_close(y.numpy(), G.oracle_all_rows(oracle, dl, x), f"shared workspace {out}x{n_in} batch {batch}")


def test_gemv_invariants_on_gpu(G, oracle):
    """Full codebook and ones vector, evaluated by the HIP path itself."""
    B = G.B
    v, out, n_in = 10, 128, 1000
    K = 1 << v
    rng = np.random.default_rng(2)
    Sg = np.where(rng.normal(size=(out, n_in)) >= 0, 1.0, -1.0)
    bits = (Sg > 0).astype(np.int64).reshape(out, n_in // v, v)
    idx = (bits << np.arange(v)).sum(axis=2).astype(np.int32)
    layer = S.Layer(out, n_in, v, K, np.arange(K, dtype=np.uint32), idx,
                    np.ones(out, np.float32), np.zeros(out, np.float32))
    dl = G.DeviceLayer(layer, oracle)
    xi = rng.integers(-4, 5, size=(1, n_in)).astype(np.float16)
    y = G.gemv(dl, xi.view(np.uint16), B.BTC_F32)
    assert np.array_equal(y, (xi.astype(np.float64) @ Sg.T))         # small integers: exact in fp32
    ones = np.ones((1, n_in), np.float16)
    y1 = G.gemv(dl, ones.view(np.uint16), B.BTC_F32)
    assert np.array_equal(y1[0], Sg.sum(axis=1))


# ------------------------------------------------------------------------- GEMM
GEMM_SMALL = [
    # out, in, v, K, M, x_dtype
    (256, 640, 10, 256, 128, "bf16"), (300, 1000, 10, 256, 200, "bf16"), (130, 1283, 10, 512, 65, "bf16"),
    (128, 5120, 10, 256, 256, "bf16"), (140, 810, 9, 1024, 130, "bf16"), (64, 700, 10, 128, 17, "f16"),
    (100, 333, 4, 9, 33, "bf16"), (90, 512, 16, 7132, 40, "f16"), (70, 250, 20, 65536, 9, "bf16"),
    (33, 640, 32, 2, 5, "bf16"), (50, 231, 7, 100, 3, "f16"), (1, 10, 10, 512, 1, "bf16"),
    # tiled kernel (v = 10, in % 16 == 0): ragged M and out, out % 4 != 0 (scalar epilogue), every index
    # width it has a table for, long rows with few outputs (k split), more than one block of activation rows
    (301, 1600, 10, 256, 300, "bf16"), (300, 5136, 10, 512, 100, "f16"), (97, 2080, 10, 1024, 70, "bf16"),
    (512, 1616, 10, 128, 513, "bf16"), (2100, 800, 10, 256, 64, "bf16"), (45, 4000, 10, 64, 2, "f16"),
    # up to 64 rows: served by the decode engine of btc_gemv in blocks of 16 (bf16 and fp16 operands, chunk
    # lengths 10 and 9, a last block of one row, rows of X that are not 16-byte aligned)
    (140, 810, 9, 1024, 33, "bf16"), (300, 5136, 10, 512, 12, "f16"), (97, 2080, 10, 1024, 30, "bf16"),
    (523, 1002, 10, 256, 49, "bf16"), (13, 648, 10, 100, 16, "bf16"),
    # 17..64 rows at chunk length 10: two or four blocks of activation rows per table read; several row
    # tiles and column shares, ragged everything, every index width
    (700, 5128, 10, 512, 33, "bf16"), (1030, 2570, 10, 256, 64, "f16"), (300, 13824, 10, 128, 17, "bf16"),
    (261, 2082, 10, 1024, 32, "f16"), (77, 650, 10, 512, 63, "bf16"),
    # 65..128 rows on a matrix of more than 6 MB: 64 rows, then the rest (again that kernel, or the decode engine)
    (5200, 12800, 10, 512, 70, "bf16"), (5200, 12800, 10, 512, 100, "f16"),
]


@pytest.mark.parametrize("out,n_in,v,K,M,xd", GEMM_SMALL)
def test_gemm_small_full_compare(G, oracle, out, n_in, v, K, M, xd):
    B = G.B
    say(f"gemm small out={out} in={n_in} v={v} K={K} M={M} {xd}")
    layer, x = S.make_case(9, out, n_in, v, K, M, x_dtype=xd)
    dl = G.DeviceLayer(layer, oracle)
    xk = B.BTC_BF16 if xd == "bf16" else B.BTC_F16
    y_ref = oracle.linear(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, x, n_in, v, K, x_kind=xd)
    for yd in (B.BTC_F32, B.BTC_BF16 if xd == "bf16" else B.BTC_F16):
        y = G.gemm(dl, x, xk, yd)
        # bf16 output included: rounding to 8 significant bits is at most 2^-8 relative per element
        # (3.9e-3 < 1e-2 on the largest one) and 2^-8 / sqrt(7) = 1.5e-3 in the L2 ratio for significands
        # spread evenly over [1, 2) -- inside the bar that every other output type is held to (outputs of
        # fewer than 256 elements, where one element can sit at the worst case of its rounding: per element)
        (G.assert_close_bf16_out if yd == B.BTC_BF16 else G.assert_close)(y, y_ref, "gemm")
    y2 = G.gemm(dl, x, xk, B.BTC_F32)
    y3 = G.gemm(dl, x, xk, B.BTC_F32)
    assert np.array_equal(y2, y3), "two runs differ"


# Many activation rows and enough 256 x 160 output tiles to fill the chip: the route that expands the signs
# into bytes once per call and streams both operands into LDS.  Ragged last block of activation rows (one
# row, a few rows), out % 4 != 0 (scalar stores), a last k-tile that is partly or wholly past `in`, fp16
# and bf16, 10-bit indices, and chunk lengths other than 10 (the general expansion, also with a codebook
# that no LDS table holds).
GEMM_WIDE = [
    # out, in, v, K, M, x_dtype
    (6007, 400, 10, 256, 1300, "bf16"), (6100, 528, 10, 700, 1281, "f16"), (6000, 320, 8, 100, 1290, "bf16"),
    (5930, 336, 12, 3000, 1537, "bf16"), (9000, 240, 10, 512, 1024, "f16"),
]


@pytest.mark.parametrize("out,n_in,v,K,M,xd", GEMM_WIDE)
def test_gemm_many_rows_full_compare(G, oracle, out, n_in, v, K, M, xd):
    B = G.B
    say(f"gemm many rows out={out} in={n_in} v={v} K={K} M={M} {xd}")
    layer, x = S.make_case(11, out, n_in, v, K, M, x_dtype=xd)
    dl = G.DeviceLayer(layer, oracle)
    xk = B.BTC_BF16 if xd == "bf16" else B.BTC_F16
    y_ref = G.oracle_all_rows(oracle, dl, x, xd)
    for yd in (B.BTC_F32, B.BTC_BF16 if xd == "bf16" else B.BTC_F16):
        y = G.gemm(dl, x, xk, yd)
        (G.assert_close_bf16_out if yd == B.BTC_BF16 else G.assert_close)(y, y_ref, "gemm, many rows")
    y2 = G.gemm(dl, x, xk, B.BTC_F32)
    y3 = G.gemm(dl, x, xk, B.BTC_F32)
    assert np.array_equal(y2, y3), "two runs differ"


@pytest.mark.parametrize("case", S.config_cases(3), ids=lambda c: f"{c['out']}x{c['n_in']}M{c['batch']}")
def test_gemm_config_3_full_size(G, oracle, case):
    B = G.B
    say(f"gemm full {case}")
    layer, x = S.make_case(**case)
    dl = G.DeviceLayer(layer, oracle)
    y = G.gemm(dl, x, B.BTC_BF16, B.BTC_F32)
    assert np.all(np.isfinite(y))
    M = x.shape[0]
    # (1) every weight row, for a band of activation rows that touches every block of 256 activation rows
    # (first, last and two inner rows of each block)
    band = np.unique(np.concatenate([[b0, b0 + 37, b0 + 130, min(b0 + 255, M - 1)] for b0 in range(0, M, 256)]))
    band = band[band < M]
    y_band = G.oracle_all_rows(oracle, dl, x[band], "bf16")
    G.assert_close(y[band], y_band, f"gemm {case}, all weight rows of {len(band)} activation rows")
    # (2) every activation row, for sampled weight rows
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, layer.out - 1], rng.choice(layer.out, size=96, replace=False)]))
    y_ref = oracle.linear(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, x, layer.n_in, layer.v,
                          layer.K, x_kind="bf16", rows=rows)
    G.assert_close(y[:, rows], y_ref, f"gemm {case}, sampled weight rows")
