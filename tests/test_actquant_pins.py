"""Pins of the oracle's activation quantisation (min-max, one offset and step per activation row; section
"Activation Quantization on sub-bit LLMs") and of the layer on quantised activations.  None of them re-types the
routine: they check what the definition fixes -- the range of the codes, the ends of the range, the bound on the
reconstruction error, exactness on rows that are already on the grid, order preservation, and that the layer on
dequantised activations that happen to be fp16 numbers is the (separately pinned) fp16 layer."""
import numpy as np
import pytest

import btc_synth as S


def _rows(seed, M, n, kind="f16", scale=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.normal(0.0, scale, size=(M, n))
    if kind == "f16":
        return x.astype(np.float16).view(np.uint16)
    return S.f32_to_bf16_bits(x.astype(np.float32))


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_codes_cover_the_range_and_reconstruct_within_half_a_step(oracle, bits, kind):
    xb = _rows(1, 7, 1000, kind, scale=3.0)
    q, lo, step = oracle.quantize_rows(xb, kind, bits)
    x = oracle.widen(xb, kind)
    L = (1 << bits) - 1
    assert q.min() >= 0 and q.max() <= L
    for m in range(x.shape[0]):
        assert q[m, np.argmin(x[m])] == 0 and q[m, np.argmax(x[m])] == L
        assert float(lo[m]) == x[m].min()
        # step = (max - min) / L up to two fp32 roundings
        assert abs(float(step[m]) - (x[m].max() - x[m].min()) / L) <= 2.0 ** -22 * float(step[m])
    xr = oracle.dequantize_rows(q, lo, step)
    # half a step, plus the fp32 rounding of the quotient that decided the code
    assert np.all(np.abs(xr - x) <= (0.5 + 1e-5) * step[:, None].astype(np.float64))


@pytest.mark.parametrize("bits", [8, 4])
def test_rows_on_the_grid_come_back_exactly(oracle, bits):
    L = (1 << bits) - 1
    rng = np.random.default_rng(2)
    k = rng.integers(0, L + 1, size=(5, 300))
    k[:, 0], k[:, 1] = 0, L                      # both ends present
    lo0, st0 = -3.0, 0.03125                     # binary fractions: lo + st * k is an fp16 number
    x = (lo0 + st0 * k).astype(np.float16)
    assert np.array_equal(x.astype(np.float64), lo0 + st0 * k)
    q, lo, step = oracle.quantize_rows(x.view(np.uint16), "f16", bits)
    assert np.array_equal(q, k) and np.all(lo == np.float32(lo0)) and np.all(step == np.float32(st0))
    assert np.array_equal(oracle.dequantize_rows(q, lo, step), x.astype(np.float64))


def test_constant_row_and_order(oracle):
    x = np.full((1, 64), 1.5, dtype=np.float16)
    q, lo, step = oracle.quantize_rows(x.view(np.uint16), "f16", 8)
    assert not q.any() and lo[0] == np.float32(1.5) and step[0] == np.float32(1.0)
    xb = _rows(3, 4, 513, "bf16")
    q, lo, step = oracle.quantize_rows(xb, "bf16", 4)
    x = oracle.widen(xb, "bf16")
    for m in range(4):                           # a larger activation never gets a smaller code
        order = np.argsort(x[m], kind="stable")
        assert np.all(np.diff(q[m][order]) >= 0)


def test_ties_go_to_the_even_code(oracle):
    # lo = 0, step = 1 (range 255 over 255 levels): 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, 254.5 -> 254
    x = np.array([[0.0, 255.0, 0.5, 1.5, 2.5, 254.5, 7.0]], dtype=np.float16)
    q, lo, step = oracle.quantize_rows(x.view(np.uint16), "f16", 8)
    assert step[0] == np.float32(1.0) and list(q[0]) == [0, 255, 0, 2, 2, 254, 7]


def test_layer_on_grid_activations_is_the_fp16_layer(oracle):
    """Quantised activations whose reconstruction is an fp16 row: the layer on (q, lo, step) must equal the
    fp16 layer (pinned in test_oracle_pins.py) on that row, to the last bit of the fp64 sums' inputs."""
    layer, _ = S.make_case(4, 37, 250, 10, 256, 1)
    packed = oracle.pack(layer.idx, layer.K)
    rng = np.random.default_rng(5)
    k = rng.integers(0, 256, size=(3, 250))
    k[:, 0], k[:, 1] = 0, 255
    x = (-2.0 + 0.015625 * k).astype(np.float16)
    q, lo, step = oracle.quantize_rows(x.view(np.uint16), "f16", 8)
    assert np.array_equal(q, k)
    y_q = oracle.linear_aq(packed, layer.codebook, layer.alpha, layer.mu, q, lo, step, 250, 10, 256)
    y_x = oracle.linear(packed, layer.codebook, layer.alpha, layer.mu, x.view(np.uint16), 250, 10, 256)
    assert np.array_equal(y_q, y_x)


def test_quantisation_error_of_the_layer_is_bounded(oracle):
    """|y(x) - y(x_hat)| <= sum_k |W_hat[i][k]| * step / 2: the layer is linear and every activation moves by at
    most half a step."""
    layer, xb = S.make_case(6, 40, 330, 10, 256, 4)
    packed = oracle.pack(layer.idx, layer.K)
    for bits in (8, 4):
        q, lo, step = oracle.quantize_rows(xb, "f16", bits)
        y_q = oracle.linear_aq(packed, layer.codebook, layer.alpha, layer.mu, q, lo, step, 330, 10, 256)
        y_x = oracle.linear(packed, layer.codebook, layer.alpha, layer.mu, xb, 330, 10, 256)
        W = oracle.materialise(packed, layer.codebook, layer.alpha, layer.mu, 330, 10, 256)
        bound = np.abs(W).sum(axis=1)[None, :] * (0.5 + 1e-5) * step[:, None].astype(np.float64)
        assert np.all(np.abs(y_q - y_x) <= bound)
        assert np.any(np.abs(y_q - y_x) > 0)
