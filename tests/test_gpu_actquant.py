"""GPU parity of the layer on quantised activations (btc_quantize_rows, btc_weight_rowsums, btc_gemm_aq) against
the oracle: the integer codes, offsets and steps bit for bit (both sides decide them in fp32, operation by
operation), the row sums of W_hat and the layer's outputs -- every output -- to the floating-point bar of the
other parity tests; 8 and 4 bits, fp16 and bf16 activations, one row (the decode engines), a few rows, and
enough rows for the prefill kernels, ragged shapes, a constant row, a row with outlier channels."""
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


def _quantize(G, xb, kind, bits):
    import torch
    B = G.B
    M, n = xb.shape
    Q = G.GuardedOutput(M, n, torch.uint8)
    lo = torch.empty(M, dtype=torch.float32, device="cuda")
    step = torch.empty(M, dtype=torch.float32, device="cuda")
    qsum = torch.empty(M, dtype=torch.float32, device="cuda")
    B.btc_quantize_rows(G.dev(xb), B.BTC_BF16 if kind == "bf16" else B.BTC_F16, M, n, bits, Q.payload, lo, step, qsum)
    Q.check_guards()
    return Q.payload.view(M, n), lo, step, qsum


QUANT_CASES = [(1, 10, "f16"), (3, 4096, "f16"), (5, 5120, "bf16"), (2, 13824, "f16"), (17, 333, "bf16"), (64, 1001, "f16")]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,n,kind", QUANT_CASES)
def test_codes_offsets_and_steps_bit_exact(G, oracle, M, n, kind, bits):
    print(f"quantize M={M} n={n} {kind} bits={bits}", flush=True)
    rng = np.random.Generator(np.random.PCG64(100 + M))
    xb = S.draw_x(rng, M, n, kind, outlier_frac=0.01)
    if M >= 3:
        xb[1, :] = xb[1, 0]                              # a constant row
    Q, lo, step, qsum = _quantize(G, xb, kind, bits)
    q_ref, lo_ref, step_ref = oracle.quantize_rows(xb, kind, bits)
    assert np.array_equal(lo.cpu().numpy(), lo_ref) and np.array_equal(step.cpu().numpy(), step_ref)
    assert np.array_equal(Q.cpu().numpy().astype(np.int32), q_ref)
    assert np.array_equal(qsum.cpu().numpy().astype(np.int64), q_ref.sum(axis=1))


AQ_CASES = [
    # out, in, v, K, M, kind, bits
    (300, 4096, 10, 512, 1, "f16", 8), (5120, 5120, 10, 256, 1, "f16", 8), (2100, 13824, 10, 256, 1, "bf16", 4),
    (777, 1234, 10, 100, 5, "f16", 8), (1030, 2570, 10, 256, 16, "bf16", 8), (260, 810, 9, 1024, 33, "f16", 4),
    (1500, 1600, 10, 256, 300, "bf16", 8), (90, 512, 16, 7132, 40, "f16", 8),
    # enough rows and output tiles to fill the chip: int8 operands on the integer matrix cores (ragged last block
    # of rows, out % 4 != 0, a last k-tile partly past `in`, 4-bit codes, a chunk length other than 10)
    (6007, 400, 10, 256, 1300, "bf16", 8), (6100, 528, 10, 700, 1281, "f16", 4), (6000, 320, 8, 100, 1290, "bf16", 8),
    (9000, 256, 10, 512, 1024, "f16", 8),
]


@pytest.mark.parametrize("out,n_in,v,K,M,kind,bits", AQ_CASES)
def test_layer_on_quantised_activations(G, oracle, out, n_in, v, K, M, kind, bits):
    import torch
    B = G.B
    print(f"gemm_aq out={out} in={n_in} v={v} K={K} M={M} {kind} bits={bits}", flush=True)
    layer, xb = S.make_case(31, out, n_in, v, K, M, x_dtype=kind, outlier_frac=0.01)
    dl = G.DeviceLayer(layer, oracle)
    Q, lo, step, _ = _quantize(G, xb, kind, bits)
    q_ref, lo_ref, step_ref = oracle.quantize_rows(xb, kind, bits)
    assert np.array_equal(Q.cpu().numpy().astype(np.int32), q_ref)
    # sum_k W_hat[i][k]: the oracle's materialised matrix added up row by row
    ws1 = torch.full((B.btc_aq_workspace_bytes(dl.shape, 1),), 0xFF, dtype=torch.uint8, device="cuda")
    wsum = torch.empty(out, dtype=torch.float32, device="cuda")
    B.btc_weight_rowsums(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, wsum, ws1)
    wsum_ref = np.concatenate([oracle.materialise(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, n_in, v, K,
                                                  rows=np.arange(r0, min(out, r0 + 2048))).sum(axis=1)
                               for r0 in range(0, out, 2048)])
    G.assert_close(wsum.cpu().numpy().astype(np.float64)[None, :], wsum_ref[None, :], "row sums of W_hat")
    y_ref = np.concatenate([oracle.linear_aq(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, q_ref, lo_ref,
                                             step_ref, n_in, v, K, rows=np.arange(r0, min(out, r0 + 2048)))
                            for r0 in range(0, out, 2048)], axis=1)
    ws = torch.full((B.btc_aq_workspace_bytes(dl.shape, M),), 0xFF, dtype=torch.uint8, device="cuda")
    for yd, tdt in ((B.BTC_F32, torch.float32), (B.BTC_F16 if kind == "f16" else B.BTC_BF16,
                                                 torch.float16 if kind == "f16" else torch.bfloat16)):
        Y = G.GuardedOutput(M, out, tdt)
        B.btc_gemm_aq(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, wsum, Q, lo, step, M, Y.payload, yd, ws)
        Y.check_guards()
        (G.assert_close_bf16_out if yd == B.BTC_BF16 else G.assert_close)(Y.numpy(), y_ref, "layer on quantised activations")


def test_argument_errors(G):
    import torch
    B = G.B
    from paper_2506_12040_amd import binding as BB
    x = torch.zeros(2, 64, dtype=torch.float16, device="cuda")
    Q = torch.zeros(2, 64, dtype=torch.uint8, device="cuda")
    lo = torch.zeros(4, dtype=torch.float32, device="cuda")
    st = torch.zeros(4, dtype=torch.float32, device="cuda")
    for bits in (0, 3, 16):
        with pytest.raises(BB.BtcError) as e:
            B.btc_quantize_rows(x, B.BTC_F16, 2, 64, bits, Q, lo, st)
        assert e.value.status == BB.BTC_ERR_UNSUPPORTED
    with pytest.raises(BB.BtcError) as e:
        B.btc_quantize_rows(x, B.BTC_F32, 2, 64, 8, Q, lo, st)
    assert e.value.status == BB.BTC_ERR_UNSUPPORTED
    with pytest.raises(BB.BtcError) as e:
        B.btc_quantize_rows(None, B.BTC_F16, 2, 64, 8, Q, lo, st)
    assert e.value.status == BB.BTC_ERR_NULL
    s = B.btc_shape_init(64, 64, 10, 256)
    small = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(BB.BtcError) as e:
        B.btc_gemm_aq(s, Q, Q, lo, lo, lo, Q, lo, st, 2, x, B.BTC_F16, small)
    assert e.value.status == BB.BTC_ERR_WORKSPACE
