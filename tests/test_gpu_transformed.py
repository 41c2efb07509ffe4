"""GPU parity of btc_gemv_transformed (the decode product behind the online activation transform, one call) against
the oracle: y = linear(fp16(transform(x))), every output.  Cases the fused engine covers (factors 64 x 64 and
64 x 80 with v = 10, 7..10 index bits, few and many rows, tiny and large activations) and cases that run as two
launches (other factor sizes, v = 9, long vectors, no prepared operands).  The fused result is also held against
the two-launch result of the library itself, which differs only where the fp16 rounding of a transformed
activation falls the other way, and the transformed row it hands out against a product computed from it."""
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


# out, n1, n2, v, K, prepared?, activation scale
CASES = [
    (5120, 64, 80, 10, 256, True, 1.0), (13824, 64, 80, 10, 256, True, 1.0), (5120, 108, 128, 10, 256, True, 1.0),
    (4096, 64, 64, 10, 512, True, 1.0), (1000, 86, 128, 10, 128, True, 1.0), (2048, 64, 128, 10, 1024, True, 1.0),
    (33, 64, 64, 10, 128, True, 1.0), (11008, 64, 64, 10, 1024, True, 1.0), (1234, 64, 80, 10, 700, True, 1.0),
    (300, 37, 48, 10, 256, True, 1.0), (64, 5, 16, 10, 256, True, 1.0), (777, 128, 128, 10, 200, True, 1.0),
    (5120, 64, 80, 10, 256, True, 2.0 ** -12), (5120, 64, 80, 10, 256, True, 300.0),
    (5120, 64, 80, 10, 256, False, 1.0), (3000, 64, 81, 9, 256, True, 1.0), (512, 50, 50, 10, 256, True, 1.0),
    (700, 64, 80, 16, 4096, True, 1.0), (2000, 128, 224, 10, 512, True, 1.0),
]


def _fp16_bits(a):
    return np.ascontiguousarray(a.astype(np.float16)).view(np.uint16)


def _same_up_to_rounding(got, ref, n):
    """Two fp16 rows that should be the same rounding of the same numbers: a few elements (about one in a thousand:
    those within the arithmetic's error of a rounding boundary) may fall to the neighbouring fp16 value, none
    further -- except outputs that are tiny next to the row (cancellation), which are held to the absolute error
    of the fp32 sums, 1e-6 of the row's largest element."""
    diff = np.nonzero(got != ref)[0]
    assert len(diff) <= max(4, n // 200), len(diff)
    g = got[diff].view(np.float16).astype(np.float64)
    r = ref[diff].view(np.float16).astype(np.float64)
    big = np.max(np.abs(ref.view(np.float16).astype(np.float64)))
    assert np.all(np.abs(g - r) <= np.maximum(np.abs(r) * 2.0 ** -10, 1e-6 * big)), (g, r)


@pytest.mark.parametrize("out,n1,n2,v,K,prep,scale", CASES)
def test_transformed_layer_matches_the_oracle(G, oracle, out, n1, n2, v, K, prep, scale):
    import torch
    B = G.B
    n = n1 * n2
    print(f"gemv_transformed out={out} n1={n1} n2={n2} v={v} K={K} prepared={prep} scale={scale}", flush=True)
    layer, x = S.make_case(53, out, n, v, K, 1)
    if scale != 1.0:
        x = _fp16_bits(x.view(np.float16).astype(np.float64) * scale)
    bits, P1, P2 = S.draw_transform(11 + n1 + n2, n1, n2)
    dl = G.DeviceLayer(layer, oracle)
    xt = oracle.transform(x, bits, P1, P2, "f16")                       # float64 [1][n]
    xt_bits = _fp16_bits(xt)
    y_ref = np.concatenate([oracle.linear(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, xt_bits, n, v, K,
                                          rows=np.arange(r0, min(out, r0 + 2048))) for r0 in range(0, out, 2048)], axis=1)
    P1_d, P2_d, bits_d, x_d = G.dev(P1), G.dev(P2), G.dev(bits), G.dev(x)
    prepared = None
    nb = B.btc_transform_prepared_bytes(n1, n2)
    if prep and nb:
        prepared = torch.full((nb,), 0x7F, dtype=torch.uint8, device="cuda")
        B.btc_transform_prepare(n1, n2, P1_d, P2_d, prepared)
    ws = torch.zeros(B.btc_gemv_transformed_workspace_bytes(dl.shape), dtype=torch.uint8, device="cuda")
    # the fused engine needs no workspace; the two launches refuse to run without one
    fused = prepared is not None and v == 10 and 128 <= K <= 1024 and (n1, n2) in ((64, 64), (64, 80))
    # prepared operands exist for the fused pairs and for the pairs with a matrix-core kernel for one row
    assert (nb > 0) == ((n1, n2) in ((64, 64), (64, 80), (64, 128), (86, 128), (108, 128)))
    if not fused:
        from paper_2506_12040_amd import binding as BB
        with pytest.raises(BB.BtcError) as e:
            B.btc_gemv_transformed(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, x_d, n1, n2, bits_d, P1_d, P2_d,
                                   prepared, torch.empty(out, dtype=torch.float32, device="cuda"), B.BTC_F32, None)
        assert e.value.status == BB.BTC_ERR_WORKSPACE
    ys = {}
    for yd, tdt in ((B.BTC_F32, torch.float32), (B.BTC_F16, torch.float16)):
        Y = G.GuardedOutput(1, out, tdt)
        XT = G.GuardedOutput(1, n, torch.float16)
        B.btc_gemv_transformed(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, x_d, n1, n2, bits_d, P1_d, P2_d,
                               prepared, Y.payload, yd, None if fused else ws, xt_out=XT.payload if yd == B.BTC_F32 else None)
        Y.check_guards()
        XT.check_guards()
        ys[yd] = Y.numpy()
        G.assert_close(ys[yd], y_ref, "transformed layer")
        if yd == B.BTC_F32:
            # the row handed out: the oracle's up to the rounding of a few elements, and exactly the row the product used
            got = XT.payload.cpu().numpy().view(np.uint16)
            _same_up_to_rounding(got, xt_bits[0], n)
            Y3 = torch.empty(out, dtype=torch.float32, device="cuda")
            ws3 = torch.zeros(B.btc_workspace_bytes(dl.shape, 1, False), dtype=torch.uint8, device="cuda")
            if fused:
                B.btc_gemv_engine(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, XT.payload, 1, Y3, B.BTC_F32, 7, ws3)
                assert torch.equal(Y3, Y.payload.view(-1)), "fused product and product of the stored row differ"
    # the library's own two launches
    xt_d = torch.empty(n, dtype=torch.float16, device="cuda")
    B.btc_transform(x_d, B.BTC_F16, 1, n1, n2, bits_d, P1_d, P2_d, xt_d, B.BTC_F16)
    ws2 = torch.zeros(B.btc_workspace_bytes(dl.shape, 1, False), dtype=torch.uint8, device="cuda")
    Y2 = torch.empty(out, dtype=torch.float32, device="cuda")
    B.btc_gemv(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, xt_d, 1, Y2, B.BTC_F32, ws2)
    y2 = Y2.cpu().numpy().astype(np.float64)[None, :]
    rel = np.linalg.norm(ys[B.BTC_F32] - y2) / np.linalg.norm(y2)
    assert rel <= 2e-4, rel
    # the transformed row itself, rounded: at most a few elements may differ from the oracle's rounding, by one ulp
    got = xt_d.cpu().numpy().view(np.uint16)
    _same_up_to_rounding(got, xt_bits[0], n)


@pytest.mark.parametrize("out,n1,n2,K,count", [(5120, 64, 80, 256, 3), (13824, 64, 80, 256, 2), (1000, 64, 64, 512, 4),
                                                (3000, 108, 128, 256, 2), (400, 7, 32, 256, 3)])
def test_grouped_transformed_layer(G, oracle, out, n1, n2, K, count):
    """Several matrices behind one transformed row: every output of every matrix against the oracle; where the fused
    engine covers the setting the result is bit for bit that of the single fused calls."""
    import torch
    B = G.B
    n, v = n1 * n2, 10
    print(f"gemv_transformed_multi out={out} n1={n1} n2={n2} K={K} count={count}", flush=True)
    layers, x = [], None
    for m in range(count):
        layer, xm = S.make_case(90 + m, out, n, v, K, 1)
        layers.append(G.DeviceLayer(layer, oracle))
        x = xm if x is None else x
    bits, P1, P2 = S.draw_transform(5 + n1, n1, n2)
    xt_bits = _fp16_bits(oracle.transform(x, bits, P1, P2, "f16"))
    P1_d, P2_d, bits_d, x_d = G.dev(P1), G.dev(P2), G.dev(bits), G.dev(x)
    nb = B.btc_transform_prepared_bytes(n1, n2)
    prepared = None
    if nb:
        prepared = torch.empty(nb, dtype=torch.uint8, device="cuda")
        B.btc_transform_prepare(n1, n2, P1_d, P2_d, prepared)
    shape = layers[0].shape
    ws = torch.zeros(B.btc_gemv_transformed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    Ys = [G.GuardedOutput(1, out, torch.float32) for _ in range(count)]
    B.btc_gemv_transformed_multi(shape, [l.packed for l in layers], [l.codebook for l in layers],
                                 [l.alpha for l in layers], [l.mu for l in layers], x_d, n1, n2, bits_d, P1_d, P2_d,
                                 prepared, [Y.payload for Y in Ys], B.BTC_F32, ws)
    fused = (n1, n2) in ((64, 64), (64, 80))
    for m, (l, Y) in enumerate(zip(layers, Ys)):
        Y.check_guards()
        G.assert_close(Y.numpy(), G.oracle_all_rows(oracle, l, xt_bits), f"matrix {m}")
        if fused:
            y1 = torch.empty(out, dtype=torch.float32, device="cuda")
            B.btc_gemv_transformed(shape, l.packed, l.codebook, l.alpha, l.mu, x_d, n1, n2, bits_d, P1_d, P2_d, prepared,
                                   y1, B.BTC_F32, None)
            assert torch.equal(y1, Y.payload.view(-1)), f"matrix {m}: grouped and single fused call differ"


def test_prepare_argument_errors(G):
    import torch
    B = G.B
    from paper_2506_12040_amd import binding as BB
    P = torch.zeros(128 * 128, dtype=torch.float32, device="cuda")
    buf = torch.zeros(1 << 17, dtype=torch.uint8, device="cuda")
    assert B.btc_transform_prepared_bytes(64, 80) > 0 and B.btc_transform_prepared_bytes(64, 81) == 0
    assert B.btc_transform_prepared_bytes(129, 64) == 0 and B.btc_transform_prepared_bytes(64, 144) == 0
    assert B.btc_transform_prepared_bytes(108, 128) == (4 * 8 + 4 * 7) * 2048
    with pytest.raises(BB.BtcError) as e:
        B.btc_transform_prepare(64, 81, P, P, buf)
    assert e.value.status == BB.BTC_ERR_UNSUPPORTED
    with pytest.raises(BB.BtcError) as e:
        B.btc_transform_prepare(64, 80, P, P, buf[:1024])
    assert e.value.status == BB.BTC_ERR_WORKSPACE
    with pytest.raises(BB.BtcError) as e:
        B.btc_transform_prepare(64, 80, P, None, buf)
    assert e.value.status == BB.BTC_ERR_NULL
    s = B.btc_shape_init(64, 5120, 10, 256)
    t = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    with pytest.raises(BB.BtcError) as e:      # n1 n2 != in
        B.btc_gemv_transformed(s, t, t, t, t, t, 64, 64, t, t, t, None, t, B.BTC_F32, t)
    assert e.value.status == BB.BTC_ERR_SHAPE
    with pytest.raises(BB.BtcError) as e:      # the transformed row must not land on the input
        B.btc_gemv_transformed(s, t, t, t, t, t, 64, 80, t, t, t, None, t[4096:], B.BTC_F32, t, xt_out=t)
    assert e.value.status == BB.BTC_ERR_UNSUPPORTED
    with pytest.raises(BB.BtcError) as e:      # two launches need the workspace
        B.btc_gemv_transformed(s, t, t, t, t, t, 64, 80, t, t, t, None, t, B.BTC_F32, None)
    assert e.value.status == BB.BTC_ERR_WORKSPACE
