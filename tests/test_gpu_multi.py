"""GPU parity of btc_gemv_multi (up to four matrices of one shape on one activation row, one launch where the
engine on the 4-bit matrix cores covers the setting): every output of every matrix against the oracle, and bit for
bit against that engine's result for each matrix alone; settings the engine does not cover run as separate calls."""
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


# out, in, v, K, count
CASES = [
    (5120, 5120, 10, 256, 3), (13824, 5120, 10, 256, 2), (1024, 8192, 10, 512, 2), (4096, 4096, 10, 512, 4),
    (33, 4100, 10, 128, 3), (2000, 1230, 9, 1024, 4), (5120, 13824, 10, 256, 2), (16, 640, 10, 256, 4),
    (2048, 28672, 10, 128, 2), (300, 999, 7, 100, 3), (700, 2048, 16, 4096, 2), (5120, 5120, 10, 256, 1),
]


@pytest.mark.parametrize("out,n_in,v,K,count", CASES)
def test_multi_matches_the_oracle_and_the_single_calls(G, oracle, out, n_in, v, K, count):
    import torch
    B = G.B
    from paper_2506_12040_amd import binding as BB
    print(f"gemv_multi out={out} in={n_in} v={v} K={K} count={count}", flush=True)
    layers = []
    x = None
    for m in range(count):
        layer, xm = S.make_case(70 + m, out, n_in, v, K, 1)
        layers.append(G.DeviceLayer(layer, oracle))
        x = xm if x is None else x
    x_d = G.dev(x)
    shape = layers[0].shape
    ws = torch.zeros(B.btc_workspace_bytes(shape, 1, False), dtype=torch.uint8, device="cuda")
    for yd, tdt in ((B.BTC_F32, torch.float32), (B.BTC_F16, torch.float16)):
        Ys = [G.GuardedOutput(1, out, tdt) for _ in range(count)]
        B.btc_gemv_multi(shape, [l.packed for l in layers], [l.codebook for l in layers], [l.alpha for l in layers],
                         [l.mu for l in layers], x_d, [Y.payload for Y in Ys], yd, ws)
        for m, (l, Y) in enumerate(zip(layers, Ys)):
            Y.check_guards()
            G.assert_close(Y.numpy(), G.oracle_all_rows(oracle, l, x), f"matrix {m}")
            if count == 1:
                continue                      # a single matrix is an ordinary btc_gemv call
            y1 = torch.empty(out, dtype=tdt, device="cuda")
            try:
                B.btc_gemv_engine(shape, l.packed, l.codebook, l.alpha, l.mu, x_d, 1, y1, yd, 7, ws)
            except BB.BtcError:
                continue                      # the engine does not cover the setting: separate calls were made
            assert torch.equal(y1, Y.payload.view(-1)), f"matrix {m}: one launch and single call differ"


# outs, in, v, K: matrices that differ in their number of rows only (q, k, v under grouped-query attention: the 70B
# shapes at the three bit settings; ragged and tiny row counts; a setting the one-launch engine does not cover)
ROWS_CASES = [
    ((8192, 1024, 1024), 8192, 10, 512), ((8192, 1024, 1024), 8192, 9, 1024), ((8192, 1024, 1024), 8192, 10, 128),
    ((33, 700, 16, 5), 4100, 10, 128), ((4096, 17), 4096, 10, 512), ((1, 5120), 5120, 10, 256),
    ((5000, 5120, 40), 13824, 10, 256), ((300, 64), 999, 7, 100),
]


@pytest.mark.parametrize("outs,n_in,v,K", ROWS_CASES)
def test_multi_shapes_matches_the_oracle_and_the_single_calls(G, oracle, outs, n_in, v, K):
    import torch
    B = G.B
    from paper_2506_12040_amd import binding as BB
    print(f"gemv_multi_shapes outs={outs} in={n_in} v={v} K={K}", flush=True)
    layers = []
    x = None
    for m, out in enumerate(outs):
        layer, xm = S.make_case(90 + m, out, n_in, v, K, 1)
        layers.append(G.DeviceLayer(layer, oracle))
        x = xm if x is None else x
    x_d = G.dev(x)
    ws = torch.zeros(max(B.btc_workspace_bytes(l.shape, 1, False) for l in layers), dtype=torch.uint8, device="cuda")
    for yd, tdt in ((B.BTC_F32, torch.float32), (B.BTC_F16, torch.float16)):
        Ys = [G.GuardedOutput(1, out, tdt) for out in outs]
        B.btc_gemv_multi_shapes([l.shape for l in layers], [l.packed for l in layers], [l.codebook for l in layers],
                                [l.alpha for l in layers], [l.mu for l in layers], x_d, [Y.payload for Y in Ys], yd, ws)
        for m, (l, Y) in enumerate(zip(layers, Ys)):
            Y.check_guards()
            G.assert_close(Y.numpy(), G.oracle_all_rows(oracle, l, x), f"matrix {m}")
            y1 = torch.empty(outs[m], dtype=tdt, device="cuda")
            try:
                B.btc_gemv_engine(l.shape, l.packed, l.codebook, l.alpha, l.mu, x_d, 1, y1, yd, 7, ws)
            except BB.BtcError:
                continue                      # the engine does not cover the setting: separate calls were made
            assert torch.equal(y1, Y.payload.view(-1)), f"matrix {m}: one launch and single call differ"


def test_configuration_2_as_the_benchmark_launches_it(G, oracle):
    """The 13B decoder-layer step the way bench.py launches it: q, k, v (three copies of the 5120x5120 layer of the
    recipe, rows rotated as the benchmark rotates them) in one launch, gate and up (two copies of 13824x5120) in
    one launch; Zipf(1.1) indices; every output of every matrix against the oracle."""
    import torch
    B = G.B
    cases = [c for c in S.config_cases(2)]
    for case, count in ((cases[0], 3), (cases[1], 2)):
        layer, x = S.make_case(**case)
        print(f"config 2 grouped: {layer.out}x{layer.n_in} x {count}", flush=True)
        dl = G.DeviceLayer(layer, oracle)
        shifts = [((L * 7 + r * 3 + 1) * 37) % layer.out for (L, r) in ((0, 0), (0, 1), (1, 2))][:count]
        packed2d = dl.packed.view(layer.out, -1)
        copies = [torch.roll(packed2d, shifts=sft, dims=0).contiguous() for sft in shifts]
        ws = torch.zeros(B.btc_workspace_bytes(dl.shape, 1, False), dtype=torch.uint8, device="cuda")
        Ys = [G.GuardedOutput(1, layer.out, torch.float16) for _ in range(count)]
        B.btc_gemv_multi(dl.shape, copies, [dl.codebook] * count, [dl.alpha] * count, [dl.mu] * count, G.dev(x),
                         [Y.payload for Y in Ys], B.BTC_F16, ws)
        for sft, Y in zip(shifts, Ys):
            Y.check_guards()
            # rolling the packed rows by s moves weight row i to row i + s: y[i + s] = alpha[i + s] * d[i] + mu[i + s] * sum(x);
            # the oracle of the rolled matrix is computed from the rolled index matrix
            rolled = np.roll(dl.packed_host, sft, axis=0)
            y_ref = np.concatenate([oracle.linear(rolled, dl.codebook_host, layer.alpha, layer.mu, x, layer.n_in, layer.v,
                                                  layer.K, rows=np.arange(r0, min(layer.out, r0 + 4096)))
                                    for r0 in range(0, layer.out, 4096)], axis=1)
            G.assert_close(Y.numpy(), y_ref, f"rolled by {sft}")


def test_argument_errors(G):
    import torch
    B = G.B
    from paper_2506_12040_amd import binding as BB
    s = B.btc_shape_init(64, 640, 10, 256)
    t = torch.zeros(1 << 14, dtype=torch.int32, device="cuda")
    with pytest.raises(BB.BtcError) as e:
        B.btc_gemv_multi(s, [t] * 5, [t] * 5, [t] * 5, [t] * 5, t, [t] * 5, B.BTC_F32, t)
    assert e.value.status == BB.BTC_ERR_UNSUPPORTED
    with pytest.raises(BB.BtcError) as e:
        B.btc_gemv_multi(s, [t, None], [t, t], [t, t], [t, t], t, [t, t], B.BTC_F32, t)
    assert e.value.status == BB.BTC_ERR_NULL
    s2 = B.btc_shape_init(32, 650, 10, 256)       # another row length: not one launch, not one input
    with pytest.raises(BB.BtcError) as e:
        B.btc_gemv_multi_shapes([s, s2], [t, t], [t, t], [t, t], [t, t], t, [t, t], B.BTC_F32, t)
    assert e.value.status == BB.BTC_ERR_SHAPE
    s3 = B.btc_shape_init(32, 640, 10, 128)       # another codebook size
    with pytest.raises(BB.BtcError) as e:
        B.btc_gemv_multi_shapes([s, s3], [t, t], [t, t], [t, t], [t, t], t, [t, t], B.BTC_F32, t)
    assert e.value.status == BB.BTC_ERR_SHAPE
