"""Every decode engine against the oracle, and the dispatcher's choice against the best engine.

btc_gemv picks one of several engines; since one of them serves most calls, the others are reached here through
the hook btc_gemv_engine, on shapes each of them covers (every output compared with the oracle).  The second
test times every engine that covers a shape, on seeded shapes off the benchmark grid, and asserts that the engine
btc_gemv picks is within 15 % of the fastest one (plus half a microsecond of timer noise)."""
import numpy as np
import pytest

import btc_synth as S

pytestmark = pytest.mark.gpu

ENGINE_NAMES = {1: "expand", 2: "lut", 3: "mfma_one", 4: "mfma", 5: "tiled", 6: "generic", 7: "fp4", 8: "code"}


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_util
    return gpu_util


def _run_engine(G, dl, x, engine, y_dtype=None, dirty_ws=False):
    import torch
    B = G.B
    from paper_2506_12040_amd import binding as BB
    batch = x.shape[0]
    y_dtype = BB.BTC_F32 if y_dtype is None else y_dtype
    y = G.GuardedOutput(batch, dl.layer.out, torch.float32 if y_dtype == BB.BTC_F32 else torch.float16)
    ws = torch.zeros(max(16, B.btc_workspace_bytes(dl.shape, batch, False)), dtype=torch.uint8, device="cuda")
    try:
        BB.btc_gemv_engine(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, G.dev(x), batch, y.payload, y_dtype, engine, ws)
    except BB.BtcError as e:
        if e.status == BB.BTC_ERR_UNSUPPORTED:
            return None
        raise
    y.check_guards()
    assert int(ws.count_nonzero()) == 0, "engine did not hand the workspace back zero-filled"
    return y.numpy()


ENGINE_CASES = [
    # out, in, v, K, batch, dist
    (300, 4096, 10, 512, 1, "uniform"), (129, 5120, 10, 256, 1, "zipf"), (200, 8192, 9, 1024, 1, "uniform"),
    (200, 8192, 10, 128, 1, "uniform"), (70, 13824, 10, 256, 1, "zipf"), (260, 11008, 10, 512, 1, "uniform"),
    (1, 10, 10, 512, 1, "uniform"), (33, 1003, 10, 512, 1, "uniform"), (523, 5128, 10, 100, 1, "uniform"),
    (5000, 4096, 10, 512, 1, "uniform"), (9000, 2000, 10, 256, 1, "uniform"), (17, 15360, 10, 512, 1, "uniform"),
    (300, 5000, 9, 512, 1, "uniform"), (77, 2701, 9, 300, 1, "zipf"), (2100, 12006, 9, 1024, 1, "uniform"),
    (96, 4096, 10, 512, 4, "uniform"), (131, 6408, 10, 256, 7, "zipf"), (50, 333, 4, 9, 1, "uniform"),
    (31, 260, 8, 85, 2, "uniform"), (40, 330, 16, 7132, 4, "uniform"), (1030, 10240, 10, 256, 16, "uniform"),
    # long vectors and large codebooks (the vector-length study's settings): codebook in LDS as 16-bit or 32-bit
    # patterns, or gathered from memory; ragged last chunk, more chunks than one per lane, an odd number of rows
    (1500, 4096, 16, 65536, 1, "uniform"), (700, 3000, 20, 65536, 1, "uniform"), (333, 2050, 12, 3000, 1, "zipf"),
    (4099, 1234, 14, 9000, 1, "uniform"), (64, 16000, 18, 32768, 1, "uniform"), (257, 998, 6, 40, 1, "uniform"),
    (90, 5000, 32, 100, 1, "uniform"),
]


@pytest.mark.parametrize("out,n_in,v,K,batch,dist", ENGINE_CASES)
def test_every_engine_matches_the_oracle(G, oracle, out, n_in, v, K, batch, dist):
    print(f"engines out={out} in={n_in} v={v} K={K} batch={batch} {dist}", flush=True)
    layer, x = S.make_case(21, out, n_in, v, K, batch, dist=dist, outlier_frac=0.01)
    dl = G.DeviceLayer(layer, oracle)
    y_ref = G.oracle_all_rows(oracle, dl, x)
    ran = []
    for engine in sorted(ENGINE_NAMES):
        y = _run_engine(G, dl, x, engine)
        if y is None:
            continue
        G.assert_close(y, y_ref, f"engine {ENGINE_NAMES[engine]}")
        ran.append(ENGINE_NAMES[engine])
    print("   covered by:", ", ".join(ran), flush=True)
    assert "generic" in ran


def test_fp4_engine_is_exact_on_integers(G, oracle):
    """The four E5M2 pieces of a (block-scaled) fp16 number add up to it exactly and +-1 is exact in E2M1, so
    small-integer activations give the exact integer row sums, and a single non-zero activation -- a subnormal,
    the largest finite number, a value with all eleven significant bits set -- comes back bit for bit."""
    from paper_2506_12040_amd import binding as BB
    v, out, n_in = 10, 200, 3000
    K = 1 << v
    rng = np.random.default_rng(5)
    Sg = np.where(rng.normal(size=(out, n_in)) >= 0, 1.0, -1.0)
    bits = (Sg > 0).astype(np.int64).reshape(out, n_in // v, v)
    idx = (bits << np.arange(v)).sum(axis=2).astype(np.int32)
    layer = S.Layer(out, n_in, v, K, np.arange(K, dtype=np.uint32), idx, np.ones(out, np.float32), np.zeros(out, np.float32))
    dl = G.DeviceLayer(layer, oracle)
    xi = rng.integers(-64, 65, size=(1, n_in)).astype(np.float16)
    y = _run_engine(G, dl, xi.view(np.uint16), BB.BTC_ENGINE_FP4)
    assert y is not None and np.array_equal(y, xi.astype(np.float64) @ Sg.T)
    # one non-zero activation at a time: the product is +-x itself, bit for bit
    for val in (np.float16(2047.0), np.float16(6e-8), np.float16(65504.0), np.float16(-0.333251953125)):
        xs = np.zeros((1, n_in), np.float16)
        xs[0, 1234] = val
        y = _run_engine(G, dl, xs.view(np.uint16), BB.BTC_ENGINE_FP4)
        assert np.array_equal(y[0], Sg[:, 1234] * np.float64(val)), val
    # activations of very different magnitudes in one row: tiny ones next to a huge one lose nothing that fp32
    # accumulation would keep, and an all-tiny row is as accurate as an ordinary one
    for scale in (1.0, 2.0 ** -12, 2.0 ** -20, 300.0):
        xs = (rng.normal(size=(1, n_in)) * scale).astype(np.float16)
        y = _run_engine(G, dl, xs.view(np.uint16), BB.BTC_ENGINE_FP4)
        ref = xs.astype(np.float64) @ Sg.T
        assert np.linalg.norm(y - ref) <= 3e-6 * np.linalg.norm(ref), scale


def _off_grid_shapes(seed, n):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        v, K = [(10, 512), (10, 256), (10, 128), (9, 1024), (10, 1024), (9, 512)][int(rng.integers(0, 6))]
        out = int(rng.choice([int(rng.integers(600, 3000)), int(rng.integers(3000, 9000)), int(rng.integers(9000, 30000))]))
        n_in = 2 * int(rng.choice([int(rng.integers(1000, 3000)), int(rng.integers(3000, 7000)), int(rng.integers(7000, 15000))]))
        shapes.append((out, n_in, v, K))
    return shapes


@pytest.mark.parametrize("out,n_in,v,K", _off_grid_shapes(20250701, 20))
def test_dispatcher_picks_a_near_best_engine(G, oracle, out, n_in, v, K):
    """Times btc_gemv (engine 0) and every engine that covers the shape for one activation row, on a matrix that
    is streamed from memory (rotating copies), and compares."""
    import torch
    from paper_2506_12040_amd import binding as BB
    print(f"engine choice out={out} in={n_in} v={v} K={K}", flush=True)
    s = BB.btc_shape_init(out, n_in, v, K)
    layer, x = S.make_case(33, min(out, 512), n_in, v, K, 1)
    ph = oracle.pack(layer.idx, K)
    base = torch.from_numpy(np.tile(ph, (-(-out // ph.shape[0]), 1))[:out].view(np.int32).copy()).cuda()
    nbytes = out * s.words_per_row * 4
    ncopies = int(min(24, max(4, -(-(300 << 20) // nbytes))))       # more than the 256 MB last-level cache in total
    copies = [torch.roll(base, shifts=(c * 37 + 1) % out, dims=0).contiguous() for c in range(ncopies)]
    cb = np.zeros(1 << s.b, np.uint32)
    cb[:K] = layer.codebook
    cbd, xd = G.dev(cb), G.dev(x)
    al, mu = G.dev(np.resize(layer.alpha, out)), G.dev(np.resize(layer.mu, out))
    y = torch.empty(out, dtype=torch.float16, device="cuda")
    ws = torch.zeros(max(16, BB.btc_workspace_bytes(s, 1, False)), dtype=torch.uint8, device="cuda")
    times = {}
    for engine in [0] + sorted(ENGINE_NAMES):
        if engine in (5, 6):        # the prefill kernel and the fallback are never candidates for one row here
            continue
        try:
            BB.btc_gemv_engine(s, copies[0], cbd, al, mu, xd, 1, y, BB.BTC_F16, engine, ws)
        except BB.BtcError as e:
            assert e.status == BB.BTC_ERR_UNSUPPORTED
            continue
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for c in copies:
                BB.btc_gemv_engine(s, c, cbd, al, mu, xd, 1, y, BB.BTC_F16, engine, ws)
        best = 1e9
        for _ in range(3):
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(4):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / (4 * ncopies))
        times[engine] = best
    assert int(ws.count_nonzero()) == 0
    chosen = times.pop(0)
    fastest = min(times.values())
    print("   btc_gemv %.2f us; " % chosen + ", ".join(f"{ENGINE_NAMES[e]} {t:.2f}" for e, t in sorted(times.items())), flush=True)
    assert chosen <= 1.15 * fastest + 0.5, (chosen, times)
