"""GPU parity on seeded random shapes against the CPU oracle (every output; for the largest btc_gemm cases
sampled weight rows for all activation rows plus all weight rows for a band of activation rows).  First set: the engines
that feed table entries straight into matrix-core operands (2..16 activation rows, one row on wide matrices,
btc_gemm with up to 64 rows).  Second set: every other route -- 65..128 rows on large matrices, the tiled
kernel at any M, one row with arbitrary chunk length and codebook size, btc_gemm on settings only the generic
kernel covers.  Third set: btc_transform, btc_assign and btc_update on random sizes.  Shapes are drawn so that ragged row tiles, ragged last chunks, activation rows
that are not 16-byte aligned and every supported index width come up; the tolerances are those of the other
parity tests."""
import numpy as np
import pytest

import btc_synth as S

pytestmark = pytest.mark.gpu

K_OF = {10: [100, 128, 200, 256, 300, 512, 700, 1024], 9: [128, 256, 512]}


def _cases(seed, n):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        v = 10 if rng.random() < 0.75 else 9
        K = int(rng.choice(K_OF[v]))
        out = int(rng.integers(1, 3000))
        n_in = 2 * int(rng.integers(300, 9000))
        mode = int(rng.integers(0, 4))
        s = int(rng.integers(1, 1000))
        if mode == 0:      # several rows on the decode engine
            cases.append(("gemv", s, out, n_in, v, K, int(rng.integers(3, 17)), "f16"))
        elif mode == 1:    # btc_gemm with few rows
            cases.append(("gemm", s, out, n_in, v, K, int(rng.integers(1, 65)), "bf16" if rng.random() < 0.6 else "f16"))
        elif mode == 2:    # one row, wide matrix, 9 or 10 index bits
            Kw = int(rng.choice([300, 512, 700, 1024] if v == 10 else [300, 512]))
            cases.append(("gemv", s, int(rng.integers(1, 2000)), 2 * int(rng.integers(5200, 12000)), v, Kw, 1, "f16"))
        else:              # two rows
            cases.append(("gemv", s, out, n_in, v, K, 2, "f16"))
    return cases


def _wide_cases(seed, n):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        mode = int(rng.integers(0, 4))
        s = int(rng.integers(1, 1000))
        xd = "bf16" if rng.random() < 0.6 else "f16"
        if mode == 0:      # 65..128 rows, 6 MB of indices or more
            cases.append(("gemm", s, int(rng.integers(3000, 8200)), 16 * int(rng.integers(400, 1000)), 10,
                          int(rng.choice([128, 256, 512, 1024])), int(rng.integers(65, 129)), xd))
        elif mode == 1:    # tiled kernel, ragged M and out
            cases.append(("gemm", s, int(rng.integers(1, 3000)), 16 * int(rng.integers(40, 600)), 10,
                          int(rng.choice([100, 256, 512, 1024])), int(rng.integers(129, 700)), xd))
        elif mode == 2:    # one row, any chunk length and codebook size
            v = int(rng.choice([4, 7, 8, 9, 10, 12, 16]))
            K = int(rng.integers(2, min(2 ** v, 4096) + 1))
            cases.append(("gemv", s, int(rng.integers(1, 9000)), int(rng.integers(20, 15000)), v, K, 1, "f16"))
        else:              # btc_gemm outside the tuned settings
            v = int(rng.choice([4, 8, 9, 12]))
            K = int(rng.integers(2, min(2 ** v, 2048) + 1))
            cases.append(("gemm", s, int(rng.integers(1, 1500)), int(rng.integers(20, 4000)), v, K,
                          int(rng.integers(1, 200)), "bf16"))
    return cases


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_util
    return gpu_util


@pytest.mark.parametrize("kind,seed,out,n_in,v,K,rows,xd", _cases(20250612, 28) + _wide_cases(20250613, 24))
def test_random_shape(G, oracle, kind, seed, out, n_in, v, K, rows, xd):
    B = G.B
    print(f"random {kind} seed={seed} out={out} in={n_in} v={v} K={K} rows={rows} {xd}", flush=True)
    layer, x = S.make_case(seed, out, n_in, v, K, rows, x_dtype=xd)
    dl = G.DeviceLayer(layer, oracle)
    if kind == "gemv":       # every output
        y = G.gemv(dl, x, B.BTC_F32)
        G.assert_close(y, G.oracle_all_rows(oracle, dl, x, xd), f"{kind} {out}x{n_in} v{v} K{K} rows={rows} {xd}")
        return
    y = G.gemm(dl, x, B.BTC_BF16 if xd == "bf16" else B.BTC_F16, B.BTC_F32)
    if rows * out * n_in <= 6e9:     # every output where the oracle's plain loop takes seconds
        G.assert_close(y, G.oracle_all_rows(oracle, dl, x, xd), f"{kind} {out}x{n_in} v{v} K{K} rows={rows} {xd}")
        return
    rng = np.random.default_rng(seed)
    sel = np.unique(np.concatenate([[0, out - 1], rng.choice(out, size=min(96, out), replace=False)]))
    y_ref = oracle.linear(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, x, n_in, v, K, rows=sel, x_kind=xd)
    G.assert_close(y[:, sel], y_ref, f"{kind} {out}x{n_in} v{v} K{K} rows={rows} {xd}")
    band = np.unique(np.concatenate([[0, rows - 1], rng.choice(rows, size=min(8, rows), replace=False)]))
    G.assert_close(y[band], G.oracle_all_rows(oracle, dl, x[band], xd), f"{kind} band of activation rows")


def _aux_cases(seed, n):
    """Seeded random calls of btc_transform, btc_assign and btc_update."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        s = int(rng.integers(1, 100000))
        if rng.random() < 0.4:
            n2 = int(rng.choice([int(rng.integers(1, 257)), 16 * int(rng.integers(1, 17)), 8 * int(rng.integers(1, 33))]))
            cases.append(("transform", s, int(rng.integers(1, 129)), n2, int(rng.choice([1, 2, 5, 16, 40, 64, 65, 100, 300])),
                          "bf16" if rng.random() < 0.6 else "f16", str(rng.choice(["f32", "f16", "bf16"]))))
        else:
            K = int(rng.choice([1, 2, 3, 17, 128, 256, 512, 1000, 1024, 4096, 20000]))
            N = int(rng.choice([1, 3, 255, 1024, 4099, 70001, 300007])) if K <= 4096 else int(rng.choice([1, 1000, 5003]))
            cases.append(("cluster", s, N, int(rng.choice([1, 2, 4, 7, 9, 10, 11, 12, 13, 16, 20, 32])), K, "", ""))
    return cases


@pytest.mark.parametrize("kind,seed,a,b,c,xd,yd", _aux_cases(20250614, 40))
def test_random_transform_and_clustering_calls(G, oracle, kind, seed, a, b, c, xd, yd):
    import torch
    B = G.B
    rng = np.random.default_rng(seed)
    print(f"random {kind} seed={seed} {a} {b} {c} {xd} {yd}", flush=True)
    if kind == "transform":
        n1, n2, M = a, b, c
        y_dtype = {"f32": B.BTC_F32, "f16": B.BTC_F16, "bf16": B.BTC_BF16}[yd]
        bits, P1, P2 = S.draw_transform(seed, n1, n2)
        xb = S.draw_x(rng, M, n1 * n2, xd)
        out = G.GuardedOutput(M, n1 * n2, {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[yd])
        B.btc_transform(G.dev(xb), B.BTC_BF16 if xd == "bf16" else B.BTC_F16, M, n1, n2, G.dev(bits), G.dev(P1), G.dev(P2),
                        out.payload, y_dtype)
        out.check_guards()
        y = out.numpy()
        rows = np.unique(rng.integers(0, M, size=min(M, 4 if n1 * n2 > 4000 else 16)))
        ref = oracle.transform(xb[rows], bits, P1, P2, xd)
        rel = np.linalg.norm(y[rows] - ref) / np.linalg.norm(ref)
        mabs = np.max(np.abs(y[rows] - ref)) / np.max(np.abs(ref))
        tol = (1e-5, 1e-5) if yd == "f32" else (2e-3, 1e-2)
        assert rel <= tol[0] and mabs <= tol[1] and np.isfinite(y).all(), (rel, mabs)
        return
    N, v, K = a, b, c
    mask = np.uint32((1 << v) - 1 if v < 32 else 0xFFFFFFFF)
    cb = (rng.integers(0, 1 << 32, size=K, dtype=np.uint64).astype(np.uint32)) & mask
    vec = rng.integers(0, 1 << 32, size=N, dtype=np.uint64).astype(np.uint32)
    if rng.random() < 0.5:      # near the centroids, junk above bit v
        vec = (cb[rng.integers(0, K, size=N)] ^ (np.uint32(1) << rng.integers(0, v, size=N).astype(np.uint32))) | (vec & ~mask)
    z = G.GuardedOutput(1, N, torch.int32)
    d = G.GuardedOutput(1, N, torch.int32)
    B.btc_assign(G.dev(vec), N, v, G.dev(cb), K, z.payload, d.payload)
    z.check_guards()
    d.check_guards()
    z_ref, d_ref = oracle.assign(vec, v, cb)
    assert np.array_equal(z.payload.cpu().numpy(), z_ref) and np.array_equal(d.payload.cpu().numpy(), d_ref)
    if N * K <= 4e8:
        zz = z_ref if rng.random() < 0.5 else rng.integers(0, K, size=N).astype(np.int32)
        ws = torch.zeros(B.btc_update_workspace_bytes(v, K), dtype=torch.uint8, device="cuda")
        cbd = G.dev(cb.copy())
        B.btc_update(G.dev(vec), G.dev(zz), N, v, cbd, K, ws)
        torch.cuda.synchronize()
        assert not bool(ws.any())
        assert np.array_equal(cbd.cpu().numpy().view(np.uint32), oracle.update(vec, zz, v, cb))
