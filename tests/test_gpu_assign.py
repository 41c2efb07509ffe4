"""GPU parity of btc_assign (E-step: nearest centroid by Hamming distance) against the CPU oracle, through the
C ABI.  Integer work: indices and distances must match bit for bit, ties included (lowest index)."""
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


def _vectors(rng, N, v, cb):
    """Sign patterns clustered around the centroids (a centroid with up to three flipped elements), some exact
    copies, some uniform ones; junk in the bits above v, which the call must ignore."""
    base = cb[rng.integers(0, cb.shape[0], size=N)].astype(np.uint64)
    flips = np.zeros(N, dtype=np.uint64)
    for _ in range(3):
        on = rng.random(N) < 0.4
        flips ^= np.where(on, np.uint64(1) << rng.integers(0, v, size=N).astype(np.uint64), np.uint64(0))
    vec = base ^ flips
    uni = rng.random(N) < 0.2
    vec = np.where(uni, rng.integers(0, 1 << v, size=N, dtype=np.uint64), vec)
    junk = rng.integers(0, 1 << 32, size=N, dtype=np.uint64) & ~np.uint64((1 << v) - 1) & np.uint64(0xFFFFFFFF)
    return (vec | junk).astype(np.uint32)


def _run(G, vec, v, cb, want_dist=True):
    import torch
    B = G.B
    N = vec.shape[0]
    z = G.GuardedOutput(1, N, torch.int32)
    d = G.GuardedOutput(1, N, torch.int32) if want_dist else None
    B.btc_assign(G.dev(vec), N, v, G.dev(cb), cb.shape[0], z.payload, d.payload if d else None)
    z.check_guards()
    zz = z.payload.cpu().numpy()
    if d is None:
        return zz, None
    d.check_guards()
    return zz, d.payload.cpu().numpy()


CASES = [(1, 10, 256), (1023, 10, 256), (100001, 10, 512), (5000, 9, 1024), (4097, 4, 5), (3000, 16, 4096),
         (2000, 20, 65536), (777, 32, 100), (2048, 10, 1), (50000, 10, 128), (1025, 1, 2),
         # many short vectors: the route that assigns the 2^v patterns once and looks the vectors up
         (262147, 12, 1000), (65536, 10, 256), (65535, 10, 256), (40001, 9, 1024), (300, 2, 3)]


@pytest.mark.parametrize("N,v,K", CASES)
def test_assign_matches_oracle(G, oracle, N, v, K):
    print(f"assign N={N} v={v} K={K}", flush=True)
    rng = np.random.default_rng(N + 31 * v + K)
    if 2 <= K <= (1 << min(v, 20)) or (v == 9 and K == 1024):
        cb = S.draw_codebook(rng, v, K)                     # distinct patterns (v = 9, K = 1024: every pattern twice)
    else:
        cb = (rng.integers(0, 1 << 32, size=K, dtype=np.uint64) & np.uint64((1 << v) - 1)).astype(np.uint32)
    vec = _vectors(rng, N, v, cb)
    z, d2 = _run(G, vec, v, cb)
    z_ref, d_ref = oracle.assign(vec, v, cb)
    assert np.array_equal(z, z_ref) and np.array_equal(d2, d_ref)


def test_assign_without_distances(G, oracle):
    rng = np.random.default_rng(5)
    cb = S.draw_codebook(rng, 10, 256)
    vec = _vectors(rng, 3001, 10, cb)
    z, _ = _run(G, vec, 10, cb, want_dist=False)
    assert np.array_equal(z, oracle.assign(vec, 10, cb)[0])


def test_assign_13b_matrix_full_size(G, oracle):
    """All 2 621 440 length-10 vectors of a 5120 x 5120 sign matrix against 256 centroids (the size the benchmark times)."""
    rng = np.random.default_rng(7)
    cb = S.draw_codebook(rng, 10, 256)
    vec = _vectors(rng, 5120 * 512, 10, cb)
    z, d2 = _run(G, vec, 10, cb)
    z_ref, d_ref = oracle.assign(vec, 10, cb)
    assert np.array_equal(z, z_ref) and np.array_equal(d2, d_ref)


# ---- M-step (btc_update): majority vote per cluster, bit-exact

def _update(G, vec, z, v, cb, ws=None):
    import torch
    B = G.B
    K = cb.shape[0]
    if ws is None:
        ws = torch.zeros(B.btc_update_workspace_bytes(v, K), dtype=torch.uint8, device="cuda")
    cbd = G.dev(cb.copy())
    B.btc_update(G.dev(vec), G.dev(z.astype(np.int32)), vec.shape[0], v, cbd, K, ws)
    torch.cuda.synchronize()
    assert not bool(ws.any()), "workspace not handed back zero-filled"
    return cbd.cpu().numpy().view(np.uint32), ws


UPDATE_CASES = [(1, 10, 256), (5000, 10, 256), (100001, 10, 512), (30000, 9, 1024), (4097, 4, 5), (60000, 16, 4096),
                (3000, 20, 65536), (777, 32, 100), (2048, 10, 1), (1025, 1, 2), (400000, 10, 1400)]


@pytest.mark.parametrize("N,v,K", UPDATE_CASES)
def test_update_matches_oracle(G, oracle, N, v, K):
    print(f"update N={N} v={v} K={K}", flush=True)
    rng = np.random.default_rng(N + 7 * v + K)
    cb = (rng.integers(0, 1 << 32, size=K, dtype=np.uint64) & np.uint64((1 << v) - 1)).astype(np.uint32)
    vec = _vectors(rng, N, v, cb)
    z = rng.integers(0, K, size=N).astype(np.int32)
    if K > 2:
        z[z == K // 2] = 0                                   # an empty cluster keeps its centroid
    new, _ = _update(G, vec, z, v, cb)
    assert np.array_equal(new, oracle.update(vec, z, v, cb))


def test_one_clustering_round_on_the_gpu(G, oracle):
    """E-step then M-step on the GPU, twice through one workspace, against the oracle's round."""
    import torch
    rng = np.random.default_rng(21)
    v, K, N = 10, 256, 200000
    cb = S.draw_codebook(rng, v, K)
    vec = _vectors(rng, N, v, cb)
    ws = None
    cb_ref = cb
    for _ in range(2):
        z, _ = _run(G, vec, v, cb_ref)
        z_ref, _ = oracle.assign(vec, v, cb_ref)
        assert np.array_equal(z, z_ref)
        new, ws = _update(G, vec, z, v, cb_ref, ws)
        cb_ref = oracle.update(vec, z_ref, v, cb_ref)
        assert np.array_equal(new, cb_ref)


def test_update_rejects_an_assignment_out_of_range(G):
    import torch
    B = G.B
    rng = np.random.default_rng(22)
    v, K, N = 10, 64, 5000
    cb = S.draw_codebook(rng, v, K)
    vec = rng.integers(0, 1 << v, size=N).astype(np.uint32)
    z = rng.integers(0, K, size=N).astype(np.int32)
    z[1234] = K
    ws = torch.zeros(B.btc_update_workspace_bytes(v, K), dtype=torch.uint8, device="cuda")
    cbd = G.dev(cb.copy())
    with pytest.raises(B.BtcError) as e:
        B.btc_update(G.dev(vec), G.dev(z), N, v, cbd, K, ws)
    assert e.value.status == B.binding.BTC_ERR_INDEX_RANGE
    torch.cuda.synchronize()
    assert np.array_equal(cbd.cpu().numpy().view(np.uint32), cb) and not bool(ws.any())
