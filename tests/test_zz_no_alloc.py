"""btc_gemv_static -- the entry point that allocates nothing and keeps its scratch memory in a static device
array -- against btc_gemv with a caller workspace, called through the C ABI: same kernels, so the outputs must be
identical bit for bit.  Two calls in a row per pair of shapes, the second with a smaller input, on shapes whose
engines do park partial sums in the scratch memory (several activation rows; settings only the table engine
covers) and on one that needs none; a call that would need more than the static array is refused."""
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


def _both(G, oracle, out, n_in, v, K, batch, seed):
    import torch
    from paper_2506_12040_amd import binding as BB
    layer, x = S.make_case(seed, out, n_in, v, K, batch)
    dl = G.DeviceLayer(layer, oracle)
    xd = G.dev(x)
    y_ws = G.GuardedOutput(batch, out, torch.float16)
    ws = torch.zeros(max(16, BB.btc_workspace_bytes(dl.shape, batch, False)), dtype=torch.uint8, device="cuda")
    BB.btc_gemv(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, xd, batch, y_ws.payload, BB.BTC_F16, ws)
    y_ws.check_guards()
    y_st = G.GuardedOutput(batch, out, torch.float16)
    BB.btc_gemv_static(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, xd, batch, y_st.payload, BB.BTC_F16)
    y_st.check_guards()
    a, b = y_ws.numpy(), y_st.numpy()
    assert np.array_equal(a, b), f"btc_gemv_static differs from btc_gemv on {out}x{n_in} v{v} K{K} batch {batch}"
    G.assert_close(b, G.oracle_all_rows(oracle, dl, x), "btc_gemv_static")
    return len(ws)


PAIRS = [
    # (larger call, smaller call): out, in, v, K, batch
    ((9000, 4096, 10, 512, 16), (700, 3008, 10, 64, 4)),      # matrix-core decode engine: partial sums in scratch
    ((3000, 6000, 8, 85, 1), (300, 1000, 8, 85, 1)),          # only the table engine covers v = 8: tagged slots
    ((4096, 11008, 10, 512, 4), (130, 2049, 10, 512, 3)),
    ((8192, 8192, 10, 512, 1), (50, 333, 4, 9, 1)),           # engines without scratch memory
]


@pytest.mark.parametrize("big,small", PAIRS)
def test_static_scratch_entry_point_matches_btc_gemv(G, oracle, big, small):
    print(f"btc_gemv_static {big} then {small}", flush=True)
    n1 = _both(G, oracle, *big, seed=41)
    n2 = _both(G, oracle, *small, seed=42)
    print(f"   workspace bytes btc_gemv would need: {n1}, {n2}", flush=True)
    _both(G, oracle, *big, seed=43)       # and the larger one again after the smaller


def test_static_scratch_entry_point_refuses_oversize(G, oracle):
    import torch
    from paper_2506_12040_amd import binding as BB
    s = BB.btc_shape_init(28672, 28672, 10, 512)
    need = BB.btc_workspace_bytes(s, 16, False)
    assert need > (8 << 20), need
    dummy = torch.zeros(1 << 20, dtype=torch.int32, device="cuda")
    with pytest.raises(BB.BtcError) as e:     # the size check comes before anything is read or enqueued
        BB.btc_gemv_static(s, dummy, dummy, dummy, dummy, dummy, 16, dummy, BB.BTC_F16)
    assert e.value.status == BB.BTC_ERR_WORKSPACE
