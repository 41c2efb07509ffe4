"""GPU parity of btc_gemv_groups (several (alpha, mu) groups per weight row) against the oracle: every output,
1..4 groups, tuned and untuned settings, ragged last chunks, chunk lengths whose map bits straddle words, a
codebook too large for LDS, group maps that are random, constant, and sorted by magnitude-like runs."""
import numpy as np
import pytest

import btc_synth as S
from test_groups_pins import pack_groups

pytestmark = pytest.mark.gpu

CASES = [
    # out, in, v, K, G
    (300, 4096, 10, 256, 3), (5120, 5120, 10, 256, 3), (1000, 13824, 10, 256, 2), (77, 1234, 9, 1024, 4),
    (513, 999, 7, 100, 3), (64, 330, 16, 20000, 2), (40, 2000, 32, 2, 4), (9, 10, 10, 512, 1), (1, 17, 4, 9, 3),
]


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import gpu_util
    return gpu_util


@pytest.mark.parametrize("out,n_in,v,K,ng", CASES)
def test_groups_layer_matches_the_oracle(G, oracle, out, n_in, v, K, ng):
    import torch
    B = G.B
    print(f"groups out={out} in={n_in} v={v} K={K} G={ng}", flush=True)
    layer, x = S.make_case(41, out, n_in, v, K, 1)
    rng = np.random.default_rng(out + ng)
    g = rng.integers(0, ng, size=(out, n_in))
    g[0, :] = ng - 1                                     # a row in one group
    if out > 2:
        g[2, :] = np.sort(g[2, :])                       # runs
    alpha = np.abs(rng.normal(0, 0.02, size=(out, ng))).astype(np.float32)
    mu = rng.normal(0, 0.002, size=(out, ng)).astype(np.float32)
    gm = pack_groups(g)
    dl = G.DeviceLayer(layer, oracle)
    y_ref = np.concatenate([oracle.linear_groups(dl.packed_host, dl.codebook_host, alpha, mu, gm, x, n_in, v, K,
                                                 rows=np.arange(r0, min(out, r0 + 2048)))
                            for r0 in range(0, out, 2048)], axis=1)
    for yd, tdt in ((B.BTC_F32, torch.float32), (B.BTC_F16, torch.float16)):
        Y = G.GuardedOutput(1, out, tdt)
        B.btc_gemv_groups(dl.shape, dl.packed, dl.codebook, G.dev(alpha), G.dev(mu), G.dev(gm), ng, G.dev(x), Y.payload, yd)
        Y.check_guards()
        G.assert_close(Y.numpy(), y_ref, "layer with groups")


def test_argument_errors(G):
    import torch
    B = G.B
    from paper_2506_12040_amd import binding as BB
    s = B.btc_shape_init(64, 64, 10, 256)
    t = torch.zeros(4096, dtype=torch.int32, device="cuda")
    for ng in (0, 5):
        with pytest.raises(BB.BtcError) as e:
            B.btc_gemv_groups(s, t, t, t, t, t, ng, t, t, B.BTC_F32)
        assert e.value.status == BB.BTC_ERR_UNSUPPORTED
    with pytest.raises(BB.BtcError) as e:
        B.btc_gemv_groups(s, t, t, t, t, None, 2, t, t, B.BTC_F32)
    assert e.value.status == BB.BTC_ERR_NULL
