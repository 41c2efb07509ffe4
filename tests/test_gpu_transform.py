"""GPU parity of btc_transform (the online activation transform X <- X D (P1 kron P2)) against the CPU oracle,
through the C ABI.  fp32 output is held to the accuracy of fp32 accumulation (rel-L2 <= 1e-5, max-abs <= 1e-5 of
the largest output); fp16 / bf16 outputs add one rounding to nearest (half an ulp: 2^-11 / 2^-8 relative per
element) and are held to the tolerances of the other parity tests (rel-L2 <= 2e-3, max-abs <= 1e-2)."""
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


def _run(G, xb, kind, bits, P1, P2, y_dtype):
    import torch
    B = G.B
    M, n = xb.shape
    tdt = {B.BTC_F32: torch.float32, B.BTC_F16: torch.float16, B.BTC_BF16: torch.bfloat16}[y_dtype]
    out = G.GuardedOutput(M, n, tdt)
    B.btc_transform(G.dev(xb), B.BTC_BF16 if kind == "bf16" else B.BTC_F16, M, P1.shape[0], P2.shape[0],
                    G.dev(bits), G.dev(P1), G.dev(P2), out.payload, y_dtype)
    out.check_guards()
    return out.numpy()


def _check(y, y_ref, y_dtype, B, what):
    rel = np.linalg.norm(y - y_ref) / np.linalg.norm(y_ref)
    mabs = np.max(np.abs(y - y_ref)) / np.max(np.abs(y_ref))
    tol = (1e-5, 1e-5) if y_dtype == B.BTC_F32 else (2e-3, 1e-2)
    assert rel <= tol[0] and mabs <= tol[1], (what, rel, mabs)


# (n1, n2, M, activation type, output type): the factor pairs of the LLaMA-2 widths (4096 = 64 x 64,
# 5120 = 64 x 80, 11008 = 86 x 128, 13824 = 108 x 128, 8192 = 64 x 128, 28672 = 128 x 224), then ragged and
# degenerate ones (a last column block that is not full, odd n2, a factor of 1, the largest factors).
CASES = [
    (64, 64, 1, "f16", "f32"), (64, 80, 1, "f16", "f16"), (64, 80, 4, "f16", "f32"), (64, 80, 16, "bf16", "bf16"),
    (86, 128, 3, "f16", "f32"), (108, 128, 2, "bf16", "f32"), (64, 128, 5, "f16", "f16"), (128, 224, 1, "f16", "f32"),
    (7, 13, 9, "f16", "f32"), (1, 9, 3, "bf16", "f32"), (5, 1, 2, "f16", "f32"), (100, 83, 4, "f16", "f32"),
    (3, 250, 7, "bf16", "f16"), (128, 256, 1, "f16", "f32"), (32, 32, 300, "bf16", "f32"), (16, 24, 2000, "f16", "f16"),
]


@pytest.mark.parametrize("n1,n2,M,kind,yd", CASES)
def test_transform_matches_oracle(G, oracle, n1, n2, M, kind, yd):
    B = G.B
    print(f"transform n1={n1} n2={n2} M={M} {kind}->{yd}", flush=True)
    y_dtype = {"f32": B.BTC_F32, "f16": B.BTC_F16, "bf16": B.BTC_BF16}[yd]
    bits, P1, P2 = S.draw_transform(100 + n1 + n2, n1, n2)
    xb = S.draw_x(np.random.default_rng(n1 * 1000 + n2 + M), M, n1 * n2, kind)
    y = _run(G, xb, kind, bits, P1, P2, y_dtype)
    _check(y, oracle.transform(xb, bits, P1, P2, kind), y_dtype, B, (n1, n2, M, kind, yd))


@pytest.mark.parametrize("kind,yd", [("bf16", "bf16"), ("f16", "f32")])
def test_transform_prefill_size_sampled_rows(G, oracle, kind, yd):
    """2048 rows of 5120 channels (the prefill size of the benchmark).  The oracle forms the n x n matrix T per
    call, so it recomputes rows spread over the blocks of rows the kernel deals to its waves (rows are independent
    of one another); the remaining rows are only checked to be finite."""
    B = G.B
    n1, n2, M = 64, 80, 2048
    y_dtype = {"f32": B.BTC_F32, "bf16": B.BTC_BF16}[yd]
    bits, P1, P2 = S.draw_transform(77, n1, n2)
    xb = S.draw_x(np.random.default_rng(4), M, n1 * n2, kind)
    y = _run(G, xb, kind, bits, P1, P2, y_dtype)
    rows = np.unique(np.concatenate([[0, 1, 2046, 2047], np.arange(5, 2048, 97)]))
    _check(y[rows], oracle.transform(xb[rows], bits, P1, P2, kind), y_dtype, B, "sampled rows")
    assert np.isfinite(y).all()


def test_transform_identity_and_signs_exact(G, oracle):
    """Identity factors: the output is the input with its signs flipped, bit for bit (fp16 in, fp16 out)."""
    B = G.B
    n1, n2, M = 12, 20, 5
    bits, _, _ = S.draw_transform(5, n1, n2)
    xb = S.draw_x(np.random.default_rng(8), M, n1 * n2, "f16")
    y = _run(G, xb, "f16", bits, np.eye(n1, dtype=np.float32), np.eye(n2, dtype=np.float32), B.BTC_F16)
    assert np.array_equal(y, oracle.transform(xb, bits, np.eye(n1, dtype=np.float32), np.eye(n2, dtype=np.float32)))


# The matrix-core path (bf16 activations, n2 a multiple of 16, 64 rows or more): ragged blocks of 32 rows i1 / j1
# (108 = 3 x 32 + 12, 33 = 32 + 1), a last block of 32 columns that is half empty (48, 80, 16), fewer steps than the
# prefetch depth (n2 = 16, 32), every block count 1..4, rows that do not divide among the waves.
MFMA_CASES = [(108, 128, 100, "f32"), (128, 224, 70, "f32"), (40, 16, 200, "f32"), (33, 48, 130, "bf16"),
              (96, 32, 64, "f16"), (64, 80, 257, "f32"), (20, 96, 65, "f32"), (128, 256, 66, "bf16")]


@pytest.mark.parametrize("n1,n2,M,yd", MFMA_CASES)
def test_transform_matrix_core_path_sampled_rows(G, oracle, n1, n2, M, yd):
    B = G.B
    print(f"transform (matrix cores) n1={n1} n2={n2} M={M} bf16->{yd}", flush=True)
    y_dtype = {"f32": B.BTC_F32, "f16": B.BTC_F16, "bf16": B.BTC_BF16}[yd]
    bits, P1, P2 = S.draw_transform(300 + n1 + n2, n1, n2)
    xb = S.draw_x(np.random.default_rng(n1 + n2 + M), M, n1 * n2, "bf16")
    y = _run(G, xb, "bf16", bits, P1, P2, y_dtype)
    rows = np.unique(np.array([0, 1, 2, 3, 4, M // 2, M - 5, M - 4, M - 3, M - 2, M - 1]))
    if n1 * n2 > 8192:
        rows = rows[[0, 3, len(rows) // 2, -1]]          # the oracle forms n x n entries per row
    _check(y[rows], oracle.transform(xb[rows], bits, P1, P2, "bf16"), y_dtype, B, (n1, n2, M, yd))
    assert np.isfinite(y).all()
