"""Helpers for the GPU parity tests: move a synthetic layer to the device, call
the C-ABI through the binding, fetch results, compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2506_12040_amd as B

REL_L2_TOL = 2e-3       # ||y - y*||_2 / ||y*||_2
MAX_ABS_TOL = 1e-2      # max|y - y*| / max|y*|
GUARD = 64              # guard elements on either side of an output buffer


def dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor with the same bytes (uint16/uint32 via int views)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


class DeviceLayer:
    def __init__(self, layer, oracle):
        self.layer = layer
        self.shape = B.btc_shape_init(layer.out, layer.n_in, layer.v, layer.K)
        self.packed_host = oracle.pack(layer.idx, layer.K)
        self.packed = dev(self.packed_host)
        cb = np.zeros(1 << self.shape.b, dtype=np.uint32)
        cb[: layer.K] = layer.codebook
        self.codebook_host = cb
        self.codebook = dev(cb)
        self.alpha = dev(layer.alpha)
        self.mu = dev(layer.mu)


class GuardedOutput:
    """Output buffer with canary bands before and after the payload."""

    def __init__(self, rows: int, cols: int, dtype: torch.dtype):
        self.rows, self.cols = rows, cols
        n = rows * cols
        self.canary = 12345.0 if dtype.is_floating_point else (0xA5 if dtype == torch.uint8 else 0x5A5A5A5A)
        self.buf = torch.full((n + 2 * GUARD,), self.canary, dtype=dtype, device="cuda")
        self.payload = self.buf[GUARD:GUARD + n]
        assert self.payload.data_ptr() % 16 == 0

    def check_guards(self):
        torch.cuda.synchronize()
        head = self.buf[:GUARD].cpu()
        tail = self.buf[GUARD + self.rows * self.cols:].cpu()
        assert bool((head == self.canary).all()) and bool((tail == self.canary).all()), "guard band overwritten"

    def numpy(self) -> np.ndarray:
        return self.payload.float().cpu().numpy().astype(np.float64).reshape(self.rows, self.cols)


def gemv(dl: DeviceLayer, x_bits: np.ndarray, y_dtype: int = B.BTC_F16) -> np.ndarray:
    batch = x_bits.shape[0]
    x = dev(x_bits)
    y = GuardedOutput(batch, dl.layer.out, torch.float16 if y_dtype == B.BTC_F16 else torch.float32)
    ws = torch.zeros(max(16, B.btc_workspace_bytes(dl.shape, batch, False)), dtype=torch.uint8, device="cuda")
    B.btc_gemv(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, x, batch, y.payload, y_dtype, ws)
    y.check_guards()
    return y.numpy()


_TORCH_OF = {B.BTC_F16: torch.float16, B.BTC_BF16: torch.bfloat16, B.BTC_F32: torch.float32}


def gemm(dl: DeviceLayer, x_bits: np.ndarray, x_dtype: int, y_dtype: int = B.BTC_F32) -> np.ndarray:
    M = x_bits.shape[0]
    X = dev(x_bits)
    Y = GuardedOutput(M, dl.layer.out, _TORCH_OF[y_dtype])
    # btc_gemm promises to need no particular workspace contents: hand it NaN bit patterns
    ws = torch.full((B.btc_workspace_bytes(dl.shape, M, True),), 0xFF, dtype=torch.uint8, device="cuda")
    B.btc_gemm(dl.shape, dl.packed, dl.codebook, dl.alpha, dl.mu, X, x_dtype, M, Y.payload, y_dtype, ws)
    Y.check_guards()
    return Y.numpy()


def assert_close_bf16_out(y: np.ndarray, y_ref: np.ndarray, what: str = ""):
    """bf16 OUTPUT: rounding to 8 significant bits is itself up to 2^-8 = 3.9e-3 relative per element, 2^-8 / sqrt(7) =
    1.5e-3 in the L2 ratio when the significands are spread over [1, 2).  Outputs with enough elements for that
    average are held to the same bar as every other output type; a handful of elements (a single one can sit at the
    worst case of its rounding) are held element by element to rounding plus the bar."""
    if y.size >= 256:
        return assert_close(y, y_ref, what)
    assert y.shape == y_ref.shape and np.all(np.isfinite(y)), what
    bound = (2.0 ** -8 + REL_L2_TOL) * np.abs(y_ref) + 1e-30
    assert np.all(np.abs(y - y_ref) <= bound), f"{what}: element beyond bf16 rounding + {REL_L2_TOL}"
    mx = np.max(np.abs(y_ref))
    assert np.max(np.abs(y - y_ref)) <= MAX_ABS_TOL * mx + 1e-30, what


def oracle_all_rows(oracle, dl: DeviceLayer, x_bits: np.ndarray, x_kind: str = "f16", block: int = 4096) -> np.ndarray:
    """The oracle's result for EVERY weight row, [rows of x][out], materialising W_hat a block of rows at a time
    so that a 28672 x 8192 matrix never needs more than a gigabyte."""
    layer = dl.layer
    parts = []
    for r0 in range(0, layer.out, block):
        rows = np.arange(r0, min(layer.out, r0 + block))
        parts.append(oracle.linear(dl.packed_host, dl.codebook_host, layer.alpha, layer.mu, x_bits, layer.n_in,
                                   layer.v, layer.K, x_kind=x_kind, rows=rows))
    return np.concatenate(parts, axis=1)


def assert_close(y: np.ndarray, y_ref: np.ndarray, what: str = ""):
    assert y.shape == y_ref.shape, (y.shape, y_ref.shape)
    assert np.all(np.isfinite(y)), what
    denom = np.linalg.norm(y_ref)
    rel = np.linalg.norm(y - y_ref) / denom if denom > 0 else np.linalg.norm(y)
    mx = np.max(np.abs(y_ref))
    mabs = np.max(np.abs(y - y_ref)) / mx if mx > 0 else np.max(np.abs(y))
    assert rel <= REL_L2_TOL, f"{what}: rel L2 {rel:.3e} > {REL_L2_TOL}"
    assert mabs <= MAX_ABS_TOL, f"{what}: max abs {mabs:.3e} > {MAX_ABS_TOL}"
    return rel, mabs
