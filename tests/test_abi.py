"""Host-side checks of the C-ABI library: it loads, exports every function
that include/btc.h declares, and its host-only entry points and argument
checks behave as documented.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

import btc_synth as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    import paper_2506_12040_amd as B
    if not os.path.exists(B.binding.LIB_PATH):
        from paper_2506_12040_amd import build
        build.build()
    return B


def declared_functions():
    text = open(os.path.join(ROOT, "include", "btc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(btc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(B):
    names = declared_functions()
    assert {"btc_pack", "btc_unpack", "btc_gemv", "btc_gemm", "btc_shape_init", "btc_packed_bytes",
            "btc_workspace_bytes", "btc_status_str"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n


def test_binding_has_the_same_names(B):
    for n in declared_functions():
        if n == "btc_status_str":
            continue
        assert hasattr(B.binding, n), n


@pytest.mark.parametrize("out,n_in,v,K", [(4096, 4096, 10, 512), (11008, 4096, 10, 512), (4096, 11008, 10, 512),
                                          (5120, 13824, 10, 256), (8192, 28672, 9, 1024), (8192, 8192, 10, 128),
                                          (7, 33, 4, 9), (3, 100, 20, 65536), (5, 17, 32, 2)])
def test_shape_arithmetic_matches_recipe(B, out, n_in, v, K):
    s = B.btc_shape_init(out, n_in, v, K)
    assert (s.out, s.in_, s.v, s.K) == (out, n_in, v, K)
    assert s.b == S.index_bits(K) and s.nchunks == S.num_chunks(n_in, v)
    assert s.words_per_row == S.words_per_row(n_in, v, K)
    assert B.btc_packed_bytes(s) == out * s.words_per_row * 4
    assert B.btc_workspace_bytes(s, 1, False) >= 16
    assert B.btc_workspace_bytes(s, 512, True) >= 16 + 512 * 4


def test_shape_errors(B):
    for args, code in [((0, 8, 4, 4), B.binding.BTC_ERR_SHAPE), ((8, -1, 4, 4), B.binding.BTC_ERR_SHAPE),
                       ((8, 8, 0, 4), B.binding.BTC_ERR_SHAPE), ((8, 8, 33, 4), B.binding.BTC_ERR_UNSUPPORTED),
                       ((8, 8, 4, 1), B.binding.BTC_ERR_UNSUPPORTED), ((8, 8, 4, 65537), B.binding.BTC_ERR_UNSUPPORTED)]:
        with pytest.raises(B.BtcError) as e:
            B.btc_shape_init(*args)
        assert e.value.status == code
    assert B.lib().btc_shape_init(None, 1, 1, 1, 2) == B.binding.BTC_ERR_NULL
    assert B.lib().btc_packed_bytes(None) == 0


def test_status_strings(B):
    seen = set()
    for code in range(0, -8, -1):
        s = B.status_str(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8 and B.status_str(-99) == "unknown status"


def test_argument_checks_need_no_gpu(B):
    """NULL, tampered shapes, unsupported batch/dtype and misalignment are
    rejected before anything is enqueued, so these calls are safe without a GPU."""
    L = B.lib()
    s = B.btc_shape_init(64, 100, 10, 512)
    sp = ctypes.byref(s)
    fake = ctypes.c_void_p(0x1000)       # aligned, never dereferenced by a rejected call
    odd = ctypes.c_void_p(0x1004)
    E = B.binding
    assert L.btc_gemv(None, sp, None, fake, fake, fake, fake, 1, fake, E.BTC_F16, None, 0) == E.BTC_ERR_NULL
    assert L.btc_gemv(None, sp, fake, fake, fake, fake, fake, 0, fake, E.BTC_F16, None, 0) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv(None, sp, fake, fake, fake, fake, fake, 17, fake, E.BTC_F16, None, 0) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv(None, sp, fake, fake, fake, fake, fake, 1, fake, E.BTC_BF16, None, 0) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv(None, sp, odd, fake, fake, fake, fake, 1, fake, E.BTC_F16, None, 0) == E.BTC_ERR_ALIGN
    assert L.btc_gemm(None, sp, fake, fake, fake, fake, fake, E.BTC_BF16, 0, fake, E.BTC_F32, fake, 1 << 20) == E.BTC_ERR_SHAPE
    assert L.btc_gemm(None, sp, fake, fake, fake, fake, fake, E.BTC_F32, 8, fake, E.BTC_F32, fake, 1 << 20) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemm(None, sp, fake, fake, fake, fake, fake, E.BTC_BF16, 8, fake, E.BTC_F32, fake, 8) == E.BTC_ERR_WORKSPACE
    assert L.btc_gemm(None, sp, fake, fake, fake, fake, fake, E.BTC_BF16, 8, fake, E.BTC_F32, None, 0) == E.BTC_ERR_WORKSPACE
    assert L.btc_pack(None, sp, fake, fake, None, 0) == E.BTC_ERR_WORKSPACE
    assert L.btc_pack(None, sp, None, fake, fake, 16) == E.BTC_ERR_NULL
    assert L.btc_unpack(None, sp, fake, odd) == E.BTC_ERR_ALIGN
    assert L.btc_unpack(None, None, fake, fake) == E.BTC_ERR_NULL
    assert L.btc_transform(None, None, E.BTC_F16, 1, 4, 4, fake, fake, fake, fake, E.BTC_F16) == E.BTC_ERR_NULL
    other = ctypes.c_void_p(0x2000)
    assert L.btc_transform(None, fake, E.BTC_F16, 0, 4, 4, fake, fake, fake, other, E.BTC_F16) == E.BTC_ERR_SHAPE
    assert L.btc_transform(None, fake, E.BTC_F16, 1, 129, 4, fake, fake, fake, other, E.BTC_F16) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_transform(None, fake, E.BTC_F16, 1, 4, 257, fake, fake, fake, other, E.BTC_F16) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_transform(None, fake, E.BTC_F32, 1, 4, 4, fake, fake, fake, other, E.BTC_F16) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_transform(None, fake, E.BTC_F16, 1, 4, 4, fake, fake, fake, fake, E.BTC_F16) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_transform(None, fake, E.BTC_F16, 1, 4, 4, fake, odd, fake, other, E.BTC_F16) == E.BTC_ERR_ALIGN
    assert L.btc_assign(None, None, 8, 10, fake, 4, fake, None) == E.BTC_ERR_NULL
    assert L.btc_assign(None, fake, 0, 10, fake, 4, fake, None) == E.BTC_ERR_SHAPE
    assert L.btc_assign(None, fake, 8, 33, fake, 4, fake, None) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_assign(None, fake, 8, 10, fake, 65537, fake, None) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_assign(None, fake, 8, 10, fake, 4, odd, None) == E.BTC_ERR_ALIGN
    assert L.btc_update_workspace_bytes(10, 256) == 256 * 11 * 4 + 16 and L.btc_update_workspace_bytes(33, 4) == 0
    assert L.btc_update(None, fake, None, 8, 10, fake, 4, fake, 1 << 20) == E.BTC_ERR_NULL
    assert L.btc_update(None, fake, fake, 0, 10, fake, 4, fake, 1 << 20) == E.BTC_ERR_SHAPE
    assert L.btc_update(None, fake, fake, 8, 0, fake, 4, fake, 1 << 20) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_update(None, fake, fake, 8, 10, fake, 4, fake, 8) == E.BTC_ERR_WORKSPACE
    assert L.btc_update(None, fake, fake, 8, 10, odd, 4, fake, 1 << 20) == E.BTC_ERR_ALIGN
    t = B.btc_shape_init(64, 100, 10, 512)
    t.words_per_row += 1                 # a shape edited after btc_shape_init
    assert L.btc_unpack(None, ctypes.byref(t), fake, fake) == E.BTC_ERR_SHAPE


def test_argument_checks_of_the_later_entry_points(B):
    """btc_gemv_multi, btc_gemv_multi_shapes, btc_gemv_groups, btc_transform_prepare, btc_gemv_transformed(_multi), btc_quantize_rows,
    btc_gemm_aq: rejected calls return before anything is enqueued."""
    L = B.lib()
    E = B.binding
    s = B.btc_shape_init(64, 5120, 10, 256)
    sp = ctypes.byref(s)
    fake, odd, other = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004), ctypes.c_void_p(0x2000)
    arr = lambda *ps: (ctypes.c_void_p * len(ps))(*[p.value if p is not None else None for p in ps])
    four = arr(fake, fake, fake, fake)
    # several matrices in one launch
    assert L.btc_gemv_multi(None, sp, 0, four, four, four, four, fake, four, E.BTC_F16, None, 0) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv_multi(None, sp, 5, four, four, four, four, fake, four, E.BTC_F16, None, 0) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv_multi(None, sp, 2, None, four, four, four, fake, four, E.BTC_F16, None, 0) == E.BTC_ERR_NULL
    assert L.btc_gemv_multi(None, sp, 2, arr(fake, None), four, four, four, fake, four, E.BTC_F16, None, 0) == E.BTC_ERR_NULL
    assert L.btc_gemv_multi(None, sp, 2, arr(fake, odd), four, four, four, fake, four, E.BTC_F16, None, 0) == E.BTC_ERR_ALIGN
    assert L.btc_gemv_multi(None, sp, 2, four, four, four, four, fake, four, E.BTC_BF16, None, 0) == E.BTC_ERR_UNSUPPORTED
    # ... whose numbers of rows differ
    s_kv, s_in, s_K = B.btc_shape_init(8, 5120, 10, 256), B.btc_shape_init(8, 5130, 10, 256), B.btc_shape_init(8, 5120, 10, 128)
    shp = lambda *ss: (ctypes.POINTER(type(s)) * len(ss))(*[ctypes.pointer(x) if x is not None else None for x in ss])
    two = arr(fake, fake)
    assert L.btc_gemv_multi_shapes(None, None, 2, two, two, two, two, fake, two, E.BTC_F16, None, 0) == E.BTC_ERR_NULL
    assert L.btc_gemv_multi_shapes(None, shp(s, None), 2, two, two, two, two, fake, two, E.BTC_F16, None, 0) == E.BTC_ERR_NULL
    assert L.btc_gemv_multi_shapes(None, shp(s, s_kv), 5, two, two, two, two, fake, two, E.BTC_F16, None, 0) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv_multi_shapes(None, shp(s, s_in), 2, two, two, two, two, fake, two, E.BTC_F16, None, 0) == E.BTC_ERR_SHAPE
    assert L.btc_gemv_multi_shapes(None, shp(s, s_K), 2, two, two, two, two, fake, two, E.BTC_F16, None, 0) == E.BTC_ERR_SHAPE
    assert L.btc_gemv_multi_shapes(None, shp(s, s_kv), 2, arr(fake, odd), two, two, two, fake, two, E.BTC_F16, None, 0) == E.BTC_ERR_ALIGN
    assert L.btc_gemv_multi_shapes(None, shp(s, s_kv), 2, two, two, two, arr(fake, None), fake, two, E.BTC_F16, None, 0) == E.BTC_ERR_NULL
    # several (alpha, mu) groups per row
    assert L.btc_gemv_groups(None, sp, fake, fake, fake, fake, fake, 0, fake, fake, E.BTC_F32) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv_groups(None, sp, fake, fake, fake, fake, fake, 5, fake, fake, E.BTC_F32) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_gemv_groups(None, sp, fake, fake, fake, fake, None, 2, fake, fake, E.BTC_F32) == E.BTC_ERR_NULL
    assert L.btc_gemv_groups(None, sp, fake, fake, fake, fake, odd, 2, fake, fake, E.BTC_F32) == E.BTC_ERR_ALIGN
    assert L.btc_gemv_groups(None, sp, fake, fake, fake, fake, fake, 2, fake, fake, E.BTC_BF16) == E.BTC_ERR_UNSUPPORTED
    # the transform inside the product
    assert L.btc_transform_prepared_bytes(64, 80) == (3 * 5 + 2 * 4) * 2048 and L.btc_transform_prepared_bytes(64, 81) == 0
    assert L.btc_transform_prepared_bytes(108, 128) == (4 * 8 + 4 * 7) * 2048 and L.btc_transform_prepared_bytes(128, 224) == 0
    assert L.btc_transform_prepare(None, 64, 80, None, fake, fake, 1 << 20) == E.BTC_ERR_NULL
    assert L.btc_transform_prepare(None, 0, 80, fake, fake, fake, 1 << 20) == E.BTC_ERR_SHAPE
    assert L.btc_transform_prepare(None, 64, 81, fake, fake, fake, 1 << 20) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_transform_prepare(None, 64, 80, fake, fake, fake, 1024) == E.BTC_ERR_WORKSPACE
    assert L.btc_transform_prepare(None, 64, 80, fake, odd, fake, 1 << 20) == E.BTC_ERR_ALIGN
    gt = lambda *a: L.btc_gemv_transformed(None, sp, fake, fake, fake, fake, *a)
    assert gt(fake, 64, 64, fake, fake, fake, None, None, other, E.BTC_F32, fake, 1 << 24) == E.BTC_ERR_SHAPE     # n1 n2 != in
    assert gt(fake, 64, 80, None, fake, fake, None, None, other, E.BTC_F32, fake, 1 << 24) == E.BTC_ERR_NULL
    assert gt(fake, 64, 80, fake, fake, fake, None, None, other, E.BTC_BF16, fake, 1 << 24) == E.BTC_ERR_UNSUPPORTED
    assert gt(fake, 64, 80, fake, fake, fake, None, fake, other, E.BTC_F32, fake, 1 << 24) == E.BTC_ERR_UNSUPPORTED   # xt_out == x
    assert gt(fake, 64, 80, fake, fake, fake, None, None, other, E.BTC_F32, None, 0) == E.BTC_ERR_WORKSPACE       # two launches
    assert gt(fake, 64, 80, fake, odd, fake, None, None, other, E.BTC_F32, fake, 1 << 24) == E.BTC_ERR_ALIGN
    assert L.btc_gemv_transformed_workspace_bytes(sp) >= 5120 * 2 + 16 and L.btc_gemv_transformed_workspace_bytes(None) == 0
    assert L.btc_gemv_transformed_multi(None, sp, 5, four, four, four, four, fake, 64, 80, fake, fake, fake, None, None,
                                        four, E.BTC_F32, fake, 1 << 24) == E.BTC_ERR_UNSUPPORTED
    # the layer on activation codes
    assert L.btc_quantize_rows(None, None, E.BTC_F16, 1, 64, 8, fake, fake, fake, None) == E.BTC_ERR_NULL
    assert L.btc_quantize_rows(None, fake, E.BTC_F16, 0, 64, 8, other, fake, fake, None) == E.BTC_ERR_SHAPE
    assert L.btc_quantize_rows(None, fake, E.BTC_F16, 1, 64, 5, other, fake, fake, None) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_quantize_rows(None, fake, E.BTC_F32, 1, 64, 8, other, fake, fake, None) == E.BTC_ERR_UNSUPPORTED
    assert L.btc_aq_workspace_bytes(sp, 1) > 0 and L.btc_aq_workspace_bytes(None, 1) == 0
    assert L.btc_gemm_aq(None, sp, fake, fake, fake, fake, fake, fake, fake, fake, 0, other, E.BTC_F32, fake, 1 << 26) == E.BTC_ERR_SHAPE
    assert L.btc_gemm_aq(None, sp, fake, fake, fake, fake, None, fake, fake, fake, 1, other, E.BTC_F32, fake, 1 << 26) == E.BTC_ERR_NULL
    assert L.btc_gemm_aq(None, sp, fake, fake, fake, fake, fake, fake, fake, fake, 1, other, E.BTC_F32, fake, 64) == E.BTC_ERR_WORKSPACE
