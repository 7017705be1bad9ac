"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2310_05218_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2310_05218_amd import build
        build.build()
    return B.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "swconv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sw_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_out_dim_and_constants(L):
    assert B.sw_workspace_bytes() == 0
    assert B.sw_version() >= 100
    assert B.sw_out_dim(56, 3, 1, 1) == 56
    assert B.sw_out_dim(65536, 9, 1, 0) == 65528
    assert B.sw_out_dim(7, 3, 2, 1) == 4
    assert B.sw_out_dim(2, 3, 1, 0) <= 0
    assert B.sw_out_dim(0, 3, 1, 0) <= 0 and B.sw_out_dim(5, 3, 0, 0) <= 0 and B.sw_out_dim(5, 3, 1, -1) <= 0
    for s in range(0, 9):
        assert len(B.status_string(s)) > 0


# Fake, never dereferenced device addresses: every call below must fail on the host.
X, W_, Y = 0x100000, 0x900000, 0x1100000


def test_conv1d_argument_errors(L):
    f = L.sw_conv1d
    assert f(None, W_, Y, 4, 100, 9, 1, 0, None) == B.SW_ERR_NULL
    assert f(X, None, Y, 4, 100, 9, 1, 0, None) == B.SW_ERR_NULL
    assert f(X, W_, None, 4, 100, 9, 1, 0, None) == B.SW_ERR_NULL
    assert f(X, W_, Y, 0, 100, 9, 1, 0, None) == B.SW_ERR_SHAPE
    assert f(X, W_, Y, 4, 0, 9, 1, 0, None) == B.SW_ERR_SHAPE
    assert f(X, W_, Y, 4, 100, 0, 1, 0, None) == B.SW_ERR_SHAPE
    assert f(X, W_, Y, 4, 100, 9, 0, 0, None) == B.SW_ERR_SHAPE
    assert f(X, W_, Y, 4, 100, 9, 1, -1, None) == B.SW_ERR_SHAPE
    assert f(X, W_, Y, 4, 5, 9, 1, 0, None) == B.SW_ERR_SHAPE          # filter longer than the row
    assert f(X, W_, Y, 1 << 20, 1 << 20, 9, 1, 0, None) == B.SW_ERR_SHAPE  # too many elements
    assert f(X, W_, Y, 4, 100, 65, 1, 0, None) == B.SW_ERR_UNSUPPORTED
    assert f(X, W_, Y, 4, 100, 9, 1, 9, None) == B.SW_ERR_UNSUPPORTED  # pad >= k
    assert f(X + 2, W_, Y, 4, 100, 9, 1, 0, None) == B.SW_ERR_ALIGN
    assert f(X, W_, Y + 1, 4, 100, 9, 1, 0, None) == B.SW_ERR_ALIGN
    assert f(X, W_, X + 4 * 50, 4, 100, 9, 1, 0, None) == B.SW_ERR_ALIAS
    assert f(X, Y + 16, Y, 4, 100, 9, 1, 0, None) == B.SW_ERR_ALIAS


def test_pool1d_argument_errors(L):
    f = L.sw_pool1d
    assert f(None, Y, 4, 100, 8, 1, 0, None) == B.SW_ERR_NULL
    assert f(X, None, 4, 100, 8, 1, 1, None) == B.SW_ERR_NULL
    assert f(X, Y, 4, 100, 8, 1, 2, None) == B.SW_ERR_UNSUPPORTED       # unknown mode
    assert f(X, Y, 4, 100, 101, 1, 0, None) == B.SW_ERR_SHAPE
    assert f(X, Y, 4, 100, 8, 0, 0, None) == B.SW_ERR_SHAPE
    assert f(X, Y, 4, 1000, 65, 1, 0, None) == B.SW_ERR_UNSUPPORTED
    assert f(X, X, 4, 100, 8, 1, 0, None) == B.SW_ERR_ALIAS


def test_pool2d_argument_errors(L):
    f = L.sw_pool2d
    ok = (2, 16, 8, 8, 3, 3, 2, 1)
    assert f(None, Y, *ok, 0, None) == B.SW_ERR_NULL
    assert f(X, None, *ok, 1, None) == B.SW_ERR_NULL
    for i in range(7):                       # N, C, H, W, R, S, stride <= 0
        bad = list(ok)
        bad[i] = 0
        assert f(X, Y, *bad, 0, None) == B.SW_ERR_SHAPE, i
    assert f(X, Y, 2, 16, 8, 8, 3, 3, 2, -1, 0, None) == B.SW_ERR_SHAPE
    assert f(X, Y, 2, 16, 2, 8, 5, 3, 1, 1, 0, None) == B.SW_ERR_SHAPE          # window > padded plane
    assert f(X, Y, 4096, 4096, 64, 64, 3, 3, 1, 1, 0, None) == B.SW_ERR_SHAPE   # > 2^31-1 elements
    assert f(X, Y, *ok, 2, None) == B.SW_ERR_UNSUPPORTED                        # unknown mode
    assert f(X, Y, 2, 16, 100, 100, 65, 3, 1, 1, 0, None) == B.SW_ERR_UNSUPPORTED
    assert f(X, Y, 2, 16, 8, 8, 3, 3, 1, 2, 1, None) == B.SW_ERR_UNSUPPORTED    # 2*pad > window
    assert f(X + 2, Y, *ok, 0, None) == B.SW_ERR_ALIGN
    assert f(X, Y + 1, *ok, 0, None) == B.SW_ERR_ALIGN
    assert f(X, X + 64, *ok, 0, None) == B.SW_ERR_ALIAS


@pytest.mark.parametrize("name", ["sw_conv2d", "sw_conv2d_s8"])
def test_conv2d_argument_errors(L, name):
    f = getattr(L, name)
    ok = (2, 16, 16, 8, 8, 3, 3, 1, 1)
    assert f(None, W_, Y, *ok, None) == B.SW_ERR_NULL
    assert f(X, None, Y, *ok, None) == B.SW_ERR_NULL
    assert f(X, W_, None, *ok, None) == B.SW_ERR_NULL
    for i in range(8):                       # N, C_in, C_out, H, W, R, S, stride <= 0
        bad = list(ok)
        bad[i] = 0
        assert f(X, W_, Y, *bad, None) == B.SW_ERR_SHAPE, i
    assert f(X, W_, Y, 2, 16, 16, 8, 8, 3, 3, 1, -1, None) == B.SW_ERR_SHAPE
    assert f(X, W_, Y, 2, 16, 16, 2, 8, 5, 3, 1, 1, None) == B.SW_ERR_SHAPE       # filter > padded input
    assert f(X, W_, Y, 4096, 4096, 16, 64, 64, 3, 3, 1, 1, None) == B.SW_ERR_SHAPE  # > 2^31-1 elements
    assert f(X, W_, Y, 2, 16, 16, 100, 100, 65, 3, 1, 1, None) == B.SW_ERR_UNSUPPORTED
    assert f(X, W_, Y + 2, *ok, None) == B.SW_ERR_ALIGN
    assert f(X, W_, X, *ok, None) == B.SW_ERR_ALIAS
    assert f(X, Y + 64, Y, *ok, None) == B.SW_ERR_ALIAS


def test_conv2d_f32_alignment_and_s8_accumulator_bound(L):
    ok = (2, 16, 16, 8, 8, 3, 3, 1, 1)
    assert L.sw_conv2d(X + 2, W_, Y, *ok, None) == B.SW_ERR_ALIGN
    assert L.sw_conv2d(X, W_ + 1, Y, *ok, None) == B.SW_ERR_ALIGN
    # int8 inputs need no alignment, so odd addresses get as far as the shape checks
    assert L.sw_conv2d_s8(X + 1, W_ + 3, Y, 1, 16384, 1, 8, 8, 3, 3, 1, 1, None) == B.SW_ERR_SHAPE  # 147456 terms


def test_requant_argument_errors(L):
    f = L.sw_conv2d_s8_requant
    B_, SC = 0x1900000, 0x1a00000
    ok = (2, 16, 16, 8, 8, 3, 3, 1, 1)
    assert f(X, W_, B_, None, Y, *ok, 0, None) == B.SW_ERR_NULL
    assert f(None, W_, B_, SC, Y, *ok, 0, None) == B.SW_ERR_NULL
    assert f(X, W_, B_, SC, Y, 2, 16, 16, 8, 8, 0, 3, 1, 1, 0, None) == B.SW_ERR_SHAPE
    assert f(X, W_, B_, SC, Y, 1, 16384, 1, 8, 8, 3, 3, 1, 1, 0, None) == B.SW_ERR_SHAPE   # 147456 terms
    assert f(X, W_, B_ + 2, SC, Y, *ok, 0, None) == B.SW_ERR_ALIGN
    assert f(X, W_, B_, SC + 1, Y, *ok, 0, None) == B.SW_ERR_ALIGN
    assert f(X, W_, B_, SC, X + 5, *ok, 0, None) == B.SW_ERR_ALIAS
    assert f(X, W_, B_, Y + 8, Y, *ok, 0, None) == B.SW_ERR_ALIAS


def test_depthwise_argument_errors(L):
    f = L.sw_conv2d_depthwise
    ok = (2, 16, 8, 8, 3, 3, 1, 1)
    assert f(None, W_, Y, *ok, None) == B.SW_ERR_NULL
    for i in range(7):
        bad = list(ok)
        bad[i] = 0
        assert f(X, W_, Y, *bad, None) == B.SW_ERR_SHAPE, i
    assert f(X, W_, Y, 2, 16, 4, 4, 7, 7, 1, 0, None) == B.SW_ERR_SHAPE
    assert f(X, W_, X + 64, *ok, None) == B.SW_ERR_ALIAS


def test_block_argument_errors(L):
    f = L.sw_dw_pw_block
    WD, BD, WP, BP = 0x2100000, 0x2200000, 0x2300000, 0x2400000
    ok = (2, 16, 32, 8, 8)                      # N, C, C_out, H, W
    assert f(None, WD, BD, WP, BP, Y, *ok, 1, 0, None) == B.SW_ERR_NULL
    assert f(X, None, BD, WP, BP, Y, *ok, 1, 0, None) == B.SW_ERR_NULL
    assert f(X, WD, BD, None, BP, Y, *ok, 1, 0, None) == B.SW_ERR_NULL
    assert f(X, WD, BD, WP, BP, None, *ok, 1, 0, None) == B.SW_ERR_NULL
    for i in range(5):
        bad = list(ok)
        bad[i] = 0
        assert f(X, WD, BD, WP, BP, Y, *bad, 1, 0, None) == B.SW_ERR_SHAPE, i
    assert f(X, WD, BD + 2, WP, BP, Y, *ok, 1, 0, None) == B.SW_ERR_ALIGN
    assert f(X, WD, BD, WP, BP, X + 64, *ok, 1, 0, None) == B.SW_ERR_ALIAS
    assert f(X, WD, BD, Y + 16, BP, Y, *ok, 1, 0, None) == B.SW_ERR_ALIAS
    assert f(X, WD, None, WP, Y + 32, Y, *ok, 1, 0, None) == B.SW_ERR_ALIAS


def test_s8_nhwc_argument_errors(L):
    f, g = L.sw_conv2d_s8_nhwc, L.sw_conv2d_s8_nhwc_requant
    B_, SC = 0x2100000, 0x2200000
    ok = (2, 8, 8, 32, 64, 3, 3, 1, 1)          # N, H, W, C_in, C_out, R, S, stride, pad
    assert f(None, W_, Y, *ok, None) == B.SW_ERR_NULL
    assert g(X, W_, B_, None, Y, *ok, 0, None) == B.SW_ERR_NULL
    assert g(X, W_, B_, SC, None, *ok, 0, None) == B.SW_ERR_NULL
    for i in range(8):
        bad = list(ok)
        bad[i] = 0
        assert f(X, W_, Y, *bad, None) == B.SW_ERR_SHAPE, i
        assert g(X, W_, B_, SC, Y, *bad, 0, None) == B.SW_ERR_SHAPE, i
    assert f(X, W_, Y + 2, *ok, None) == B.SW_ERR_ALIGN
    assert f(X, W_, X + 64, *ok, None) == B.SW_ERR_ALIAS
    assert g(X, W_, B_, SC + 2, Y, *ok, 0, None) == B.SW_ERR_ALIGN
    assert g(X, W_, B_, Y + 8, Y, *ok, 0, None) == B.SW_ERR_ALIAS
    # 131072 products of magnitude 2^14 could leave int32
    assert f(X, W_, Y, 1, 64, 64, 4096, 8, 6, 6, 1, 0, None) == B.SW_ERR_SHAPE


def test_bf16_argument_errors(L):
    f = L.sw_conv2d_depthwise_bf16
    ok = (2, 16, 8, 8, 3, 3, 1, 1)
    assert f(None, W_, Y, *ok, None) == B.SW_ERR_NULL
    for i in range(7):
        bad = list(ok)
        bad[i] = 0
        assert f(X, W_, Y, *bad, None) == B.SW_ERR_SHAPE, i
    assert f(X + 1, W_, Y, *ok, None) == B.SW_ERR_ALIGN        # bf16 planes: 2-byte aligned
    assert f(X, W_ + 2, Y, *ok, None) == B.SW_ERR_ALIGN        # the fp32 filter: 4-byte aligned
    assert f(X, W_, X + 64, *ok, None) == B.SW_ERR_ALIAS
    assert f(X, Y + 2 * 2 * 16 * 64 - 4, Y, *ok, None) == B.SW_ERR_ALIAS   # the filter's last bytes under y


def test_dilated_argument_errors(L):
    f, g = L.sw_conv2d_dilated, L.sw_conv2d_depthwise_dilated
    ok = (2, 16, 64, 12, 12, 3, 3, 1, 2, 2)
    okd = (2, 16, 12, 12, 3, 3, 1, 2, 2)
    assert f(None, W_, Y, *ok, None) == B.SW_ERR_NULL and g(X, None, Y, *okd, None) == B.SW_ERR_NULL
    for bad_dil in (0, -1):
        assert f(X, W_, Y, *ok[:-1], bad_dil, None) == B.SW_ERR_SHAPE
        assert g(X, W_, Y, *okd[:-1], bad_dil, None) == B.SW_ERR_SHAPE
    # span 6 * 2 + 1 = 13 > 12: the dilated filter does not fit the unpadded plane
    assert f(X, W_, Y, 2, 16, 64, 12, 12, 7, 7, 1, 0, 2, None) == B.SW_ERR_SHAPE
    assert g(X, W_, Y, 2, 16, 12, 12, 7, 7, 1, 0, 2, None) == B.SW_ERR_SHAPE
    assert f(X, W_, X + 64, *ok, None) == B.SW_ERR_ALIAS
    assert g(X + 2, W_, Y, *okd, None) == B.SW_ERR_ALIGN


def test_bias_relu_argument_errors(L):
    f = L.sw_conv2d_bias_relu
    B_ = 0x2100000
    ok = (2, 16, 64, 8, 8, 3, 3, 1, 1)
    assert f(None, W_, B_, Y, *ok, 0, None) == B.SW_ERR_NULL
    assert f(X, W_, B_, None, *ok, 1, None) == B.SW_ERR_NULL
    for i in range(8):
        bad = list(ok)
        bad[i] = 0
        assert f(X, W_, B_, Y, *bad, 0, None) == B.SW_ERR_SHAPE, i
    assert f(X, W_, B_ + 2, Y, *ok, 0, None) == B.SW_ERR_ALIGN
    assert f(X, W_, Y + 16, Y, *ok, 0, None) == B.SW_ERR_ALIAS
    assert f(X, W_, B_, X + 64, *ok, 0, None) == B.SW_ERR_ALIAS


def test_depthwise_bias_relu_argument_errors(L):
    f = L.sw_conv2d_depthwise_bias_relu
    B_ = 0x2100000
    ok = (2, 16, 8, 8, 3, 3, 1, 1)
    assert f(None, W_, B_, Y, *ok, 0, None) == B.SW_ERR_NULL
    for i in range(7):
        bad = list(ok)
        bad[i] = 0
        assert f(X, W_, B_, Y, *bad, 0, None) == B.SW_ERR_SHAPE, i
    assert f(X, W_, B_ + 2, Y, *ok, 0, None) == B.SW_ERR_ALIGN
    assert f(X, W_, Y + 16, Y, *ok, 0, None) == B.SW_ERR_ALIAS


def test_jit_entry_point_argument_errors(L):
    f = L.sw_conv2d_depthwise_jit
    ok = (2, 16, 56, 56, 9, 9, 1, 4)
    assert f(None, W_, Y, *ok, None) == B.SW_ERR_NULL
    for i in range(7):
        bad = list(ok)
        bad[i] = 0
        assert f(X, W_, Y, *bad, None) == B.SW_ERR_SHAPE, i
    assert f(X, W_, X + 64, *ok, None) == B.SW_ERR_ALIAS
    assert f(X, W_, Y + 2, *ok, None) == B.SW_ERR_ALIGN


# geometries inside the generated kernel's range: H, W, R, S, pad
JIT_GEOMETRIES = [(56, 56, 1, 1, 0), (56, 56, 3, 3, 1), (56, 56, 9, 9, 4), (56, 56, 11, 11, 5), (56, 56, 17, 17, 8),
                  (56, 56, 29, 29, 14), (56, 56, 33, 33, 16), (64, 64, 9, 9, 0), (56, 56, 5, 9, 2), (48, 52, 7, 7, 3)]


@pytest.mark.parametrize("geometry", JIT_GEOMETRIES)
def test_generated_source_compiles_for_its_whole_range(L, geometry):
    """The run-time compiler accepts the generated kernel (its static_asserts included) for each geometry; the
    compile step needs no device."""
    H, W, R, S, pad = geometry
    assert B.sw_jit_compile_check(H, W, R, S, 1, pad) == B.SW_OK


def test_jit_range_and_errors(L):
    assert B.sw_jit_compile_check(56, 56, 9, 9, 3, 4) == B.SW_ERR_UNSUPPORTED      # stride 3
    assert B.sw_jit_compile_check(8, 8, 3, 3, 1, 1) == B.SW_ERR_UNSUPPORTED        # small plane
    assert B.sw_jit_compile_check(56, 24, 3, 3, 1, 1) == B.SW_ERR_UNSUPPORTED      # most lanes of the 8 x 8 grid idle
    assert B.sw_jit_compile_check_dilated(56, 56, 3, 3, 1, 32, 32) == B.SW_ERR_UNSUPPORTED   # span 65
    assert B.sw_jit_compile_check_dilated(56, 56, 3, 3, 1, 2, 0) == B.SW_ERR_SHAPE
    assert B.sw_jit_compile_check_dilated(56, 56, 3, 3, 2, 1, 1) == B.SW_OK         # stride 2: builds
    assert B.sw_jit_compile_check_dilated(28, 28, 5, 5, 1, 4, 2) == B.SW_OK         # four outputs per lane, dilation 2
    assert B.sw_jit_compile_check(58, 58, 3, 3, 1, 1) == B.SW_ERR_UNSUPPORTED      # output above 56 x 56
    assert B.sw_jit_compile_check(56, 56, 12, 12, 1, 4) == B.SW_ERR_UNSUPPORTED    # W_out = 53
    assert B.sw_jit_compile_check(56, 56, 9, 9, 1, 6) == B.SW_ERR_UNSUPPORTED      # output larger than the plane
    assert B.sw_jit_compile_check(56, 56, 37, 37, 1, 18) == B.SW_ERR_UNSUPPORTED   # window above 37 KB
    assert B.sw_jit_compile_check(0, 56, 9, 9, 1, 4) == B.SW_ERR_SHAPE
    assert B.sw_jit_compile_check(4, 4, 9, 9, 1, 0) == B.SW_ERR_SHAPE              # filter larger than the plane
    assert B.sw_jit_prepare_depthwise(56, 56, 9, 9, 1, -1) == B.SW_ERR_SHAPE
    assert B.sw_jit_prepare_depthwise(8, 8, 3, 3, 1, 1) == B.SW_ERR_UNSUPPORTED
    assert B.sw_jit_cached_kernels() >= 0


def test_binding_refuses_host_tensors(L):
    import torch

    x = torch.zeros(2, 16)
    w = torch.zeros(3)
    with pytest.raises(ValueError):
        B.sw_conv1d(x, w)


def test_float_nhwc_argument_errors(L):
    for f, esz in ((L.sw_conv2d_nhwc, 4), (L.sw_conv2d_bf16_nhwc, 2), (L.sw_conv2d_f16_nhwc, 2)):
        B_ = 0x2100000
        ok = (2, 8, 8, 32, 64, 3, 3, 1, 1, 1)      # N, H, W, C_in, C_out, R, S, stride, pad, dilation
        assert f(None, W_, None, Y, *ok, 0, None) == B.SW_ERR_NULL
        assert f(X, None, None, Y, *ok, 0, None) == B.SW_ERR_NULL
        assert f(X, W_, None, None, *ok, 0, None) == B.SW_ERR_NULL
        for i in (0, 1, 2, 3, 4, 5, 6, 7, 9):       # every extent, the stride and the dilation
            bad = list(ok)
            bad[i] = 0
            assert f(X, W_, None, Y, *bad, 0, None) == B.SW_ERR_SHAPE, i
        assert f(X, W_, None, Y, 2, 8, 8, 32, 64, 3, 3, 1, 1, 5, 0, None) == B.SW_ERR_SHAPE   # span 11 > 8 + 2
        assert f(X + 1, W_, None, Y, *ok, 0, None) == B.SW_ERR_ALIGN
        assert f(X, W_, None, Y + esz // 2, *ok, 0, None) == B.SW_ERR_ALIGN
        assert f(X, W_, B_ + 2, Y, *ok, 0, None) == B.SW_ERR_ALIGN                             # the fp32 bias
        assert f(X, W_, None, X + 64, *ok, 0, None) == B.SW_ERR_ALIAS
        assert f(X, W_, Y + 16, Y, *ok, 0, None) == B.SW_ERR_ALIAS


def test_probe_argument_errors_and_operation_counts(L):
    # the measurement aids refuse bad arguments before anything is enqueued
    assert L.sw_probe(B.SW_PROBE_FMA_F32, 0, None) == B.SW_ERR_SHAPE
    assert L.sw_probe(99, 10, None) == B.SW_ERR_UNSUPPORTED
    waves = 256 * 8
    assert L.sw_probe_ops(B.SW_PROBE_MFMA_F32, 3) == waves * 3 * 8 * 2 * 32 * 32 * 2
    assert L.sw_probe_ops(B.SW_PROBE_MFMA_I8, 3) == waves * 3 * 8 * 2 * 32 * 32 * 32
    assert L.sw_probe_ops(B.SW_PROBE_FMA_F32, 3) == waves * 3 * 48 * 4 * 2 * 64
    # sixteen rounds of nine FMAs (64 lanes) and one 16 x 16 x 4 matrix product
    assert L.sw_probe_ops(B.SW_PROBE_FMA_MFMA_F32, 3) == waves * 3 * 16 * (9 * 2 * 64 + 2 * 16 * 16 * 4)
    assert L.sw_probe_ops(B.SW_PROBE_MFMA_F32_FED, 3) == 256 * 4 * 3 * 8 * 2 * 32 * 32 * 2
    assert L.sw_probe_ops(B.SW_PROBE_MFMA_F32_FED2, 3) == 2 * L.sw_probe_ops(B.SW_PROBE_MFMA_F32_FED, 3)
    assert L.sw_probe_ops(B.SW_PROBE_MFMA_BF16, 3) == waves * 3 * 8 * 2 * 32 * 32 * 16
    assert L.sw_probe_ops(99, 3) == 0 and L.sw_probe_ops(B.SW_PROBE_FMA_F32, 0) == 0
