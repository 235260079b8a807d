"""The C-ABI library loads, exports every declared symbol and validates arguments (no GPU needed).

Validation runs on the host before any launch, so these calls use made-up device
addresses: a non-zero status means nothing was launched or dereferenced.
"""
import ctypes
import os
import re

import pytest

from paper_1802_04730_amd import build as tcbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tc355.h")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(tcbuild.LIB):
        tcbuild.build(force=True)
    from paper_1802_04730_amd import tc355
    return tc355.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tc_[a-z0-9_]+|tc355_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert {"tc_tbmm", "tc_mlp_fcrelu", "tc_group_conv", "tc_kron", "tc_group_conv_infer",
            "tc_mlp_fcrelu_workspace_bytes", "tc_status_string", "tc355_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    from paper_1802_04730_amd import tc355
    assert sorted(tc355.EXPORTS) == names


def test_status_strings(L):
    for code in range(8):
        s = L.tc_status_string(code).decode()
        assert s.startswith("TC_")
    assert L.tc355_version() >= 100


def test_group_conv_infer(L):
    oh, ow = ctypes.c_int64(), ctypes.c_int64()
    assert L.tc_group_conv_infer(58, 58, 3, 3, ctypes.byref(oh), ctypes.byref(ow)) == 0
    assert (oh.value, ow.value) == (56, 56)
    assert L.tc_group_conv_infer(7, 7, 3, 3, ctypes.byref(oh), ctypes.byref(ow)) == 0
    assert (oh.value, ow.value) == (5, 5)
    assert L.tc_group_conv_infer(2, 7, 3, 3, ctypes.byref(oh), ctypes.byref(ow)) == 2
    assert L.tc_group_conv_infer(7, 7, 0, 3, ctypes.byref(oh), ctypes.byref(ow)) == 2
    assert L.tc_group_conv_infer(7, 7, 3, 3, None, ctypes.byref(ow)) == 1


A, B_, C_ = 0x10000, 0x20000, 0x30000  # fake, 16-byte aligned "device" addresses


def test_tbmm_validation(L):
    assert L.tc_tbmm(None, B_, C_, 1, 2, 3, 4, None) == 1
    assert L.tc_tbmm(A, B_, C_, 1, 0, 3, 4, None) == 2
    assert L.tc_tbmm(A, B_, C_, -1, 2, 3, 4, None) == 2
    assert L.tc_tbmm(A, B_, A, 1, 2, 3, 4, None) == 3
    assert L.tc_tbmm(A + 4, B_, C_, 1, 2, 3, 4, None) == 4
    assert L.tc_tbmm(A, B_, C_, 1, 1 << 20, 1 << 20, 4, None) == 7
    assert L.tc_tbmm(A, B_, C_, 0, 2, 3, 4, None) == 0  # empty batch: nothing to do


def test_tbmm_ws_validation_and_workspace_size(L):
    W_ = 0x80000
    assert L.tc_tbmm_ws(None, B_, C_, 1, 2, 3, 4, W_, 1 << 20, None) == 1
    assert L.tc_tbmm_ws(A, B_, C_, 1, 0, 3, 4, W_, 1 << 20, None) == 2
    assert L.tc_tbmm_ws(A, B_, A, 1, 2, 3, 4, W_, 1 << 20, None) == 3
    assert L.tc_tbmm_ws(A, B_, C_, 1, 2, 3, 4, W_ + 4, 1 << 20, None) == 4     # misaligned workspace
    assert L.tc_tbmm_ws(A, B_, C_, 1, 2, 3, 4, C_, 1 << 20, None) == 3         # the workspace is the output
    assert L.tc_tbmm_ws(A, B_, C_, 0, 2, 3, 4, None, 0, None) == 0             # no workspace, empty batch
    # the paper's largest transposed matmul (Section 7): 32 reduction blocks x one block of 128 rows of X,
    # 64 KiB of digit records and 1 KiB of inverse scales each
    assert L.tc_tbmm_workspace_bytes(1, 128, 16384, 4096) == 32 * (65536 + 1024)
    assert L.tc_tbmm_workspace_bytes(3, 256, 16384, 2048) == 3 * 2 * 16 * (65536 + 1024)
    for shape in ((500, 26, 72, 26), (1, 128, 1024, 1024), (1, 128, 256, 32), (0, 128, 16384, 4096), (1, -128, 16384, 4096),
                  (1, 1 << 40, 1 << 40, 4096)):
        assert L.tc_tbmm_workspace_bytes(*shape) == 0


def test_kron_and_gconv_validation(L):
    assert L.tc_kron(A, B_, C_, None, 1, 2, 2, 2, 2, None) == 1
    assert L.tc_kron(A, B_, C_, 0x40000, 1, 2, 0, 2, 2, None) == 2
    assert L.tc_kron(A, B_, C_, C_, 1, 2, 2, 2, 2, None) == 3
    assert L.tc_kron(A, B_, C_, 0x40008, 1, 2, 2, 2, 2, None) == 4
    assert L.tc_kron(A, B_, C_, 0x40000, 0, 2, 2, 2, 2, None) == 0
    assert L.tc_group_conv(A, B_, None, None, 1, 1, 1, 1, 5, 5, 3, 3, None) == 1
    assert L.tc_group_conv(A, B_, None, C_, 1, 1, 1, 1, 2, 5, 3, 3, None) == 2
    assert L.tc_group_conv(A, B_, None, C_, 1, 0, 1, 1, 5, 5, 3, 3, None) == 2
    assert L.tc_group_conv(A, B_, C_, C_, 1, 1, 1, 1, 5, 5, 3, 3, None) == 3
    assert L.tc_group_conv(A, B_ + 8, None, C_, 1, 1, 1, 1, 5, 5, 3, 3, None) == 4
    assert L.tc_group_conv(A, B_, None, C_, 0, 1, 1, 1, 5, 5, 3, 3, None) == 0


def test_extents_whose_products_overflow_int64_are_unsupported_not_undefined(L):
    """Every extent product is formed without overflow: 2^32 x 2^32 = 2^64 must read as "too large", not as 0."""
    big = 1 << 32
    assert L.tc_group_conv(A, B_, None, C_, 1, 1, 1, 1, big, big, 3, 3, None) == 7
    assert L.tc_group_conv(A, B_, None, C_, 1, big, big, 1, 5, 5, 3, 3, None) == 7
    assert L.tc_group_conv(A, B_, None, C_, 1 << 62, 1, 1, 1, 5, 5, 3, 3, None) == 7
    assert L.tc_sconv2d(A, B_, None, C_, big, big, 1, 5, 5, 3, 3, 2, 2, None) == 7
    assert L.tc_sconv2d(A, B_, None, C_, 1, 1, 1, big, big, 3, 3, 1, 1, None) == 7
    assert L.tc_tbmm(A, B_, C_, 1, big, big, 1, None) == 7
    assert L.tc_tbmm(A, B_, C_, 1 << 62, 2, 3, 4, None) == 7
    assert L.tc_kron(A, B_, C_, 0x40000, 1, big, big, 2, 2, None) == 7
    assert L.tc_kron(A, B_, C_, 0x40000, 1 << 62, 2, 2, 2, 2, None) == 7
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    T, I, O = (vp * 1)(0x50000), (vp * 1)(0x70000), (vp * 1)(0x90000)
    assert L.tc_lut(1, T, I, O, (i64 * 1)(1000), (i64 * 1)(big), 64, big, None) == 7
    assert L.tc_lut(1, T, I, O, (i64 * 1)(1000), (i64 * 1)(50), big, big, None) == 7
    dims = (i64 * 2)(big, big)
    Wp, bp, Op = (vp * 1)(0x50000), (vp * 1)(0x60000), (vp * 1)(0x90000)
    assert L.tc_mlp_fcrelu(A, 1, 1, dims, Wp, bp, Op, None, 0, None) == 7
    assert L.tc_mlp_fcrelu(A, big, 1, (i64 * 2)(big, 4), Wp, bp, Op, None, 0, None) == 7


def test_sconv2d_validation_and_infer(L):
    oh, ow = ctypes.c_int64(), ctypes.c_int64()
    assert L.tc_sconv2d_infer(56, 56, 3, 3, 2, 2, ctypes.byref(oh), ctypes.byref(ow)) == 0
    assert (oh.value, ow.value) == (27, 27)
    assert L.tc_sconv2d_infer(10, 9, 3, 2, 2, 3, ctypes.byref(oh), ctypes.byref(ow)) == 0
    assert (oh.value, ow.value) == (4, 3)
    assert L.tc_sconv2d_infer(3, 3, 3, 3, 5, 5, ctypes.byref(oh), ctypes.byref(ow)) == 0
    assert (oh.value, ow.value) == (1, 1)
    assert L.tc_sconv2d_infer(2, 7, 3, 3, 1, 1, ctypes.byref(oh), ctypes.byref(ow)) == 2
    assert L.tc_sconv2d_infer(7, 7, 3, 3, 0, 1, ctypes.byref(oh), ctypes.byref(ow)) == 2
    assert L.tc_sconv2d_infer(7, 7, 3, 3, 1, 1, None, ctypes.byref(ow)) == 1
    assert L.tc_sconv2d(A, B_, None, None, 1, 1, 1, 5, 5, 3, 3, 2, 2, None) == 1
    assert L.tc_sconv2d(A, B_, None, C_, 1, 1, 1, 2, 5, 3, 3, 2, 2, None) == 2
    assert L.tc_sconv2d(A, B_, None, C_, 1, 0, 1, 5, 5, 3, 3, 2, 2, None) == 2
    assert L.tc_sconv2d(A, B_, None, C_, 1, 1, 1, 5, 5, 3, 3, 2, -1, None) == 2
    assert L.tc_sconv2d(A, B_, C_, C_, 1, 1, 1, 5, 5, 3, 3, 2, 2, None) == 3
    assert L.tc_sconv2d(A, B_ + 8, None, C_, 1, 1, 1, 5, 5, 3, 3, 2, 2, None) == 4
    assert L.tc_sconv2d(A, B_, None, C_, 1 << 12, 1 << 10, 1, 1 << 5, 1 << 5, 3, 3, 2, 2, None) == 7
    assert L.tc_sconv2d(A, B_, None, C_, 0, 1, 1, 5, 5, 3, 3, 2, 2, None) == 0


def test_lut_validation(L):
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    T = (vp * 2)(0x50000, 0x60000)
    I = (vp * 2)(0x70000, 0x80000)
    O = (vp * 2)(0x90000, 0xA0000)
    E = (i64 * 2)(1000, 2000)
    Ls = (i64 * 2)(50, 7)
    assert L.tc_lut(2, T, I, O, E, Ls, 64, 0, None) == 0  # empty batch: nothing to do
    assert L.tc_lut(2, None, I, O, E, Ls, 64, 4, None) == 1
    assert L.tc_lut(2, T, (vp * 2)(0x70000, None), O, E, Ls, 64, 4, None) == 1
    assert L.tc_lut(0, T, I, O, E, Ls, 64, 4, None) == 2
    assert L.tc_lut(9, T, I, O, E, Ls, 64, 4, None) == 2
    assert L.tc_lut(2, T, I, O, E, Ls, 0, 4, None) == 2
    assert L.tc_lut(2, T, I, O, (i64 * 2)(1000, 0), Ls, 64, 4, None) == 2
    assert L.tc_lut(2, T, I, O, E, (i64 * 2)(50, -1), 64, 4, None) == 2
    assert L.tc_lut(2, T, I, (vp * 2)(0x90000, 0x50000), E, Ls, 64, 4, None) == 3
    assert L.tc_lut(2, T, I, (vp * 2)(0x90000, 0x90000), E, Ls, 64, 4, None) == 3
    assert L.tc_lut(2, T, I, (vp * 2)(0x90000, 0xA0004), E, Ls, 64, 4, None) == 4
    assert L.tc_lut(2, T, I, O, (i64 * 2)(1000, 1 << 40), Ls, 64, 4, None) == 7


def test_mlp_validation(L):
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    dims = (i64 * 3)(8, 6, 4)
    W = (vp * 2)(0x50000, 0x60000)
    b = (vp * 2)(0x70000, 0x80000)
    O = (vp * 2)(0x90000, 0xA0000)
    need = L.tc_mlp_fcrelu_workspace_bytes(5, 2, dims)
    assert need >= 5 * 6 * 8 and need % 256 == 0
    assert L.tc_mlp_fcrelu_workspace_bytes(5, 1, dims) == 0
    assert L.tc_mlp_fcrelu_workspace_bytes(5, 0, dims) == 0
    assert L.tc_mlp_fcrelu(None, 5, 2, dims, W, b, O, 0xB0000, need, None) == 1
    assert L.tc_mlp_fcrelu(A, 5, 0, dims, W, b, O, 0xB0000, need, None) == 2
    assert L.tc_mlp_fcrelu(A, 5, 9, dims, W, b, O, 0xB0000, need, None) == 2
    bad = (i64 * 3)(8, 0, 4)
    assert L.tc_mlp_fcrelu(A, 5, 2, bad, W, b, O, 0xB0000, need, None) == 2
    Onull = (vp * 2)(0x90000, None)
    assert L.tc_mlp_fcrelu(A, 5, 2, dims, W, b, Onull, 0xB0000, need, None) == 1
    Oalias = (vp * 2)(0x90000, A)
    assert L.tc_mlp_fcrelu(A, 5, 2, dims, W, b, Oalias, 0xB0000, need, None) == 3
    assert L.tc_mlp_fcrelu(A, 5, 2, dims, W, b, O, None, 0, None) == 5
    assert L.tc_mlp_fcrelu(A, 5, 2, dims, W, b, O, 0xB0000, need - 1, None) == 5
    assert L.tc_mlp_fcrelu(A, 5, 2, dims, W, b, O, 0xB0010, need, None) == 5
    assert L.tc_mlp_fcrelu(A, 0, 2, dims, W, b, O, 0xB0000, need, None) == 0


def test_product_package_does_not_reach_the_oracle():
    pkg = os.path.join(ROOT, "paper_1802_04730_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "tc_oracle" not in text, f
