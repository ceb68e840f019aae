"""Host-side checks of the C-ABI boundary that need no GPU: the library loads,
exports every symbol the header declares, and rejects bad arguments before any
HIP call."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2104_10949_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2104_10949_amd import build
        build.build()
    return binding.lib()


def header_symbols():
    text = open(os.path.join(ROOT, "include", "cg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cg_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_entry_points():
    syms = header_symbols()
    for name in ("cg_share_matmul", "cg_share_conv2d", "cg_share_add", "cg_share_mul_public",
                 "cg_reconstruct", "cg_status_string", "cg_version"):
        assert name in syms


def test_library_exports_every_declared_symbol(L):
    from paper_2104_10949_amd import binding
    for name in header_symbols():
        assert hasattr(L, name), name
    assert sorted(binding.EXPORTS) == header_symbols()
    for name in binding.EXPORTS:        # every entry point is called with declared argument types
        assert getattr(L, name).argtypes is not None, name
    assert binding.version() >= 100
    assert binding.status_string(0) == "CG_OK"
    for s in range(1, 8):
        assert binding.status_string(s).startswith("CG_ERR_")


P = 0x10000  # fake, well-aligned, non-null "device" addresses; never dereferenced on the host


def test_matmul_validation_happens_before_any_device_work(L):
    from paper_2104_10949_amd import binding as b
    f = L.cg_share_matmul
    ok = [P, 2 * P, 3 * P, 4 * P, 5 * P]
    assert f(0, *ok[1:], 4, 4, 4, None) == b.CG_ERR_NULL
    assert f(*ok[:4], 0, 4, 4, 4, None) == b.CG_ERR_NULL
    assert f(*ok, 0, 4, 4, None) == b.CG_ERR_SHAPE
    assert f(*ok, 4, -1, 4, None) == b.CG_ERR_SHAPE
    assert f(*ok, 4, 4, 0, None) == b.CG_ERR_SHAPE
    assert f(*ok, 1 << 40, 1 << 40, 4, None) == b.CG_ERR_SHAPE          # M*N*8 overflows int64
    assert f(P + 4, *ok[1:], 4, 4, 4, None) == b.CG_ERR_ALIGN
    assert f(*ok[:4], P + 8, 4, 4, 4, None) == b.CG_ERR_ALIAS              # z inside x_i
    assert f(*ok[:4], 4 * P + 64, 4, 4, 4, None) == b.CG_ERR_ALIAS         # z inside y_ip1
    big = [1 << 40, 2 << 40, 3 << 40, 4 << 40, 5 << 40]
    assert f(*big, 4, 4, (1 << 30) + 1, None) == b.CG_ERR_UNSUPPORTED     # rows of up to 2^30 words are addressed
    assert f(*big, 1 << 31, 1, 1, None) == b.CG_ERR_UNSUPPORTED


def test_accumulating_entry_points_validate_like_the_plain_ones(L):
    from paper_2104_10949_amd import binding as b
    ok = [P, 2 * P, 3 * P, 4 * P, 5 * P]
    f = L.cg_share_matmul_acc
    assert f(0, *ok[1:], 4, 4, 4, None) == b.CG_ERR_NULL
    assert f(*ok[:4], 0, 4, 4, 4, None) == b.CG_ERR_NULL
    assert f(*ok, 4, 0, 4, None) == b.CG_ERR_SHAPE
    assert f(*ok[:4], 5 * P + 4, 4, 4, 4, None) == b.CG_ERR_ALIGN
    assert f(*ok[:4], P + 8, 4, 4, 4, None) == b.CG_ERR_ALIAS              # z inside x_i
    big = [1 << 40, 2 << 40, 3 << 40, 4 << 40, 5 << 40]
    assert f(*big, 4, 4, (1 << 30) + 1, None) == b.CG_ERR_UNSUPPORTED
    h = L.cg_share_matmul_f64limb                                          # the float64 comparator: same checks
    assert h(0, *ok[1:], 4, 4, 4, None) == b.CG_ERR_NULL
    assert h(*ok, 4, 4, 0, None) == b.CG_ERR_SHAPE
    assert h(*ok[:4], P + 8, 4, 4, 4, None) == b.CG_ERR_ALIAS
    assert h(*big, 4, 4, (1 << 20) + 1, None) == b.CG_ERR_UNSUPPORTED
    g = L.cg_share_conv2d_acc
    d = b.ConvDesc(1, 8, 8, 3, 4, 3, 3, 1, 1, 1, 1)
    assert g(*big, None, None) == b.CG_ERR_NULL
    assert g(*big[:4], 0, ctypes.byref(d), None) == b.CG_ERR_NULL
    assert g(*big[:4], big[1] + 16, ctypes.byref(d), None) == b.CG_ERR_ALIAS
    assert g(*big, ctypes.byref(b.ConvDesc(1, 8, 8, 3, 4, 11, 3, 1, 1, 1, 1)), None) == b.CG_ERR_SHAPE


def test_workspace_entry_points_validate_like_the_plain_ones(L):
    from paper_2104_10949_amd import binding as b
    big = [1 << 40, 2 << 40, 3 << 40, 4 << 40, 5 << 40]
    ws = 6 << 40
    f = L.cg_share_matmul_ws
    assert f(0, *big[1:], 4, 4, 4, ws, 1 << 20, None) == b.CG_ERR_NULL
    assert f(*big, 4, 0, 4, ws, 1 << 20, None) == b.CG_ERR_SHAPE
    assert f(*big, 128, 64, 64, 0, 1 << 20, None) == b.CG_ERR_NULL            # digit route needs scratch memory
    assert f(*big, 128, 64, 64, ws + 8, 1 << 20, None) == b.CG_ERR_ALIGN
    need = L.cg_share_matmul_workspace_bytes(128, 64, 64)
    assert need == (2 * 128 + 2 * 64) * 2 * 256
    assert f(*big, 128, 64, 64, ws, need - 1, None) == b.CG_ERR_WORKSPACE
    assert f(*big, 128, 64, 64, big[0] + 256, need, None) == b.CG_ERR_ALIAS   # scratch inside x_i
    assert L.cg_share_matmul_workspace_bytes(128, 64, 65) == 0               # odd K: no digit route
    assert L.cg_share_matmul_workspace_bytes(64, 64, 64) == 0                # few rows: computes as the plain call
    assert L.cg_share_matmul_workspace_bytes(-1, 64, 64) == 0
    d = b.ConvDesc(2, 8, 8, 32, 16, 3, 3, 1, 1, 1, 1)
    need = L.cg_share_conv2d_workspace_bytes(ctypes.byref(d))
    assert need == 2 * (2 * 8 * 8 * 32 * 8) + 2 * (16 * 9 * 256)
    assert L.cg_share_conv2d_ws(*big, ctypes.byref(d), ws, need - 1, None) == b.CG_ERR_WORKSPACE
    d3 = b.ConvDesc(2, 8, 8, 3, 16, 3, 3, 1, 1, 1, 1)
    assert L.cg_share_conv2d_workspace_bytes(ctypes.byref(d3)) == 0          # Cin = 3: direct route only
    assert L.cg_share_conv2d_workspace_bytes(None) == 0


def test_conv_validation(L):
    from paper_2104_10949_amd import binding as b
    f = L.cg_share_conv2d
    ok = [1 << 40, 2 << 40, 3 << 40, 4 << 40, 5 << 40]

    def desc(**kw):
        base = dict(B=1, H=8, W=8, Cin=3, Cout=4, kh=3, kw=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1)
        base.update(kw)
        return ctypes.byref(b.ConvDesc(**base))

    assert f(*ok, None, None) == b.CG_ERR_NULL
    assert f(0, *ok[1:], desc(), None) == b.CG_ERR_NULL
    assert f(*ok, desc(B=0), None) == b.CG_ERR_SHAPE
    assert f(*ok, desc(stride_h=0), None) == b.CG_ERR_SHAPE
    assert f(*ok, desc(pad_w=-1), None) == b.CG_ERR_SHAPE
    assert f(*ok, desc(kh=11, pad_h=1), None) == b.CG_ERR_SHAPE            # empty output
    assert f(*ok, desc(H=1 << 50), None) == b.CG_ERR_SHAPE
    assert f(ok[0] + 2, *ok[1:], desc(), None) == b.CG_ERR_ALIGN
    assert f(*ok[:4], ok[0] + 16, desc(), None) == b.CG_ERR_ALIAS
    assert f(*ok, desc(H=1 << 14, W=1 << 14), None) == b.CG_ERR_UNSUPPORTED  # one image too large for a view


def test_elementwise_validation(L):
    from paper_2104_10949_amd import binding as b
    a = [P, 2 * P, 3 * P, 4 * P, 5 * P, 6 * P]
    assert L.cg_share_add(*a[:5], 0, 16, None) == b.CG_ERR_NULL
    assert L.cg_share_add(*a[:5], 6 * P + 1, 16, None) == b.CG_ERR_ALIGN
    assert L.cg_share_add(*a[:4], P + 8, 6 * P, 16, None) == b.CG_ERR_ALIAS     # za partially overlaps xa
    assert L.cg_share_add(*a[:4], 5 * P, 5 * P + 8, 16, None) == b.CG_ERR_ALIAS  # za overlaps zb
    assert L.cg_share_add(*a, 0, None) == b.CG_OK                               # n == 0: nothing to do
    assert L.cg_share_mul_public(P, 2 * P, 3, 0, 4 * P, 8, None) == b.CG_ERR_NULL
    assert L.cg_share_mul_public(P, 2 * P, 3, P + 16, 4 * P, 8, None) == b.CG_ERR_ALIAS
    assert L.cg_share_add_public(P, 2 * P, 3, 3, 3 * P, 4 * P, 8, None) == b.CG_ERR_SHAPE
    assert L.cg_share_add_public(P, 2 * P, 3, -1, 3 * P, 4 * P, 8, None) == b.CG_ERR_SHAPE
    assert L.cg_reconstruct(P, 2 * P, 0, 4 * P, 8, None) == b.CG_ERR_NULL
    assert L.cg_reconstruct(P, 2 * P, 3 * P, 3 * P + 8, 8, None) == b.CG_ERR_ALIAS
    assert L.cg_reconstruct(P, 2 * P, 3 * P, 4 * P, 0, None) == b.CG_OK


def test_transposed_matmul_validation(L):
    from paper_2104_10949_amd import binding as b
    big = [1 << 40, 2 << 40, 3 << 40, 4 << 40, 5 << 40]
    f = L.cg_share_matmul_t
    assert f(*big, 4, 4, 4, 2, 0, None) == b.CG_ERR_SHAPE
    assert f(*big, 4, 4, 4, 0, -1, None) == b.CG_ERR_SHAPE
    assert f(0, *big[1:], 4, 4, 4, 1, 1, None) == b.CG_ERR_NULL
    assert f(*big, 4, 0, 4, 1, 1, None) == b.CG_ERR_SHAPE
    assert f(*big, (1 << 22) + 1, 4, 4, 1, 0, None) == b.CG_ERR_UNSUPPORTED
    assert f(*big, 4, (1 << 22) + 1, 4, 0, 1, None) == b.CG_ERR_UNSUPPORTED


def test_mul_and_pool_validation(L):
    from paper_2104_10949_amd import binding as b
    q = [P, 2 * P, 3 * P, 4 * P, 5 * P]
    assert L.cg_share_mul(*q, 0, 0, None) == b.CG_OK
    assert L.cg_share_mul(0, *q[1:], 8, 8, None) == b.CG_ERR_NULL
    assert L.cg_share_mul(*q, 8, 0, None) == b.CG_ERR_SHAPE
    assert L.cg_share_mul(*q, 8, 3, None) == b.CG_ERR_SHAPE          # period must divide n
    assert L.cg_share_mul(*q, 8, 16, None) == b.CG_ERR_SHAPE
    assert L.cg_share_mul(*q[:4], P + 8, 8, 8, None) == b.CG_ERR_ALIAS
    assert L.cg_share_mul(*q[:4], 3 * P, 8, 4, None) == b.CG_ERR_ALIAS  # in place over a broadcast y
    d = b.PoolDesc(1, 8, 8, 4, 2, 2, 2, 2, 0, 0)
    assert L.cg_share_sum_pool2d(P, 2 * P, 3 * P, 4 * P, None, None) == b.CG_ERR_NULL
    assert L.cg_share_sum_pool2d(0, 2 * P, 3 * P, 4 * P, ctypes.byref(d), None) == b.CG_ERR_NULL
    assert L.cg_share_sum_pool2d(P, 2 * P, P + 64, 4 * P, ctypes.byref(d), None) == b.CG_ERR_ALIAS
    bad = b.PoolDesc(1, 2, 2, 4, 3, 3, 1, 1, 0, 0)
    assert L.cg_share_sum_pool2d(P, 2 * P, 3 * P, 4 * P, ctypes.byref(bad), None) == b.CG_ERR_SHAPE
    bad = b.PoolDesc(1, 8, 8, 4, 2, 2, 0, 2, 0, 0)
    assert L.cg_share_sum_pool2d(P, 2 * P, 3 * P, 4 * P, ctypes.byref(bad), None) == b.CG_ERR_SHAPE


def test_prf_entry_points_validation(L):
    from paper_2104_10949_amd import binding as b
    k = bytes(16)
    assert L.cg_zero_share(None, k, 0, 0, P, 8, None) == b.CG_ERR_NULL
    assert L.cg_zero_share(k, k, 0, 0, 0, 8, None) == b.CG_ERR_NULL
    assert L.cg_zero_share(k, k, 0, 0, P + 4, 8, None) == b.CG_ERR_ALIGN
    assert L.cg_zero_share(k, k, 0, (1 << 64) - 4, P, 8, None) == b.CG_ERR_SHAPE   # index range wraps
    assert L.cg_zero_share(k, k, 0, 0, 0, 0, None) == b.CG_OK
    assert L.cg_reshare(0, k, k, 0, 0, P, 8, None) == b.CG_ERR_NULL
    assert L.cg_reshare(P, k, None, 0, 0, P, 8, None) == b.CG_ERR_NULL
    assert L.cg_reshare(P, k, k, 0, 0, P + 8, 8, None) == b.CG_ERR_ALIAS           # partial overlap
    assert L.cg_reshare(0, k, k, 0, 0, 0, 0, None) == b.CG_OK


def test_conv_backward_validation(L):
    from paper_2104_10949_amd import binding as b
    ok = [1 << 40, 2 << 40, 3 << 40, 4 << 40, 5 << 40]

    def desc(**kw):
        base = dict(B=2, H=8, W=8, Cin=4, Cout=6, kh=3, kw=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1)
        base.update(kw)
        return ctypes.byref(b.ConvDesc(**base))

    for f in (L.cg_share_conv2d_dgrad, L.cg_share_conv2d_wgrad):
        assert f(*ok, None, None) == b.CG_ERR_NULL
        assert f(*ok[:4], 0, desc(), None) == b.CG_ERR_NULL
        assert f(*ok, desc(Cout=0), None) == b.CG_ERR_SHAPE
        assert f(*ok, desc(kh=11, pad_h=1), None) == b.CG_ERR_SHAPE
        assert f(ok[0] + 4, *ok[1:], desc(), None) == b.CG_ERR_ALIGN
        assert f(*ok[:4], ok[0] + 8, desc(), None) == b.CG_ERR_ALIAS          # output inside the gradient
        assert f(*ok[:4], ok[2] + 8, desc(), None) == b.CG_ERR_ALIAS          # output inside the second operand
    # documented limits: contraction of the input gradient, rows of the weight gradient's transposed operand
    assert L.cg_share_conv2d_dgrad(*ok, desc(Cout=1 << 18, kh=3, kw=3), None) == b.CG_ERR_UNSUPPORTED
    assert L.cg_share_conv2d_wgrad(*ok, desc(Cout=(1 << 22) + 1), None) == b.CG_ERR_UNSUPPORTED


def test_static_scratch_entry_point_validates_and_bounds_its_size(L):
    from paper_2104_10949_amd import binding as b
    f = L.cg_share_matmul_static
    G = 1 << 32   # fake pointers far enough apart for 128 MB operands
    far = [G, 2 * G, 3 * G, 4 * G, 5 * G]
    assert f(0, *far[1:], 4, 4, 4, None) == b.CG_ERR_NULL
    assert f(*far, 4, 0, 4, None) == b.CG_ERR_SHAPE
    assert f(*far[:4], far[0] + 8, 4, 4, 4, None) == b.CG_ERR_ALIAS
    # 2 * (4096 + 4096) rows of 4096 words as digit planes are 512 MiB: beyond the fixed array, refused on the host
    assert L.cg_share_matmul_workspace_bytes(4096, 4096, 4096) > b.STATIC_SCRATCH_BYTES
    assert f(*far, 4096, 4096, 4096, None) == b.CG_ERR_WORKSPACE
    text = open(os.path.join(ROOT, "include", "cg.h")).read()
    assert re.search(r"#define\s+CG_STATIC_SCRATCH_BYTES\s+\(64u << 20\)", text) and b.STATIC_SCRATCH_BYTES == 64 << 20


def test_truncation_and_binary_gate_validation(L):
    from paper_2104_10949_amd import binding as b
    k = bytes(16)
    f = L.cg_trunc1_local
    assert f(P, None, None, k, 0, 0, 16, None, 0, 2 * P, 8, None) == b.CG_ERR_NULL
    assert f(P, None, k, k, 0, 0, 64, None, 0, 2 * P, 8, None) == b.CG_ERR_SHAPE
    assert f(P, None, k, k, 0, 0, -1, None, 0, 2 * P, 8, None) == b.CG_ERR_SHAPE
    assert f(0, None, k, k, 0, 0, 16, None, 0, 2 * P, 8, None) == b.CG_ERR_NULL
    assert f(P, P + 4, k, k, 0, 0, 16, None, 0, 2 * P, 8, None) == b.CG_ERR_ALIGN
    assert f(P, None, k, k, 0, 0, 16, None, 0, P + 8, 8, None) == b.CG_ERR_ALIAS
    assert f(P, None, k, k, 0, (1 << 64) - 2, 16, None, 0, 2 * P, 8, None) == b.CG_ERR_SHAPE
    assert f(0, None, k, k, 0, 0, 16, None, 0, 0, 0, None) == b.CG_OK
    # a mask stream that coincides with one of the two alpha streams (same key AND same nonce) blinds nothing
    k1, k2, k3 = bytes(range(16)), bytes(range(16, 32)), bytes(range(32, 48))
    assert f(P, None, k1, k2, 5, 0, 16, bytes(k1), 5, 2 * P, 8, None) == b.CG_ERR_SHAPE
    assert f(P, None, k1, k2, 5, 0, 16, bytes(k2), 5, 2 * P, 8, None) == b.CG_ERR_SHAPE
    assert f(0, None, k1, k2, 5, 0, 16, k1, 5, 0, 0, None) == b.CG_ERR_SHAPE       # checked even for n == 0
    assert f(0, None, k1, k2, 5, 0, 16, k1, 6, 0, 0, None) == b.CG_OK              # another nonce is fine
    assert f(0, None, k1, k2, 5, 0, 16, k3, 5, 0, 0, None) == b.CG_OK              # another key is fine
    assert L.cg_prf_words(None, 0, 0, P, 8, None) == b.CG_ERR_NULL
    assert L.cg_prf_words(k, 0, 0, P + 2, 8, None) == b.CG_ERR_ALIGN
    assert L.cg_prf_words(k, 0, 0, 0, 0, None) == b.CG_OK
    a = [P, 2 * P, 3 * P, 4 * P]
    assert L.cg_bshare_and(*a, 0, 8, None) == b.CG_ERR_NULL
    assert L.cg_bshare_and(*a, P + 8, 8, None) == b.CG_ERR_ALIAS
    assert L.cg_bshare_xor(*a, 5 * P, 5 * P + 8, 8, None) == b.CG_ERR_ALIAS        # the two outputs overlap
    assert L.cg_bshare_prefix_stage(*a, 0, 5 * P, 6 * P, 8, None) == b.CG_ERR_SHAPE
    assert L.cg_bshare_prefix_stage(*a, 64, 5 * P, 6 * P, 8, None) == b.CG_ERR_SHAPE
    assert L.cg_bshare_prefix_stage(*a, 1, None, 0, 8, None) == b.CG_ERR_NULL
    assert L.cg_bshare_prefix_stage(*a, 1, None, 6 * P, 0, None) == b.CG_OK
    assert L.cg_bshare_carry_level(*a, None, P + 64, 4, 4, None) == b.CG_ERR_ALIAS   # output inside an input
    assert L.cg_bshare_carry_level(*a, None, 6 * P, 1 << 40, 1 << 40, None) == b.CG_ERR_SHAPE
    assert L.cg_bit_transpose64(P, 2 * P, 65, None) == b.CG_ERR_SHAPE
    assert L.cg_bit_transpose64(P, P + 64, 128, None) == b.CG_ERR_ALIAS
    assert L.cg_bits_unpack(P, 0, 8, None) == b.CG_ERR_NULL
    six = [P, 2 * P, 3 * P, 4 * P, 5 * P, 6 * P]
    assert L.cg_bshare_csa(*six, 7 * P, 8 * P, 7 * P + 8, 8, None) == b.CG_ERR_ALIAS  # sum and carry overlap
    assert L.cg_bshare_csa(*six, 7 * P, 0, 9 * P, 8, None) == b.CG_ERR_NULL           # outputs are required
    assert L.cg_bshare_csa(P, None, None, 4 * P + 4, None, None, 7 * P, 8 * P, 9 * P, 8, None) == b.CG_ERR_ALIGN
    assert L.cg_bshare_csa(P, None, None, 4 * P, None, None, 7 * P, 8 * P, 4 * P + 8, 8, None) == b.CG_ERR_ALIAS
    assert L.cg_bshare_half_adder(*a, 5 * P, 6 * P, 0, 8, None) == b.CG_ERR_NULL


def test_bias_entry_points_validation(L):
    from paper_2104_10949_amd import binding as b
    a = [P, 2 * P, 3 * P, 4 * P, 5 * P, 6 * P]
    assert L.cg_share_bias_add(*a, 12, 5, None) == b.CG_ERR_SHAPE               # period does not divide n
    assert L.cg_share_bias_add(*a, 12, 0, None) == b.CG_ERR_SHAPE
    assert L.cg_share_bias_add(*a[:4], 3 * P, 6 * P, 12, 4, None) == b.CG_ERR_ALIAS   # output over the bias
    assert L.cg_share_bias_add(*a, 0, 0, None) == b.CG_OK
    assert L.cg_share_col_sum(P, 2 * P, 0, 4 * P, 8, 4, None) == b.CG_ERR_NULL
    assert L.cg_share_col_sum(P, 2 * P, P + 8, 4 * P, 8, 4, None) == b.CG_ERR_ALIAS
    assert L.cg_share_col_sum(P, 2 * P, 3 * P, 3 * P + 8, 8, 4, None) == b.CG_ERR_ALIAS
    assert L.cg_share_col_sum(P, 2 * P, 3 * P, 4 * P, 1 << 62, 8, None) == b.CG_ERR_SHAPE
    assert L.cg_share_col_sum(0, 0, 0, 0, 8, 0, None) == b.CG_OK


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2104_10949_amd import binding as b
    x = torch.zeros((2, 2), dtype=torch.int64)
    with pytest.raises(ValueError):
        b._ptr(x)
    with pytest.raises(TypeError):
        b._ptr(torch.zeros((2, 2), dtype=torch.float32))
