"""ctypes front end of the C oracle in ``ring_oracle.c``.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the product package never does.

All functions take and return numpy arrays of dtype uint64 (ring elements of
Z_{2^64}) or float64 (reals before encoding / after decoding).  The ring
products, convolutions, element-wise share operations, the PRF and the
truncation steps forward to the C routine of the same name, which writes the
paper's definition out as plain loops.  The binary-share section further down
(the adder circuits for the most significant bit, their gates and the bit-plane
helpers) is numpy arithmetic of this module's own: XOR / AND / shifts on whole
arrays, written gate by gate, and pinned by the plain integer sum of the shares
in ``tests/test_oracle_msb.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ring_oracle.c")
_LIB = os.path.join(_HERE, "libring_oracle.so")

_u64p = ctypes.POINTER(ctypes.c_uint64)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64
_sz = ctypes.c_size_t


def build(force: bool = False) -> str:
    """Compile ``ring_oracle.c`` with gcc into ``libring_oracle.so`` beside it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-march=native", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_set_num_threads.argtypes = [ctypes.c_int]
        L.oracle_set_num_threads.restype = None
        L.oracle_encode.argtypes = [_f64p, _u64p, _sz, ctypes.c_int]
        L.oracle_decode.argtypes = [_u64p, _f64p, _sz, ctypes.c_int]
        L.oracle_share.argtypes = [_u64p] * 6 + [_sz]
        L.oracle_reconstruct.argtypes = [_u64p] * 4 + [_sz]
        L.oracle_share_add.argtypes = [_u64p] * 6 + [_sz]
        L.oracle_share_mul_public.argtypes = [_u64p, _u64p, ctypes.c_uint64, _u64p, _u64p, _sz]
        L.oracle_share_add_public.argtypes = [_u64p, _u64p, ctypes.c_uint64, ctypes.c_int, _u64p, _u64p, _sz]
        L.oracle_matmul_u64.argtypes = [_u64p, _u64p, _u64p, _i64, _i64, _i64]
        L.oracle_conv_out_dim.argtypes = [_i64] * 4
        L.oracle_conv_out_dim.restype = _i64
        L.oracle_conv2d_u64.argtypes = [_u64p, _u64p, _u64p] + [_i64] * 11
        L.oracle_party_matmul.argtypes = [_u64p] * 5 + [_i64] * 3
        L.oracle_party_matmul.restype = ctypes.c_int
        L.oracle_party_conv2d.argtypes = [_u64p] * 5 + [_i64] * 11
        L.oracle_party_conv2d.restype = ctypes.c_int
        L.oracle_conv2d_dgrad_u64.argtypes = [_u64p, _u64p, _u64p] + [_i64] * 11
        L.oracle_conv2d_wgrad_u64.argtypes = [_u64p, _u64p, _u64p] + [_i64] * 11
        L.oracle_party_conv2d_dgrad.argtypes = [_u64p] * 5 + [_i64] * 11
        L.oracle_party_conv2d_dgrad.restype = ctypes.c_int
        L.oracle_party_conv2d_wgrad.argtypes = [_u64p] * 5 + [_i64] * 11
        L.oracle_party_conv2d_wgrad.restype = ctypes.c_int
        L.oracle_party_matmul_at.argtypes = [_u64p] * 4 + [_i64] * 3
        L.oracle_party_matmul_at.restype = ctypes.c_uint64
        L.oracle_party_conv2d_at.argtypes = [_u64p] * 4 + [_i64] * 13
        L.oracle_party_conv2d_at.restype = ctypes.c_uint64
        L.oracle_party_mul.argtypes = [_u64p] * 5 + [_sz, _sz]
        L.oracle_share_bias_add.argtypes = [_u64p] * 6 + [_sz, _sz]
        L.oracle_share_col_sum.argtypes = [_u64p] * 4 + [_sz, _sz]
        L.oracle_sum_pool2d.argtypes = [_u64p, _u64p] + [_i64] * 10
        u8p = ctypes.POINTER(ctypes.c_uint8)
        L.oracle_aes128_encrypt_block.argtypes = [u8p, u8p, u8p]
        L.oracle_prf_words.argtypes = [u8p, ctypes.c_uint64, ctypes.c_uint64, _u64p, _sz]
        L.oracle_zero_share.argtypes = [u8p, u8p, ctypes.c_uint64, ctypes.c_uint64, _u64p, _sz]
        L.oracle_zero_share.restype = ctypes.c_int
        L.oracle_reshare.argtypes = [_u64p, u8p, u8p, ctypes.c_uint64, ctypes.c_uint64, _u64p, _sz]
        L.oracle_reshare.restype = ctypes.c_int
        L.oracle_bshare_and.argtypes = [_u64p] * 5 + [_sz]
        L.oracle_bzero_share.argtypes = [u8p, u8p, ctypes.c_uint64, ctypes.c_uint64, _u64p, _sz]
        L.oracle_bzero_share.restype = ctypes.c_int
        L.oracle_trunc1_local.argtypes = [_u64p, _u64p, u8p, u8p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int,
                                          u8p, ctypes.c_uint64, _u64p, _sz]
        L.oracle_trunc1_local.restype = ctypes.c_int
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the C loops may use from now on (timing reports only; results do not depend on it)."""
    lib().oracle_set_num_threads(int(n))


def _u(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint64:
        raise TypeError(f"ring tensors are uint64, got {a.dtype}")
    return a


def _p(a: np.ndarray):
    return a.ctypes.data_as(_u64p)


def encode(x, t: int = 16) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint64)
    lib().oracle_encode(x.ctypes.data_as(_f64p), _p(out), x.size, int(t))
    return out


def decode(z, bits: int) -> np.ndarray:
    z = _u(z)
    out = np.empty(z.shape, dtype=np.float64)
    lib().oracle_decode(_p(z), out.ctypes.data_as(_f64p), z.size, int(bits))
    return out


def share(x, r0, r1):
    """Split x into (s0, s1, s2) with s0 = r0, s1 = r1, s2 = x - r0 - r1."""
    x, r0, r1 = _u(x), _u(r0), _u(r1)
    assert x.shape == r0.shape == r1.shape
    s = [np.empty(x.shape, dtype=np.uint64) for _ in range(3)]
    lib().oracle_share(_p(x), _p(r0), _p(r1), _p(s[0]), _p(s[1]), _p(s[2]), x.size)
    return tuple(s)


def party_pair(shares, i: int):
    """Party i's replicated pair (s_i, s_{i+1 mod 3})."""
    return shares[i % 3], shares[(i + 1) % 3]


def reconstruct(s0, s1, s2) -> np.ndarray:
    s0, s1, s2 = _u(s0), _u(s1), _u(s2)
    assert s0.shape == s1.shape == s2.shape
    out = np.empty(s0.shape, dtype=np.uint64)
    lib().oracle_reconstruct(_p(s0), _p(s1), _p(s2), _p(out), s0.size)
    return out


def share_add(xa, xb, ya, yb):
    xa, xb, ya, yb = _u(xa), _u(xb), _u(ya), _u(yb)
    za, zb = np.empty_like(xa), np.empty_like(xb)
    lib().oracle_share_add(_p(xa), _p(xb), _p(ya), _p(yb), _p(za), _p(zb), xa.size)
    return za, zb


def share_mul_public(xa, xb, alpha: int):
    xa, xb = _u(xa), _u(xb)
    za, zb = np.empty_like(xa), np.empty_like(xb)
    lib().oracle_share_mul_public(_p(xa), _p(xb), ctypes.c_uint64(alpha % (1 << 64)), _p(za), _p(zb), xa.size)
    return za, zb


def share_add_public(xa, xb, gamma: int, party: int):
    xa, xb = _u(xa), _u(xb)
    za, zb = np.empty_like(xa), np.empty_like(xb)
    lib().oracle_share_add_public(_p(xa), _p(xb), ctypes.c_uint64(gamma % (1 << 64)), int(party),
                                  _p(za), _p(zb), xa.size)
    return za, zb


def matmul(A, Y) -> np.ndarray:
    """C[m,n] = sum_k A[m,k] * Y[n,k] mod 2^64; A is [M,K], Y is [N,K]."""
    A, Y = _u(A), _u(Y)
    M, K = A.shape
    N, K2 = Y.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.uint64)
    lib().oracle_matmul_u64(_p(A), _p(Y), _p(C), M, N, K)
    return C


def conv_out_dim(n: int, k: int, stride: int, pad: int) -> int:
    return int(lib().oracle_conv_out_dim(n, k, stride, pad))


def conv2d(X, W, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """X NHWC [B,H,W,Cin], W [Cout,kh,kw,Cin] -> Z NHWC [B,Ho,Wo,Cout]."""
    X, W = _u(X), _u(W)
    B, H, Wd, Cin = X.shape
    Cout, kh, kw, Cin2 = W.shape
    assert Cin == Cin2
    sh, sw = stride
    ph, pw = pad
    Ho, Wo = conv_out_dim(H, kh, sh, ph), conv_out_dim(Wd, kw, sw, pw)
    Z = np.empty((B, Ho, Wo, Cout), dtype=np.uint64)
    lib().oracle_conv2d_u64(_p(X), _p(W), _p(Z), B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw)
    return Z


def party_matmul(x_i, x_ip1, y_i, y_ip1) -> np.ndarray:
    x_i, x_ip1, y_i, y_ip1 = _u(x_i), _u(x_ip1), _u(y_i), _u(y_ip1)
    M, K = x_i.shape
    N, _ = y_i.shape
    assert x_ip1.shape == (M, K) and y_i.shape == (N, K) and y_ip1.shape == (N, K)
    z = np.empty((M, N), dtype=np.uint64)
    rc = lib().oracle_party_matmul(_p(x_i), _p(x_ip1), _p(y_i), _p(y_ip1), _p(z), M, N, K)
    if rc != 0:
        raise MemoryError("oracle_party_matmul")
    return z


def party_matmul_t(x_i, x_ip1, y_i, y_ip1, trans_x: bool, trans_y: bool) -> np.ndarray:
    """party_matmul on operands that are stored transposed: the stored arrays are transposed back
    (a copy, no arithmetic) and handed to the same C routine."""
    t = lambda a, flag: np.ascontiguousarray(_u(a).T) if flag else _u(a)
    return party_matmul(t(x_i, trans_x), t(x_ip1, trans_x), t(y_i, trans_y), t(y_ip1, trans_y))


def party_conv2d(x_i, x_ip1, w_i, w_ip1, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    x_i, x_ip1, w_i, w_ip1 = _u(x_i), _u(x_ip1), _u(w_i), _u(w_ip1)
    B, H, Wd, Cin = x_i.shape
    Cout, kh, kw, _ = w_i.shape
    assert x_ip1.shape == x_i.shape and w_ip1.shape == w_i.shape and w_i.shape[3] == Cin
    sh, sw = stride
    ph, pw = pad
    Ho, Wo = conv_out_dim(H, kh, sh, ph), conv_out_dim(Wd, kw, sw, pw)
    z = np.empty((B, Ho, Wo, Cout), dtype=np.uint64)
    rc = lib().oracle_party_conv2d(_p(x_i), _p(x_ip1), _p(w_i), _p(w_ip1), _p(z),
                                   B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw)
    if rc != 0:
        raise MemoryError("oracle_party_conv2d")
    return z


def _conv_dims(x_shape, w_shape, g_shape, stride, pad):
    B, H, Wd, Cin = x_shape
    Cout, kh, kw, Cin2 = w_shape
    assert Cin == Cin2
    Ho, Wo = conv_out_dim(H, kh, stride[0], pad[0]), conv_out_dim(Wd, kw, stride[1], pad[1])
    assert tuple(g_shape) == (B, Ho, Wo, Cout), (g_shape, (B, Ho, Wo, Cout))
    return B, H, Wd, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1]


def conv2d_dgrad(G, W, x_shape, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """Gradient of conv2d(X, W) with respect to X: G [B,Ho,Wo,Cout], W [Cout,kh,kw,Cin] -> [B,H,W,Cin]."""
    G, W = _u(G), _u(W)
    dims = _conv_dims(x_shape, W.shape, G.shape, stride, pad)
    DX = np.empty(tuple(x_shape), dtype=np.uint64)
    lib().oracle_conv2d_dgrad_u64(_p(G), _p(W), _p(DX), *dims)
    return DX


def conv2d_wgrad(G, X, w_shape, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """Gradient of conv2d(X, W) with respect to W: G [B,Ho,Wo,Cout], X [B,H,W,Cin] -> [Cout,kh,kw,Cin]."""
    G, X = _u(G), _u(X)
    dims = _conv_dims(X.shape, w_shape, G.shape, stride, pad)
    DW = np.empty(tuple(w_shape), dtype=np.uint64)
    lib().oracle_conv2d_wgrad_u64(_p(G), _p(X), _p(DW), *dims)
    return DW


def party_conv2d_dgrad(g_i, g_ip1, w_i, w_ip1, x_shape, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    g_i, g_ip1, w_i, w_ip1 = _u(g_i), _u(g_ip1), _u(w_i), _u(w_ip1)
    assert g_ip1.shape == g_i.shape and w_ip1.shape == w_i.shape
    dims = _conv_dims(x_shape, w_i.shape, g_i.shape, stride, pad)
    dx = np.empty(tuple(x_shape), dtype=np.uint64)
    if lib().oracle_party_conv2d_dgrad(_p(g_i), _p(g_ip1), _p(w_i), _p(w_ip1), _p(dx), *dims) != 0:
        raise MemoryError("oracle_party_conv2d_dgrad")
    return dx


def party_conv2d_wgrad(g_i, g_ip1, x_i, x_ip1, w_shape, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    g_i, g_ip1, x_i, x_ip1 = _u(g_i), _u(g_ip1), _u(x_i), _u(x_ip1)
    assert g_ip1.shape == g_i.shape and x_ip1.shape == x_i.shape
    dims = _conv_dims(x_i.shape, w_shape, g_i.shape, stride, pad)
    dw = np.empty(tuple(w_shape), dtype=np.uint64)
    if lib().oracle_party_conv2d_wgrad(_p(g_i), _p(g_ip1), _p(x_i), _p(x_ip1), _p(dw), *dims) != 0:
        raise MemoryError("oracle_party_conv2d_wgrad")
    return dw


def party_matmul_at(x_i, x_ip1, y_i, y_ip1, m: int, n: int) -> int:
    x_i, x_ip1, y_i, y_ip1 = _u(x_i), _u(x_ip1), _u(y_i), _u(y_ip1)
    K = x_i.shape[1]
    return int(lib().oracle_party_matmul_at(_p(x_i), _p(x_ip1), _p(y_i), _p(y_ip1), m, n, K))


def party_conv2d_at(x_i, x_ip1, w_i, w_ip1, b, ho, wo, co, stride=(1, 1), pad=(0, 0)) -> int:
    x_i, x_ip1, w_i, w_ip1 = _u(x_i), _u(x_ip1), _u(w_i), _u(w_ip1)
    _, H, Wd, Cin = x_i.shape
    _, kh, kw, _ = w_i.shape
    return int(lib().oracle_party_conv2d_at(_p(x_i), _p(x_ip1), _p(w_i), _p(w_ip1), b, ho, wo, co,
                                            H, Wd, Cin, kh, kw, stride[0], stride[1], pad[0], pad[1]))


def _key(key: bytes):
    if len(key) != 16:
        raise ValueError("AES-128 keys are 16 bytes")
    return (ctypes.c_uint8 * 16).from_buffer_copy(bytes(key))


def aes128_encrypt_block(key: bytes, block: bytes) -> bytes:
    out = (ctypes.c_uint8 * 16)()
    lib().oracle_aes128_encrypt_block(_key(key), _key(block), out)
    return bytes(out)


def prf_words(key: bytes, nonce: int, first: int, n: int) -> np.ndarray:
    """F(key, first + j) for j < n (AES-128 counter mode, see ring_oracle.c)."""
    out = np.empty(n, dtype=np.uint64)
    lib().oracle_prf_words(_key(key), nonce, first, _p(out), n)
    return out


def zero_share(key_self: bytes, key_prev: bytes, nonce: int, first: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint64)
    if lib().oracle_zero_share(_key(key_self), _key(key_prev), nonce, first, _p(out), n):
        raise MemoryError("oracle_zero_share")
    return out


def reshare(z, key_self: bytes, key_prev: bytes, nonce: int, first: int) -> np.ndarray:
    z = _u(z)
    out = np.empty(z.shape, dtype=np.uint64)
    if lib().oracle_reshare(_p(z), _key(key_self), _key(key_prev), nonce, first, _p(out), z.size):
        raise MemoryError("oracle_reshare")
    return out


def trunc1_local(z, msg, key_self: bytes, key_prev: bytes, nonce: int, first: int, d: int,
                 key_mask=None, mask_nonce: int = 0) -> np.ndarray:
    """One party's local step of the share truncation: asr(z + alpha + msg, d) - F(key_mask, .)."""
    z = _u(z)
    m = None if msg is None else _u(msg)
    out = np.empty(z.shape, dtype=np.uint64)
    rc = lib().oracle_trunc1_local(_p(z), None if m is None else _p(m), _key(key_self), _key(key_prev), nonce, first,
                                   d, None if key_mask is None else _key(key_mask), mask_nonce, _p(out), z.size)
    if rc != 0:
        raise MemoryError("oracle_trunc1_local") if rc == -1 else ValueError("shift outside [0, 63]")
    return out


def trunc1_protocol(z, keys, nonce: int, first: int, d: int, mask_nonce: int):
    """All three parties' steps of the two-round share truncation on the additive product shares
    z = (z_0, z_1, z_2); keys = (k_0, k_1, k_2), P_i holding k_i and k_{i-1}.  Messages are plain
    assignments here.  Returns the new shares (s_0, s_1, s_2); P_i ends up with (s_i, s_{i+1})."""
    k0, k1, k2 = keys
    # round 1: P_2 blinds its share and sends it to P_1
    msg = reshare(z[2], k2, k1, nonce, first)
    # local steps
    s0 = trunc1_local(z[0], None, k0, k2, nonce, first, d)                       # P_0
    s1 = trunc1_local(z[1], msg, k1, k0, nonce, first, d, k1, mask_nonce)        # P_1 (mask key shared with P_2)
    s2 = prf_words(k1, mask_nonce, first, _u(z[2]).size).reshape(_u(z[2]).shape)  # P_2 and P_1: the mask itself
    # round 2: P_1 -> P_0: s1, P_0 -> P_2: s0 (no arithmetic)
    return s0, s1, s2


# ---- binary replicated shares and the adder circuit for the most significant bit ----------------
def bshare_and(x_i, x_ip1, y_i, y_ip1) -> np.ndarray:
    """One party's local step of an AND gate on binary shares (64 gates per word)."""
    x_i, x_ip1, y_i, y_ip1 = _u(x_i), _u(x_ip1), _u(y_i), _u(y_ip1)
    assert x_i.shape == x_ip1.shape == y_i.shape == y_ip1.shape
    z = np.empty(x_i.shape, dtype=np.uint64)
    lib().oracle_bshare_and(_p(x_i), _p(x_ip1), _p(y_i), _p(y_ip1), _p(z), x_i.size)
    return z


def bzero_share(key_self: bytes, key_prev: bytes, nonce: int, first: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint64)
    if lib().oracle_bzero_share(_key(key_self), _key(key_prev), nonce, first, _p(out), n):
        raise MemoryError("oracle_bzero_share")
    return out


def breshare(z, key_self: bytes, key_prev: bytes, nonce: int, first: int) -> np.ndarray:
    """z ^ beta: the blinded XOR share a party passes on after an AND gate."""
    z = _u(z)
    return z ^ bzero_share(key_self, key_prev, nonce, first, z.size).reshape(z.shape)


def csa_local(a_i, a_ip1, b_i, b_ip1, c_i, c_ip1):
    """One party's local step of a carry-save (full) adder on three binary sharings: the sum S = A ^ B ^ C as a
    pair (XOR gates only), and its XOR share of the carry majority(A, B, C) = ((A ^ C) & (B ^ C)) ^ C before
    blinding (one AND gate by the three-term formula; the party adds its own component C_i)."""
    a_i, a_ip1, b_i, b_ip1, c_i, c_ip1 = (_u(v) for v in (a_i, a_ip1, b_i, b_ip1, c_i, c_ip1))
    s_i, s_ip1 = a_i ^ b_i ^ c_i, a_ip1 ^ b_ip1 ^ c_ip1
    carry = bshare_and(a_i ^ c_i, a_ip1 ^ c_ip1, b_i ^ c_i, b_ip1 ^ c_ip1) ^ c_i
    return s_i, s_ip1, carry


def half_adder_local(s_i, s_ip1, t_i, t_ip1):
    """One party's local step of a half adder on two binary sharings: propagate P = S ^ T as a pair and its
    XOR share of generate G = S & T before blinding."""
    s_i, s_ip1, t_i, t_ip1 = (_u(v) for v in (s_i, s_ip1, t_i, t_ip1))
    return s_i ^ t_i, s_ip1 ^ t_ip1, bshare_and(s_i, s_ip1, t_i, t_ip1)


def ks_stage_local(p_i, p_ip1, g_i, g_ip1, shift: int, last: bool = False):
    """One party's local step of one stage of the parallel-prefix adder on (propagate, generate) words:
    g' = g ^ (p & (g << shift)), p' = p & (p << shift), both AND gates by the three-term formula; the party
    adds its own component g_i.  Returns (p', g') as this party's XOR shares (p' is None for the last stage)."""
    p_i, p_ip1, g_i, g_ip1 = _u(p_i), _u(p_ip1), _u(g_i), _u(g_ip1)
    sh = np.uint64(shift)
    g_new = g_i ^ bshare_and(p_i, p_ip1, g_i << sh, g_ip1 << sh)
    p_new = None if last else bshare_and(p_i, p_ip1, p_i << sh, p_ip1 << sh)
    return p_new, g_new


def msb_protocol(x, keys, nonce: int):
    """All three parties' steps of the addition circuit on x = (x_0, x_1, x_2), the arithmetic shares of a
    tensor (P_i holds x_i and x_{i+1}).  Each x_k is taken as a binary sharing with one non-zero component;
    a carry-save step (one AND round) reduces the three addends to two, and a 64-bit parallel-prefix adder
    (one AND round for the first generate word, six stages) adds those.  Messages are plain assignments.
    Returns (sum, msb): binary sharings, as triples, of the 64-bit sum and of its top bit (in bit 0)."""
    x = [_u(a) for a in x]
    n, shape = x[0].size, x[0].shape
    zero = np.zeros(shape, dtype=np.uint64)
    pair = lambda v, i: (v[i], v[(i + 1) % 3])
    counter = [0]

    def and_gate(X, Y):
        first = counter[0]
        counter[0] += n
        return tuple(breshare(bshare_and(*pair(X, i), *pair(Y, i)), keys[i], keys[(i - 1) % 3], nonce, first)
                     for i in range(3))

    xor = lambda X, Y: tuple(a ^ b for a, b in zip(X, Y))
    A, B, C = (x[0], zero, zero), (zero, x[1], zero), (zero, zero, x[2])
    # carry-save: S = A ^ B ^ C, carry = majority(A, B, C) = ((A ^ C) & (B ^ C)) ^ C
    S = xor(xor(A, B), C)
    carry = xor(and_gate(xor(A, C), xor(B, C)), C)
    T = tuple(c << np.uint64(1) for c in carry)
    # parallel-prefix adder of S and T
    P0 = xor(S, T)
    G = and_gate(S, T)
    P = P0
    for stage, shift in enumerate((1, 2, 4, 8, 16, 32)):
        last = stage == 5
        first = counter[0]
        counter[0] += 2 * n
        new_p, new_g = [], []
        for i in range(3):
            p_loc, g_loc = ks_stage_local(*pair(P, i), *pair(G, i), shift, last)
            ks, kp = keys[i], keys[(i - 1) % 3]
            new_g.append(breshare(g_loc, ks, kp, nonce, first))
            if not last:
                new_p.append(breshare(p_loc, ks, kp, nonce, first + n))
        G = tuple(new_g)
        if not last:
            P = tuple(new_p)
    total = xor(P0, tuple(g << np.uint64(1) for g in G))
    msb = tuple(t >> np.uint64(63) for t in total)
    return total, msb


# ---- the same sign bit from a circuit pruned to it, on bit planes ---------------------------------
def bit_planes(x) -> np.ndarray:
    """64 x 64 bit transpose of a flat tensor of n = 64 m words: plane b (row b of the result, m words) holds
    bit b of every element, element 64 w + e in bit e of word w.  Written with numpy's bit unpacking."""
    x = _u(x).reshape(-1)
    assert x.size % 64 == 0
    m = x.size // 64
    bits = np.unpackbits(x.view(np.uint8).reshape(x.size, 8), axis=1, bitorder="little")      # [n, 64]: bit b of element i
    per_plane = bits.T.reshape(64, m, 64)                                                    # [b, w, e]
    packed = np.packbits(per_plane, axis=2, bitorder="little")                               # [b, w, 8 bytes]
    return np.ascontiguousarray(packed).view(np.uint64).reshape(64, m)


def bits_unpack(plane, n: int) -> np.ndarray:
    """Inverse for a single plane: word i of the result is bit i % 64 of plane[i // 64]."""
    plane = _u(plane).reshape(-1)
    bits = np.unpackbits(plane.view(np.uint8), bitorder="little")[:n]
    return bits.astype(np.uint64)


def carry_level_local(p_i, p_ip1, g_i, g_ip1, last: bool = False):
    """One party's local step of one level of the carry tree on planes [2k, m] -> [k, m]: neighbouring
    segments (hi = plane 2j+1, lo = plane 2j) are merged by g' = g_hi ^ (p_hi & g_lo), p' = p_hi & p_lo."""
    p_i, p_ip1, g_i, g_ip1 = _u(p_i), _u(p_ip1), _u(g_i), _u(g_ip1)
    hi, lo = slice(1, None, 2), slice(0, None, 2)
    c = np.ascontiguousarray
    g_new = g_i[hi] ^ bshare_and(c(p_i[hi]), c(p_ip1[hi]), c(g_i[lo]), c(g_ip1[lo]))
    p_new = None if last else bshare_and(c(p_i[hi]), c(p_ip1[hi]), c(p_i[lo]), c(p_ip1[lo]))
    return p_new, g_new


def msb_protocol_sliced(x, keys, nonce: int):
    """The sign bit of x_0 + x_1 + x_2 from a circuit pruned to that one output, evaluated on bit planes
    (n = 64 m elements).  Local: every party transposes its two shares into planes.  Carry-save step on all 64
    planes (one AND round), first generate word (one AND round), then a binary tree over the 64 positions
    "below bit 63" (leaf q holds bit q - 1, leaf 0 is empty) that merges neighbouring segments, six AND rounds
    on 32, 16, 8, 4, 2, 1 planes.  254 plane-sized AND gates instead of the 832 of the word-parallel adder.
    Returns the binary sharing (triple of [m] words) of the packed sign bits."""
    x = [_u(a).reshape(-1) for a in x]
    n = x[0].size
    m = n // 64
    zero = np.zeros((64, m), dtype=np.uint64)
    pair = lambda v, i: (v[i], v[(i + 1) % 3])
    counter = [0]

    def blind(z, i):
        first = counter[0]
        return breshare(z.reshape(-1), keys[i], keys[(i - 1) % 3], nonce, first).reshape(z.shape)

    def and_gate(X, Y):
        out = tuple(blind(bshare_and(*pair(X, i), *pair(Y, i)), i) for i in range(3))
        counter[0] += X[0].size
        return out

    xor = lambda X, Y: tuple(a ^ b for a, b in zip(X, Y))
    planes = [bit_planes(a) for a in x]
    A, B, C = (planes[0], zero, zero), (zero, planes[1], zero), (zero, zero, planes[2])
    S = xor(xor(A, B), C)
    carry = xor(and_gate(xor(A, C), xor(B, C)), C)
    up = lambda v: np.concatenate([np.zeros((1, m), dtype=np.uint64), v[:63]])       # one bit position up, plane-wise
    T = tuple(up(c) for c in carry)
    P0 = xor(S, T)
    G0 = and_gate(S, T)
    # leaves of the tree: position q = bit q - 1 (the carry into bit 63 is the generate of bits 0..62)
    P, G = tuple(up(p) for p in P0), tuple(up(g) for g in G0)
    while P[0].shape[0] > 1:
        last = P[0].shape[0] == 2
        loc = [carry_level_local(*pair(P, i), *pair(G, i), last) for i in range(3)]
        G = tuple(blind(loc[i][1], i) for i in range(3))
        counter[0] += G[0].size
        if not last:
            P = tuple(blind(loc[i][0], i) for i in range(3))
            counter[0] += P[0].size
        else:
            P = tuple(g[:1] for g in G)   # only the shape is used from here on
    return tuple(p0[63] ^ g[0] for p0, g in zip(P0, G))


def party_mul(x_i, x_ip1, y_i, y_ip1) -> np.ndarray:
    """Element-wise local multiplication step; y is broadcast along the leading dimensions of x
    (y.size must divide x.size and match x's trailing elements)."""
    x_i, x_ip1, y_i, y_ip1 = _u(x_i), _u(x_ip1), _u(y_i), _u(y_ip1)
    assert x_i.shape == x_ip1.shape and y_i.shape == y_ip1.shape and x_i.size % max(y_i.size, 1) == 0
    z = np.empty(x_i.shape, dtype=np.uint64)
    if x_i.size:
        lib().oracle_party_mul(_p(x_i), _p(x_ip1), _p(y_i), _p(y_ip1), _p(z), x_i.size, y_i.size)
    return z


def share_bias_add(xa, xb, ba, bb):
    """(xa + ba, xb + bb) with the bias [cols] broadcast over the rows of x [..., cols]."""
    xa, xb, ba, bb = _u(xa), _u(xb), _u(ba), _u(bb)
    cols = ba.size
    assert xa.shape == xb.shape and bb.size == cols and xa.shape[-1] == cols
    za, zb = np.empty(xa.shape, dtype=np.uint64), np.empty(xa.shape, dtype=np.uint64)
    lib().oracle_share_bias_add(_p(xa), _p(xb), _p(ba), _p(bb), _p(za), _p(zb), xa.size // cols, cols)
    return za, zb


def share_col_sum(xa, xb):
    """Column sums of both components of x [..., cols] over all leading dimensions."""
    xa, xb = _u(xa), _u(xb)
    cols = xa.shape[-1]
    za, zb = np.empty(cols, dtype=np.uint64), np.empty(cols, dtype=np.uint64)
    lib().oracle_share_col_sum(_p(xa), _p(xb), _p(za), _p(zb), xa.size // cols, cols)
    return za, zb


def sum_pool2d(X, window, stride, pad=(0, 0)) -> np.ndarray:
    X = _u(X)
    B, H, Wd, C = X.shape
    kh, kw = window
    Ho, Wo = conv_out_dim(H, kh, stride[0], pad[0]), conv_out_dim(Wd, kw, stride[1], pad[1])
    Z = np.empty((B, Ho, Wo, C), dtype=np.uint64)
    lib().oracle_sum_pool2d(_p(X), _p(Z), B, H, Wd, C, kh, kw, stride[0], stride[1], pad[0], pad[1])
    return Z
