"""Pins for the CPU oracle (no GPU).

The oracle is checked against things other than itself: Python big-integer
brute force, closed forms, algebraic identities the paper states, an explicit
patch-matrix formulation built here with numpy indexing, output sizes the
paper prints, and an fp64 product of the decoded operands.
"""
import os

import numpy as np
import pytest

from oracle import ring_oracle as ro
from paper_2104_10949_amd import workloads as wl

MOD = 1 << 64
HERE = os.path.dirname(os.path.abspath(__file__))


def ring(shape, seed):
    return wl.draw_ring(shape, seed)


def to_int(a):
    return [int(v) for v in np.asarray(a).reshape(-1)]


# ---------------------------------------------------------------- brute force
def bf_matmul(A, Y):
    M, K = A.shape
    N = Y.shape[0]
    a, y = A.tolist(), Y.tolist()
    return np.array([[sum(a[m][k] * y[n][k] for k in range(K)) % MOD for n in range(N)]
                     for m in range(M)], dtype=np.uint64).reshape(M, N)


def bf_conv(X, W, stride, pad):
    B, H, Wd, C = X.shape
    Co, kh, kw, _ = W.shape
    sh, sw = stride
    ph, pw = pad
    Ho = (H + 2 * ph - kh) // sh + 1
    Wo = (Wd + 2 * pw - kw) // sw + 1
    x, w = X.tolist(), W.tolist()
    Z = np.zeros((B, Ho, Wo, Co), dtype=np.uint64)
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Co):
                    acc = 0
                    for r in range(kh):
                        for s in range(kw):
                            hi, wi = ho * sh - ph + r, wo * sw - pw + s
                            if 0 <= hi < H and 0 <= wi < Wd:
                                for c in range(C):
                                    acc += x[b][hi][wi][c] * w[co][r][s][c]
                    Z[b, ho, wo, co] = acc % MOD
    return Z


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 1), (3, 2, 5), (8, 8, 8), (5, 7, 6), (1, 4, 9)])
def test_matmul_bigint_bruteforce(M, N, K):
    A, Y = ring((M, K), 11 + M + 10 * N + 100 * K), ring((N, K), 12 + M + 10 * N + 100 * K)
    assert np.array_equal(ro.matmul(A, Y), bf_matmul(A, Y))


def test_matmul_is_not_symmetric_in_its_operands():
    # a transposed or swapped operand must fail the brute-force pin above; show the
    # pin has teeth on a non-square case
    A, Y = ring((3, 4), 5), ring((2, 4), 6)
    C = ro.matmul(A, Y)
    assert C.shape == (3, 2)
    assert np.array_equal(C.T, ro.matmul(Y, A))  # (A Y^T)^T = Y A^T
    assert not np.array_equal(C, bf_matmul(A[:, ::-1].copy(), Y))


@pytest.mark.parametrize("shape,wshape,stride,pad", [
    ((1, 3, 3, 1), (1, 1, 1, 1), (1, 1), (0, 0)),
    ((2, 5, 4, 3), (2, 3, 3, 3), (1, 1), (1, 1)),
    ((1, 7, 6, 2), (3, 3, 2, 2), (2, 1), (0, 1)),
    ((1, 6, 6, 1), (2, 5, 5, 1), (2, 2), (2, 2)),
    ((2, 4, 5, 2), (1, 2, 3, 2), (1, 2), (1, 0)),
])
def test_conv_bigint_bruteforce(shape, wshape, stride, pad):
    X, W = ring(shape, 21 + sum(shape)), ring(wshape, 22 + sum(wshape))
    assert np.array_equal(ro.conv2d(X, W, stride, pad), bf_conv(X, W, stride, pad))


# ---------------------------------------------------------------- closed forms
def test_matmul_identity_right_operand():
    X = ring((6, 5), 31)
    assert np.array_equal(ro.matmul(X, np.eye(5, dtype=np.uint64)), X)


@pytest.mark.parametrize("K", [1, 7, 256, 1000])
def test_matmul_all_minus_one(K):
    A = np.full((3, K), MOD - 1, dtype=np.uint64)
    Y = np.full((2, K), MOD - 1, dtype=np.uint64)
    assert np.array_equal(ro.matmul(A, Y), np.full((3, 2), K, dtype=np.uint64))


def test_matmul_wraps_to_zero():
    A = np.full((2, 9), 1 << 32, dtype=np.uint64)
    assert not ro.matmul(A, A).any()                       # 2^32 * 2^32 = 2^64 = 0
    H = np.full((1, 1), 1 << 63, dtype=np.uint64)
    assert not ro.matmul(H, np.full((1, 1), 2, dtype=np.uint64)).any()   # 2^63 * 2 = 0
    assert ro.matmul(H, np.full((1, 1), 3, dtype=np.uint64))[0, 0] == 1 << 63


@pytest.mark.parametrize("word", wl.ADVERSARIAL_WORDS)
def test_matmul_constant_words(word):
    K = 37
    A = np.full((2, K), word, dtype=np.uint64)
    Y = np.full((3, K), word, dtype=np.uint64)
    expect = (K * word * word) % MOD
    assert np.array_equal(ro.matmul(A, Y), np.full((2, 3), expect, dtype=np.uint64))


def test_matmul_linearity():
    A, A2, Y = ring((4, 9), 41), ring((4, 9), 42), ring((5, 9), 43)
    alpha = np.uint64(0x9E3779B97F4A7C15)
    with np.errstate(over="ignore"):
        assert np.array_equal(ro.matmul(A * alpha, Y), ro.matmul(A, Y) * alpha)
        assert np.array_equal(ro.matmul(A + A2, Y), ro.matmul(A, Y) + ro.matmul(A2, Y))
        assert np.array_equal(ro.matmul(A, Y * alpha), ro.matmul(A, Y) * alpha)


# ---------------------------------------------------------------- convolution
def patch_matrix(X, kh, kw, stride, pad):
    """Explicit (B*Ho*Wo) x (kh*kw*Cin) patch matrix, zero padded, by numpy indexing."""
    B, H, Wd, C = X.shape
    sh, sw = stride
    ph, pw = pad
    Xp = np.zeros((B, H + 2 * ph, Wd + 2 * pw, C), dtype=np.uint64)
    Xp[:, ph:ph + H, pw:pw + Wd, :] = X
    Ho = (H + 2 * ph - kh) // sh + 1
    Wo = (Wd + 2 * pw - kw) // sw + 1
    rows = []
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                rows.append(Xp[b, ho * sh:ho * sh + kh, wo * sw:wo * sw + kw, :].reshape(-1))
    return np.stack(rows), (B, Ho, Wo)


@pytest.mark.parametrize("shape,wshape,stride,pad", [
    ((2, 9, 8, 3), (5, 3, 3, 3), (1, 1), (1, 1)),
    ((1, 12, 12, 4), (6, 5, 5, 4), (1, 1), (2, 2)),
    ((2, 11, 10, 3), (4, 7, 7, 3), (2, 2), (3, 3)),
    ((1, 32, 32, 3), (2, 11, 11, 3), (4, 4), (9, 9)),
    ((3, 8, 8, 16), (8, 1, 1, 16), (2, 2), (0, 0)),
])
def test_conv_equals_patch_matrix_times_weights(shape, wshape, stride, pad):
    X, W = ring(shape, 51 + sum(shape)), ring(wshape, 52 + sum(wshape))
    P, (B, Ho, Wo) = patch_matrix(X, wshape[1], wshape[2], stride, pad)
    Z = ro.matmul(P, W.reshape(wshape[0], -1)).reshape(B, Ho, Wo, wshape[0])
    assert np.array_equal(ro.conv2d(X, W, stride, pad), Z)


def test_conv_1x1_is_matmul():
    X, W = ring((2, 5, 6, 7), 61), ring((4, 1, 1, 7), 62)
    Z = ro.conv2d(X, W)
    assert np.array_equal(Z.reshape(-1, 4), ro.matmul(X.reshape(-1, 7), W.reshape(4, 7)))


def test_conv_delta_kernel_shifts_with_zero_border():
    X = ring((1, 6, 7, 1), 63)
    for r in range(3):
        for s in range(3):
            W = np.zeros((1, 3, 3, 1), dtype=np.uint64)
            W[0, r, s, 0] = 1
            Z = ro.conv2d(X, W, (1, 1), (1, 1))
            E = np.zeros_like(X)
            for ho in range(6):
                for wo in range(7):
                    hi, wi = ho - 1 + r, wo - 1 + s
                    if 0 <= hi < 6 and 0 <= wi < 7:
                        E[0, ho, wo, 0] = X[0, hi, wi, 0]
            assert np.array_equal(Z, E)


def test_conv_output_sizes_printed_in_the_paper():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "conv_output_dims.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for hw, k, pad, stride, out in (map(int, r) for r in rows):
        assert ro.conv_out_dim(hw, k, stride, pad) == out
        X, W = ring((1, hw, hw, 1), 64), ring((1, k, k, 1), 65)
        assert ro.conv2d(X, W, (stride, stride), (pad, pad)).shape == (1, out, out, 1)


# ---------------------------------------------------------------- sharing
def test_share_reconstruct_identity():
    edge = np.array([0, 1, 1 << 63, MOD - 1, 0x8080808080808080], dtype=np.uint64)
    x = np.concatenate([edge, ring((1000,), 71)])
    s = ro.share(x, ring(x.shape, 72), ring(x.shape, 73))
    assert np.array_equal(ro.reconstruct(*s), x)
    # python integers, independent of numpy wraparound
    for xs, a, b, c in zip(to_int(x), *map(to_int, s)):
        assert (a + b + c) % MOD == xs
    # the two random shares are the supplied randomness, the third is determined
    assert np.array_equal(s[0], ring(x.shape, 72)) and np.array_equal(s[1], ring(x.shape, 73))
    # replicated pairs: party i holds (s_i, s_{i+1})
    assert ro.party_pair(s, 2)[1] is s[0] and ro.party_pair(s, 0)[1] is s[1]


def test_linear_ops_on_shares():
    n = 257
    x, y = ring((n,), 81), ring((n,), 82)
    sx = ro.share(x, ring((n,), 83), ring((n,), 84))
    sy = ro.share(y, ring((n,), 85), ring((n,), 86))
    alpha, gamma = 0xDEADBEEFCAFEF00D, 0x0123456789ABCDEF
    add, mul, addc = [], [], []
    for i in range(3):
        xa, xb = ro.party_pair(sx, i)
        ya, yb = ro.party_pair(sy, i)
        add.append(ro.share_add(xa, xb, ya, yb))
        mul.append(ro.share_mul_public(xa, xb, alpha))
        addc.append(ro.share_add_public(xa, xb, gamma, i))
    for res, expect in ((add, [(a + b) % MOD for a, b in zip(to_int(x), to_int(y))]),
                        (mul, [(alpha * a) % MOD for a in to_int(x)]),
                        (addc, [(a + gamma) % MOD for a in to_int(x)])):
        # replicated consistency: party i's second component is party i+1's first
        for i in range(3):
            assert np.array_equal(res[i][1], res[(i + 1) % 3][0])
        rec = ro.reconstruct(res[0][0], res[1][0], res[2][0])
        assert to_int(rec) == expect
    # the public constant lands in share 0 only
    assert np.array_equal(addc[1][0], sx[1]) and np.array_equal(addc[2][0], sx[2])


# ---------------------------------------------------------------- party product
def bf_party(xi, xi1, yi, yi1):
    M, K = xi.shape
    N = yi.shape[0]
    a, a1, b, b1 = xi.tolist(), xi1.tolist(), yi.tolist(), yi1.tolist()
    return np.array([[sum(a[m][k] * b[n][k] + a1[m][k] * b[n][k] + a[m][k] * b1[n][k] for k in range(K)) % MOD
                      for n in range(N)] for m in range(M)], dtype=np.uint64)


def test_party_matmul_is_the_papers_three_terms():
    xi, xi1, yi, yi1 = ring((4, 6), 91), ring((4, 6), 92), ring((3, 6), 93), ring((3, 6), 94)
    z = ro.party_matmul(xi, xi1, yi, yi1)
    assert np.array_equal(z, bf_party(xi, xi1, yi, yi1))
    for m in range(4):
        for n in range(3):
            assert ro.party_matmul_at(xi, xi1, yi, yi1, m, n) == int(z[m, n])
    # x_{i+1} * y_{i+1} is NOT part of party i's sum
    with np.errstate(over="ignore"):
        assert not np.array_equal(z, ro.matmul(xi + xi1, yi + yi1))
        assert np.array_equal(z, ro.matmul(xi + xi1, yi + yi1) - ro.matmul(xi1, yi1))


@pytest.mark.parametrize("trans_x,trans_y", [(False, True), (True, False), (True, True)])
def test_party_matmul_on_transposed_storage(trans_x, trans_y):
    """party_matmul_t takes operands stored [K, rows]: pinned, on a non-square case, against the big-integer
    three-term formula applied to the operands transposed back by plain indexing (a wrong axis fails: M, N
    and K all differ)."""
    M, N, K = 5, 3, 7
    xi, xi1, yi, yi1 = ring((M, K), 95), ring((M, K), 96), ring((N, K), 97), ring((N, K), 98)
    want = bf_party(xi, xi1, yi, yi1)

    def stored(a, t):   # [rows, K] -> what the caller keeps in memory
        if not t:
            return a
        return np.array([[a[r, k] for r in range(a.shape[0])] for k in range(a.shape[1])], dtype=np.uint64)
    got = ro.party_matmul_t(stored(xi, trans_x), stored(xi1, trans_x), stored(yi, trans_y), stored(yi1, trans_y),
                            trans_x, trans_y)
    assert got.shape == (M, N) and np.array_equal(got, want)


@pytest.mark.parametrize("M,N,K", [(5, 4, 7), (16, 9, 33)])
def test_three_parties_sum_to_the_plaintext_product(M, N, K):
    x, y = ring((M, K), 101), ring((N, K), 102)
    sx = ro.share(x, ring((M, K), 103), ring((M, K), 104))
    sy = ro.share(y, ring((N, K), 105), ring((N, K), 106))
    z = [ro.party_matmul(*ro.party_pair(sx, i), *ro.party_pair(sy, i)) for i in range(3)]
    assert np.array_equal(ro.reconstruct(*z), ro.matmul(x, y))
    assert np.array_equal(ro.reconstruct(*z), bf_matmul(x, y))


def test_three_parties_sum_to_the_plaintext_conv():
    xs, ws, stride, pad = (2, 6, 5, 3), (4, 3, 3, 3), (2, 1), (1, 1)
    x, w = ring(xs, 111), ring(ws, 112)
    sx = ro.share(x, ring(xs, 113), ring(xs, 114))
    sw = ro.share(w, ring(ws, 115), ring(ws, 116))
    z = [ro.party_conv2d(*ro.party_pair(sx, i), *ro.party_pair(sw, i), stride, pad) for i in range(3)]
    assert np.array_equal(ro.reconstruct(*z), bf_conv(x, w, stride, pad))
    zi = z[1]
    xa, xb = ro.party_pair(sx, 1)
    wa, wb = ro.party_pair(sw, 1)
    with np.errstate(over="ignore"):
        three = bf_conv(xa, wa, stride, pad) + bf_conv(xb, wa, stride, pad) + bf_conv(xa, wb, stride, pad)
    assert np.array_equal(zi, three)
    for idx in [(0, 0, 0, 0), (1, 2, 4, 3), (0, 1, 2, 1)]:
        assert ro.party_conv2d_at(xa, xb, wa, wb, *idx, stride, pad) == int(zi[idx])


# ---------------------------------------------------------------- fixed point
def test_encode_known_values():
    t = 16
    vals = np.array([0.0, 1.0, -1.0, 0.5, 2.0 ** -16, -(2.0 ** -16), 0.5 * 2.0 ** -16, 1.5 * 2.0 ** -16,
                     2.5 * 2.0 ** -16, 3.25, -3.25])
    enc = to_int(ro.encode(vals, t))
    assert enc == [0, 65536, MOD - 65536, 32768, 1, MOD - 1, 0, 2, 2, 212992, MOD - 212992]
    assert np.array_equal(ro.decode(ro.encode(vals[:6], t), t), vals[:6])
    assert to_int(ro.encode(np.array([1.0]), 20)) == [1 << 20]


@pytest.mark.parametrize("cfg,layer_idx", [(1, 0), (2, 0), (2, 2)])
def test_fixed_point_product_decodes_to_the_real_product(cfg, layer_idx):
    """Secret-shared fixed-point matmul, decoded at scale 2^(2t), against the fp64
    product of the operands on the 2^-t grid: within 2^-12 absolute."""
    L = wl.config_layers(cfg)[layer_idx]
    seed = wl.layer_seed(cfg, layer_idx)
    t = wl.FRAC_BITS
    X = wl.draw_reals(L.x_shape, L.x_dist, seed)
    Y = wl.draw_reals(L.w_shape, L.w_dist, seed + 1)
    ex, ey = ro.encode(X, t), ro.encode(Y, t)
    Xg, Yg = ro.decode(ex, t), ro.decode(ey, t)
    assert np.max(np.abs(Xg - X)) <= 2.0 ** -(t + 1) and np.max(np.abs(Yg - Y)) <= 2.0 ** -(t + 1)
    sx = ro.share(ex, wl.draw_ring(ex.shape, seed + 2), wl.draw_ring(ex.shape, seed + 3))
    sy = ro.share(ey, wl.draw_ring(ey.shape, seed + 4), wl.draw_ring(ey.shape, seed + 5))
    z = [ro.party_matmul(*ro.party_pair(sx, i), *ro.party_pair(sy, i)) for i in range(3)]
    got = ro.decode(ro.reconstruct(*z), 2 * t)
    assert np.max(np.abs(got - Xg @ Yg.T)) <= 2.0 ** -12
    # against the un-rounded reals the error is bounded by the encoding error
    kmax = L.K * (np.max(np.abs(X)) + np.max(np.abs(Y))) * 2.0 ** -(t + 1) + L.K * 2.0 ** -(2 * t + 2)
    assert np.max(np.abs(got - X @ Y.T)) <= kmax


# ---------------------------------------------------------------- element-wise product, pooling
def test_party_mul_is_the_three_term_scalar_protocol():
    n = 23
    xi, xi1, yi, yi1 = ring((n,), 201), ring((n,), 202), ring((n,), 203), ring((n,), 204)
    z = ro.party_mul(xi, xi1, yi, yi1)
    for j in range(n):
        a, a1, b, b1 = int(xi[j]), int(xi1[j]), int(yi[j]), int(yi1[j])
        assert int(z[j]) == (a * b + a1 * b + a * b1) % MOD
    # the diagonal of the outer-product matmul with K = 1 is the element-wise product
    full = ro.party_matmul(xi.reshape(n, 1), xi1.reshape(n, 1), yi.reshape(n, 1), yi1.reshape(n, 1))
    assert np.array_equal(np.diagonal(full), z)


def test_party_mul_broadcast_and_three_party_sum():
    shape, C = (2, 3, 4, 6), 6
    x, a = ring(shape, 211), ring((C,), 212)
    sx = ro.share(x, ring(shape, 213), ring(shape, 214))
    sa = ro.share(a, ring((C,), 215), ring((C,), 216))
    z = [ro.party_mul(*ro.party_pair(sx, i), *ro.party_pair(sa, i)) for i in range(3)]
    opened = ro.reconstruct(*z)
    xs, as_ = x.tolist(), a.tolist()
    for idx in np.ndindex(*shape):
        assert int(opened[idx]) == (int(x[idx]) * as_[idx[-1]]) % MOD


def bf_sum_pool(X, window, stride, pad):
    B, H, Wd, C = X.shape
    kh, kw = window
    Ho = (H + 2 * pad[0] - kh) // stride[0] + 1
    Wo = (Wd + 2 * pad[1] - kw) // stride[1] + 1
    x = X.tolist()
    Z = np.zeros((B, Ho, Wo, C), dtype=np.uint64)
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for c in range(C):
                    acc = 0
                    for r in range(kh):
                        for s in range(kw):
                            hi, wi = ho * stride[0] - pad[0] + r, wo * stride[1] - pad[1] + s
                            if 0 <= hi < H and 0 <= wi < Wd:
                                acc += x[b][hi][wi][c]
                    Z[b, ho, wo, c] = acc % MOD
    return Z


@pytest.mark.parametrize("shape,window,stride,pad", [
    ((1, 4, 4, 1), (2, 2), (2, 2), (0, 0)), ((2, 7, 6, 3), (3, 3), (2, 2), (1, 1)),
    ((1, 10, 10, 2), (3, 3), (2, 2), (0, 0)), ((2, 5, 4, 5), (2, 3), (1, 2), (0, 1)),
])
def test_sum_pool_bruteforce(shape, window, stride, pad):
    X = ring(shape, 221 + sum(shape))
    assert np.array_equal(ro.sum_pool2d(X, window, stride, pad), bf_sum_pool(X, window, stride, pad))


def test_sum_pool_closed_forms_and_paper_sizes():
    X = ring((2, 6, 6, 3), 231)
    assert np.array_equal(ro.sum_pool2d(X, (1, 1), (1, 1)), X)                  # 1x1 window: identity
    whole = ro.sum_pool2d(X, (6, 6), (6, 6))
    for b in range(2):
        for c in range(3):
            assert int(whole[b, 0, 0, c]) == sum(int(v) for v in X[b, :, :, c].reshape(-1)) % MOD
    # pooling is the convolution with a per-channel all-ones kernel
    W = np.zeros((3, 2, 2, 3), dtype=np.uint64)
    for c in range(3):
        W[c, :, :, c] = 1
    assert np.array_equal(ro.sum_pool2d(X, (2, 2), (2, 2)), ro.conv2d(X, W, (2, 2), (0, 0)))
    # sizes printed in the paper's AlexNet / VGG tables: 10x10 with 3x3/2 -> 4x4; 32x32 with 2x2/2 -> 16x16
    assert ro.sum_pool2d(ring((1, 10, 10, 1), 232), (3, 3), (2, 2)).shape == (1, 4, 4, 1)
    assert ro.sum_pool2d(ring((1, 32, 32, 1), 233), (2, 2), (2, 2)).shape == (1, 16, 16, 1)
    # linear, hence local on shares: pooling the shares and opening = pooling the secret
    s = ro.share(X, ring(X.shape, 234), ring(X.shape, 235))
    pooled = [ro.sum_pool2d(v, (3, 3), (2, 2), (1, 1)) for v in s]
    assert np.array_equal(ro.reconstruct(*pooled), ro.sum_pool2d(X, (3, 3), (2, 2), (1, 1)))


# ---------------------------------------------------------------- bias of a linear layer
def test_bias_add_and_its_gradient():
    rows, cols = 37, 11
    x, b = ring((rows, cols), 501), ring((cols,), 502)
    sx = ro.share(x, ring(x.shape, 503), ring(x.shape, 504))
    sb = ro.share(b, ring(b.shape, 505), ring(b.shape, 506))
    outs = [ro.share_bias_add(*ro.party_pair(sx, i), *ro.party_pair(sb, i)) for i in range(3)]
    # party i's first component is share i: the three open to x + b, row by row, in Python integers
    opened = ro.reconstruct(outs[0][0], outs[1][0], outs[2][0])
    want = [[(int(x[r, c]) + int(b[c])) % MOD for c in range(cols)] for r in range(rows)]
    assert opened.tolist() == want
    # replicated form is kept: party i's second component is party i+1's first
    for i in range(3):
        assert np.array_equal(outs[i][1], outs[(i + 1) % 3][0])
    sums = [ro.share_col_sum(*ro.party_pair(sx, i)) for i in range(3)]
    opened = ro.reconstruct(sums[0][0], sums[1][0], sums[2][0])
    assert opened.tolist() == [sum(int(x[r, c]) for r in range(rows)) % MOD for c in range(cols)]
    # on a 4-d tensor the leading dimensions are all rows
    x4 = ring((2, 3, 4, 5), 507)
    za, _ = ro.share_col_sum(x4, x4)
    assert za.tolist() == [sum(int(v) for v in x4[..., c].reshape(-1)) % MOD for c in range(5)]
    # adjoint pair: <x + 1 b^T, g> - <x, g> = <b, colsum(g)>
    g = ring((rows, cols), 508)
    za, _ = ro.share_bias_add(x, x, b, b)
    ga, _ = ro.share_col_sum(g, g)
    dot = lambda u, v: sum(int(p) * int(q) for p, q in zip(u.reshape(-1).tolist(), v.reshape(-1).tolist())) % MOD
    assert (dot(za, g) - dot(x, g)) % MOD == dot(b, ga)
