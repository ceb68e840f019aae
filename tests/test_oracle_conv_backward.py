"""Pins for the oracle's convolution backward products (no GPU).

The two gradients are pinned to things other than themselves: the exact adjoint identity
over Z_{2^64} against the forward convolution (itself pinned by big-integer brute force),
the textbook "correlate the incoming gradient with the flipped, transposed filter" form
built from the pinned forward routine, a patch-matrix form built with numpy indexing,
big-integer brute force on tiny inputs, and a library autograd (float64 on small integers,
where every sum is exact).
"""
import numpy as np
import pytest
import torch

from oracle import ring_oracle as ro
from paper_2104_10949_amd import workloads as wl
from test_oracle_pins import MOD, bf_conv, patch_matrix

CASES = [
    # x shape (B,H,W,Cin), w shape (Cout,kh,kw,Cin), stride, pad
    ((2, 6, 5, 3), (4, 3, 3, 3), (1, 1), (1, 1)),
    ((1, 7, 7, 2), (3, 3, 3, 2), (1, 1), (0, 0)),
    ((2, 8, 6, 4), (5, 5, 3, 4), (1, 1), (2, 1)),
    ((2, 9, 8, 3), (2, 3, 3, 3), (2, 2), (1, 1)),
    ((1, 11, 10, 2), (3, 7, 7, 2), (2, 2), (3, 3)),
    ((1, 12, 12, 1), (2, 4, 4, 1), (4, 4), (0, 0)),
    ((3, 5, 5, 6), (7, 1, 1, 6), (1, 1), (0, 0)),
    ((2, 6, 7, 2), (3, 2, 3, 2), (1, 2), (1, 0)),
]


def ring(shape, seed):
    return wl.draw_ring(shape, seed)


def dot(a, b) -> int:
    """Inner product over the ring with Python integers."""
    return sum(int(u) * int(v) for u, v in zip(a.reshape(-1).tolist(), b.reshape(-1).tolist())) % MOD


def g_shape(xs, ws, stride, pad):
    Ho = (xs[1] + 2 * pad[0] - ws[1]) // stride[0] + 1
    Wo = (xs[2] + 2 * pad[1] - ws[2]) // stride[1] + 1
    return (xs[0], Ho, Wo, ws[0])


@pytest.mark.parametrize("xs,ws,stride,pad", CASES)
def test_gradients_are_the_adjoints_of_the_forward_map(xs, ws, stride, pad):
    # <conv(X, W), G> = <X, dgrad(G, W)> = <W, wgrad(G, X)> holds exactly mod 2^64
    X, W, G = ring(xs, 1), ring(ws, 2), ring(g_shape(xs, ws, stride, pad), 3)
    lhs = dot(ro.conv2d(X, W, stride, pad), G)
    assert dot(X, ro.conv2d_dgrad(G, W, xs, stride, pad)) == lhs
    assert dot(W, ro.conv2d_wgrad(G, X, ws, stride, pad)) == lhs


@pytest.mark.parametrize("xs,ws,stride,pad", CASES[:4])
def test_adjoint_identity_pins_every_entry(xs, ws, stride, pad):
    # pairing with unit tensors reads single entries: DX[j] = <conv(e_j, W), G>, DW[j] = <conv(X, e_j), G>
    X, W, G = ring(xs, 4), ring(ws, 5), ring(g_shape(xs, ws, stride, pad), 6)
    DX, DW = ro.conv2d_dgrad(G, W, xs, stride, pad), ro.conv2d_wgrad(G, X, ws, stride, pad)
    rng = np.random.default_rng(7)
    for _ in range(12):
        j = tuple(int(rng.integers(0, n)) for n in xs)
        E = np.zeros(xs, dtype=np.uint64)
        E[j] = 1
        assert int(DX[j]) == dot(bf_conv(E, W, stride, pad), G)
        j = tuple(int(rng.integers(0, n)) for n in ws)
        E = np.zeros(ws, dtype=np.uint64)
        E[j] = 1
        assert int(DW[j]) == dot(bf_conv(X, E, stride, pad), G)


@pytest.mark.parametrize("xs,ws,stride,pad", [c for c in CASES if c[2] == (1, 1)])
def test_stride1_dgrad_is_a_correlation_with_the_flipped_transposed_filter(xs, ws, stride, pad):
    W, G = ring(ws, 8), ring(g_shape(xs, ws, stride, pad), 9)
    Wt = np.ascontiguousarray(W[:, ::-1, ::-1, :].transpose(3, 1, 2, 0))   # [Cin, kh, kw, Cout], taps reversed
    full = (ws[1] - 1 - pad[0], ws[2] - 1 - pad[1])
    assert np.array_equal(ro.conv2d_dgrad(G, W, xs, stride, pad), ro.conv2d(G, Wt, (1, 1), full))


@pytest.mark.parametrize("xs,ws,stride,pad", CASES)
def test_wgrad_is_gradient_transposed_times_patch_matrix(xs, ws, stride, pad):
    X, G = ring(xs, 10), ring(g_shape(xs, ws, stride, pad), 11)
    P, _ = patch_matrix(X, ws[1], ws[2], stride, pad)             # [pixels, kh*kw*Cin]
    Gt = np.ascontiguousarray(G.reshape(-1, ws[0]).T)             # [Cout, pixels]
    DW = ro.matmul(Gt, np.ascontiguousarray(P.T)).reshape(ws)     # right operand of matmul is [N, K]
    assert np.array_equal(ro.conv2d_wgrad(G, X, ws, stride, pad), DW)


@pytest.mark.parametrize("xs,ws,stride,pad", CASES)
def test_against_library_autograd_on_small_integers(xs, ws, stride, pad):
    rng = np.random.default_rng(12)
    X = rng.integers(-8, 9, size=xs)
    W = rng.integers(-8, 9, size=ws)
    G = rng.integers(-8, 9, size=g_shape(xs, ws, stride, pad))
    xt = torch.tensor(X.transpose(0, 3, 1, 2), dtype=torch.float64, requires_grad=True)   # NCHW
    wt = torch.tensor(W.transpose(0, 3, 1, 2), dtype=torch.float64, requires_grad=True)   # [Cout,Cin,kh,kw]
    z = torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad)
    z.backward(torch.tensor(G.transpose(0, 3, 1, 2), dtype=torch.float64))
    want_dx = xt.grad.numpy().transpose(0, 2, 3, 1).astype(np.int64).astype(np.uint64)
    want_dw = wt.grad.numpy().transpose(0, 2, 3, 1).astype(np.int64).astype(np.uint64)
    u = lambda a: a.astype(np.int64).astype(np.uint64)
    assert np.array_equal(ro.conv2d_dgrad(u(G), u(W), xs, stride, pad), want_dx)
    assert np.array_equal(ro.conv2d_wgrad(u(G), u(X), ws, stride, pad), want_dw)


def test_party_gradients_are_three_terms_and_sum_to_the_plaintext_gradients():
    xs, ws, stride, pad = (2, 6, 5, 3), (4, 3, 3, 3), (2, 1), (1, 1)
    gs = g_shape(xs, ws, stride, pad)
    x, w, g = ring(xs, 20), ring(ws, 21), ring(gs, 22)
    sx = ro.share(x, ring(xs, 23), ring(xs, 24))
    sw = ro.share(w, ring(ws, 25), ring(ws, 26))
    sg = ro.share(g, ring(gs, 27), ring(gs, 28))
    dx = [ro.party_conv2d_dgrad(*ro.party_pair(sg, i), *ro.party_pair(sw, i), xs, stride, pad) for i in range(3)]
    dw = [ro.party_conv2d_wgrad(*ro.party_pair(sg, i), *ro.party_pair(sx, i), ws, stride, pad) for i in range(3)]
    assert np.array_equal(ro.reconstruct(*dx), ro.conv2d_dgrad(g, w, xs, stride, pad))
    assert np.array_equal(ro.reconstruct(*dw), ro.conv2d_wgrad(g, x, ws, stride, pad))
    ga, gb = ro.party_pair(sg, 2)
    wa, wb = ro.party_pair(sw, 2)
    xa, xb = ro.party_pair(sx, 2)
    with np.errstate(over="ignore"):
        three_dx = (ro.conv2d_dgrad(ga, wa, xs, stride, pad) + ro.conv2d_dgrad(gb, wa, xs, stride, pad) +
                    ro.conv2d_dgrad(ga, wb, xs, stride, pad))
        three_dw = (ro.conv2d_wgrad(ga, xa, ws, stride, pad) + ro.conv2d_wgrad(gb, xa, ws, stride, pad) +
                    ro.conv2d_wgrad(ga, xb, ws, stride, pad))
    assert np.array_equal(dx[2], three_dx)
    assert np.array_equal(dw[2], three_dw)
