"""Softmax on shares, assembled from the library's local steps as the paper's training section describes it
(Sec. III-C): maximum by a tree of comparisons (sign bit of differences), exponential by the limit form
(1 + x/m)^m with m a power of two (repeated squaring), reciprocal by Newton-Raphson from the fixed start 1/Y.
Every party's local step runs on the GPU through the C-ABI; messages are device-to-device assignments."""
import numpy as np
import pytest

from tests.gpu_util import gpu_mul_trunc, gpu_relu, gpu_trunc, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KEYS = (bytes(range(16)), bytes(range(16, 32)), bytes(range(32, 48)))
T = 16           # fractional bits
LOG_M = 8        # m = 256 in (1 + x/m)^m
NEWTON = 7       # iterations for 1/y, y in [1, 10]


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import ring_oracle as ro
    from paper_2104_10949_amd import binding as cg
    from paper_2104_10949_amd import workloads as wl
    cg.lib()
    return cg, ro, wl


def float_model(x):
    """The same approximations in float64, without shares or fixed point."""
    y = x - x.max(axis=1, keepdims=True)
    e = (1 + y / 2 ** LOG_M) ** (2 ** LOG_M)
    s = e.sum(axis=1, keepdims=True)
    z = np.full_like(s, 1 / x.shape[1])
    for _ in range(NEWTON):
        z = 2 * z - s * z * z
    return e * z


def test_softmax_on_shares(env):
    cg, ro, wl = env
    batch, d = 64, 10
    rng = np.random.default_rng(5)
    x_real = np.rint(rng.normal(0, 2, size=(batch, d)) * 2 ** T) / 2 ** T
    enc = ro.encode(x_real, T)
    X = tuple(cg.to_device(s) for s in ro.share(enc, wl.draw_ring(enc.shape, 1), wl.draw_ring(enc.shape, 2)))
    nonce = [5000]

    def fresh():
        nonce[0] += 4
        return nonce[0]

    sub = lambda U, V: tuple(u - v for u, v in zip(U, V))        # linear combinations of shares are local
    add = lambda U, V: tuple(u + v for u, v in zip(U, V))
    const = lambda c, like: tuple(torch.full_like(like, int(round(c * 2 ** T))) if k == 0 else torch.zeros_like(like)
                                  for k in range(3))             # a public constant lives in share 0

    say("softmax: maximum by a comparison tree")
    cols = [tuple(s[:, j].contiguous() for s in X) for j in range(d)]
    while len(cols) > 1:
        nxt = []
        for a, b in zip(cols[0::2], cols[1::2]):
            nxt.append(add(b, gpu_relu(cg, sub(a, b), KEYS, fresh())))        # max(a, b) = b + relu(a - b)
        if len(cols) % 2:
            nxt.append(cols[-1])
        cols = nxt
    mx = cols[0]
    opened_max = cg.to_host(cg.cg_reconstruct(*mx)).astype(np.int64)
    assert np.array_equal(opened_max, enc.astype(np.int64).max(axis=1))      # comparisons are exact

    say("softmax: exponential by repeated squaring")
    Y = tuple((x - m[:, None]).contiguous() for x, m in zip(X, mx))
    U = add(const(1.0, Y[0]), gpu_trunc(cg, Y, KEYS, fresh(), LOG_M))        # 1 + y / m
    for _ in range(LOG_M):
        U = gpu_mul_trunc(cg, U, U, KEYS, fresh(), T)
    say("softmax: reciprocal of the row sums by Newton-Raphson")
    S = tuple(u.sum(dim=1, keepdim=True).contiguous() for u in U)            # sums of shares are local
    Z = const(1.0 / d, S[0])
    for _ in range(NEWTON):
        Z2 = gpu_mul_trunc(cg, Z, Z, KEYS, fresh(), T)
        SZ2 = gpu_mul_trunc(cg, S, Z2, KEYS, fresh(), T)
        Z = sub(add(Z, Z), SZ2)
    say("softmax: quotient")
    Zb = tuple(z.expand(-1, d).contiguous() for z in Z)
    P = gpu_mul_trunc(cg, U, Zb, KEYS, fresh(), T)
    torch.cuda.synchronize()
    got = cg.to_host(cg.cg_reconstruct(*P)).astype(np.int64) / 2 ** T
    model = float_model(x_real)
    e = np.exp(x_real - x_real.max(axis=1, keepdims=True))
    exact = e / e.sum(axis=1, keepdims=True)
    assert np.max(np.abs(got - model)) < 5e-3          # shares and fixed point against the same approximations
    assert np.max(np.abs(got - exact)) < 3e-2          # the approximations themselves
    assert np.all(np.abs(got.sum(axis=1) - 1) < 2e-2)
    assert np.array_equal(np.argmax(got, axis=1), np.argmax(exact, axis=1))
