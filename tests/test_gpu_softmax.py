"""Softmax on shares, assembled from the library's local steps as the paper's training section describes it
(Sec. III-C): maximum by a tree of comparisons (sign bit of differences), exponential by the limit form
(1 + x/m)^m with m a power of two (repeated squaring), reciprocal by Newton-Raphson from the fixed start 1/Y.
Every party's local step runs on the GPU through the C-ABI; messages are device-to-device assignments."""
import numpy as np
import pytest

from tests.gpu_util import gpu_softmax, say, softmax_float_model

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

    say("softmax on shares: comparison tree, repeated squaring, Newton-Raphson")
    P, mx = gpu_softmax(cg, X, KEYS, fresh, T, LOG_M, NEWTON)
    opened_max = cg.to_host(cg.cg_reconstruct(*mx)).astype(np.int64)
    assert np.array_equal(opened_max, enc.astype(np.int64).max(axis=1))      # comparisons are exact
    torch.cuda.synchronize()
    got = cg.to_host(cg.cg_reconstruct(*P)).astype(np.int64) / 2 ** T
    model = softmax_float_model(x_real, LOG_M, NEWTON)
    e = np.exp(x_real - x_real.max(axis=1, keepdims=True))
    exact = e / e.sum(axis=1, keepdims=True)
    assert np.max(np.abs(got - model)) < 5e-3          # shares and fixed point against the same approximations
    assert np.max(np.abs(got - exact)) < 3e-2          # the approximations themselves
    assert np.all(np.abs(got.sum(axis=1) - 1) < 2e-2)
    assert np.array_equal(np.argmax(got, axis=1), np.argmax(exact, axis=1))
