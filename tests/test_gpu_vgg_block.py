"""A VGG-style block evaluated with every value on shares: two 3x3 convolutions, each followed by the truncation
protocol and ReLU (sign-bit circuit + share products), then 2x2 max pooling as a tree of comparisons
(max(a, b) = b + ReLU(a - b)).  Every party's local step runs on the GPU through the C-ABI; messages are
device-to-device assignments.  Only the pooled output is opened; it must match a float64 evaluation of the same
grid-rounded parameters."""
import numpy as np
import pytest

from tests.gpu_util import gpu_relu, gpu_trunc, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KEYS = (bytes(range(16)), bytes(range(16, 32)), bytes(range(32, 48)))
T = 16


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import ring_oracle as ro
    from paper_2104_10949_amd import binding as cg
    from paper_2104_10949_amd import workloads as wl
    cg.lib()
    return cg, ro, wl


def test_conv_relu_conv_relu_maxpool_on_shares(env):
    cg, ro, wl = env
    rng = np.random.default_rng(31)
    grid = lambda a: np.rint(a * 2 ** T) / 2 ** T
    B, H, W, C0, C1 = 2, 16, 16, 3, 64
    seed = [500]

    def share_dev(real):
        enc = ro.encode(real, T)
        seed[0] += 2
        return tuple(cg.to_device(s) for s in ro.share(enc, wl.draw_ring(enc.shape, seed[0]), wl.draw_ring(enc.shape, seed[0] + 1)))

    nonce = [20000]

    def fresh():
        nonce[0] += 4
        return nonce[0]

    x_real = grid(rng.uniform(0, 1, size=(B, H, W, C0)))
    w_real = [grid(rng.normal(0, 0.2, size=(C1, 3, 3, C0))), grid(rng.normal(0, 0.05, size=(C1, 3, 3, C1)))]
    b_real = [grid(rng.normal(0, 0.1, size=(C1,))) for _ in range(2)]
    act = share_dev(x_real)
    Wt = [share_dev(w) for w in w_real]
    Bs = [share_dev(b) for b in b_real]

    for l in range(2):
        say(f"VGG block on shares: convolution {l}, truncation, ReLU")
        z = []
        for i in range(3):
            zi = cg.cg_share_conv2d(act[i], act[(i + 1) % 3], Wt[l][i], Wt[l][(i + 1) % 3], stride=(1, 1), pad=(1, 1))
            bi = Bs[l][i] << T
            zi, _ = cg.cg_share_bias_add(zi, zi, bi, bi)
            z.append(zi)
        act = gpu_relu(cg, gpu_trunc(cg, tuple(z), KEYS, fresh(), T), KEYS, fresh())

    say("VGG block on shares: 2x2 max pooling by comparisons")
    corner = lambda dh, dw: tuple(s[:, dh::2, dw::2, :].contiguous() for s in act)
    sub = lambda U, V: tuple(u - v for u, v in zip(U, V))
    add = lambda U, V: tuple(u + v for u, v in zip(U, V))
    smax = lambda U, V: add(V, gpu_relu(cg, sub(U, V), KEYS, fresh()))
    pooled = smax(smax(corner(0, 0), corner(0, 1)), smax(corner(1, 0), corner(1, 1)))
    torch.cuda.synchronize()
    got = cg.to_host(cg.cg_reconstruct(*pooled)).astype(np.int64) / 2 ** T

    a = torch.from_numpy(x_real).permute(0, 3, 1, 2)
    for l in range(2):
        wt = torch.from_numpy(w_real[l]).permute(0, 3, 1, 2)
        a = torch.relu(torch.nn.functional.conv2d(a, wt, torch.from_numpy(b_real[l]), padding=1))
    want = torch.nn.functional.max_pool2d(a, 2).permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape == (B, H // 2, W // 2, C1)
    assert np.max(np.abs(got - want)) < 2e-3
    assert np.mean(want > 0) > 0.3            # the comparison has something to say
