"""One stochastic-gradient step of a fully connected classifier with every value on shares (the private-training
pipeline of Sec. III-C assembled from the library's local steps): forward products with bias and truncation, ReLU
from the sign-bit circuit, softmax, cross-entropy gradient, backward products with transposed operands, bias
gradients by column sums, and the update with the learning rate folded into the truncation.  Every party's local
step runs on the GPU through the C-ABI; messages are device-to-device assignments.  Only test code opens values:
the updated parameters are compared with a float64 step on the same grid-rounded parameters."""
import numpy as np
import pytest

from tests.gpu_util import gpu_relu, gpu_share_mult, gpu_softmax, gpu_trunc, say, softmax_float_model

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KEYS = (bytes(range(16)), bytes(range(16, 32)), bytes(range(32, 48)))
T = 16            # fractional bits
LOG_M = 8
NEWTON = 7
LOG_LR = 1        # learning rate 2^-LOG_LR on the batch-mean gradient
DIMS = (784, 128, 128, 10)
BATCH = 64        # a power of two, so that the mean folds into the truncation


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import ring_oracle as ro
    from paper_2104_10949_amd import binding as cg
    from paper_2104_10949_amd import workloads as wl
    cg.lib()
    return cg, ro, wl


def test_one_sgd_step_on_shares(env):
    cg, ro, wl = env
    rng = np.random.default_rng(77)
    grid = lambda a: np.rint(a * 2 ** T) / 2 ** T
    seed = [100]

    def share_dev(real):
        enc = ro.encode(real, T)
        seed[0] += 2
        return tuple(cg.to_device(s) for s in ro.share(enc, wl.draw_ring(enc.shape, seed[0]), wl.draw_ring(enc.shape, seed[0] + 1)))

    nonce = [9000]

    def fresh():
        nonce[0] += 4
        return nonce[0]

    def product(L, R, trans_l, trans_r):
        """The three parties' additive results of L R^T on replicated sharings (operands possibly stored transposed)."""
        return tuple(cg.cg_share_matmul_t(L[i], L[(i + 1) % 3], R[i], R[(i + 1) % 3], trans_l, trans_r) for i in range(3))

    opened = lambda S: cg.to_host(cg.cg_reconstruct(*S)).astype(np.int64)

    x_real = grid(rng.uniform(0, 1, size=(BATCH, DIMS[0])))
    labels = rng.integers(0, DIMS[-1], size=BATCH)
    y_real = np.eye(DIMS[-1])[labels]
    W_real = [grid(rng.normal(0, 0.05, size=(DIMS[l + 1], DIMS[l]))) for l in range(3)]
    b_real = [grid(rng.normal(0, 0.1, size=(DIMS[l + 1],))) for l in range(3)]
    X, Y = share_dev(x_real), share_dev(y_real)
    W = [share_dev(w) for w in W_real]
    B = [share_dev(b) for b in b_real]

    # forward
    acts, masks = [X], []
    for l in range(3):
        say(f"training step: forward layer {l}")
        z = []
        for i in range(3):
            zi = cg.cg_share_matmul(acts[l][i], acts[l][(i + 1) % 3], W[l][i], W[l][(i + 1) % 3])
            bi = B[l][i] << T                                   # bias joins at the product's scale: a public shift
            zi, _ = cg.cg_share_bias_add(zi, zi, bi, bi)
            z.append(zi)
        pre = gpu_trunc(cg, tuple(z), KEYS, fresh(), T)
        if l < 2:
            a, keep = gpu_relu(cg, pre, KEYS, fresh(), with_mask=True)
            acts.append(a)
            masks.append(keep)
    say("training step: softmax")
    P, _ = gpu_softmax(cg, pre, KEYS, fresh, T, LOG_M, NEWTON)

    # backward and update; dz holds the gradient of the batch SUM, the mean and the rate go into the shift
    shift = int(np.log2(BATCH)) + LOG_LR
    dz = tuple(p - y for p, y in zip(P, Y))
    new_W, new_B = [None] * 3, [None] * 3
    for l in (2, 1, 0):
        say(f"training step: backward layer {l}")
        dW = gpu_trunc(cg, product(dz, acts[l], True, True), KEYS, fresh(), T + shift)
        db = []
        for i in range(3):
            s, _ = cg.cg_share_col_sum(dz[i], dz[i])
            db.append(s)
        db = gpu_trunc(cg, tuple(db), KEYS, fresh(), shift)
        new_W[l] = tuple(w - g for w, g in zip(W[l], dW))
        new_B[l] = tuple(b - g for b, g in zip(B[l], db))
        if l:
            da = gpu_trunc(cg, product(dz, W[l], False, True), KEYS, fresh(), T)
            dz = gpu_share_mult(cg, da, masks[l - 1], KEYS, fresh(), 0)      # 0 / 1 integers: no rescaling
    torch.cuda.synchronize()

    # float64 step with the same approximations of softmax and the ReLU pattern the shares produced
    mask_open = [opened(m) for m in masks]
    a_f, pre_f = [x_real], None
    for l in range(3):
        pre_f = a_f[l] @ W_real[l].T + b_real[l]
        if l < 2:
            assert set(np.unique(mask_open[l])) <= {0, 1}
            assert np.mean(mask_open[l] != (pre_f >= 0)) < 2e-3          # signs differ only next to zero
            a_f.append(pre_f * mask_open[l])
    p_f = softmax_float_model(pre_f, LOG_M, NEWTON)
    assert np.max(np.abs(opened(P) / 2 ** T - p_f)) < 1e-2
    dz_f = p_f - y_real
    lr = 2.0 ** -shift
    for l in (2, 1, 0):
        gW, gb = dz_f.T @ a_f[l], dz_f.sum(axis=0)
        got_W, got_b = opened(new_W[l]) / 2 ** T, opened(new_B[l]) / 2 ** T
        step_W, step_b = got_W - W_real[l], got_b - b_real[l]
        say(f"layer {l}: max update error W {np.max(np.abs(step_W + lr * gW)):.2e} b {np.max(np.abs(step_b + lr * gb)):.2e} "
            f"relative {np.linalg.norm(step_W + lr * gW) / np.linalg.norm(lr * gW):.2e}")
        assert np.max(np.abs(step_W + lr * gW)) < 2e-4, l          # a few units of 2^-16
        assert np.max(np.abs(step_b + lr * gb)) < 2e-4, l
        assert np.linalg.norm(step_W + lr * gW) < 0.06 * np.linalg.norm(lr * gW), l   # first layer's updates are near the grid step
        if l:
            dz_f = (dz_f @ W_real[l]) * mask_open[l - 1]

    # the step lowers the exact cross-entropy of the batch
    def loss(Ws, bs):
        a = x_real
        for l in range(3):
            a = a @ Ws[l].T + bs[l]
            if l < 2:
                a = np.maximum(a, 0)
        a = a - a.max(axis=1, keepdims=True)
        return float(np.mean(np.log(np.exp(a).sum(axis=1)) - a[np.arange(BATCH), labels]))

    before = loss(W_real, b_real)
    after = loss([opened(w) / 2 ** T for w in new_W], [opened(b) / 2 ** T for b in new_B])
    assert after < before - 1e-3, (before, after)
