"""Seeded sweep of random shapes through every product entry point against the CPU oracle, bit for bit.
The shapes mix round numbers with their neighbours (31, 32, 33, ...), so that tile tails, K tails, split
launches, the streamed distributions, strided gradients and every address generator come up without being
listed one by one."""
import numpy as np
import pytest

from tests.gpu_util import first_mismatch, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SPECIAL = (1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 192, 255, 256, 257, 512)
BUDGET = 4e8        # ring MACs per case: the oracle takes a fraction of a second


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import ring_oracle as ro
    from paper_2104_10949_amd import binding as cg
    cg.lib()
    return cg, ro


def dim(rng, hi, specials=SPECIAL):
    if rng.random() < 0.5:
        return int(rng.choice([s for s in specials if s <= hi]))
    return int(rng.integers(1, hi + 1))


def words(rng, shape):
    if rng.integers(0, 4) == 0:      # every digit at an extreme
        return np.full(shape, [0xFFFFFFFFFFFFFFFF, 0x8080808080808080, 0x7F7F7F7F7F7F7F7F][int(rng.integers(0, 3))],
                       dtype=np.uint64)
    return rng.integers(0, 1 << 64, size=shape, dtype=np.uint64, endpoint=False)


def matmul_case(cg, ro, rng, op):
    while True:
        M, N, K = dim(rng, 3000), dim(rng, 1500), dim(rng, 6000)
        if M * N * K <= BUDGET:
            break
    tx, ty = (bool(rng.integers(0, 2)), bool(rng.integers(0, 2))) if op == "matmul_t" else (False, False)
    desc = f"{op} M={M} N={N} K={K} trans=({tx},{ty})"
    L, R = [words(rng, (M, K)) for _ in range(2)], [words(rng, (N, K)) for _ in range(2)]
    want = ro.party_matmul(L[0], L[1], R[0], R[1])
    dl = [cg.to_device(np.ascontiguousarray(a.T) if tx else a) for a in L]
    dr = [cg.to_device(np.ascontiguousarray(a.T) if ty else a) for a in R]
    if op == "matmul_t":
        got = cg.cg_share_matmul_t(*dl, *dr, tx, ty)
    elif op == "matmul_f64limb":
        got = cg.cg_share_matmul_f64limb(*dl, *dr)
    elif op == "matmul_acc":
        init = words(rng, (M, N))
        with np.errstate(over="ignore"):
            want = want + init
        got = cg.cg_share_matmul_acc(*dl, *dr, cg.to_device(init))
    else:
        got = cg.cg_share_matmul(*dl, *dr)
    return desc, cg.to_host(got), want


def conv_case(cg, ro, rng, op):
    while True:
        B, H, W = dim(rng, 6, (1, 2, 3)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        Cin, Cout = dim(rng, 160, (1, 3, 16, 32, 64, 96, 128)), dim(rng, 160, (1, 8, 32, 64, 96, 128))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        st = (int(rng.choice([1, 1, 2, 3])), int(rng.choice([1, 1, 2, 3])))
        pd = (int(rng.integers(0, kh + 1)), int(rng.integers(0, kw + 1)))
        if H + 2 * pd[0] < kh or W + 2 * pd[1] < kw:
            continue
        Ho, Wo = (H + 2 * pd[0] - kh) // st[0] + 1, (W + 2 * pd[1] - kw) // st[1] + 1
        if B * Ho * Wo * Cout * kh * kw * Cin <= BUDGET:
            break
    xs, ws, zs = (B, H, W, Cin), (Cout, kh, kw, Cin), (B, Ho, Wo, Cout)
    desc = f"{op} x={xs} w={ws} stride={st} pad={pd}"
    dev = cg.to_device
    if op in ("conv2d", "conv2d_acc"):
        x, w = [words(rng, xs) for _ in range(2)], [words(rng, ws) for _ in range(2)]
        want = ro.party_conv2d(*x, *w, st, pd)
        if op == "conv2d_acc":
            init = words(rng, zs)
            with np.errstate(over="ignore"):
                want = want + init
            got = cg.cg_share_conv2d_acc(dev(x[0]), dev(x[1]), dev(w[0]), dev(w[1]), dev(init), stride=st, pad=pd)
        else:
            got = cg.cg_share_conv2d(dev(x[0]), dev(x[1]), dev(w[0]), dev(w[1]), stride=st, pad=pd)
    elif op == "dgrad":
        g, w = [words(rng, zs) for _ in range(2)], [words(rng, ws) for _ in range(2)]
        want = ro.party_conv2d_dgrad(*g, *w, xs, st, pd)
        got = torch.full(xs, 0x5A5A5A5A, dtype=torch.int64, device="cuda")      # stale words would show
        cg.cg_share_conv2d_dgrad(dev(g[0]), dev(g[1]), dev(w[0]), dev(w[1]), xs, stride=st, pad=pd, dx_i=got)
    else:
        g, x = [words(rng, zs) for _ in range(2)], [words(rng, xs) for _ in range(2)]
        want = ro.party_conv2d_wgrad(*g, *x, ws, st, pd)
        got = torch.full(ws, 0x5A5A5A5A, dtype=torch.int64, device="cuda")
        cg.cg_share_conv2d_wgrad(dev(g[0]), dev(g[1]), dev(x[0]), dev(x[1]), ws, stride=st, pad=pd, dw_i=got)
    return desc, cg.to_host(got), want


OPS = ("matmul", "matmul_t", "matmul_f64limb", "matmul_acc", "conv2d", "conv2d_acc", "dgrad", "wgrad")


@pytest.mark.parametrize("chunk", range(8))
def test_random_shapes_match_the_oracle(env, chunk):
    cg, ro = env
    for seed in range(31000 + 60 * chunk, 31000 + 60 * (chunk + 1)):
        rng = np.random.default_rng(seed)
        op = OPS[int(rng.integers(0, len(OPS)))]
        desc, got, want = (matmul_case if op.startswith("matmul") else conv_case)(cg, ro, rng, op)
        say(f"seed {seed}: {desc}")
        msg = first_mismatch(np.asarray(got).view(np.uint64).reshape(want.shape), want)
        assert not msg, f"seed {seed} {desc}: {msg}"
