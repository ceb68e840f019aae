"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle, bit for bit."""
import numpy as np
import pytest

from tests.gpu_util import first_mismatch, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def cg():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2104_10949_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def ro():
    from oracle import ring_oracle
    return ring_oracle


@pytest.fixture(scope="module")
def wl():
    from paper_2104_10949_amd import workloads
    return workloads


ROUTES = ["direct", "workspace"]


def make_workspace(nbytes):
    # poisoned scratch memory: nothing may depend on its previous contents
    return torch.full((max(nbytes, 16) // 8 + 2,), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")


def run_matmul(cg, ops, route="direct"):
    d = [cg.to_device(a) for a in ops]
    if route == "direct":
        z = cg.cg_share_matmul(*d)
    else:
        M, K = ops[0].shape
        ws = make_workspace(cg.cg_share_matmul_workspace_bytes(M, ops[2].shape[0], K))
        z = cg.cg_share_matmul_ws(*d, ws)
    torch.cuda.synchronize()
    return cg.to_host(z)


def run_conv(cg, ops, stride, pad, route="direct"):
    d = [cg.to_device(a) for a in ops]
    if route == "direct":
        z = cg.cg_share_conv2d(*d, stride=stride, pad=pad)
    else:
        ws = make_workspace(cg.cg_share_conv2d_workspace_bytes(ops[0].shape, ops[2].shape, stride, pad))
        z = cg.cg_share_conv2d_ws(*d, ws, stride=stride, pad=pad)
    torch.cuda.synchronize()
    return cg.to_host(z)


MATMUL_SHAPES = [
    (1, 1, 1), (1, 1, 2), (3, 5, 7), (32, 32, 32), (33, 31, 34), (17, 63, 65), (128, 64, 32),
    (129, 65, 33), (130, 70, 100), (200, 100, 31), (256, 256, 256), (300, 129, 130), (64, 200, 512),
    (5, 1000, 96), (1000, 3, 40),
    (32, 130, 2048), (7, 300, 4100), (1, 128, 2048),   # small batch, long K: the 32-row tile
    (3, 70001, 40), (70001, 3, 40), (2, 2, 30000),      # very wide, very tall, very deep
    (1568, 256, 2304), (700, 520, 3000), (1000, 136, 5000),   # tile counts that take the streamed distribution
]


@pytest.mark.parametrize("route", ROUTES)
@pytest.mark.parametrize("M,N,K", MATMUL_SHAPES)
def test_matmul_random_shares(cg, ro, wl, M, N, K, route):
    say(f"cg_share_matmul random M={M} N={N} K={K} route={route}")
    seed = 7000 + M * 31 + N * 17 + K
    ops = (wl.draw_ring((M, K), seed), wl.draw_ring((M, K), seed + 1),
           wl.draw_ring((N, K), seed + 2), wl.draw_ring((N, K), seed + 3))
    got = run_matmul(cg, ops, route)
    want = ro.party_matmul(*ops)
    assert not first_mismatch(got, want), first_mismatch(got, want)


@pytest.mark.parametrize("route", ROUTES)
@pytest.mark.parametrize("word", [0x8080808080808080, 0xFFFFFFFFFFFFFFFF, 0x7F7F7F7F7F7F7F7F, 0, 1,
                                  0x8000000000000000, 0x00000000FFFFFFFF, 0x0100000000000000,
                                  0x80FF7F0080FF7F00])
def test_matmul_adversarial_constant_words(cg, ro, word, route):
    M, N, K = 70, 40, 300
    say(f"cg_share_matmul constant word 0x{word:016x} M={M} N={N} K={K} route={route}")
    x = np.full((M, K), word, dtype=np.uint64)
    y = np.full((N, K), word, dtype=np.uint64)
    got = run_matmul(cg, (x, x, y, y), route)
    want = ro.party_matmul(x, x, y, y)
    assert not first_mismatch(got, want), first_mismatch(got, want)
    assert int(got[0, 0]) == (3 * K * word * word) % (1 << 64)


@pytest.mark.parametrize("route,K", [("direct", 257), ("direct", 258), ("workspace", 258)])
def test_matmul_mixed_adversarial_words(cg, ro, wl, route, K):
    M, N = 96, 80
    say(f"cg_share_matmul adversarial word mix M={M} N={N} K={K} route={route}")
    words = np.array(wl.ADVERSARIAL_WORDS, dtype=np.uint64)
    rng = np.random.default_rng(99)
    ops = tuple(words[rng.integers(0, len(words), size=s)] for s in ((M, K), (M, K), (N, K), (N, K)))
    got = run_matmul(cg, ops, route)
    want = ro.party_matmul(*ops)
    assert not first_mismatch(got, want), first_mismatch(got, want)


@pytest.mark.parametrize("route", ROUTES)
@pytest.mark.parametrize("K", [8192, 16352, 16384, 16400, 40000])
def test_matmul_long_k_crosses_accumulator_folds(cg, ro, wl, K, route):
    """Worst-case digits (every byte 0x80, every digit product +2^14) through one
    or more folds of the 32-bit partial sums, plus random words."""
    M, N = 40, 33
    say(f"cg_share_matmul long K={K} worst-case bytes route={route}")
    x = np.full((M, K), 0x8080808080808080, dtype=np.uint64)
    y = np.full((N, K), 0x8080808080808080, dtype=np.uint64)
    got = run_matmul(cg, (x, x, y, y), route)
    expect = (3 * K * 0x8080808080808080 * 0x8080808080808080) % (1 << 64)
    assert np.all(got == np.uint64(expect))
    say(f"cg_share_matmul long K={K} random")
    ops = (wl.draw_ring((M, K), K), wl.draw_ring((M, K), K + 1), wl.draw_ring((N, K), K + 2),
           wl.draw_ring((N, K), K + 3))
    got = run_matmul(cg, ops, route)
    want = ro.party_matmul(*ops)
    assert not first_mismatch(got, want), first_mismatch(got, want)


@pytest.mark.parametrize("route", ROUTES)
def test_matmul_long_k_without_split_k_folds_in_place(cg, ro, wl, route):
    """256 output tiles (no split-K) and K = 16400 = 513 slices: the 32-bit partial sums are folded
    into z twice, the second time by read-add-write.  Worst-case digits over the whole output, then
    random words on sampled rows."""
    M, N, K = 2048, 1024, 16400
    say(f"cg_share_matmul M={M} N={N} K={K}: two folds per block, no split-K, route={route}")
    x = np.full((M, K), 0x8080808080808080, dtype=np.uint64)
    y = np.full((N, K), 0x8080808080808080, dtype=np.uint64)
    got = run_matmul(cg, (x, x, y, y), route)
    expect = (3 * K * 0x8080808080808080 * 0x8080808080808080) % (1 << 64)
    assert np.all(got == np.uint64(expect))
    ops = (wl.draw_ring((M, K), 51), wl.draw_ring((M, K), 52), wl.draw_ring((N, K), 53), wl.draw_ring((N, K), 54))
    got = run_matmul(cg, ops, route)
    for r0 in (0, 1000, 2040):
        want = ro.party_matmul(ops[0][r0:r0 + 8], ops[1][r0:r0 + 8], ops[2], ops[3])
        assert not first_mismatch(got[r0:r0 + 8], want), f"rows {r0}.."


# Left operands of few rows take a kernel of their own (one 16 x 16 block of z per thread block, the slices of K
# shared out over its waves, K split over blocks as well when z has few blocks).
FEW_ROWS_SHAPES = [
    (16, 16, 32), (1, 1, 2), (32, 512, 512), (32, 200, 512), (8, 1000, 2048),    # the fully connected layers of the configs
    (17, 33, 70), (33, 47, 1026), (64, 64, 1024), (49, 300, 512),                # ragged in every dimension, 2-4 row blocks
    (5, 7, 20000), (16, 40, 4100),                                               # K split over blocks, ragged last range
    (2, 3, 130816), (2, 3, 130818),                                              # the longest K it takes; just beyond
    (16, 5000, 64), (3, 70001, 2),                                               # many column blocks
    (32, 4608, 256), (32, 4609, 256),                                            # either side of its work limit
]


@pytest.mark.parametrize("route", ["plain", "acc"])
@pytest.mark.parametrize("M,N,K", FEW_ROWS_SHAPES)
def test_matmul_few_rows(cg, ro, wl, M, N, K, route):
    say(f"cg_share_matmul few rows M={M} N={N} K={K} route={route}")
    ops = (wl.draw_ring((M, K), 91), wl.draw_ring((M, K), 92), wl.draw_ring((N, K), 93), wl.draw_ring((N, K), 94))
    dev = [cg.to_device(a) for a in ops]
    want = ro.party_matmul(*ops)
    if route == "plain":
        got = cg.cg_share_matmul(*dev)
    else:
        base = wl.draw_ring((M, N), 95)
        got = cg.to_device(base)
        cg.cg_share_matmul_acc(*dev, got)
        with np.errstate(over="ignore"):
            want = want + base
    torch.cuda.synchronize()
    assert not first_mismatch(cg.to_host(got), want), first_mismatch(cg.to_host(got), want)


@pytest.mark.parametrize("word", [0x8080808080808080, 0xFFFFFFFFFFFFFFFF, 0x7F7F7F7F7F7F7F7F, 0x80FF7F0080FF7F00])
def test_matmul_few_rows_worst_case_digits_over_the_longest_wave_range(cg, ro, word):
    """Every digit product at its extreme through as many slices as one wave ever accumulates before its fold."""
    M, N, K = 16, 4096, 130816      # 256 blocks of z: K is not split, each of a block's 8 waves takes 511 slices
    say(f"cg_share_matmul few rows constant word 0x{word:016x} M={M} N={N} K={K}")
    x = torch.full((M, K), word - (1 << 64) if word >> 63 else word, dtype=torch.int64, device="cuda")
    y = torch.full((N, K), word - (1 << 64) if word >> 63 else word, dtype=torch.int64, device="cuda")
    got = cg.cg_share_matmul(x, x, y, y)
    torch.cuda.synchronize()
    assert np.all(cg.to_host(got) == np.uint64((3 * K * word * word) % (1 << 64)))


@pytest.mark.parametrize("shape", [(3, 2, (1 << 20) + (1 << 17) + 6),      # even K, one ragged tile
                                   (5, 70, (1 << 20) + 33),                # odd K, two column tiles
                                   (130, 3, (1 << 20) + 2)])               # two row tiles: row offsets beyond 2^31 bytes
@pytest.mark.parametrize("route", ["plain", "ws", "acc"])
def test_matmul_rows_longer_than_a_buffer_view_addresses(cg, ro, wl, shape, route):
    M, N, K = shape
    if route != "plain" and M != 3:
        pytest.skip("the other entry points share the plain call's path for long rows; one shape covers them")
    say(f"cg_share_matmul M={M} N={N} K={K} (> 2^20: 64-bit row addresses), route {route}")
    ops = (wl.draw_ring((M, K), 71), wl.draw_ring((M, K), 72), wl.draw_ring((N, K), 73), wl.draw_ring((N, K), 74))
    dev = [cg.to_device(a) for a in ops]
    want = ro.party_matmul(*ops)
    if route == "plain":
        got = cg.cg_share_matmul(*dev)
    elif route == "ws":
        assert cg.cg_share_matmul_workspace_bytes(M, N, K) == 0
        got = cg.cg_share_matmul_ws(*dev, torch.empty(16, dtype=torch.int64, device="cuda"))
    else:
        base = wl.draw_ring((M, N), 75)
        got = cg.to_device(base)
        cg.cg_share_matmul_acc(*dev, got)
        want = want + base
    torch.cuda.synchronize()
    assert not first_mismatch(cg.to_host(got), want), first_mismatch(cg.to_host(got), want)


@pytest.mark.parametrize("trans", [(1, 0), (0, 1), (1, 1)])
def test_matmul_transposed_operands_with_a_long_contraction(cg, ro, wl, trans):
    tx, ty = trans
    M, N, K = 70, 9, (1 << 20) + 36
    say(f"cg_share_matmul_t M={M} N={N} K={K} trans_x={tx} trans_y={ty}")
    L_ = (wl.draw_ring((M, K), 81), wl.draw_ring((M, K), 82))
    R_ = (wl.draw_ring((N, K), 83), wl.draw_ring((N, K), 84))
    x = [cg.to_device(np.ascontiguousarray(a.T) if tx else a) for a in L_]
    y = [cg.to_device(np.ascontiguousarray(a.T) if ty else a) for a in R_]
    got = cg.cg_share_matmul_t(*x, *y, bool(tx), bool(ty))
    torch.cuda.synchronize()
    want = ro.party_matmul(*L_, *R_)
    assert not first_mismatch(cg.to_host(got), want), first_mismatch(cg.to_host(got), want)


def test_matmul_largest_k_of_the_buffer_view_route(cg, ro, wl):
    M, N, K = 3, 2, 1 << 20
    say(f"cg_share_matmul M={M} N={N} K=2^20 (the longest row a buffer view addresses)")
    ops = (wl.draw_ring((M, K), 61), wl.draw_ring((M, K), 62), wl.draw_ring((N, K), 63), wl.draw_ring((N, K), 64))
    got = run_matmul(cg, ops)
    want = ro.party_matmul(*ops)
    assert not first_mismatch(got, want), first_mismatch(got, want)


def test_matmul_unaligned_views_take_the_8_byte_path(cg, ro, wl):
    M, N, K = 50, 37, 64
    say("cg_share_matmul with 8-byte-aligned (not 16) operand pointers")
    ops = (wl.draw_ring((M, K), 1), wl.draw_ring((M, K), 2), wl.draw_ring((N, K), 3), wl.draw_ring((N, K), 4))
    dev = []
    for a in ops:
        buf = torch.empty(a.size + 1, dtype=torch.int64, device="cuda")
        view = buf[1:].view(a.shape)
        view.copy_(torch.from_numpy(a.view(np.int64)))
        assert view.data_ptr() % 16 == 8
        dev.append(view)
    z = cg.cg_share_matmul(*dev)
    torch.cuda.synchronize()
    want = ro.party_matmul(*ops)
    assert not first_mismatch(cg.to_host(z), want)


CONV_CASES = [
    # B, H, W, Cin, Cout, kh, kw, stride, pad
    (1, 4, 4, 1, 1, 1, 1, (1, 1), (0, 0)),
    (2, 8, 8, 3, 5, 3, 3, (1, 1), (1, 1)),
    (2, 9, 7, 3, 64, 5, 5, (1, 1), (2, 2)),
    (1, 32, 32, 3, 70, 11, 11, (4, 4), (9, 9)),
    (3, 10, 12, 32, 40, 3, 3, (1, 1), (1, 1)),
    (2, 12, 12, 64, 130, 3, 3, (2, 2), (1, 1)),
    (2, 14, 14, 64, 96, 1, 1, (1, 1), (0, 0)),
    (2, 14, 14, 64, 96, 1, 1, (2, 2), (0, 0)),
    (1, 30, 30, 3, 64, 7, 7, (2, 2), (3, 3)),
    (2, 6, 5, 16, 33, 2, 3, (1, 2), (1, 0)),
    (5, 3, 3, 96, 20, 3, 3, (1, 1), (1, 1)),
    (2, 7, 7, 6, 10, 1, 1, (1, 1), (0, 0)),
    (4, 5, 5, 7, 9, 1, 1, (1, 1), (0, 0)),
    (200, 1, 1, 32, 16, 3, 3, (1, 1), (1, 1)),
    (1, 12, 12, 32, 40, 9, 9, (1, 1), (4, 4)),       # 81 taps: more than the tap mask of the 32-channel gather holds, general gather
    (2, 10, 11, 64, 70, 9, 8, (2, 1), (4, 3)),
    (2, 11, 12, 32, 40, 4, 8, (1, 1), (1, 3)),       # 32 taps: the largest window of the 32-channel gather
    (2, 11, 12, 32, 40, 5, 7, (1, 1), (2, 3)),       # 35 taps
    # 32-tap windows of other shapes, padded up to the window's own size: every bit of the tap mask, the mask's last
    # bit included, is set for some pixel and clear for another
    (1, 3, 40, 32, 8, 1, 32, (1, 1), (0, 31)),
    (1, 40, 3, 32, 8, 32, 1, (1, 1), (31, 0)),
    (2, 9, 9, 32, 16, 8, 4, (1, 2), (7, 3)),
    (1, 6, 20, 32, 8, 2, 16, (1, 1), (1, 15)),
    (1, 5, 5, 32, 8, 6, 5, (1, 1), (5, 4)),          # 30 taps, windows larger than the image
    (8, 14, 14, 256, 256, 3, 3, (1, 1), (1, 1)),     # 13 x 4 tiles, 72 slices: streamed distribution
    (3, 21, 21, 96, 200, 3, 3, (1, 1), (1, 1)),
]


@pytest.mark.parametrize("route", ROUTES)
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_random_shares(cg, ro, wl, case, route):
    B, H, W, Cin, Cout, kh, kw, stride, pad = case
    say(f"cg_share_conv2d random {case} route={route}")
    seed = 9000 + sum(case[:7])
    xs, ws = (B, H, W, Cin), (Cout, kh, kw, Cin)
    ops = (wl.draw_ring(xs, seed), wl.draw_ring(xs, seed + 1), wl.draw_ring(ws, seed + 2),
           wl.draw_ring(ws, seed + 3))
    got = run_conv(cg, ops, stride, pad, route)
    want = ro.party_conv2d(*ops, stride, pad)
    assert not first_mismatch(got, want), first_mismatch(got, want)


@pytest.mark.parametrize("route", ROUTES)
def test_matmul_operand_larger_than_2_gib(cg, ro, wl, route):
    """Left operand shares of 2.3 GB each: block views are rebased, offsets stay 32-bit.
    Sampled outputs and the last (ragged) tile rows against the oracle."""
    M, N, K = 70001, 96, 4096
    say(f"cg_share_matmul M={M} N={N} K={K} (x shares > 2 GiB) route={route}")
    rng = np.random.default_rng(4242)
    xa = rng.integers(0, 1 << 64, size=(M, K), dtype=np.uint64, endpoint=False)
    xb = rng.integers(0, 1 << 64, size=(M, K), dtype=np.uint64, endpoint=False)
    ya, yb = wl.draw_ring((N, K), 4243), wl.draw_ring((N, K), 4244)
    assert xa.nbytes > (1 << 31)
    got = run_matmul(cg, (xa, xb, ya, yb), route)
    rows = sorted(set([0, 1, 127, 128, 65535, 65536, 65537, 69999, 70000] +
                      [int(v) for v in rng.integers(0, M, size=40)]))
    for m in rows:
        want = ro.party_matmul(xa[m:m + 1], xb[m:m + 1], ya, yb)
        assert np.array_equal(got[m:m + 1], want), f"row {m}"
    for m, n in zip(rng.integers(0, M, size=200), rng.integers(0, N, size=200)):
        assert int(got[m, n]) == ro.party_matmul_at(xa, xb, ya, yb, int(m), int(n))


def test_conv_input_larger_than_2_gib(cg, ro, wl):
    """Convolution whose input shares exceed 2 GiB (per-block view rebasing on image boundaries)."""
    B, H, W, Cin, Cout = 460, 96, 96, 64, 64
    say(f"cg_share_conv2d B={B} {H}x{W}x{Cin} -> {Cout}, 3x3 pad 1 (x shares > 2 GiB)")
    rng = np.random.default_rng(777)
    xs, ws = (B, H, W, Cin), (Cout, 3, 3, Cin)
    xa = rng.integers(0, 1 << 64, size=xs, dtype=np.uint64, endpoint=False)
    xb = rng.integers(0, 1 << 64, size=xs, dtype=np.uint64, endpoint=False)
    wa, wb = wl.draw_ring(ws, 778), wl.draw_ring(ws, 779)
    assert xa.nbytes > (1 << 31)
    for route in ROUTES:
        got = run_conv(cg, (xa, xb, wa, wb), (1, 1), (1, 1), route)
        assert got.shape == (B, H, W, Cout)
        for b in (0, 1, 230, 458, 459):   # whole images, first, middle and last
            want = ro.party_conv2d(xa[b:b + 1], xb[b:b + 1], wa, wb, (1, 1), (1, 1))
            assert np.array_equal(got[b:b + 1], want), f"image {b} route {route}"
        for b, ho, wo, co in zip(rng.integers(0, B, 100), rng.integers(0, H, 100), rng.integers(0, W, 100),
                                 rng.integers(0, Cout, 100)):
            want = ro.party_conv2d_at(xa, xb, wa, wb, int(b), int(ho), int(wo), int(co), (1, 1), (1, 1))
            assert int(got[b, ho, wo, co]) == want


def test_workspace_errors(cg):
    say("workspace argument errors")
    x = torch.zeros((128, 64), dtype=torch.int64, device="cuda")
    y = torch.zeros((64, 64), dtype=torch.int64, device="cuda")
    need = cg.cg_share_matmul_workspace_bytes(128, 64, 64)
    assert need == (2 * 128 + 2 * 64) * 2 * 256
    assert cg.cg_share_matmul_workspace_bytes(128, 64, 63) == 0     # odd K: direct route only
    assert cg.cg_share_matmul_workspace_bytes(0, 64, 64) == 0
    assert cg.cg_share_matmul_workspace_bytes(64, 64, 64) == 0      # few rows: the plain call's kernel is the fast one
    small = torch.zeros(need // 8 - 1, dtype=torch.int64, device="cuda")
    with pytest.raises(cg.CgError) as e:
        cg.cg_share_matmul_ws(x, x, y, y, small)
    assert e.value.status == cg.CG_ERR_WORKSPACE
    with pytest.raises(cg.CgError) as e:
        cg.cg_share_matmul_ws(x, x, y, y, None)
    assert e.value.status == cg.CG_ERR_NULL
    with pytest.raises(cg.CgError) as e:
        cg.cg_share_matmul_ws(x, x, y, y, x.view(-1))               # workspace overlaps an operand
    assert e.value.status in (cg.CG_ERR_ALIAS, cg.CG_ERR_WORKSPACE)
    # odd K never touches the workspace
    xo = torch.zeros((8, 7), dtype=torch.int64, device="cuda")
    cg.cg_share_matmul_ws(xo, xo, xo, xo, None)
    torch.cuda.synchronize()


def test_three_parties_reconstruct_to_the_product_config1(cg, ro, wl):
    """Config 1: 256^3 matmul of fixed-point N(0,1) reals, all three parties on the GPU,
    outputs opened on the GPU and compared with the plaintext product."""
    L = wl.config_layers(1)[0]
    seed = wl.layer_seed(1, 0)
    say("config 1: three parties, reconstruct, decode")
    t = wl.FRAC_BITS
    X, Y = wl.draw_reals(L.x_shape, L.x_dist, seed), wl.draw_reals(L.w_shape, L.w_dist, seed + 1)
    ex, ey = ro.encode(X, t), ro.encode(Y, t)
    sx = ro.share(ex, wl.draw_ring(ex.shape, seed + 2), wl.draw_ring(ex.shape, seed + 3))
    sy = ro.share(ey, wl.draw_ring(ey.shape, seed + 4), wl.draw_ring(ey.shape, seed + 5))
    dx, dy = [cg.to_device(s) for s in sx], [cg.to_device(s) for s in sy]
    z = []
    for i in range(3):
        zi = cg.cg_share_matmul(dx[i], dx[(i + 1) % 3], dy[i], dy[(i + 1) % 3])
        torch.cuda.synchronize()
        want = ro.party_matmul(sx[i], sx[(i + 1) % 3], sy[i], sy[(i + 1) % 3])
        assert not first_mismatch(cg.to_host(zi), want), f"party {i}"
        z.append(zi)
    opened = cg.to_host(cg.cg_reconstruct(*z))
    torch.cuda.synchronize()
    assert np.array_equal(opened, ro.matmul(ex, ey))
    got = ro.decode(opened, 2 * t)
    assert np.max(np.abs(got - ro.decode(ex, t) @ ro.decode(ey, t).T)) <= 2.0 ** -12


@pytest.mark.parametrize("n", [0, 1, 2, 3, 255, 256, 257, 1 << 16, (1 << 20) + 3])
def test_elementwise_ops(cg, ro, wl, n):
    say(f"element-wise share ops n={n}")
    a, b, c, d = (wl.draw_ring((n,), 500 + i) for i in range(4))
    da, db, dc, dd = (cg.to_device(v) for v in (a, b, c, d))
    alpha, gamma = 0x9E3779B97F4A7C15, 0xFEDCBA9876543210
    za, zb = cg.cg_share_add(da, db, dc, dd)
    wa, wb = ro.share_add(a, b, c, d)
    assert np.array_equal(cg.to_host(za), wa) and np.array_equal(cg.to_host(zb), wb)
    za, zb = cg.cg_share_mul_public(da, db, alpha)
    wa, wb = ro.share_mul_public(a, b, alpha)
    assert np.array_equal(cg.to_host(za), wa) and np.array_equal(cg.to_host(zb), wb)
    for party in range(3):
        za, zb = cg.cg_share_add_public(da, db, gamma, party)
        wa, wb = ro.share_add_public(a, b, gamma, party)
        assert np.array_equal(cg.to_host(za), wa) and np.array_equal(cg.to_host(zb), wb)
    out = cg.cg_reconstruct(da, db, dc)
    assert np.array_equal(cg.to_host(out), ro.reconstruct(a, b, c))
    # in place
    ea, eb = da.clone(), db.clone()
    cg.cg_share_add(ea, eb, dc, dd, za=ea, zb=eb)
    wa, wb = ro.share_add(a, b, c, d)
    assert np.array_equal(cg.to_host(ea), wa) and np.array_equal(cg.to_host(eb), wb)


def test_elementwise_and_gates_beyond_one_grid_trip(cg, ro, wl):
    """The element-wise kernels cap their grid (2^23 words per trip) and walk further with a grid stride: n just
    above that cap plus 2^20 + 3 words reaches the second trip, its partial last chunk and the odd tail word,
    with 16-byte-aligned pointers and with pointers offset by one word (the 8-byte path)."""
    n = (1 << 23) + (1 << 20) + 3
    say(f"element-wise ops and gates across a second grid trip, n={n}")
    a, b, c, d = (wl.draw_ring((n + 1,), 700 + i) for i in range(4))
    keys = PRF_KEYS
    for off in (0, 1):
        ha, hb, hc, hd = (v[off:off + n] for v in (a, b, c, d))
        da, db, dc, dd = (cg.to_device(v)[off:off + n] for v in (a, b, c, d))
        za, zb = cg.cg_share_add(da, db, dc, dd)
        wa, wb = ro.share_add(ha, hb, hc, hd)
        assert not first_mismatch(cg.to_host(za), wa) and not first_mismatch(cg.to_host(zb), wb)
        out = cg.cg_reconstruct(da, db, dc)
        assert not first_mismatch(cg.to_host(out), ro.reconstruct(ha, hb, hc))
        g = cg.cg_bshare_and(da, db, dc, dd)
        assert not first_mismatch(cg.to_host(g), ro.bshare_and(ha, hb, hc, hd))
        r = cg.cg_reshare(da, keys[0], keys[2], 0x1234, 5)
        assert not first_mismatch(cg.to_host(r), ro.reshare(ha, keys[0], keys[2], 0x1234, 5))
        del da, db, dc, dd, za, zb, out, g, r
    # column sums and the zero fill at a size beyond their grid caps: 2^19 + 1 columns, 17 rows
    rows, cols = 17, (1 << 19) + 1
    xa, xb = wl.draw_ring((rows, cols), 710), wl.draw_ring((rows, cols), 711)
    sa, sb = cg.cg_share_col_sum(cg.to_device(xa), cg.to_device(xb))
    wa, wb = ro.share_col_sum(xa, xb)
    assert not first_mismatch(cg.to_host(sa), wa) and not first_mismatch(cg.to_host(sb), wb)


def test_elementwise_unaligned(cg, ro, wl):
    n = 1001
    say("element-wise ops on 8-byte-aligned views")
    a, b, c = (wl.draw_ring((n,), 600 + i) for i in range(3))
    dev = []
    for v in (a, b, c):
        buf = torch.empty(n + 1, dtype=torch.int64, device="cuda")
        buf[1:].copy_(torch.from_numpy(v.view(np.int64)))
        dev.append(buf[1:])
    out = cg.cg_reconstruct(*dev)
    assert np.array_equal(cg.to_host(out), ro.reconstruct(a, b, c))


PRF_KEYS = [bytes(range(16)), bytes(range(16, 32)), bytes([7 * i % 251 for i in range(16)])]


@pytest.mark.parametrize("n,first", [(1, 0), (1, 1), (2, 0), (2, 1), (3, 5), (255, 2), (256, 3), (1000, 0),
                                     (65537, 11), ((1 << 20) + 1, (1 << 40) + 7)])
def test_zero_share_matches_the_oracle(cg, ro, n, first):
    say(f"cg_zero_share n={n} first={first}")
    nonce = 0xA5A5000011112222
    for i in range(3):
        got = cg.to_host(cg.cg_zero_share(PRF_KEYS[i], PRF_KEYS[(i - 1) % 3], nonce, first, n))
        want = ro.zero_share(PRF_KEYS[i], PRF_KEYS[(i - 1) % 3], nonce, first, n)
        assert not first_mismatch(got, want), first_mismatch(got, want)
    assert cg.cg_zero_share(PRF_KEYS[0], PRF_KEYS[2], nonce, first, 0).numel() == 0


def test_reshare_after_matmul_opens_to_the_product(cg, ro, wl):
    M, N, K = 130, 70, 96
    say(f"three parties: cg_share_matmul + cg_reshare + cg_reconstruct, M={M} N={N} K={K}")
    x, y = wl.draw_ring((M, K), 31), wl.draw_ring((N, K), 32)
    sx = ro.share(x, wl.draw_ring((M, K), 33), wl.draw_ring((M, K), 34))
    sy = ro.share(y, wl.draw_ring((N, K), 35), wl.draw_ring((N, K), 36))
    dx, dy = [cg.to_device(s) for s in sx], [cg.to_device(s) for s in sy]
    blinded = []
    for i in range(3):
        z = cg.cg_share_matmul(dx[i], dx[(i + 1) % 3], dy[i], dy[(i + 1) % 3])
        zh = cg.to_host(z)
        b = cg.cg_reshare(z, PRF_KEYS[i], PRF_KEYS[(i - 1) % 3], nonce=5, first=3)
        want = ro.reshare(zh, PRF_KEYS[i], PRF_KEYS[(i - 1) % 3], 5, 3)
        assert not first_mismatch(cg.to_host(b), want), f"party {i}"
        # in place
        cg.cg_reshare(z, PRF_KEYS[i], PRF_KEYS[(i - 1) % 3], nonce=5, first=3, out=z)
        assert np.array_equal(cg.to_host(z), want)
        blinded.append(b)
    # party i's new replicated pair is (blinded_i, blinded_{i+1}); opening gives x y^T
    assert np.array_equal(cg.to_host(cg.cg_reconstruct(*blinded)), ro.matmul(x, y))


@pytest.mark.parametrize("trans_x,trans_y", [(False, True), (True, True), (True, False), (False, False)])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (128, 64, 32), (129, 65, 33), (130, 70, 100),
                                   (300, 129, 130), (64, 200, 513), (1000, 3, 40), (5, 1000, 96), (40, 33, 16400)])
def test_matmul_transposed_operands(cg, ro, wl, M, N, K, trans_x, trans_y):
    say(f"cg_share_matmul_t M={M} N={N} K={K} trans_x={trans_x} trans_y={trans_y}")
    seed = 12000 + M * 31 + N * 17 + K
    xs = (K, M) if trans_x else (M, K)
    ys = (K, N) if trans_y else (N, K)
    ops = (wl.draw_ring(xs, seed), wl.draw_ring(xs, seed + 1), wl.draw_ring(ys, seed + 2), wl.draw_ring(ys, seed + 3))
    d = [cg.to_device(a) for a in ops]
    z = cg.cg_share_matmul_t(*d, trans_x, trans_y)
    torch.cuda.synchronize()
    want = ro.party_matmul_t(*ops, trans_x, trans_y)
    got = cg.to_host(z)
    assert not first_mismatch(got, want), first_mismatch(got, want)


def test_fc_backward_products_open_to_the_gradients(cg, ro, wl):
    """Forward Z = X W^T; backward dX = dZ W and dW = dZ^T X as share products on the
    stored tensors, all three parties, opened and compared with the ring products."""
    Mb, Nout, Kin = 96, 40, 136
    say(f"FC backward on shares: batch {Mb}, {Kin} -> {Nout}")
    X, W, dZ = wl.draw_ring((Mb, Kin), 1), wl.draw_ring((Nout, Kin), 2), wl.draw_ring((Mb, Nout), 3)
    sh = lambda a, s: ro.share(a, wl.draw_ring(a.shape, s), wl.draw_ring(a.shape, s + 1))
    sX, sW, sdZ = sh(X, 10), sh(W, 20), sh(dZ, 30)
    dX_, dW_, ddZ = ([cg.to_device(v) for v in s] for s in (sX, sW, sdZ))
    p = lambda t, i: (t[i], t[(i + 1) % 3])
    dX = [cg.cg_share_matmul_t(*p(ddZ, i), *p(dW_, i), False, True) for i in range(3)]
    dW = [cg.cg_share_matmul_t(*p(ddZ, i), *p(dX_, i), True, True) for i in range(3)]
    torch.cuda.synchronize()
    assert np.array_equal(cg.to_host(cg.cg_reconstruct(*dX)), ro.matmul(dZ, np.ascontiguousarray(W.T)))
    assert np.array_equal(cg.to_host(cg.cg_reconstruct(*dW)),
                          ro.matmul(np.ascontiguousarray(dZ.T), np.ascontiguousarray(X.T)))


def test_calls_can_be_captured_in_a_hip_graph_and_replayed(cg, ro, wl):
    """Every entry point only enqueues kernels on the caller's stream (split-K clears its output with
    a fill kernel, not a memset), so a sequence of calls can be captured once and replayed.  Each replay,
    with fresh inputs copied in between, must equal the eager result."""
    M, N, K = 192, 130, 512          # 2 x 3 tiles -> split-K with the zero-fill kernel
    say(f"HIP graph capture/replay of cg_share_matmul + cg_reshare + cg_share_add, M={M} N={N} K={K}")
    key_a, key_b = bytes(range(16)), bytes(range(32, 48))
    x = [torch.empty((M, K), dtype=torch.int64, device="cuda") for _ in range(2)]
    y = [torch.empty((N, K), dtype=torch.int64, device="cuda") for _ in range(2)]
    z = torch.empty((M, N), dtype=torch.int64, device="cuda")
    zb = torch.empty_like(z)
    sa, sb = torch.empty_like(z), torch.empty_like(z)

    def run():
        cg.cg_share_matmul(x[0], x[1], y[0], y[1], z_i=z)
        cg.cg_reshare(z, key_a, key_b, nonce=9, first=0, out=zb)
        cg.cg_share_add(z, zb, zb, z, za=sa, zb=sb)

    def fill(seed):
        host = [wl.draw_ring((M, K), seed), wl.draw_ring((M, K), seed + 1),
                wl.draw_ring((N, K), seed + 2), wl.draw_ring((N, K), seed + 3)]
        for dst, h in zip(x + y, host):
            dst.copy_(torch.from_numpy(h.view(np.int64)))
        torch.cuda.synchronize()
        return host

    fill(100)
    run()                      # warm-up outside capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        host = fill(200 + 10 * rep)
        graph.replay()
        torch.cuda.synchronize()
        want_z = ro.party_matmul(*host)
        want_zb = ro.reshare(want_z, key_a, key_b, 9, 0)
        with np.errstate(over="ignore"):
            want_s = want_z + want_zb
        assert np.array_equal(cg.to_host(z), want_z), f"replay {rep}: product"
        assert np.array_equal(cg.to_host(zb), want_zb), f"replay {rep}: reshare"
        assert np.array_equal(cg.to_host(sa), want_s) and np.array_equal(cg.to_host(sb), want_s), f"replay {rep}"
        # eager work between replays
        run()
        torch.cuda.synchronize()
        assert np.array_equal(cg.to_host(z), want_z)


@pytest.mark.parametrize("shape,period", [((1,), 1), ((7,), 7), ((1000,), 1000), ((1001,), 1001), ((4, 5, 6, 8), 8),
                                          ((2, 9, 9, 3), 3), ((3, 64, 64, 64), 64), ((1 << 20,), 1 << 20),
                                          ((33, 1 << 10), 1 << 10)])
def test_share_mul_elementwise_and_broadcast(cg, ro, wl, shape, period):
    say(f"cg_share_mul shape={shape} period={period}")
    x = [wl.draw_ring(shape, 700 + i) for i in range(2)]
    y = [wl.draw_ring((period,), 710 + i) for i in range(2)]
    got = cg.to_host(cg.cg_share_mul(*[cg.to_device(v) for v in x + y]))
    want = ro.party_mul(*x, *y)
    assert not first_mismatch(got, want), first_mismatch(got, want)
    # in place over x_i
    dx = [cg.to_device(v) for v in x]
    cg.cg_share_mul(dx[0], dx[1], cg.to_device(y[0]), cg.to_device(y[1]), z_i=dx[0])
    assert np.array_equal(cg.to_host(dx[0]), want)


def test_share_mul_three_parties_open_to_the_product(cg, ro, wl):
    shape, C = (4, 7, 7, 32), 32
    say("cg_share_mul: per-channel secret scale, three parties, opened")
    x, a = wl.draw_ring(shape, 720), wl.draw_ring((C,), 721)
    sx = ro.share(x, wl.draw_ring(shape, 722), wl.draw_ring(shape, 723))
    sa = ro.share(a, wl.draw_ring((C,), 724), wl.draw_ring((C,), 725))
    dx, da = [cg.to_device(v) for v in sx], [cg.to_device(v) for v in sa]
    z = [cg.cg_share_mul(dx[i], dx[(i + 1) % 3], da[i], da[(i + 1) % 3]) for i in range(3)]
    with np.errstate(over="ignore"):
        assert np.array_equal(cg.to_host(cg.cg_reconstruct(*z)), x * a)


@pytest.mark.parametrize("shape,window,stride,pad", [
    ((1, 4, 4, 1), (2, 2), (2, 2), (0, 0)), ((2, 10, 10, 96), (3, 3), (2, 2), (0, 0)),
    ((3, 32, 32, 64), (2, 2), (2, 2), (0, 0)), ((2, 7, 6, 3), (3, 3), (2, 2), (1, 1)),
    ((2, 9, 8, 5), (2, 3), (1, 2), (0, 1)), ((8, 56, 56, 64), (3, 3), (2, 2), (1, 1)),
    ((2, 7, 7, 2048), (7, 7), (7, 7), (0, 0)),
])
def test_sum_pool_matches_the_oracle(cg, ro, wl, shape, window, stride, pad):
    say(f"cg_share_sum_pool2d shape={shape} window={window} stride={stride} pad={pad}")
    xa, xb = wl.draw_ring(shape, 730), wl.draw_ring(shape, 731)
    za, zb = cg.cg_share_sum_pool2d(cg.to_device(xa), cg.to_device(xb), window, stride, pad)
    assert not first_mismatch(cg.to_host(za), ro.sum_pool2d(xa, window, stride, pad))
    assert not first_mismatch(cg.to_host(zb), ro.sum_pool2d(xb, window, stride, pad))


@pytest.mark.parametrize("shape", [(1, 1), (3, 7), (37, 11), (128, 64), (1000, 10), (2, 9, 9, 3), (32, 16, 16, 256),
                                   (5, 1000), (70000, 6)])
def test_bias_add_and_bias_gradient(cg, ro, wl, shape):
    say(f"cg_share_bias_add / cg_share_col_sum shape={shape}")
    cols = shape[-1]
    xa, xb = wl.draw_ring(shape, 610), wl.draw_ring(shape, 611)
    ba, bb = wl.draw_ring((cols,), 612), wl.draw_ring((cols,), 613)
    d = [cg.to_device(a) for a in (xa, xb, ba, bb)]
    za, zb = cg.cg_share_bias_add(*d)
    wa, wb = ro.share_bias_add(xa, xb, ba, bb)
    assert not first_mismatch(cg.to_host(za), wa) and not first_mismatch(cg.to_host(zb), wb)
    sa, sb = cg.cg_share_col_sum(d[0], d[1])
    wa, wb = ro.share_col_sum(xa, xb)
    assert not first_mismatch(cg.to_host(sa), wa) and not first_mismatch(cg.to_host(sb), wb)
    # in place over x
    cg.cg_share_bias_add(*d, za=d[0], zb=d[1])
    wa, wb = ro.share_bias_add(xa, xb, ba, bb)
    assert not first_mismatch(cg.to_host(d[0]), wa) and not first_mismatch(cg.to_host(d[1]), wb)


F64LIMB_SHAPES = [(1, 1, 1), (16, 16, 4), (64, 64, 8), (65, 63, 9), (100, 130, 77), (200, 96, 1000),
                  (33, 40, 40000)]          # the last folds its float64 accumulators more than once


@pytest.mark.parametrize("M,N,K", F64LIMB_SHAPES)
def test_float64_block_comparator_matches_the_oracle(cg, ro, wl, M, N, K):
    """The product on 16-bit blocks in float64 (Sec. II-B) gives the same words as the definition."""
    say(f"matmul_f64limb M={M} N={N} K={K}")
    ops = [wl.draw_ring((M, K), 1), wl.draw_ring((M, K), 2), wl.draw_ring((N, K), 3), wl.draw_ring((N, K), 4)]
    got = cg.to_host(cg.cg_share_matmul_f64limb(*(cg.to_device(a) for a in ops)))
    assert not first_mismatch(got, ro.party_matmul(*ops))


@pytest.mark.parametrize("word", [0xFFFFFFFFFFFFFFFF, 0xFFFF0000FFFF0000, 0x8000800080008000])
def test_float64_block_comparator_stays_exact_on_extreme_blocks(cg, ro, word):
    """Every block at its maximum for the longest accumulation the kernel allows between folds."""
    M, N, K = 32, 32, 70000
    say(f"matmul_f64limb constant words {word:#x}")
    ops = [np.full((M, K), word, dtype=np.uint64), np.full((M, K), word, dtype=np.uint64),
           np.full((N, K), word, dtype=np.uint64), np.full((N, K), word, dtype=np.uint64)]
    got = cg.to_host(cg.cg_share_matmul_f64limb(*(cg.to_device(a) for a in ops)))
    assert not first_mismatch(got, ro.party_matmul(*ops))
