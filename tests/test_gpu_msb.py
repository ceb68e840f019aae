"""GPU parity of the binary-share gates and of the whole addition circuit for the most significant bit,
every party's local steps through the C-ABI, messages as device-to-device assignments, against the CPU
oracle bit for bit, and against plain integer addition of the shares."""
import numpy as np
import pytest

from tests.gpu_util import first_mismatch, gpu_msb_circuit, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KEYS = (bytes(range(16)), bytes(range(16, 32)), bytes(range(32, 48)))


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


@pytest.mark.parametrize("n", [1, 2, 3, 255, 256, 257, 100003, (1 << 20) + 1])
def test_gates_match_the_oracle(cg, ro, wl, n):
    say(f"binary-share gates n={n}")
    h = [wl.draw_ring((n,), 50 + k + n) for k in range(4)]
    d = [cg.to_device(a) for a in h]
    assert not first_mismatch(cg.to_host(cg.cg_bshare_and(*d)), ro.bshare_and(*h))
    za, zb = cg.cg_bshare_xor(*d)
    assert not first_mismatch(cg.to_host(za), h[0] ^ h[2]) and not first_mismatch(cg.to_host(zb), h[1] ^ h[3])
    for shift, last in ((1, False), (8, False), (32, True), (63, False)):
        p_out, g_out = cg.cg_bshare_prefix_stage(*d, shift, last)
        want_p, want_g = ro.ks_stage_local(*h, shift, last)
        assert not first_mismatch(cg.to_host(g_out), want_g)
        assert (p_out is None) == last
        if not last:
            assert not first_mismatch(cg.to_host(p_out), want_p)
    for first in (0, 1, 7):
        got = cg.to_host(cg.cg_bzero_share(KEYS[1], KEYS[0], 9, first, n))
        assert not first_mismatch(got, ro.bzero_share(KEYS[1], KEYS[0], 9, first, n))
        got = cg.to_host(cg.cg_breshare(d[0], KEYS[1], KEYS[0], 9, first))
        assert not first_mismatch(got, ro.breshare(h[0], KEYS[1], KEYS[0], 9, first))


def test_gates_on_unaligned_views_and_in_place(cg, ro, wl):
    n = 1001
    h = [wl.draw_ring((n + 1,), 70 + k) for k in range(4)]
    d = [cg.to_device(a)[1:] for a in h]          # 8-byte aligned only
    hv = [a[1:] for a in h]
    say("binary-share gates, 8-byte aligned views")
    assert not first_mismatch(cg.to_host(cg.cg_bshare_and(*d).contiguous()), ro.bshare_and(*hv))
    p_out, g_out = cg.cg_bshare_prefix_stage(*d, 4)
    want_p, want_g = ro.ks_stage_local(*hv, 4)
    assert not first_mismatch(cg.to_host(p_out.contiguous()), want_p)
    assert not first_mismatch(cg.to_host(g_out.contiguous()), want_g)
    # in place: outputs over the first components
    dd = [cg.to_device(a) for a in h]
    cg.cg_bshare_prefix_stage(*dd, 2, p_out=dd[0], g_out=dd[2])
    want_p, want_g = ro.ks_stage_local(*h, 2)
    assert not first_mismatch(cg.to_host(dd[0]), want_p) and not first_mismatch(cg.to_host(dd[2]), want_g)


def test_addition_circuit_matches_the_oracle_and_plain_addition(cg, ro, wl):
    n = 50000
    say(f"addition circuit on binary shares, n={n}")
    edge = [(1 << 63) - 1, 1, 0], [(1 << 64) - 1, 1, 0], [(1 << 64) - 1] * 3, [5, (1 << 64) - 7, 0]
    x = [wl.draw_ring((n,), 80 + k) for k in range(3)]
    for j, e in enumerate(edge):
        for k in range(3):
            x[k][j] = e[k]
    total = gpu_msb_circuit(cg, [cg.to_device(a) for a in x], KEYS, nonce=6)
    torch.cuda.synchronize()
    want_total, want_msb = ro.msb_protocol(x, KEYS, nonce=6)
    for got, want in zip(total, want_total):
        assert not first_mismatch(cg.to_host(got), want)
    with np.errstate(over="ignore"):
        plain = x[0] + x[1] + x[2]
    opened = cg.to_host(total[0]) ^ cg.to_host(total[1]) ^ cg.to_host(total[2])
    assert not first_mismatch(opened, plain)
    assert np.array_equal(opened >> np.uint64(63), want_msb[0] ^ want_msb[1] ^ want_msb[2])


def test_gate_argument_errors(cg):
    z = torch.zeros(32, dtype=torch.int64, device="cuda")
    for shift in (0, 64, -1):
        with pytest.raises(cg.CgError) as e:
            cg.cg_bshare_prefix_stage(z, z, z, z, shift)
        assert e.value.status == cg.CG_ERR_SHAPE
    with pytest.raises(cg.CgError) as e:
        cg.cg_bshare_and(z[:16], z[:16], z[:16], z[:16], z_i=z[8:24])
    assert e.value.status == cg.CG_ERR_ALIAS
    with pytest.raises(cg.CgError) as e:
        cg.cg_bshare_prefix_stage(z[:16], z[:16], z[:16], z[:16], 1, p_out=z[16:], g_out=z[16:])
    assert e.value.status == cg.CG_ERR_ALIAS


def test_relu_assembled_from_sign_bit_and_products(cg, ro, wl):
    """ReLU on shares end to end, every local step on the GPU: the adder circuit for the sign bit, its three
    binary shares read as arithmetic sharings, two integer XORs (u + v - 2uv) and the final (1 - b) x, each
    product being cg_share_mul + cg_reshare.  The opened result equals max(x, 0) exactly, and every party's
    shares equal the oracle's run of the same steps."""
    n = 20000
    say(f"ReLU from the sign bit and three products, n={n}")
    rng = np.random.default_rng(61)
    xs = rng.integers(-(1 << 40), 1 << 40, size=n, dtype=np.int64)
    xs[:4] = [0, -1, 1, -(1 << 40)]
    x = xs.astype(np.uint64)
    X = ro.share(x, wl.draw_ring(x.shape, 62), wl.draw_ring(x.shape, 63))
    Xd = [cg.to_device(a) for a in X]
    total = gpu_msb_circuit(cg, Xd, KEYS, nonce=7)
    msb = [(t >> 63) & 1 for t in total]                       # a word shift of a share is local
    zero = torch.zeros_like(Xd[0])
    B = [tuple(msb[k] if j == k else zero for j in range(3)) for k in range(3)]

    def mult(U, V, first):
        out = []
        for i in range(3):
            zi = cg.cg_share_mul(U[i], U[(i + 1) % 3], V[i], V[(i + 1) % 3])
            out.append(cg.cg_reshare(zi, KEYS[i], KEYS[(i - 1) % 3], 8, first, out=zi))
        return tuple(out)

    def xor_arith(U, V, first):
        P = mult(U, V, first)
        return tuple(u + v - 2 * p for u, v, p in zip(U, V, P))   # linear combination of shares: local

    D = xor_arith(B[0], B[1], 0)
    Bsum = xor_arith(D, B[2], n)
    keep = tuple((1 if k == 0 else 0) - b for k, b in enumerate(Bsum))
    R = mult(Xd, keep, 2 * n)
    torch.cuda.synchronize()
    opened = cg.to_host(cg.cg_reconstruct(*R)).astype(np.int64)
    assert np.array_equal(opened, np.maximum(xs, 0))
    # the oracle's run of the same steps, share by share
    _, msb_o = ro.msb_protocol(X, KEYS, nonce=7)
    zo = np.zeros_like(x)
    Bo = [tuple(msb_o[k] if j == k else zo for j in range(3)) for k in range(3)]

    def mult_o(U, V, first):
        return tuple(ro.reshare(ro.party_mul(U[i], U[(i + 1) % 3], V[i], V[(i + 1) % 3]), KEYS[i], KEYS[(i - 1) % 3], 8, first)
                     for i in range(3))

    def xor_o(U, V, first):
        P = mult_o(U, V, first)
        with np.errstate(over="ignore"):
            return tuple(u + v - np.uint64(2) * p for u, v, p in zip(U, V, P))

    Bs_o = xor_o(xor_o(Bo[0], Bo[1], 0), Bo[2], n)
    with np.errstate(over="ignore"):
        keep_o = tuple((np.uint64(1) if k == 0 else np.uint64(0)) - b for k, b in enumerate(Bs_o))
    Ro = mult_o(X, keep_o, 2 * n)
    for got, want in zip(R, Ro):
        assert not first_mismatch(cg.to_host(got), want)


@pytest.mark.parametrize("m", [1, 2, 7, 8, 9, 64, 1001])
def test_bit_planes_and_unpack(cg, ro, wl, m):
    from tests.gpu_util import first_mismatch as fm
    n = 64 * m
    say(f"cg_bit_transpose64 / cg_bits_unpack n={n}")
    x = wl.draw_ring((n,), 900 + m)
    planes = cg.cg_bit_transpose64(cg.to_device(x))
    want = ro.bit_planes(x)
    assert not fm(cg.to_host(planes), want)
    for b in (0, 31, 63):
        for nn in (n, n - 1, max(1, n - 63)):
            got = cg.to_host(cg.cg_bits_unpack(planes[b], nn))
            assert not fm(got, ro.bits_unpack(want[b], nn))


@pytest.mark.parametrize("k,m", [(1, 1), (1, 6), (2, 5), (32, 40), (16, 1001), (4, 2)])
def test_carry_level_matches_the_oracle(cg, ro, wl, k, m):
    say(f"cg_bshare_carry_level k={k} m={m}")
    h = [wl.draw_ring((2 * k, m), 950 + j + k + m) for j in range(4)]
    d = [cg.to_device(a) for a in h]
    for last in (False, True):
        p_out, g_out = cg.cg_bshare_carry_level(*d, last)
        want_p, want_g = ro.carry_level_local(*h, last)
        assert not first_mismatch(cg.to_host(g_out), want_g)
        assert (p_out is None) == last
        if not last:
            assert not first_mismatch(cg.to_host(p_out), want_p)


def test_pruned_circuit_matches_the_oracle_and_the_sign_of_the_sum(cg, ro, wl):
    from tests.gpu_util import gpu_msb_sliced
    n = 64 * 700
    say(f"sign bit from the pruned circuit on bit planes, n={n}")
    x = [wl.draw_ring((n,), 980 + k) for k in range(3)]
    edge = [((1 << 63) - 1, 1, 0), ((1 << 64) - 1, 1, 0), ((1 << 64) - 1,) * 3, (5, (1 << 64) - 7, 0), (0, 0, 0),
            (1 << 62, (1 << 62) - 1, 1)]
    for j, e in enumerate(edge):
        for k in range(3):
            x[k][j * 3] = e[k]
    msb = gpu_msb_sliced(cg, [cg.to_device(a) for a in x], KEYS, nonce=9)
    torch.cuda.synchronize()
    want = ro.msb_protocol_sliced(x, KEYS, nonce=9)
    for got, w in zip(msb, want):
        assert not first_mismatch(cg.to_host(got), w)
    opened = cg.to_host(msb[0]) ^ cg.to_host(msb[1]) ^ cg.to_host(msb[2])
    with np.errstate(over="ignore"):
        plain = x[0] + x[1] + x[2]
    assert np.array_equal(ro.bits_unpack(opened, n), plain >> np.uint64(63))


@pytest.mark.parametrize("n", [1, 2, 255, 256, 100003])
def test_adder_cells_match_the_oracle(cg, ro, wl, n):
    say(f"cg_bshare_csa / cg_bshare_half_adder n={n}")
    h = [wl.draw_ring((n,), 1100 + k + n) for k in range(6)]
    d = [cg.to_device(a) for a in h]
    got = cg.cg_bshare_csa(*d)
    want = ro.csa_local(*h)
    for g, w in zip(got, want):
        assert not first_mismatch(cg.to_host(g), w)
    got = cg.cg_bshare_half_adder(*d[:4])
    want = ro.half_adder_local(*h[:4])
    for g, w in zip(got, want):
        assert not first_mismatch(cg.to_host(g), w)
    # components that are zero everywhere may be left out
    zero = np.zeros(n, dtype=np.uint64)
    for absent in [(1, 2, 4, 5), (0, 3), (0, 1, 2, 3, 4), (5,)]:
        got = cg.cg_bshare_csa(*(None if k in absent else d[k] for k in range(6)))
        want = ro.csa_local(*(zero if k in absent else h[k] for k in range(6)))
        for g, w in zip(got, want):
            assert not first_mismatch(cg.to_host(g), w), absent
    # in place: sum over a, propagate over s
    cg.cg_bshare_csa(*d, s_i=d[0], s_ip1=d[1], carry_i=d[4])
    want = ro.csa_local(*h)
    for g, w in zip((d[0], d[1], d[4]), want):
        assert not first_mismatch(cg.to_host(g), w)


def test_pruned_circuit_built_from_adder_cells_gives_the_same_shares(cg, ro, wl):
    """The pruned circuit with its first two rounds taken by the fused cells: same blinded shares as the
    gate-by-gate assembly, since the cells compute the same local values."""
    from tests.gpu_util import gpu_msb_sliced
    n = 64 * 300
    say(f"pruned circuit from adder cells, n={n}")
    x = [wl.draw_ring((n,), 1200 + k) for k in range(3)]
    dx = [cg.to_device(a) for a in x]
    ref = gpu_msb_sliced(cg, dx, KEYS, nonce=11)
    got = gpu_msb_sliced(cg, dx, KEYS, nonce=11, cells=True)
    torch.cuda.synchronize()
    for g, r in zip(got, ref):
        assert not first_mismatch(cg.to_host(g), cg.to_host(r))
    want = ro.msb_protocol_sliced(x, KEYS, nonce=11)
    for g, w in zip(got, want):
        assert not first_mismatch(cg.to_host(g), w)


def test_relu_is_the_same_with_either_sign_bit_circuit(cg, ro, wl):
    from tests.gpu_util import gpu_relu
    n = 64 * 100
    say(f"ReLU with the word-parallel and the pruned sign-bit circuit, n={n}")
    rng = np.random.default_rng(77)
    xs = rng.integers(-(1 << 45), 1 << 45, size=n, dtype=np.int64)
    x = xs.astype(np.uint64)
    X = tuple(cg.to_device(s) for s in ro.share(x, wl.draw_ring(x.shape, 78), wl.draw_ring(x.shape, 79)))
    for sliced in (False, True):
        R = gpu_relu(cg, X, KEYS, nonce=20, sliced=sliced)
        opened = cg.to_host(cg.cg_reconstruct(*R)).astype(np.int64)
        assert np.array_equal(opened, np.maximum(xs, 0)), f"sliced={sliced}"
