"""Pins for the oracle's binary-share gates and the addition circuit for the most significant bit (no GPU).

Pinned by the plain definitions: the three parties' AND outputs XOR to x & y; zero shares XOR to zero and are
the FIPS-pinned PRF words; and the whole circuit, run on arithmetic shares, opens to the 64-bit sum of the
shares computed by ordinary integer addition (every bit, not only the top one), including inputs whose carries
ripple through all 64 positions.
"""
import numpy as np
import pytest

from oracle import ring_oracle as ro
from paper_2104_10949_amd import workloads as wl

MOD = 1 << 64
KEYS = (bytes(range(16)), bytes(range(16, 32)), bytes(range(32, 48)))


def bshare(v, seed):
    s0, s1 = wl.draw_ring(v.shape, seed), wl.draw_ring(v.shape, seed + 1)
    return s0, s1, v ^ s0 ^ s1


def test_and_gate_is_the_three_term_formula_and_opens_to_the_and():
    x, y = wl.draw_ring((300,), 1), wl.draw_ring((300,), 2)
    X, Y = bshare(x, 3), bshare(y, 5)
    z = [ro.bshare_and(X[i], X[(i + 1) % 3], Y[i], Y[(i + 1) % 3]) for i in range(3)]
    assert np.array_equal(z[0] ^ z[1] ^ z[2], x & y)
    i = 1
    want = [(int(X[1][j]) & int(Y[1][j])) ^ (int(X[2][j]) & int(Y[1][j])) ^ (int(X[1][j]) & int(Y[2][j]))
            for j in range(300)]
    assert [int(v) for v in z[i]] == want


def test_binary_zero_shares_cancel_and_are_prf_words():
    n, nonce, first = 101, 9, 7
    b = [ro.bzero_share(KEYS[i], KEYS[(i - 1) % 3], nonce, first, n) for i in range(3)]
    assert not (b[0] ^ b[1] ^ b[2]).any()
    assert np.array_equal(b[1], ro.prf_words(KEYS[1], nonce, first, n) ^ ro.prf_words(KEYS[0], nonce, first, n))
    z = wl.draw_ring((n,), 11)
    assert np.array_equal(ro.breshare(z, KEYS[1], KEYS[0], nonce, first), z ^ b[1])


def test_prefix_stage_matches_bit_level_definition():
    # opened over the three parties, one stage computes g' = g | (p & g<<s), p' = p & p<<s when p & g = 0
    p, g = wl.draw_ring((200,), 21), wl.draw_ring((200,), 22)
    g = g & ~p
    P, G = bshare(p, 23), bshare(g, 25)
    for shift in (1, 4, 32):
        outs = [ro.ks_stage_local(P[i], P[(i + 1) % 3], G[i], G[(i + 1) % 3], shift) for i in range(3)]
        p_new = outs[0][0] ^ outs[1][0] ^ outs[2][0]
        g_new = outs[0][1] ^ outs[1][1] ^ outs[2][1]
        sh = np.uint64(shift)
        assert np.array_equal(p_new, p & (p << sh))
        assert np.array_equal(g_new, g ^ (p & (g << sh)))
        assert np.array_equal(g_new, g | (p & (g << sh)))   # disjoint, so XOR is OR


def open3(t):
    return t[0] ^ t[1] ^ t[2]


def test_circuit_opens_to_the_integer_sum_of_the_shares():
    n = 4000
    x = (wl.draw_ring((n,), 31), wl.draw_ring((n,), 32), wl.draw_ring((n,), 33))
    total, msb = ro.msb_protocol(x, KEYS, nonce=3)
    with np.errstate(over="ignore"):
        want = x[0] + x[1] + x[2]
    assert np.array_equal(open3(total), want)
    assert np.array_equal(open3(msb), want >> np.uint64(63))


def test_circuit_on_carry_chains_and_signs():
    top = (1 << 63) - 1
    cases = [
        (top, 1, 0),                 # carry ripples through 63 positions into the sign bit
        (MOD - 1, 1, 0),             # ripples through all 64 and out
        (MOD - 1, MOD - 1, MOD - 1), # two carries per column
        (0, 0, 0), (1 << 63, 0, 0), (1 << 63, 1 << 63, 0), (1 << 62, 1 << 62, 0),
        (0x5555555555555555, 0xAAAAAAAAAAAAAAAA, 1), (0x8080808080808080, 0x8080808080808080, 0x8080808080808080),
        (5, MOD - 7, 0),             # small negative secret
        (MOD - 3, 2, 1),             # secret zero from wrapping shares
    ]
    x = tuple(np.array([c[k] for c in cases], dtype=np.uint64) for k in range(3))
    total, msb = ro.msb_protocol(x, KEYS, nonce=4)
    want = [(a + b + c) % MOD for a, b, c in cases]
    assert [int(v) for v in open3(total)] == want
    assert [int(v) for v in open3(msb)] == [w >> 63 for w in want]


def test_sign_of_fixed_point_values():
    rng = np.random.default_rng(41)
    reals = rng.normal(0, 3, size=2000)
    enc = ro.encode(reals, 16)
    shares = ro.share(enc, wl.draw_ring(enc.shape, 42), wl.draw_ring(enc.shape, 43))
    _, msb = ro.msb_protocol(shares, KEYS, nonce=5)
    assert np.array_equal(open3(msb).astype(bool), np.rint(reals * 65536) < 0)


def arithmetic_mult(X, Y, nonce, first):
    """The multiplication protocol on replicated arithmetic sharings given as triples (oracle steps only)."""
    z = []
    for i in range(3):
        zi = ro.party_mul(X[i], X[(i + 1) % 3], Y[i], Y[(i + 1) % 3])
        z.append(ro.reshare(zi, KEYS[i], KEYS[(i - 1) % 3], nonce, first))
    return tuple(z)


def test_relu_from_the_sign_bit_and_three_products():
    """ReLU assembled from the pieces: the sign bit b = b_0 ^ b_1 ^ b_2 from the adder circuit; each b_k read as
    an arithmetic sharing with one non-zero component (the paper's re-interpretation trick in the other
    direction); XOR over the integers, u ^ v = u + v - 2uv, costs one product each; relu(x) = (1 - b) x one
    more.  (The paper uses the bit-injection protocol of ABY3 here, whose steps it does not list; this test
    only needs the multiplication protocol.)  Multiplying by a bit needs no rescaling, so the result is exact."""
    rng = np.random.default_rng(61)
    xs = rng.integers(-(1 << 40), 1 << 40, size=3000, dtype=np.int64)
    xs[:4] = [0, -1, 1, -(1 << 40)]
    x = xs.astype(np.uint64)
    X = ro.share(x, wl.draw_ring(x.shape, 62), wl.draw_ring(x.shape, 63))
    _, msb = ro.msb_protocol(X, KEYS, nonce=7)
    zero = np.zeros_like(x)
    B = [tuple(msb[k] if j == k else zero for j in range(3)) for k in range(3)]   # arithmetic sharings of b_0, b_1, b_2
    n = x.size

    def xor_arith(U, V, first):
        P = arithmetic_mult(U, V, 8, first)
        with np.errstate(over="ignore"):
            return tuple(u + v - np.uint64(2) * p for u, v, p in zip(U, V, P))

    D = xor_arith(B[0], B[1], 0)
    Bsum = xor_arith(D, B[2], n)
    assert np.array_equal(ro.reconstruct(*Bsum), (xs < 0).astype(np.uint64))
    with np.errstate(over="ignore"):
        keep = tuple((np.uint64(1) if k == 0 else np.uint64(0)) - b for k, b in enumerate(Bsum))   # 1 - b: the constant joins share 0
    R = arithmetic_mult(X, keep, 8, 2 * n)
    assert np.array_equal(ro.reconstruct(*R).astype(np.int64), np.maximum(xs, 0))


# ---------------------------------------------------------------- the pruned circuit on bit planes
def test_bit_planes_definition():
    rng = np.random.default_rng(71)
    x = rng.integers(0, 1 << 63, size=128, dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, size=128, dtype=np.uint64)
    planes = ro.bit_planes(x)
    assert planes.shape == (64, 2)
    for b in (0, 1, 31, 32, 62, 63):
        for w in range(2):
            want = sum(((int(x[64 * w + e]) >> b) & 1) << e for e in range(64))
            assert int(planes[b, w]) == want
    assert np.array_equal(ro.bits_unpack(planes[63], 128), x >> np.uint64(63))
    # transposing twice returns the words (a 64 x 64 bit transpose is an involution on each block of 64)
    assert np.array_equal(ro.bit_planes(planes.T.reshape(-1)).T.reshape(-1), x)


def test_pruned_circuit_gives_the_sign_of_the_integer_sum():
    n = 64 * 50
    x = [wl.draw_ring((n,), 81 + k) for k in range(3)]
    top = (1 << 63) - 1
    edge = [(top, 1, 0), (MOD - 1, 1, 0), (MOD - 1, MOD - 1, MOD - 1), (0, 0, 0), (1 << 63, 0, 0), (1 << 63, 1 << 63, 0),
            (1 << 62, 1 << 62, 0), (0x5555555555555555, 0xAAAAAAAAAAAAAAAA, 1), (5, MOD - 7, 0), (MOD - 3, 2, 1),
            (top, 0, 0), (1 << 62, (1 << 62) - 1, 1)]
    for j, e in enumerate(edge):
        for k in range(3):
            x[k][j * 5] = e[k]
    msb = ro.msb_protocol_sliced(x, KEYS, nonce=9)
    with np.errstate(over="ignore"):
        plain = x[0] + x[1] + x[2]
    opened = msb[0] ^ msb[1] ^ msb[2]
    assert np.array_equal(ro.bits_unpack(opened, n), plain >> np.uint64(63))
    # and it agrees with the word-parallel adder's sign bit
    _, msb_word = ro.msb_protocol(x, KEYS, nonce=10)
    assert np.array_equal(ro.bits_unpack(opened, n), msb_word[0] ^ msb_word[1] ^ msb_word[2])


def test_full_and_half_adder_steps_open_to_the_bitwise_definitions():
    a, b, c = (wl.draw_ring((257,), 90 + k) for k in range(3))
    A, B, C = bshare(a, 93), bshare(b, 95), bshare(c, 97)
    outs = [ro.csa_local(A[i], A[(i + 1) % 3], B[i], B[(i + 1) % 3], C[i], C[(i + 1) % 3]) for i in range(3)]
    assert np.array_equal(outs[0][0] ^ outs[1][0] ^ outs[2][0], a ^ b ^ c)
    assert np.array_equal(outs[0][2] ^ outs[1][2] ^ outs[2][2], (a & b) | (a & c) | (b & c))
    for i in range(3):                      # the sum keeps the replicated form
        assert np.array_equal(outs[i][1], outs[(i + 1) % 3][0])
    # one column of the adder: a + b + c = sum + 2 carry, bit by bit
    for j in range(5):
        for bit in (0, 17, 63):
            abc = [(int(v[j]) >> bit) & 1 for v in (a, b, c)]
            s_bit = (int(outs[0][0][j] ^ outs[1][0][j] ^ outs[2][0][j]) >> bit) & 1
            c_bit = (int(outs[0][2][j] ^ outs[1][2][j] ^ outs[2][2][j]) >> bit) & 1
            assert sum(abc) == s_bit + 2 * c_bit
    S, T = bshare(a, 101), bshare(b, 103)
    outs = [ro.half_adder_local(S[i], S[(i + 1) % 3], T[i], T[(i + 1) % 3]) for i in range(3)]
    assert np.array_equal(outs[0][0] ^ outs[1][0] ^ outs[2][0], a ^ b)
    assert np.array_equal(outs[0][2] ^ outs[1][2] ^ outs[2][2], a & b)
