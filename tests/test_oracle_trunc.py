"""Pins for the oracle's share-truncation step (no GPU).

The step is a protocol with an error term, so it is pinned by what the mathematics fixes: the
signed shift against Python's floor division on edge words, every party's formula re-derived with
Python integers from the (FIPS-pinned) PRF words, the opened result within one unit in the last
place of floor(x / 2^d) for values far from the ring's size, exactness for d = 0 and for summands
that are multiples of 2^d, and the known failure when the two summands wrap.
"""
import numpy as np
import pytest

from oracle import ring_oracle as ro
from paper_2104_10949_amd import workloads as wl

MOD = 1 << 64
K0, K1, K2 = bytes(range(16)), bytes(range(16, 32)), bytes(range(32, 48))
SAME = bytes(16)   # key_self == key_prev makes alpha vanish


def signed(v: int) -> int:
    return v - MOD if v >= 1 << 63 else v


def floor_shift(v: int, d: int) -> int:
    return (signed(v) >> d) % MOD     # Python's >> on negative integers rounds down


EDGE = [0, 1, 2, 3, 0xFFFF, 0x10000, 0x10001, (1 << 63) - 1, 1 << 63, (1 << 63) + 1, MOD - 1, MOD - 2,
        MOD - 0x10000, MOD - 0x10001, 0x8080808080808080, 0x7F7F7F7F7F7F7F7F, 0x00000000FFFFFFFF, 0xFFFFFFFF00000000]


@pytest.mark.parametrize("d", [0, 1, 7, 16, 20, 32, 62, 63])
def test_signed_shift_on_edge_words(d):
    z = np.array(EDGE, dtype=np.uint64)
    got = ro.trunc1_local(z, None, SAME, SAME, 5, 3, d)
    assert [int(v) for v in got] == [floor_shift(v, d) for v in EDGE]
    # with a second summand the shift applies to the wrapped sum
    m = np.array(EDGE[::-1], dtype=np.uint64)
    got = ro.trunc1_local(z, m, SAME, SAME, 5, 3, d)
    assert [int(v) for v in got] == [floor_shift((a + b) % MOD, d) for a, b in zip(EDGE, EDGE[::-1])]


def test_shift_outside_the_word_is_rejected():
    z = np.zeros(4, dtype=np.uint64)
    for d in (-1, 64, 100):
        with pytest.raises(ValueError):
            ro.trunc1_local(z, None, SAME, SAME, 0, 0, d)


@pytest.mark.parametrize("first", [0, 1, 6, 7])
def test_local_step_is_shift_of_blinded_sum_minus_mask(first):
    n, d, nonce, mnonce = 37, 16, 11, 12
    z, m = wl.draw_ring((n,), 71), wl.draw_ring((n,), 72)
    a_self, a_prev = ro.prf_words(K1, nonce, first, n), ro.prf_words(K0, nonce, first, n)
    r = ro.prf_words(K1, mnonce, first, n)
    want = [(floor_shift((int(z[j]) + int(a_self[j]) - int(a_prev[j]) + int(m[j])) % MOD, d) - int(r[j])) % MOD
            for j in range(n)]
    got = ro.trunc1_local(z, m, K1, K0, nonce, first, d, K1, mnonce)
    assert [int(v) for v in got] == want
    # without message and mask: P_0's step
    want0 = [floor_shift((int(z[j]) + int(a_self[j]) - int(a_prev[j])) % MOD, d) for j in range(n)]
    assert [int(v) for v in ro.trunc1_local(z, None, K1, K0, nonce, first, d)] == want0


def additive_shares(x, seed):
    z0, z1 = wl.draw_ring(x.shape, seed), wl.draw_ring(x.shape, seed + 1)
    with np.errstate(over="ignore"):
        return z0, z1, x - z0 - z1


@pytest.mark.parametrize("d,bits", [(16, 40), (20, 44), (1, 30), (32, 48)])
def test_opened_result_is_within_one_unit_of_the_floor(d, bits):
    n = 20000
    rng = np.random.default_rng(300 + d)
    xs = rng.integers(-(1 << bits), 1 << bits, size=n, dtype=np.int64)
    x = xs.astype(np.uint64)
    s = ro.trunc1_protocol(additive_shares(x, 310 + d), (K0, K1, K2), nonce=21, first=5, d=d, mask_nonce=22)
    opened = ro.reconstruct(*s).astype(np.int64)
    err = opened - (xs >> d)                      # numpy's >> on int64 rounds down
    assert set(np.unique(err).tolist()) <= {-1, 0}
    assert (err == -1).any() and (err == 0).any()  # the error is real, and not systematic
    # the mask is the third share, and nothing else
    assert np.array_equal(s[2], ro.prf_words(K1, 22, 5, n))


def test_d_zero_is_a_plain_resharing():
    x = wl.draw_ring((500,), 400)
    s = ro.trunc1_protocol(additive_shares(x, 401), (K0, K1, K2), nonce=1, first=0, d=0, mask_nonce=2)
    assert np.array_equal(ro.reconstruct(*s), x)


def test_exact_when_both_summands_are_multiples_of_the_divisor():
    d = 16
    rng = np.random.default_rng(410)
    a = rng.integers(-(1 << 40), 1 << 40, size=300, dtype=np.int64) << d
    b = rng.integers(-(1 << 40), 1 << 40, size=300, dtype=np.int64) << d
    s0 = ro.trunc1_local(a.astype(np.uint64), None, SAME, SAME, 0, 0, d)
    s1 = ro.trunc1_local(b.astype(np.uint64), None, SAME, SAME, 0, 0, d)
    with np.errstate(over="ignore"):
        assert np.array_equal((s0 + s1).astype(np.int64), (a + b) >> d)


def test_wrapping_summands_break_the_result_as_the_bound_says():
    # two positive summands whose sum wraps to -2: the shifted summands miss floor(-2 / 2) = -1 by 2^63
    a = np.array([(1 << 63) - 1], dtype=np.uint64)
    s0 = ro.trunc1_local(a, None, SAME, SAME, 0, 0, 1)
    s1 = ro.trunc1_local(a, None, SAME, SAME, 0, 0, 1)
    assert (int(s0[0]) + int(s1[0])) % MOD == (1 << 63) - 2
    assert floor_shift((2 * ((1 << 63) - 1)) % MOD, 1) == MOD - 1
