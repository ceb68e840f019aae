"""Pins for the oracle's PRF, zero shares and reshare step (no GPU)."""
import os

import numpy as np

from oracle import ring_oracle as ro
from paper_2104_10949_amd import workloads as wl

MOD = 1 << 64
HERE = os.path.dirname(os.path.abspath(__file__))
K0, K1, K2 = bytes(range(16)), bytes(range(16, 32)), bytes([7 * i % 251 for i in range(16)])


def test_aes128_published_vectors():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "aes128_fips197.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for key, pt, ct in rows:
        assert ro.aes128_encrypt_block(bytes.fromhex(key), bytes.fromhex(pt)).hex() == ct


def test_aes_is_a_permutation_of_the_block_and_key_sensitive():
    pt = bytes(16)
    outs = {ro.aes128_encrypt_block(bytes([i]) + bytes(15), pt) for i in range(64)}
    assert len(outs) == 64
    outs = {ro.aes128_encrypt_block(K0, bytes([i]) + bytes(15)) for i in range(64)}
    assert len(outs) == 64


def test_prf_word_layout_matches_the_counter_mode_reading():
    nonce = 0x1122334455667788
    w = ro.prf_words(K0, nonce, 0, 6)
    for block in range(3):
        pt = block.to_bytes(8, "little") + nonce.to_bytes(8, "little")
        ct = ro.aes128_encrypt_block(K0, pt)
        assert int(w[2 * block]) == int.from_bytes(ct[:8], "little")
        assert int(w[2 * block + 1]) == int.from_bytes(ct[8:], "little")
    # a stream can be continued at any index, odd ones included
    full = ro.prf_words(K1, nonce, 0, 37)
    for first in (1, 2, 5, 16, 36):
        assert np.array_equal(ro.prf_words(K1, nonce, first, 37 - first), full[first:])
    big = (1 << 40) + 3
    assert np.array_equal(ro.prf_words(K1, nonce, big, 4)[1:], ro.prf_words(K1, nonce, big + 1, 3))
    assert not np.array_equal(ro.prf_words(K1, nonce, 0, 8), ro.prf_words(K1, nonce + 1, 0, 8))


def test_zero_shares_sum_to_zero_over_the_three_parties():
    n, nonce = 1001, 42
    keys = [K0, K1, K2]
    alpha = [ro.zero_share(keys[i], keys[(i - 1) % 3], nonce, 7, n) for i in range(3)]
    total = [(int(a) + int(b) + int(c)) % MOD for a, b, c in zip(*alpha)]
    assert not any(total)
    assert all(a.any() for a in alpha)
    f = [ro.prf_words(k, nonce, 7, n) for k in keys]
    with np.errstate(over="ignore"):
        assert np.array_equal(alpha[1], f[1] - f[0])      # alpha_i = F(k_i) - F(k_{i-1})
        assert np.array_equal(alpha[0], f[0] - f[2])


def test_reshare_keeps_the_opened_value():
    M, N, K = 6, 5, 9
    x, y = wl.draw_ring((M, K), 1), wl.draw_ring((N, K), 2)
    sx = ro.share(x, wl.draw_ring((M, K), 3), wl.draw_ring((M, K), 4))
    sy = ro.share(y, wl.draw_ring((N, K), 5), wl.draw_ring((N, K), 6))
    keys = [K0, K1, K2]
    z = [ro.party_matmul(*ro.party_pair(sx, i), *ro.party_pair(sy, i)) for i in range(3)]
    blinded = [ro.reshare(z[i], keys[i], keys[(i - 1) % 3], 99, 0) for i in range(3)]
    assert np.array_equal(ro.reconstruct(*blinded), ro.matmul(x, y))
    for i in range(3):
        assert not np.array_equal(blinded[i], z[i])
        with np.errstate(over="ignore"):
            assert np.array_equal(blinded[i] - z[i],
                                  ro.zero_share(keys[i], keys[(i - 1) % 3], 99, 0, M * N).reshape(M, N))
