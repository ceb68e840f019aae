"""Helpers shared by the GPU parity tests."""
import sys

import numpy as np


def say(msg: str) -> None:
    """Name the case before the GPU step that runs it, flushed, so a fault can be traced."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def first_mismatch(got: np.ndarray, want: np.ndarray) -> str:
    if got.shape != want.shape:
        return f"shape {got.shape} != {want.shape}"
    bad = np.argwhere(got != want)
    if bad.size == 0:
        return ""
    idx = tuple(int(v) for v in bad[0])
    return (f"{len(bad)} of {got.size} elements differ; first at {idx}: "
            f"got 0x{int(got[idx]):016x} want 0x{int(want[idx]):016x}")


def gpu_msb_circuit(cg, x_dev, KEYS, nonce):
    """The circuit of the oracle's msb_protocol, every local step on the GPU through the C-ABI."""
    n = x_dev[0].numel()
    import torch
    zero = torch.zeros_like(x_dev[0])
    pair = lambda v, i: (v[i], v[(i + 1) % 3])
    counter = [0]

    def and_gate(X, Y):
        first = counter[0]
        counter[0] += n
        return tuple(cg.cg_breshare(cg.cg_bshare_and(*pair(X, i), *pair(Y, i)), KEYS[i], KEYS[(i - 1) % 3], nonce, first)
                     for i in range(3))

    def xor(X, Y):
        # share-wise XOR; run through the pair entry point party by party (component i is party i's first)
        return tuple(cg.cg_bshare_xor(*pair(X, i), *pair(Y, i))[0] for i in range(3))

    A, B, C = (x_dev[0], zero, zero), (zero, x_dev[1], zero), (zero, zero, x_dev[2])
    S = xor(xor(A, B), C)
    carry = xor(and_gate(xor(A, C), xor(B, C)), C)
    T = tuple(c << 1 for c in carry)              # a word shift of a share is local
    P0 = xor(S, T)
    G = and_gate(S, T)
    P = P0
    for stage, shift in enumerate((1, 2, 4, 8, 16, 32)):
        last = stage == 5
        first = counter[0]
        counter[0] += 2 * n
        new_p, new_g = [], []
        for i in range(3):
            p_loc, g_loc = cg.cg_bshare_prefix_stage(*pair(P, i), *pair(G, i), shift, last)
            new_g.append(cg.cg_breshare(g_loc, KEYS[i], KEYS[(i - 1) % 3], nonce, first, out=g_loc))
            if not last:
                new_p.append(cg.cg_breshare(p_loc, KEYS[i], KEYS[(i - 1) % 3], nonce, first + n, out=p_loc))
        G = tuple(new_g)
        if not last:
            P = tuple(new_p)
    total = xor(P0, tuple(g << 1 for g in G))
    return total


def gpu_share_mult(cg, U, V, keys, nonce, first):
    """The multiplication protocol on replicated arithmetic sharings held as triples of GPU tensors:
    every party's three-term product and blinding on the GPU, the message a plain assignment."""
    out = []
    for i in range(3):
        zi = cg.cg_share_mul(U[i], U[(i + 1) % 3], V[i], V[(i + 1) % 3])
        out.append(cg.cg_reshare(zi, keys[i], keys[(i - 1) % 3], nonce, first, out=zi))
    return tuple(out)


def gpu_relu(cg, X, keys, nonce, sliced=False, with_mask=False):
    """ReLU of a replicated arithmetic sharing X = (x_0, x_1, x_2): sign bit from the adder circuit, its three
    binary shares read as arithmetic sharings, two integer XORs (u + v - 2uv) and (1 - b) x.  Uses the PRF
    streams `nonce` (binary gates) and `nonce + 1` (products).  sliced=True takes the sign bit from the pruned
    circuit on bit planes (the element count must then be a multiple of 64)."""
    import torch
    n = X[0].numel()
    if sliced:
        planes = gpu_msb_sliced(cg, [x.reshape(-1) for x in X], keys, nonce, cells=True)
        msb = [cg.cg_bits_unpack(p, n).view_as(X[0]) for p in planes]
    else:
        total = gpu_msb_circuit(cg, list(X), keys, nonce)
        msb = [(t >> 63) & 1 for t in total]
    zero = torch.zeros_like(X[0])
    B = [tuple(msb[k] if j == k else zero for j in range(3)) for k in range(3)]

    def xor_arith(U, V, first):
        P = gpu_share_mult(cg, U, V, keys, nonce + 1, first)
        return tuple(u + v - 2 * p for u, v, p in zip(U, V, P))

    b = xor_arith(xor_arith(B[0], B[1], 0), B[2], n)
    keep = tuple((1 if k == 0 else 0) - s for k, s in enumerate(b))
    out = gpu_share_mult(cg, X, keep, keys, nonce + 1, 2 * n)
    return (out, keep) if with_mask else out          # keep = sharing of relu'(x) as an unscaled integer 0 / 1


def gpu_msb_sliced(cg, x_dev, KEYS, nonce, cells=False):
    """The oracle's msb_protocol_sliced with every local step on the GPU through the C-ABI: returns the
    binary sharing (triple of [m] words) of the packed sign bits of x_0 + x_1 + x_2 (n = 64 m elements).
    cells=True takes the first two rounds with the fused adder cells instead of single gates."""
    import torch
    n = x_dev[0].numel()
    m = n // 64
    pair = lambda v, i: (v[i], v[(i + 1) % 3])
    counter = [0]

    def blind(z, i):
        return cg.cg_breshare(z, KEYS[i], KEYS[(i - 1) % 3], nonce, counter[0], out=z)

    def and_gate(X, Y):
        out = tuple(blind(cg.cg_bshare_and(*pair(X, i), *pair(Y, i)), i) for i in range(3))
        counter[0] += X[0].numel()
        return out

    def xor(X, Y):
        return tuple(cg.cg_bshare_xor(*pair(X, i), *pair(Y, i))[0] for i in range(3))

    planes = [cg.cg_bit_transpose64(a.reshape(-1)) for a in x_dev]
    zero = torch.zeros_like(planes[0])
    A, B, C = (planes[0], zero, zero), (zero, planes[1], zero), (zero, zero, planes[2])
    up = lambda v: torch.cat([torch.zeros_like(v[:1]), v[:63]])        # one bit position up: a move of planes
    if cells:
        # the three summands are sharings with a single non-zero share: zero components are passed as None
        An, Bn, Cn = (planes[0], None, None), (None, planes[1], None), (None, None, planes[2])
        loc = [cg.cg_bshare_csa(*pair(An, i), *pair(Bn, i), *pair(Cn, i)) for i in range(3)]
        S = tuple(loc[i][0] for i in range(3))
        carry = tuple(blind(loc[i][2], i) for i in range(3))
        counter[0] += n
        T = tuple(up(c) for c in carry)
        loc = [cg.cg_bshare_half_adder(*pair(S, i), *pair(T, i)) for i in range(3)]
        P0 = tuple(loc[i][0] for i in range(3))
        G0 = tuple(blind(loc[i][2], i) for i in range(3))
        counter[0] += n
    else:
        S = xor(xor(A, B), C)
        carry = xor(and_gate(xor(A, C), xor(B, C)), C)
        T = tuple(up(c) for c in carry)
        P0 = xor(S, T)
        G0 = and_gate(S, T)
    P, G = tuple(up(p) for p in P0), tuple(up(g) for g in G0)
    while P[0].shape[0] > 1:
        last = P[0].shape[0] == 2
        loc = [cg.cg_bshare_carry_level(*pair(P, i), *pair(G, i), last) for i in range(3)]
        G = tuple(blind(loc[i][1], i) for i in range(3))
        counter[0] += G[0].numel()
        if not last:
            P = tuple(blind(loc[i][0], i) for i in range(3))
            counter[0] += P[0].numel()
        else:
            P = G
    return tuple(p0[63] ^ g[0] for p0, g in zip(P0, G))                # XOR of shares: local
