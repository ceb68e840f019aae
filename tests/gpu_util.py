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


def gpu_trunc(cg, z, keys, nonce, d):
    """The two-round truncation protocol on a 3-out-of-3 additive sharing z = (z_0, z_1, z_2) of GPU tensors
    (e.g. the outputs of the local products, or a replicated sharing read as its three shares): returns the
    replicated sharing (s_0, s_1, s_2) of about z / 2^d.  PRF streams `nonce` and `nonce + 1`."""
    n = z[0].numel()
    msg = cg.cg_reshare(z[2], keys[2], keys[1], nonce, 0)
    s0 = cg.cg_trunc1_local(z[0], None, keys[0], keys[2], nonce, 0, d)
    s1 = cg.cg_trunc1_local(z[1], msg, keys[1], keys[0], nonce, 0, d, keys[1], nonce + 1)
    s2 = cg.cg_prf_words(keys[1], nonce + 1, 0, n).view_as(s0)
    return (s0, s1, s2)


def gpu_mul_trunc(cg, U, V, keys, nonce, t):
    """Fixed-point product of two replicated sharings at scale 2^t: every party's three-term product on the GPU,
    then the truncation protocol on the three additive results (its first step blinds them)."""
    z = tuple(cg.cg_share_mul(U[i], U[(i + 1) % 3], V[i], V[(i + 1) % 3]) for i in range(3))
    return gpu_trunc(cg, z, keys, nonce, t)



def softmax_float_model(x, log_m, newton):
    """The approximations of gpu_softmax in float64, without shares or fixed point."""
    y = x - x.max(axis=1, keepdims=True)
    e = (1 + y / 2 ** log_m) ** (2 ** log_m)
    s = e.sum(axis=1, keepdims=True)
    z = np.full_like(s, 1 / x.shape[1])
    for _ in range(newton):
        z = 2 * z - s * z * z
    return e * z


def gpu_softmax(cg, X, keys, fresh, t, log_m, newton):
    """Row-wise softmax of a replicated sharing X [batch, d] at scale 2^t, from local steps on the GPU: maximum by a
    tree of comparisons, (1 + x/m)^m with m = 2^log_m by repeated squaring, reciprocal of the row sums by `newton`
    Newton-Raphson iterations from the fixed start 1/d.  `fresh()` hands out unused PRF nonces (4 apart).
    Returns (softmax sharing, sharing of the row maxima)."""
    import torch
    d = X[0].shape[1]
    sub = lambda U, V: tuple(u - v for u, v in zip(U, V))        # linear combinations of shares are local
    add = lambda U, V: tuple(u + v for u, v in zip(U, V))
    const = lambda c, like: tuple(torch.full_like(like, int(round(c * 2 ** t))) if k == 0 else torch.zeros_like(like)
                                  for k in range(3))             # a public constant lives in share 0
    cols = [tuple(s[:, j].contiguous() for s in X) for j in range(d)]
    while len(cols) > 1:
        nxt = [add(b, gpu_relu(cg, sub(a, b), keys, fresh())) for a, b in zip(cols[0::2], cols[1::2])]   # max = b + relu(a - b)
        if len(cols) % 2:
            nxt.append(cols[-1])
        cols = nxt
    mx = cols[0]
    Y = tuple((x - m[:, None]).contiguous() for x, m in zip(X, mx))
    U = add(const(1.0, Y[0]), gpu_trunc(cg, Y, keys, fresh(), log_m))        # 1 + y / m
    for _ in range(log_m):
        U = gpu_mul_trunc(cg, U, U, keys, fresh(), t)
    S = tuple(u.sum(dim=1, keepdim=True).contiguous() for u in U)            # sums of shares are local
    Z = const(1.0 / d, S[0])
    for _ in range(newton):
        Z2 = gpu_mul_trunc(cg, Z, Z, keys, fresh(), t)
        SZ2 = gpu_mul_trunc(cg, S, Z2, keys, fresh(), t)
        Z = sub(add(Z, Z), SZ2)
    Zb = tuple(z.expand(-1, d).contiguous() for z in Z)
    return gpu_mul_trunc(cg, U, Zb, keys, fresh(), t), mx
