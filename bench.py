#!/usr/bin/env python3
"""Benchmark of one party's local linear-layer products on replicated shares over Z_{2^64}.

One "step" is one pass of the hot path over one batch: every layer of the
VGG16-shaped configuration (batch 32, 64x64x3 input, thirteen 3x3 convolutions
and three fully connected layers), each computed by one party from its four
share tensors with cg_share_conv2d / cg_share_matmul, or with their *_ws
variants (caller-supplied scratch memory, allocated once outside the timed
region) for the layers where the library's own rule says that route is faster;
--plain times the plain calls only, and the default line reports both.  Inputs
are uniform 64-bit words (the distribution of any two of the three shares),
seeded, resident in HBM before the timed region.

Prints ONE JSON line: effective 64-bit ring MAC/s (three ring products per
party and output element, as the protocol states them), the int8-MFMA roofline
fraction of the share-product kernel measured over the same timed region, the
CPU oracle timed on the host cores for the same workload, and (object "rows")
the largest GEMM shapes, the other convolution configurations, the streaming
kernels against the HBM peak and the small fully connected layers warm and cold.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "Z_2^64 share-GEMM effective 64-bit MAC/s (1 party) + % MFMA peak"
INT8_PEAK_TOPS = 5000.0  # MI355X dense int8 MFMA, published: 5.0 POP/s (2 ops per MAC)
HBM_PEAK_GBS = 8000.0    # MI355X HBM3E, published: 8 TB/s
LAST_LEVEL_CACHE_BYTES = 256 << 20
DIGIT_MACS_PER_RING_MAC_TRIPLE = 72  # 2 ring products x 36 signed-byte digit pairs per (m, n, k)
WORKLOAD_CONFIG = 4
# HBM bytes per share_gemm_kernel launch on the config-4 step, from the two rocprofv3 --pmc runs summarised in
# profiles/share_gemm_config4_hbm_traffic.txt (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000 by the 1 GiB copy calibration).
PROFILED_TRAFFIC_CONFIG4 = {"read_bytes_per_launch": 65.8e6, "write_bytes_per_launch": 22.6e6,
                            "algorithmic_bytes_per_launch": 61.0e6,
                            "conversion_pass_per_scratch_route_layer": {"read_bytes": 47.8e6, "write_bytes": 43.5e6},
                            "source": "profiles/share_gemm_config4_hbm_traffic.txt"}


def parse_args():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=250)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=WORKLOAD_CONFIG, choices=[1, 2, 3, 4, 5],
                    help="benchmark configuration (default: the VGG16-shaped one)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-min-s", type=float, default=10.0,
                    help="repeat whole passes of the CPU oracle until this many seconds are collected")
    ap.add_argument("--cpu-budget-s", type=float, default=30.0,
                    help="stop adding layers to the CPU-oracle sample after this many seconds")
    ap.add_argument("--layers", action="store_true", help="also print a per-layer table to stderr")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the register-only MFMA issue-rate measurement")
    ap.add_argument("--plain", action="store_true",
                    help="time the plain entry points only (no layer takes the route with scratch memory)")
    ap.add_argument("--no-rows", action="store_true",
                    help="skip the rows printed beside the step by default (largest share-GEMM shapes, totals of the "
                         "other configurations, streaming kernels, warm/cold fully connected layers)")
    ap.add_argument("--extras", action="store_true",
                    help="after the step, also time the rows outside the five configurations (square share products, "
                         "the paper's Fig. 1 convolution shapes, backward products, element-wise and PRF kernels) and "
                         "add them to the JSON line under \"extras\"")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="after the timed region, run one plain device copy of this many MiB (a kernel of "
                         "known traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def _rnd(torch, shape, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randint(-2 ** 63, 2 ** 63 - 1, tuple(shape), dtype=torch.int64, device="cuda", generator=g)


def _timed(torch, fn, warm=3, iters=10, lead=None):
    """Mean duration in ms of `iters` calls after `warm` untimed ones, HIP events on the launch stream.
    `lead`: GPU work enqueued ahead of the first event, long enough for the host to enqueue all timed calls
    meanwhile; launches of a few microseconds are then timed as the GPU runs them back to back, not at the rate
    at which Python issues them."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if lead is not None:
        lead()
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def measure_rows(torch, cg, wl, headline_config):
    """Rows reported beside the timed step in every run (not part of `value`): the largest share-GEMM shapes,
    the totals of the other convolution configurations, the streaming kernels against the HBM peak, and the
    HBM-bound fully connected layers with warm and cold operands."""
    out = {}
    # ---- largest GEMM shapes: plain entry point and the digit-plane route with caller scratch
    rows = []
    for M, N, K in [(4096, 4096, 4096), (8192, 8192, 2048)]:
        ops = [_rnd(torch, (M, K), 1), _rnd(torch, (M, K), 2), _rnd(torch, (N, K), 3), _rnd(torch, (N, K), 4)]
        z = torch.empty((M, N), dtype=torch.int64, device="cuda")
        ws = torch.empty(cg.cg_share_matmul_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
        ops_per = 2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * M * N * K
        ms = _timed(torch, lambda: cg.cg_share_matmul(*ops, z_i=z), warm=2, iters=8)
        ms_ws = _timed(torch, lambda: cg.cg_share_matmul_ws(*ops, ws, z_i=z), warm=2, iters=8)
        rows.append({"gemm": [M, N, K], "cg_share_matmul_ms": round(ms, 4),
                     "ring_macs_per_s": 3.0 * M * N * K / (ms * 1e-3),
                     "int8_tops": round(ops_per / (ms * 1e-3) / 1e12, 1),
                     "frac_of_peak": round(ops_per / (ms * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4),
                     "cg_share_matmul_ws_ms": round(ms_ws, 4),
                     "ws_frac_of_peak": round(ops_per / (ms_ws * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)})
        if (M, N, K) == (4096, 4096, 4096):
            # the same launches on all-zero shares: control flow and memory traffic do not depend on the data,
            # the power the matrix cores draw does (share words are uniformly random, the worst case), so the gap
            # to the rows above is what the chip's power limit costs and these are what the schedule itself reaches
            for t in ops:
                t.zero_()
            ms0 = _timed(torch, lambda: cg.cg_share_matmul(*ops, z_i=z), warm=2, iters=8)
            ms0_ws = _timed(torch, lambda: cg.cg_share_matmul_ws(*ops, ws, z_i=z), warm=2, iters=8)
            rows[-1]["all_zero_operands"] = {
                "cg_share_matmul_ms": round(ms0, 4),
                "frac_of_peak": round(ops_per / (ms0 * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4),
                "cg_share_matmul_ws_ms": round(ms0_ws, 4),
                "ws_frac_of_peak": round(ops_per / (ms0_ws * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)}
        del ops, z, ws
    out["largest_gemm_shapes"] = rows
    # ---- the other convolution configurations: one step = all their layers, same method as the headline step
    rows = []
    for cfg in (3, 5):
        if cfg == headline_config:
            continue
        layers = wl.config_layers(cfg)
        dev, outs = [], []
        for li, L in enumerate(layers):
            dev.append([_rnd(torch, L.x_shape, 7 * li + 1), _rnd(torch, L.x_shape, 7 * li + 2),
                        _rnd(torch, L.w_shape, 7 * li + 3), _rnd(torch, L.w_shape, 7 * li + 4)])
            outs.append(torch.empty(L.z_shape, dtype=torch.int64, device="cuda"))

        def step():
            for L, ops, z in zip(layers, dev, outs):
                for _ in range(L.repeat):
                    if L.kind == "conv":
                        cg.cg_share_conv2d(*ops, stride=(L.stride, L.stride), pad=(L.pad, L.pad), z_i=z)
                    else:
                        cg.cg_share_matmul(*ops, z_i=z)
        ms = _timed(torch, step, warm=3, iters=20)
        mnk = sum(L.mnk * L.repeat for L in layers)
        tops = 2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * mnk / (ms * 1e-3) / 1e12
        rows.append({"config": cfg, "layers": sum(L.repeat for L in layers), "ms_per_step": round(ms, 4),
                     "ring_macs_per_s": 3.0 * mnk / (ms * 1e-3), "int8_tops": round(tops, 1),
                     "frac_of_peak": round(tops / INT8_PEAK_TOPS, 4)})
        del dev, outs
    out["other_configs"] = rows
    # ---- element-wise share operations: HBM-bound, 2^26 words per stream (beyond the 256 MB last-level cache)
    n = 1 << 26
    a, b, c, d = (_rnd(torch, (n,), s) for s in (1, 2, 3, 4))
    o1, o2 = torch.empty_like(a), torch.empty_like(a)
    rows = []
    for name, nbytes, fn in [
        ("cg_share_add", 48, lambda: cg.cg_share_add(a, b, c, d, za=o1, zb=o2)),
        ("cg_share_mul_public", 32, lambda: cg.cg_share_mul_public(a, b, 12345, za=o1, zb=o2)),
        ("cg_reconstruct", 32, lambda: cg.cg_reconstruct(a, b, c, out=o1)),
    ]:
        ms = _timed(torch, fn, warm=2, iters=5)
        gbs = nbytes * n / (ms * 1e-3) / 1e9
        rows.append({"name": name, "words": n, "ms": round(ms, 4), "GB_per_s": round(gbs, 1),
                     "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)})
    out["streaming"] = rows
    del a, b, c, d, o1, o2
    # ---- HBM-bound fully connected layers: warm = the same operands every launch (they stay in the last-level
    # cache), cold = rotating through enough distinct operand sets to exceed it
    rows = []
    fcs = [L for L in wl.config_layers(4) if L.kind == "matmul"] + [L for L in wl.config_layers(5) if L.kind == "matmul"]
    lead_ops = [_rnd(torch, (2048, 2048), 900 + i) for i in range(4)]
    lead_z = torch.empty((2048, 2048), dtype=torch.int64, device="cuda")

    def lead():   # about 4 ms of GPU work (see _timed)
        for _ in range(8):
            cg.cg_share_matmul(*lead_ops, z_i=lead_z)
    for L in fcs:
        nbytes = L.algorithmic_bytes
        sets = max(2, int(2 * LAST_LEVEL_CACHE_BYTES // nbytes) + 1)
        sets = min(sets, 160)
        pool = [[_rnd(torch, L.x_shape, 10 * i + 1), _rnd(torch, L.x_shape, 10 * i + 2),
                 _rnd(torch, L.w_shape, 10 * i + 3), _rnd(torch, L.w_shape, 10 * i + 4)] for i in range(sets)]
        z = torch.empty(L.z_shape, dtype=torch.int64, device="cuda")
        warm_ms = _timed(torch, lambda: cg.cg_share_matmul(*pool[0], z_i=z), warm=3, iters=20, lead=lead)
        it = [0]

        def cold():
            cg.cg_share_matmul(*pool[it[0] % sets], z_i=z)
            it[0] += 1
        cold_ms = _timed(torch, cold, warm=sets, iters=sets, lead=lead)
        rows.append({"name": L.name, "gemm": list(L.gemm), "algorithmic_bytes": nbytes, "operand_sets": sets,
                     "warm_us": round(warm_ms * 1e3, 2), "cold_us": round(cold_ms * 1e3, 2),
                     "hbm_time_us": round(nbytes / (HBM_PEAK_GBS * 1e9) * 1e6, 2),
                     "cold_GB_per_s": round(nbytes / (cold_ms * 1e-3) / 1e9, 1)})
        del pool, z
    out["fc_warm_cold"] = rows
    return out


def measure_extras(torch, cg, wl, config_layers):
    """Rows outside the timed step: every figure is the mean of 10 launches after 3 warm-ups, HIP events on the
    launch stream, uniform random words resident in HBM."""
    def rnd(shape, seed):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        return torch.randint(-2 ** 63, 2 ** 63 - 1, tuple(shape), dtype=torch.int64, device="cuda", generator=g)

    def timed(fn, warm=3, iters=10):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters

    def row(name, mnk, ms):
        tops = 2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * mnk / (ms * 1e-3) / 1e12
        return {"name": name, "ms": round(ms, 4), "ring_macs_per_s": 3.0 * mnk / (ms * 1e-3),
                "int8_tops": round(tops, 1), "frac_of_peak": round(tops / INT8_PEAK_TOPS, 4)}

    out = {"square_products": [], "fig1_conv_shapes": [], "backward_config4": [], "streaming": []}
    for M, N, K in [(1024, 1024, 1024), (4096, 4096, 4096), (8192, 8192, 2048), (8192, 8192, 8192)]:
        ops = [rnd((M, K), 1), rnd((M, K), 2), rnd((N, K), 3), rnd((N, K), 4)]
        z = torch.empty((M, N), dtype=torch.int64, device="cuda")
        out["square_products"].append(row(f"matmul {M}x{N}x{K}", M * N * K, timed(lambda: cg.cg_share_matmul(*ops, z_i=z))))
        del ops, z
    # the paper's embedding (16-bit blocks in float64, float64 matrix instruction) against the int8 route, same product
    out["limb_choice"] = []
    for M, N, K in [(2048, 2048, 2048), (4096, 4096, 4096)]:
        ops = [rnd((M, K), 1), rnd((M, K), 2), rnd((N, K), 3), rnd((N, K), 4)]
        z = torch.empty((M, N), dtype=torch.int64, device="cuda")
        ms8 = timed(lambda: cg.cg_share_matmul(*ops, z_i=z))
        ms64 = timed(lambda: cg.cg_share_matmul_f64limb(*ops, z_i=z), warm=1, iters=3)
        out["limb_choice"].append({
            "name": f"matmul {M}x{N}x{K}", "int8_digits_ms": round(ms8, 4), "float64_blocks_ms": round(ms64, 4),
            "float64_blocks_ring_macs_per_s": 3.0 * M * N * K / (ms64 * 1e-3),
            "float64_blocks_tflops": round(2.0 * 20 * M * N * K / (ms64 * 1e-3) / 1e12, 1),
            "int8_over_float64": round(ms64 / ms8, 2)})
        del ops, z
    # shapes of the paper's Fig. 1 (its times are whole-protocol times on three V100s over a LAN: context only)
    fig1 = [("11x11 3->64 s4 p2", (1, n, n, 3), (64, 11, 11, 3), 4, 2) for n in (64, 128, 256, 512)]
    fig1 += [("11x11 3->64 s4 p2 on 32x32x3", (b, 32, 32, 3), (64, 11, 11, 3), 4, 2) for b in (32, 128, 512)]
    fig1 += [("3x3 512->512 p1", (1, n, n, 512), (512, 3, 3, 512), 1, 1) for n in (8, 16, 32, 64)]
    for name, xs, ws, st, pd in fig1:
        ops = [rnd(xs, 1), rnd(xs, 2), rnd(ws, 3), rnd(ws, 4)]
        zs = cg.conv_out_shape(xs, ws, (st, st), (pd, pd))
        z = torch.empty(zs, dtype=torch.int64, device="cuda")
        ms = timed(lambda: cg.cg_share_conv2d(*ops, stride=(st, st), pad=(pd, pd), z_i=z))
        out["fig1_conv_shapes"].append(row(f"{name}, input {xs[0]}x{xs[1]}x{xs[2]}x{xs[3]}",
                                           zs[0] * zs[1] * zs[2] * ws[0] * ws[1] * ws[2] * ws[3], ms))
        del ops, z
    # forward / input-gradient / weight-gradient products of a configuration's convolution layers
    def backward_rows(layers, key):
        tot = {"forward": 0.0, "dgrad": 0.0, "wgrad": 0.0}
        strided = {"forward": 0.0, "dgrad": 0.0}
        mnk = mnk_strided = 0
        for li, L in enumerate(layers):
            if L.kind != "conv":
                continue
            xs, ws, zs = L.x_shape, L.w_shape, L.z_shape
            g, w, x = [rnd(zs, 1), rnd(zs, 2)], [rnd(ws, 3), rnd(ws, 4)], [rnd(xs, 5), rnd(xs, 6)]
            dx, dw = torch.empty(xs, dtype=torch.int64, device="cuda"), torch.empty(ws, dtype=torch.int64, device="cuda")
            z = torch.empty(zs, dtype=torch.int64, device="cuda")
            st, pd = (L.stride, L.stride), (L.pad, L.pad)
            fwd = timed(lambda: cg.cg_share_conv2d(*x, *w, stride=st, pad=pd, z_i=z)) * L.repeat
            dg = timed(lambda: cg.cg_share_conv2d_dgrad(*g, *w, xs, stride=st, pad=pd, dx_i=dx)) * L.repeat
            tot["forward"] += fwd
            tot["dgrad"] += dg
            tot["wgrad"] += timed(lambda: cg.cg_share_conv2d_wgrad(*g, *x, ws, stride=st, pad=pd, dw_i=dw)) * L.repeat
            mnk += L.mnk * L.repeat
            if L.stride > 1 and li > 0:      # the first layer's input gradient is never needed
                strided["forward"] += fwd
                strided["dgrad"] += dg
                mnk_strided += L.mnk * L.repeat
            del g, w, x, dx, dw, z
        for k, ms in tot.items():
            out[key].append(row(f"{k}, all convolution layers", mnk, ms))
        if mnk_strided:
            for k, ms in strided.items():
                out[key].append(row(f"{k}, strided layers after the first", mnk_strided, ms))

    backward_rows(config_layers, "backward_config4")
    out["backward_config5"] = []
    backward_rows(wl.config_layers(5), "backward_config5")
    # The multiplication protocol's message z_i + alpha_i for one large convolution (32x32x128 -> 128, batch 32):
    # product then reshare pass, against the product folded into an output that already holds alpha_i (which
    # depends on no data and can be produced while the party waits for the previous round's messages).
    xs, ws = (32, 32, 32, 128), (128, 3, 3, 128)
    x, w = [rnd(xs, 1), rnd(xs, 2)], [rnd(ws, 3), rnd(ws, 4)]
    z = torch.empty(cg.conv_out_shape(xs, ws, (1, 1), (1, 1)), dtype=torch.int64, device="cuda")
    ka, kb = bytes(range(16)), bytes(range(16, 32))
    nz = z.numel()
    out["reshare_in_fold"] = [
        {"name": "cg_share_conv2d", "ms": round(timed(lambda: cg.cg_share_conv2d(*x, *w, pad=(1, 1), z_i=z)), 4)},
        {"name": "cg_share_conv2d + cg_reshare", "ms": round(timed(lambda: cg.cg_reshare(
            cg.cg_share_conv2d(*x, *w, pad=(1, 1), z_i=z), ka, kb, 1, 0, out=z)), 4)},
        {"name": "cg_zero_share + cg_share_conv2d_acc", "ms": round(timed(lambda: cg.cg_share_conv2d_acc(
            *x, *w, cg.cg_zero_share(ka, kb, 1, 0, nz, out=z.view(-1)).view(z.shape), pad=(1, 1))), 4)},
        {"name": "cg_share_conv2d_acc alone (alpha_i produced earlier)", "ms": round(timed(
            lambda: cg.cg_share_conv2d_acc(*x, *w, z, pad=(1, 1))), 4)},
    ]
    del x, w, z
    # HBM- and ALU-bound kernels next to the products; n words per stream, beyond the 256 MB last-level cache
    n = 1 << 26
    a, b, c, d = (rnd((n,), s) for s in (1, 2, 3, 4))
    o1, o2 = torch.empty_like(a), torch.empty_like(a)
    k0, k1 = bytes(range(16)), bytes(range(16, 32))
    for name, nbytes, fn in [
        ("cg_share_add", 48, lambda: cg.cg_share_add(a, b, c, d, za=o1, zb=o2)),
        ("cg_share_mul_public", 32, lambda: cg.cg_share_mul_public(a, b, 12345, za=o1, zb=o2)),
        ("cg_reconstruct", 32, lambda: cg.cg_reconstruct(a, b, c, out=o1)),
        ("cg_share_mul", 40, lambda: cg.cg_share_mul(a, b, c, d, z_i=o1)),
        ("cg_reshare", 16, lambda: cg.cg_reshare(a, k0, k1, 1, 0, out=o1)),
        ("cg_trunc1_local (message, mask)", 24, lambda: cg.cg_trunc1_local(a, b, k1, k0, 1, 0, 16, k1, 2, out=o1)),
    ]:
        ms = timed(fn, warm=2, iters=5)
        out["streaming"].append({"name": name, "words": n, "ms": round(ms, 4), "words_per_s": n / (ms * 1e-3),
                                 "GB_per_s": round(nbytes * n / (ms * 1e-3) / 1e9, 1)})
    # One party's local work for the sign bit of n words (carry-save step + 64-bit parallel-prefix adder on
    # binary shares: 8 rounds of AND gates, each followed by the PRF blinding), message passing excluded.
    n = 1 << 24
    x0, x1, t0, t1, p0, p1, g0, g1 = (rnd((n,), s) for s in range(11, 19))
    k0, k1 = bytes(range(16)), bytes(range(16, 32))

    def msb_local():
        cg.cg_bshare_xor(x0, x1, t0, t1, za=p0, zb=p1)              # A ^ C, B ^ C, S = A ^ B ^ C: three XOR gates
        cg.cg_bshare_xor(x1, x0, t1, t0, za=g0, zb=g1)
        cg.cg_bshare_xor(p0, p1, g0, g1, za=t0, zb=t1)
        cg.cg_breshare(cg.cg_bshare_and(p0, p1, g0, g1, z_i=t0), k0, k1, 3, 0, out=t0)          # majority
        cg.cg_bshare_xor(t0, t1, x0, x1, za=g0, zb=g1)              # ... ^ C, then P0 = S ^ T
        cg.cg_bshare_xor(g0, g1, p0, p1, za=p0, zb=p1)
        cg.cg_breshare(cg.cg_bshare_and(p0, p1, g0, g1, z_i=g0), k0, k1, 3, n, out=g0)          # G = S & T
        first = 2 * n
        for stage, shift in enumerate((1, 2, 4, 8, 16, 32)):
            last = stage == 5
            cg.cg_bshare_prefix_stage(p0, p1, g0, g1, shift, last, p_out=None if last else t0, g_out=t1)
            cg.cg_breshare(t1, k0, k1, 3, first, out=g0)
            if not last:
                cg.cg_breshare(t0, k0, k1, 3, first + n, out=p0)
            first += 2 * n
        cg.cg_bshare_xor(p0, p1, g0, g1, za=t0, zb=t1)              # sum = P0 ^ (G << 1)

    ms = timed(msb_local, warm=2, iters=5)
    out["sign_bit_circuit_local"] = [{"name": "word-parallel adder: one party's local steps", "words": n,
                                      "ms": round(ms, 4), "words_per_s": n / (ms * 1e-3),
                                      "and_rounds": 8, "prf_blinded_words_per_input_word": 13}]

    # The same for the circuit pruned to the sign bit on bit planes: two transposes, 64-plane gates for the
    # carry-save step and the first generate word, then the carry tree on 32, 16, 8, 4, 2, 1 planes.
    m = n // 64
    pl = [torch.empty((64, m), dtype=torch.int64, device="cuda") for _ in range(8)]
    a0, a1, s0, s1, c0, c1, q0, q1 = pl

    def msb_local_sliced():
        cg.cg_bit_transpose64(x0, out=a0)
        cg.cg_bit_transpose64(x1, out=a1)
        # carry-save cell on the three sharings x_0, x_1, x_2, each with a single non-zero share: of the six pair
        # components of party i only A's first (x_i) and B's second (x_{i+1}) are not zero; carry blinded
        cg.cg_bshare_csa(a0, None, None, a1, None, None, s_i=q0, s_ip1=q1, carry_i=s0)
        cg.cg_breshare(s0, k0, k1, 4, 0, out=s0)
        # half-adder cell: propagate pair and generate share, generate blinded
        cg.cg_bshare_half_adder(q0, q1, s0, s1, p_i=c0, p_ip1=c1, g_i=q0)
        cg.cg_breshare(q0, k0, k1, 4, n, out=q0)
        first, P, G = 2 * n, (c0, c1), (q0, q1)
        while P[0].shape[0] > 1:
            last = P[0].shape[0] == 2
            p_loc, g_loc = cg.cg_bshare_carry_level(P[0], P[1], G[0], G[1], last)
            cg.cg_breshare(g_loc, k0, k1, 4, first, out=g_loc)
            first += g_loc.numel()
            if not last:
                cg.cg_breshare(p_loc, k0, k1, 4, first, out=p_loc)
                first += p_loc.numel()
            P = (g_loc, g_loc) if last else (p_loc, p_loc)   # the second component would arrive from the next party
            G = (g_loc, g_loc)
        cg.cg_bits_unpack(G[0][0], n, out=x0)                       # back to one word per element

    ms = timed(msb_local_sliced, warm=2, iters=5)
    out["sign_bit_circuit_local"].append({"name": "pruned circuit on bit planes: one party's local steps", "words": n,
                                          "ms": round(ms, 4), "words_per_s": n / (ms * 1e-3), "and_rounds": 8,
                                          "prf_blinded_words_per_input_word": round(253 / 64, 2)})
    return out


def main() -> int:
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one party's local product); "
              f"--gpus {args.gpus} is not supported. Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2104_10949_amd import binding as cg
    from paper_2104_10949_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback for the product path", file=sys.stderr)
        return 3
    cg.lib()  # fails loudly if libcg.so has not been built
    torch.cuda.set_device(0)

    layers = wl.config_layers(args.config)
    host_ops, dev_ops, outs = [], [], []
    for li, L in enumerate(layers):
        ops = wl.party_operands(L, wl.layer_seed(args.config, li))
        host_ops.append(ops)
        dev_ops.append([cg.to_device(a) for a in ops])
        outs.append(torch.empty(L.z_shape, dtype=torch.int64, device="cuda"))
    torch.cuda.synchronize()

    # Route per layer.  The library offers every product with and without caller-supplied scratch memory (the
    # *_ws entry points: operands split into digit planes once, then a product kernel without split work); its
    # own rule of thumb (cg_share_*_prefers_workspace) says which one to call for a shape.  The scratch buffer
    # is allocated here, once, outside the timed region, like the operands; --plain times the plain calls only.
    def prefers_ws(L) -> bool:
        if args.plain:
            return False
        if L.kind == "conv":
            return cg.cg_share_conv2d_prefers_workspace(L.x_shape, L.w_shape, (L.stride, L.stride), (L.pad, L.pad))
        return cg.cg_share_matmul_prefers_workspace(*L.gemm)

    def ws_bytes(L) -> int:
        if L.kind == "conv":
            return cg.cg_share_conv2d_workspace_bytes(L.x_shape, L.w_shape, (L.stride, L.stride), (L.pad, L.pad))
        return cg.cg_share_matmul_workspace_bytes(*L.gemm)
    use_ws = [prefers_ws(L) for L in layers]
    scratch = torch.empty(max([ws_bytes(L) for L, u in zip(layers, use_ws) if u] + [16]), dtype=torch.uint8,
                          device="cuda")

    def run_layer(li: int, plain: bool = False) -> None:
        L = layers[li]
        for _ in range(L.repeat):
            if L.kind == "conv":
                if use_ws[li] and not plain:
                    cg.cg_share_conv2d_ws(*dev_ops[li], scratch, stride=(L.stride, L.stride), pad=(L.pad, L.pad),
                                          z_i=outs[li])
                else:
                    cg.cg_share_conv2d(*dev_ops[li], stride=(L.stride, L.stride), pad=(L.pad, L.pad), z_i=outs[li])
            elif use_ws[li] and not plain:
                cg.cg_share_matmul_ws(*dev_ops[li], scratch, z_i=outs[li])
            else:
                cg.cg_share_matmul(*dev_ops[li], z_i=outs[li])

    def step(plain: bool = False) -> None:
        for li in range(len(layers)):
            run_layer(li, plain)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps

    # spread of single steps (separate pass, one event pair per step)
    n_single = min(args.steps, 50)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_single + 1)]
    marks[0].record()
    for i in range(n_single):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    single = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(n_single))
    step_spread = {"median_ms": round(single[len(single) // 2], 5), "min_ms": round(single[0], 5),
                   "max_ms": round(single[-1], 5)}

    total_mnk = sum(L.mnk * L.repeat for L in layers)
    launches = sum(L.repeat for L in layers)
    value = 3.0 * total_mnk / (ms_per_step * 1e-3)
    # the same step through the plain entry points only (no scratch memory anywhere)
    plain_ms_per_step = ms_per_step if not any(use_ws) else _timed(torch, lambda: step(True), warm=3,
                                                                    iters=max(10, args.steps // 4))

    # Per-layer durations of the share-product kernel, HIP events on the launch stream,
    # measured right after the timed region on the same buffers.
    per_layer_ms = []
    reps = max(3, min(args.steps, 10))
    lead_steps = max(1, min(100, int(1.0 / max(ms_per_step, 1e-3)) + 1))   # about a millisecond of queued work
    for li, L in enumerate(layers):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(lead_steps):   # keeps the GPU busy while the host enqueues the timed launches (see _timed)
            step()
        a.record()
        for _ in range(reps):
            run_layer(li)
        b.record()
        torch.cuda.synchronize()
        per_layer_ms.append(a.elapsed_time(b) / (reps * L.repeat))
    kernel_ms_sum = sum(ms * L.repeat for ms, L in zip(per_layer_ms, layers))

    def mfma_ceiling(random_bytes: bool, k64: bool = True) -> float:
        """int8 TOP/s of a register-only MFMA loop on all compute units (2 waves per SIMD): the 16x16x64 form the
        share-product kernel issues (k64) or the 32x32x32 form."""
        import ctypes
        import numpy as np
        from paper_2104_10949_amd import build as hip_build
        probe = ctypes.CDLL(hip_build.PROBE_LIB)
        fn = probe.cg_probe_mfma16_rate if k64 else probe.cg_probe_mfma_rate
        fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 3 + [ctypes.c_void_p]
        fn.restype = ctypes.c_int
        if random_bytes:
            ops = cg.to_device(wl.draw_ring((8192,), 12345))
        else:
            ops = cg.to_device(np.full((8192,), 0x0101010101010101, dtype=np.uint64))
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        sink = torch.empty(n_cu * 512, dtype=torch.int32, device="cuda")
        # (long enough that the kernel's start-up, about 0.4 ms for the 16x16x64 loop, is under 5 % of the run)
        iters, stream = 20000, torch.cuda.current_stream().cuda_stream

        def launch():
            rc = fn(ops.data_ptr(), sink.data_ptr(), n_cu, 2, iters, stream)
            if rc != 0:
                raise RuntimeError(f"MFMA probe returned {rc}")
        launch()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        launch()
        b.record()
        torch.cuda.synchronize()
        macs = n_cu * 8 * iters * (32 * 16384.0 if k64 else 8 * 32768.0)
        return 2.0 * macs / (a.elapsed_time(b) * 1e-3) / 1e12

    def mfma_f64_ceiling() -> float:
        """float64 MAC/s of a register-only v_mfma_f64_16x16x4_f64 loop on all compute units, with
        random 16-bit integer operands (the paper's limb width)."""
        import ctypes
        import numpy as np
        from paper_2104_10949_amd import build as hip_build
        probe = ctypes.CDLL(hip_build.PROBE_LIB)
        probe.cg_probe_mfma_f64_rate.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 3 + [ctypes.c_void_p]
        probe.cg_probe_mfma_f64_rate.restype = ctypes.c_int
        limbs = (wl.draw_ring((8192,), 54321) & np.uint64(0xFFFF)).astype(np.float64)
        ops = torch.from_numpy(limbs).cuda()
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        sink = torch.empty(n_cu * 512, dtype=torch.float64, device="cuda")
        iters, stream = 4000, torch.cuda.current_stream().cuda_stream

        def launch():
            rc = probe.cg_probe_mfma_f64_rate(ops.data_ptr(), sink.data_ptr(), n_cu, 2, iters, stream)
            if rc != 0:
                raise RuntimeError(f"cg_probe_mfma_f64_rate returned {rc}")
        launch()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        launch()
        b.record()
        torch.cuda.synchronize()
        return n_cu * 8 * iters * 8 * 1024.0 / (a.elapsed_time(b) * 1e-3)

    if args.calib_copy_mib > 0:
        n = args.calib_copy_mib * (1 << 20) // 8
        src = torch.arange(n, dtype=torch.int64, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)  # reads n*8 bytes, writes n*8 bytes
        torch.cuda.synchronize()

    int8_ops_per_step = 2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * total_mnk
    achieved_tops = int8_ops_per_step / (kernel_ms_sum * 1e-3) / 1e12
    big = max(range(len(layers)), key=lambda i: layers[i].mnk)
    big_tops = 2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * layers[big].mnk / (per_layer_ms[big] * 1e-3) / 1e12
    roofline = {
        "bound": "mfma", "kernel": "share_gemm_kernel (int8 MFMA, i32 accumulate)",
        "achieved": round(achieved_tops, 2), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
        "frac": round(achieved_tops / INT8_PEAK_TOPS, 4),
        "launches_per_step": launches,
        "avg_launch_ms": round(kernel_ms_sum / launches, 5),
        "ops_per_launch": int8_ops_per_step / launches,
        "largest_layer": {"name": layers[big].name, "gemm": list(layers[big].gemm),
                          "ms": round(per_layer_ms[big], 5), "achieved": round(big_tops, 2),
                          "frac": round(big_tops / INT8_PEAK_TOPS, 4)},
        # every layer whose M*N*K equals the largest one's (several layers of the VGG-shaped stack tie)
        "largest_layers": [{"name": L.name, "gemm": list(L.gemm), "ms": round(ms, 5),
                            "frac": round(2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * L.mnk / (ms * 1e-3) / 1e12
                                          / INT8_PEAK_TOPS, 4)}
                           for L, ms in zip(layers, per_layer_ms) if L.mnk == layers[big].mnk],
        # the same layers as one figure: their int8 ops over their summed time
        "largest_layers_together": (lambda ties: {
            "layers": len(ties), "ms": round(sum(ms for _, ms in ties), 5),
            "frac": round(sum(2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * L.mnk for L, _ in ties)
                          / (sum(ms for _, ms in ties) * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)})(
            [(L, ms) for L, ms in zip(layers, per_layer_ms) if L.mnk == layers[big].mnk]),
        "traffic": PROFILED_TRAFFIC_CONFIG4 if args.config == WORKLOAD_CONFIG else None,
    }
    # Per layer: measured time against t_roof = max(int8 ops / peak, algorithmic bytes / HBM peak) and the larger term.
    per_layer = []
    for L, ms in zip(layers, per_layer_ms):
        t_mfma = 2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * L.mnk / (INT8_PEAK_TOPS * 1e12)
        t_hbm = L.algorithmic_bytes / 8e12
        per_layer.append({"name": L.name, "gemm": list(L.gemm), "repeat": L.repeat, "us": round(ms * 1e3, 2),
                          "t_roof_us": round(max(t_mfma, t_hbm) * 1e6, 2), "bound": "mfma" if t_mfma >= t_hbm else "hbm",
                          "frac_of_roof": round(max(t_mfma, t_hbm) / (ms * 1e-3), 4)})
    roofline["layers"] = per_layer
    if not args.no_mfma_probe:
        # register-only MFMA loop on the same box: what the matrix cores sustain at the power limit
        peak_const, peak_random = mfma_ceiling(False), mfma_ceiling(True)
        roofline["measured_mfma_loop"] = {
            "instruction": "v_mfma_i32_16x16x64_i8",
            "constant_operands": round(peak_const, 1), "random_operands": round(peak_random, 1), "unit": "TOP/s",
            "random_operands_32x32x32_form": round(mfma_ceiling(True, k64=False), 1),
            "frac_of_random_operand_loop": round(achieved_tops / peak_random, 4),
            "largest_layer_frac_of_random_operand_loop": round(big_tops / peak_random, 4)}
        # Limb-choice check: the paper's embedding (four 16-bit limbs in float64, 10 limb products per ring
        # product) would need 20 float64 MACs per (m,n,k) for the fused two-product form; even at the measured
        # float64 MFMA issue rate that caps the effective ring MAC/s below what the int8 kernel delivers.
        f64_macs = mfma_f64_ceiling()
        roofline["fp64_limb_route_upper_bound"] = {
            "measured_f64_mfma_macs_per_s": f64_macs, "f64_macs_per_mnk": 20,
            "effective_ring_macs_per_s_at_100pct": 3.0 * f64_macs / 20.0,
            "int8_kernel_vs_bound": round(value / (3.0 * f64_macs / 20.0), 2)}

    if args.layers:
        for L, ms in zip(layers, per_layer_ms):
            m, n, k = L.gemm
            tops = 2.0 * DIGIT_MACS_PER_RING_MAC_TRIPLE * L.mnk / (ms * 1e-3) / 1e12
            print(f"{L.name:28s} M={m:7d} N={n:5d} K={k:5d} x{L.repeat}  {ms * 1e3:9.1f} us  "
                  f"{3.0 * L.mnk / (ms * 1e-3):.3e} ringMAC/s  {tops:7.1f} TOP/s ({100 * tops / INT8_PEAK_TOPS:4.1f}%)  "
                  f"{L.algorithmic_bytes / (ms * 1e-3) / 1e9:7.0f} GB/s", file=sys.stderr)

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ring_oracle as ro  # the benchmark's cpu_baseline leg only
        done_mnk, t_cpu, covered, passes = 0, 0.0, [], 0
        # whole passes over the workload until about 10 s of CPU work are collected (one pass at least,
        # cut short at the budget)
        while t_cpu < args.cpu_min_s and t_cpu <= args.cpu_budget_s:
            for li, L in enumerate(layers):
                if t_cpu > args.cpu_budget_s:
                    break
                t0 = time.perf_counter()
                if L.kind == "conv":
                    ro.party_conv2d(*host_ops[li], (L.stride, L.stride), (L.pad, L.pad))
                else:
                    ro.party_matmul(*host_ops[li])
                t_cpu += time.perf_counter() - t0
                done_mnk += L.mnk
                if passes == 0:
                    covered.append(L.name)
            passes += 1
        # the same oracle on ONE thread, on configuration 1 (256^3, the three parties' products)
        c1 = wl.config_layers(1)[0]
        ops1 = wl.party_operands(c1, wl.layer_seed(1, 0))
        all_threads = ro.num_threads()
        ro.set_num_threads(1)
        t0, n1 = time.perf_counter(), 0
        while time.perf_counter() - t0 < 1.0:
            ro.party_matmul(*ops1)
            n1 += 1
        t_one = time.perf_counter() - t0
        ro.set_num_threads(all_threads)
        single_thread = {"value": 3.0 * c1.mnk * n1 / t_one, "unit": "ring MAC/s", "cores": 1,
                         "sample": f"{n1} party products of config 1 (matmul 256^3) on one thread"}
        cpu = {"value": 3.0 * done_mnk / t_cpu, "unit": "ring MAC/s", "cores": ro.num_threads(),
               "single_thread_config1": single_thread,
               "kind": "oracle", "seconds": round(t_cpu, 2),
               "sample": (f"{passes} pass(es) over {len(covered)} of {len(layers)} layers of config {args.config} at "
                          f"full size, one party ({covered[0]} .. {covered[-1]}), {3 * done_mnk:.3e} ring MACs")}

    rows = None if args.no_rows else measure_rows(torch, cg, wl, args.config)
    extras = measure_extras(torch, cg, wl, layers) if args.extras else None

    out = {
        "metric": METRIC, "value": value, "unit": "ring MAC/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "step_spread": step_spread,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "dtype_note": "u64 ring elements as 8 signed-byte digits on int8 MFMA, i32 accumulate, exact",
        "data": "synthetic",
        "config": {"workload": {1: "config 1: share matmul 256^3",
                                2: "config 2: FC stack 784-128-128-10, batch 128",
                                3: "config 3: small CNN conv layers, batch 128, 32x32x3",
                                4: "config 4: VGG16-shaped 13 conv + 3 FC on shares, batch 32, 64x64x3",
                                5: "config 5: ResNet-50-shaped 53 conv + 1 FC on shares, batch 8, 224x224x3"}[args.config],
                   "layers": launches, "ring_macs_per_step": 3 * total_mnk,
                   "layers_on_the_scratch_memory_route": [L.name for L, u in zip(layers, use_ws) if u],
                   "scratch_bytes": int(scratch.numel()),
                   "plain_entry_points_only": {"ms_per_step": plain_ms_per_step,
                                               "ring_macs_per_s": 3.0 * total_mnk / (plain_ms_per_step * 1e-3)},
                   "parties_timed": 1, "fixed_point_bits": wl.FRAC_BITS},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "rows": rows,
        "extras": extras,
        "paper_context": "CryptGPU reports no isolated local-product rate; derived from its Fig. 1 "
                         "(3 V100, LAN, whole protocol): about 6e9-1.1e10 effective ring MAC/s",
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
