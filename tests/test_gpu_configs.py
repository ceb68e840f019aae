"""Full-size GPU parity on the five benchmark configurations: every output element of every
layer, one party, bit for bit against the CPU oracle, in the launch configuration bench.py times."""
import numpy as np
import pytest

from tests.gpu_util import first_mismatch, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import ring_oracle as ro
    from paper_2104_10949_amd import binding as cg
    from paper_2104_10949_amd import workloads as wl
    cg.lib()
    return cg, ro, wl


def check_layer(cg, ro, wl, cfg, li, L):
    """Both routes (allocation-free entry point, and the *_ws entry point bench.py times) against the oracle."""
    say(f"config {cfg} layer {li} {L.name} gemm={L.gemm}")
    ops = wl.party_operands(L, wl.layer_seed(cfg, li))
    dev = [cg.to_device(a) for a in ops]
    sp = ((L.stride, L.stride), (L.pad, L.pad))
    if L.kind == "conv":
        z = cg.cg_share_conv2d(*dev, stride=sp[0], pad=sp[1])
        ws = torch.empty(cg.cg_share_conv2d_workspace_bytes(L.x_shape, L.w_shape, *sp) // 8 + 2,
                         dtype=torch.int64, device="cuda")
        z2 = cg.cg_share_conv2d_ws(*dev, ws, stride=sp[0], pad=sp[1])
        want = ro.party_conv2d(*ops, *sp)
    else:
        z = cg.cg_share_matmul(*dev)
        ws = torch.empty(cg.cg_share_matmul_workspace_bytes(*L.gemm) // 8 + 2, dtype=torch.int64, device="cuda")
        z2 = cg.cg_share_matmul_ws(*dev, ws)
        want = ro.party_matmul(*ops)
    torch.cuda.synchronize()
    for route, out in (("direct", z), ("workspace", z2)):
        got = cg.to_host(out)
        assert got.shape == tuple(L.z_shape)
        msg = first_mismatch(got, want)
        assert not msg, f"config {cfg} {L.name} route {route}: {msg}"


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_config_every_layer_bit_exact(env, cfg):
    cg, ro, wl = env
    for li, L in enumerate(wl.config_layers(cfg)):
        check_layer(cg, ro, wl, cfg, li, L)


@pytest.mark.parametrize("cfg", [4, 5])
def test_config_backward_products_every_layer_bit_exact(env, cfg):
    """Input and weight gradients of every convolution layer of the VGG16-shaped and the ResNet-50-shaped
    configuration at full size (the shapes bench.py --extras times; the second brings the strided 3x3 layers, the
    strided 1x1 projections and the 7x7 stem), one party, every element against the oracle."""
    cg, ro, wl = env
    for li, L in enumerate(wl.config_layers(cfg)):
        if L.kind != "conv":
            continue
        say(f"config {cfg} backward, layer {li} {L.name}")
        seed = wl.layer_seed(cfg, li) + 500
        g = [wl.draw_ring(L.z_shape, seed), wl.draw_ring(L.z_shape, seed + 1)]
        w = [wl.draw_ring(L.w_shape, seed + 2), wl.draw_ring(L.w_shape, seed + 3)]
        x = [wl.draw_ring(L.x_shape, seed + 4), wl.draw_ring(L.x_shape, seed + 5)]
        dg, dw, dx = ([cg.to_device(a) for a in t] for t in (g, w, x))
        sp = ((L.stride, L.stride), (L.pad, L.pad))
        got_dx = cg.cg_share_conv2d_dgrad(*dg, *dw, L.x_shape, stride=sp[0], pad=sp[1])
        got_dw = cg.cg_share_conv2d_wgrad(*dg, *dx, L.w_shape, stride=sp[0], pad=sp[1])
        torch.cuda.synchronize()
        msg = first_mismatch(cg.to_host(got_dx), ro.party_conv2d_dgrad(*g, *w, L.x_shape, *sp))
        assert not msg, f"{L.name} input gradient: {msg}"
        msg = first_mismatch(cg.to_host(got_dw), ro.party_conv2d_wgrad(*g, *x, L.w_shape, *sp))
        assert not msg, f"{L.name} weight gradient: {msg}"


def test_config4_step_replayed_from_a_hip_graph_is_bit_exact(env):
    """A caller may capture the 16-layer step once and replay it (measured: no faster than host launches here,
    the GPU is never idle between them); every replay must give the oracle's outputs, also with eager work and
    fresh inputs between replays."""
    cg, ro, wl = env
    layers = wl.config_layers(4)
    host = [list(wl.party_operands(L, wl.layer_seed(4, li))) for li, L in enumerate(layers)]
    dev = [[cg.to_device(a) for a in ops] for ops in host]
    outs = [torch.empty(L.z_shape, dtype=torch.int64, device="cuda") for L in layers]

    def step():
        for L, d, z in zip(layers, dev, outs):
            if L.kind == "conv":
                cg.cg_share_conv2d(*d, stride=(L.stride, L.stride), pad=(L.pad, L.pad), z_i=z)
            else:
                cg.cg_share_matmul(*d, z_i=z)

    def oracle_outputs():
        return [ro.party_conv2d(*ops, (L.stride, L.stride), (L.pad, L.pad)) if L.kind == "conv"
                else ro.party_matmul(*ops) for L, ops in zip(layers, host)]

    say("config 4: capture the step into a HIP graph")
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    want = oracle_outputs()
    for rep in range(3):
        say(f"config 4: graph replay {rep}")
        for z in outs:
            z.fill_(0x5A5A5A5A5A5A5A5A)          # eager work between replays; stale outputs would show
        if rep == 2:
            # new activations for the two largest layers, same buffers: the graph must read them afresh
            for li in (1, 3):
                for j in (0, 1):
                    host[li][j] = wl.draw_ring(layers[li].x_shape, 4242 + 10 * li + j)
                    dev[li][j].copy_(torch.from_numpy(host[li][j].view(np.int64)))
            want = oracle_outputs()
        graph.replay()
        torch.cuda.synchronize()
        for L, z, w in zip(layers, outs, want):
            msg = first_mismatch(cg.to_host(z), w)
            assert not msg, f"replay {rep} {L.name}: {msg}"


def test_config3_alternate_reading_conv2_at_16x16(env):
    cg, ro, wl = env
    L = wl.config3(alt=True)[1]
    check_layer(cg, ro, wl, 3, 11, L)


def test_config2_all_three_parties_open_to_the_fixed_point_product(env):
    """FC stack, first layer: the three parties' outputs open to enc(X) enc(W)^T and decode to
    the real product within 2^-12."""
    cg, ro, wl = env
    L = wl.config_layers(2)[0]
    seed = wl.layer_seed(2, 0)
    t = wl.FRAC_BITS
    say("config 2 fc1: three parties, open, decode")
    X, W = wl.draw_reals(L.x_shape, L.x_dist, seed), wl.draw_reals(L.w_shape, L.w_dist, seed + 1)
    ex, ew = ro.encode(X, t), ro.encode(W, t)
    sx = ro.share(ex, wl.draw_ring(ex.shape, seed + 2), wl.draw_ring(ex.shape, seed + 3))
    sw = ro.share(ew, wl.draw_ring(ew.shape, seed + 4), wl.draw_ring(ew.shape, seed + 5))
    dx, dw = [cg.to_device(s) for s in sx], [cg.to_device(s) for s in sw]
    z = [cg.cg_share_matmul(dx[i], dx[(i + 1) % 3], dw[i], dw[(i + 1) % 3]) for i in range(3)]
    opened = cg.to_host(cg.cg_reconstruct(*z))
    assert np.array_equal(opened, ro.matmul(ex, ew))
    assert np.max(np.abs(ro.decode(opened, 2 * t) - ro.decode(ex, t) @ ro.decode(ew, t).T)) <= 2.0 ** -12


def test_protocol_steps_replayed_from_a_hip_graph_match_eager_runs(env):
    """The entry points around the products (zero share, accumulating convolution, class-by-class strided input
    gradient, weight gradient, truncation step, bit transpose, carry-save cell, binary reshare) captured into
    one graph: every replay, with eager work and new inputs in between, must give what the eager calls give."""
    cg, ro, wl = env
    k0, k1 = bytes(range(16)), bytes(range(16, 32))
    xs, ws, st, pd = (4, 14, 14, 64), (96, 3, 3, 64), (2, 2), (1, 1)
    zs = cg.conv_out_shape(xs, ws, st, pd)
    x = [cg.to_device(wl.draw_ring(xs, 70 + j)) for j in range(2)]
    w = [cg.to_device(wl.draw_ring(ws, 72 + j)) for j in range(2)]
    g = [cg.to_device(wl.draw_ring(zs, 74 + j)) for j in range(2)]
    n = int(np.prod(zs))
    assert n % 64 == 0
    z = torch.empty(zs, dtype=torch.int64, device="cuda")
    dx = torch.empty(xs, dtype=torch.int64, device="cuda")
    dw = torch.empty(ws, dtype=torch.int64, device="cuda")
    tr = torch.empty(zs, dtype=torch.int64, device="cuda")
    planes = [torch.empty((64, n // 64), dtype=torch.int64, device="cuda") for _ in range(2)]
    s0, s1, carry = (torch.empty((64, n // 64), dtype=torch.int64, device="cuda") for _ in range(3))
    outs = [z, dx, dw, tr, s0, s1, carry]

    def step():
        cg.cg_zero_share(k0, k1, 9, 0, n, out=z.view(-1))
        cg.cg_share_conv2d_acc(*x, *w, z, stride=st, pad=pd)                        # the reshared product
        cg.cg_share_conv2d_dgrad(*g, *w, xs, stride=st, pad=pd, dx_i=dx)            # four launches after a fill
        cg.cg_share_conv2d_wgrad(*g, *x, ws, stride=st, pad=pd, dw_i=dw)
        cg.cg_trunc1_local(z, g[0], k1, k0, 10, 0, 16, k1, 11, out=tr)
        cg.cg_bit_transpose64(z.view(-1), out=planes[0])
        cg.cg_bit_transpose64(tr.view(-1), out=planes[1])
        cg.cg_bshare_csa(planes[0], None, None, planes[1], None, None, s_i=s0, s_ip1=s1, carry_i=carry)
        cg.cg_breshare(carry, k0, k1, 12, 0, out=carry)

    say("protocol steps: eager run, then capture")
    step()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        say(f"protocol steps: graph replay {rep}")
        for o in outs:
            o.fill_(0x3C3C3C3C3C3C3C3C)
        if rep == 2:                                   # new activations and gradient in the same buffers
            x[0].copy_(cg.to_device(wl.draw_ring(xs, 170)))
            g[1].copy_(cg.to_device(wl.draw_ring(zs, 171)))
            step()
            torch.cuda.synchronize()
            want = [o.clone() for o in outs]
            for o in outs:
                o.fill_(0x3C3C3C3C3C3C3C3C)
        graph.replay()
        torch.cuda.synchronize()
        for name, o, w_ in zip(("z", "dx", "dw", "trunc", "sum", "sum'", "carry"), outs, want):
            assert torch.equal(o, w_), f"replay {rep}: {name}"
