"""cg_share_matmul_static (the entry point that allocates nothing, for callers that cannot allocate) against
cg_share_matmul_ws, the existing entry point whose kernels it shares, and against the CPU oracle: two calls in
a row on the library's fixed scratch array, the second with a smaller input."""
import numpy as np
import pytest

from tests.gpu_util import first_mismatch, say

pytestmark = pytest.mark.gpu


def test_static_scratch_matches_workspace_entry_point_twice():
    import torch
    from oracle import ring_oracle as ro
    from paper_2104_10949_amd import binding as cg
    from paper_2104_10949_amd import workloads as wl

    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    cg.lib()
    # the second product is smaller in every dimension: it reuses the front of the array the first one filled
    for case, (M, N, K) in enumerate([(300, 200, 1000), (70, 130, 96)]):
        say(f"cg_share_matmul_static call {case}: M={M} N={N} K={K}")
        host = [wl.draw_ring(s, 9100 + 10 * case + j) for j, s in enumerate([(M, K), (M, K), (N, K), (N, K)])]
        dev = [cg.to_device(a) for a in host]
        need = cg.cg_share_matmul_workspace_bytes(M, N, K)
        assert 0 < need <= cg.STATIC_SCRATCH_BYTES
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        want_ws = cg.cg_share_matmul_ws(*dev, ws)
        got = cg.cg_share_matmul_static(*dev)
        torch.cuda.synchronize()
        got_h, ws_h = cg.to_host(got), cg.to_host(want_ws)
        assert np.array_equal(got_h, ws_h), first_mismatch(got_h, ws_h)
        want = ro.party_matmul(*host)
        assert np.array_equal(got_h, want), first_mismatch(got_h, want)


def test_static_scratch_rejects_products_beyond_its_size():
    import torch
    from paper_2104_10949_amd import binding as cg

    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    M = N = K = 2048
    assert cg.cg_share_matmul_workspace_bytes(M, N, K) > cg.STATIC_SCRATCH_BYTES
    x = torch.zeros((M, K), dtype=torch.int64, device="cuda")
    y = torch.zeros((N, K), dtype=torch.int64, device="cuda")
    z = torch.full((M, N), 7, dtype=torch.int64, device="cuda")
    say("cg_share_matmul_static beyond the scratch size: must refuse and launch nothing")
    with pytest.raises(cg.CgError) as e:
        cg.cg_share_matmul_static(x, x.clone(), y, y.clone(), z_i=z)
    assert e.value.status == cg.CG_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((z == 7).all())
