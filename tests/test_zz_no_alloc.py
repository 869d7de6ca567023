"""The allocation-free entry point grawa_lgrawa_update_static against grawa_lgrawa_update (the same
kernels behind a plan): bit-identical parameters, center and weights, on two calls in a row of which
the second has the smaller input (the fixed scratch array keeps the first call's contents), for fp32 and
bf16 gradients, ragged layer lists and a benchmark-sized problem; plus its limits and that it
allocates nothing."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2403_04206_amd import grawa, workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RAGGED = [1, 3, 8193, 2, 5, 8191, 20000, 7, 1, 1, 4096, 33, 16385, 6]


def say(msg):
    print("[case] " + msg, flush=True)


def both_ways(w, x, g, lam, check_alloc=False):
    """Run the plan-based update and the static one on clones; everything must be bit-identical."""
    P, K, L = w.P, w.K, w.L
    off_dev = torch.from_numpy(w.offsets).to(DEV)
    xa, xb = x.clone(), x.clone()
    ca = torch.full((W.round_up(P, 4),), float("nan"), device=DEV)
    cb = ca.clone()
    wa = torch.full((K, L), float("nan"), device=DEV)
    wb = wa.clone()
    with grawa.Plan(K, P, w.offsets) as plan:
        plan.lgrawa_update(xa[:, :P], g[:, :P], lam, center_out=ca, weights_out=wa)
        torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
    grawa.lgrawa_update_static(xb[:, :P], g[:, :P], off_dev, lam, center_out=cb, weights_out=wb)
    torch.cuda.synchronize()
    after = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
    if check_alloc:                      # the device's free memory does not move across the call
        assert after == before, "allocation across the static call: %r -> %r" % (before, after)
    assert torch.equal(wa, wb), "weights differ"
    assert torch.equal(ca[:P], cb[:P]), "center differs"
    assert torch.equal(xa, xb), "parameters differ"
    assert not torch.isnan(wb).any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_matches_plan_twice_in_a_row(dtype):
    # first a larger problem, then a smaller one (fewer workers, fewer and shorter layers): what the
    # first call left in the scratch array must not leak into the second
    w1, x1, g1 = W.make_small(801, 16, RAGGED + [50000, 12, 70001], grad_dtype=dtype, device=DEV)
    w2, x2, g2 = W.make_small(802, 5, RAGGED[:6], grad_dtype=dtype, ld_pad=8, device=DEV)
    say("static twice in a row dtype=%s  P=%d then P=%d" % (dtype, w1.P, w2.P))
    both_ways(w1, x1, g1, 0.3)                 # the first call on the device also looks up the array
    both_ways(w2, x2, g2, 0.25, check_alloc=True)
    both_ways(w1, x1, g1, 0.3, check_alloc=True)


@pytest.mark.parametrize("K,sizes", [(1, [7]), (3, [1, 1, 1, 1, 1]), (4, [8192]), (4, [8193]), (33, RAGGED[:8]),
                                     (70, [300, 5, 1000, 1, 257]), (8, [2048] * 40), (2, [1] * 3000)])
def test_static_layouts(K, sizes):
    w, x, g = W.make_small(810 + K, K, sizes, device=DEV)
    say("static layout K=%d L=%d P=%d" % (K, w.L, w.P))
    both_ways(w, x, g, 0.5)


def test_static_benchmark_size():
    # configurations 3 (the largest: 354 M parameters, 7 MiB of the fixed workspace), 4 (K = 32, 161 layers),
    # 2 (K = 16, 80 ragged layers) on the streaming path, then the small configuration 0 right after them
    for idx in (3, 4, 2, 0):
        w = W.config(idx)
        say("static %s K=%d L=%d P=%d" % (w.name, w.K, w.L, w.P))
        x, g = W.make_inputs(w, device=DEV)
        both_ways(w, x, g, w.lam, check_alloc=True)
        del x, g
        torch.cuda.empty_cache()


def test_static_limits_launch_nothing():
    L = grawa.lib()
    f = L.grawa_lgrawa_update_static
    z, a, odd = C.c_void_p(0), C.c_void_p(0x1000), C.c_void_p(0x1004)
    assert f(0, 16, 1, a, a, 16, a, 16, 0, 0.1, z, z, z) == grawa.ERR_INVALID_ARG       # K < 1
    assert f(2, 16, 1, z, a, 16, a, 16, 0, 0.1, z, z, z) == grawa.ERR_INVALID_ARG       # no offsets
    assert f(2, 16, 17, a, a, 16, a, 16, 0, 0.1, z, z, z) == grawa.ERR_INVALID_ARG      # L > P
    assert f(2, 16, 1, odd, a, 16, a, 16, 0, 0.1, z, z, z) == grawa.ERR_ALIGNMENT       # offsets not 8-byte aligned
    assert f(2, 16, 1, a, a, 8, a, 16, 0, 0.1, z, z, z) == grawa.ERR_INVALID_ARG        # ldx < P
    assert f(2, 16, 1, a, a, 16, a, 16, 0, 1.5, z, z, z) == grawa.ERR_INVALID_ARG       # lambda
    assert f(grawa.MAX_WORKERS + 1, 16, 1, a, a, 16, a, 16, 0, 0.1, z, z, z) == grawa.ERR_UNSUPPORTED
    # more scratch than the fixed array holds: 2^33 columns need 128 MiB of cell map alone
    big = 1 << 33
    assert f(2, big, 1, a, a, big, a, big, 0, 0.1, z, z, z) == grawa.ERR_UNSUPPORTED
    # and a worker count whose partial sums do not fit: K = 1024, 2^28 columns
    assert f(1024, 1 << 28, 1, a, a, 1 << 28, a, 1 << 28, 0, 0.1, z, z, z) == grawa.ERR_UNSUPPORTED


def test_static_under_graph_capture():
    # what the entry point is for: recorded into a HIP graph (after one eager call on the device, which looks
    # up the array) and replayed, with eager work in between, it gives bit for bit what the plan-based call gives
    w, x, g = W.make_small(830, 16, RAGGED, device=DEV)
    P, K, L = w.P, w.K, w.L
    say("static under graph capture K=%d P=%d" % (K, P))
    off_dev = torch.from_numpy(w.offsets).to(DEV)
    xs = x.clone()
    cen_g, cen_e = torch.empty(W.round_up(P, 4), device=DEV), torch.empty(W.round_up(P, 4), device=DEV)
    wts_g, wts_e = torch.empty((K, L), device=DEV), torch.empty((K, L), device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                       # warm-up outside the capture
        grawa.lgrawa_update_static(xs[:, :P], g[:, :P], off_dev, 0.3)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        grawa.lgrawa_update_static(xs[:, :P], g[:, :P], off_dev, 0.3, center_out=cen_g, weights_out=wts_g)
    with grawa.Plan(K, P, w.offsets) as plan:
        for rep in range(3):
            xe = x.clone() + rep
            xs.copy_(xe)
            plan.lgrawa_update(xe[:, :P], g[:, :P], 0.3, center_out=cen_e, weights_out=wts_e)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(xs, xe), "replay %d differs" % rep
            assert torch.equal(cen_g[:P], cen_e[:P]) and torch.equal(wts_g, wts_e)
