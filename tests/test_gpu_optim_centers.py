"""GPU parity of the local optimizer of the experiments (Appendix B.2.2: SGD with Nesterov momentum
and weight decay) and of the two competing center rules of Appendix F (EASGD, LSGD)."""
import numpy as np
import pytest
import torch

from oracle import grawa_oracle as orc
from paper_2403_04206_amd import grawa, workloads as W
from parity_util import TIGHT, assert_params_close, grads_to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RAGGED = [1, 3, 8193, 2, 5, 8191, 20000, 7, 1, 1, 4096, 33, 16385, 6]


def say(msg):
    print("[case] " + msg, flush=True)


@pytest.mark.parametrize("K", [1, 3, 8, 33])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_nesterov_steps(K, dtype):
    for ld_pad in (0, 8):
        w, x, g0 = W.make_small(700 + K, K, RAGGED, grad_dtype=dtype, ld_pad=ld_pad, device=DEV)
        P = w.P
        say("nesterov K=%d dtype=%s ld_pad=%d P=%d" % (K, dtype, ld_pad, P))
        grads = [g0] + [W.make_small(710 + K + t, K, RAGGED, grad_dtype=dtype, ld_pad=ld_pad, device=DEV)[2] for t in (1, 2)]
        lr, mom, wd = 0.1, 0.9, 5e-4
        xh = W.to_numpy_params(x)
        xg = x.clone()
        buf = torch.zeros_like(x)
        ref_x, ref_b = xh[:, :P].astype(np.float64), np.zeros((K, P))
        sx = np.abs(ref_x)
        sb = np.zeros((K, P))
        for t, g in enumerate(grads):
            gh = W.to_numpy_grads(g)
            grawa.local_nesterov(xg[:, :P], g[:, :P], buf[:, :P], lr, mom, wd)
            ref_x, ref_b = orc.nesterov_sgd(ref_x, ref_b, gh, lr, mom, wd, P=P)
            # operand scales: what the step adds up, element by element
            gabs = np.abs(grads_to_f64(gh)[:, :P])
            sb = mom * sb + gabs + wd * sx
            sx = sx + lr * (gabs + wd * sx + mom * sb)
            torch.cuda.synchronize()
            got_x, got_b = xg.cpu().numpy(), buf.cpu().numpy()
            tol = (t + 1) * TIGHT                             # fp32 state is carried from step to step
            assert_params_close(got_x[:, :P], ref_x, w.offsets, tol, "x after step %d" % (t + 1), sx.max(axis=0))
            assert_params_close(got_b[:, :P], ref_b, w.offsets, tol, "buf after step %d" % (t + 1), sb.max(axis=0))
        np.testing.assert_array_equal(got_x[:, P:], xh[:, P:])
        assert not got_b[:, P:].any()


def test_nesterov_reductions_and_errors():
    w, x, g = W.make_small(720, 3, [1000, 29], device=DEV)
    P = w.P
    xa, xb = x.clone(), x.clone()
    buf = torch.zeros_like(x)
    grawa.local_nesterov(xa[:, :P], g[:, :P], buf[:, :P], 0.1, 0.0, 0.0)     # no momentum, no decay: plain SGD
    grawa.local_sgd(xb[:, :P], g[:, :P], 0.1)
    torch.cuda.synchronize()
    assert torch.equal(xa, xb)
    assert torch.equal(buf[:, :P], g[:, :P])
    for mom, wd in ((-0.1, 0.0), (0.9, -1.0), (float("nan"), 0.0)):
        with pytest.raises(grawa.GrawaError) as e:
            grawa.local_nesterov(xa[:, :P], g[:, :P], buf[:, :P], 0.1, mom, wd)
        assert e.value.status == grawa.ERR_INVALID_ARG
    short = buf[:, :P - 4].contiguous()                                      # buffer rows shorter than P
    with pytest.raises(ValueError):                                          # the binding refuses it ...
        grawa.local_nesterov(xa[:, :P], g[:, :P], short, 0.1, 0.9, 0.0)
    st = grawa.lib().grawa_local_nesterov(xa.data_ptr(), xa.stride(0), g.data_ptr(), g.stride(0), 0, short.data_ptr(),
                                          short.stride(0), 3, P, 0.1, 0.9, 0.0, None)
    assert st in (grawa.ERR_INVALID_ARG, grawa.ERR_ALIGNMENT)              # ... and so does the library (ldb < P)


@pytest.mark.parametrize("K", [1, 4, 7, 16, 33, 70])
def test_easgd_update(K):
    sizes = RAGGED if K <= 16 else RAGGED[:8]
    for ld_pad in (0, 8):
        w, x, _ = W.make_small(730 + K, K, sizes, ld_pad=ld_pad, device=DEV)
        P = w.P
        say("easgd K=%d ld_pad=%d P=%d" % (K, ld_pad, P))
        xh = W.to_numpy_params(x)
        cen = 0.05 * torch.randn(W.round_up(P, 4), device=DEV, generator=torch.Generator(device=DEV).manual_seed(K))
        ch = cen.cpu().numpy().astype(np.float64)
        xg = x.clone()
        with grawa.Plan(K, P, w.offsets) as plan:
            plan.easgd_update(xg[:, :P], 0.3, 0.25, cen)
            torch.cuda.synchronize()
        ref_x, ref_c = orc.easgd_update(xh, ch[:P], 0.3, 0.25, P=P)
        sc = np.maximum(np.abs(xh[:, :P].astype(np.float64)).max(axis=0), np.abs(ch[:P]))
        got = xg.cpu().numpy()
        assert_params_close(got[:, :P], ref_x, w.offsets, TIGHT, "easgd x", sc)
        assert_params_close(cen.cpu().numpy()[:P], ref_c, w.offsets, TIGHT, "easgd center", sc)
        np.testing.assert_array_equal(got[:, P:], xh[:, P:])
        np.testing.assert_array_equal(cen.cpu().numpy()[P:].astype(np.float64), ch[P:])


def test_easgd_limits():
    w, x, _ = W.make_small(740, 4, [500, 12], device=DEV)
    P = w.P
    cen = torch.randn(P, device=DEV)
    c0, x0 = cen.clone(), x.clone()
    with grawa.Plan(4, P, w.offsets) as plan:
        for rho in (-0.1, 1.5, float("nan")):
            with pytest.raises(grawa.GrawaError) as e:
                plan.easgd_update(x[:, :P], 0.3, rho, cen)
            assert e.value.status == grawa.ERR_INVALID_ARG
        with pytest.raises(TypeError):                      # the center is required (binding) ...
            plan.easgd_update(x[:, :P], 0.3, 0.5, None)
        assert grawa.lib().grawa_easgd_update(plan._h, x.data_ptr(), x.stride(0), 0.3, 0.5, None, None) == \
            grawa.ERR_INVALID_ARG                           # ... and by the library
        plan.easgd_update(x[:, :P], 0.0, 0.0, cen)          # rho = 0 keeps the center, lambda = 0 the workers
        torch.cuda.synchronize()
        assert torch.equal(cen, c0) and torch.equal(x, x0)
        # rho = 1: the center is the plain average, i.e. the GRAWA center with equal weights
        xa, xb = x.clone(), x.clone()
        ca, cb = cen.clone(), torch.empty_like(cen)
        plan.easgd_update(xa[:, :P], 0.4, 1.0, ca)
        plan.center_pull(xb[:, :P], torch.full((4,), 0.25, device=DEV), 0.4, center_out=cb)
        torch.cuda.synchronize()
        torch.testing.assert_close(ca, cb, rtol=0, atol=1e-5 * float(x.abs().max() + c0.abs().max()))
        torch.testing.assert_close(xa, xb, rtol=0, atol=1e-5 * float(x.abs().max() + c0.abs().max()))


@pytest.mark.parametrize("K", [1, 4, 16, 33, 70])
def test_lsgd_update(K):
    sizes = RAGGED if K <= 16 else RAGGED[:8]
    w, x, _ = W.make_small(750 + K, K, sizes, device=DEV)
    P = w.P
    say("lsgd K=%d P=%d" % (K, P))
    xh = W.to_numpy_params(x)
    losses = torch.rand(K, device=DEV, generator=torch.Generator(device=DEV).manual_seed(K))
    if K >= 4:
        losses[K // 2] = losses.min()                        # a tie: the first smallest leads
        losses[1] = losses[K // 2]
    xg = x.clone()
    cen = torch.empty(W.round_up(P, 4), device=DEV)
    lead = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    with grawa.Plan(K, P, w.offsets) as plan:
        plan.lsgd_update(xg[:, :P], losses, 0.3, center_out=cen, leader_out=lead)
        torch.cuda.synchronize()
    ref_x, ref_lead = orc.lsgd_update(xh, losses.cpu().numpy().astype(np.float64), 0.3, P=P)
    assert int(lead.item()) == ref_lead                      # an index: exact
    got = xg.cpu().numpy()
    np.testing.assert_array_equal(cen.cpu().numpy()[:P], xh[ref_lead, :P])      # the center is a copy of the leader
    np.testing.assert_array_equal(got[ref_lead], xh[ref_lead])                  # which does not move
    sc = np.abs(xh[:, :P].astype(np.float64)).max(axis=0)
    assert_params_close(got[:, :P], ref_x, w.offsets, TIGHT, "lsgd x", sc)
    np.testing.assert_array_equal(got[:, P:], xh[:, P:])
