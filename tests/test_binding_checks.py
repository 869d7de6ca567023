"""Host-only checks of the Python binding's argument validation: the C side sees only pointers and
strides, so a tensor with too few rows, a narrow column view with a large stride, a short center or a
table of the wrong shape would become an out-of-range device access.  The binding must refuse all of
them before anything reaches the library.  CPU tensors stand in for device memory (the device check is
switched off); no call here passes validation, so nothing is launched."""
import ctypes as C

import pytest
import torch

from paper_2403_04206_amd import grawa

K, P, L = 4, 100, 3


@pytest.fixture()
def plan(monkeypatch):
    monkeypatch.setattr(grawa, "_REQUIRE_DEVICE", False)

    class Reached:
        def __getattr__(self, name):
            def fn(*args):
                raise AssertionError("%s was reached: validation let a bad argument through" % name)
            return fn
    monkeypatch.setattr(grawa, "lib", lambda: Reached())
    p = grawa.Plan.__new__(grawa.Plan)
    p.K, p.P, p.L = K, P, L
    p._h = C.c_void_p(0)
    return p


def good():
    x = torch.zeros((K, 104))[:, :P]
    g = torch.zeros((K, 104))[:, :P]
    return x, g


def test_validators_accept_well_formed_tensors(monkeypatch):
    monkeypatch.setattr(grawa, "_REQUIRE_DEVICE", False)
    x, g = good()
    assert grawa._params(x, K, P)[1] == 104
    assert grawa._grads(g.to(torch.bfloat16), K, P)[2] == grawa.BF16
    assert grawa._grads(g, K, P)[2] == grawa.F32
    assert grawa._vector(torch.zeros(P), P, "c").value
    assert grawa._vector(None, P, "c").value in (0, None)
    assert grawa._table(torch.zeros((K, L)), (K, L), "w").value
    assert grawa._params(torch.zeros((1, P)), 1, P)[1] == P            # one row: any stride


def test_cpu_tensors_are_refused_when_the_device_is_required():
    x, g = good()
    with pytest.raises(TypeError):
        grawa._params(x, K, P)
    with pytest.raises(TypeError):
        grawa._grads(g, K, P)
    with pytest.raises(TypeError):
        grawa._vector(torch.zeros(P), P, "center")
    with pytest.raises(TypeError):
        grawa._table(torch.zeros((K, L)), (K, L), "weights")


def test_update_calls_refuse_bad_x_and_g(plan):
    x, g = good()
    bad_x = [
        (torch.zeros((K - 1, 104))[:, :P], ValueError),               # fewer than K rows
        (torch.zeros((K, 104))[:, :P - 4], ValueError),               # narrower than P
        (torch.zeros((K, 104), dtype=torch.float64)[:, :P], TypeError),
        (torch.zeros((104, K)).t()[:, :P], TypeError),                 # column stride != 1
        (torch.zeros(K * 104), TypeError),                             # not 2-D
        (torch.zeros((K, 104))[:, ::2][:, :P // 2], TypeError),       # strided columns
    ]
    for t, exc in bad_x:
        with pytest.raises(exc):
            plan.lgrawa_update(t, g, 0.1)
        with pytest.raises(exc):
            plan.mgrawa_update(t, g, 0.1)
        with pytest.raises(exc):
            plan.center_pull(t, torch.zeros(K), 0.1)
        with pytest.raises(exc):
            plan.local_lgrawa_update(t, 0.1)
        with pytest.raises(exc):
            plan.easgd_update(t, 0.1, 0.5, torch.zeros(P))
    bad_g = [
        (torch.zeros((K - 1, 104))[:, :P], ValueError),
        (torch.zeros((K, 104))[:, :P - 1], ValueError),
        (torch.zeros((K, 104), dtype=torch.float16)[:, :P], TypeError),
        (torch.zeros((K, 104), dtype=torch.int32)[:, :P], TypeError),
    ]
    for t, exc in bad_g:
        with pytest.raises(exc):
            plan.lgrawa_update(x, t, 0.1)
        with pytest.raises(exc):
            plan.grad_norms(t)
        with pytest.raises(exc):
            plan.lgrawa_update_sgd(x, g, 0.1, t, 0.1)
        with pytest.raises(exc):
            plan.local_step_scored(x, t, 0.1, 0.9)
    with pytest.raises(TypeError):                                     # g and g_sgd of different types
        plan.mgrawa_update_sgd(x, g, 0.1, g.to(torch.bfloat16), 0.1)


def test_overlapping_rows_are_refused(plan):
    # torch itself refuses a view that overruns its storage; rows that overlap it does allow
    x, g = good()
    overlapping = torch.as_strided(torch.zeros(4 * P), (K, P), (P - 4, 1))
    with pytest.raises(ValueError, match="row stride"):
        plan.lgrawa_update(overlapping, g, 0.1)
    with pytest.raises(ValueError, match="row stride"):
        plan.lgrawa_update(x, overlapping, 0.1)


def test_outputs_and_side_inputs_are_checked(plan):
    x, g = good()
    for cen in (torch.zeros(P - 1), torch.zeros(P, dtype=torch.float64), torch.zeros((1, P)), torch.zeros(2 * P)[::2]):
        with pytest.raises((TypeError, ValueError)):
            plan.lgrawa_update(x, g, 0.1, center_out=cen)
        with pytest.raises((TypeError, ValueError)):
            plan.local_step_scored(x, g, 0.1, 0.9, center=cen)
        with pytest.raises((TypeError, ValueError)):
            plan.easgd_update(x, 0.1, 0.5, cen)
        with pytest.raises((TypeError, ValueError)):
            grawa.local_sgd_prox(x, g, 0.1, cen, 0.05, 16.0)
    with pytest.raises(TypeError):
        plan.easgd_update(x, 0.1, 0.5, None)                          # the EASGD center is required
    for wts in (torch.zeros((K, L + 1)), torch.zeros((L, K)), torch.zeros(K * L), torch.zeros((K, L), dtype=torch.float64),
                torch.zeros((K, 2 * L))[:, ::2]):
        with pytest.raises((TypeError, ValueError)):
            plan.lgrawa_update(x, g, 0.1, weights_out=wts)
        with pytest.raises((TypeError, ValueError)):
            plan.local_lgrawa_update(x, 0.1, est_out=wts)
        with pytest.raises((TypeError, ValueError)):
            plan.grad_norms(g, norms_out=wts)
    with pytest.raises(ValueError):
        plan.mgrawa_update(x, g, 0.1, weights_out=torch.zeros(K + 1))
    with pytest.raises(ValueError):
        plan.center_pull(x, torch.zeros((K, L + 1)), 0.1)
    with pytest.raises(ValueError):
        plan.center_pull(x, torch.zeros(K - 1), 0.1)
    with pytest.raises((TypeError, ValueError)):
        plan.lsgd_update(x, torch.zeros(K - 1), 0.1)                  # losses shorter than K
    with pytest.raises(TypeError):
        plan.lsgd_update(x, torch.zeros(K, dtype=torch.float64), 0.1)
    with pytest.raises(TypeError):
        plan.lsgd_update(x, torch.zeros(K), 0.1, leader_out=torch.zeros(1, dtype=torch.int64))
    with pytest.raises(TypeError):
        plan.lsgd_update(x, None, 0.1)


def test_planless_steps_check_their_shapes(plan):
    x, g = good()
    with pytest.raises(ValueError):
        grawa.local_sgd(x, torch.zeros((K - 1, 104))[:, :P], 0.1)     # g with fewer rows than x
    with pytest.raises(ValueError):
        grawa.local_sgd(x, g[:, :P - 8], 0.1)                          # g narrower than x
    with pytest.raises(ValueError):
        grawa.local_sgd(x, g, 0.1, P=P + 8)                            # P beyond both
    with pytest.raises(ValueError):
        grawa.local_nesterov(x, g, torch.zeros((K, 96)), 0.1, 0.9)     # momentum buffer too narrow
    with pytest.raises(ValueError):
        grawa.local_nesterov(x, g, torch.zeros((K + 1, 104))[:, :P], 0.1, 0.9)
    with pytest.raises(TypeError):
        grawa.local_nesterov(x, g, torch.zeros((K, 104), dtype=torch.bfloat16)[:, :P], 0.1, 0.9)
    with pytest.raises(TypeError):
        grawa.lgrawa_update_static(x, g, torch.zeros(L + 1, dtype=torch.int32), 0.1)    # offsets must be int64
    with pytest.raises(ValueError):
        grawa.lgrawa_update_static(x, g, torch.zeros(L + 1, dtype=torch.int64), 0.1, weights_out=torch.zeros((K, L + 1)))
