"""The paper's motivating example (Sec. 3 "Motivating Example", Appendix C) run through the library.

Four workers start from the corners (0.25, 0.25), (0.25, 10), (10, 0.25), (10, 10) of the plane and
minimise the two-dimensional Vincent function f(x, y) = -sin(10 ln x) - sin(10 ln y) with plain SGD
(learning rate 0.01); after every 4 local steps a distributed optimizer pulls them toward its center.
All minimisers have the value -2 but sit in valleys of different width (the curvature at a minimiser
is 100 / x^2 per coordinate), which is what the example is about: the gradient-norm weighted centers
end in a wider valley than the EASGD and LSGD centers.

The function and its gradient are the "model" here and are evaluated with torch on the device; every
optimizer step (local SGD step, the five distributed phases) is a call into the library.  The
pulling strength is not given in the paper; 0.5 is used (0.3 gives the same picture).
"""
from __future__ import annotations

import torch

from . import grawa

START = ((0.25, 0.25), (0.25, 10.0), (10.0, 0.25), (10.0, 10.0))
POLICIES = ("easgd", "lsgd", "grawa", "mgrawa", "lgrawa")


def vincent(x: torch.Tensor) -> torch.Tensor:
    """f per worker; x: [K, 2], positive."""
    return -torch.sin(10.0 * torch.log(x)).sum(dim=1)


def vincent_grad(x: torch.Tensor) -> torch.Tensor:
    return -10.0 * torch.cos(10.0 * torch.log(x)) / x


def curvature(x: torch.Tensor) -> torch.Tensor:
    """Second derivative of f along each coordinate (100 / x^2 at a minimiser)."""
    u = 10.0 * torch.log(x)
    return (100.0 * torch.sin(u) + 10.0 * torch.cos(u)) / (x * x)


def run(policy: str, rounds: int = 60, tau: int = 4, lr: float = 0.01, lam: float = 0.5, rho: float = 0.5,
        device: str = "cuda:0", observer=None):
    """Runs `rounds` rounds of tau local SGD steps and one distributed phase.  Returns a dict with the
    final points x [4, 2], their losses, and the trajectory [rounds * (tau + 1) + 1, 4, 2].
    observer(name, x_before, g, x_after, extra), if given, is called after every library call with
    copies of the state (for checks against a reference)."""
    if policy not in POLICIES:
        raise ValueError("policy must be one of %r" % (POLICIES,))
    K, P, ld = len(START), 2, 4                          # rows padded to 16 bytes
    x = torch.ones((K, ld), dtype=torch.float32, device=device)
    x[:, :P] = torch.tensor(START, dtype=torch.float32, device=device)
    g = torch.zeros((K, ld), dtype=torch.float32, device=device)
    center = torch.zeros(ld, dtype=torch.float32, device=device)
    center[:P] = x[:, :P].mean(dim=0)                    # EASGD's center starts at the workers' mean
    traj = [x[:, :P].clone()]
    xv, gv = x[:, :P], g[:, :P]

    def call(name, fn, extra=None):
        before = x.clone() if observer else None
        fn()
        if observer:
            torch.cuda.synchronize()
            observer(name, before[:, :P], g[:, :P].clone(), x[:, :P].clone(), extra)
        traj.append(x[:, :P].clone())

    with grawa.Plan(K, P, [0, 1, 2]) as plan:            # every coordinate is a "layer"
        for _ in range(rounds):
            for _ in range(tau):
                gv.copy_(vincent_grad(xv))
                call("local_sgd", lambda: grawa.local_sgd(xv, gv, lr))
            gv.copy_(vincent_grad(xv))                   # the gradients the weights are taken from
            if policy == "easgd":
                c0 = center.clone()
                call("easgd", lambda: plan.easgd_update(xv, lam, rho, center), {"center_before": c0[:P]})
            elif policy == "lsgd":
                losses = vincent(xv).contiguous()
                call("lsgd", lambda: plan.lsgd_update(xv, losses, lam), {"losses": losses.clone()})
            elif policy == "grawa":
                call("grawa", lambda: plan.mgrawa_update(xv, gv, lam, mode=grawa.NORM_FLAT))
            elif policy == "mgrawa":
                call("mgrawa", lambda: plan.mgrawa_update(xv, gv, lam))
            else:
                call("lgrawa", lambda: plan.lgrawa_update(xv, gv, lam))
        torch.cuda.synchronize()
    return {"x": x[:, :P].clone(), "loss": vincent(x[:, :P]), "curvature": curvature(x[:, :P]),
            "trajectory": torch.stack(traj)}


if __name__ == "__main__":
    for pol in POLICIES:
        out = run(pol)
        print("%-7s final points %s  loss %s  curvature %s" % (
            pol, [[round(v, 3) for v in r] for r in out["x"].tolist()],
            [round(v, 3) for v in out["loss"].tolist()], [round(v, 2) for v in out["curvature"][0].tolist()]))
