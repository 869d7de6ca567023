"""Float64 reference run of the paper's motivating example (Sec. 3; Appendix C) for the tests: the
Vincent function and its gradient in numpy, every optimizer step through the CPU reference."""
import numpy as np

from oracle import grawa_oracle as orc

START = np.array([(0.25, 0.25), (0.25, 10.0), (10.0, 0.25), (10.0, 10.0)])
POLICIES = ("easgd", "lsgd", "grawa", "mgrawa", "lgrawa")
OFF = np.array([0, 1, 2])


def loss(x):
    return -np.sin(10.0 * np.log(x)).sum(axis=1)


def grad(x):
    return -10.0 * np.cos(10.0 * np.log(x)) / x


def curvature(x):
    u = 10.0 * np.log(x)
    return (100.0 * np.sin(u) + 10.0 * np.cos(u)) / (x * x)


def phase(policy, x, g, lam, rho=0.5, center=None, losses=None):
    """One distributed phase on float32 states through the reference; returns (x_new float64, center or None)."""
    if policy == "easgd":
        return orc.easgd_update(x, center, lam, rho)
    if policy == "lsgd":
        return orc.lsgd_update(x, losses, lam)[0], None
    if policy == "grawa":
        return orc.mgrawa_update(x, g, OFF, lam, mode="flat")["x"], None
    if policy == "mgrawa":
        return orc.mgrawa_update(x, g, OFF, lam)["x"], None
    return orc.lgrawa_update(x, g, OFF, lam)["x"], None


def simulate(policy, rounds=60, tau=4, lr=0.01, lam=0.5, rho=0.5):
    """Workers kept in float32 between steps (as the library stores them), gradients of the float32
    points evaluated in float64 and rounded to float32."""
    x = START.astype(np.float32)
    center = x.astype(np.float64).mean(axis=0)
    for _ in range(rounds):
        for _ in range(tau):
            g = grad(x.astype(np.float64)).astype(np.float32)
            x = orc.local_sgd(x, g, lr).astype(np.float32)
        g = grad(x.astype(np.float64)).astype(np.float32)
        xn, c = phase(policy, x, g, lam, rho, center, loss(x.astype(np.float64)))
        if c is not None:
            center = c.astype(np.float32).astype(np.float64)
        x = xn.astype(np.float32)
    xd = x.astype(np.float64)
    return {"x": xd, "loss": loss(xd), "curvature": curvature(xd)}
