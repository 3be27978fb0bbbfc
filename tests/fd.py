"""Central finite differences of a scalar loss w.r.t. named float64 arrays."""
import numpy as np


def central_fd(loss_fn, params: dict, name: str, rel_step=1e-6):
    base = params[name]
    g = np.zeros_like(base)
    it = np.nditer(base, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        h = rel_step * max(1.0, abs(base[i]))
        p = dict(params); a = base.copy(); a[i] += h; p[name] = a
        up = loss_fn(p)
        a = base.copy(); a[i] -= h; p[name] = a
        dn = loss_fn(p)
        g[i] = (up - dn) / (2 * h)
    return g


def assert_close(a, b, rtol, what=""):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    scale = max(np.abs(b).max(), 1e-30)
    err = np.abs(a - b).max() / scale
    assert err <= rtol, f"{what}: max|a-b|/max|b| = {err:.3e} > {rtol}"
