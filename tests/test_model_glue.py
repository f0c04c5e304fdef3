"""Central differences pin the norm derivatives that the oracle-side stack model uses (CPU only)."""
import numpy as np

from model_glue import ln_bwd, ln_fwd, rms_bwd, rms_fwd


def _fd(f, x, dy, h=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        g[i] = ((f(xp) - f(xm)) * dy).sum() / (2 * h)
    return g


def test_rmsnorm_derivatives():
    rng = np.random.default_rng(0)
    x, g, dy = rng.standard_normal((5, 12)), rng.standard_normal(12), rng.standard_normal((5, 12))
    y, r = rms_fwd(x, g, 1e-6)
    np.testing.assert_allclose(y, x / np.sqrt((x * x).mean(1, keepdims=True) + 1e-6) * g)
    dx, dg, _ = rms_bwd(x, g, r, dy)
    np.testing.assert_allclose(dx, _fd(lambda v: rms_fwd(v, g, 1e-6)[0], x, dy), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dg, _fd(lambda v: rms_fwd(x, v, 1e-6)[0], g, dy), rtol=1e-6, atol=1e-8)


def test_layernorm_derivatives():
    rng = np.random.default_rng(1)
    x, g, b, dy = rng.standard_normal((4, 10)), rng.standard_normal(10), rng.standard_normal(10), rng.standard_normal((4, 10))
    y, st = ln_fwd(x, g, b, 1e-5)
    np.testing.assert_allclose(y.mean(1), (b + 0 * x).mean(1) + ((x - x.mean(1, keepdims=True)) / np.sqrt(x.var(1, keepdims=True) + 1e-5) * g).mean(1))
    dx, dg, db = ln_bwd(g, st, dy)
    np.testing.assert_allclose(dx, _fd(lambda v: ln_fwd(v, g, b, 1e-5)[0], x, dy), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dg, _fd(lambda v: ln_fwd(x, v, b, 1e-5)[0], g, dy), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db, dy.sum(0))
