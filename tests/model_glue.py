"""Pre-norm glue of the small test models in fp64 numpy (RMSNorm, LayerNorm and their derivatives): not part of the
method, used by the oracle-side model of `test_gpu_stack_oracle.py`; pinned by central differences in
`test_model_glue.py`."""
import numpy as np


def rms_fwd(x, g, eps):
    r = 1.0 / np.sqrt((x * x).mean(axis=1, keepdims=True) + eps)
    return x * r * g, r


def rms_bwd(x, g, r, dy):
    u = dy * g
    dx = r * u - x * r ** 3 * (u * x).mean(axis=1, keepdims=True)
    return dx, (dy * x * r).sum(axis=0), None


def ln_fwd(x, g, b, eps):
    mu = x.mean(axis=1, keepdims=True)
    r = 1.0 / np.sqrt(((x - mu) ** 2).mean(axis=1, keepdims=True) + eps)
    xh = (x - mu) * r
    return xh * g + b, (xh, r)


def ln_bwd(g, st, dy):
    xh, r = st
    u = dy * g
    dx = r * (u - u.mean(axis=1, keepdims=True) - xh * (u * xh).mean(axis=1, keepdims=True))
    return dx, (dy * xh).sum(axis=0), dy.sum(axis=0)


