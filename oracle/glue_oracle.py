"""Oracle for the layer glue - TEST INFRASTRUCTURE, not product code.

The operators that sit between the blocks of a pre-norm decoder layer and are the same for a dense and a sparse
model: RMSNorm, LayerNorm (each with the residual addition in front of it), the embedding lookup with an optional
learned position table, and the mean cross-entropy loss over a vocabulary.  The paper leaves them untouched (its
Sec. 3.1 prunes the coupled pairs only), so nothing here follows an equation of the paper: each function is the
textbook definition in fp64 numpy, written out plainly, and each is pinned by central differences, closed forms or
brute force in tests/test_oracle_glue.py.  Only tests/ may import this module; it shares no code with the HIP path.
"""
import numpy as np


def rms_fwd(x, g, eps):
    """y = x / sqrt(mean(x^2) + eps) * g, row by row.  Returns (y, r) with r the reciprocal root per row."""
    r = 1.0 / np.sqrt((x * x).mean(axis=1, keepdims=True) + eps)
    return x * r * g, r


def rms_bwd(x, g, r, dy):
    """-> (dx, dg, None) of rms_fwd."""
    u = dy * g
    dx = r * u - x * r ** 3 * (u * x).mean(axis=1, keepdims=True)
    return dx, (dy * x * r).sum(axis=0), None


def ln_fwd(x, g, b, eps):
    """y = (x - mean) / sqrt(var + eps) * g + b, row by row (biased variance).  Returns (y, (xhat, r))."""
    mu = x.mean(axis=1, keepdims=True)
    r = 1.0 / np.sqrt(((x - mu) ** 2).mean(axis=1, keepdims=True) + eps)
    xh = (x - mu) * r
    return xh * g + b, (xh, r)


def ln_bwd(g, st, dy):
    """-> (dx, dg, db) of ln_fwd; st = (xhat, r) as returned by it."""
    xh, r = st
    u = dy * g
    dx = r * (u - u.mean(axis=1, keepdims=True) - xh * (u * xh).mean(axis=1, keepdims=True))
    return dx, (dy * xh).sum(axis=0), dy.sum(axis=0)


def embed_fwd(ids, table, pos=None, L=None):
    """x[t] = table[ids[t]] (+ pos[t mod L])."""
    x = table[ids].copy()
    if pos is not None:
        x += pos[np.arange(len(ids)) % L]
    return x


def embed_bwd(ids, dx, vocab, pos_len=None):
    """-> (dtable [vocab, d], dpos [pos_len, d] or None): every row of dx added to the row of its token,
    and to the row of its position."""
    dtable = np.zeros((vocab, dx.shape[1]))
    for t, v in enumerate(ids):
        dtable[v] += dx[t]
    dpos = None
    if pos_len is not None:
        dpos = np.zeros((pos_len, dx.shape[1]))
        for t in range(len(ids)):
            dpos[t % pos_len] += dx[t]
    return dtable, dpos


def xent(logits, targets):
    """Mean over the rows of -log softmax(logits)[target].  Returns (loss, row losses, dlogits of the mean)."""
    T = logits.shape[0]
    z = logits - logits.max(axis=1, keepdims=True)
    lse = np.log(np.exp(z).sum(axis=1, keepdims=True))
    logp = z - lse
    rows = -logp[np.arange(T), targets]
    dl = np.exp(logp)
    dl[np.arange(T), targets] -= 1.0
    return rows.mean(), rows, dl / T
