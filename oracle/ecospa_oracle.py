"""CPU oracle for EcoSpa's coupled structured sparsification and the reduced layer maths.

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 numpy restatement of what the
paper's method computes, used only to check the GPU library (tests, the smoke check and
the benchmark's CPU-baseline leg).  The product path never imports it, and it imports
nothing from the product.

Conventions
-----------
* Storage is the Linear-layer layout ``W[out_features, in_features]`` (``y = x W^T``).
  The paper writes ``X W`` with ``W_in in R^{d_m x d}`` (Sec. 2.1, Eq. 3), so the paper's
  "column j of W_in" is stored row j of ``w1`` here, and "row j of W_out" is stored
  column j of ``w2``.
* A coupled pair has ``groups`` independent inner spaces of ``n`` dimensions each
  (``groups`` = number of heads for the attention pairs of Eq. 4, 1 for the FFN pair).
* ``unit`` consecutive inner dimensions are scored and removed together; ``unit=2`` is the
  2x2 rotary block of Eq. 6, whose Frobenius norm no position rotation changes.
* All arithmetic is fp64 on the inputs as given (already rounded to their storage type).

Every function states the passage of the paper it follows.  Parity status: every function
here is pinned by tests that do not go through this file's own formulas (library SVD,
autograd of independently written dense layers, finite differences, brute force over
subsets, Proposition 1, the printed values of Table 7, and a library optimizer for the update).
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

PAIR_QK = 0      # W_i^Q / W_i^K: rows of stored W_q and rows of stored W_k are aligned (Eq. 4)
PAIR_VO = 1      # W_i^V / W_i^O: rows of stored W_v and columns of stored W_o (Eq. 4)
PAIR_FFN = 2     # W_in / W_out (Eq. 7)
PAIR_FFN_GATED = 3   # W_1 = W_gate (.) W_up, W_2 = W_down (footnote to Eq. 8; App. B.2)

ACT_GELU_ERF = 0
ACT_GELU_TANH = 1
ACT_SWIGLU = 2


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


# --------------------------------------------------------------------------------------
# Step 1: per-dimension coupled score (Eq. 10; selection criterion of Eq. 12)
# --------------------------------------------------------------------------------------
def coupled_score(kind: int, w1, w2, groups: int, n: int, unit: int = 1, w1b=None, rep1: int = 1,
                  rep2: int = 1) -> np.ndarray:
    """upsilon[g, u] = r[g, u] / ||r[g, :]||_2 with r = ||a||_2 * ||b||_2 over each unit.

    a_j is stored row j of ``w1`` (of the elementwise product ``w1 * w1b`` for the gated
    FFN); b_j is stored row j of ``w2`` for the QK pair and stored column j of ``w2``
    otherwise.  For ``unit > 1`` the norms are Frobenius norms over the unit's rows/columns.
    An all-zero group scores 0 everywhere.

    Grouped-query attention (Eq. 5): the pairs W_i^Q W_g(i)^K^T of the rep1 query heads of a group
    share the inner dimensions of one key head, so dimension j leaves all of them together; a_j is then
    column j of the group's query matrices stacked on each other, i.e. ||a_j||^2 adds the rep1 heads'
    squared norms (``w1`` holds groups * rep1 heads of n rows, the heads of a group side by side).  In
    the same way rep2 heads of W^O share one value head (``w2`` holds groups * rep2 heads of n columns).
    """
    w1 = _f64(w1)
    w2 = _f64(w2)
    if kind == PAIR_FFN_GATED:
        w1 = w1 * _f64(w1b)
    assert n % unit == 0 and w1.shape[0] == groups * rep1 * n
    a_sq = (w1 * w1).sum(axis=1).reshape(groups, rep1, n).sum(axis=1).reshape(-1)
    if kind == PAIR_QK:
        assert w2.shape[0] == groups * rep2 * n
        b_sq = (w2 * w2).sum(axis=1)
    else:
        assert w2.shape[1] == groups * rep2 * n
        b_sq = (w2 * w2).sum(axis=0)
    b_sq = b_sq.reshape(groups, rep2, n).sum(axis=1).reshape(-1)
    nu = n // unit
    a_u = a_sq.reshape(groups, nu, unit).sum(axis=2)
    b_u = b_sq.reshape(groups, nu, unit).sum(axis=2)
    r = np.sqrt(a_u) * np.sqrt(b_u)
    nrm = np.sqrt((r * r).sum(axis=1, keepdims=True))
    out = np.zeros_like(r)
    np.divide(r, nrm, out=out, where=nrm > 0)
    return out


# --------------------------------------------------------------------------------------
# Step 2: keep the k most important units (Sec. 3.2 "rank upsilon_i"; Alg. 1 removal loop)
# --------------------------------------------------------------------------------------
def select_topk(scores, k: int) -> np.ndarray:
    """Indices of the k largest scores of every row, returned ascending, as int32.

    Order: larger value first; equal values (``-0 == +0``) keep the lower index; NaN ranks
    below every number.  Exactly one index set is correct for given scores.
    """
    s = np.asarray(scores)
    assert s.ndim == 2 and 0 <= k <= s.shape[1]
    out = np.empty((s.shape[0], k), dtype=np.int32)
    for g in range(s.shape[0]):
        v = s[g].astype(np.float64)
        isnan = np.isnan(v)
        v = np.where(isnan, 0.0, v) + 0.0          # +0.0 folds -0 into +0
        # lexsort: last key is the primary one
        order = np.lexsort((np.arange(v.size), -v, isnan))
        out[g] = np.sort(order[:k])
    return out


# --------------------------------------------------------------------------------------
# Step 3: aligned gather into smaller dense matrices, and its inverse (Def. 1; Alg. 1)
# --------------------------------------------------------------------------------------
# --------------------------------------------------------------------------------------
# Pair-level importance (Eq. 8) and the cumulative-threshold removal rule (Alg. 1)
# --------------------------------------------------------------------------------------
def pair_fisher(kind: int, g1, g2, groups: int, n: int, n_samples: float, g1b=None, rep1: int = 1,
                rep2: int = 1) -> np.ndarray:
    """I_hat[g] of Eq. 8 for each of the ``groups`` coupled pairs of one layer.

    ``g1``, ``g2`` (and ``g1b``) are the loss gradients of the pair's matrices in the storage
    layout of the weights themselves.  For pair g the two members are the group's rows of
    ``g1`` and its rows (QK) or columns (otherwise) of ``g2``; each member contributes the
    mean of its squared entries, the two means are averaged (the factor 1/2 and 1/|W_k| of
    Eq. 8), and the result is divided by the number of samples |D|.  For the gated FFN the
    first member is the pair (W_gate, W_up) - the paper defines W_1 from both (footnote to
    Eq. 8) - so its mean runs over the entries of both gradient matrices.  With grouped-query
    attention (Eq. 5) a member is made of the rep1 (rep2) heads that share the group's inner
    dimensions, and its mean runs over all of them.
    """
    g1, g2, g1b = _f64(g1), _f64(g2), _f64(g1b)
    out = np.zeros(groups)
    for g in range(groups):
        rows1 = slice(g * rep1 * n, (g + 1) * rep1 * n)
        rows2 = slice(g * rep2 * n, (g + 1) * rep2 * n)
        first = g1[rows1]
        if kind == PAIR_FFN_GATED:
            first = np.concatenate([first, g1b[rows1]])
        second = g2[rows2] if kind == PAIR_QK else g2[:, rows2]
        out[g] = 0.5 * ((first ** 2).sum() / first.size + (second ** 2).sum() / second.size) / n_samples
    return out


def theta_mass(scores) -> np.ndarray:
    """Integer mass of each score used by the threshold rule: floor(min(max(s, 0), 1) * 2^32), NaN -> 0.

    The rule compares sums of scores with a threshold; summing integers makes that comparison
    independent of the order of summation, so that exactly one result is correct.
    """
    s = np.asarray(scores, dtype=np.float32).astype(np.float64)
    s = np.where(np.isnan(s), 0.0, s)
    return np.floor(np.clip(s, 0.0, 1.0) * 4294967296.0).astype(np.uint64)


def select_theta(scores, theta: float):
    """Alg. 1's removal loop for each row of ``scores[groups, n_units]``: the unit with the smallest score
    is removed while the units that remain still hold at least the fraction ``theta`` of the group's
    total score (the scores of a group are compared as fractions of their sum, which leaves the ranking
    of Eq. 10 untouched); at least one unit is always kept.

    Order of removal: ascending score under the ordering of select_topk (NaN first, -0 = +0), and among
    equal scores the higher index first, so that ties keep the lower index.  Masses are the integers of
    theta_mass(); the kept-mass bound is ceil(theta * total) evaluated in fp64.
    Returns (idx, k): idx[g] holds the k[g] kept indices in ascending order, padded with -1.
    """
    sc = np.asarray(scores, dtype=np.float32)
    if sc.ndim == 1:
        sc = sc[None, :]
    groups, n = sc.shape
    idx = np.full((groups, n), -1, dtype=np.int32)
    ks = np.zeros(groups, dtype=np.int32)
    theta = float(np.float32(theta))
    for g in range(groups):
        row = sc[g]
        q = [int(v) for v in theta_mass(row)]
        total = sum(q)
        bound = int(np.ceil(np.float64(theta) * np.float64(total)))
        key = np.where(np.isnan(row), -np.inf, row.astype(np.float64))
        key = np.where(key == 0.0, 0.0, key)
        order = sorted(range(n), key=lambda i: (key[i], -i))      # removal order
        kept_mass, removed = total, set()
        for i in order:
            if len(removed) == n - 1 or kept_mass - q[i] < bound:
                break
            kept_mass -= q[i]
            removed.add(i)
        kept = [i for i in range(n) if i not in removed]
        ks[g] = len(kept)
        idx[g, :len(kept)] = kept
    return idx, ks


def select_pairs(fisher, n_select: int) -> np.ndarray:
    """Alg. 1's choice among the coupled pairs: the n_select pairs whose importance (Eq. 8) is smallest,
    as ascending int32 indices.  Smaller value first, NaN before every number, ``-0 == +0``, equal
    values go to the lower index."""
    f = [float(v) for v in np.asarray(fisher).reshape(-1)]
    assert 0 <= n_select <= len(f)
    left = list(range(len(f)))
    chosen = []
    for _ in range(n_select):                      # repeatedly take the least important pair still left
        best = left[0]
        for i in left[1:]:
            if f[best] != f[best]:                 # a NaN already leads; an earlier index keeps it
                break
            if f[i] != f[i] or f[i] < f[best]:
                best = i
        left.remove(best)
        chosen.append(best)
    return np.array(sorted(chosen), dtype=np.int32)


def compact_ragged(src, idx, ks, axis: int, n: int, kp: int, unit: int = 1) -> np.ndarray:
    """Aligned gather with a kept count of its own for every group (what the removal loop of Alg. 1
    leaves): group g keeps the units idx[g, :ks[g]]; every group is padded with zeros to kp units, so
    the result is one dense matrix."""
    src = np.asarray(src)
    idx = np.asarray(idx)
    groups = idx.shape[0]
    vec = src.ndim == 1
    m = src.reshape(1, -1) if vec else (src.T if axis == 0 else src)       # inner axis last
    out = np.zeros((m.shape[0], groups * kp * unit), dtype=src.dtype)
    for g in range(groups):
        assert 0 <= ks[g] <= kp
        for i in range(int(ks[g])):
            for u in range(unit):
                out[:, (g * kp + i) * unit + u] = m[:, g * n + int(idx[g, i]) * unit + u]
    return out.reshape(-1) if vec else (out.T if axis == 0 else out)


def scatter_ragged(cmp, idx, ks, axis: int, n: int, kp: int, unit: int = 1, base=None) -> np.ndarray:
    """Inverse of :func:`compact_ragged`: kept units back in place, zeros everywhere else - or, with `base`
    (a full-size array), the contents of `base` everywhere else: compact parameters and optimizer state
    written back before the importance is estimated again (Alg. 1: only what was kept has been updated)."""
    cmp = np.asarray(cmp)
    idx = np.asarray(idx)
    groups = idx.shape[0]
    vec = cmp.ndim == 1
    m = cmp.reshape(1, -1) if vec else (cmp.T if axis == 0 else cmp)
    if base is None:
        out = np.zeros((m.shape[0], groups * n), dtype=cmp.dtype)
    else:
        base = np.asarray(base)
        out = (base.reshape(1, -1) if vec else (base.T if axis == 0 else base)).astype(cmp.dtype, copy=True)
        assert out.shape == (m.shape[0], groups * n)
    for g in range(groups):
        for i in range(int(ks[g])):
            for u in range(unit):
                out[:, g * n + int(idx[g, i]) * unit + u] = m[:, (g * kp + i) * unit + u]
    return out.reshape(-1) if vec else (out.T if axis == 0 else out)


def individual_keep(w1, w2, n: int, k: int):
    """The baseline of Appendix A (Def. 2, individual sparsification), for one pair with a single group:
    the k inner dimensions of W_1 with the largest ||a_j|| and, independently, the k of W_2 with the
    largest ||b_j|| (ties keep the lower index, as everywhere).  Returns (idx_1, idx_2), ascending int32
    [1, k] each; gathering W_1 with idx_1 and W_2 with idx_2 re-pairs whatever is left, position by position."""
    w1, w2 = _f64(w1), _f64(w2)
    na = np.sqrt((w1 * w1).sum(axis=1))          # ||a_j||: rows of stored W_1
    nb = np.sqrt((w2 * w2).sum(axis=0))          # ||b_j||: columns of stored W_2
    assert na.size == n and nb.size == n
    return select_topk(na[None, :], k), select_topk(nb[None, :], k)


def kept_positions(idx, n: int, unit: int = 1) -> np.ndarray:
    """Flat positions, over all groups, of the kept inner dimensions (ascending per group)."""
    idx = np.asarray(idx, dtype=np.int64)
    g = np.arange(idx.shape[0], dtype=np.int64)[:, None, None]
    u = np.arange(unit, dtype=np.int64)[None, None, :]
    return (g * n + idx[:, :, None] * unit + u).reshape(-1)


def compact(src, idx, axis: int, n: int, unit: int = 1) -> np.ndarray:
    """Keep the rows (axis 0) or columns (axis 1) named by idx[groups, k], in that order."""
    pos = kept_positions(idx, n, unit)
    src = np.asarray(src)
    return src[pos] if axis == 0 else src[:, pos]


def scatter(cmp, idx, axis: int, n: int, unit: int = 1, groups: int | None = None) -> np.ndarray:
    """Inverse of :func:`compact`: kept rows/columns back in place, zeros elsewhere."""
    idx = np.asarray(idx)
    groups = idx.shape[0] if groups is None else groups
    pos = kept_positions(idx, n, unit)
    cmp = np.asarray(cmp)
    if cmp.ndim == 1:
        out = np.zeros(groups * n, dtype=cmp.dtype)
        out[pos] = cmp
    elif axis == 0:
        out = np.zeros((groups * n, cmp.shape[1]), dtype=cmp.dtype)
        out[pos] = cmp
    else:
        out = np.zeros((cmp.shape[0], groups * n), dtype=cmp.dtype)
        out[:, pos] = cmp
    return out


# --------------------------------------------------------------------------------------
# Step 4/5, FFN block (Eq. 3; gated form of the footnote to Eq. 8)
# --------------------------------------------------------------------------------------
def _gelu(hh, act):
    if act == ACT_GELU_ERF:
        return hh * 0.5 * (1.0 + _erf(hh / np.sqrt(2.0)))
    c = np.sqrt(2.0 / np.pi)
    return 0.5 * hh * (1.0 + np.tanh(c * (hh + 0.044715 * hh ** 3)))


def _gelu_grad(hh, act):
    if act == ACT_GELU_ERF:
        cdf = 0.5 * (1.0 + _erf(hh / np.sqrt(2.0)))
        pdf = np.exp(-0.5 * hh * hh) / np.sqrt(2.0 * np.pi)
        return cdf + hh * pdf
    c = np.sqrt(2.0 / np.pi)
    u = c * (hh + 0.044715 * hh ** 3)
    th = np.tanh(u)
    return 0.5 * (1.0 + th) + 0.5 * hh * (1.0 - th * th) * c * (1.0 + 3 * 0.044715 * hh * hh)


def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def ffn_fwd(x, w1, b1, w2, b2, act: int, w1b=None):
    """Y = act(X W_1^T + b_1) W_2^T + b_2; gated: A = silu(X W_gate^T) * (X W_up^T).

    Returns (Y, saved) with saved = dict(h=..., hu=..., a=...).
    """
    x, w1, w2, w1b, b1, b2 = map(_f64, (x, w1, w2, w1b, b1, b2))
    h = x @ w1.T
    if b1 is not None:
        h = h + b1
    if act == ACT_SWIGLU:
        hu = x @ w1b.T
        a = h * _sigmoid(h) * hu
    else:
        hu = None
        a = _gelu(h, act)
    y = a @ w2.T
    if b2 is not None:
        y = y + b2
    return y, {"h": h, "hu": hu, "a": a}


def ffn_bwd(x, dy, w1, w2, act: int, saved, w1b=None):
    """Gradients of L = <dY, Y> for :func:`ffn_fwd` (plain chain rule).

    Returns dict(dx, dw1, db1, dw2, db2[, dw1b]).
    """
    x, dy, w1, w2, w1b = map(_f64, (x, dy, w1, w2, w1b))
    h, hu, a = saved["h"], saved["hu"], saved["a"]
    g = {"dw2": dy.T @ a, "db2": dy.sum(axis=0)}
    da = dy @ w2
    if act == ACT_SWIGLU:
        sg = _sigmoid(h)
        dh = da * hu * sg * (1.0 + h * (1.0 - sg))
        dhu = da * h * sg
        g["dw1b"] = dhu.T @ x
        g["dx"] = dh @ w1 + dhu @ w1b
    else:
        dh = da * _gelu_grad(h, act)
        g["dx"] = dh @ w1
    g["dw1"] = dh.T @ x
    g["db1"] = dh.sum(axis=0)
    return g


# --------------------------------------------------------------------------------------
# Step 4/5, attention block (Eq. 1-2, rewritten per head as Eq. 4; rotary form Eq. 6)
# --------------------------------------------------------------------------------------
def rope_angles(idx_blocks, L: int, d_h: int, base: float = 10000.0) -> np.ndarray:
    """angle[h, t, i] = t * base^(-2 p / d_h) for the kept rotary block p = idx_blocks[h, i].

    Blocks keep the frequency they had in the unpruned head of width d_h (the position
    matrices are "adjusted to match the new dimensions", footnote to Eq. 10).
    """
    p = np.asarray(idx_blocks, dtype=np.float64)
    theta = base ** (-2.0 * p / d_h)
    t = np.arange(L, dtype=np.float64)
    return t[None, :, None] * theta[:, None, :]


def _rotate(z, ang):
    """Rotate adjacent pairs (2i, 2i+1) of the last axis of z[L, k] by ang[L, k/2]."""
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(z)
    z0, z1 = z[:, 0::2], z[:, 1::2]
    out[:, 0::2] = z0 * c - z1 * s
    out[:, 1::2] = z0 * s + z1 * c
    return out


def attn_fwd(x, wq, wk, wv, wo, B: int, L: int, scale: float, causal: bool,
             bq=None, bk=None, bv=None, bo=None, angles=None):
    """Multi-head attention on per-head matrices.

    wq, wk: [h, k_qk, d]; wv: [h, k_vo, d]; wo: [h, d, k_vo] (head i's columns of W^O);
    optional biases bq, bk: [h, k_qk], bv: [h, k_vo], bo: [d]; angles: [h, L, k_qk/2] or None.
    Y[b] = sum_i softmax(scale * Q_i K_i^T (+ causal mask)) V_i W_o,i^T + b_o.
    Grouped-query attention (Eq. 5): wk, wv (bk, bv) may hold fewer heads, h_kv dividing h; query head i
    then uses key/value head g(i) = i // (h / h_kv) (its angles are those of the query head).
    Returns (Y[B*L, d], saved) where saved holds q, k (rotated), v, p, o per (b, head).
    """
    x, wq, wk, wv, wo, bq, bk, bv, bo = map(_f64, (x, wq, wk, wv, wo, bq, bk, bv, bo))
    h = wq.shape[0]
    m = h // wk.shape[0]                          # query heads per key/value head
    assert wk.shape[0] * m == h and wv.shape[0] == wk.shape[0]
    d = x.shape[1]
    y = np.zeros((B * L, d))
    sv = {"q": {}, "k": {}, "v": {}, "p": {}, "o": {}}
    mask = np.triu(np.ones((L, L), dtype=bool), k=1) if causal else None
    for b in range(B):
        xb = x[b * L:(b + 1) * L]
        for i in range(h):
            q = xb @ wq[i].T
            k = xb @ wk[i // m].T
            v = xb @ wv[i // m].T
            if bq is not None:
                q = q + bq[i]
            if bk is not None:
                k = k + bk[i // m]
            if bv is not None:
                v = v + bv[i // m]
            if angles is not None:
                q = _rotate(q, angles[i])
                k = _rotate(k, angles[i])
            s = (q @ k.T) * scale
            if causal:
                s = np.where(mask, -np.inf, s)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=1, keepdims=True)
            o = p @ v
            y[b * L:(b + 1) * L] += o @ wo[i].T
            for nm, val in (("q", q), ("k", k), ("v", v), ("p", p), ("o", o)):
                sv[nm][(b, i)] = val
    if bo is not None:
        y = y + bo
    return y, sv


def attn_bwd(x, dy, wq, wk, wv, wo, B: int, L: int, scale: float, saved, angles=None):
    """Gradients of L = <dY, Y> for :func:`attn_fwd`.

    Returns dict(dx, dwq, dwk, dwv, dwo, dbq, dbk, dbv, dbo) in the per-head shapes of the inputs.
    """
    x, dy, wq, wk, wv, wo = map(_f64, (x, dy, wq, wk, wv, wo))
    h = wq.shape[0]
    m = h // wk.shape[0]                          # query heads per key/value head (Eq. 5)
    g = {"dx": np.zeros_like(x), "dwq": np.zeros_like(wq), "dwk": np.zeros_like(wk),
         "dwv": np.zeros_like(wv), "dwo": np.zeros_like(wo),
         "dbq": np.zeros(wq.shape[:2]), "dbk": np.zeros(wk.shape[:2]), "dbv": np.zeros(wv.shape[:2]),
         "dbo": dy.sum(axis=0)}
    for b in range(B):
        sl = slice(b * L, (b + 1) * L)
        xb, dyb = x[sl], dy[sl]
        for i in range(h):
            q, k, v, p, o = (saved[nm][(b, i)] for nm in ("q", "k", "v", "p", "o"))
            do = dyb @ wo[i]
            g["dwo"][i] += dyb.T @ o
            dv = p.T @ do
            dp = do @ v.T
            ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
            dq = scale * (ds @ k)
            dk = scale * (ds.T @ q)
            if angles is not None:
                dq = _rotate(dq, -angles[i])
                dk = _rotate(dk, -angles[i])
            g["dwq"][i] += dq.T @ xb
            g["dwk"][i // m] += dk.T @ xb
            g["dwv"][i // m] += dv.T @ xb
            g["dbq"][i] += dq.sum(axis=0)
            g["dbk"][i // m] += dk.sum(axis=0)
            g["dbv"][i // m] += dv.sum(axis=0)
            g["dx"][sl] += dq @ wq[i] + dk @ wk[i // m] + dv @ wv[i // m]
    return g


# --------------------------------------------------------------------------------------
# Parameter update on the compact tensors (Alg. 1 "Update W"; AdamW is the optimizer of the GPT-2 and
# DeiT runs of Sec. 4.1, and Alg. 1 removes the moments of removed rows/columns with them)
# --------------------------------------------------------------------------------------
def adamw_step(w, g, m, v, t: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
               weight_decay: float = 0.01):
    """One AdamW update (Adam with decoupled weight decay, Loshchilov & Hutter) of step number t >= 1.

    m' = beta1 m + (1 - beta1) g,  v' = beta2 v + (1 - beta2) g^2,
    w' = w - lr * ( (m' / (1 - beta1^t)) / (sqrt(v' / (1 - beta2^t)) + eps) + weight_decay * w ).
    Returns (w', m', v') in fp64.  Elementwise, so it acts on compact tensors exactly as on the kept
    entries of full ones.
    """
    w, g, m, v = map(_f64, (w, g, m, v))
    m1 = beta1 * m + (1.0 - beta1) * g
    v1 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m1 / (1.0 - beta1 ** t)
    vhat = v1 / (1.0 - beta2 ** t)
    w1 = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    return w1, m1, v1


# --------------------------------------------------------------------------------------
# helpers for tests: per-head views of stored matrices
# --------------------------------------------------------------------------------------
def heads_rows(w, h: int) -> np.ndarray:
    """Stored [h*k, d] -> [h, k, d]."""
    w = np.asarray(w)
    return w.reshape(h, w.shape[0] // h, w.shape[1])


def heads_cols(w, h: int) -> np.ndarray:
    """Stored [d, h*k] -> [h, d, k]."""
    w = np.asarray(w)
    return np.ascontiguousarray(w.reshape(w.shape[0], h, w.shape[1] // h).transpose(1, 0, 2))


def rel_fro(a, b) -> float:
    """||a - b||_F / ||b||_F (b is the reference); 0 if both are zero."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    num = np.linalg.norm(a - b)
    return float(num / den) if den > 0 else float(num)
