"""Pins for the oracle's choice among coupled pairs (Alg. 1, "top-K with smallest importance") and its
aligned gather/scatter with a kept count per group, against library sorts, the uniform gather (pinned
elsewhere), adjointness, and the exactness of zero padding in the attention and FFN maths (no GPU, no
product code)."""
import numpy as np
import pytest

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import synth


# ---- choice among pairs ---------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(4))
def test_select_pairs_distinct_values_is_a_sort(seed):
    rng = np.random.default_rng(seed)
    f = rng.permutation(np.arange(37)).astype(np.float32) * np.float32(0.25) - np.float32(3.0)
    for m in (1, 5, 36, 37):
        want = np.sort(np.argsort(f, kind="stable")[:m])
        assert np.array_equal(O.select_pairs(f, m), want)
        # without ties the chosen pairs are exactly those the (separately pinned) top-k leaves out
        rest = O.select_topk(f[None, :], 37 - m)[0]
        assert sorted(set(range(37)) - set(rest.tolist())) == want.tolist()


def test_select_pairs_ties_nan_and_signed_zero():
    f = np.array([0.5, 0.25, 0.25, np.nan, 0.25, -0.0, 0.0, 1.0], dtype=np.float32)
    assert O.select_pairs(f, 1).tolist() == [3]                    # NaN: least important
    assert O.select_pairs(f, 2).tolist() == [3, 5]                 # -0 == +0: lower index
    assert O.select_pairs(f, 3).tolist() == [3, 5, 6]
    assert O.select_pairs(f, 5).tolist() == [1, 2, 3, 5, 6]        # of three equal values the two lower indices
    assert O.select_pairs(f, 8).tolist() == list(range(8))
    assert O.select_pairs(f, 0).size == 0


def test_select_pairs_every_chosen_value_is_not_above_any_other():
    rng = np.random.default_rng(7)
    f = rng.integers(0, 6, 50).astype(np.float32)
    for m in (3, 17, 40):
        c = O.select_pairs(f, m)
        rest = np.setdiff1d(np.arange(50), c)
        assert len(c) == m and f[c].max() <= f[rest].min()
        edge = f[c].max()                                            # ties at the boundary go to the lower index
        tied_in, tied_out = c[f[c] == edge], rest[f[rest] == edge]
        assert tied_out.size == 0 or tied_in.max() < tied_out.min()


# ---- ragged gather / scatter ------------------------------------------------------------------
def _ragged_case(seed, groups, n, unit):
    rng = np.random.default_rng(seed)
    nu = n // unit
    ks = rng.integers(0, nu + 1, groups)
    ks[0] = nu
    idx = -np.ones((groups, nu), dtype=np.int32)
    for g in range(groups):
        idx[g, :ks[g]] = np.sort(rng.choice(nu, ks[g], replace=False))
    return idx, ks.astype(np.int32)


@pytest.mark.parametrize("axis", (0, 1))
@pytest.mark.parametrize("unit", (1, 2))
def test_ragged_gather_with_equal_counts_is_the_uniform_gather_padded(axis, unit):
    groups, n, k, kp = 3, 8, 3, 4
    rng = np.random.default_rng(2)
    idx = np.stack([np.sort(rng.choice(n // unit, k, replace=False)) for _ in range(groups)]).astype(np.int32)
    w = synth.normal(9, 1, (groups * n, 5) if axis == 0 else (5, groups * n)).astype(np.float64)
    got = O.compact_ragged(w, idx, np.full(groups, k), axis, n, kp, unit)
    uni = O.compact(w, idx, axis, n, unit)
    gm, um = (got.T, uni.T) if axis == 0 else (got, uni)
    gm = gm.reshape(5, groups, kp * unit)
    np.testing.assert_array_equal(gm[:, :, :k * unit].reshape(5, -1), um)
    assert np.all(gm[:, :, k * unit:] == 0)


@pytest.mark.parametrize("axis", (0, 1))
@pytest.mark.parametrize("unit", (1, 2))
def test_ragged_scatter_inverts_gather_and_is_its_adjoint(axis, unit):
    groups, n = 4, 12
    idx, ks = _ragged_case(5, groups, n, unit)
    kp = n // unit + 1
    w = synth.normal(10, 1, (groups * n, 6) if axis == 0 else (6, groups * n)).astype(np.float64)
    c = O.compact_ragged(w, idx, ks, axis, n, kp, unit)
    back = O.scatter_ragged(c, idx, ks, axis, n, kp, unit)
    keep = np.zeros(groups * n, dtype=bool)
    for g in range(groups):
        for i in idx[g, :ks[g]]:
            keep[g * n + i * unit:g * n + (i + 1) * unit] = True
    want = np.where(keep[:, None], w, 0.0) if axis == 0 else np.where(keep[None, :], w, 0.0)
    np.testing.assert_array_equal(back, want)
    y = synth.normal(10, 2, c.shape).astype(np.float64)
    np.testing.assert_allclose((c * y).sum(), (w * O.scatter_ragged(y, idx, ks, axis, n, kp, unit)).sum(), rtol=1e-13)
    # vectors (biases) follow the same map
    b = synth.normal(10, 3, (groups * n,)).astype(np.float64)
    cb = O.compact_ragged(b, idx, ks, 1, n, kp, unit)
    assert cb.shape == (groups * kp * unit,)
    np.testing.assert_array_equal(cb, O.compact_ragged(b[None, :], idx, ks, 1, n, kp, unit)[0])


@pytest.mark.parametrize("axis", (0, 1))
@pytest.mark.parametrize("unit", (1, 2))
def test_scatter_into_a_base_touches_only_the_kept_slots(axis, unit):
    groups, n = 3, 12
    idx, ks = _ragged_case(8, groups, n, unit)
    kp = n // unit
    shape = (groups * n, 5) if axis == 0 else (5, groups * n)
    base = synth.normal(14, 1, shape).astype(np.float64)
    c = synth.normal(14, 2, (groups * kp * unit, 5) if axis == 0 else (5, groups * kp * unit)).astype(np.float64)
    got = O.scatter_ragged(c, idx, ks, axis, n, kp, unit, base=base)
    keep = np.zeros(groups * n, dtype=bool)
    for g in range(groups):
        for i in idx[g, :ks[g]]:
            keep[g * n + i * unit:g * n + (i + 1) * unit] = True
    km = keep[:, None] if axis == 0 else keep[None, :]
    # outside the kept slots the base survives, inside them the zero-filling scatter's values stand
    np.testing.assert_array_equal(np.where(km, 0.0, got), np.where(km, 0.0, base))
    np.testing.assert_array_equal(np.where(km, got, 0.0), O.scatter_ragged(c, idx, ks, axis, n, kp, unit))
    # gathering again returns what was written (padding slots of c aside), and a base of zeros is the plain scatter
    back = O.compact_ragged(got, idx, ks, axis, n, kp, unit)
    np.testing.assert_array_equal(back, O.compact_ragged(O.scatter_ragged(c, idx, ks, axis, n, kp, unit), idx, ks, axis, n, kp, unit))
    np.testing.assert_array_equal(O.scatter_ragged(c, idx, ks, axis, n, kp, unit, base=np.zeros(shape)),
                                  O.scatter_ragged(c, idx, ks, axis, n, kp, unit))
    # writing back what was gathered from the base changes nothing
    np.testing.assert_array_equal(O.scatter_ragged(O.compact_ragged(base, idx, ks, axis, n, kp, unit), idx, ks, axis, n, kp, unit, base=base), base)


# ---- zero padding is exact in the layer maths: a ragged layer equals its padded dense form ---------------
def test_padded_heads_equal_the_sum_of_ragged_heads():
    """Eq. 4 is a sum over heads, each with an inner width of its own: heads of unequal width computed one
    by one give what a single call gives on the widths padded to a common size with zero rows/columns."""
    h, d, B, L = 3, 10, 2, 7
    kq, kv, kp = [2, 4, 6], [5, 1, 3], 6
    x = synth.normal(12, 0, (B * L, d)).astype(np.float64)
    dy = synth.normal(12, 9, (B * L, d)).astype(np.float64)
    wq = [synth.normal(12, 1 + i, (kq[i], d)) * 0.3 for i in range(h)]
    wk = [synth.normal(12, 11 + i, (kq[i], d)) * 0.3 for i in range(h)]
    wv = [synth.normal(12, 21 + i, (kv[i], d)) * 0.3 for i in range(h)]
    wo = [synth.normal(12, 31 + i, (d, kv[i])) * 0.3 for i in range(h)]
    ang = [O.rope_angles(np.arange(kq[i] // 2)[None, :] * 2 + i, L, 16)[0] for i in range(h)]
    y_sum, dx_sum, dwq = np.zeros((B * L, d)), np.zeros((B * L, d)), []
    for i in range(h):
        yi, sv = O.attn_fwd(x, wq[i][None], wk[i][None], wv[i][None], wo[i][None], B, L, 0.37, True, angles=ang[i][None])
        gi = O.attn_bwd(x, dy, wq[i][None], wk[i][None], wv[i][None], wo[i][None], B, L, 0.37, sv, angles=ang[i][None])
        y_sum += yi
        dx_sum += gi["dx"]
        dwq.append(gi["dwq"][0])

    def pad_rows(ws, k):
        return np.stack([np.concatenate([w, np.zeros((k - w.shape[0], d))]) for w in ws])

    wo_p = np.stack([np.concatenate([w, np.zeros((d, kp - w.shape[1]))], axis=1) for w in wo])
    ang_p = np.stack([np.concatenate([a, np.zeros((L, kp // 2 - a.shape[1]))], axis=1) for a in ang])
    wq_p, wk_p, wv_p = pad_rows(wq, kp), pad_rows(wk, kp), pad_rows(wv, kp)
    y, sv = O.attn_fwd(x, wq_p, wk_p, wv_p, wo_p, B, L, 0.37, True, angles=ang_p)
    g = O.attn_bwd(x, dy, wq_p, wk_p, wv_p, wo_p, B, L, 0.37, sv, angles=ang_p)
    np.testing.assert_allclose(y, y_sum, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dx"], dx_sum, rtol=1e-12, atol=1e-13)
    for i in range(h):
        np.testing.assert_allclose(g["dwq"][i, :kq[i]], dwq[i], rtol=1e-12, atol=1e-13)
        assert np.all(g["dwq"][i, kq[i]:] == 0) and np.all(g["dwk"][i, kq[i]:] == 0)     # padding never trains
        assert np.all(g["dwv"][i, kv[i]:] == 0) and np.all(g["dwo"][i][:, kv[i]:] == 0)


@pytest.mark.parametrize("act", (O.ACT_GELU_ERF, O.ACT_SWIGLU))
def test_padded_ffn_units_contribute_nothing(act):
    T, d, k, kp = 9, 6, 5, 8
    x = synth.normal(13, 0, (T, d)).astype(np.float64)
    dy = synth.normal(13, 1, (T, d)).astype(np.float64)
    w1, w2 = synth.normal(13, 2, (k, d)) * 0.5, synth.normal(13, 3, (d, k)) * 0.5
    w1b = synth.normal(13, 4, (k, d)) * 0.5 if act == O.ACT_SWIGLU else None
    z = np.zeros((kp - k, d))
    y0, s0 = O.ffn_fwd(x, w1, None, w2, None, act, w1b=w1b)
    y1, s1 = O.ffn_fwd(x, np.concatenate([w1, z]), None, np.concatenate([w2, z.T], axis=1), None, act,
                       w1b=None if w1b is None else np.concatenate([w1b, z]))
    np.testing.assert_allclose(y1, y0, rtol=1e-13, atol=1e-14)
    g0 = O.ffn_bwd(x, dy, w1, w2, act, s0, w1b=w1b)
    g1 = O.ffn_bwd(x, dy, np.concatenate([w1, z]), np.concatenate([w2, z.T], axis=1), act, s1,
                   w1b=None if w1b is None else np.concatenate([w1b, z]))
    np.testing.assert_allclose(g1["dx"], g0["dx"], rtol=1e-13, atol=1e-14)
    assert np.all(g1["dw1"][k:] == 0) and np.all(g1["dw2"][:, k:] == 0)
