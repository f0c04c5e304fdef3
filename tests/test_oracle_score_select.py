"""Pins for the oracle's score / select / compact steps against facts the paper and the
mathematics fix (no GPU, no product code)."""
import itertools
import os

import numpy as np
import pytest

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import synth


def _pair(seed, m, n, p, std=1.0):
    """A[m,n] with columns a_j, B[n,p] with rows b_j (the paper's Appendix A notation),
    returned in storage layout: w1 = A^T [n,m], w2 = B^T [p,n]."""
    A = synth.normal(seed, 100, (m, n), std).astype(np.float64)
    Bm = synth.normal(seed, 101, (n, p), std).astype(np.float64)
    return A, Bm, np.ascontiguousarray(A.T), np.ascontiguousarray(Bm.T)


# ---- score -----------------------------------------------------------------------------
def test_score_unit_l2_norm_and_scaling_invariance():
    _, _, w1, w2 = _pair(1, 24, 40, 17)
    v = O.coupled_score(O.PAIR_FFN, w1, w2, 1, 40)
    assert v.shape == (1, 40)
    assert abs(np.linalg.norm(v) - 1.0) < 1e-14
    # Eq. 10 is homogeneous of degree 0 in each matrix
    v2 = O.coupled_score(O.PAIR_FFN, 3.5 * w1, 0.01 * w2, 1, 40)
    np.testing.assert_allclose(v2, v, rtol=1e-13)
    # moving a factor c_j from a_j to b_j leaves a_j b_j^T, hence the score, unchanged
    c = np.exp(synth.normal(1, 102, (40,)).astype(np.float64))
    v3 = O.coupled_score(O.PAIR_FFN, w1 * c[:, None], w2 / c[None, :], 1, 40)
    np.testing.assert_allclose(v3, v, rtol=1e-12)


def test_score_is_norm_of_removed_outer_product():
    """Eq. 12: ||a_j b_j^T||_F = ||a_j|| ||b_j||; check against the explicit rank-1 matrices."""
    A, Bm, w1, w2 = _pair(2, 9, 7, 11)
    r = np.array([np.linalg.norm(np.outer(A[:, j], Bm[j])) for j in range(7)])
    v = O.coupled_score(O.PAIR_FFN, w1, w2, 1, 7)[0]
    np.testing.assert_allclose(v, r / np.linalg.norm(r), rtol=1e-13)


def test_score_tsvd_special_case_matches_lapack():
    """Eq. 9: with W_1 = U Sigma^(1/2), W_2 = Sigma^(1/2) V^T the pair norms are the singular
    values, so upsilon = sigma / ||sigma||_2 and top-k is the Eckart-Young truncation."""
    M = synth.normal(3, 103, (30, 22)).astype(np.float64)
    U, s, Vt = np.linalg.svd(M, full_matrices=False)
    perm = np.random.Generator(np.random.Philox(key=[3, 9])).permutation(22)
    A = (U * np.sqrt(s))[:, perm]            # columns a_j
    Bm = (np.sqrt(s)[:, None] * Vt)[perm]    # rows b_j
    v = O.coupled_score(O.PAIR_FFN, A.T.copy(), Bm.T.copy(), 1, 22)[0]
    np.testing.assert_allclose(v, s[perm] / np.linalg.norm(s), rtol=1e-10)
    for k in (1, 5, 21):
        idx = O.select_topk(v[None].astype(np.float32), k)
        Ac = O.compact(A.T.copy(), idx, 0, 22).T
        Bc = O.compact(Bm.T.copy(), idx, 1, 22).T
        err = np.linalg.norm(M - Ac @ Bc)
        assert abs(err - np.sqrt((s[k:] ** 2).sum())) < 1e-10


def test_score_qk_uses_rows_of_both_and_groups_normalise_separately():
    h, dh, d = 3, 8, 10
    wq = synth.normal(4, 104, (h * dh, d)).astype(np.float64)
    wk = synth.normal(4, 105, (h * dh, d)).astype(np.float64)
    v = O.coupled_score(O.PAIR_QK, wq, wk, h, dh)
    assert v.shape == (h, dh)
    np.testing.assert_allclose(np.linalg.norm(v, axis=1), 1.0, rtol=1e-14)
    for g in range(h):
        for j in range(dh):
            # ||column j of W_i^Q W_i^K^T's rank-1 term||_F
            r = np.linalg.norm(np.outer(wq[g * dh + j], wk[g * dh + j]))
            rn = np.sqrt(sum(np.linalg.norm(np.outer(wq[g * dh + t], wk[g * dh + t])) ** 2 for t in range(dh)))
            assert abs(v[g, j] - r / rn) < 1e-13
    # scaling one head must not change another head's scores
    wq2 = wq.copy()
    wq2[:dh] *= 7.0
    np.testing.assert_allclose(O.coupled_score(O.PAIR_QK, wq2, wk, h, dh), v, rtol=1e-13)


def test_score_vo_uses_columns_of_wo():
    h, dh, d = 2, 4, 6
    wv = synth.normal(5, 104, (h * dh, d)).astype(np.float64)
    wo = synth.normal(5, 105, (d, h * dh)).astype(np.float64)
    v = O.coupled_score(O.PAIR_VO, wv, wo, h, dh)
    for g in range(h):
        r = np.array([np.linalg.norm(np.outer(wv[g * dh + j], wo[:, g * dh + j])) for j in range(dh)])
        np.testing.assert_allclose(v[g], r / np.linalg.norm(r), rtol=1e-13)


def test_score_rotary_block_is_rotation_invariant():
    """Eq. 6: W^Q P_t only rotates each 2-dim block, so the unit=2 score cannot depend on t, s."""
    h, dh, d = 2, 8, 12
    wq = synth.normal(6, 104, (h * dh, d)).astype(np.float64)
    wk = synth.normal(6, 105, (h * dh, d)).astype(np.float64)
    v = O.coupled_score(O.PAIR_QK, wq, wk, h, dh, unit=2)
    assert v.shape == (h, dh // 2)

    def rot(w, t):
        out = w.copy()
        for g in range(h):
            for p in range(dh // 2):
                th = t * 10000.0 ** (-2.0 * p / dh)
                c, s = np.cos(th), np.sin(th)
                r0, r1 = w[g * dh + 2 * p], w[g * dh + 2 * p + 1]
                out[g * dh + 2 * p] = c * r0 - s * r1
                out[g * dh + 2 * p + 1] = s * r0 + c * r1
        return out

    v2 = O.coupled_score(O.PAIR_QK, rot(wq, 17.0), rot(wk, 3.0), h, dh, unit=2)
    np.testing.assert_allclose(v2, v, rtol=1e-12)
    # and unit=2 is the Frobenius norm over the two rows
    a = np.sqrt((wq[0] ** 2).sum() + (wq[1] ** 2).sum())
    b = np.sqrt((wk[0] ** 2).sum() + (wk[1] ** 2).sum())
    a2 = np.sqrt((wq[2] ** 2).sum() + (wq[3] ** 2).sum())
    b2 = np.sqrt((wk[2] ** 2).sum() + (wk[3] ** 2).sum())
    assert abs(v[0, 0] / v[0, 1] - (a * b) / (a2 * b2)) < 1e-12


def test_score_gated_is_hadamard_of_gate_and_up():
    n, d = 6, 5
    wg = synth.normal(7, 104, (n, d)).astype(np.float64)
    wu = synth.normal(7, 105, (n, d)).astype(np.float64)
    wd = synth.normal(7, 106, (d, n)).astype(np.float64)
    v = O.coupled_score(O.PAIR_FFN_GATED, wg, wd, 1, n, w1b=wu)[0]
    r = np.array([np.sqrt(sum((wg[j, i] * wu[j, i]) ** 2 for i in range(d))) * np.linalg.norm(wd[:, j])
                  for j in range(n)])
    np.testing.assert_allclose(v, r / np.linalg.norm(r), rtol=1e-13)
    # it is NOT the product of the separate row norms
    r_wrong = np.linalg.norm(wg, axis=1) * np.linalg.norm(wu, axis=1) * np.linalg.norm(wd, axis=0)
    assert np.abs(v - r_wrong / np.linalg.norm(r_wrong)).max() > 1e-3


def test_score_zero_group_is_zero():
    v = O.coupled_score(O.PAIR_FFN, np.zeros((4, 3)), np.ones((3, 4)), 1, 4)
    assert np.all(v == 0)


# ---- select ----------------------------------------------------------------------------
def _brute_select(v, k):
    """Lexicographically smallest subset among those maximising the kept score mass."""
    best, best_sum = None, -np.inf
    for c in itertools.combinations(range(len(v)), k):
        s = float(sum(sorted(v[list(c)])))  # order independent sum
        if s > best_sum + 1e-15:
            best, best_sum = c, s
    return np.array(best, dtype=np.int32)


@pytest.mark.parametrize("n,k", [(6, 1), (6, 3), (7, 6), (8, 4), (9, 9), (5, 0)])
def test_select_matches_brute_force_distinct(n, k):
    v = np.abs(synth.normal(11 + n, 110, (n,))).astype(np.float32)
    idx = O.select_topk(v[None], k)[0]
    if k == 0:
        assert idx.size == 0
        return
    np.testing.assert_array_equal(idx, _brute_select(v.astype(np.float64), k))
    assert np.all(np.diff(idx) > 0)


def test_select_ties_keep_lower_index():
    v = np.array([[0.5, 0.25, 0.5, 0.25, 0.5, 0.25, 0.125, 0.5]], dtype=np.float32)
    np.testing.assert_array_equal(O.select_topk(v, 2)[0], [0, 2])
    np.testing.assert_array_equal(O.select_topk(v, 5)[0], [0, 1, 2, 4, 7])
    np.testing.assert_array_equal(O.select_topk(v, 6)[0], [0, 1, 2, 3, 4, 7])
    # exactly-tied values, powers of two so sums are exact: brute force agrees
    for k in range(1, 8):
        np.testing.assert_array_equal(O.select_topk(v, k)[0], _brute_select(v[0].astype(np.float64), k))
    # all equal -> first k
    np.testing.assert_array_equal(O.select_topk(np.zeros((1, 9), np.float32), 4)[0], [0, 1, 2, 3])


def test_select_signed_zero_and_nan():
    v = np.array([[-0.0, 0.0, np.nan, 1.0, -1.0, np.nan, 0.0]], dtype=np.float32)
    np.testing.assert_array_equal(O.select_topk(v, 1)[0], [3])
    np.testing.assert_array_equal(O.select_topk(v, 3)[0], [0, 1, 3])      # -0 ties with +0
    np.testing.assert_array_equal(O.select_topk(v, 5)[0], [0, 1, 3, 4, 6])
    np.testing.assert_array_equal(O.select_topk(v, 6)[0], [0, 1, 2, 3, 4, 6])  # NaN last, lower index first


def test_select_n_minus_1_drops_argmin_pair():
    """Def. 1 / Eq. 12: one removal takes the pair with minimal ||a_j|| ||b_j||."""
    A, Bm, w1, w2 = _pair(12, 13, 21, 9)
    v = O.coupled_score(O.PAIR_FFN, w1, w2, 1, 21)
    idx = O.select_topk(v.astype(np.float32), 20)[0]
    dropped = sorted(set(range(21)) - set(idx.tolist()))
    prods = np.linalg.norm(A, axis=0) * np.linalg.norm(Bm, axis=1)
    assert dropped == [int(np.argmin(prods))]


# ---- compact / scatter -----------------------------------------------------------------
def test_compact_scatter_roundtrip_and_mask():
    G, n, d = 3, 8, 5
    w = synth.normal(13, 104, (G * n, d))
    idx = np.array([[0, 3, 7], [1, 2, 4], [5, 6, 7]], dtype=np.int32)
    c = O.compact(w, idx, 0, n)
    assert c.shape == (9, d)
    np.testing.assert_array_equal(c[4], w[8 + 2])
    full = O.scatter(c, idx, 0, n)
    mask = np.zeros(G * n, bool)
    mask[O.kept_positions(idx, n)] = True
    np.testing.assert_array_equal(full, w * mask[:, None])
    np.testing.assert_array_equal(O.compact(full, idx, 0, n), c)
    # columns, with unit 2
    wt = np.ascontiguousarray(w.T)
    idx2 = np.array([[0, 2], [1, 3], [0, 1]], dtype=np.int32)
    c2 = O.compact(wt, idx2, 1, n, unit=2)
    np.testing.assert_array_equal(c2[:, :4], wt[:, [0, 1, 4, 5]])
    np.testing.assert_array_equal(c2[:, 4:8], wt[:, [8 + 2, 8 + 3, 8 + 6, 8 + 7]])
    f2 = O.scatter(c2, idx2, 1, n, unit=2)
    np.testing.assert_array_equal(O.compact(f2, idx2, 1, n, unit=2), c2)
    # keep everything = identity
    all_idx = np.tile(np.arange(n, dtype=np.int32), (G, 1))
    np.testing.assert_array_equal(O.compact(w, all_idx, 0, n), w)


# ---- score + select + compact together ---------------------------------------------------
def test_prop1_single_removal_error_is_min_norm_product():
    """Prop. 1 (Eq. 14-15): ||AB - A_new B_new||_F = min_j ||a_j|| ||b_j||, error = a_j* b_j*^T."""
    for seed in range(5):
        A, Bm, w1, w2 = _pair(20 + seed, 15, 12, 18)
        v = O.coupled_score(O.PAIR_FFN, w1, w2, 1, 12)
        idx = O.select_topk(v.astype(np.float32), 11)
        Ac = O.compact(w1, idx, 0, 12).T
        Bc = O.compact(w2, idx, 1, 12).T
        delta = A @ Bm - Ac @ Bc
        prods = np.linalg.norm(A, axis=0) * np.linalg.norm(Bm, axis=1)
        j = int(np.argmin(prods))
        np.testing.assert_allclose(delta, np.outer(A[:, j], Bm[j]), atol=1e-12)
        assert abs(np.linalg.norm(delta) - prods.min()) < 1e-12


def test_orthogonal_columns_topk_is_brute_force_optimum():
    """With mutually orthogonal a_j the squared error is additive over removed pairs, so the
    coupled top-k minimises the true Frobenius error over all C(n,k) aligned subsets."""
    n, m, p = 7, 10, 6
    Q, _ = np.linalg.qr(synth.normal(30, 104, (m, n)).astype(np.float64))
    A = Q * np.exp(synth.normal(30, 105, (n,)).astype(np.float64))
    Bm = synth.normal(30, 106, (n, p)).astype(np.float64)
    P = A @ Bm
    v = O.coupled_score(O.PAIR_FFN, A.T.copy(), Bm.T.copy(), 1, n)
    for k in (2, 3, 5):
        idx = O.select_topk(v.astype(np.float32), k)[0]
        err = np.linalg.norm(P - A[:, idx] @ Bm[idx])
        best = min(np.linalg.norm(P - A[:, list(c)] @ Bm[list(c)])
                   for c in itertools.combinations(range(n), k))
        assert abs(err - best) < 1e-12
        removed = sorted(set(range(n)) - set(idx.tolist()))
        add = np.sqrt(sum(np.linalg.norm(A[:, j]) ** 2 * np.linalg.norm(Bm[j]) ** 2 for j in removed))
        assert abs(err - add) < 1e-12


def _table7(golden_dir):
    rows = {}
    with open(os.path.join(golden_dir, "table7_random_pairs.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                n, d1, d2, pr = line.split()
                rows[int(n)] = (float(d1), float(d2), float(pr))
    return rows


@pytest.mark.parametrize("n,trials,rtol", [(100, 1500, 0.01), (500, 120, 0.01), (1000, 40, 0.01)])
def test_table7_coupled_column(golden_dir, n, trials, rtol):
    """Table 7, coupled column: average ||Delta_1||_F over random N(0,1) n x n pairs when the
    whole chain (score -> keep n-1 -> compact -> product difference) is run."""
    want = _table7(golden_dir)[n][0]
    g = np.random.Generator(np.random.Philox(key=[77, n]))
    tot = 0.0
    for _ in range(trials):
        A = g.standard_normal((n, n))
        Bm = g.standard_normal((n, n))
        w1, w2 = A.T, Bm.T
        v = O.coupled_score(O.PAIR_FFN, w1, w2, 1, n)
        idx = O.select_topk(v.astype(np.float32), n - 1)
        Ac = O.compact(w1, idx, 0, n).T
        Bc = O.compact(w2, idx, 1, n).T
        if n <= 100:
            tot += np.linalg.norm(A @ Bm - Ac @ Bc)
        else:
            # Delta_1 = sum over removed pairs of a_j b_j^T (Eq. 14): form it from the removed pair
            j = (set(range(n)) - set(idx[0].tolist())).pop()
            tot += np.linalg.norm(np.outer(A[:, j], Bm[j]))
    got = tot / trials
    assert abs(got - want) / want < rtol, (got, want)


def test_table7_individual_column_n100(golden_dir):
    """Table 7, individual column at n=100: delete argmin||a_k|| from A and argmin||b_l|| from B
    independently, re-index, multiply (Def. 2).  Checks the paper's matrices are N(0,1) and that
    the coupled error wins with the printed frequency."""
    want1, want2, wantp = _table7(golden_dir)[100]
    g = np.random.Generator(np.random.Philox(key=[78, 100]))
    n, trials = 100, 800
    t1 = t2 = 0.0
    wins = 0
    for _ in range(trials):
        A = g.standard_normal((n, n))
        Bm = g.standard_normal((n, n))
        v = O.coupled_score(O.PAIR_FFN, A.T, Bm.T, 1, n)
        idx = O.select_topk(v.astype(np.float32), n - 1)
        d1 = np.linalg.norm(A @ Bm - O.compact(A.T, idx, 0, n).T @ O.compact(Bm.T, idx, 1, n).T)
        ka = int(np.argmin(np.linalg.norm(A, axis=0)))
        lb = int(np.argmin(np.linalg.norm(Bm, axis=1)))
        d2 = np.linalg.norm(A @ Bm - np.delete(A, ka, axis=1) @ np.delete(Bm, lb, axis=0))
        t1 += d1
        t2 += d2
        wins += d1 < d2
    assert abs(t1 / trials - want1) / want1 < 0.015
    assert abs(t2 / trials - want2) / want2 < 0.05
    assert abs(100.0 * wins / trials - wantp) < 1.5


def test_individual_keep_is_the_independent_argmin_removal():
    """Def. 2 of Appendix A with one removal: the dropped indices are the argmin of each member's own norms,
    and the re-paired product is that of numpy's delete (library routines, written independently)."""
    g = np.random.Generator(np.random.Philox(key=[79, 1]))
    for n in (5, 40):
        A, Bm = g.standard_normal((n, n + 3)).T, g.standard_normal((n, n + 2))      # A: (n+3) x n, B: n x (n+2)
        i1, i2 = O.individual_keep(A.T, Bm.T, n, n - 1)
        ka, lb = int(np.argmin(np.linalg.norm(A, axis=0))), int(np.argmin(np.linalg.norm(Bm, axis=1)))
        assert sorted(set(range(n)) - set(i1[0].tolist())) == [ka]
        assert sorted(set(range(n)) - set(i2[0].tolist())) == [lb]
        got = O.compact(A.T, i1, 0, n).T @ O.compact(Bm.T, i2, 1, n).T
        np.testing.assert_allclose(got, np.delete(A, ka, axis=1) @ np.delete(Bm, lb, axis=0), rtol=1e-13, atol=1e-13)
    # keeping k < n - 1: each member keeps its own k largest norms
    A, Bm = g.standard_normal((7, 9)), g.standard_normal((9, 4))
    i1, i2 = O.individual_keep(A.T, Bm.T, 9, 4)
    assert set(i1[0].tolist()) == set(np.argsort(-np.linalg.norm(A, axis=0), kind="stable")[:4].tolist())
    assert set(i2[0].tolist()) == set(np.argsort(-np.linalg.norm(Bm, axis=1), kind="stable")[:4].tolist())
