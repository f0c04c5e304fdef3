"""Pins of the glue oracle (CPU only): central differences, closed forms, brute force and adjointness."""
import numpy as np

from oracle.glue_oracle import embed_bwd, embed_fwd, ln_bwd, ln_fwd, rms_bwd, rms_fwd, xent


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


def test_cross_entropy_closed_forms_and_derivative():
    rng = np.random.default_rng(2)
    T, V = 6, 9
    tgt = rng.integers(0, V, T)
    # equal logits: every class has probability 1/V
    loss, rows, dl = xent(np.full((T, V), 3.25), tgt)
    assert abs(loss - np.log(V)) < 1e-12 and np.allclose(rows, np.log(V))
    want = np.full((T, V), 1.0 / V)
    want[np.arange(T), tgt] -= 1.0
    np.testing.assert_allclose(dl, want / T, atol=1e-15)
    # one overwhelming logit on the target: loss -> 0; on another class: loss -> the gap
    lg = np.zeros((T, V))
    lg[np.arange(T), tgt] = 60.0
    assert xent(lg, tgt)[0] < 1e-20
    lg2 = np.zeros((T, V))
    lg2[np.arange(T), (tgt + 1) % V] = 60.0
    assert abs(xent(lg2, tgt)[0] - 60.0) < 1e-9
    # general case: the row losses by the definition with plain sums, the gradient by central differences, rows sum to 0
    lg = rng.standard_normal((T, V)) * 3
    loss, rows, dl = xent(lg, tgt)
    p = np.exp(lg) / np.exp(lg).sum(1, keepdims=True)
    np.testing.assert_allclose(rows, -np.log(p[np.arange(T), tgt]), rtol=1e-12)
    np.testing.assert_allclose(dl, _fd(lambda v: np.array(xent(v, tgt)[0]), lg, np.array(1.0)), rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(dl.sum(1), 0, atol=1e-15)
    # shifting a row by a constant changes nothing
    np.testing.assert_allclose(xent(lg + rng.standard_normal((T, 1)) * 50, tgt)[0], loss, rtol=1e-12)


def test_embedding_lookup_and_its_adjoint():
    rng = np.random.default_rng(3)
    V, d, L, Bsz = 7, 5, 4, 3
    ids = np.array([2, 2, 6, 0, 2, 5, 5, 0, 1, 2, 6, 6])
    table, pos = rng.standard_normal((V, d)), rng.standard_normal((L, d))
    x = embed_fwd(ids, table, pos, L)
    assert np.array_equal(x[5], table[5] + pos[1]) and np.array_equal(x[11], table[6] + pos[3])
    assert np.array_equal(embed_fwd(ids, table)[4], table[2])
    dx = rng.standard_normal((Bsz * L, d))
    dt, dp = embed_bwd(ids, dx, V, L)
    # by hand: token 2 appears at 0, 1, 4, 9; token 3 and 4 never
    np.testing.assert_allclose(dt[2], dx[0] + dx[1] + dx[4] + dx[9])
    assert not dt[3].any() and not dt[4].any()
    np.testing.assert_allclose(dp[1], dx[1] + dx[5] + dx[9])
    # a library routine for the same sum, and the adjoint identity <lookup(table, pos), dx> = <table, dtable> + <pos, dpos>
    ref = np.zeros((V, d))
    np.add.at(ref, ids, dx)
    np.testing.assert_allclose(dt, ref)
    np.testing.assert_allclose((x * dx).sum(), (table * dt).sum() + (pos * dp).sum(), rtol=1e-12)
    assert embed_bwd(ids, dx, V)[1] is None
