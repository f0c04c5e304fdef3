"""Pins for the oracle's AdamW update: a library optimizer run in fp64, the closed form of the first step,
and the alignment property Alg. 1 relies on (updating gathered tensors = gathering updated tensors)."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import synth


@pytest.mark.parametrize("wd,eps", [(0.0, 1e-8), (0.01, 1e-8), (0.1, 1e-3)])
def test_adamw_matches_library_optimizer(wd, eps):
    w0 = synth.normal(60, 0, (7, 5)).astype(np.float64)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.8, 0.95), eps=eps, weight_decay=wd)
    w, m, v = w0, np.zeros_like(w0), np.zeros_like(w0)
    for t in range(1, 8):
        g = synth.normal(60, t, (7, 5)).astype(np.float64) * (10.0 ** (t % 3 - 1))
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        w, m, v = O.adamw_step(w, g, m, v, t, 3e-3, 0.8, 0.95, eps, wd)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-15)
    st = opt.state[p]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12)


def test_adamw_first_step_closed_form():
    """From zero moments the bias-corrected moments of step 1 are g and g^2: the step is
    lr * (g / (|g| + eps) + wd * w) whatever the betas."""
    w = np.array([1.0, -2.0, 0.5, 0.0])
    g = np.array([0.3, -4.0, 0.0, 1e-9])
    for b1, b2 in ((0.9, 0.999), (0.5, 0.7)):
        w1, m1, v1 = O.adamw_step(w, g, np.zeros(4), np.zeros(4), 1, 0.1, b1, b2, 1e-8, 0.2)
        np.testing.assert_allclose(w1, w - 0.1 * (g / (np.abs(g) + 1e-8) + 0.2 * w), rtol=1e-12)
        np.testing.assert_allclose(m1, (1 - b1) * g, rtol=1e-15)
        np.testing.assert_allclose(v1, (1 - b2) * g * g, rtol=1e-15)
    # zero gradient and zero moments: only the decay acts; an all-zero (padding) entry stays zero
    w1, m1, v1 = O.adamw_step(w, np.zeros(4), np.zeros(4), np.zeros(4), 5, 0.1, 0.9, 0.999, 1e-8, 0.2)
    np.testing.assert_allclose(w1, w * (1 - 0.1 * 0.2), rtol=1e-15)
    assert w1[3] == 0 and not m1.any() and not v1.any()


def test_adamw_commutes_with_the_aligned_gather():
    """Removing the moments of removed rows with the rows themselves (Alg. 1) loses nothing: steps on the
    gathered (w, m, v) equal the gathered result of steps on the full tensors."""
    n, d, k = 12, 4, 5
    idx = np.sort(np.random.default_rng(3).choice(n, k, replace=False))[None, :].astype(np.int32)
    w, m, v = (synth.normal(61, i, (n, d)).astype(np.float64) for i in range(3))
    v = v * v
    wc, mc, vc = (O.compact(a, idx, 0, n) for a in (w, m, v))
    for t in (3, 4):
        g = synth.normal(61, 10 + t, (n, d)).astype(np.float64)
        w, m, v = O.adamw_step(w, g, m, v, t, 1e-2)
        wc, mc, vc = O.adamw_step(wc, O.compact(g, idx, 0, n), mc, vc, t, 1e-2)
    for full, cmp in ((w, wc), (m, mc), (v, vc)):
        np.testing.assert_array_equal(O.compact(full, idx, 0, n), cmp)
