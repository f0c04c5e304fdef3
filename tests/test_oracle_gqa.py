"""Pins for the oracle's grouped-query coupling (Eq. 5): the group-joint score against explicit removal errors
of the stacked coupled matrices, and the attention with shared key/value heads against torch autograd with
repeated heads (a library routine) and against the multi-head oracle on replicated heads."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import synth


def _gqa_weights(seed, d, h, hkv, dh, scale=1.0):
    wq = synth.normal(seed, 1, (h * dh, d)).astype(np.float64) * scale
    wk = synth.normal(seed, 2, (hkv * dh, d)).astype(np.float64) * scale
    wv = synth.normal(seed, 3, (hkv * dh, d)).astype(np.float64) * scale
    wo = synth.normal(seed, 4, (d, h * dh)).astype(np.float64) * scale
    return wq, wk, wv, wo


@pytest.mark.parametrize("h,hkv", [(4, 2), (6, 2), (3, 1)])
def test_group_joint_score_is_the_removal_error_of_the_groups_pairs(h, hkv):
    """Removing inner dimension j of a group takes the term q_ij k_gj^T out of every pair W_i^Q W_g^K^T of the
    group (Eq. 5); the root of the summed squared Frobenius errors, formed from explicit products, is the
    unnormalised score - for QK and, with the roles of the members exchanged, for VO."""
    d, dh = 9, 5
    m = h // hkv
    wq, wk, wv, wo = _gqa_weights(30 + h, d, h, hkv, dh)
    s_qk = O.coupled_score(O.PAIR_QK, wq, wk, hkv, dh, rep1=m)
    s_vo = O.coupled_score(O.PAIR_VO, wv, wo, hkv, dh, rep2=m)
    for g in range(hkv):
        err_qk, err_vo = np.zeros(dh), np.zeros(dh)
        for j in range(dh):
            keep = [c for c in range(dh) if c != j]
            for i in range(g * m, (g + 1) * m):
                Q, K = wq[i * dh:(i + 1) * dh].T, wk[g * dh:(g + 1) * dh].T          # [d, dh]: columns are q_ij, k_gj
                err_qk[j] += np.linalg.norm(Q @ K.T - Q[:, keep] @ K[:, keep].T) ** 2
                V, Oi = wv[g * dh:(g + 1) * dh].T, wo[:, i * dh:(i + 1) * dh].T     # V: [d, dh], O_i: [dh, d] rows o_ij
                err_vo[j] += np.linalg.norm(V @ Oi - V[:, keep] @ Oi[keep]) ** 2
        for got, err in ((s_qk[g], err_qk), (s_vo[g], err_vo)):
            r = np.sqrt(err)
            np.testing.assert_allclose(got, r / np.linalg.norm(r), rtol=1e-12)
            assert int(np.argmin(got)) == int(np.argmin(err))        # the unit that goes first costs the least


def test_group_joint_score_with_one_head_per_group_is_the_multi_head_score():
    d, h, dh = 8, 3, 6
    wq, wk, wv, wo = _gqa_weights(40, d, h, h, dh)
    np.testing.assert_array_equal(O.coupled_score(O.PAIR_QK, wq, wk, h, dh, rep1=1), O.coupled_score(O.PAIR_QK, wq, wk, h, dh))
    # replicated key heads: the joint score of a group of identical query heads is the single head's
    wq2 = np.concatenate([wq[:dh], wq[:dh], wq[dh:2 * dh], wq[dh:2 * dh]])
    np.testing.assert_allclose(O.coupled_score(O.PAIR_QK, wq2, wk[:2 * dh], 2, dh, rep1=2),
                               O.coupled_score(O.PAIR_QK, wq[:2 * dh], wk[:2 * dh], 2, dh), rtol=1e-13)
    # rotary units: Frobenius norms over the unit's rows of all heads of the group
    s = O.coupled_score(O.PAIR_QK, wq, wk[:dh], 1, dh, unit=2, rep1=3)
    a = sum((wq[i * dh:(i + 1) * dh] ** 2).sum(axis=1).reshape(dh // 2, 2).sum(axis=1) for i in range(3))
    b = (wk[:dh] ** 2).sum(axis=1).reshape(dh // 2, 2).sum(axis=1)
    r = np.sqrt(a * b)
    np.testing.assert_allclose(s[0], r / np.linalg.norm(r), rtol=1e-13)


def _torch_gqa(x, dy, wq, wk, wv, wo, B, L, h, hkv, dh, causal, scale):
    tx, tq, tk, tv, to = (torch.from_numpy(a.copy()).requires_grad_(True) for a in (x, wq, wk, wv, wo))
    d = x.shape[1]
    xb = tx.reshape(B, L, d)
    q = F.linear(xb, tq).reshape(B, L, h, dh).transpose(1, 2)
    k = F.linear(xb, tk).reshape(B, L, hkv, dh).transpose(1, 2).repeat_interleave(h // hkv, dim=1)
    v = F.linear(xb, tv).reshape(B, L, hkv, dh).transpose(1, 2).repeat_interleave(h // hkv, dim=1)
    s = q @ k.transpose(-1, -2) * scale
    if causal:
        s = s.masked_fill(torch.ones(L, L, dtype=torch.bool).triu(1), float("-inf"))
    y = F.linear((torch.softmax(s, dim=-1) @ v).transpose(1, 2).reshape(B * L, h * dh), to)
    (y * torch.from_numpy(dy)).sum().backward()
    return y.detach().numpy(), [t.grad.numpy() for t in (tx, tq, tk, tv, to)]


@pytest.mark.parametrize("h,hkv,causal", [(4, 2, True), (6, 2, False), (4, 1, True)])
def test_gqa_attention_matches_torch_autograd(h, hkv, causal):
    B, L, d, dh = 2, 7, 10, 4
    wq, wk, wv, wo = _gqa_weights(50 + h, d, h, hkv, dh, 0.5)
    x = synth.normal(51, 0, (B * L, d)).astype(np.float64)
    dy = synth.normal(51, 9, (B * L, d)).astype(np.float64)
    scale = dh ** -0.5
    args = (O.heads_rows(wq, h), O.heads_rows(wk, hkv), O.heads_rows(wv, hkv), O.heads_cols(wo, h))
    y, sv = O.attn_fwd(x, *args, B, L, scale, causal)
    g = O.attn_bwd(x, dy, *args, B, L, scale, sv)
    yt, (dx, dq, dk, dv, do) = _torch_gqa(x, dy, wq, wk, wv, wo, B, L, h, hkv, dh, causal, scale)
    np.testing.assert_allclose(y, yt, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dx"], dx, rtol=1e-8, atol=1e-11)
    np.testing.assert_allclose(g["dwq"].reshape(h * dh, d), dq, rtol=1e-8, atol=1e-11)
    np.testing.assert_allclose(g["dwk"].reshape(hkv * dh, d), dk, rtol=1e-8, atol=1e-11)
    np.testing.assert_allclose(g["dwv"].reshape(hkv * dh, d), dv, rtol=1e-8, atol=1e-11)
    np.testing.assert_allclose(g["dwo"].transpose(1, 0, 2).reshape(d, h * dh), do, rtol=1e-8, atol=1e-11)


def test_gqa_equals_multi_head_attention_on_replicated_heads():
    B, L, d, h, hkv, dh = 2, 6, 8, 4, 2, 4
    m = h // hkv
    wq, wk, wv, wo = _gqa_weights(60, d, h, hkv, dh, 0.5)
    x = synth.normal(61, 0, (B * L, d)).astype(np.float64)
    dy = synth.normal(61, 9, (B * L, d)).astype(np.float64)
    ang = O.rope_angles(np.tile(np.arange(dh // 2), (h, 1)), L, dh)
    hq, hk, hv, ho = O.heads_rows(wq, h), O.heads_rows(wk, hkv), O.heads_rows(wv, hkv), O.heads_cols(wo, h)
    y, sv = O.attn_fwd(x, hq, hk, hv, ho, B, L, 0.5, True, angles=ang)
    g = O.attn_bwd(x, dy, hq, hk, hv, ho, B, L, 0.5, sv, angles=ang)
    rk, rv = np.repeat(hk, m, axis=0), np.repeat(hv, m, axis=0)
    y2, sv2 = O.attn_fwd(x, hq, rk, rv, ho, B, L, 0.5, True, angles=ang)
    g2 = O.attn_bwd(x, dy, hq, rk, rv, ho, B, L, 0.5, sv2, angles=ang)
    np.testing.assert_allclose(y, y2, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(g["dx"], g2["dx"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dwk"], g2["dwk"].reshape(hkv, m, dh, d).sum(axis=1), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dwv"], g2["dwv"].reshape(hkv, m, dh, d).sum(axis=1), rtol=1e-12, atol=1e-14)


def test_pair_importance_of_a_group_is_the_mean_over_all_its_heads():
    """Eq. 8 with shared heads: each member's mean squared gradient runs over every head of the group - element
    loops, and the constant-gradient closed form c^2 / |D|."""
    hkv, m, dh, d, D = 2, 3, 4, 5, 7.0
    gq = synth.normal(70, 1, (hkv * m * dh, d)).astype(np.float64)
    gk = synth.normal(70, 2, (hkv * dh, d)).astype(np.float64)
    go = synth.normal(70, 3, (d, hkv * m * dh)).astype(np.float64)
    got_qk = O.pair_fisher(O.PAIR_QK, gq, gk, hkv, dh, D, rep1=m)
    got_vo = O.pair_fisher(O.PAIR_VO, gk, go, hkv, dh, D, rep2=m)
    for g in range(hkv):
        s1 = sum(gq[r, c] ** 2 for r in range(g * m * dh, (g + 1) * m * dh) for c in range(d)) / (m * dh * d)
        s2 = sum(gk[r, c] ** 2 for r in range(g * dh, (g + 1) * dh) for c in range(d)) / (dh * d)
        s3 = sum(go[r, c] ** 2 for r in range(d) for c in range(g * m * dh, (g + 1) * m * dh)) / (m * dh * d)
        np.testing.assert_allclose(got_qk[g], 0.5 * (s1 + s2) / D, rtol=1e-13)
        np.testing.assert_allclose(got_vo[g], 0.5 * (s2 + s3) / D, rtol=1e-13)
    c = O.pair_fisher(O.PAIR_QK, np.full_like(gq, 0.5), np.full_like(gk, 0.5), hkv, dh, D, rep1=m)
    np.testing.assert_allclose(c, np.full(hkv, 0.25 / D), rtol=1e-14)
