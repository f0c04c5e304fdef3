"""GPU tests of the multi-layer harness (pre-norm decoder stack around the library's blocks): a small stack
against the same model written with torch's fp32 operators and autograd - dense through the library (all units
kept) and sparse (= the dense model with the pruned rows and columns zeroed, Def. 1) - and the bookkeeping of
the training state: compact master weights and moments, their write-back and the next estimate."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd.stack import DecoderStack
from util import host

pytestmark = pytest.mark.gpu

GPT = dict(B=2, L=64, d=128, h=2, d_h=64, d_ff=256, gated=False, rope=False, bias=True)
LLAMA = dict(B=2, L=64, d=128, h=2, d_h=64, d_ff=264, gated=True, rope=True, bias=False)
LLAMA_GQA = dict(LLAMA, h=4, h_kv=2, d=256)      # two query heads per key/value head
VOCAB = 512


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def _kept_mask(idx, groups, n, unit):
    """bool[groups * n]: inner dimensions the index lists keep."""
    m = torch.zeros(groups * n, dtype=torch.bool, device="cuda")
    pos = (torch.arange(groups, device="cuda")[:, None] * n + idx.long() * unit).reshape(-1)
    for u in range(unit):
        m[pos + u] = True
    return m


def _rope(x, L, d_h):
    """Interleaved pairs (2p, 2p+1) rotated by t * 10000^(-2p/d_h) (Eq. 6); x: [B, L, h, d_h]."""
    p = torch.arange(d_h // 2, device=x.device, dtype=torch.float64)
    ang = torch.arange(L, device=x.device, dtype=torch.float64)[:, None] * (10000.0 ** (-2.0 * p / d_h))[None, :]
    c, s = ang.cos().float()[None, :, None, :], ang.sin().float()[None, :, None, :]
    a, b = x[..., 0::2], x[..., 1::2]
    return torch.stack([a * c - b * s, a * s + b * c], dim=-1).flatten(-2)


def _reference(st: DecoderStack, ids, targets):
    """The masked dense model in fp32 torch operators; returns logits, loss and the leaves with gradients."""
    cfg, Bsz, L, d, h, dh = st.cfg, st.Bsz, st.L, st.d, st.h, st.d_h
    leaves = {}

    def leaf(name, t):
        leaves[name] = t.detach().float().clone().requires_grad_(True)
        return leaves[name]

    def norm(x, ps, name):
        g = leaf(name + ".g", ps[0].w)
        if st.rms:
            return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + st.eps) * g
        return F.layer_norm(x, (d,), g, leaf(name + ".b", ps[1].w), st.eps)

    x = leaf("emb", st.emb.w)[ids]
    if st.pos is not None:
        x = (x.view(Bsz, L, d) + leaf("pos", st.pos.w)).view(Bsz * L, d)
    causal = torch.ones(L, L, dtype=torch.bool, device="cuda").tril()
    for li, ly in enumerate(st.layers):
        unit = 2 if cfg["rope"] else 1
        hkv = st.h_kv
        rep = h // hkv          # a group's query heads (and heads of W_o) keep the dimensions of their key/value head
        mk_, mv_ = _kept_mask(ly.idx[0], hkv, dh, unit).float(), _kept_mask(ly.idx[1], hkv, dh, 1).float()
        mqk = mk_.view(hkv, 1, dh).expand(hkv, rep, dh).reshape(-1)
        mvo = mv_.view(hkv, 1, dh).expand(hkv, rep, dh).reshape(-1)
        mff = _kept_mask(ly.idx[2], 1, st.d_ff, 1).float()
        f = ly.full["w"]
        wq, wk = leaf(f"{li}.wq", f["wq"]) * mqk[:, None], leaf(f"{li}.wk", f["wk"]) * mk_[:, None]
        wv, wo = leaf(f"{li}.wv", f["wv"]) * mv_[:, None], leaf(f"{li}.wo", f["wo"]) * mvo[None, :]
        h1 = norm(x, ly.norm[0], f"{li}.n1")
        q, k, v = h1 @ wq.T, h1 @ wk.T, h1 @ wv.T
        if cfg["bias"]:
            q, k, v = q + leaf(f"{li}.bq", f["bq"]) * mqk, k + leaf(f"{li}.bk", f["bk"]) * mk_, v + leaf(f"{li}.bv", f["bv"]) * mv_
        q = q.view(Bsz, L, h, dh)
        k, v = (t.view(Bsz, L, hkv, dh).repeat_interleave(rep, dim=2) for t in (k, v))
        if cfg["rope"]:
            q, k = _rope(q, L, dh), _rope(k, L, dh)
        s = torch.einsum("blhd,bmhd->bhlm", q, k) * dh ** -0.5
        p = s.masked_fill(~causal, float("-inf")).softmax(-1)
        o = torch.einsum("bhlm,bmhd->blhd", p, v).reshape(Bsz * L, h * dh)
        a = o @ wo.T
        if cfg["bias"]:
            a = a + leaf(f"{li}.bo", f["bo"])
        x = x + a
        h2 = norm(x, ly.norm[1], f"{li}.n2")
        w1, w2 = leaf(f"{li}.w1", f["w1"]) * mff[:, None], leaf(f"{li}.w2", f["w2"]) * mff[None, :]
        if cfg["gated"]:
            w1b = leaf(f"{li}.w1b", f["w1b"]) * mff[:, None]
            act = F.silu(h2 @ w1.T) * (h2 @ w1b.T)
        else:
            act = F.gelu(h2 @ w1.T + leaf(f"{li}.b1", f["b1"]) * mff)
        y = act @ w2.T
        if cfg["bias"]:
            y = y + leaf(f"{li}.b2", f["b2"])
        x = x + y
    logits = norm(x, st.norm_f, "nf") @ leaf("lm", st.lm.w).T
    loss = F.cross_entropy(logits, targets)
    loss.backward()
    return logits.detach(), loss.detach(), leaves


def _rel(got, want):
    return O.rel_fro(host(got), host(want))


@pytest.mark.parametrize("cfg", [GPT, LLAMA, LLAMA_GQA], ids=["gpt2_like", "llama_like", "llama_gqa"])
@pytest.mark.parametrize("keep", [(1, 1), (1, 2)], ids=["dense", "half"])
def test_stack_matches_masked_dense_torch_model(ctx, cfg, keep):
    st = DecoderStack(ctx, cfg, n_layers=2, vocab=VOCAB, keep=keep, seed=3)
    gen = torch.Generator(device="cuda").manual_seed(11)
    ids = torch.randint(0, VOCAB, (st.T,), device="cuda", generator=gen)
    tgt = torch.randint(0, VOCAB, (st.T,), device="cuda", generator=gen)
    logits = st.forward(ids).clone()      # backward turns the buffer into the gradient of the logits
    loss = st.backward(ids, tgt)
    ref_logits, ref_loss, leaves = _reference(st, ids, tgt)
    assert _rel(logits, ref_logits) <= 2e-2
    assert abs(float(loss) - float(ref_loss)) <= 2e-3 * abs(float(ref_loss))
    tol = 3e-2          # bf16 activations and gradients through two layers, against fp32
    assert _rel(st.lm.g, leaves["lm"].grad) <= tol
    assert _rel(st.emb.g, leaves["emb"].grad) <= tol
    if st.pos is not None:
        assert _rel(st.pos.g, leaves["pos"].grad) <= tol
    assert _rel(st.norm_f[0].g, leaves["nf.g"].grad) <= tol
    for li, ly in enumerate(st.layers):
        a, f = ly.attn["w"], ly.ffn["w"]
        unit = 2 if cfg["rope"] else 1
        kq, kv, kf = a.k_qk_units * unit, a.k_vo, f.k
        # compact gradients against the reference's gradients gathered with the same indices; pruned entries of the
        # reference carry no gradient (their partner row/column is zero)
        rep = st.h // st.h_kv
        gq = O.compact(host(leaves[f"{li}.wq"].grad), np.repeat(ly.idx[0].cpu().numpy(), rep, axis=0), 0, st.d_h, unit)
        got = host(a.dwqkv_c[:a.nq]).reshape(st.h, a.kp_qk, st.d)[:, :kq].reshape(-1, st.d)
        assert O.rel_fro(got, gq) <= tol, f"layer {li} dW_q"
        go = O.compact(host(leaves[f"{li}.wo"].grad), np.repeat(ly.idx[1].cpu().numpy(), rep, axis=0), 1, st.d_h, 1)
        got = host(a.dwo_c).reshape(st.d, st.h, a.kp_vo)[:, :, :kv].reshape(st.d, -1)
        assert O.rel_fro(got, go) <= tol, f"layer {li} dW_o"
        g1 = O.compact(host(leaves[f"{li}.w1"].grad), ly.idx[2].cpu().numpy(), 0, st.d_ff, 1)
        assert O.rel_fro(host(f.gate_rows(f.dw1_c)[:kf]), g1) <= tol, f"layer {li} dW_1"
        g2 = O.compact(host(leaves[f"{li}.w2"].grad), ly.idx[2].cpu().numpy(), 1, st.d_ff, 1)
        assert O.rel_fro(host(f.dw2_c[:, :kf]), g2) <= tol, f"layer {li} dW_2"
        assert _rel(ly.norm[0][0].g, leaves[f"{li}.n1.g"].grad) <= tol
        if keep == (1, 2):
            pruned = ~_kept_mask(ly.idx[2], 1, st.d_ff, 1)
            assert float(leaves[f"{li}.w1"].grad[pruned].abs().max()) == 0.0


@pytest.mark.parametrize("cfg", [GPT, LLAMA], ids=["gpt2_like", "llama_like"])
def test_training_state_stays_compact_and_is_written_back(ctx, cfg):
    st = DecoderStack(ctx, cfg, n_layers=2, vocab=VOCAB, keep=(1, 2), seed=5, lr=3e-3, weight_decay=0.01)
    gen = torch.Generator(device="cuda").manual_seed(2)
    ids = torch.randint(0, VOCAB, (st.T,), device="cuda", generator=gen)
    tgt = torch.roll(ids, -1)
    init = [{n: t.clone() for n, t in ly.full["mst"].items()} for ly in st.layers]
    idx0 = [[i.clone() for i in ly.idx] for ly in st.layers]
    losses = [float(st.train_step(ids, tgt)) for _ in range(8)]
    assert losses[-1] < losses[0] - 0.1, losses                       # the same batch again and again: the loss falls
    # the working copies are the rounded master weights, and the transposed copies follow them
    for ly in st.layers:
        a, f = ly.attn, ly.ffn
        assert torch.equal(a["w"].wqkv_c, a["mst"].wqkv_c.to(torch.bfloat16))
        assert torch.equal(f["w"].w2_c, f["mst"].w2_c.to(torch.bfloat16))
        assert torch.equal(a["w"].wqkv_t, a["w"].wqkv_c.T) and torch.equal(f["w"].w2_t, f["w"].w2_c.T)
    # until the next estimate the full-size arrays are untouched
    for ly, w0 in zip(st.layers, init):
        for n, t in ly.full["mst"].items():
            if n not in ("bo", "b2"):                    # the output biases belong to no pair: they train in place
                assert torch.equal(t, w0[n]), n
    cm = [{"w1": ly.ffn["mst"].gate_rows(ly.ffn["mst"].w1_c).clone(), "m_w2": ly.ffn["m"].w2_c.clone(), "wq": ly.attn["mst"].wqkv_c.clone()} for ly in st.layers]
    st.prune()
    for li, (ly, w0) in enumerate(zip(st.layers, init)):
        unit = 2 if cfg["rope"] else 1
        kept_ff = _kept_mask(idx0[li][2], 1, st.d_ff, 1)
        kept_qk = _kept_mask(idx0[li][0], st.h, st.d_h, unit)
        full = ly.full["mst"]
        # written back: kept rows hold the trained values, pruned rows what they held before
        kf = st.k[2]
        assert torch.equal(full["w1"][kept_ff], cm[li]["w1"][:kf])
        assert torch.equal(full["w1"][~kept_ff], w0["w1"][~kept_ff])
        assert torch.equal(ly.full["m"]["w2"][:, kept_ff], cm[li]["m_w2"][:, :kf])
        assert float(ly.full["m"]["w2"][:, ~kept_ff].abs().max()) == 0.0
        kq = st.k[0] * unit
        got = full["wq"][kept_qk].reshape(st.h, kq, st.d)
        assert torch.equal(got, cm[li]["wq"][:ly.attn["mst"].nq].reshape(st.h, -1, st.d)[:, :kq])
        assert torch.equal(full["wq"][~kept_qk], w0["wq"][~kept_qk])
        assert torch.equal(ly.full["w"]["w1"][kept_ff], cm[li]["w1"][:kf].to(torch.bfloat16))
        # the new choice is the library's selection on the scores of the written-back master weights, and every family
        # holds the gather of its full-size array by that choice
        s = st.ctx.ecospa_coupled_score([ly.ffn["mst"].pair()])[0]
        assert np.array_equal(ly.idx[2].cpu().numpy(), O.select_topk(s.cpu().numpy(), kf))
        new_ff = ly.idx[2][0].long()
        assert torch.equal(ly.ffn["mst"].gate_rows(ly.ffn["mst"].w1_c)[:kf], full["w1"][new_ff])
        assert torch.equal(ly.ffn["v"].w2_c[:, :kf], ly.full["v"]["w2"][:, new_ff])
        assert torch.equal(ly.ffn["w"].gate_rows(ly.ffn["w"].w1_c)[:kf], ly.full["w"]["w1"][new_ff])
    # and training goes on from the new compact state
    more = [float(st.train_step(ids, tgt)) for _ in range(3)]
    assert all(np.isfinite(more)) and more[-1] < losses[0]


@pytest.mark.parametrize("cfg", [GPT, LLAMA], ids=["gpt2_like", "llama_like"])
def test_inference_stack_forward_only(ctx, cfg):
    st = DecoderStack(ctx, cfg, n_layers=2, vocab=VOCAB, keep=(3, 10), seed=7, train=False)
    ids = torch.randint(0, VOCAB, (st.T,), device="cuda")
    logits = st.forward(ids)
    assert logits.shape == (st.T, VOCAB) and bool(torch.isfinite(logits.float()).all())
    assert "mst" not in st.layers[0].full
    ref_logits, _, _ = _reference(st, ids, torch.zeros_like(ids))
    assert _rel(logits, ref_logits) <= 2e-2
