"""One forward+backward of a small two-layer stack through the harness (`stack.py`: the library's blocks, the
output projection and the glue around them) against the fp64 oracle: the oracle's attention and FFN functions
chained with the embedding, pre-norms (RMSNorm / LayerNorm), residual additions, output projection and mean
cross-entropy written out here in numpy.  What is compared: logits, loss, and every gradient the step produces."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd.stack import DecoderStack
from oracle.glue_oracle import ln_bwd, ln_fwd, rms_bwd, rms_fwd
from util import assert_close, host

pytestmark = pytest.mark.gpu

GPT = dict(B=2, L=72, d=128, h=2, d_h=64, d_ff=256, gated=False, rope=False, bias=True)
LLAMA = dict(B=2, L=72, d=128, h=2, d_h=64, d_ff=264, gated=True, rope=True, bias=False)
VOCAB = 320


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def _oracle_step(st, ids, tgt):
    """fp64 forward and backward of the stack `st` on its own (bf16-rounded) parameters and kept indices."""
    cfg, Bsz, L, d, h, dh, T = st.cfg, st.Bsz, st.L, st.d, st.h, st.d_h, st.T
    unit = 2 if cfg["rope"] else 1
    oact = O.ACT_SWIGLU if cfg["gated"] else O.ACT_GELU_ERF
    scale = dh ** -0.5
    emb, lm = host(st.emb.w), host(st.lm.w)

    def norm_fwd(x, ps):
        if st.rms:
            y, r = rms_fwd(x, host(ps[0].w), st.eps)
            return y, (x, r)
        return ln_fwd(x, host(ps[0].w), host(ps[1].w), st.eps)

    def norm_bwd(ps, saved, dy):
        if st.rms:
            return rms_bwd(saved[0], host(ps[0].w), saved[1], dy)
        return ln_bwd(host(ps[0].w), saved, dy)

    x = emb[ids]
    if st.pos is not None:
        x = (x.reshape(Bsz, L, d) + host(st.pos.w)).reshape(T, d)
    tape = []
    for ly in st.layers:
        iq, iv, iff = (i.cpu().numpy() for i in ly.idx)
        f = {n: host(t) for n, t in ly.full["w"].items()}
        w = dict(wq=O.heads_rows(O.compact(f["wq"], iq, 0, dh, unit), h), wk=O.heads_rows(O.compact(f["wk"], iq, 0, dh, unit), h),
                 wv=O.heads_rows(O.compact(f["wv"], iv, 0, dh), h), wo=O.heads_cols(O.compact(f["wo"], iv, 1, dh), h),
                 w1=O.compact(f["w1"], iff, 0, st.d_ff), w2=O.compact(f["w2"], iff, 1, st.d_ff),
                 w1b=O.compact(f["w1b"], iff, 0, st.d_ff) if cfg["gated"] else None)
        kw, b1, b2 = {}, None, None
        if cfg["bias"]:
            kw = dict(bq=O.compact(f["bq"], iq, 0, dh, unit).reshape(h, -1), bk=O.compact(f["bk"], iq, 0, dh, unit).reshape(h, -1),
                      bv=O.compact(f["bv"], iv, 0, dh).reshape(h, -1), bo=f["bo"])
            b1, b2 = O.compact(f["b1"], iff, 0, st.d_ff), f["b2"]
        ang = O.rope_angles(iq, L, dh) if cfg["rope"] else None
        h1, n1 = norm_fwd(x, ly.norm[0])
        a, sva = O.attn_fwd(h1, w["wq"], w["wk"], w["wv"], w["wo"], Bsz, L, scale, True, angles=ang, **kw)
        x = x + a
        h2, n2 = norm_fwd(x, ly.norm[1])
        y, svf = O.ffn_fwd(h2, w["w1"], b1, w["w2"], b2, oact, w1b=w["w1b"])
        x = x + y
        tape.append((w, ang, h1, n1, sva, h2, n2, svf))
    hf, nf = norm_fwd(x, st.norm_f)
    logits = hf @ lm.T
    z = logits - logits.max(axis=1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
    loss = -logp[np.arange(T), tgt].mean()
    dl = np.exp(logp)
    dl[np.arange(T), tgt] -= 1.0
    dl /= T
    out = {"logits": logits, "loss": loss, "lm": dl.T @ hf, "layers": []}
    dx, out["nf_g"], _ = norm_bwd(st.norm_f, nf, dl @ lm)
    for ly, (w, ang, h1, n1, sva, h2, n2, svf) in zip(reversed(st.layers), reversed(tape)):
        gf = O.ffn_bwd(h2, dx, w["w1"], w["w2"], oact, svf, w1b=w["w1b"])
        d2, g2, _ = norm_bwd(ly.norm[1], n2, gf["dx"])
        dx = dx + d2
        ga = O.attn_bwd(h1, dx, w["wq"], w["wk"], w["wv"], w["wo"], Bsz, L, scale, sva, angles=ang)
        d1, g1, _ = norm_bwd(ly.norm[0], n1, ga["dx"])
        dx = dx + d1
        out["layers"].insert(0, {"ffn": gf, "attn": ga, "n1_g": g1, "n2_g": g2})
    demb = np.zeros_like(emb)
    np.add.at(demb, ids, dx)
    out["emb"] = demb
    out["pos"] = dx.reshape(Bsz, L, d).sum(axis=0)
    return out


@pytest.mark.parametrize("cfg", [GPT, LLAMA], ids=["gpt2_like", "llama_like"])
def test_two_layer_step_against_the_oracle(ctx, cfg):
    st = DecoderStack(ctx, cfg, n_layers=2, vocab=VOCAB, keep=(1, 2), seed=9)
    gen = torch.Generator(device="cuda").manual_seed(4)
    ids = torch.randint(0, VOCAB, (st.T,), device="cuda", generator=gen)
    tgt = torch.randint(0, VOCAB, (st.T,), device="cuda", generator=gen)
    # steps 1-3 of the harness against the oracle: scores of the fp32 master weights, then the choice on those scores
    for li, ly in enumerate(st.layers):
        m = {n: host(t) for n, t in ly.full["mst"].items()}
        unit = 2 if cfg["rope"] else 1
        want = [O.coupled_score(O.PAIR_QK, m["wq"], m["wk"], st.h, st.d_h, unit), O.coupled_score(O.PAIR_VO, m["wv"], m["wo"], st.h, st.d_h),
                O.coupled_score(O.PAIR_FFN_GATED if cfg["gated"] else O.PAIR_FFN, m["w1"], m["w2"], 1, st.d_ff, w1b=m.get("w1b"))]
        for j in range(3):
            s = st.scores[3 * li + j]
            assert_close(s, want[j], "f32", f"layer {li} score {j}")
            assert np.array_equal(ly.idx[j].cpu().numpy(), O.select_topk(s.cpu().numpy(), st.k[j]))
    logits = st.forward(ids).clone()      # backward turns the buffer into the gradient of the logits
    loss = st.backward(ids, tgt)
    torch.cuda.synchronize()
    o = _oracle_step(st, ids.cpu().numpy(), tgt.cpu().numpy())
    # bf16 activations, residual stream and gradients through two layers against fp64: the bf16 bound for what a
    # single block produces, half as much again for gradients that have crossed the whole stack
    assert_close(logits, o["logits"], "bf16", "logits")
    assert abs(float(loss) - o["loss"]) <= 2e-3 * abs(o["loss"])
    deep = 3e-2

    def rel(got, want, what):
        e = O.rel_fro(host(got) if isinstance(got, torch.Tensor) else got, want)
        assert e <= deep, f"{what}: {e:.3e}"

    rel(st.lm.g, o["lm"], "dW of the output projection")
    rel(st.emb.g, o["emb"], "embedding gradient")
    rel(st.norm_f[0].g, o["nf_g"], "final norm gain")
    if st.pos is not None:
        rel(st.pos.g, o["pos"], "position table gradient")
    unit = 2 if cfg["rope"] else 1
    for li, (ly, g) in enumerate(zip(st.layers, o["layers"])):
        a, f = ly.attn["w"], ly.ffn["w"]
        kq, kv, kf = a.k_qk_units * unit, a.k_vo, f.k
        got = host(a.dwqkv_c)
        rel(got[:a.nq].reshape(st.h, a.kp_qk, st.d)[:, :kq], g["attn"]["dwq"], f"layer {li} dW_q")
        rel(got[a.nq:a.nq + a.nk].reshape(st.h, a.kp_qk, st.d)[:, :kq], g["attn"]["dwk"], f"layer {li} dW_k")
        rel(got[a.nq + a.nk:].reshape(st.h, a.kp_vo, st.d)[:, :kv], g["attn"]["dwv"], f"layer {li} dW_v")
        rel(host(a.dwo_c).reshape(st.d, st.h, a.kp_vo)[:, :, :kv].transpose(1, 0, 2), g["attn"]["dwo"], f"layer {li} dW_o")
        rel(f.dw2_c[:, :kf], g["ffn"]["dw2"], f"layer {li} dW_2")
        if cfg["gated"]:
            rel(f.gate_rows(f.dw1_c)[:kf], g["ffn"]["dw1"], f"layer {li} dW_gate")
            rel(f.up_rows(f.dw1_c)[:kf], g["ffn"]["dw1b"], f"layer {li} dW_up")
        else:
            rel(f.dw1_c[:kf], g["ffn"]["dw1"], f"layer {li} dW_1")
            rel(f.db1_c[:kf], g["ffn"]["db1"], f"layer {li} db_1")
            rel(f.db2, g["ffn"]["db2"], f"layer {li} db_2")
            rel(a.dbo, g["attn"]["dbo"], f"layer {li} db_o")
        rel(ly.norm[0][0].g, g["n1_g"], f"layer {li} first norm gain")
        rel(ly.norm[1][0].g, g["n2_g"], f"layer {li} second norm gain")
