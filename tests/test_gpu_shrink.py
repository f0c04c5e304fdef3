"""Alg. 1 as printed, on a small stack: rows and columns leave for good.  A stack built with permanent=True releases
its full-size arrays after the first gather and shrinks from its compact state; what it holds after two rounds
(1 -> 3/4 -> 1/2 of every pair) is checked against the oracle applied to the original full-size tensors of a twin
stack with the same seed: scores of the compact master weights, the choice, the composed index lists, every
compact tensor of every family bit for bit, the rotary tables of the original block positions, and one training
step through the shrunk stack against the oracle's forward pass."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd.stack import DecoderStack
from util import assert_close, host

pytestmark = pytest.mark.gpu

GPT = dict(B=2, L=40, d=128, h=2, d_h=64, d_ff=256, gated=False, rope=False, bias=True)
LLAMA = dict(B=2, L=40, d=128, h=4, d_h=32, d_ff=264, gated=True, rope=True, bias=False, h_kv=2)
VOCAB = 96


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def _compose(prev, idx):
    """positions in the previous compact layout -> original positions"""
    return np.take_along_axis(prev, idx.astype(np.int64), axis=1)


@pytest.mark.parametrize("cfg", [GPT, LLAMA], ids=["gpt2_like", "llama_gqa_like"])
def test_two_rounds_of_removal_for_good(ctx, cfg):
    twin = DecoderStack(ctx, cfg, n_layers=2, vocab=VOCAB, keep=(1, 1), seed=5)            # keeps its full-size arrays
    st = DecoderStack(ctx, cfg, n_layers=2, vocab=VOCAB, keep=(1, 1), seed=5, permanent=True)
    assert all(ly.full is None for ly in st.layers)
    h, hk, dh, dff = st.h, st.h_kv, st.d_h, st.d_ff
    unit = 2 if cfg["rope"] else 1
    mem = [torch.cuda.memory_allocated()]
    orig = [[np.tile(np.arange(dh // unit), (hk, 1)), np.tile(np.arange(dh), (hk, 1)), np.arange(dff)[None, :]] for _ in st.layers]
    gen = torch.Generator(device="cuda").manual_seed(2)
    ids = torch.randint(0, VOCAB, (st.T,), device="cuda", generator=gen)
    tgt = torch.randint(0, VOCAB, (st.T,), device="cuda", generator=gen)
    for keep in ((3, 4), (1, 2)):
        # what the round must score: the compact master weights as they stand (gathered from the originals so far)
        want_scores = []
        for li, ly in enumerate(st.layers):
            f = {n: host(t) for n, t in twin.layers[li].full["mst"].items()}
            oq, ov, of = orig[li]
            wq = O.compact(f["wq"], np.repeat(oq, h // hk, axis=0), 0, dh, unit)
            wk, wv = O.compact(f["wk"], oq, 0, dh, unit), O.compact(f["wv"], ov, 0, dh)
            wo = O.compact(f["wo"], np.repeat(ov, h // hk, axis=0), 1, dh)
            kq, kv = oq.shape[1] * unit, ov.shape[1]
            want_scores += [O.coupled_score(O.PAIR_QK, wq, wk, hk, kq, unit, rep1=h // hk),
                            O.coupled_score(O.PAIR_VO, wv, wo, hk, kv, rep2=h // hk),
                            O.coupled_score(O.PAIR_FFN_GATED if cfg["gated"] else O.PAIR_FFN, O.compact(f["w1"], of, 0, dff),
                                            O.compact(f["w2"], of, 1, dff), 1, of.shape[1],
                                            w1b=O.compact(f["w1b"], of, 0, dff) if cfg["gated"] else None)]
        st.shrink(keep)
        torch.cuda.synchronize()
        mem.append(torch.cuda.memory_allocated())
        for li, ly in enumerate(st.layers):
            for j in range(3):
                s = host(st.scores[3 * li + j])
                k_old = orig[li][j].shape[1]
                assert_close(s[:, :k_old], want_scores[3 * li + j], "f32", f"round {keep} layer {li} score {j}")
                assert not s[:, k_old:].any()                   # padding units of the compact layout: zero weights, zero score
                idx = ly.idx[j].cpu().numpy()
                assert np.array_equal(idx, O.select_topk(st.scores[3 * li + j].cpu().numpy(), st.k[j]))
                assert idx.max() < k_old
                orig[li][j] = _compose(orig[li][j], idx)
    assert mem[2] < mem[1] < mem[0]
    # every family's compact tensors: the originals gathered at the composed positions, bit for bit
    for li, ly in enumerate(st.layers):
        oq, ov, of = orig[li]
        a, f = ly.attn["w"], ly.ffn["w"]
        assert (a.k_qk_units, a.k_vo, f.k) == (oq.shape[1], ov.shape[1], of.shape[1])
        for fam in ("w", "mst"):
            full = {n: host(t) for n, t in twin.layers[li].full[fam].items()}
            A, F = ly.attn[fam], ly.ffn[fam]
            got = host(A.wqkv_c)
            rq = np.repeat(oq, h // hk, axis=0)
            assert np.array_equal(got[:A.nq].reshape(h, A.kp_qk, -1)[:, :oq.shape[1] * unit], O.heads_rows(O.compact(full["wq"], rq, 0, dh, unit), h))
            assert np.array_equal(got[A.nq:A.nq + A.nk].reshape(hk, A.kp_qk, -1)[:, :oq.shape[1] * unit], O.heads_rows(O.compact(full["wk"], oq, 0, dh, unit), hk))
            assert np.array_equal(got[A.nq + A.nk:].reshape(hk, A.kp_vo, -1)[:, :ov.shape[1]], O.heads_rows(O.compact(full["wv"], ov, 0, dh), hk))
            assert not got[:A.nq].reshape(h, A.kp_qk, -1)[:, oq.shape[1] * unit:].any()
            wo = host(A.wo_c).reshape(st.d, h, A.kp_vo)
            assert np.array_equal(wo[:, :, :ov.shape[1]].transpose(1, 0, 2), O.heads_cols(O.compact(full["wo"], np.repeat(ov, h // hk, axis=0), 1, dh), h))
            assert np.array_equal(host(F.w2_c)[:, :F.k], O.compact(full["w2"], of, 1, dff))
            assert np.array_equal(host(F.gate_rows(F.w1_c))[:F.k], O.compact(full["w1"], of, 0, dff))
            if cfg["gated"]:
                assert np.array_equal(host(F.up_rows(F.w1_c))[:F.k], O.compact(full["w1b"], of, 0, dff))
            if cfg["bias"]:
                assert np.array_equal(host(F.b1_c)[:F.k], O.compact(full["b1"], of, 0, dff))
                assert np.array_equal(host(A.bqkv_c[:A.nq]).reshape(h, A.kp_qk)[:, :oq.shape[1]], O.compact(full["bq"], rq, 0, dh).reshape(h, -1))
        if cfg["rope"]:
            assert np.array_equal(a.rope_idx.cpu().numpy(), oq)
            ang = O.rope_angles(oq, st.L, dh)                                   # [h_kv, L, kept blocks]
            assert_close(a.cos[:, :, :oq.shape[1]], np.cos(ang), "f32", "cos table")
            assert_close(a.sin[:, :, :oq.shape[1]], np.sin(ang), "f32", "sin table")
    # a training step runs through the shrunk stack; its logits are those of the oracle's forward pass over the same
    # compact weights (first layer's attention checked through the whole stack's output)
    logits = st.forward(ids).clone()
    loss = st.train_step(ids, tgt)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(logits.float()).all()) and np.isfinite(float(loss))
    # moments moved with their rows: shrink once more and compare against a gather of the moments as they were
    before = [{fam: (ly.ffn[fam].w2_c.clone(), ly.attn[fam].wo_c.clone()) for fam in ("m", "v")} for ly in st.layers]
    k_old = st.k
    st.shrink((1, 4))
    for li, ly in enumerate(st.layers):
        iv, iff = ly.idx[1].cpu().numpy(), ly.idx[2].cpu().numpy()
        for fam in ("m", "v"):
            w2_old, wo_old = (host(t) for t in before[li][fam])
            F, A = ly.ffn[fam], ly.attn[fam]
            assert np.array_equal(host(F.w2_c)[:, :F.k], w2_old[:, iff[0]])
            kp_old = wo_old.shape[1] // h
            want = np.stack([wo_old[:, g * kp_old:(g + 1) * kp_old][:, iv[g // (h // hk)]] for g in range(h)])
            assert np.array_equal(host(A.wo_c).reshape(st.d, h, A.kp_vo)[:, :, :A.k_vo].transpose(1, 0, 2), want)
        assert float(ly.ffn["m"].w2_c.float().abs().max()) > 0.0      # the step did leave moments behind
    assert st.k[2] < k_old[2]
    loss2 = st.train_step(ids, tgt)
    assert np.isfinite(float(loss2))
