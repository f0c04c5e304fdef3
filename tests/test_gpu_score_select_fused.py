"""GPU parity of ecospa_score_select (steps 1 and 2 in two launches) against the fp64 oracle: the scores within the fp32
tolerance, the indices bit-exact given the scores the GPU wrote."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd import synth
from util import assert_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def check(scores, idx, want_scores, ks):
    for s, i, w, k in zip(scores, idx, want_scores, ks):
        assert s.shape == w.shape and i.shape == (w.shape[0], k)
        assert_close(s, w, "f32", "score")
        np.testing.assert_array_equal(i.cpu().numpy(), O.select_topk(s.cpu().numpy(), k))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("h,dh,d,unit,dff,gated", [(16, 64, 1024, 1, 4096, False), (32, 64, 2048, 2, 5461, True),
                                                   (3, 64, 192, 1, 200, False), (2, 8, 24, 2, 37, True),
                                                   (20, 128, 320, 1, 70, False)])
def test_layer_pairs(ctx, h, dh, d, unit, dff, gated, dtype):
    """The three pairs of a layer; head groups of up to 64 units go to wavefront teams, wider heads (128) and the FFN
    pair to workgroup teams, whatever the number of groups."""
    t = synth.attn_layer(4, 1, 2, d, h, dh, dtype=dtype, structure="pretrained", bias=False)
    f = synth.ffn_layer(5, 2, d, dff, gated=gated, dtype=dtype, bias=False)
    kind = O.PAIR_FFN_GATED if gated else O.PAIR_FFN
    want = [O.coupled_score(O.PAIR_QK, t["wq"], t["wk"], h, dh, unit),
            O.coupled_score(O.PAIR_VO, t["wv"], t["wo"], h, dh),
            O.coupled_score(kind, f["w1"], f["w2"], 1, dff, w1b=f.get("w1b"))]
    g = {k: dev(v, dtype) for k, v in t.items()}
    fw = {k: dev(v, dtype) for k, v in f.items() if k in ("w1", "w2", "w1b")}
    mk = B.Context.make_pair
    pairs = [mk(B.PAIR_QK, g["wq"], g["wk"], h, dh, unit), mk(B.PAIR_VO, g["wv"], g["wo"], h, dh, 1),
             mk(kind, fw["w1"], fw["w2"], 1, dff, 1, fw.get("w1b"))]
    ks = [max(1, dh // unit // 2), dh // 2, max(1, dff // 2)]
    scores, idx = ctx.ecospa_score_select(pairs, ks)
    check(scores, idx, want, ks)
    # the second member stored with its units as rows, and every count from 1 to all
    wo_r, w2_r = g["wo"].t().contiguous(), fw["w2"].t().contiguous()
    pairs_r = [pairs[0], mk(B.PAIR_VO, g["wv"], wo_r, h, dh, 1, w2_rows=True),
               mk(kind, fw["w1"], w2_r, 1, dff, 1, fw.get("w1b"), w2_rows=True)]
    for ks in ([1, 1, 1], [dh // unit, dh, dff]):
        scores, idx = ctx.ecospa_score_select(pairs_r, ks)
        check(scores, idx, want, ks)


def test_ties_go_to_the_lower_index(ctx):
    t = synth.ffn_layer(11, 2, 64, 256, dtype="bf16", structure="ties", bias=False)
    w1, w2 = dev(t["w1"], "bf16"), dev(t["w2"], "bf16")
    scores, idx = ctx.ecospa_score_select([B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, 256, 1)], [128])
    s = scores[0].cpu().numpy()
    assert np.array_equal(s[0, 0:4], s[0, 4:8])
    np.testing.assert_array_equal(idx[0].cpu().numpy(), O.select_topk(s, 128))


def test_many_pairs_span_several_launches(ctx):
    pairs, want, keep, ks = [], [], [], []
    for i in range(60):
        t = synth.ffn_layer(100 + i, 2, 40, 56 + i, dtype="bf16", bias=False)
        w1, w2 = dev(t["w1"], "bf16"), dev(t["w2"], "bf16")
        keep += [w1, w2]
        pairs.append(B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, 56 + i, 1))
        want.append(O.coupled_score(O.PAIR_FFN, t["w1"], t["w2"], 1, 56 + i))
        ks.append(7 + i // 2)
    scores, idx = ctx.ecospa_score_select(pairs, ks)
    check(scores, idx, want, ks)


def test_errors_before_any_launch(ctx):
    t = synth.ffn_layer(3, 2, 16, 32, dtype="f32", bias=False)
    w1, w2 = dev(t["w1"]), dev(t["w2"])
    p = [B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, 32, 1)]
    idx = [torch.empty((1, 40), dtype=torch.int32, device="cuda")]
    for k in (0, 33):
        with pytest.raises(B.EcospaError) as e:
            ctx.ecospa_score_select(p, [k], idx=idx)
        assert e.value.code == B.ERR_K


@pytest.mark.parametrize("n", [8192, 8193, 11008, 70000])
def test_large_groups_take_the_uncached_selection_path(ctx, n):
    """More than 8 units per thread of a selecting workgroup: the keys are read again from the scores in every pass."""
    t = synth.ffn_layer(7, 2, 24, n, dtype="bf16", bias=False)
    w1, w2 = dev(t["w1"], "bf16"), dev(t["w2"], "bf16")
    want = [O.coupled_score(O.PAIR_FFN, t["w1"], t["w2"], 1, n)]
    ks = [n // 3]
    scores, idx = ctx.ecospa_score_select([B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, n, 1)], ks)
    check(scores, idx, want, ks)


def test_grouped_query_pairs(ctx):
    """Query heads that share a key/value head (Eq. 5): one score row and one index list per key/value head."""
    h, hkv, dh, d = 8, 2, 64, 96
    t = synth.attn_layer(9, 1, 2, d, h, dh, dtype="bf16", structure="pretrained", bias=False)
    wq, wo = dev(t["wq"], "bf16"), dev(t["wo"], "bf16")
    wk, wv = dev(t["wk"][:hkv * dh], "bf16"), dev(t["wv"][:hkv * dh], "bf16")
    mk = B.Context.make_pair
    pairs = [mk(B.PAIR_QK, wq, wk, hkv, dh, 2, rep1=h // hkv), mk(B.PAIR_VO, wv, wo, hkv, dh, 1, rep2=h // hkv)]
    ks = [10, 20]
    ref = ctx.ecospa_coupled_score(pairs)
    scores, idx = ctx.ecospa_score_select(pairs, ks)
    for s, r, i, k in zip(scores, ref, idx, ks):
        assert_close(s, r.cpu().numpy().astype(np.float64), "f32", "gqa score")     # the separate call is checked against the oracle elsewhere
        np.testing.assert_array_equal(i.cpu().numpy(), O.select_topk(s.cpu().numpy(), k))
