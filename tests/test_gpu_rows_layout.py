"""The second member of a pair stored with its units as rows ([units, d]: the orientation of B in App. A.1) instead of
the Linear layout [d, units]: scores and pair importances against the oracle (which sees the matrix in the layout it is
written for), and blocks that gather rows only against blocks built on the Linear layout - same index lists, same
compact matrices bit for bit, same forward and backward results bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd import synth
from paper_2511_11641_amd.layer import AttnBlock, FfnBlock, rows_aligned
from util import assert_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def tr(t):
    return t.t().contiguous()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,d,gated", [(1024, 256, False), (1073, 264, False), (5461, 2048, True), (37, 8, True)])
def test_score_and_importance_ffn_rows_layout(ctx, n, d, gated, dtype):
    t = synth.ffn_layer(3, 4, d, n, gated=gated, dtype=dtype, structure="pretrained", bias=False)
    kind = O.PAIR_FFN_GATED if gated else O.PAIR_FFN
    w1, w2, w1b = dev(t["w1"], dtype), tr(dev(t["w2"], dtype)), dev(t.get("w1b"), dtype)
    pair = B.Context.make_pair(kind, w1, w2, 1, n, 1, w1b, w2_rows=True)
    assert pair.d2 == d and pair.ld2 == d
    got = ctx.ecospa_coupled_score([pair])[0]
    assert_close(got, O.coupled_score(kind, t["w1"], t["w2"], 1, n, w1b=t.get("w1b")), "f32", "ffn score, units as rows")
    fi = ctx.ecospa_pair_fisher([pair], 64.0)[0]
    assert_close(fi, O.pair_fisher(kind, t["w1"], t["w2"], 1, n, 64.0, g1b=t.get("w1b")), "f32", "Eq. 8, units as rows")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("h,hk,dh,d", [(16, 16, 64, 1024), (8, 2, 64, 512), (3, 3, 64, 192)])
def test_score_vo_rows_layout(ctx, h, hk, dh, d, dtype):
    t = synth.attn_layer(4, 1, 2, d, h, dh, dtype=dtype, structure="pretrained", bias=False)
    wv = t["wv"][:hk * dh]
    want = O.coupled_score(O.PAIR_VO, wv, t["wo"], hk, dh, rep2=h // hk)
    pair = B.Context.make_pair(B.PAIR_VO, dev(wv, dtype), tr(dev(t["wo"], dtype)), hk, dh, 1, rep2=h // hk, w2_rows=True)
    keep = pair
    assert_close(ctx.ecospa_coupled_score([keep])[0], want, "f32", "vo score, units as rows")


@pytest.mark.parametrize("gated,n,k", [(False, 1024, 512), (True, 1365, 409), (False, 200, 77)])
def test_ffn_block_rows_layout_equals_linear_layout(ctx, gated, n, k):
    d, Bsz, L = 256, 2, 96
    t = synth.ffn_layer(11, Bsz * L, d, n, gated=gated, dtype="bf16", bias=not gated)
    g = {kk: dev(v, "bf16") for kk, v in t.items()}
    act = B.ACT_SWIGLU if gated else B.ACT_GELU_ERF
    lin = FfnBlock(ctx, g["w1"], g.get("b1"), rows_aligned(g["w2"]), g.get("b2"), act, g.get("w1b"), transposed=True)
    row = FfnBlock(ctx, g["w1"], g.get("b1"), tr(g["w2"]), g.get("b2"), act, g.get("w1b"), transposed=True, w2_rows=True)
    s_lin, s_row = lin.score(), row.score()
    assert_close(s_row, s_lin.double().cpu().numpy(), "f32", "scores of the two layouts")
    idx = ctx.ecospa_select_topk(s_lin, k)
    lin.compact(idx).alloc(Bsz, L)
    row.compact(idx).alloc(Bsz, L)
    for name in ("w1_c", "w2_c", "w1_t", "w2_t"):
        assert torch.equal(getattr(lin, name), getattr(row, name)), name
    y1, y2 = lin.fwd(g["x"]).clone(), row.fwd(g["x"]).clone()
    assert torch.equal(y1, y2)
    dx1, dx2 = lin.bwd(g["x"], g["dy"]).clone(), row.bwd(g["x"], g["dy"]).clone()
    assert torch.equal(dx1, dx2) and torch.equal(lin.dw1_c, row.dw1_c) and torch.equal(lin.dw2_c, row.dw2_c)
    # removal for good from the rows layout: the transposed copy is what the next round gathers from
    row.rebase()
    idx2 = ctx.ecospa_select_topk(row.score(), k // 2)
    row.compact(idx2)
    lin.rebase()
    lin.compact(idx2)
    assert torch.equal(row.w2_c, lin.w2_c) and torch.equal(row.w1_c, lin.w1_c)


@pytest.mark.parametrize("rope,h,hk", [(False, 4, 4), (True, 4, 2)])
def test_attn_block_rows_layout_equals_linear_layout(ctx, rope, h, hk):
    d, dh, Bsz, L = 256, 64, 2, 80
    t = synth.attn_layer(12, Bsz, L, d, h, dh, dtype="bf16", bias=not rope)
    g = {kk: dev(v, "bf16") for kk, v in t.items()}
    for nm in ("wk", "wv", "bk", "bv"):
        if g.get(nm) is not None:
            g[nm] = g[nm][:hk * dh].contiguous()
    mk = lambda wo, rows: AttnBlock(ctx, g["wq"], g["wk"], g["wv"], wo, g.get("bq"), g.get("bk"), g.get("bv"), g.get("bo"), h, dh,
                                    rope=rope, h_kv=hk, transposed=True, wo_rows=rows)
    lin, row = mk(g["wo"], False), mk(tr(g["wo"]), True)
    (q1, v1), (q2, v2) = lin.score(), row.score()
    assert torch.equal(q1, q2)
    assert_close(v2, v1.double().cpu().numpy(), "f32", "vo scores of the two layouts")
    unit = 2 if rope else 1
    iq, iv = ctx.ecospa_select_topk(q1, 32 // unit), ctx.ecospa_select_topk(v1, 32)
    lin.compact(iq, iv).alloc(Bsz, L)
    row.compact(iq, iv).alloc(Bsz, L)
    for name in ("wqkv_c", "wo_c", "wqkv_t", "wo_t"):
        assert torch.equal(getattr(lin, name), getattr(row, name)), name
    assert torch.equal(lin.fwd(g["x"]), row.fwd(g["x"]))
    assert torch.equal(lin.bwd(g["x"], g["dy"]), row.bwd(g["x"], g["dy"]))
    assert torch.equal(lin.dwo_c, row.dwo_c) and torch.equal(lin.dwqkv_c, row.dwqkv_c)
