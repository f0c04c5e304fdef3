"""GPU parity (through the C ABI) of the reduced attention block forward/backward against the
fp64 oracle: compacted heads, separate kept widths for QK and VO, causal and full masks, RoPE."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd import synth
from paper_2511_11641_amd.layer import AttnBlock
from util import assert_close, dev, host, pad_cols, pad_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def run_attn_case(ctx, seed, Bsz, L, d, h, dh, k_qk, k_vo, *, rope, causal, bias=True, structure="scratch",
                  wscale=1.0, dtype="bf16", transposed=False):
    """k_qk counts kept dimensions (even when rope: kept rotary blocks = k_qk / 2)."""
    t = synth.attn_layer(seed, Bsz, L, d, h, dh, dtype=dtype, structure=structure, bias=bias)
    if wscale != 1.0:
        for nm in ("wq", "wk", "wv", "wo"):
            t[nm] = synth.round_to(t[nm] * np.float32(wscale), dtype)
    unit = 2 if rope else 1
    vqk = O.coupled_score(O.PAIR_QK, t["wq"], t["wk"], h, dh, unit)
    vvo = O.coupled_score(O.PAIR_VO, t["wv"], t["wo"], h, dh)
    iq = O.select_topk(vqk.astype(np.float32), k_qk // unit)
    iv = O.select_topk(vvo.astype(np.float32), k_vo)
    g = {nm: dev(a, dtype) for nm, a in t.items()}
    blk = AttnBlock(ctx, g["wq"], g["wk"], g["wv"], g["wo"], g.get("bq"), g.get("bk"), g.get("bv"), g.get("bo"),
                    h, dh, rope=rope, causal=causal, transposed=transposed, bias_grads=True)
    blk.compact(torch.from_numpy(iq).cuda(), torch.from_numpy(iv).cuda()).alloc(Bsz, L)
    y = blk.fwd(g["x"])
    dx = blk.bwd(g["x"], g["dy"])
    torch.cuda.synchronize()

    scale = 1.0 / np.sqrt(dh)
    ang = O.rope_angles(iq, L, dh) if rope else None
    wq = O.heads_rows(O.compact(t["wq"], iq, 0, dh, unit), h)
    wk = O.heads_rows(O.compact(t["wk"], iq, 0, dh, unit), h)
    wv = O.heads_rows(O.compact(t["wv"], iv, 0, dh), h)
    wo = O.heads_cols(O.compact(t["wo"], iv, 1, dh), h)
    kw = {}
    if bias:
        kw = dict(bq=O.compact(t["bq"], iq, 0, dh, unit).reshape(h, -1),
                  bk=O.compact(t["bk"], iq, 0, dh, unit).reshape(h, -1),
                  bv=O.compact(t["bv"], iv, 0, dh).reshape(h, -1), bo=t["bo"])
    yo, sv = O.attn_fwd(t["x"], wq, wk, wv, wo, Bsz, L, scale, causal, angles=ang, **kw)
    go = O.attn_bwd(t["x"], t["dy"], wq, wk, wv, wo, Bsz, L, scale, sv, angles=ang)

    kq, kpq, kpv = k_qk, blk.kp_qk, blk.kp_vo
    errs = {"y": assert_close(y, yo, dtype, "y"), "dx": assert_close(dx, go["dx"], dtype, "dx")}
    want_dw = np.concatenate([pad_rows(go["dwq"].reshape(h * kq, d), h, kq, kpq),
                              pad_rows(go["dwk"].reshape(h * kq, d), h, kq, kpq),
                              pad_rows(go["dwv"].reshape(h * k_vo, d), h, k_vo, kpv)])
    errs["dwqkv"] = assert_close(blk.dwqkv_c, want_dw, dtype, "dwqkv")
    nq = h * kpq
    errs["dwq"] = assert_close(blk.dwqkv_c[:nq], want_dw[:nq], dtype, "dwq")
    errs["dwk"] = assert_close(blk.dwqkv_c[nq:2 * nq], want_dw[nq:2 * nq], dtype, "dwk")
    errs["dwv"] = assert_close(blk.dwqkv_c[2 * nq:], want_dw[2 * nq:], dtype, "dwv")
    want_db = np.concatenate([pad_rows(go["dbq"].reshape(-1), h, kq, kpq), pad_rows(go["dbk"].reshape(-1), h, kq, kpq),
                              pad_rows(go["dbv"].reshape(-1), h, k_vo, kpv)])
    errs["dbq"] = assert_close(blk.dbqkv_c[:nq], want_db[:nq], dtype, "dbq")
    errs["dbv"] = assert_close(blk.dbqkv_c[2 * nq:], want_db[2 * nq:], dtype, "dbv")
    # the key bias shifts every score of a row equally, so its true gradient is ~0: compare absolutely
    dbk = host(blk.dbqkv_c[nq:2 * nq])
    assert np.abs(dbk - want_db[nq:2 * nq]).max() <= 2e-2 * max(np.abs(want_db[:nq]).max(), 1e-6), "dbk"
    want_dwo = pad_cols(go["dwo"].transpose(1, 0, 2).reshape(d, h * k_vo), h, k_vo, kpv)
    errs["dwo"] = assert_close(blk.dwo_c, want_dwo, dtype, "dwo")
    errs["dbo"] = assert_close(blk.dbo, go["dbo"], dtype, "dbo")
    # log-sum-exp the forward pass keeps
    lse = host(blk.lse).reshape(Bsz, h, L)
    for b in (0, Bsz - 1):
        for i in (0, h - 1):
            s = (sv["q"][(b, i)] @ sv["k"][(b, i)].T) * scale
            if causal:
                s = np.where(np.triu(np.ones((L, L), bool), 1), -np.inf, s)
            ref = np.log(np.exp(s - s.max(1, keepdims=True)).sum(1)) + s.max(1)
            np.testing.assert_allclose(lse[b, i], ref, atol=5e-2)
    return errs


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("k_qk,k_vo", [(32, 32), (64, 64), (48, 19), (20, 64), (16, 48)])
def test_attn_small_no_rope(ctx, k_qk, k_vo, causal):
    # L = 200: two query tiles with a ragged tail, four key tiles with a ragged tail
    run_attn_case(ctx, 31, 2, 200, 128, 3, 64, k_qk, k_vo, rope=False, causal=causal, wscale=6.0)


@pytest.mark.parametrize("k_qk,k_vo", [(32, 32), (64, 64), (38, 21)])
def test_attn_small_rope(ctx, k_qk, k_vo):
    run_attn_case(ctx, 32, 2, 130, 128, 4, 64, k_qk, k_vo, rope=True, causal=True, bias=False, wscale=6.0)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("k_qk,k_vo", [(128, 128), (96, 80), (72, 32), (32, 112), (128, 64), (64, 100)])
def test_attn_heads_of_128_dims_no_rope(ctx, k_qk, k_vo, causal):
    """Heads of 128 dims (the LLaMA-7B shape), dense and at keep ratios that leave more than 64: the 128-wide kernels,
    alone and mixed with the narrower ones on the other side of the pair."""
    run_attn_case(ctx, 41, 2, 200, 256, 2, 128, k_qk, k_vo, rope=False, causal=causal, wscale=4.0)


@pytest.mark.parametrize("k_qk,k_vo,transposed", [(128, 128, False), (96, 72, True), (80, 128, False)])
def test_attn_heads_of_128_dims_rope(ctx, k_qk, k_vo, transposed):
    run_attn_case(ctx, 42, 2, 300, 256, 3, 128, k_qk, k_vo, rope=True, causal=True, bias=False, wscale=4.0, transposed=transposed)


def test_attn_tiny_sequence(ctx):
    run_attn_case(ctx, 33, 3, 5, 64, 2, 64, 32, 32, rope=True, causal=True, wscale=6.0)


def test_attn_gpt2_medium_heads(ctx):
    """16 heads x 64 at d=1024, keep 32/32, L=1024 (one batch element keeps the oracle quick)."""
    run_attn_case(ctx, 34, 1, 1024, 1024, 16, 64, 32, 32, rope=False, causal=True, structure="pretrained")


def test_attn_llama_heads(ctx):
    """32 heads x 64 at d=2048, RoPE, keep 16 of 32 rotary blocks and 32 of 64 value dims, L=256."""
    run_attn_case(ctx, 35, 2, 256, 2048, 32, 64, 32, 32, rope=True, causal=True, bias=False, structure="pretrained")


@pytest.mark.parametrize("k_qk,k_vo,rope", [(32, 32, False), (48, 19, False), (32, 64, True)])
def test_attn_backward_with_transposed_weight_copies(ctx, k_qk, k_vo, rope):
    """The input-gradient contractions read transposed copies of the compact weights: same results to tolerance."""
    run_attn_case(ctx, 33, 2, 200, 256, 4, 64, k_qk, k_vo, rope=rope, causal=True, transposed=True)
    run_attn_case(ctx, 34, 8, 1024, 1024, 16, 64, 32, 32, rope=rope, causal=True, transposed=True)


@pytest.mark.parametrize("rope,transposed", [(False, False), (True, True)])
def test_attn_few_tokens_split_contractions(ctx, rope, transposed):
    """2 x 128 tokens at d = 2048: the projections and the gradient of the attention output run split along K."""
    run_attn_case(ctx, 36, 2, 128, 2048, 16, 64, 32, 32, rope=rope, causal=True, transposed=transposed)


@pytest.mark.parametrize("rope,L,d", [(False, 200, 256), (True, 128, 2048)])
def test_attn_forward_only_keeps_nothing_and_agrees(ctx, rope, L, d):
    """Forward without saved tensors (inference): bit for bit the training forward's output."""
    h, dh = (4, 64) if d == 256 else (16, 64)
    t = synth.attn_layer(37, 2, L, d, h, dh, dtype="bf16")
    g = {nm: dev(a, "bf16") for nm, a in t.items()}
    blk = AttnBlock(ctx, g["wq"], g["wk"], g["wv"], g["wo"], g["bq"], g["bk"], g["bv"], g["bo"], h, dh, rope=rope, causal=True, bias_grads=True)
    rng = np.random.default_rng(L)
    units = dh // (2 if rope else 1)
    iq = torch.from_numpy(np.stack([np.sort(rng.choice(units, units // 2, replace=False)) for _ in range(h)]).astype(np.int32)).cuda()
    iv = torch.from_numpy(np.stack([np.sort(rng.choice(dh, 32, replace=False)) for _ in range(h)]).astype(np.int32)).cuda()
    blk.compact(iq, iv).alloc(2, L)
    y_train = blk.fwd(g["x"]).clone()
    blk.qkv.fill_(float("nan"))
    y_inf = blk.fwd(g["x"], save=False)
    assert torch.equal(y_inf, y_train)
    assert bool(torch.isnan(blk.qkv.float()).all())


def test_attn_backward_with_optional_outputs(ctx):
    """The input gradient alone and the weight/bias gradients without it equal what the full backward writes."""
    h, dh, L, d = 4, 64, 200, 256
    t = synth.attn_layer(38, 2, L, d, h, dh, dtype="bf16")
    g = {nm: dev(a, "bf16") for nm, a in t.items()}
    blk = AttnBlock(ctx, g["wq"], g["wk"], g["wv"], g["wo"], g["bq"], g["bk"], g["bv"], g["bo"], h, dh, rope=True, causal=True, bias_grads=True)
    rng = np.random.default_rng(9)
    iq = torch.from_numpy(np.stack([np.sort(rng.choice(dh // 2, 16, replace=False)) for _ in range(h)]).astype(np.int32)).cuda()
    iv = torch.from_numpy(np.stack([np.sort(rng.choice(dh, 32, replace=False)) for _ in range(h)]).astype(np.int32)).cuda()
    blk.compact(iq, iv).alloc(2, L)
    blk.fwd(g["x"])
    dx = blk.bwd(g["x"], g["dy"]).clone()
    names = ("dwqkv_c", "dbqkv_c", "dwo_c", "dbo")
    full = {nm: getattr(blk, nm).clone() for nm in names}
    for nm in names:
        getattr(blk, nm).fill_(float("nan"))
    only_dx = torch.full_like(dx, float("nan"))
    ctx.ecospa_coupled_bwd(blk._desc, g["x"], g["dy"], blk.saved, only_dx, B.Grads())
    assert torch.equal(only_dx, dx)
    assert all(bool(torch.isnan(getattr(blk, nm).float()).all()) for nm in names)
    ctx.ecospa_coupled_bwd(blk._desc, g["x"], g["dy"], blk.saved, None, blk.grads)
    for nm, want in full.items():
        assert torch.equal(getattr(blk, nm), want), nm


def test_attn_keep_all_is_dense(ctx):
    run_attn_case(ctx, 36, 2, 256, 256, 4, 64, 64, 64, rope=True, causal=True, wscale=4.0)


def test_attn_is_deterministic(ctx):
    t = synth.attn_layer(37, 2, 300, 128, 2, 64, dtype="bf16")
    g = {nm: dev(a, "bf16") for nm, a in t.items()}
    blk = AttnBlock(ctx, g["wq"], g["wk"], g["wv"], g["wo"], g["bq"], g["bk"], g["bv"], g["bo"], 2, 64, rope=False, bias_grads=True)
    idx = torch.arange(0, 64, 2, dtype=torch.int32).repeat(2, 1).cuda()
    blk.compact(idx, idx).alloc(2, 300)
    outs = []
    for _ in range(2):
        blk.fwd(g["x"])
        blk.bwd(g["x"], g["dy"])
        outs.append([blk.y.clone(), blk.dx.clone(), blk.dwqkv_c.clone(), blk.dwo_c.clone(), blk.dbqkv_c.clone()])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_attn_fp32_is_reported_unsupported(ctx):
    t = synth.attn_layer(38, 1, 16, 64, 2, 32, dtype="f32")
    g = {nm: dev(a, "f32") for nm, a in t.items()}
    blk = AttnBlock(ctx, g["wq"], g["wk"], g["wv"], g["wo"], None, None, None, None, 2, 32, rope=False, bias_grads=True)
    idx = torch.arange(16, dtype=torch.int32).repeat(2, 1).cuda()
    blk.compact(idx, idx).alloc(1, 16)
    with pytest.raises(B.EcospaError) as e:
        blk.fwd(g["x"])
    assert e.value.code == B.ERR_DTYPE
