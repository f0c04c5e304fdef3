"""GPU parity (through the C ABI) of steps 1-3 against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd import synth
from util import assert_close, dev, host, interleave_rows, pad_cols, pad_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


# ---- score -----------------------------------------------------------------------------------
FFN_SHAPES = [  # (n, d, gated)
    (1024, 256, False),   # the fp32 single-pair configuration
    (1073, 264, False),   # ragged kept-dimension counts as in the paper's Tables 10-11
    (4096, 1024, False),
    (5461, 2048, True),
    (37, 8, True),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("structure", ["scratch", "pretrained"])
@pytest.mark.parametrize("n,d,gated", FFN_SHAPES)
def test_score_ffn(ctx, n, d, gated, structure, dtype):
    t = synth.ffn_layer(3, 4, d, n, gated=gated, dtype=dtype, structure=structure, bias=False)
    kind = O.PAIR_FFN_GATED if gated else O.PAIR_FFN
    want = O.coupled_score(kind, t["w1"], t["w2"], 1, n, w1b=t.get("w1b"))
    w1, w2, w1b = dev(t["w1"], dtype), dev(t["w2"], dtype), dev(t.get("w1b"), dtype)
    got = ctx.ecospa_coupled_score([B.Context.make_pair(kind, w1, w2, 1, n, 1, w1b)])[0]
    assert got.shape == (1, n)
    assert_close(got, want, "f32", "ffn score")
    assert abs(float(got.double().pow(2).sum().sqrt()) - 1.0) < 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("h,dh,d,unit", [(16, 64, 1024, 1), (32, 64, 2048, 2), (3, 64, 192, 1), (2, 8, 24, 2)])
def test_score_attention_pairs_batched(ctx, h, dh, d, unit, dtype):
    t = synth.attn_layer(4, 1, 2, d, h, dh, dtype=dtype, structure="pretrained", bias=False)
    f = synth.ffn_layer(5, 2, d, 200, dtype=dtype, bias=False)
    want = [O.coupled_score(O.PAIR_QK, t["wq"], t["wk"], h, dh, unit),
            O.coupled_score(O.PAIR_VO, t["wv"], t["wo"], h, dh),
            O.coupled_score(O.PAIR_FFN, f["w1"], f["w2"], 1, 200)]
    g = {k: dev(v, dtype) for k, v in t.items()}
    fw1, fw2 = dev(f["w1"], dtype), dev(f["w2"], dtype)
    mk = B.Context.make_pair
    got = ctx.ecospa_coupled_score([mk(B.PAIR_QK, g["wq"], g["wk"], h, dh, unit),
                                    mk(B.PAIR_VO, g["wv"], g["wo"], h, dh, 1),
                                    mk(B.PAIR_FFN, fw1, fw2, 1, 200, 1)])
    for a, b, nm in zip(got, want, ("qk", "vo", "ffn")):
        assert a.shape == b.shape
        assert_close(a, b, "f32", nm)


def test_score_many_pairs_spans_several_launch_batches(ctx):
    pairs, want, keep = [], [], []
    for i in range(30):
        t = synth.ffn_layer(100 + i, 2, 40, 56 + i, dtype="bf16", bias=False)
        w1, w2 = dev(t["w1"], "bf16"), dev(t["w2"], "bf16")
        keep += [w1, w2]
        pairs.append(B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, 56 + i, 1))
        want.append(O.coupled_score(O.PAIR_FFN, t["w1"], t["w2"], 1, 56 + i))
    got = ctx.ecospa_coupled_score(pairs)
    for a, b in zip(got, want):
        assert_close(a, b, "f32", "batched score")


def test_score_zero_group_and_strided_views(ctx):
    n, d = 64, 48
    big1 = torch.randn(n, d + 16, device="cuda", dtype=torch.float32)
    big2 = torch.randn(d, n + 8, device="cuda", dtype=torch.float32)
    w1, w2 = big1[:, :d], big2[:, :n]          # leading dimensions larger than the extents
    w1[5].zero_()
    got = ctx.ecospa_coupled_score([B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, n, 1)])[0]
    want = O.coupled_score(O.PAIR_FFN, host(w1), host(w2), 1, n)
    assert_close(got, want, "f32", "strided")
    assert float(got[0, 5]) == 0.0
    z = torch.zeros(n, d, device="cuda", dtype=torch.float32)
    got = ctx.ecospa_coupled_score([B.Context.make_pair(B.PAIR_FFN, z, w2.contiguous(), 1, n, 1)])[0]
    assert torch.all(got == 0)


# ---- select ----------------------------------------------------------------------------------
@pytest.mark.parametrize("groups,n,k", [(1, 1024, 512), (16, 64, 32), (16, 64, 48), (16, 64, 19), (1, 4096, 2048),
                                        (1, 4096, 1228), (1, 5461, 2730), (32, 32, 16), (3, 7, 7), (2, 300, 1),
                                        (1, 70000, 35000)])
def test_select_bit_exact(ctx, groups, n, k):
    s = np.abs(synth.normal(7, 200, (groups, n))).astype(np.float32)
    got = ctx.ecospa_select_topk(dev(s), k)
    np.testing.assert_array_equal(got.cpu().numpy(), O.select_topk(s, k))


def test_select_ties_signed_zero_nan_inf(ctx):
    g = np.random.Generator(np.random.Philox(key=[9, 1]))
    n = 777
    s = g.integers(0, 12, size=(5, n)).astype(np.float32) / 8.0          # heavy exact ties
    s[1, ::7] = -0.0
    s[1, 1::7] = 0.0
    s[2, ::5] = np.nan
    s[2, 1::9] = -np.inf
    s[2, 2::11] = np.inf
    s[3] = 0.25
    s[4] = -s[4]
    for k in (1, 2, 100, 388, 776, 777):
        got = ctx.ecospa_select_topk(dev(s), k).cpu().numpy()
        np.testing.assert_array_equal(got, O.select_topk(s, k), err_msg=f"k={k}")


def test_select_on_gpu_scores_of_tied_weights(ctx):
    """Duplicated inner dimensions give exactly tied scores; the lower index must win."""
    t = synth.ffn_layer(11, 2, 64, 256, dtype="bf16", structure="ties", bias=False)
    w1, w2 = dev(t["w1"], "bf16"), dev(t["w2"], "bf16")
    sc = ctx.ecospa_coupled_score([B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, 256, 1)])[0]
    s = sc.cpu().numpy()
    assert np.array_equal(s[0, 0:4], s[0, 4:8])          # ties really are exact on the GPU
    got = ctx.ecospa_select_topk(sc, 128).cpu().numpy()
    np.testing.assert_array_equal(got, O.select_topk(s, 128))


# ---- compact / scatter -----------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("groups,n,unit,k,kp,other", [(1, 1024, 1, 512, 512, 256), (16, 64, 1, 19, 32, 1024),
                                                      (32, 64, 2, 16, 16, 2048), (1, 5461, 1, 2730, 2736, 520),
                                                      (3, 10, 1, 4, 4, 7), (2, 12, 2, 3, 5, 9)])
def test_compact_and_scatter_both_axes(ctx, groups, n, unit, k, kp, other, dtype):
    nu = n // unit
    sc = np.abs(synth.normal(13, 201, (groups, nu))).astype(np.float32)
    idx_np = O.select_topk(sc, k)
    idx = torch.from_numpy(idx_np).cuda()
    src_np = synth.round_to(synth.normal(13, 202, (groups * n, other)), dtype)
    src = dev(src_np, dtype)
    # rows
    got = ctx.ecospa_compact(src, idx, 0, groups, n, unit, kp)
    want = pad_rows(O.compact(src_np, idx_np, 0, n, unit), groups, k * unit, kp * unit)
    np.testing.assert_array_equal(host(got), want)
    back = ctx.ecospa_scatter(got, idx, 0, groups, n, unit, kp)
    np.testing.assert_array_equal(host(back), O.scatter(O.compact(src_np, idx_np, 0, n, unit), idx_np, 0, n, unit))
    # columns
    srcT = src.t().contiguous()
    got = ctx.ecospa_compact(srcT, idx, 1, groups, n, unit, kp)
    want = pad_cols(O.compact(src_np.T, idx_np, 1, n, unit), groups, k * unit, kp * unit)
    np.testing.assert_array_equal(host(got), want)
    back = ctx.ecospa_scatter(got, idx, 1, groups, n, unit, kp)
    np.testing.assert_array_equal(host(back), O.scatter(O.compact(src_np.T, idx_np, 1, n, unit), idx_np, 1, n, unit))
    # vector (bias)
    vec = src[:, 0].contiguous()
    got = ctx.ecospa_compact(vec, idx, 1, groups, n, unit, kp)
    want = pad_rows(O.compact(src_np[:, 0], idx_np, 0, n, unit), groups, k * unit, kp * unit)
    np.testing.assert_array_equal(host(got), want)


def test_compact_keep_all_is_identity(ctx):
    w = dev(synth.normal(14, 203, (4 * 16, 40)), "bf16")
    idx = torch.arange(16, dtype=torch.int32).repeat(4, 1).cuda()
    assert torch.equal(ctx.ecospa_compact(w, idx, 0, 4, 16, 1, 16), w)


def test_rope_table(ctx):
    h, L, dh = 3, 50, 16
    idx_np = np.array([[0, 3, 7], [1, 2, 4], [5, 6, 7]], dtype=np.int32)
    cos, sin = ctx.ecospa_rope_table(torch.from_numpy(idx_np).cuda(), h, L, 3, 4, dh)
    ang = O.rope_angles(idx_np, L, dh)
    np.testing.assert_allclose(host(cos)[:, :, :3], np.cos(ang), atol=2e-7)
    np.testing.assert_allclose(host(sin)[:, :, :3], np.sin(ang), atol=2e-7)
    assert torch.all(cos[:, :, 3] == 1) and torch.all(sin[:, :, 3] == 0)


def test_select_and_compact_batches_match_single_calls(ctx):
    """The one-launch batch entry points give bit-identical results to item-by-item calls."""
    rng = np.random.default_rng(5)
    shapes = [(16, 64, 32), (3, 100, 37), (1, 4096, 2048), (2, 5461, 2730), (1, 7, 7)]
    scores = [torch.from_numpy(rng.standard_normal((g, n)).astype(np.float32)).cuda() for g, n, _ in shapes]
    scores[1][:, 10:20] = scores[1][:, 30:40]          # exact ties
    single = [ctx.ecospa_select_topk(s, k) for s, (_, _, k) in zip(scores, shapes)]
    outs = [torch.empty_like(i) for i in single]
    ctx.ecospa_select_topk_batch([ctx.select_item(s, k, o) for s, (_, _, k), o in zip(scores, shapes, outs)])
    for a, b, s, (_, _, k) in zip(single, outs, scores, shapes):
        assert torch.equal(a, b)
        assert np.array_equal(b.cpu().numpy(), O.select_topk(s.cpu().numpy(), k))
    # gathers and a scatter of different dtypes / axes in one launch
    g, n, k = shapes[0]
    idx = single[0]
    w_rows = torch.randn(g * n, 72, device="cuda").to(torch.bfloat16)
    w_cols = torch.randn(40, g * n, device="cuda")
    bias = torch.randn(g * n, device="cuda").to(torch.bfloat16)
    items, want = [], []
    for src, axis, kp in ((w_rows, 0, 48), (w_cols, 1, 32), (bias, 1, 32)):
        want.append(ctx.ecospa_compact(src, idx, axis, g, n, 1, kp))
        dst = torch.full_like(want[-1], 7)
        items.append((ctx.map_item(src, dst, idx, axis, g, n, 1, kp), dst))
    full = ctx.ecospa_scatter(want[1], idx, 1, g, n, 1, 32)
    dst = torch.full_like(full, 7)
    items.append((ctx.map_item(want[1], dst, idx, 1, g, n, 1, 32, scatter=True), dst))
    want.append(full)
    ctx.ecospa_compact_batch([it for it, _ in items])
    for (_, got), w in zip(items, want):
        assert torch.equal(got, w)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols,pad", [(2048, 1024, 0), (1536, 1024, 0), (64, 64, 0), (130, 72, 8), (7, 301, 3), (1, 1, 0)])
def test_transposed_copies_are_exact(ctx, rows, cols, pad, dtype):
    """dst = src^T, bit for bit (numpy's transpose is the definition), with leading dimensions wider than the rows."""
    a = synth.round_to(synth.normal(300, rows + cols, (rows, cols + pad)), dtype)
    src = dev(a, dtype)[:, :cols]
    dst_full = torch.full((cols, rows + pad), 7.0, dtype=src.dtype, device="cuda")
    ctx.ecospa_transpose_batch([B.Context.transpose_item(src, dst_full[:, :rows])])
    assert np.array_equal(host(dst_full[:, :rows]), a[:, :cols].T.astype(np.float64))
    assert torch.all(dst_full[:, rows:] == 7.0)                         # nothing written past the rows
    with pytest.raises(B.EcospaError) as e:
        it = B.Context.transpose_item(src, dst_full[:, :rows])
        it.ld_dst = rows - 1
        ctx.ecospa_transpose_batch([it])
    assert e.value.code == B.ERR_SHAPE


# ---- the debugging aid for the caller's contract on index lists ----------------------------------------
def test_check_indices_accepts_what_select_writes_and_names_bad_lists(ctx):
    s = torch.rand((6, 100), device="cuda")
    idx = ctx.ecospa_select_topk(s, 37)
    assert ctx.ecospa_check_indices(idx, 100)
    bad = idx.clone()
    bad[3, 10] = bad[3, 9]                      # not strictly ascending
    assert not ctx.ecospa_check_indices(bad, 100)
    bad = idx.clone()
    bad[5, 36] = 100                            # out of range
    assert not ctx.ecospa_check_indices(bad, 100)
    bad = idx.clone()
    bad[0, 0] = -1
    assert not ctx.ecospa_check_indices(bad, 100)
    # ragged lists: only the first k_group[g] entries count, what lies behind them may be anything (-1 padding)
    idx_t, k_t = ctx.ecospa_select_theta(s / s.sum(dim=1, keepdim=True), 0.8)
    assert ctx.ecospa_check_indices(idx_t, 100, k_group=k_t)
    k_bad = k_t.clone()
    k_bad[2] = 101                              # a count the list cannot hold
    assert not ctx.ecospa_check_indices(idx_t, 100, k_group=k_bad)
    k_bad = k_t.clone()
    k_bad[1] = min(int(k_t[1]) + 1, 100)        # reaches into the -1 padding (unless the row kept everything)
    if int(k_t[1]) < 100:
        assert not ctx.ecospa_check_indices(idx_t, 100, k_group=k_bad)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n,k", [(1073, 536), (5461, 2730), (37, 11)])
def test_column_gather_of_an_odd_width_with_padded_rows(ctx, n, k, dtype):
    """A second member with an odd inner width (d_ff = 5461) stored with a padded leading dimension: its column gather
    takes the path that fetches whole 16-byte pieces; bit-exact against the oracle, scatter back included."""
    rows = 70
    w = synth.round_to(synth.normal(61, 330, (rows, n)), dtype)
    idx = np.sort(np.random.default_rng(n).choice(n, k, replace=False)).astype(np.int32)[None, :]
    ld = (n + 31) // 32 * 32
    buf = torch.full((rows, ld), 7.0, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    buf[:, :n] = dev(w, dtype)
    src = buf[:, :n]
    kp = (k + 15) // 16 * 16
    got = ctx.ecospa_compact(src, torch.from_numpy(idx).cuda(), 1, 1, n, kp=kp)
    want = pad_cols(O.compact(w, idx, 1, n), 1, k, kp)
    assert np.array_equal(host(got), want.astype(np.float64))
    back = torch.full((rows, ld), 3.0, dtype=buf.dtype, device="cuda")
    ctx.ecospa_scatter(got, torch.from_numpy(idx).cuda(), 1, 1, n, kp=kp, out=back[:, :n])
    assert np.array_equal(host(back[:, :n]), O.scatter(O.compact(w, idx, 1, n), idx, 1, n).astype(np.float64))
    assert bool((back[:, n:] == 3.0).all())          # the padding of the rows is not touched


# ---- row gathers that write their transposed copy themselves, interleaved second source -------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("groups,n,unit,k,kp,other", [(1, 1024, 1, 512, 512, 256), (16, 64, 1, 19, 32, 1024),
                                                      (32, 64, 2, 16, 16, 2048), (1, 5461, 1, 2730, 2736, 520),
                                                      (3, 10, 1, 4, 4, 7), (2, 12, 2, 3, 5, 9), (1, 200, 1, 77, 80, 136)])
def test_row_gather_with_transposed_copy(ctx, groups, n, unit, k, kp, other, dtype):
    nu = n // unit
    sc = np.abs(synth.normal(17, 301, (groups, nu))).astype(np.float32)
    idx_np = O.select_topk(sc, k)
    idx = torch.from_numpy(idx_np).cuda()
    src_np = synth.round_to(synth.normal(17, 302, (groups * n, other)), dtype)
    src = dev(src_np, dtype)
    want = pad_rows(O.compact(src_np, idx_np, 0, n, unit), groups, k * unit, kp * unit)
    slots = groups * kp * unit
    dst = torch.full((slots, other), 7.0, dtype=src.dtype, device="cuda")
    # a transposed copy wider than the matrix (the columns of a larger buffer), the slots beside it untouched
    dst_t_buf = torch.full((other, slots + 8), 7.0, dtype=src.dtype, device="cuda")
    ctx.ecospa_compact_batch([ctx.map_item(src, dst, idx, 0, groups, n, unit, kp, dst_t=dst_t_buf[:, :slots])])
    np.testing.assert_array_equal(host(dst), want)
    np.testing.assert_array_equal(host(dst_t_buf[:, :slots]), want.T)
    assert bool((dst_t_buf[:, slots:] == 7.0).all())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,k,kp,other,with_t", [(1024, 512, 512, 256, True), (5461, 2730, 2736, 520, True),
                                                 (37, 18, 32, 8, True), (37, 18, 32, 9, True), (200, 77, 80, 136, False)])
def test_row_gather_of_two_interleaved_sources(ctx, n, k, kp, other, with_t, dtype):
    """(gate, up) row pairs of a gated FFN's first matrix out of W_gate and W_up in one copy."""
    sc = np.abs(synth.normal(19, 401, (1, n))).astype(np.float32)
    idx_np = O.select_topk(sc, k)
    idx = torch.from_numpy(idx_np).cuda()
    a_np = synth.round_to(synth.normal(19, 402, (n, other)), dtype)
    b_np = synth.round_to(synth.normal(19, 403, (n, other)), dtype)
    a, b = dev(a_np, dtype), dev(b_np, dtype)
    want = interleave_rows(pad_rows(O.compact(a_np, idx_np, 0, n, 1), 1, k, kp), pad_rows(O.compact(b_np, idx_np, 0, n, 1), 1, k, kp))
    dst = torch.full((2 * kp, other), 7.0, dtype=a.dtype, device="cuda")
    dst_t = torch.full((other, 2 * kp), 7.0, dtype=a.dtype, device="cuda") if with_t else None
    ctx.ecospa_compact_batch([ctx.map_item(a, dst, idx, 0, 1, n, 1, kp, dst_t=dst_t, src_b=b)])
    np.testing.assert_array_equal(host(dst), want)
    if with_t:
        np.testing.assert_array_equal(host(dst_t), want.T)


def test_row_gather_with_transposed_copy_ragged_counts_and_shared_lists(ctx):
    """Per-group kept counts from device memory and heads that share an index list (Eq. 5), transposed copy included."""
    groups, n, kp, other, div = 8, 64, 32, 200, 2
    rng = np.random.default_rng(5)
    kg = rng.integers(0, kp + 1, size=groups // div).astype(np.int32)
    idx_np = np.full((groups // div, n), -1, dtype=np.int32)
    for g in range(groups // div):
        idx_np[g, :kg[g]] = np.sort(rng.choice(n, size=kg[g], replace=False))
    src_np = synth.round_to(synth.normal(21, 1, (groups * n, other)), "bf16")
    want = np.zeros((groups * kp, other))
    for g in range(groups):
        rows = idx_np[g // div, :kg[g // div]]
        want[g * kp:g * kp + len(rows)] = src_np[g * n + rows]
    src = dev(src_np, "bf16")
    dst = torch.empty((groups * kp, other), dtype=torch.bfloat16, device="cuda")
    dst_t = torch.empty((other, groups * kp), dtype=torch.bfloat16, device="cuda")
    ctx.ecospa_compact_batch([ctx.map_item(src, dst, torch.from_numpy(idx_np).cuda(), 0, groups, n, 1, kp,
                                           k_group=torch.from_numpy(kg).cuda(), idx_div=div, dst_t=dst_t)])
    np.testing.assert_array_equal(host(dst), want)
    np.testing.assert_array_equal(host(dst_t), want.T)


def test_transposed_copy_only_with_row_gathers(ctx):
    src = torch.zeros((64, 16), device="cuda")
    idx = torch.arange(8, dtype=torch.int32, device="cuda").view(1, 8)
    dst_t = torch.zeros((64, 8), device="cuda")
    for axis, scatter in ((1, 0), (0, 1)):
        dst = torch.zeros((64, 8) if axis == 1 else (64, 16), device="cuda")
        item = ctx.map_item(dst if scatter else src, src if scatter else dst, idx, axis, 1, 64 if scatter or axis == 0 else 16, 1, 8,
                            scatter=scatter, dst_t=dst_t)
        with pytest.raises(B.EcospaError) as e:
            ctx.ecospa_compact_batch([item])
        assert e.value.code == B.ERR_SHAPE


# ---- the rotary tables of the kept blocks from the gather launch itself ----------------------------------------------
@pytest.mark.parametrize("ragged", [False, True])
def test_gather_launch_fills_the_rotary_tables(ctx, ragged):
    """ecospa_compact_batch with a table descriptor: the same gathers, and tables bit-identical to those of the launch
    of their own (whose values are checked against the oracle's angles in the attention tests)."""
    h, dh, L, d, k, kp = 6, 64, 77, 40, 11, 16
    rng = np.random.default_rng(17)
    idx_np = np.stack([np.sort(rng.choice(dh // 2, size=k, replace=False)) for _ in range(h)]).astype(np.int32)
    idx = torch.from_numpy(idx_np).cuda()
    src_np = synth.round_to(synth.normal(23, 1, (h * dh, d)), "bf16")
    src = dev(src_np, "bf16")
    dst = torch.empty((h * 2 * kp, d), dtype=torch.bfloat16, device="cuda")
    kg = None
    if ragged:
        kg = torch.from_numpy(rng.integers(0, k + 1, size=h).astype(np.int32)).cuda()
        want_cos, want_sin = ctx.ecospa_rope_table_ragged(idx, kg, L, kp, dh)
    else:
        want_cos, want_sin = ctx.ecospa_rope_table(idx, h, L, k, kp, dh)
    cos = torch.full((h, L, kp), 7.0, device="cuda")
    sin = torch.full((h, L, kp), 7.0, device="cuda")
    item = ctx.map_item(src, dst, idx, 0, h, dh, 2, kp, k_group=kg)
    ctx.ecospa_compact_batch([item], ctx.rope_item(idx, h, L, k, kp, dh, 10000.0, cos, sin, k_group=kg))
    assert torch.equal(cos, want_cos) and torch.equal(sin, want_sin)
    ref = torch.empty_like(dst)
    ctx.ecospa_compact_batch([ctx.map_item(src, ref, idx, 0, h, dh, 2, kp, k_group=kg)])
    assert torch.equal(dst, ref)
    if not ragged:
        want = pad_rows(O.compact(src_np, idx_np, 0, dh, 2), h, 2 * k, 2 * kp)
        np.testing.assert_array_equal(host(dst), want)
    # a bad table descriptor is refused before anything is launched
    dst.fill_(3.0)
    with pytest.raises(B.EcospaError) as e:
        ctx.ecospa_compact_batch([item], ctx.rope_item(idx, h, L, k, kp, 1, 10000.0, cos, sin, k_group=kg))
    assert e.value.code == B.ERR_SHAPE
    assert bool((dst == 3.0).all())
