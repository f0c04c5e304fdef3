"""The layer glue of the library (normalisation with the residual addition in front, embedding lookup and its gradient,
mean cross-entropy) against the fp64 glue oracle, on inputs rounded to bf16: ragged row counts, widths from one chunk
per lane to the widest supported, vocabularies with a ragged tail and at the size of the stack workloads."""
import numpy as np
import pytest
import torch

from oracle import glue_oracle as G
from paper_2511_11641_amd import binding as B
from util import assert_close, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def bf(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).cuda()


def each_element_rounded(got, want, what):
    """For tensors with a few entries far above the rest (a token that occurs a thousand times, the target's entry of a
    softmax gradient) a bound relative to the tensor's RMS says little: every element to bf16 rounding of its own size
    (half a unit in the last place = 2^-9; fp32 sums in between: 2^-8 leaves room for them)."""
    g, w = host(got), np.asarray(want, dtype=np.float64)
    bad = np.abs(g - w) > 2.0 ** -8 * np.abs(w) + 1e-12
    assert not bad.any(), f"{what}: {int(bad.sum())} elements off, worst {np.abs(g - w).max():.3e} at {np.unravel_index(np.abs(g - w).argmax(), w.shape)}"


@pytest.mark.parametrize("kind", ["rms", "layer"])
@pytest.mark.parametrize("T,d", [(5, 8), (77, 128), (300, 1000), (1500, 2048), (66, 4096), (2051, 1024)])
@pytest.mark.parametrize("with_res", [False, True])
def test_norm_forward_backward(ctx, kind, T, d, with_res):
    rng = np.random.default_rng(T * 7 + d)
    layer = kind == "layer"
    x, res, dy, dres = (bf(rng.standard_normal((T, d)) * s) for s in (1.0, 0.5, 1.0, 0.7))
    x = x + 0.75 if layer else x                     # a mean worth subtracting
    gain, bias = bf(1.0 + 0.2 * rng.standard_normal(d)), bf(0.1 * rng.standard_normal(d))
    eps = 1e-5 if layer else 1e-6
    code = B.NORM_LAYER if layer else B.NORM_RMS
    y, x_out, dx = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    stat = torch.empty((T, 2) if layer else (T,), dtype=torch.float32, device="cuda")
    dgain, dbias = torch.empty_like(gain), torch.empty_like(gain)
    ctx.ecospa_norm_fwd(code, x, gain, bias if layer else None, eps, y, res=res if with_res else None,
                        x_out=x_out if with_res else None, stat=stat)
    s_in = x_out if with_res else x
    ctx.ecospa_norm_bwd(code, s_in, gain, stat, dy, dx, dgain, dbias=dbias if layer else None, dres=dres if with_res else None)
    torch.cuda.synchronize()
    # the oracle sees the stream as the library stores it: the sum rounded to bf16
    xs = host(x) + host(res) if with_res else host(x)
    if with_res:
        assert_close(x_out, xs, "bf16", "x + res")
        xs = host(x_out)
    if layer:
        want_y, st = G.ln_fwd(xs, host(gain), host(bias), eps)
        want_dx, want_dg, want_db = G.ln_bwd(host(gain), st, host(dy))
        assert_close(stat[:, 0], xs.mean(axis=1), "f32", "row means")
        assert_close(stat[:, 1], st[1][:, 0], "f32", "row reciprocal deviations")
    else:
        want_y, r = G.rms_fwd(xs, host(gain), eps)
        want_dx, want_dg, want_db = G.rms_bwd(xs, host(gain), r, host(dy))
        assert_close(stat, r[:, 0], "f32", "row reciprocal roots")
    if with_res:
        want_dx = want_dx + host(dres)
    assert_close(y, want_y, "bf16", "y")
    assert_close(dx, want_dx, "bf16", "dx")
    assert_close(dgain, want_dg, "bf16", "dgain")
    if layer:
        assert_close(dbias, want_db, "bf16", "dbias")
    # in place on the stream and its gradient, and bit for bit the same as out of place
    if with_res:
        x2, d2 = x.clone(), dres.clone()
        y2 = torch.empty_like(x)
        ctx.ecospa_norm_fwd(code, x2, gain, bias if layer else None, eps, y2, res=res, x_out=x2, stat=stat)
        ctx.ecospa_norm_bwd(code, x2, gain, stat, dy, d2, dgain, dbias=dbias if layer else None, dres=d2)
        assert torch.equal(x2, x_out) and torch.equal(y2, y) and torch.equal(d2, dx)


def test_norm_without_statistics_is_the_same_forward(ctx):
    rng = np.random.default_rng(0)
    x, g = bf(rng.standard_normal((33, 256))), bf(rng.standard_normal(256))
    a, b = torch.empty_like(x), torch.empty_like(x)
    st = torch.empty(33, dtype=torch.float32, device="cuda")
    ctx.ecospa_norm_fwd(B.NORM_RMS, x, g, None, 1e-6, a, stat=st)
    ctx.ecospa_norm_fwd(B.NORM_RMS, x, g, None, 1e-6, b)
    assert torch.equal(a, b)


@pytest.mark.parametrize("T,L,d,V", [(12, 4, 8, 7), (96, 32, 136, 50), (4096, 256, 2048, 32000), (1024, 1024, 4096, 300)])
def test_embedding_lookup_and_gradient(ctx, T, L, d, V):
    rng = np.random.default_rng(T + V)
    ids_np = rng.integers(0, V, T)
    ids_np[: T // 3] = ids_np[0]                          # one token many times: a long sum in position order
    ids = torch.from_numpy(ids_np).cuda()
    table, pos, dx = bf(rng.standard_normal((V, d))), bf(rng.standard_normal((L, d))), bf(rng.standard_normal((T, d)))
    out = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    ctx.ecospa_embed_fwd(ids, table, out)
    assert torch.equal(out, table[ids])                    # a copy of rows: exact
    ctx.ecospa_embed_fwd(ids, table, out, pos=pos)
    assert_close(out, G.embed_fwd(ids_np, host(table), host(pos), L), "bf16", "lookup + position")
    dtable = torch.full((V, d), 7.0, dtype=torch.bfloat16, device="cuda")       # stale contents must go
    dpos = torch.empty((L, d), dtype=torch.bfloat16, device="cuda")
    ctx.ecospa_embed_bwd(ids, dx, dtable, dpos=dpos)
    want_t, want_p = G.embed_bwd(ids_np, host(dx), V, L)
    each_element_rounded(dtable, want_t, "table gradient")
    each_element_rounded(dpos, want_p, "position gradient")
    unused = np.setdiff1d(np.arange(V), ids_np)
    assert not dtable[torch.from_numpy(unused).cuda()].any()
    again = torch.empty_like(dtable)
    ctx.ecospa_embed_bwd(ids, dx, again)
    assert torch.equal(again, dtable)                      # fixed order of every sum


def test_embedding_ids_outside_the_table(ctx):
    V, d = 10, 16
    ids = torch.tensor([3, -1, 10, 3, 9], device="cuda")
    table = bf(np.arange(V * d).reshape(V, d) % 13)
    out = torch.empty((5, d), dtype=torch.bfloat16, device="cuda")
    ctx.ecospa_embed_fwd(ids, table, out)
    assert torch.equal(out[0], table[3]) and not out[1].any() and not out[2].any() and torch.equal(out[4], table[9])
    dx = bf(np.ones((5, d)))
    dtable = torch.empty((V, d), dtype=torch.bfloat16, device="cuda")
    ctx.ecospa_embed_bwd(ids, dx, dtable)
    assert float(dtable[3, 0]) == 2.0 and float(dtable[9, 0]) == 1.0 and float(dtable.float().sum()) == 3.0 * d


@pytest.mark.parametrize("T,V,ld", [(7, 8, 8), (37, 320, 320), (50, 1003, 1008), (19, 32000, 32000), (5, 65536, 65536), (300, 5000, 5120)])
def test_cross_entropy(ctx, T, V, ld):
    rng = np.random.default_rng(V)
    full = bf(rng.standard_normal((T, ld)) * 4.0)
    logits = full[:, :V]
    tgt_np = rng.integers(0, V, T)
    tgt_np[0], tgt_np[-1] = V - 1, 0
    tgt = torch.from_numpy(tgt_np).cuda()
    rows, loss = torch.empty(T, dtype=torch.float32, device="cuda"), torch.zeros((), dtype=torch.float32, device="cuda")
    dfull = torch.zeros_like(full)
    ctx.ecospa_xent(logits, tgt, rows, loss, dlogits=dfull[:, :V])
    want_loss, want_rows, want_dl = G.xent(host(logits), tgt_np)
    assert_close(rows, want_rows, "f32", "row losses")
    assert abs(float(loss) - want_loss) <= 1e-5 * abs(want_loss)
    each_element_rounded(dfull[:, :V], want_dl, "dlogits")
    assert not dfull[:, V:].any()                          # the padding of the rows is not written
    # loss only; and in place on the logits, bit for bit the same
    loss2 = torch.zeros_like(loss)
    ctx.ecospa_xent(logits, tgt, rows, loss2)
    assert torch.equal(loss2, loss)
    inplace = full.clone()
    ctx.ecospa_xent(inplace[:, :V], tgt, rows, loss2, dlogits=inplace[:, :V])
    assert torch.equal(inplace[:, :V], dfull[:, :V]) and torch.equal(loss2, loss)


def test_cross_entropy_target_outside_the_vocabulary(ctx):
    rng = np.random.default_rng(5)
    T, V = 6, 64
    logits = bf(rng.standard_normal((T, V)))
    tgt_np = rng.integers(0, V, T)
    tgt = torch.from_numpy(tgt_np).cuda()
    tgt[2] = -100
    rows, loss = torch.empty(T, dtype=torch.float32, device="cuda"), torch.zeros((), dtype=torch.float32, device="cuda")
    dl = torch.empty_like(logits)
    ctx.ecospa_xent(logits, tgt, rows, loss, dlogits=dl)
    _, want_rows, want_dl = G.xent(host(logits), np.where(tgt_np < 0, 0, tgt_np))
    want_rows[2] = 0.0
    want_dl[2] = 0.0
    assert float(rows[2]) == 0.0 and not dl[2].any()
    assert_close(rows, want_rows, "f32", "row losses")
    assert abs(float(loss) - want_rows.mean()) <= 1e-5 * want_rows.mean()
    each_element_rounded(dl, want_dl, "dlogits")
