"""The entry point that allocates nothing (ecospa_coupled_score_static: partial sums in a fixed array inside the
library's device image) against the entry point it is a variant of (ecospa_coupled_score, partial sums in the caller's
workspace), through the C ABI: two calls in a row, the second with a smaller input, and the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd import synth
from util import assert_close, dev

pytestmark = pytest.mark.gpu


def _layer_pairs(seed, d, h, dh, dff, gated, unit, dtype):
    a = synth.attn_layer(seed, 1, 2, d, h, dh, dtype=dtype, structure="pretrained", bias=False)
    f = synth.ffn_layer(seed + 1, 2, d, dff, gated=gated, dtype=dtype, structure="pretrained", bias=False)
    g = {k: dev(v, dtype) for k, v in a.items()}
    gf = {k: dev(v, dtype) for k, v in f.items()}
    mk = B.Context.make_pair
    pairs = [mk(B.PAIR_QK, g["wq"], g["wk"], h, dh, unit), mk(B.PAIR_VO, g["wv"], g["wo"], h, dh, 1),
             mk(B.PAIR_FFN_GATED if gated else B.PAIR_FFN, gf["w1"], gf["w2"], 1, dff, 1, gf.get("w1b"))]
    want = [O.coupled_score(O.PAIR_QK, a["wq"], a["wk"], h, dh, unit), O.coupled_score(O.PAIR_VO, a["wv"], a["wo"], h, dh),
            O.coupled_score(O.PAIR_FFN_GATED if gated else O.PAIR_FFN, f["w1"], f["w2"], 1, dff, w1b=f.get("w1b"))]
    return pairs, want, (g, gf)


def test_static_scratch_score_equals_workspace_score_on_two_calls_in_a_row():
    ctx = B.Context("cuda:0")
    # first call: a LLaMA-1B-shaped layer's three pairs; second call, right behind it on the same stream: a much smaller
    # layer, whose partial sums overwrite the beginning of what the first call left in the fixed array
    for seed, (d, h, dh, dff, gated, unit, dtype) in ((70, (2048, 32, 64, 5461, True, 2, "bf16")), (72, (192, 3, 64, 200, False, 1, "f32"))):
        pairs, want, keep = _layer_pairs(seed, d, h, dh, dff, gated, unit, dtype)
        ref = ctx.ecospa_coupled_score(pairs)
        out = [torch.full_like(r, float("nan")) for r in ref]
        before = torch.cuda.memory_allocated()
        ctx.ecospa_coupled_score_static(pairs, out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        for got, r, w, nm in zip(out, ref, want, ("qk", "vo", "ffn")):
            assert torch.equal(got, r), f"{nm}: differs from the workspace entry point"      # same kernels, same order of sums
            assert_close(got, w, "f32", nm)
            assert abs(float(got.double().pow(2).sum(dim=1).sqrt()[0]) - 1.0) < 1e-5


def test_static_scratch_limit_and_validation():
    ctx = B.Context("cuda:0")
    lib = ctx.lib
    limit = lib.ecospa_coupled_score_static_max_bytes()
    assert limit == 2 << 20
    w1 = torch.zeros((300000, 8), device="cuda")
    w2 = torch.zeros((8, 300000), device="cuda")
    big = (B.Pair * 1)(B.Context.make_pair(B.PAIR_FFN, w1, w2, 1, 300000, 1))
    assert lib.ecospa_score_workspace_bytes(big, 1) > limit
    out = torch.full((1, 300000), 7.0, device="cuda")
    ptrs = (C.c_void_p * 1)(out.data_ptr())
    assert lib.ecospa_coupled_score_static(ctx.h, big, 1, ptrs) == B.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                       # nothing was launched
    assert lib.ecospa_coupled_score_static(ctx.h, big, 0, ptrs) == B.ERR_SHAPE
    assert lib.ecospa_coupled_score_static(ctx.h, None, 1, ptrs) == B.ERR_NULL
