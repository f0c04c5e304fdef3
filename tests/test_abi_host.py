"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and validates arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2511_11641_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load()


@pytest.fixture()
def ctx(lib):
    h = C.c_void_p()
    assert lib.ecospa_create(C.byref(h), None) == B.OK
    yield h
    lib.ecospa_destroy(h)


def test_every_declared_symbol_is_exported(lib):
    text = open(os.path.join(ROOT, "include", "ecospa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ecospa_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    for code in range(9):
        assert lib.ecospa_status_string(code)
    assert b"unknown" in lib.ecospa_status_string(99)


def test_select_validation(lib, ctx):
    f = lib.ecospa_select_topk
    assert f(ctx, 256, 1, 8, 0, 256) == B.ERR_K
    assert f(ctx, 256, 1, 8, 9, 256) == B.ERR_K
    assert f(ctx, 256, 0, 8, 1, 256) == B.ERR_SHAPE
    assert f(ctx, None, 1, 8, 1, 256) == B.ERR_NULL
    assert f(None, 256, 1, 8, 1, 256) == B.ERR_NULL


def test_compact_validation(lib, ctx):
    for f in (lib.ecospa_compact, lib.ecospa_scatter):
        ok = dict(src=256, dst=512, dtype=B.F32, axis=0, groups=2, n=8, unit=1, k=4, kp=4, other=16, ls=16, ld=16, idx=768)

        def call(**kw):
            a = dict(ok, **kw)
            return f(ctx, a["src"], a["dst"], a["dtype"], a["axis"], a["groups"], a["n"], a["unit"], a["k"], a["kp"],
                     a["other"], a["ls"], a["ld"], a["idx"])

        assert call(src=None) == B.ERR_NULL
        assert call(idx=None) == B.ERR_NULL
        assert call(dtype=7) == B.ERR_DTYPE
        assert call(axis=2) == B.ERR_SHAPE
        assert call(unit=3) == B.ERR_SHAPE          # n % unit
        assert call(k=0) == B.ERR_K
        assert call(k=9) == B.ERR_K
        assert call(kp=3) == B.ERR_K
        assert call(ls=8) == B.ERR_SHAPE
        assert call(axis=1, ls=8, ld=8) == B.ERR_SHAPE   # axis 1 needs ld >= slots


def test_map_item_validation(lib, ctx):
    """Batched gathers/scatters: every item is validated before anything is launched (the pointers are never touched)."""
    def item(**kw):
        a = dict(src=256, dst=512, dtype=B.F32, axis=0, groups=4, n=8, unit=1, k=4, kp=4, scatter=0, other=16, ls=16, ld=16,
                 idx=768, k_group=None, ld_idx=0, idx_div=0)
        a.update(kw)
        return B.MapItem(a["src"], a["dst"], a["dtype"], a["axis"], a["groups"], a["n"], a["unit"], a["k"], a["kp"], a["scatter"],
                         a["other"], a["ls"], a["ld"], a["idx"], a["k_group"], a["ld_idx"], a["idx_div"])

    def call(*items):
        arr = (B.MapItem * len(items))(*items)
        return lib.ecospa_compact_batch(ctx, arr, len(items))

    assert call(item(scatter=3)) == B.ERR_SHAPE              # 0 gather, 1 zero-filling scatter, 2 merging scatter
    assert call(item(scatter=-1)) == B.ERR_SHAPE
    assert call(item(), item(dst=None)) == B.ERR_NULL        # a bad item anywhere in the batch stops the whole call
    assert call(item(k_group=1024, kp=0, ld_idx=8)) == B.ERR_K       # ragged: capacities must be positive
    assert call(item(k_group=1024, kp=4, ld_idx=0)) == B.ERR_K
    assert call(item(idx_div=3)) == B.ERR_SHAPE              # heads per shared index list must divide the heads
    assert call(item(ld_idx=3)) == B.ERR_K                   # index lists closer together than k
    assert lib.ecospa_compact_batch(ctx, None, 1) == B.ERR_NULL
    arr = (B.MapItem * 1)(item())
    assert lib.ecospa_compact_batch(ctx, arr, 0) == B.ERR_SHAPE


def test_score_validation(lib, ctx):
    p = B.Pair(B.PAIR_FFN, B.F32, 1, 8, 1, 4, 4, 256, None, 512, 4, 0, 8)
    arr = (B.Pair * 1)(p)
    out = (C.c_void_p * 1)(1024)
    assert lib.ecospa_score_workspace_bytes(arr, 1) > 0
    assert lib.ecospa_coupled_score(ctx, arr, 1, out) == B.ERR_WORKSPACE   # no workspace attached
    bad = B.Pair(B.PAIR_FFN_GATED, B.F32, 1, 8, 1, 4, 4, 256, None, 512, 4, 0, 8)
    assert lib.ecospa_coupled_score(ctx, (B.Pair * 1)(bad), 1, out) == B.ERR_NULL   # gated needs w1b
    bad = B.Pair(B.PAIR_FFN, B.F32, 1, 8, 3, 4, 4, 256, None, 512, 4, 0, 8)
    assert lib.ecospa_coupled_score(ctx, (B.Pair * 1)(bad), 1, out) == B.ERR_SHAPE  # n % unit
    bad = B.Pair(9, B.F32, 1, 8, 1, 4, 4, 256, None, 512, 4, 0, 8)
    assert lib.ecospa_coupled_score(ctx, (B.Pair * 1)(bad), 1, out) == B.ERR_DTYPE
    bad = B.Pair(B.PAIR_FFN, B.F32, 1, 8, 1, 4, 4, 256, None, 512, 4, 0, 7)
    assert lib.ecospa_coupled_score(ctx, (B.Pair * 1)(bad), 1, out) == B.ERR_SHAPE  # ld2 < groups*n
    assert lib.ecospa_score_workspace_bytes((B.Pair * 1)(bad), 1) == 0
    # second member stored with its units as rows: ld2 counts against d2 = 4, not against the 8 units
    rows = B.Pair(B.PAIR_FFN, B.F32, 1, 8, 1, 4, 4, 256, None, 512, 4, 0, 4, 0, 0, 1)
    assert lib.ecospa_coupled_score(ctx, (B.Pair * 1)(rows), 1, out) == B.ERR_WORKSPACE
    bad = B.Pair(B.PAIR_FFN, B.F32, 1, 8, 1, 4, 4, 256, None, 512, 4, 0, 3, 0, 0, 1)
    assert lib.ecospa_coupled_score(ctx, (B.Pair * 1)(bad), 1, out) == B.ERR_SHAPE
    # ... and needs no partial sums per row range: a smaller workspace than the column form
    assert lib.ecospa_score_workspace_bytes((B.Pair * 1)(rows), 1) <= lib.ecospa_score_workspace_bytes(arr, 1)


def test_block_validation(lib, ctx):
    d = B.BlockDesc()
    d.block, d.dtype, d.B, d.L, d.d_model = B.BLOCK_FFN, B.BF16, 2, 16, 64
    d.kp_ff, d.act, d.w_1, d.w_2, d.ld_w1, d.ld_w2 = 32, B.ACT_GELU_ERF, 256, 512, 64, 32
    need = lib.ecospa_block_workspace_bytes(C.byref(d))
    assert need > 0
    assert lib.ecospa_coupled_fwd(ctx, C.byref(d), 1024, 2048, None) == B.ERR_WORKSPACE
    d2 = B.BlockDesc.from_buffer_copy(d)
    d2.kp_ff = 30
    assert lib.ecospa_block_workspace_bytes(C.byref(d2)) == 0
    assert lib.ecospa_coupled_fwd(ctx, C.byref(d2), 1024, 2048, None) == B.ERR_SHAPE
    d2 = B.BlockDesc.from_buffer_copy(d)
    d2.act = 5
    assert lib.ecospa_coupled_fwd(ctx, C.byref(d2), 1024, 2048, None) == B.ERR_DTYPE
    d2 = B.BlockDesc.from_buffer_copy(d)
    d2.w_1 = None
    assert lib.ecospa_coupled_fwd(ctx, C.byref(d2), 1024, 2048, None) == B.ERR_NULL
    d2 = B.BlockDesc.from_buffer_copy(d)
    d2.ld_w1 = 60
    assert lib.ecospa_coupled_fwd(ctx, C.byref(d2), 1024, 2048, None) == B.ERR_SHAPE
    assert lib.ecospa_coupled_fwd(ctx, C.byref(d), 1028, 2048, None) == B.ERR_ALIGN
    a = B.BlockDesc()
    a.block, a.dtype, a.B, a.L, a.d_model = B.BLOCK_ATTN, B.BF16, 2, 16, 64
    a.h, a.kp_qk, a.kp_vo, a.scale, a.w_qkv, a.w_o, a.ld_wqkv, a.ld_wo = 2, 16, 24, 0.125, 256, 512, 64, 64
    assert lib.ecospa_coupled_fwd(ctx, C.byref(a), 1024, 2048, None) == B.ERR_SHAPE   # kp_vo % 16
    assert lib.ecospa_set_workspace(ctx, 257, 1024) == B.ERR_ALIGN


def test_attention_heads_wider_than_128_are_rejected_before_any_launch(lib, ctx):
    """The attention core is built for padded head widths up to 128: a wider head is a validation error of the
    descriptor itself (workspace query included), not something found after the projections have been launched."""
    a = B.BlockDesc()
    a.block, a.dtype, a.B, a.L, a.d_model = B.BLOCK_ATTN, B.BF16, 2, 16, 256
    a.h, a.kp_qk, a.kp_vo, a.scale, a.w_qkv, a.w_o, a.ld_wqkv, a.ld_wo = 2, 32, 32, 0.125, 256, 512, 256, 160
    assert lib.ecospa_block_workspace_bytes(C.byref(a)) > 0
    for kq, kv in ((144, 32), (32, 144), (256, 256), (160, 64)):
        b = B.BlockDesc.from_buffer_copy(a)
        b.kp_qk, b.kp_vo = kq, kv
        assert lib.ecospa_block_workspace_bytes(C.byref(b)) == 0
        # no workspace is attached and the data pointers are bogus: ERR_SHAPE must come first, from validation alone
        assert lib.ecospa_coupled_fwd(ctx, C.byref(b), 1024, 2048, None) == B.ERR_SHAPE
        sv, gr = B.Saved(4096, 8192, 12288, None, None), B.Grads()
        assert lib.ecospa_coupled_bwd(ctx, C.byref(b), 1024, 2048, C.byref(sv), 4096, C.byref(gr)) == B.ERR_SHAPE
    b = B.BlockDesc.from_buffer_copy(a)
    for kq, kv in ((64, 48), (80, 32), (96, 128), (128, 128)):
        b.kp_qk, b.kp_vo = kq, kv
        b.ld_wo = 2 * kv
        assert lib.ecospa_block_workspace_bytes(C.byref(b)) > 0


def test_check_indices_validation(lib, ctx):
    f = lib.ecospa_check_indices
    assert f(None, 256, 1, 8, 4, None, 8) == B.ERR_NULL
    assert f(ctx, None, 1, 8, 4, None, 8) == B.ERR_NULL
    assert f(ctx, 256, 0, 8, 4, None, 8) == B.ERR_SHAPE
    assert f(ctx, 256, 1, 0, 4, None, 8) == B.ERR_SHAPE
    assert f(ctx, 256, 1, 8, 0, None, 8) == B.ERR_K
    assert f(ctx, 256, 1, 8, 9, None, 16) == B.ERR_K          # more entries than the list holds
    assert f(ctx, 256, 1, 8, 8, None, 4) == B.ERR_K           # more entries than there are units
    assert f(ctx, 256, 1, 8, 4, None, 8) == B.ERR_WORKSPACE   # needs a flag word; nothing was launched


def test_contract_workspace_query(lib):
    q = lib.ecospa_contract_workspace_bytes
    assert q(B.BF16, 1024, 2048, 8192, 4) == 4 * 1024 * 2048 * 4
    assert q(B.BF16, 1024, 2048, 8192, 1) == 0
    own = q(B.BF16, 1024, 2048, 8192, 0)
    assert own % (1024 * 2048 * 4) == 0 and own <= 8 * 1024 * 2048 * 4
    # an output as large as a vocabulary projection: the library's own choice never reserves tens of gigabytes
    assert q(B.BF16, 8192, 32000, 2048, 0) <= 8 * 8192 * 32000 * 4
    assert q(7, 8, 8, 8, 0) == 0 and q(B.BF16, 0, 8, 8, 0) == 0 and q(B.BF16, 8, 8, 8, 65) == 0


def test_static_scratch_score_validates_before_touching_the_device(lib, ctx):
    """The entry point that allocates nothing: bad arguments and batches beyond its fixed scratch array are refused by
    host checks alone (no GPU is needed to get these answers)."""
    f = lib.ecospa_coupled_score_static
    assert lib.ecospa_coupled_score_static_max_bytes() == 2 << 20
    p = B.Pair(B.PAIR_FFN, B.F32, 1, 8, 1, 4, 4, 256, None, 512, 4, 0, 8)
    arr = (B.Pair * 1)(p)
    out = (C.c_void_p * 1)(1024)
    assert f(None, arr, 1, out) == B.ERR_NULL
    assert f(ctx, None, 1, out) == B.ERR_NULL
    assert f(ctx, arr, 0, out) == B.ERR_SHAPE
    assert f(ctx, arr, 1, (C.c_void_p * 1)(None)) == B.ERR_NULL
    bad = B.Pair(B.PAIR_FFN, B.F32, 1, 8, 3, 4, 4, 256, None, 512, 4, 0, 8)
    assert f(ctx, (B.Pair * 1)(bad), 1, out) == B.ERR_SHAPE
    big = B.Pair(B.PAIR_FFN, B.F32, 1, 300000, 1, 8, 8, 256, None, 512, 8, 0, 300000)
    assert lib.ecospa_score_workspace_bytes((B.Pair * 1)(big), 1) > lib.ecospa_coupled_score_static_max_bytes()
    assert f(ctx, (B.Pair * 1)(big), 1, out) == B.ERR_WORKSPACE


def test_glue_validation(lib, ctx):
    p = 4096      # any 16-byte aligned non-null value: nothing is launched on a validation error
    nf, nb = lib.ecospa_norm_fwd, lib.ecospa_norm_bwd
    assert nf(ctx, B.NORM_RMS, 4, 64, B.BF16, None, None, None, p, None, 1e-6, p, None) == B.ERR_NULL
    assert nf(ctx, B.NORM_RMS, 4, 64, B.BF16, p, p, None, p, None, 1e-6, p, None) == B.ERR_NULL       # res without x_out
    assert nf(ctx, B.NORM_RMS, 4, 64, B.F32, p, None, None, p, None, 1e-6, p, None) == B.ERR_DTYPE
    assert nf(ctx, 2, 4, 64, B.BF16, p, None, None, p, None, 1e-6, p, None) == B.ERR_SHAPE
    assert nf(ctx, B.NORM_RMS, 0, 64, B.BF16, p, None, None, p, None, 1e-6, p, None) == B.ERR_SHAPE
    assert nf(ctx, B.NORM_RMS, 4, 60, B.BF16, p, None, None, p, None, 1e-6, p, None) == B.ERR_SHAPE
    assert nf(ctx, B.NORM_RMS, 4, 4104, B.BF16, p, None, None, p, None, 1e-6, p, None) == B.ERR_SHAPE
    assert nf(ctx, B.NORM_RMS, 4, 64, B.BF16, p + 2, None, None, p, None, 1e-6, p, None) == B.ERR_ALIGN
    assert nb(ctx, B.NORM_LAYER, 4, 64, B.BF16, p, p, None, p, None, p, p, p) == B.ERR_NULL          # no statistics
    assert nb(ctx, B.NORM_LAYER, 4, 64, B.BF16, p, p, p, p, None, p, p, p) == B.ERR_WORKSPACE        # none attached
    assert lib.ecospa_norm_bwd_workspace_bytes(8192, 2048) >= 512 * 2 * 2048 * 4
    assert lib.ecospa_norm_bwd_workspace_bytes(0, 2048) == 0
    ef, eb = lib.ecospa_embed_fwd, lib.ecospa_embed_bwd
    assert ef(ctx, 8, 64, 100, B.BF16, None, p, None, 0, p) == B.ERR_NULL
    assert ef(ctx, 8, 64, 100, B.BF16, p, p, p, 3, p) == B.ERR_SHAPE                                  # 8 positions, table of 3
    assert ef(ctx, 8, 12, 100, B.BF16, p, p, None, 0, p) == B.ERR_SHAPE
    assert ef(ctx, 8, 64, 100, B.F32, p, p, None, 0, p) == B.ERR_DTYPE
    assert eb(ctx, 8, 8192, 100, B.BF16, p, p, p, None, 0) == B.ERR_SHAPE
    assert eb(ctx, 8, 64, 100, B.BF16, p, p + 8, p, None, 0) == B.ERR_ALIGN
    xe = lib.ecospa_xent
    assert xe(ctx, 4, 100, B.BF16, p, 104, p, None, 0, None, p) == B.ERR_NULL
    assert xe(ctx, 4, 100, B.BF16, p, 96, p, None, 0, p, p) == B.ERR_SHAPE                            # rows overlap
    assert xe(ctx, 4, 70000, B.BF16, p, 70000, p, None, 0, p, p) == B.ERR_SHAPE
    assert xe(ctx, 4, 100, B.BF16, p, 100, p, None, 0, p, p) == B.ERR_ALIGN                           # leading dimension % 8
    assert xe(ctx, 4, 100, B.F32, p, 104, p, None, 0, p, p) == B.ERR_DTYPE
