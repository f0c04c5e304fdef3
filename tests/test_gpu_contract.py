"""GPU parity of the dense contraction kernels (every workgroup tile and LDS layout variant, all
operand layouts, ragged extents, split K) against a plain fp64 matrix product."""
import numpy as np
import pytest
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd import synth
from util import assert_close, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return B.Context("cuda:0")


def _operands(seed, M, N, K, ta, tb, dtype):
    a = synth.round_to(synth.normal(seed, 300, (K, M) if ta else (M, K)), dtype)
    b = synth.round_to(synth.normal(seed, 301, (K, N) if tb else (N, K)), dtype)
    bias = synth.round_to(synth.normal(seed, 302, (N,)), dtype)
    am = a.T if ta else a
    bm = b.T if tb else b
    want = am.astype(np.float64) @ bm.astype(np.float64).T + bias.astype(np.float64)
    return a, b, bias, want


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, True), (True, False)])
@pytest.mark.parametrize("M,N,K", [(300, 264, 136), (512, 512, 256), (1000, 520, 72), (64, 1032, 648)])
def test_contract_bf16(ctx, M, N, K, ta, tb, tile):
    if ta:
        M = (M + 7) // 8 * 8
    a, b, bias, want = _operands(41, M, N, K, ta, tb, "bf16")
    got = ctx.ecospa_contract(dev(a, "bf16"), ta, dev(b, "bf16"), tb, dev(bias, "bf16"), tile=tile, splits=1)
    assert_close(got, want, "bf16", f"tile {tile}")


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
@pytest.mark.parametrize("splits", [2, 5])
def test_contract_bf16_split_k(ctx, splits, tile):
    a, b, bias, want = _operands(42, 264, 136, 1000, True, True, "bf16")
    got = ctx.ecospa_contract(dev(a, "bf16"), True, dev(b, "bf16"), True, dev(bias, "bf16"), tile=tile, splits=splits)
    assert_close(got, want, "bf16", "split k")
    again = ctx.ecospa_contract(dev(a, "bf16"), True, dev(b, "bf16"), True, dev(bias, "bf16"), tile=tile, splits=splits)
    assert torch.equal(got, again)


@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, True)])
def test_contract_f32(ctx, ta, tb):
    a, b, bias, want = _operands(43, 201, 77, 130, ta, tb, "f32")
    got = ctx.ecospa_contract(dev(a), ta, dev(b), tb, dev(bias), splits=1)
    assert_close(got, want, "f32", "fp32")
    got = ctx.ecospa_contract(dev(a), ta, dev(b), tb, dev(bias), splits=3)
    assert_close(got, want, "f32", "fp32 split")


def test_contract_model_shapes_auto_tile(ctx):
    """Projection and FFN shapes of the GPT-2-Medium layer at 50% keep, library's own tile choice."""
    for (M, N, K, ta, tb) in [(2048, 1536, 1024, False, False), (2048, 1024, 2048, False, True), (1024, 2048, 2048, True, True)]:
        a, b, bias, want = _operands(44, M, N, K, ta, tb, "bf16")
        got = ctx.ecospa_contract(dev(a, "bf16"), ta, dev(b, "bf16"), tb, dev(bias, "bf16"))
        assert_close(got, want, "bf16", f"{M}x{N}x{K}")


@pytest.mark.parametrize("M,N,K,ta,tb", [(5504, 2048, 8192, True, True),      # gate|up weight gradient of the LLaMA-1B-shaped FFN: register-prefetch kernel
                                          (2048, 2752, 8192, True, True),      # W_down gradient: the same kernel, K split in two
                                          (8192, 1280, 1024, False, False),    # FFN kept at 3/10: 256x192 tiles
                                          (8192, 2048, 2752, False, False)])   # contraction over 2752 kept units (43 whole slabs)
def test_contract_stack_shapes_sampled(ctx, M, N, K, ta, tb):
    """Full-size contractions of the multi-layer workloads through the library's own choice of kernel, tile and
    split, checked on a sampled 96 x 96 block of outputs computed in fp64 from the same bf16 operands."""
    a = synth.round_to(synth.normal(49, 310, (K, M) if ta else (M, K)), "bf16")
    b = synth.round_to(synth.normal(49, 311, (K, N) if tb else (N, K)), "bf16")
    got = ctx.ecospa_contract(dev(a, "bf16"), ta, dev(b, "bf16"), tb)
    rng = np.random.default_rng(M + N)
    ms = np.sort(np.concatenate([rng.choice(M, 92, replace=False), [0, M - 1, M // 256 * 256 - 1, min(M - 1, M // 256 * 256)]]))
    ns = np.sort(np.concatenate([rng.choice(N, 92, replace=False), [0, N - 1, N // 256 * 256 - 1, min(N - 1, N // 256 * 256)]]))
    am = (a[:, ms].T if ta else a[ms]).astype(np.float64)
    bm = (b[:, ns].T if tb else b[ns]).astype(np.float64)
    want = am @ bm.T
    block = host(got[torch.from_numpy(ms).cuda()][:, torch.from_numpy(ns).cuda()])
    assert O.rel_fro(block, want) <= 2e-2
    assert np.abs(block - want).max() <= 2e-2 * np.abs(want).max() + 1e-6


def test_contract_launch_profile_counts_flops_and_time(ctx):
    """The per-launch event profile the benchmark's roofline figure comes from: launches counted, 2MNK flops each,
    a positive device time; nothing is recorded while it is switched off."""
    a, b, bias, _ = _operands(50, 512, 256, 128, False, False, "bf16")
    ga, gb = dev(a, "bf16"), dev(b, "bf16")
    ctx.ecospa_profile_gemm(True)
    for _ in range(3):
        ctx.ecospa_contract(ga, False, gb, False, splits=1)
    n, ms, flop = ctx.ecospa_profile_gemm_read()
    assert n == 3 and flop == 3 * 2.0 * 512 * 256 * 128 and 0.0 < ms < 50.0
    ctx.ecospa_profile_gemm(False)
    ctx.ecospa_contract(ga, False, gb, False, splits=1)
    ctx.ecospa_profile_gemm(True)
    n, ms, flop = ctx.ecospa_profile_gemm_read()
    assert n == 0 and flop == 0.0
    ctx.ecospa_profile_gemm(False)


def test_contract_alignment_errors(ctx):
    a = torch.zeros((64, 72), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((60, 72), dtype=torch.bfloat16, device="cuda")     # N = 60 is not a multiple of 8
    with pytest.raises(B.EcospaError) as e:
        ctx.ecospa_contract(a, False, b, False, splits=1)
    assert e.value.code == B.ERR_ALIGN


@pytest.mark.parametrize("cfg", range(11))
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, True)])
@pytest.mark.parametrize("M,N,K", [(520, 264, 192), (256, 512, 64), (304, 136, 512)])
def test_contract_bf16_pipelined_tiles(ctx, M, N, K, ta, tb, cfg):
    """Every configuration of the software-pipelined kernel (tile = 10 + cfg): ragged M and N, one slab
    (shorter than the LDS ring), a few slabs (ring wrap-around) and many."""
    a, b, bias, want = _operands(45, M, N, K, ta, tb, "bf16")
    got = ctx.ecospa_contract(dev(a, "bf16"), ta, dev(b, "bf16"), tb, dev(bias, "bf16"), tile=21 if cfg == 10 else 10 + cfg, splits=1)
    assert_close(got, want, "bf16", f"pipelined cfg {cfg}")


@pytest.mark.parametrize("cfg", [0, 1, 2, 4])
def test_contract_bf16_pipelined_split_k(ctx, cfg):
    a, b, bias, want = _operands(46, 264, 520, 1024, True, True, "bf16")
    got = ctx.ecospa_contract(dev(a, "bf16"), True, dev(b, "bf16"), True, dev(bias, "bf16"), tile=10 + cfg, splits=4)
    assert_close(got, want, "bf16", "split k")
    again = ctx.ecospa_contract(dev(a, "bf16"), True, dev(b, "bf16"), True, dev(bias, "bf16"), tile=10 + cfg, splits=4)
    assert torch.equal(got, again)


@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, True)])
@pytest.mark.parametrize("M,N,K", [(520, 264, 192), (256, 512, 64), (304, 136, 512), (1000, 520, 128)])
def test_contract_bf16_register_staged_prefetch(ctx, M, N, K, ta, tb):
    """The two-slab register-prefetch kernel (tile = 20): ragged M and N, one slab, two, three (odd count:
    the unrolled slab pair plus a tail) and many; x W^T, dY W and dY^T X operand forms."""
    a, b, bias, want = _operands(47, M, N, K, ta, tb, "bf16")
    got = ctx.ecospa_contract(dev(a, "bf16"), ta, dev(b, "bf16"), tb, dev(bias, "bf16"), tile=20, splits=1)
    assert_close(got, want, "bf16", "register-staged prefetch")
    if ta:      # split along K: fp32 partial sums added in a fixed order
        got = ctx.ecospa_contract(dev(a, "bf16"), ta, dev(b, "bf16"), tb, dev(bias, "bf16"), tile=20, splits=2 if K >= 128 else 1)
        assert_close(got, want, "bf16", "register-staged prefetch, split")


def test_contract_bf16_register_staged_prefetch_split_k(ctx):
    a, b, bias, want = _operands(48, 264, 520, 1024, False, True, "bf16")
    got = ctx.ecospa_contract(dev(a, "bf16"), False, dev(b, "bf16"), True, dev(bias, "bf16"), tile=20, splits=4)
    assert_close(got, want, "bf16", "split k")


RS_SHAPES = [(256, 256), (192, 256), (256, 192), (128, 256), (256, 128), (192, 192), (128, 192), (192, 128), (128, 128)]


@pytest.mark.parametrize("shape", range(9), ids=[f"{a}x{b}" for a, b in RS_SHAPES])
@pytest.mark.parametrize("M,N,K,splits", [(520, 264, 192, 1),      # ragged M and N, three slabs (slab pair + tail)
                                           (256, 512, 64, 1),       # one slab
                                           (304, 136, 128, 1),      # two slabs
                                           (1000, 776, 640, 1),     # several tiles on both axes, ten slabs
                                           (392, 648, 320, 3),      # five slabs split 2 + 2 + 1
                                           (200, 1048, 1024, 4)])
def test_contract_bf16_weight_gradient_tile_shapes(ctx, M, N, K, splits, shape):
    """dY^T X (both operands K-slow) on every tile shape of the register-prefetch kernel (tile = 30 + shape), with the
    column sums of the A operand that the backward passes take from the same launch (the bias gradient)."""
    a, b, _, _ = _operands(51, M, N, K, True, True, "bf16")
    want = a.astype(np.float64).T @ b.astype(np.float64)
    got, cs = ctx.ecospa_contract_colsum(dev(a, "bf16"), dev(b, "bf16"), tile=30 + shape, splits=splits)
    assert_close(got, want, "bf16", f"{RS_SHAPES[shape]} x{splits}")
    assert_close(cs, a.astype(np.float64).sum(axis=0), "f32", "column sums of A")
    again, cs2 = ctx.ecospa_contract_colsum(dev(a, "bf16"), dev(b, "bf16"), tile=30 + shape, splits=splits)
    assert torch.equal(got, again) and torch.equal(cs, cs2)


@pytest.mark.parametrize("M,N,K", [(1024, 2048, 8192), (1536, 1024, 8192), (5504, 2048, 4096), (2048, 2752, 4096), (3072, 2048, 4096),
                                   (2048, 1024, 4096), (4096, 1024, 8192), (520, 264, 1088)])
def test_contract_weight_gradient_own_plan(ctx, M, N, K):
    """The layers' weight-gradient shapes through the library's own choice of tile shape and K split: sampled outputs in
    fp64 from the same operands, and the fused column sums of A."""
    a = synth.round_to(synth.normal(52, 320, (K, M)), "bf16")
    b = synth.round_to(synth.normal(52, 321, (K, N)), "bf16")
    got, cs = ctx.ecospa_contract_colsum(dev(a, "bf16"), dev(b, "bf16"))
    rng = np.random.default_rng(M * 7 + N)
    edge = lambda n: [0, n - 1, n // 256 * 256 - 1, min(n - 1, n // 256 * 256), n // 192 * 192 - 1, min(n - 1, n // 192 * 192)]
    ms = np.unique(np.concatenate([rng.choice(M, 90, replace=False), edge(M)]))
    ns = np.unique(np.concatenate([rng.choice(N, 90, replace=False), edge(N)]))
    want = a[:, ms].astype(np.float64).T @ b[:, ns].astype(np.float64)
    block = host(got[torch.from_numpy(ms).cuda()][:, torch.from_numpy(ns).cuda()])
    assert_close(block, want, "bf16", "sampled block")
    assert_close(cs, a.astype(np.float64).sum(axis=0), "f32", "column sums of A")
