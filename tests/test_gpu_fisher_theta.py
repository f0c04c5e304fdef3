"""GPU parity (through the C ABI) of the pair-level importance (Eq. 8) and the cumulative-threshold
rule (Alg. 1) against the oracle: importances within the fp32 tolerance, kept counts and indices bit
for bit on identical scores."""
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


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("h,dh,d,dff,gated", [(16, 64, 1024, 4096, False), (32, 64, 2048, 5461, True), (3, 8, 24, 37, True),
                                               (2, 64, 136, 1073, False)])
def test_pair_fisher_layer(ctx, h, dh, d, dff, gated, dtype):
    """Gradient-shaped tensors of a whole layer (QK, VO and FFN pairs) in one batched call."""
    a = synth.attn_layer(21, 1, 2, d, h, dh, dtype=dtype, bias=False)       # stand-ins for dW_q, dW_k, dW_v, dW_o
    f = synth.ffn_layer(22, 2, d, dff, gated=gated, dtype=dtype, bias=False)   # dW_1 (, dW_up), dW_2
    D = 96.0
    kind = O.PAIR_FFN_GATED if gated else O.PAIR_FFN
    want = [O.pair_fisher(O.PAIR_QK, a["wq"], a["wk"], h, dh, D), O.pair_fisher(O.PAIR_VO, a["wv"], a["wo"], h, dh, D),
            O.pair_fisher(kind, f["w1"], f["w2"], 1, dff, D, g1b=f.get("w1b"))]
    g = {k: dev(v, dtype) for k, v in a.items()}
    gf = {k: dev(v, dtype) for k, v in f.items() if k in ("w1", "w2", "w1b")}
    mk = B.Context.make_pair
    got = ctx.ecospa_pair_fisher([mk(B.PAIR_QK, g["wq"], g["wk"], h, dh, 1), mk(B.PAIR_VO, g["wv"], g["wo"], h, dh, 1),
                                  mk(kind, gf["w1"], gf["w2"], 1, dff, 1, gf.get("w1b"))], D)
    for x, y, nm in zip(got, want, ("qk", "vo", "ffn")):
        assert x.shape == y.shape
        assert_close(x, y, "f32", f"fisher {nm}")


def test_pair_fisher_constant_gradient_and_errors(ctx):
    g1 = torch.full((128, 64), 0.5, device="cuda")
    g2 = torch.full((32, 128), 0.5, device="cuda")
    got = ctx.ecospa_pair_fisher([B.Context.make_pair(B.PAIR_VO, g1, g2, 2, 64, 1)], 8.0)[0]
    assert torch.allclose(got.cpu(), torch.full((2,), 0.25 / 8.0), rtol=1e-6)
    with pytest.raises(B.EcospaError) as e:
        ctx.ecospa_pair_fisher([B.Context.make_pair(B.PAIR_VO, g1, g2, 2, 64, 1)], 0.0)
    assert e.value.code == B.ERR_SHAPE


def _theta_case(ctx, s, theta):
    want_idx, want_k = O.select_theta(s, theta)
    idx, k = ctx.ecospa_select_theta(torch.from_numpy(s).cuda(), theta)
    assert np.array_equal(k.cpu().numpy(), want_k), f"theta {theta}: kept counts"
    assert np.array_equal(idx.cpu().numpy(), want_idx), f"theta {theta}: kept indices"
    return want_k


@pytest.mark.parametrize("groups,n", [(1, 4096), (16, 64), (32, 32), (3, 5461), (5, 37), (2, 1)])
@pytest.mark.parametrize("theta", [0.0, 0.3, 0.9, 0.99, 1.0])
def test_select_theta_on_scores_of_the_right_shape(ctx, groups, n, theta):
    """Rows normalised like Eq. 10 (unit l2 norm), spread like pre-trained weights."""
    rng = np.random.default_rng(groups * 1000 + n)
    r = np.exp(rng.normal(0, 0.7, (groups, n)))
    s = (r / np.linalg.norm(r, axis=1, keepdims=True)).astype(np.float32)
    _theta_case(ctx, s, theta)


def test_select_theta_ties_zeros_nan_and_out_of_range_values(ctx):
    rng = np.random.default_rng(7)
    s = (rng.integers(1, 9, (6, 300)) / 2048.0).astype(np.float32)      # few distinct values: ties everywhere
    s[1, ::3] = 0.0
    s[2, 5] = np.nan
    s[2, 9] = -0.0
    s[3, :] = 0.0                                                        # massless row: one unit stays
    s[4, 7] = 3.0                                                        # clipped to 1
    s[4, 8] = -2.0
    s[5, :] = s[5, 0]                                                    # one value only
    for theta in (0.0, 0.25, 0.5, 0.75, 0.999, 1.0):
        ks = _theta_case(ctx, s, theta)
        assert ks[3] == 1


def test_select_theta_feeds_compaction(ctx):
    """The kept indices of a row are valid input of the aligned gather (ascending, in range)."""
    rng = np.random.default_rng(9)
    n, d = 256, 64
    s = rng.random((1, n)).astype(np.float32)
    s /= np.linalg.norm(s)
    idx, k = ctx.ecospa_select_theta(torch.from_numpy(s).cuda(), 0.8)
    kk = int(k[0])
    w = synth.normal(9, 1, (n, d)).astype(np.float32)
    got = ctx.ecospa_compact(dev(w), idx[:, :kk].contiguous(), axis=0, groups=1, n=n, unit=1, kp=B.round_up(kk, 16))
    want = np.zeros((B.round_up(kk, 16), d))
    want[:kk] = O.compact(w, idx.cpu().numpy()[:, :kk], 0, n)
    assert np.array_equal(got.cpu().numpy().astype(np.float64), want)


def test_select_theta_errors(ctx):
    s = torch.ones((2, 8), device="cuda")
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(B.EcospaError) as e:
            ctx.ecospa_select_theta(s, bad)
        assert e.value.code == B.ERR_K
