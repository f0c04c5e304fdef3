"""GPU parity at the vision-transformer shapes of the paper's DeiT experiments (Sec. 4.1: DeiT-Tiny d = 192,
3 heads; DeiT-Small d = 384, 6 heads; 197 tokens per image, no causal mask, GELU): one attention block and
one FFN block each, 50 % and 30 % of the inner dimensions kept, against the oracle.  The sequence length is
not a multiple of any tile and the model widths are narrower than one 256-wide contraction tile."""
import pytest

from test_gpu_attn import ctx, run_attn_case      # noqa: F401  (fixture and case runner)
from test_gpu_ffn import run_ffn_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,h", [(192, 3), (384, 6)])
@pytest.mark.parametrize("k", [32, 19])
def test_deit_attention_block(ctx, d, h, k):
    run_attn_case(ctx, 90 + h, 4, 197, d, h, 64, k, k, rope=False, causal=False, structure="pretrained")


@pytest.mark.parametrize("d", [192, 384])
@pytest.mark.parametrize("num,den", [(1, 2), (3, 10)])
def test_deit_ffn_block(ctx, d, num, den):
    n = 4 * d
    run_ffn_case(ctx, 95, 4, 197, d, n, n * num // den, "gelu", "bf16", structure="pretrained")
