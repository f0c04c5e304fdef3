"""The whole path of a layer (steps 1-3, forward, backward) recorded once into a HIP graph and replayed: the library
allocates nothing, waits for nothing and records no memset, so a replay must give, bit for bit, what the same calls
give eagerly on the inputs present at replay time - checked on three replays with new weights and inputs written in
place and eager work between them."""
import numpy as np
import pytest
import torch

from paper_2511_11641_amd import binding as B
from paper_2511_11641_amd import synth
from paper_2511_11641_amd.layer import AttnBlock, FfnBlock

pytestmark = pytest.mark.gpu


def test_layer_step_recorded_in_a_graph_replays_bit_exactly():
    Bsz, L, d, h, dh, dff = 2, 160, 128, 4, 64, 520
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = B.Context("cuda:0")                     # bound to `stream`, the stream the graph is recorded on
        a = synth.attn_layer(51, Bsz, L, d, h, dh, dtype="bf16", bias=False)
        f = synth.ffn_layer(52, Bsz * L, d, dff, gated=True, dtype="bf16", bias=False)
        up = lambda t: torch.from_numpy(t).to(torch.bfloat16).cuda()
        ga = {k: up(v) for k, v in a.items() if v is not None}
        gf = {k: up(v) for k, v in f.items() if v is not None}
        wo_r, w2_r = ga["wo"].t().contiguous(), gf["w2"].t().contiguous()
        attn = AttnBlock(ctx, ga["wq"], ga["wk"], ga["wv"], wo_r, None, None, None, None, h, dh, rope=True, causal=True,
                         transposed=True, wo_rows=True)
        ffn = FfnBlock(ctx, gf["w1"], None, w2_r, None, B.ACT_SWIGLU, gf["w1b"], transposed=True, w2_rows=True)
        pairs = attn.pairs() + [ffn.pair()]
        pair_arr = (B.Pair * len(pairs))(*pairs)
        ks = [dh // 4, dh // 2, dff // 2]
        scores = [torch.empty((p.groups, p.n // p.unit), dtype=torch.float32, device="cuda") for p in pairs]
        idx = [torch.empty((p.groups, k), dtype=torch.int32, device="cuda") for p, k in zip(pairs, ks)]
        ctx.ecospa_score_select(pair_arr, ks, scores, idx)
        items = attn.compact(idx[0], idx[1], defer=True) + ffn.compact(idx[2], defer=True)
        assert not attn.post_gather_items() and not ffn.post_gather_items()      # every copy comes out of the gather launch
        item_arr = (B.MapItem * len(items))(*items)
        ctx.ecospa_compact_batch(item_arr)
        attn.alloc(Bsz, L)
        ffn.alloc(Bsz, L)
        x, dy = ga["x"], ga["dy"]

        def step():
            ctx.ecospa_score_select(pair_arr, ks, scores, idx)
            ctx.ecospa_compact_batch(item_arr)
            attn._rope_table(L, out=(attn.cos, attn.sin))
            y1 = attn.fwd(x)
            ffn.fwd(y1)
            d1 = ffn.bwd(y1, dy)
            attn.bwd(x, d1)

        outs = lambda: [idx[0], idx[1], idx[2], attn.wqkv_c, attn.wqkv_t, attn.wo_c, ffn.w1_c, ffn.w1_t, ffn.w2_c, ffn.y, attn.dx,
                        attn.dwqkv_c, attn.dwo_c, ffn.dw1_c, ffn.dw2_c]
        for _ in range(2):      # every buffer and the workspace exist before the recording
            step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
        rng = np.random.default_rng(3)
        for trial in range(3):
            # new weights (other units win the selection) and new inputs, written in place
            for t in (ga["wq"], ga["wk"], ga["wv"], wo_r, gf["w1"], gf["w1b"], w2_r):
                t.mul_(torch.from_numpy(rng.uniform(0.5, 1.5, size=(t.shape[0], 1)).astype(np.float32)).cuda().to(t.dtype))
            x.copy_(torch.randn_like(x))
            dy.copy_(torch.randn_like(dy))
            step()
            want = [t.clone() for t in outs()]
            for t in outs():
                t.fill_(0)
            (x.float() @ x.float().t()).sum().item()      # eager work and a wait between the replays
            graph.replay()
            torch.cuda.synchronize()
            for i, (got, w) in enumerate(zip(outs(), want)):
                assert torch.equal(got, w), f"replay {trial}: output {i} differs from the eager result"
        assert not torch.equal(want[2], torch.zeros_like(want[2]))
