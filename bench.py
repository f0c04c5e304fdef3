#!/usr/bin/env python3
"""Benchmark of the coupled-sparse hot path on one MI355X.

A "step" is one pass of the whole path over one batch of a LLaMA-1B-shaped layer
(d=2048, 32 heads x 64, SwiGLU d_ff=5461, RoPE, batch 16 x seq 256, bf16) - the larger of the two layer
configurations the metric names; the GPT-2-Medium-shaped layer (d=1024, 16 heads x 64, d_ff=4096, GELU,
batch 8 x seq 1024) runs through the same code right after it and is reported inside `roofline` and `also`:
    score the QK, VO and FFN pairs (one batched call) -> select top-k at 50% keep (one call) ->
    compact every matrix (one call) -> attention fwd -> FFN fwd -> FFN bwd -> attention bwd.
Inputs are seeded synthetic tensors (weights N(0, 0.02^2), activations N(0, 1)) that are
resident in HBM before the timed region.  One JSON line is printed.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

METRIC = "coupled-sparse layer fwd+bwd tokens/s & TFLOP/s vs dense, 50% sparsity, 1 GPU"
MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the MFMA contraction kernels, averaged over the contraction launches of one sparse
# step of the headline workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/):
# (sha256 prefix of csrc/gemm*, bytes).  Reported only while the kernel sources still have that hash; otherwise null.
GEMM_TRAFFIC = ("4cc5e299fbc0ab02", 139.1e6)
HEADLINE = "c3_llama1b_layer"
SECOND = "c2_gpt2m_layer"


def model_flops(T, L, d, h, k_qk, k_vo, k_ff, causal=True, gated=False, h_kv=None):
    """fwd+bwd model flops of one layer (backward = 2x forward, recomputation not counted,
    causal attention counted at half; a gated FFN has three matrices; h_kv < h: shared key/value heads)."""
    h_kv = h if h_kv is None else h_kv
    proj = 2 * T * d * ((h + h_kv) * k_qk + h_kv * k_vo) + 2 * T * d * h * k_vo
    attn = (2 * T * L * h * (k_qk + k_vo)) * (0.5 if causal else 1.0)
    ffn = (3 if gated else 2) * 2 * T * d * k_ff
    return 3.0 * (proj + attn + ffn)


def gemm_traffic():
    """HBM bytes per contraction launch from the committed counter profile, or None once the kernel sources
    (csrc/gemm*) differ from the ones the counters were taken with."""
    import glob
    import hashlib
    import os
    pat = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2511_11641_amd", "csrc", "gemm*")
    try:
        digest = hashlib.sha256(b"".join(open(p, "rb").read() for p in sorted(glob.glob(pat)))).hexdigest()[:16]
    except OSError:
        return None
    return GEMM_TRAFFIC[1] if GEMM_TRAFFIC[0] == digest else None


class Layer:
    """One attention block followed by one FFN block, all through the C ABI."""

    def __init__(self, ctx, cfg, seed, keep_num, keep_den):
        import torch
        from paper_2511_11641_amd import binding as B, synth
        from paper_2511_11641_amd.layer import AttnBlock, FfnBlock
        self.torch, self.B_ = torch, B
        self.ctx, self.cfg = ctx, cfg
        Bsz, L, d, h, dh, dff = (cfg[k] for k in ("B", "L", "d", "h", "d_h", "d_ff"))
        dt = cfg["dtype"]
        a = synth.attn_layer(seed, Bsz, L, d, h, dh, dtype=dt, bias=cfg["bias"])
        f = synth.ffn_layer(seed + 1000, 1, d, dff, gated=cfg["gated"], dtype=dt, bias=cfg["bias"])
        self.host = {"attn": a, "ffn": f}
        tdt = torch.bfloat16 if dt == "bf16" else torch.float32
        up = lambda arr: None if arr is None else torch.from_numpy(arr).to(tdt).cuda()
        g = {k: up(v) for k, v in a.items()}
        gf = {k: up(v) for k, v in f.items() if k not in ("x", "dy")}
        # W_o and W_out stored with their units as rows ([h d_h, d], [d_ff, d]: the orientation of B in App. A.1), so that
        # steps 1-3 read and gather rows only; the [d, kp] matrices of the forward pass come out of a transposing copy
        g["wo"] = g["wo"].t().contiguous()
        gf["w2"] = gf["w2"].t().contiguous()
        self.x, self.dy = g["x"], g["dy"]
        act = B.ACT_SWIGLU if cfg["gated"] else B.ACT_GELU_ERF
        hkv = cfg.get("h_kv", h)          # grouped-query attention (Eq. 5): the first h_kv heads of W_k, W_v serve as the shared ones
        if hkv != h:
            for nm in ("wk", "wv", "bk", "bv"):
                if g.get(nm) is not None:
                    g[nm] = g[nm][:hkv * dh].contiguous()
        self.attn = AttnBlock(ctx, g["wq"], g["wk"], g["wv"], g["wo"], g.get("bq"), g.get("bk"), g.get("bv"),
                              g.get("bo"), h, dh, rope=cfg["rope"], causal=True, transposed=True, h_kv=hkv, wo_rows=True)
        self.ffn = FfnBlock(ctx, gf["w1"], gf.get("b1"), gf["w2"], gf.get("b2"), act, gf.get("w1b"), transposed=True, w2_rows=True)
        unit = 2 if cfg["rope"] else 1
        self.k_qk_units = (dh // unit) * keep_num // keep_den
        self.k_vo = dh * keep_num // keep_den
        self.k_ff = dff * keep_num // keep_den
        pairs = self.attn.pairs() + [self.ffn.pair()]
        self.pairs = (B.Pair * len(pairs))(*pairs)
        self.scores = self._sel = self._map = self._tr = self._k = self._rope = None     # descriptor arrays are built once: every buffer they name persists
        self.idx = [torch.empty((hkv, self.k_qk_units), dtype=torch.int32, device="cuda"),
                    torch.empty((hkv, self.k_vo), dtype=torch.int32, device="cuda"),
                    torch.empty((1, self.k_ff), dtype=torch.int32, device="cuda")]
        self.prune()
        self.attn.alloc(Bsz, L)
        self.ffn.alloc(Bsz, L)

    # steps 1-3
    def score(self):
        self.scores = self.ctx.ecospa_coupled_score(self.pairs, out=self.scores)

    def select(self):       # one launch for the three pairs
        if self._sel is None:
            mk = self.ctx.select_item
            sel = [mk(s, k, out) for s, k, out in zip(self.scores, (self.k_qk_units, self.k_vo, self.k_ff), self.idx)]
            self._sel = (self.B_.SelectItem * len(sel))(*sel)
        self.ctx.ecospa_select_topk_batch(self._sel)

    def compact(self):      # one launch for every matrix and bias of the layer
        if self._map is None:
            items = self.attn.compact(self.idx[0], self.idx[1], defer=True) + self.ffn.compact(self.idx[2], defer=True)
            self._map = (self.B_.MapItem * len(items))(*items)
            tr = self.attn.post_gather_items() + self.ffn.post_gather_items()
            self._tr = (self.B_.TransposeItem * len(tr))(*tr) if tr else None
        # the kept rotary blocks may have changed: their cos/sin tables are filled again by the same launch (the very
        # first compaction precedes alloc(), which makes the first tables)
        if self._rope is None and self.attn.rope and getattr(self.attn, "cos", None) is not None:
            self._rope = self.attn.rope_item()
        self.ctx.ecospa_compact_batch(self._map, self._rope)
        # transposed copies (one launch): of the gathered rows of W_o / W_out for the forward pass, of the other
        # compact matrices for the input-gradient contractions
        if self._tr is not None:
            self.ctx.ecospa_transpose_batch(self._tr)

    def score_select(self):     # steps 1 and 2 in two launches (the team that finishes a group's scores selects from them)
        if self._k is None:
            import ctypes as C
            self.score()
            n = len(self.scores)
            self._k = (C.c_int * n)(self.k_qk_units, self.k_vo, self.k_ff)
            self._sp = (C.c_void_p * n)(*[t.data_ptr() for t in self.scores])
            self._ip = (C.c_void_p * n)(*[t.data_ptr() for t in self.idx])
            self.ctx.reserve(self.ctx.lib.ecospa_score_workspace_bytes(self.pairs, n))
        self.ctx._check(self.ctx.lib.ecospa_score_select(self.ctx.h, self.pairs, len(self.pairs), self._sp, self._k, self._ip),
                        "ecospa_score_select")

    def prune(self):
        self.score_select()
        self.compact()

    # steps 4-5
    def fwd(self, save=True):
        y1 = self.attn.fwd(self.x, save)
        return self.ffn.fwd(y1, save)

    def bwd(self):
        d1 = self.ffn.bwd(self.attn.y, self.dy)
        return self.attn.bwd(self.x, d1)

    def step(self):
        self.prune()
        self.fwd()
        self.bwd()


def timed(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def timed_gpu(torch, fn, steps, warmup):
    """Device-side time per call (events on the current stream): for calls whose host cost would
    otherwise dominate."""
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def prune_stack(ctx, cfg, n_layers, keep_num, keep_den, steps, rows=True, extras=True):
    """Steps 1-3 on a stack of n_layers layers of the same shape (the re-scoring pass of a whole model):
    one batched score call, one select call, one compaction call; descriptors are built once, so
    the device-side times are not hidden behind the host.  rows: W_o and W_out are stored with their units as rows
    (every gather a row gather; the [d, kp] forms come from the transposing copies timed as `transposes`);
    otherwise in the Linear layout [out, in] (their kept units are gathered by column)."""
    import ctypes as C
    import torch
    from paper_2511_11641_amd import binding as B
    from paper_2511_11641_amd.layer import AttnBlock, FfnBlock
    d, h, dh, dff = (cfg[k] for k in ("d", "h", "d_h", "d_ff"))
    g = lambda *s: (torch.randn(*s, device="cuda") * 0.02).to(torch.bfloat16)
    layers = []
    for _ in range(n_layers):
        a = AttnBlock(ctx, g(h * dh, d), g(h * dh, d), g(h * dh, d), g(h * dh, d) if rows else g(d, h * dh), g(h * dh), g(h * dh),
                      g(h * dh), g(d), h, dh, rope=False, transposed=True, wo_rows=rows, gather_transposed=False)
        f = FfnBlock(ctx, g(dff, d), g(dff), g(dff, d) if rows else g(d, dff), g(d), B.ACT_GELU_ERF, transposed=True, w2_rows=rows,
                     gather_transposed=False)
        layers.append((a, f))
    pairs = [p for a, f in layers for p in a.pairs() + [f.pair()]]
    pair_arr = (B.Pair * len(pairs))(*pairs)
    scores = ctx.ecospa_coupled_score(pair_arr)
    ks = (dh * keep_num // keep_den, dh * keep_num // keep_den, dff * keep_num // keep_den)
    idx = [torch.empty((s.shape[0], ks[i % 3]), dtype=torch.int32, device="cuda") for i, s in enumerate(scores)]
    sel = [ctx.select_item(s, ks[i % 3], o) for i, (s, o) in enumerate(zip(scores, idx))]
    sel_arr = (B.SelectItem * len(sel))(*sel)
    ctx.ecospa_select_topk_batch(sel_arr)
    items = []
    for li, (a, f) in enumerate(layers):
        items += a.compact(idx[3 * li], idx[3 * li + 1], defer=True) + f.compact(idx[3 * li + 2], defer=True)
    item_arr = (B.MapItem * len(items))(*items)
    tr = [t for a, f in layers for t in a.post_gather_items() + f.post_gather_items()]
    tr_arr = (B.TransposeItem * len(tr))(*tr)
    t_score = timed_gpu(torch, lambda: ctx.ecospa_coupled_score(pair_arr, out=scores), steps, 3)
    t_select = timed_gpu(torch, lambda: ctx.ecospa_select_topk_batch(sel_arr), steps, 3)
    t_compact = timed_gpu(torch, lambda: ctx.ecospa_compact_batch(item_arr), steps, 3)
    t_tr = timed_gpu(torch, lambda: ctx.ecospa_transpose_batch(tr_arr), steps, 3)
    # the same gathers writing their transposed copies themselves (one launch for both; column gathers keep their pass)
    for a, f in layers:
        a.gather_transposed = f.gather_transposed = True
    fused = [it for a, f in layers for it in a._map_items(0) + f._map_items(0)]
    fused_arr = (B.MapItem * len(fused))(*fused)
    rest = [t for a, f in layers for t in a.post_gather_items() + f.post_gather_items()]
    rest_arr = (B.TransposeItem * len(rest))(*rest) if rest else None

    def gather_all():
        ctx.ecospa_compact_batch(fused_arr)
        if rest_arr is not None:
            ctx.ecospa_transpose_batch(rest_arr)
    t_fused = timed_gpu(torch, gather_all, steps, 3)
    w_bytes = n_layers * 2 * (4 * d * d + 2 * d * dff)
    keep = keep_num / keep_den
    cols = 0 if rows else n_layers * 2 * (d * d + d * dff)  # the members gathered by column: W_o, W_2
    traffic = 2 * keep * (w_bytes - cols) + (1 + keep) * cols
    head = {"layers": n_layers, "weights_MB": w_bytes / 1e6, "second_members": "units as rows" if rows else "Linear layout [out, in]",
            "score": {"us": t_score * 1e3, "gbs": w_bytes / t_score / 1e6, "frac_of_hbm_peak": w_bytes / t_score / 1e6 / HBM_PEAK_GBS},
            "select": {"us": t_select * 1e3},
            "compact": {"us": t_compact * 1e3, "kept_gbs": 2 * keep * w_bytes / t_compact / 1e6,
                        "traffic_gbs": traffic / t_compact / 1e6,
                        "frac_of_hbm_peak": traffic / t_compact / 1e6 / HBM_PEAK_GBS,
                        "note": "kept bytes read + written; traffic adds the whole 128-byte lines a column gather has to fetch (none with units as rows)"},
            "transposes": {"us": t_tr * 1e3, "note": "the transposing copies a training block keeps beside its compact matrices (4 per layer), either layout"},
            "compact_with_transposed_copies": {"us": t_fused * 1e3, "bytes_gbs": 3 * keep * w_bytes / t_fused / 1e6,
                                               "note": "row gathers that write the transposed copy themselves (kept bytes read once, written twice), "
                                                       "against compact + transposes as two passes"}}
    if not extras:
        return head
    # the two other pieces of Alg. 1: pair-level importance (Eq. 8; the weights stand in for gradient
    # tensors of the same shapes) and the cumulative-threshold rule on the FFN scores
    fisher = ctx.ecospa_pair_fisher(pair_arr, 8192.0)
    t_fisher = timed_gpu(torch, lambda: ctx.ecospa_pair_fisher(pair_arr, 8192.0, out=fisher), steps, 3)
    ffn_scores = torch.cat([scores[3 * li + 2] for li in range(n_layers)]).contiguous()
    t_theta = timed_gpu(torch, lambda: ctx.ecospa_select_theta(ffn_scores, 0.9), steps, 3)
    # Alg. 1's update on the compact tensors of the whole stack: fp32 master weights and moments, bf16 gradients,
    # bf16 working copies written back - one launch for all tensors
    opt_items, opt_keep, n_par = [], [], 0
    for a, f in layers:
        for w_c in (a.wqkv_c, a.wo_c, f.w1_c, f.w2_c):
            st = [w_c.float(), torch.zeros(w_c.shape, device="cuda"), torch.zeros(w_c.shape, device="cuda"),
                  (torch.randn(w_c.shape, device="cuda") * 1e-3).to(torch.bfloat16)]
            opt_keep.append(st)
            opt_items.append(ctx.adamw_item(st[0], st[3], st[1], st[2], w_c))
            n_par += w_c.numel()
    opt_arr = (B.AdamwItem * len(opt_items))(*opt_items)
    t_adamw = timed_gpu(torch, lambda: ctx.ecospa_adamw(opt_arr, 10, 1e-3), steps, 3)
    adamw_bytes = n_par * (2 + 3 * 4 + 3 * 4 + 2)
    return {**head,
            "pair_fisher": {"us": t_fisher * 1e3, "gbs": w_bytes / t_fisher / 1e6,
                            "frac_of_hbm_peak": w_bytes / t_fisher / 1e6 / HBM_PEAK_GBS},
            "select_theta": {"us": t_theta * 1e3, "rows": n_layers, "units": dff, "theta": 0.9},
            "adamw": {"us": t_adamw * 1e3, "params_M": n_par / 1e6, "bytes_per_param": 28, "gbs": adamw_bytes / t_adamw / 1e6,
                      "frac_of_hbm_peak": adamw_bytes / t_adamw / 1e6 / HBM_PEAK_GBS,
                      "note": "compact tensors of the stack: bf16 gradient, fp32 master + both moments read and written, bf16 working copy written"},
            "timing": "device-side events, descriptors prebuilt"}


def fp32_pair_workload(ctx, steps):
    """The fp32 single FFN pair (512 tokens, d = 256, 1024 inner dimensions, half kept): score, select, gather,
    forward and backward.  0.8 GFLOP on the vector ALU (fp32 has no place on the bf16 matrix path): ten short launches
    whose contraction loops are bound by load latency, not arithmetic; time only."""
    import torch
    from paper_2511_11641_amd import binding as B, synth
    from paper_2511_11641_amd.layer import FfnBlock
    cfg = synth.CONFIGS["c1_ffn_f32"]
    T, d, n = cfg["T"], cfg["d"], cfg["n"]
    t = synth.ffn_layer(cfg["seed"], T, d, n, dtype="f32")
    g = {nm: torch.from_numpy(a).cuda() for nm, a in t.items()}
    blk = FfnBlock(ctx, g["w1"], g["b1"], g["w2"], g["b2"], B.ACT_GELU_ERF)
    k = synth.keep_count(n, 1, 2)
    idx = torch.empty((1, k), dtype=torch.int32, device="cuda")
    pair = [blk.pair()]
    scores = ctx.ecospa_coupled_score(pair)

    def prune():
        ctx.ecospa_coupled_score(pair, out=scores)
        ctx.ecospa_select_topk_batch([ctx.select_item(scores[0], k, idx)])
        blk.compact(idx)

    prune()
    blk.alloc(1, T)

    def step():
        prune()
        blk.fwd(g["x"])
        blk.bwd(g["x"], g["dy"])

    ms = timed(torch, step, steps, 3)
    return {"workload": "c1_ffn_f32", "dtype": "f32", "tokens": T, "keep": f"{k}/{n}", "ms_per_step": ms,
            "tokens_per_s": T / (ms * 1e-3), "note": "0.8 GFLOP in ten short launches on the vector ALU: latency-bound, reported as a time only"}


def layer_workload(ctx, name, steps, warmup, h_kv=None, detail=True, keep=(1, 2)):
    """One layer configuration through the whole path: the timed sparse step at 50 % keep (`ms_per_step`), its parts,
    fwd+bwd alone, the dense layer (same library at k = n), and - with detail - the contraction kernels' own launch
    times (HIP events on the library's stream around every launch, in steps run again after the timed region) and the
    attention core's forward time.  With h_kv: the same layer with that many shared key/value heads (Eq. 5)."""
    import torch
    from paper_2511_11641_amd import synth
    cfg = dict(synth.CONFIGS[name])
    if h_kv is not None:
        cfg["h_kv"] = h_kv
    Bsz, L, d, h, dh, dff = (cfg[k] for k in ("B", "L", "d", "h", "d_h", "d_ff"))
    T = Bsz * L
    sp = Layer(ctx, cfg, cfg["seed"], keep[0], keep[1])
    ms_step = timed(torch, sp.step, steps, warmup)
    out = {"workload": name if h_kv is None else f"{name}, {h_kv} key/value heads", "batch": Bsz, "seq_len": L,
           "ms_per_step": ms_step, "tokens_per_s": T / (ms_step * 1e-3)}
    if detail:
        # break-down of the same step, each part timed on its own with device-side events (on the host clock the three
        # short pruning calls would show their Python marshalling rather than their kernels)
        parts = {nm: timed_gpu(torch, fn, steps, 2) for nm, fn in
                 (("score", sp.score), ("select", sp.select), ("score_select", sp.score_select), ("compact", sp.compact),
                  ("fwd", sp.fwd), ("bwd", sp.bwd))}
        # score and select are the two steps as separate calls (three launches); the timed step takes them through
        # ecospa_score_select (two launches): score_select
        out["parts_ms"] = parts
    ms_fb = timed(torch, lambda: (sp.fwd(), sp.bwd()), steps, 2)
    # model flops count the kept dimensions, not the zero padding of the compact layout
    fl_sp = model_flops(T, L, d, h, sp.attn.k_qk_units * sp.attn.unit, sp.attn.k_vo, sp.ffn.k, gated=cfg["gated"], h_kv=h_kv)
    out["fwd_bwd"] = {"ms": ms_fb, "tokens_per_s": T / (ms_fb * 1e-3), "model_tflops": fl_sp / (ms_fb * 1e-3) / 1e12}
    if detail:
        ctx.ecospa_profile_gemm(True)
        for _ in range(steps):
            sp.step()
        n_launch, gemm_ms, gemm_flop = ctx.ecospa_profile_gemm_read()
        ctx.ecospa_profile_gemm(False)
        gemm_tflops = gemm_flop / (gemm_ms * 1e-3) / 1e12
        out["contractions"] = {"achieved": gemm_tflops, "frac": gemm_tflops / MFMA_BF16_PEAK_TFLOPS, "launches": n_launch,
                               "launches_per_step": n_launch // max(steps, 1),
                               "avg_launch_us": gemm_ms * 1e3 / max(n_launch, 1), "flop_per_launch_avg": gemm_flop / max(n_launch, 1),
                               "us_per_step": gemm_ms * 1e3 / max(steps, 1)}
        # the attention core on its own (bound by exponentials and conversions on the vector ALU, not by the matrix
        # units): forward time minus the time of the contraction launches inside the same forward passes
        ctx.ecospa_profile_gemm(True)
        for _ in range(steps):
            sp.fwd()
        _, gemm_ms_fwd, _ = ctx.ecospa_profile_gemm_read()
        ctx.ecospa_profile_gemm(False)
        core_us = (parts["fwd"] - gemm_ms_fwd / steps) * 1e3
        exps = Bsz * h * L * (L + 1) / 2.0
        exp_peak = 256 * 4 * 16 / 4 * 2.4e9          # compute units x SIMDs x lanes per clock, transcendentals at quarter rate
        out["attention_core"] = {"fwd_us": core_us, "exponentials": exps, "exp_per_s": exps / (core_us * 1e-6),
                                 "frac_of_transcendental_peak": exps / (core_us * 1e-6) / exp_peak,
                                 "note": "causal softmax exponentials of the forward pass (incl. the rotary pass where there is one); "
                                         "at 32 kept dimensions a head has only 128 matrix flops per exponential, so the core is priced "
                                         "against the vector ALU, not the MFMA peak"}
        w_bytes = 2 * (4 * d * d + (3 if cfg["gated"] else 2) * d * dff)     # every weight of the three pairs, bf16
        out["score_gbs"] = w_bytes / (parts["score"] * 1e-3) / 1e9
        out["compact_gbs"] = w_bytes / (parts["compact"] * 1e-3) / 1e9        # kept bytes read + kept bytes written (+ transposed copies)
    del sp
    torch.cuda.empty_cache()
    de = Layer(ctx, cfg, cfg["seed"], 1, 1)        # same library at k = n: the dense layer
    ms_de = timed(torch, lambda: (de.fwd(), de.bwd()), steps, warmup)
    fl_de = model_flops(T, L, d, h, dh, dh, dff, gated=cfg["gated"], h_kv=h_kv)
    del de
    torch.cuda.empty_cache()
    out["dense_fwd_bwd"] = {"ms": ms_de, "tokens_per_s": T / (ms_de * 1e-3), "model_tflops": fl_de / (ms_de * 1e-3) / 1e12}
    out["speedup_fwd_bwd_vs_dense"] = ms_de / ms_fb
    out["speedup_whole_step_vs_dense_fwd_bwd"] = ms_de / ms_step
    return out


def mfma_ceiling(ctx):
    """What the matrix units alone sustain on this GPU with operands like the workload's (N(0, 1) bf16 values): about
    0.1 s of back-to-back pure-MFMA launches, so that the clock has settled under the power limit."""
    import torch
    src = torch.randn(65536, device="cuda").to(torch.bfloat16)
    sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    zero = torch.zeros_like(src)
    out = {}
    for nm, buf in (("normal_operands", src), ("zero_operands", zero)):
        fl = ctx.ecospa_mfma_probe(buf, sink, 2000)
        ms = timed_gpu(torch, lambda: ctx.ecospa_mfma_probe(buf, sink, 2000), 60, 20)
        out[nm + "_tflops"] = fl / (ms * 1e-3) / 1e12
    out["note"] = ("pure v_mfma_f32_32x32x16_bf16 loop on all 1024 SIMDs, no memory traffic, same run; with all-zero operands the "
                   "matrix units draw less power and the clock stays higher")
    return out


def hbm_ceilings(ctx, nbytes, steps=10):
    """What plain kernels reach on this GPU over a buffer of the size the 24-layer pruning pass reads: a streaming read
    and a 1:1 copy (the library's own probe kernels and, for the copy, torch's device copy as a second opinion)."""
    import torch
    n = int(nbytes) // 16 * 16
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    sink = torch.zeros(64, dtype=torch.uint8, device="cuda")
    t_read = timed_gpu(torch, lambda: ctx.ecospa_hbm_probe(src, sink, False), steps, 3)
    dst.zero_()
    t_copy = timed_gpu(torch, lambda: ctx.ecospa_hbm_probe(src, dst, True), steps, 3)
    ok = bool(torch.equal(src, dst))
    t_tcopy = timed_gpu(torch, lambda: dst.copy_(src), steps, 3)
    del src, dst
    torch.cuda.empty_cache()
    return {"bytes": n, "read_gbs": n / t_read / 1e6, "copy_gbs": 2 * n / t_copy / 1e6, "torch_copy_gbs": 2 * n / t_tcopy / 1e6,
            "copy_checked": ok, "note": "plain streaming read / 1:1 copy (bytes read + bytes written) of a buffer of this size, same run"}


def torch_dense_layer(name, steps):
    """Context only: the same dense layer (attention block + FFN block, no norms, no residual) forward+backward
    through torch-ROCm's own operators (vendor GEMMs, its fused attention), to show that the dense baseline of
    this library is no strawman.  Nothing of the library runs here."""
    import torch
    import torch.nn.functional as F
    from paper_2511_11641_amd import synth
    cfg = synth.CONFIGS[name]
    Bsz, L, d, h, dh, dff = (cfg[k] for k in ("B", "L", "d", "h", "d_h", "d_ff"))
    g = lambda *s: (torch.randn(*s, device="cuda") * 0.02).to(torch.bfloat16).requires_grad_(True)
    wqkv, bqkv, wo, bo, w1, b1, w2, b2 = g(3 * d, d), g(3 * d), g(d, d), g(d), g(dff, d), g(dff), g(d, dff), g(d)
    x = torch.randn(Bsz * L, d, device="cuda").to(torch.bfloat16).requires_grad_(True)
    dy = torch.randn(Bsz * L, d, device="cuda").to(torch.bfloat16)

    def step():
        q, k, v = (t.reshape(Bsz, L, h, dh).transpose(1, 2) for t in F.linear(x, wqkv, bqkv).chunk(3, dim=-1))
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(Bsz * L, d)
        y1 = F.linear(o, wo, bo)
        y2 = F.linear(F.gelu(F.linear(y1, w1, b1)), w2, b2)
        y2.backward(dy)

    ms = timed(torch, step, steps, 3)
    return {"workload": name, "ms_fwd_bwd": ms, "tokens_per_s": Bsz * L / (ms * 1e-3),
            "note": "torch-ROCm operators (vendor GEMM library, fused attention), bf16, autograd backward; context for dense_fwd_bwd"}


def inference_sweep(ctx, name, steps):
    """Forward only (inference) of the layer at batch 1 and batch 32, dense and at three keep ratios: per-layer
    time, tokens/s and the speed-up over the dense layer run through the same library."""
    import torch
    from paper_2511_11641_amd import synth
    rows = []
    for Bsz in (1, 32):
        cfg = dict(synth.CONFIGS[name], B=Bsz)
        T = Bsz * cfg["L"]
        ms_dense = None
        for num, den in ((1, 1), (3, 4), (1, 2), (3, 10)):
            lay = Layer(ctx, cfg, cfg["seed"], num, den)
            ms = timed(torch, lambda: lay.fwd(save=False), steps, 3)
            ms_dense = ms if ms_dense is None else ms_dense
            rows.append({"batch": Bsz, "seq_len": cfg["L"], "keep": f"{num}/{den}", "ms_fwd": ms,
                         "tokens_per_s": T / (ms * 1e-3), "speedup_vs_dense": ms_dense / ms})
            del lay
            torch.cuda.empty_cache()
    return {"workload": name, "pass": "forward only", "rows": rows}


def _stack_flops(st, k_qk, k_vo, k_ff, passes):
    """Model flops of the stack: the layers' contractions and attention (causal at half) plus the output projection."""
    c = st.cfg
    per_layer = model_flops(st.T, st.L, st.d, st.h, k_qk, k_vo, k_ff, gated=c["gated"]) / 3.0
    return passes * (len(st.layers) * per_layer + 2.0 * st.T * st.d * st.vocab)


def stack_training(ctx, name, n_layers, vocab, Bsz, L, keeps, steps, rescore_every=200):
    """Whole-model training step of a stack of `name`-shaped layers (embedding, pre-norm layers, output projection,
    cross-entropy, AdamW with fp32 master weights): per keep ratio the time of a plain step, of a step that first
    estimates the coupled importance again (write-back, score, select, gather of all layers), and the throughput with
    one such step in every `rescore_every`.  Every kernel of a step is the library's (norms, residuals, embedding and
    loss included); torch allocates and draws the initial weights."""
    import torch
    from paper_2511_11641_amd import synth
    from paper_2511_11641_amd.stack import DecoderStack
    cfg = dict(synth.CONFIGS[name], B=Bsz, L=L)
    T, rows, dense_ms = Bsz * L, [], None
    ids = torch.randint(0, vocab, (T,), device="cuda")
    tgt = torch.roll(ids, -1)
    for num, den in keeps:
        st = DecoderStack(ctx, cfg, n_layers, vocab, keep=(num, den), seed=1, train=True)
        ms_step = timed(torch, lambda: st.train_step(ids, tgt), steps, 2)
        ms_fwd = timed(torch, lambda: st.forward(ids), steps, 1)
        ms_bwd = timed(torch, lambda: (st.forward(ids), st.backward(ids, tgt)), steps, 1) - ms_fwd
        ms_upd = timed(torch, st.update, steps, 1)
        ms_prune = timed(torch, st.prune, max(2, steps // 2), 1)
        # the contraction kernels inside two whole steps: per-launch events on the library's stream
        ctx.ecospa_profile_gemm(True)
        st.train_step(ids, tgt)
        st.train_step(ids, tgt)
        n_launch, gemm_ms, gemm_flop = ctx.ecospa_profile_gemm_read()
        ctx.ecospa_profile_gemm(False)
        a, f = st.layers[0].attn["w"], st.layers[0].ffn["w"]
        fl = _stack_flops(st, a.k_qk_units * a.unit, a.k_vo, f.k, 3)      # kept dimensions, not the padding
        dense_ms = ms_step if (num, den) == (1, 1) else dense_ms
        amort = (rescore_every - 1) * ms_step + (ms_step + ms_prune)
        rows.append({"keep": f"{num}/{den}", "ms_step": ms_step, "ms_rescore_step": ms_step + ms_prune,
                     "tokens_per_s": rescore_every * T / (amort * 1e-3), "model_tflops": fl / (ms_step * 1e-3) / 1e12,
                     "parts_ms": {"fwd": ms_fwd, "bwd": ms_bwd, "adamw_and_transposes": ms_upd, "rescore": ms_prune},
                     "contractions": {"launches_per_step": n_launch // 2, "ms_per_step": gemm_ms / 2,
                                      "tflops": gemm_flop / (gemm_ms * 1e-3) / 1e12,
                                      "frac_of_mfma_peak": gemm_flop / (gemm_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
                     "trained_params_M": st.n_params / 1e6})
        del st
        torch.cuda.empty_cache()
    for r in rows:
        r["speedup_vs_dense"] = None if dense_ms is None else dense_ms / r["ms_step"]
    return {"workload": f"{n_layers} x {name}", "batch": Bsz, "seq_len": L, "vocab": vocab,
            "rescore_every": rescore_every, "rows": rows,
            "tokens_per_s_formula": "rescore_every * T / ((rescore_every - 1) * ms_step + ms_rescore_step)",
            "glue": "embedding, norms with the residual adds, cross-entropy: the library's kernels (no torch operator in a step); weights: device RNG, N(0, 0.02)"}


def stack_inference(ctx, name, n_layers, vocab, L, keeps, steps):
    """Forward only of the whole stack (logits for every position) at batch 1 and batch 32."""
    import torch
    from paper_2511_11641_amd import synth
    from paper_2511_11641_amd.stack import DecoderStack
    rows = []
    for Bsz in (1, 32):
        cfg = dict(synth.CONFIGS[name], B=Bsz, L=L)
        ids = torch.randint(0, vocab, (Bsz * L,), device="cuda")
        ms_dense = None
        for num, den in keeps:
            st = DecoderStack(ctx, cfg, n_layers, vocab, keep=(num, den), seed=1, train=False)
            ms = timed(torch, lambda: st.forward(ids), steps, 2)
            ms_layers = timed(torch, lambda: st.forward(ids, lm_head=False), steps, 1)
            ms_dense = ms if (num, den) == (1, 1) else ms_dense
            rows.append({"batch": Bsz, "seq_len": L, "keep": f"{num}/{den}", "ms_fwd": ms, "ms_fwd_without_output_projection": ms_layers,
                         "tokens_per_s": Bsz * L / (ms * 1e-3), "speedup_vs_dense": None if ms_dense is None else ms_dense / ms})
            del st
            torch.cuda.empty_cache()
    return {"workload": f"{n_layers} x {name}", "pass": "forward only, logits for every position", "vocab": vocab, "rows": rows}


def cpu_baseline(cfg, seed, keep_num, keep_den, sample_B):
    """The fp64 oracle, as it stands, on `sample_B` batch elements of the same workload."""
    import os
    from oracle import ecospa_oracle as O
    from paper_2511_11641_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    L, d, h, dh, dff = (cfg[k] for k in ("L", "d", "h", "d_h", "d_ff"))
    gated, rope, bias = cfg["gated"], cfg["rope"], cfg["bias"]
    a = synth.attn_layer(seed, sample_B, L, d, h, dh, dtype=cfg["dtype"], bias=bias)
    f = synth.ffn_layer(seed + 1000, 1, d, dff, gated=gated, dtype=cfg["dtype"], bias=bias)
    dy = a["dy"]
    unit = 2 if rope else 1
    act = O.ACT_SWIGLU if gated else O.ACT_GELU_ERF
    t0 = time.perf_counter()
    vq = O.coupled_score(O.PAIR_QK, a["wq"], a["wk"], h, dh, unit)
    vv = O.coupled_score(O.PAIR_VO, a["wv"], a["wo"], h, dh)
    vf = O.coupled_score(O.PAIR_FFN_GATED if gated else O.PAIR_FFN, f["w1"], f["w2"], 1, dff, w1b=f.get("w1b"))
    iq = O.select_topk(vq.astype(np.float32), (dh // unit) * keep_num // keep_den)
    iv = O.select_topk(vv.astype(np.float32), dh * keep_num // keep_den)
    iff = O.select_topk(vf.astype(np.float32), dff * keep_num // keep_den)
    wq = O.heads_rows(O.compact(a["wq"], iq, 0, dh, unit), h)
    wk = O.heads_rows(O.compact(a["wk"], iq, 0, dh, unit), h)
    wv = O.heads_rows(O.compact(a["wv"], iv, 0, dh), h)
    wo = O.heads_cols(O.compact(a["wo"], iv, 1, dh), h)
    kw, b1, b2 = {}, None, None
    if bias:
        kw = dict(bq=O.compact(a["bq"], iq, 0, dh, unit).reshape(h, -1), bk=O.compact(a["bk"], iq, 0, dh, unit).reshape(h, -1),
                  bv=O.compact(a["bv"], iv, 0, dh).reshape(h, -1), bo=a["bo"])
        b1, b2 = O.compact(f["b1"], iff, 0, dff), f["b2"]
    angles = O.rope_angles(iq, L, dh) if rope else None
    w1, w2 = O.compact(f["w1"], iff, 0, dff), O.compact(f["w2"], iff, 1, dff)
    w1b = O.compact(f["w1b"], iff, 0, dff) if gated else None
    y1, sv = O.attn_fwd(a["x"], wq, wk, wv, wo, sample_B, L, dh ** -0.5, True, angles=angles, **kw)
    _, sv2 = O.ffn_fwd(y1, w1, b1, w2, b2, act, w1b=w1b)
    g2 = O.ffn_bwd(y1, dy, w1, w2, act, sv2, w1b=w1b)
    O.attn_bwd(a["x"], g2["dx"], wq, wk, wv, wo, sample_B, L, dh ** -0.5, sv, angles=angles)
    dt = time.perf_counter() - t0
    return {"value": sample_B * L / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{sample_B} of {cfg['B']} batch elements (seq {L}) of the same layer, whole path "
                      f"score+select+compact+fwd+bwd in fp64 numpy, {dt:.1f} s"}


def stack_shrink_schedule(ctx, name, n_layers, vocab, Bsz, L, schedule, steps):
    """Alg. 1 with removal for good on a stack of `name`-shaped layers: built dense, the full-size arrays released, then
    shrunk stage by stage from its own compact state (parameters, fp32 master copies and both moments together).  Per
    stage: the time of the shrinking call, of a training step afterwards, and the device memory the process holds
    (weights in all four families, gradients, the activations of one step, the workspace)."""
    import torch
    from paper_2511_11641_amd import synth
    from paper_2511_11641_amd.stack import DecoderStack
    cfg = dict(synth.CONFIGS[name], B=Bsz, L=L)
    T = Bsz * L
    ids = torch.randint(0, vocab, (T,), device="cuda")
    tgt = torch.roll(ids, -1)
    torch.cuda.empty_cache()
    base = torch.cuda.memory_allocated()
    st = DecoderStack(ctx, cfg, n_layers, vocab, keep=(1, 1), seed=1, train=True, permanent=True)
    rows = []
    for num, den in schedule:
        ms_shrink = None
        if (num, den) != (1, 1):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            st.shrink((num, den))
            torch.cuda.synchronize()
            ms_shrink = (time.perf_counter() - t0) * 1e3
        ms_step = timed(torch, lambda: st.train_step(ids, tgt), steps, 1)
        rows.append({"keep": f"{num}/{den}", "ms_shrink": ms_shrink, "ms_step": ms_step, "tokens_per_s": T / (ms_step * 1e-3),
                     "resident_GB": (torch.cuda.memory_allocated() - base) / 1e9, "trained_params_M": st.n_params / 1e6})
    del st
    torch.cuda.empty_cache()
    return {"workload": f"{n_layers} x {name}, removal for good", "batch": Bsz, "seq_len": L, "vocab": vocab, "rows": rows,
            "note": "resident_GB: device memory held by the stack (four families of every kept tensor, gradients, one step's "
                    "activations, workspace); the dense stage holds no second full-size copy either"}


def stack_workloads(ctx):
    """The two whole-model workloads: the LLaMA-1B-shaped 24-layer training step (batch 32 x 256, vocabulary 32000,
    importance estimated again every 200 steps, 50 % keep, beside the dense model) and the GPT-2-Medium-shaped
    24-layer sweep over keep ratios (training step at batch 8 x 1024; forward only at batch 1 and 32)."""
    sweep = ((1, 1), (3, 4), (1, 2), (3, 10))
    return {
        "stack_llama1b_train": stack_training(ctx, "c3_llama1b_layer", 24, 32000, 32, 256, ((1, 1), (1, 2)), 4),
        "stack_gpt2m_train_sweep": stack_training(ctx, "c2_gpt2m_layer", 24, 50304, 8, 1024, sweep, 4),
        "stack_gpt2m_inference": stack_inference(ctx, "c2_gpt2m_layer", 24, 50304, 1024, sweep, 4),
        "stack_llama1b_shrink": stack_shrink_schedule(ctx, "c3_llama1b_layer", 24, 32000, 32, 256, ((1, 1), (3, 4), (1, 2)), 3),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the 24-layer pruning pass and the LLaMA-1B-shaped layer reported beside the main workload")
    ap.add_argument("--pmc-reference", action="store_true",
                    help="first run 3 plain device copies of a 128 MiB tensor, so that hardware byte counters read "
                         "under rocprofv3 --pmc can be scaled by what they show for a copy of known size")
    ap.add_argument("--prune-only", action="store_true",
                    help="run only the 24-layer pruning pass (score, select, compaction, Eq. 8, threshold rule, AdamW) and "
                         "print its figures (for profiler runs of the HBM-bound kernels)")
    ap.add_argument("--stacks-only", action="store_true",
                    help="run only the whole-model workloads (24-layer training step and forward-only sweep) and print their figures")
    ap.add_argument("--stack-step-only", action="store_true",
                    help="run only the LLaMA-1B-shaped 24-layer training workload at 50 %% keep (for profiler runs)")
    ap.add_argument("--sparse-only", action="store_true",
                    help="run only the timed sparse steps (for hardware-counter runs) and print a short line")
    ap.add_argument("--workload", default=None, help="with --sparse-only: c3_llama1b_layer (default) or c2_gpt2m_layer")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU hot path only: run it with --gpus 1 "
              "(nothing in this library shards across GPUs).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2511_11641_amd import binding as B, synth
    if not torch.cuda.is_available():
        print("bench.py needs an MI355X: no GPU is visible.", file=sys.stderr)
        sys.exit(2)
    name = HEADLINE
    cfg = dict(synth.CONFIGS[name])
    seed = cfg["seed"]
    ctx = B.Context("cuda:0")
    Bsz, L, d, h, dh, dff = (cfg[k] for k in ("B", "L", "d", "h", "d_h", "d_ff"))
    T = Bsz * L
    c2 = dict(synth.CONFIGS[SECOND])

    if args.pmc_reference:      # a plain device copy reads 128 MiB and writes 128 MiB per launch
        ref = torch.zeros((65536, 1024), dtype=torch.bfloat16, device="cuda")
        out_ref = torch.empty_like(ref)
        for _ in range(3):
            out_ref.copy_(ref)
        torch.cuda.synchronize()
        del ref, out_ref

    if args.prune_only:
        out = prune_stack(ctx, c2, 24, 1, 2, 20)
        out["linear_layout"] = prune_stack(ctx, c2, 24, 1, 2, 20, rows=False, extras=False)
        print(json.dumps({"prune_24_layers": out}))
        return

    if args.stack_step_only:
        print(json.dumps({"stack_llama1b_train": stack_training(ctx, "c3_llama1b_layer", 24, 32000, 32, 256, ((1, 2),), 4)}))
        return
    if args.stacks_only:
        print(json.dumps(stack_workloads(ctx)))
        return

    if args.sparse_only:
        wl = args.workload or name
        sparse = Layer(ctx, dict(synth.CONFIGS[wl]), synth.CONFIGS[wl]["seed"], 1, 2)
        ms_step = timed(torch, sparse.step, args.steps, args.warmup)
        print(json.dumps({"workload": wl, "ms_per_step": ms_step, "steps": args.steps, "warmup": args.warmup}))
        return

    main_wl = layer_workload(ctx, name, args.steps, args.warmup)
    ms_step = main_wl["ms_per_step"]
    gm = main_wl["contractions"]
    second = layer_workload(ctx, SECOND, args.steps, args.warmup)
    g2 = second["contractions"]

    # the HBM-bound steps on a whole model's weights (24 layers, 604 MB), beside what plain kernels reach on the same bytes
    prune = prune_stack(ctx, c2, 24, 1, 2, 20)
    prune["linear_layout"] = prune_stack(ctx, c2, 24, 1, 2, 20, rows=False, extras=False)   # W_o, W_out as [out, in]: column gathers
    ceil = hbm_ceilings(ctx, prune["weights_MB"] * 1e6)
    hbm = {"peak_gbs": HBM_PEAK_GBS, "workload": "steps 1-3 over 24 GPT-2-Medium-shaped layers, one call each",
           "weights_MB": prune["weights_MB"], "read_ceiling_gbs": ceil["read_gbs"],
           "copy_ceiling_gbs": max(ceil["copy_gbs"], ceil["torch_copy_gbs"]), "ceilings": ceil,
           "score": {"us": prune["score"]["us"], "gbs": prune["score"]["gbs"], "frac_of_peak": prune["score"]["frac_of_hbm_peak"],
                     "frac_of_read_ceiling": prune["score"]["gbs"] / ceil["read_gbs"]},
           "select": {"us": prune["select"]["us"]},
           "compact": {"us": prune["compact"]["us"], "kept_gbs": prune["compact"]["kept_gbs"],
                       "traffic_gbs": prune["compact"]["traffic_gbs"],
                       "frac_of_peak_kept": prune["compact"]["kept_gbs"] / HBM_PEAK_GBS,
                       "frac_of_peak_traffic": prune["compact"]["frac_of_hbm_peak"],
                       "frac_of_copy_ceiling_kept": prune["compact"]["kept_gbs"] / max(ceil["copy_gbs"], ceil["torch_copy_gbs"]),
                       "frac_of_copy_ceiling_traffic": prune["compact"]["traffic_gbs"] / max(ceil["copy_gbs"], ceil["torch_copy_gbs"])}}

    mfma = mfma_ceiling(ctx)
    out = {
        "metric": METRIC, "value": T / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "layer": "LLaMA-1B shaped: d=2048, 32 heads x 64, SwiGLU d_ff=5461, RoPE, causal, no biases",
                   "batch": Bsz, "seq_len": L, "keep": "1/2 per coupled pair (16 of 32 rotary blocks, k_vo=32, k_ff=2730)",
                   "step": "score+select+compact+attn/ffn fwd+bwd",
                   "storage": "W_q, W_k, W_v, W_gate, W_up as [out, in]; W_o and W_down with their units as rows, [units, d]",
                   "second_workload": SECOND + " (same path; its figures are in roofline." + SECOND + " and in also)"},
        "fwd_bwd": main_wl["fwd_bwd"], "dense_fwd_bwd": main_wl["dense_fwd_bwd"],
        "speedup_fwd_bwd_vs_dense": main_wl["speedup_fwd_bwd_vs_dense"],
        "speedup_whole_step_vs_dense_fwd_bwd": main_wl["speedup_whole_step_vs_dense_fwd_bwd"],
        "parts_ms": main_wl["parts_ms"], "attention_core": main_wl["attention_core"],
        "score_gbs": main_wl["score_gbs"], "compact_gbs": main_wl["compact_gbs"],
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_{pipe,mfma,rs}_kernel", "achieved": gm["achieved"],
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": gm["frac"], "traffic": gemm_traffic(),
                     "launches": gm["launches"], "launches_per_step": gm["launches_per_step"], "avg_launch_us": gm["avg_launch_us"],
                     "flop_per_launch_avg": gm["flop_per_launch_avg"],
                     "measured": f"HIP events around each launch, {args.steps} steps re-run after the timed region",
                     "step": {"ms_per_step": ms_step, "fwd_bwd_ms": main_wl["fwd_bwd"]["ms"], "dense_fwd_bwd_ms": main_wl["dense_fwd_bwd"]["ms"],
                              "speedup_fwd_bwd_vs_dense": main_wl["speedup_fwd_bwd_vs_dense"],
                              "model_tflops_fwd_bwd": main_wl["fwd_bwd"]["model_tflops"],
                              "attention_core_fwd_us": main_wl["attention_core"]["fwd_us"]},
                     SECOND: {"achieved": g2["achieved"], "frac": g2["frac"], "avg_launch_us": g2["avg_launch_us"],
                              "launches_per_step": g2["launches_per_step"], "flop_per_launch_avg": g2["flop_per_launch_avg"],
                              "ms_per_step": second["ms_per_step"], "tokens_per_s": second["tokens_per_s"],
                              "fwd_bwd_ms": second["fwd_bwd"]["ms"], "dense_fwd_bwd_ms": second["dense_fwd_bwd"]["ms"],
                              "speedup_fwd_bwd_vs_dense": second["speedup_fwd_bwd_vs_dense"],
                              "model_tflops_fwd_bwd": second["fwd_bwd"]["model_tflops"],
                              "attention_core_fwd_us": second["attention_core"]["fwd_us"], "parts_ms": second["parts_ms"]},
                     "sustained_mfma": mfma,
                     "frac_of_sustained_mfma": gm["achieved"] / mfma["normal_operands_tflops"],
                     "hbm": hbm},
        "also": second,
        "prune_24_layers": prune,
    }
    if not args.no_extras:
        out["fp32_pair"] = fp32_pair_workload(ctx, args.steps)
        out["gqa_layer"] = layer_workload(ctx, "c3_llama1b_layer", args.steps, args.warmup, h_kv=8, detail=False)
        # the paper's larger pre-training shape (32 heads of 128 dims): dense and keep 3/4 run the 128-wide attention kernels
        out["llama7b_layer"] = {f"keep_{n}_{m}": layer_workload(ctx, "llama7b_layer", 20, 3, detail=False, keep=(n, m))
                                for n, m in ((1, 2), (3, 4))}
        out["inference"] = inference_sweep(ctx, SECOND, 20)
        out["torch_dense_fwd_bwd"] = torch_dense_layer(SECOND, 20)
        out.update(stack_workloads(ctx))
    if not args.no_cpu_baseline:
        # the fp64 oracle on the whole batch of the headline layer, and of the second one (inside the same object)
        cb = cpu_baseline(cfg, seed, 1, 2, sample_B=cfg["B"])
        cb[SECOND] = cpu_baseline(c2, c2["seed"], 1, 2, sample_B=c2["B"])
        out["cpu_baseline"] = cb
        if not args.no_extras:
            # the oracle beside the multi-layer workloads: one layer timed, the stack figure is 24 times that
            # (no embedding, norms, output projection or optimizer) - extrapolated, not measured
            note = "EXTRAPOLATED: 24 x the oracle's time for one layer at 50 % keep (layers only), not a measured stack run"
            out["stack_gpt2m_train_sweep"]["cpu_oracle_extrapolated"] = {
                "tokens_per_s": cb[SECOND]["value"] / 24, "cores": cb["cores"], "note": note}
            out["stack_llama1b_train"]["cpu_oracle_extrapolated"] = {
                "tokens_per_s": cb["value"] / 24, "cores": cb["cores"], "note": note}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
