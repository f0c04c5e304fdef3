"""A stack of pre-norm decoder layers around the library's blocks: the harness of the multi-layer workloads
(a training step of the whole model with the coupled importance estimated again every so many steps, and
forward-only inference at several keep ratios).

What runs where.  Through the C ABI: the coupled scores (Eq. 10) of every pair of every layer in one call,
the selection, the aligned gather of parameters, master copies and optimizer moments (Def. 1, Alg. 1), their
write-back into the full-size arrays before the next estimate, both blocks' forward and backward
contractions, the contractions of the output projection onto the vocabulary, the AdamW update of every
tensor, and the glue that is the same for a dense and a sparse model and is no part of the method -
embedding lookup and its gradient, LayerNorm / RMSNorm with the residual addition in front of them and
their backward, the cross-entropy loss.  Torch allocates the buffers (once, when the stack is built) and
owns the stream; no torch operator runs in a forward pass, a backward pass or an update.

State between two estimates is compact: fp32 master weights and both moments live in the compact layout
and only they are updated.  Two ways to estimate again:
  * `prune()` (default): the full-size arrays stay resident so that a later estimate can bring a dimension
    back; pruned rows/columns are frozen - no gradient reaches them - until `prune()` writes the compact
    state back, scores the full-size master weights again and gathers the new choice;
  * `shrink(keep)` with `permanent=True`: Alg. 1 as printed - rows and columns are removed for good.  The
    full-size arrays are released after the first gather; every later call scores the compact master
    weights, keeps fewer units of what is left and gathers parameters, master copies and both moments
    from the compact layout into a smaller one, so the resident state falls with the kept fraction.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B
from .layer import AttnBlock, FfnBlock, rows_aligned

FAMILIES = ("w", "mst", "m", "v")      # bf16 working copy, fp32 master, first and second moment


class _Param:
    """A glue parameter (embedding, norm gain, output projection): bf16 working copy, fp32 master, moments."""

    def __init__(self, value: torch.Tensor, train: bool):
        self.w = value.to(torch.bfloat16).contiguous()
        self.g = None
        if train:
            self.mst = self.w.float()
            self.m, self.v = torch.zeros_like(self.mst), torch.zeros_like(self.mst)
            self.g = torch.zeros_like(self.w)

    def item(self):
        return B.Context.adamw_item(self.mst, self.g, self.m, self.v, self.w)


class _Layer:
    pass


class DecoderStack:
    def __init__(self, ctx: B.Context, cfg: dict, n_layers: int, vocab: int, keep=(1, 2), seed: int = 0,
                 train: bool = True, lr: float = 1e-4, weight_decay: float = 0.01, permanent: bool = False):
        """cfg: B, L, d, h, d_h, d_ff, gated, rope, bias as in synth.CONFIGS, optionally h_kv (gated: RMSNorm, no position table;
        otherwise LayerNorm with a learned position table).  keep = (num, den): every pair keeps
        floor(n * num / den) of its units; (1, 1) is the dense model through the same code."""
        self.ctx, self.cfg, self.train, self.permanent = ctx, cfg, train, permanent
        self.Bsz, self.L, self.d, self.h, self.d_h, self.d_ff = (cfg[k] for k in ("B", "L", "d", "h", "d_h", "d_ff"))
        self.h_kv = cfg.get("h_kv", self.h)      # fewer key/value heads than query heads: grouped-query attention (Eq. 5)
        self.T = self.Bsz * self.L
        self.vocab, self.lr, self.wd, self.t = vocab, lr, weight_decay, 0
        self.rms = bool(cfg["gated"])
        self.eps = 1e-6 if self.rms else 1e-5
        gen = torch.Generator(device="cuda").manual_seed(seed)
        d, h, dh, dff, hkv = self.d, self.h, self.d_h, self.d_ff, self.h_kv

        def rnd(*shape):
            return torch.randn(*shape, device="cuda", generator=gen) * 0.02

        fams = FAMILIES if train else ("w",)
        act = B.ACT_SWIGLU if cfg["gated"] else B.ACT_GELU_ERF
        unit = 2 if cfg["rope"] else 1
        num, den = keep
        self.k = ((dh // unit) * num // den, dh * num // den, dff * num // den)
        self.layers = []
        for _ in range(n_layers):
            ly = _Layer()
            names = ["wq", "wk", "wv", "wo", "w1", "w2"] + (["w1b"] if cfg["gated"] else [])
            shapes = {"wq": (h * dh, d), "wk": (hkv * dh, d), "wv": (hkv * dh, d), "wo": (d, h * dh), "w1": (dff, d),
                      "w1b": (dff, d), "w2": (d, dff)}
            bias_shapes = {"bq": h * dh, "bk": hkv * dh, "bv": hkv * dh, "bo": d, "b1": dff, "b2": d} if cfg["bias"] else {}
            init = {n: rnd(*shapes[n]).to(torch.bfloat16) for n in names}
            init.update({n: torch.zeros(s, device="cuda", dtype=torch.bfloat16) for n, s in bias_shapes.items()})
            ly.full, ly.attn, ly.ffn = {}, {}, {}
            for fam in fams:
                if fam == "w":
                    t = {n: rows_aligned(x) for n, x in init.items()}
                elif fam == "mst":
                    t = {n: rows_aligned(x.float()) for n, x in init.items()}
                else:
                    t = {n: rows_aligned(torch.zeros(x.shape, device="cuda")) for n, x in init.items()}
                ly.full[fam] = t
                ly.attn[fam] = AttnBlock(ctx, t["wq"], t["wk"], t["wv"], t["wo"], t.get("bq"), t.get("bk"), t.get("bv"),
                                         t.get("bo"), h, dh, rope=cfg["rope"], causal=True, transposed=(fam == "w" and train),
                                         h_kv=hkv, gather_transposed=False)
                ly.ffn[fam] = FfnBlock(ctx, t["w1"], t.get("b1"), t["w2"], t.get("b2"), act, t.get("w1b"),
                                       transposed=(fam == "w" and train), gather_transposed=False)
                if permanent:
                    ly.attn[fam].track_rotary_blocks()
            ly.idx = [torch.empty((hkv, self.k[0]), dtype=torch.int32, device="cuda"),
                      torch.empty((hkv, self.k[1]), dtype=torch.int32, device="cuda"),
                      torch.empty((1, self.k[2]), dtype=torch.int32, device="cuda")]
            ly.norm = [self._norm_params() for _ in range(2)]
            self.layers.append(ly)
        self.emb = _Param(rnd(vocab, d), train)
        self.pos = None if cfg["rope"] else _Param(rnd(self.L, d), train)
        self.lm = _Param(rnd(vocab, d), train)
        self.norm_f = self._norm_params()
        # the pairs that are scored: the fp32 master weights when they exist, else the working copy
        sf = "mst" if train else "w"
        self.pairs = [p for ly in self.layers for p in ly.attn[sf].pairs() + [ly.ffn[sf].pair()]]
        self.pair_arr = (B.Pair * len(self.pairs))(*self.pairs)
        self.scores = None
        self.compacted = False
        self.prune()
        if permanent:
            self._rebase()
        for ly in self.layers:
            ly.attn["w"].alloc(self.Bsz, self.L)
            ly.ffn["w"].alloc(self.Bsz, self.L)
        self._alloc_glue()
        if train:
            self._build_optimizer()

    # ---- glue ---------------------------------------------------------------------------------------
    def _norm_params(self):
        ps = [_Param(torch.ones(self.d, device="cuda"), self.train)]
        if not self.rms:
            ps.append(_Param(torch.zeros(self.d, device="cuda"), self.train))
        return ps

    def _alloc_glue(self):
        """Activations of the glue, allocated once: per normalisation its input (the residual stream at that point), its
        output and its row statistics; the stream's gradient ping-pongs between two buffers."""
        T, d, dev = self.T, self.d, "cuda"
        bf = lambda *shape: torch.empty(shape, dtype=torch.bfloat16, device=dev)
        st = lambda: torch.empty((T,) if self.rms else (T, 2), dtype=torch.float32, device=dev) if self.train else None
        n_norm = 2 * len(self.layers) + 1
        self.x0 = bf(T, d)                                         # embedding output
        keep = n_norm if self.train else 1                          # inference: one buffer serves every normalisation
        self.xs = [bf(T, d) for _ in range(keep)]                  # input of normalisation i (x0 itself for i = 0)
        self.hs = [bf(T, d) for _ in range(keep)]                  # its output
        self.stats = [st() for _ in range(keep)]
        self.logits = bf(T, self.vocab)
        if self.train:
            self.dxa, self.dxb = bf(T, d), bf(T, d)
            self.row_loss = torch.empty(T, dtype=torch.float32, device=dev)
            self.loss = torch.zeros((), dtype=torch.float32, device=dev)
            self.dhf = bf(T, d)

    def _norm_fwd(self, i, ps, x, res):
        """Normalisation i of the stack on x + res -> (the sum, the normalised rows)."""
        j = i if self.train else 0
        kind = B.NORM_RMS if self.rms else B.NORM_LAYER
        x_out = self.xs[j] if res is not None else None
        self.ctx.ecospa_norm_fwd(kind, x, ps[0].w, None if self.rms else ps[1].w, self.eps, self.hs[j], res=res, x_out=x_out,
                                 stat=self.stats[j])
        if res is None:
            self.xs[j] = x
        return self.xs[j], self.hs[j]

    def _norm_bwd(self, i, ps, dy, dres, dx):
        kind = B.NORM_RMS if self.rms else B.NORM_LAYER
        return self.ctx.ecospa_norm_bwd(kind, self.xs[i], ps[0].w, self.stats[i], dy, dx, ps[0].g,
                                        dbias=None if self.rms else ps[1].g, dres=dres)

    # ---- steps 1-3 for the whole stack -----------------------------------------------------------------
    def _descriptors(self):
        """Descriptor arrays of the stack's batched calls, built once: every buffer they name lives as long as the stack."""
        ctx = self.ctx
        fams = FAMILIES if self.train else ("w",)
        self.scores = ctx.ecospa_coupled_score(self.pair_arr)
        sel = [ctx.select_item(s, self.k[i % 3], self.layers[i // 3].idx[i % 3]) for i, s in enumerate(self.scores)]
        gather, back = [], []
        for ly in self.layers:
            for fam in fams:          # compact() with defer=True also sizes the family's compact buffers
                gather += ly.attn[fam].compact(ly.idx[0], ly.idx[1], defer=True) + ly.ffn[fam].compact(ly.idx[2], defer=True)
                if self.train and not self.permanent:
                    back += ly.attn[fam].write_back_items() + ly.ffn[fam].write_back_items()
        tr = [it for ly in self.layers for it in ly.attn["w"].transpose_items() + ly.ffn["w"].transpose_items()]
        self._sel = (B.SelectItem * len(sel))(*sel)
        self._gather = (B.MapItem * len(gather))(*gather)
        self._back = (B.MapItem * len(back))(*back) if back else None
        self._tr = (B.TransposeItem * len(tr))(*tr) if tr else None

    def prune(self):
        """Estimate the importance again and gather the new choice: write the compact state back into the full-size
        arrays (not before the first estimate), score the full-size weights (one call for all pairs of all layers),
        select (one call), gather every family (one call), refresh the transposed copies and the rotary tables."""
        ctx = self.ctx
        assert not (self.permanent and self.compacted), "a stack that removes for good estimates again through shrink()"
        if getattr(self, "_gather", None) is None:
            self._descriptors()
        if self.compacted and self._back is not None:
            ctx.ecospa_compact_batch(self._back)
        ctx.ecospa_coupled_score(self.pair_arr, out=self.scores)
        ctx.ecospa_select_topk_batch(self._sel)
        ctx.ecospa_compact_batch(self._gather)
        self._refresh_transposed()
        if self.cfg["rope"]:      # kept rotary blocks changed: new frequencies (the first tables come with alloc)
            for ly in self.layers:
                a = ly.attn["w"]
                if getattr(a, "cos", None) is not None:
                    a._rope_table(a._L, out=(a.cos, a.sin))
        self.compacted = True

    def _rebase(self):
        """The compact tensors of every family become the blocks' own; the arrays they were gathered from are released."""
        for ly in self.layers:
            for fam in ly.attn:
                ly.attn[fam].rebase()
                ly.ffn[fam].rebase()
            ly.full = None

    def shrink(self, keep):
        """Alg. 1's step for a stack that removes for good: score the compact master weights of every pair, keep
        floor(n * num / den) units of the ORIGINAL n of every pair (no more than are left), gather every family from its
        compact layout into a smaller one (one call each for scores, selection, gathers, transposed copies), rebuild the
        activations, descriptors and optimizer lists for the new widths, and release the larger buffers."""
        assert self.permanent and self.compacted
        num, den = keep
        unit = 2 if self.cfg["rope"] else 1
        k_new = ((self.d_h // unit) * num // den, self.d_h * num // den, self.d_ff * num // den)
        assert all(0 < a <= b for a, b in zip(k_new, self.k)), "the kept counts only fall"
        self.k = k_new
        sf = "mst" if self.train else "w"
        for ly in self.layers:
            ly.idx = [torch.empty((self.h_kv, k_new[0]), dtype=torch.int32, device="cuda"),
                      torch.empty((self.h_kv, k_new[1]), dtype=torch.int32, device="cuda"),
                      torch.empty((1, k_new[2]), dtype=torch.int32, device="cuda")]
        self.pairs = [p for ly in self.layers for p in ly.attn[sf].pairs() + [ly.ffn[sf].pair()]]
        self.pair_arr = (B.Pair * len(self.pairs))(*self.pairs)
        self.compacted = False              # prune() below is a first gather from the blocks' own (compact) tensors
        self._gather = None
        self.prune()
        self._rebase()
        if self.train:
            self._build_optimizer()

    def _refresh_transposed(self):
        if self._tr is not None:
            self.ctx.ecospa_transpose_batch(self._tr)

    def _build_optimizer(self):
        """Two groups of tensors: matrices (decoupled weight decay) and vectors - biases, norm gains - without it."""
        mk, mats, vecs = B.Context.adamw_item, [], []
        for ly in self.layers:
            for blk, names in ((ly.attn, (("wqkv_c", "dwqkv_c"), ("wo_c", "dwo_c"), ("bqkv_c", "dbqkv_c"), ("bo", "dbo"))),
                               (ly.ffn, (("w1_c", "dw1_c"), ("w2_c", "dw2_c"), ("b1_c", "db1_c"), ("b2", "db2")))):
                for name, grad in names:
                    if getattr(blk["w"], name) is not None:
                        (mats if name.startswith("w") else vecs).append(
                            mk(getattr(blk["mst"], name), getattr(blk["w"], grad), getattr(blk["m"], name),
                               getattr(blk["v"], name), getattr(blk["w"], name)))
            vecs += [p.item() for ps in ly.norm for p in ps]
        vecs += [p.item() for p in self.norm_f]
        mats += [self.emb.item(), self.lm.item()] + ([] if self.pos is None else [self.pos.item()])
        self.opt_mats, self.opt_vecs = (B.AdamwItem * len(mats))(*mats), (B.AdamwItem * len(vecs))(*vecs)
        self.n_params = sum(int(it.n) for it in mats + vecs)

    # ---- forward / backward / update -------------------------------------------------------------------------
    @torch.no_grad()
    def forward(self, ids: torch.Tensor, lm_head: bool = True):
        """ids: int64 [B*L] -> logits bf16 [B*L, vocab] (or the final hidden states with lm_head=False)."""
        ctx = self.ctx
        x = ctx.ecospa_embed_fwd(ids, self.emb.w, self.x0, pos=None if self.pos is None else self.pos.w)
        res = None                       # the block output that the next normalisation adds to the stream first
        for li, ly in enumerate(self.layers):
            x, ly.h1 = self._norm_fwd(2 * li, ly.norm[0], x, res)
            res = ly.attn["w"].fwd(ly.h1, save=self.train)
            x, ly.h2 = self._norm_fwd(2 * li + 1, ly.norm[1], x, res)
            res = ly.ffn["w"].fwd(ly.h2, save=self.train)
        _, self.hf = self._norm_fwd(2 * len(self.layers), self.norm_f, x, res)
        if not lm_head:
            return self.hf
        ctx.ecospa_contract(self.hf, False, self.lm.w, False, splits=1, out=self.logits)
        return self.logits

    @torch.no_grad()
    def backward(self, ids: torch.Tensor, targets: torch.Tensor):
        """Mean cross-entropy of the last forward's logits against targets; fills every gradient buffer.  The logits
        buffer holds their gradient afterwards."""
        ctx, nl = self.ctx, len(self.layers)
        ctx.ecospa_xent(self.logits, targets, self.row_loss, self.loss, dlogits=self.logits)
        dl = self.logits
        ctx.ecospa_contract(dl, True, self.hf, True, splits=1, out=self.lm.g)         # dW = dlogits^T h
        ctx.ecospa_contract(dl, False, self.lm.w, True, splits=1, out=self.dhf)       # dh = dlogits W
        dx, spare = self._norm_bwd(2 * nl, self.norm_f, self.dhf, None, self.dxa), self.dxb
        for li in reversed(range(nl)):
            ly = self.layers[li]
            dh2 = ly.ffn["w"].bwd(ly.h2, dx)
            dx, spare = self._norm_bwd(2 * li + 1, ly.norm[1], dh2, dx, spare), dx
            dh1 = ly.attn["w"].bwd(ly.h1, dx)
            dx, spare = self._norm_bwd(2 * li, ly.norm[0], dh1, dx, spare), dx
        ctx.ecospa_embed_bwd(ids, dx, self.emb.g, dpos=None if self.pos is None else self.pos.g)
        return self.loss

    def update(self):
        """AdamW on every compact tensor and glue parameter (fp32 masters and moments, bf16 working copies written by
        the same kernel), then the transposed copies the backward contractions read."""
        self.t += 1
        self.ctx.ecospa_adamw(self.opt_mats, self.t, self.lr, weight_decay=self.wd)
        self.ctx.ecospa_adamw(self.opt_vecs, self.t, self.lr, weight_decay=0.0)
        self._refresh_transposed()

    def train_step(self, ids, targets):
        self.forward(ids)
        loss = self.backward(ids, targets)
        self.update()
        return loss
