"""Thin helpers that chain the C-ABI calls for one block: score -> select -> compact -> fwd/bwd.

They only allocate tensors, fill descriptor structs and call :class:`binding.Context`; all
arithmetic happens in the library.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


def rows_aligned(t: torch.Tensor) -> torch.Tensor:
    """The same matrix with its leading dimension padded to a multiple of 32 elements, so that every row starts on a
    16-byte boundary whatever the dtype: the score, gather and transpose kernels then move 16 bytes per lane (an inner
    width such as d_ff = 5461 otherwise puts W_down on their element-wise paths)."""
    if t.dim() != 2 or t.shape[1] % 32 == 0:
        return t
    buf = torch.zeros((t.shape[0], B.round_up(t.shape[1], 32)), dtype=t.dtype, device=t.device)
    buf[:, :t.shape[1]] = t
    return buf[:, :t.shape[1]]


class FfnBlock:
    """Compacted FFN pair (W_in / W_out, or W_gate (.) W_up / W_down)."""

    def __init__(self, ctx: B.Context, w1, b1, w2, b2, act: int, w1b=None, transposed: bool = False,
                 bias_grads: Optional[bool] = None, w2_rows: bool = False, gather_transposed: bool = True):
        """w2_rows: the second matrix is stored with its units as rows, [n, d] (the orientation of B in App. A.1; how
        GPT-2 checkpoints keep W_out): it is then scored along rows and its kept units are gathered as rows into the
        transposed compact copy, from which the [d, kp] matrix of the forward pass is written by a transposing copy -
        no column gather anywhere.  transposed: keep transposed copies of the compact matrices for the backward pass (refreshed by
        :meth:`compact`; after a parameter update call :meth:`refresh_transposed`).  bias_grads: ask the backward pass
        for the bias gradients (default: for the biases the block has; True: all of them - they are column sums of the
        upstream gradients and exist with or without a bias).  gather_transposed: row gathers write the transposed
        copy of their result themselves (one launch for a compaction) instead of leaving it to a transposing copy
        afterwards (:meth:`post_gather_items` then lists only what is left)."""
        self.ctx, self.act = ctx, act
        self.gather_transposed = gather_transposed
        self.bias_grads = bias_grads
        self.transposed = transposed
        self.w1, self.b1, self.w2, self.b2, self.w1b = w1, b1, w2, b2, w1b
        self.w2_rows = w2_rows
        self.n, self.d = w1.shape
        self.gated = act == B.ACT_SWIGLU
        self.idx = None
        self.rebased = False      # True: the block's own tensors are views of its compact ones (see rebase)

    def pair(self) -> B.Pair:
        kind = B.PAIR_FFN_GATED if self.gated else B.PAIR_FFN
        return B.Context.make_pair(kind, self.w1, self.w2, 1, self.n, 1, self.w1b, w2_rows=self.w2_rows)

    def score(self) -> torch.Tensor:
        return self.ctx.ecospa_coupled_score([self.pair()])[0]

    def compact(self, idx: torch.Tensor, defer: bool = False, k_group: Optional[torch.Tensor] = None,
                k_max: Optional[int] = None):
        """Gather the kept rows/columns named by idx[1, k] into the padded compact layout (one launch).
        With defer=True the gather descriptors are returned instead, for a larger batch.  With k_group
        (int32[1] on the device, the kept count of the cumulative-threshold rule) only the first k_group[0]
        entries of idx[1, n] count; the count stays on the device, so the caller names an upper bound k_max
        (>= k_group[0]) that sizes the compact matrices - units beyond it would be dropped.
        A call that changes the padded width after :meth:`alloc` allocates the block's buffers again."""
        c = self.ctx
        if k_group is not None and k_max is None:
            raise ValueError("ragged compaction needs k_max: the kept count lives on the device")
        k = idx.shape[1] if k_group is None else int(k_max)
        self.idx, self.k, self.k_group = idx, k, k_group
        # padded width: a multiple of the contraction kernels' slab depth (64) once that costs little, so that the
        # contractions over the kept units (the second FFN matrix, the input gradient) can take the pipelined kernel
        self.kp = kp = B.round_up(k, 64 if k >= 512 else 16)
        nh = 2 * kp if self.gated else kp
        dt, dev = self.w1.dtype, self.w1.device
        assert k_group is None or not self.rebased, "a block that was rebased shrinks by fixed counts"
        resized = getattr(self, "w1_c", None) is None or self.w1_c.shape[0] != nh or self.rebased
        if resized:     # buffers are reused across re-compactions of the same width (never the ones a rebased block reads)
            self.w1_c = torch.empty((nh, self.d), dtype=dt, device=dev)
            self.b1_c = None if self.b1 is None else torch.zeros((nh,), dtype=dt, device=dev)
            self.w2_c = torch.empty((self.d, kp), dtype=dt, device=dev)
            if self.transposed:
                self.w1_t = torch.empty((self.d, nh), dtype=dt, device=dev)
            if self.transposed or self.w2_rows:
                self.w2_t = torch.empty((kp, self.d), dtype=dt, device=dev)
            if getattr(self, "_alloc_shape", None) is not None:     # descriptors, saved activations, gradients follow the new width
                self.alloc(*self._alloc_shape)
        items = self._map_items(0)
        if defer:
            return items
        c.ecospa_compact_batch(items)
        post = self.post_gather_items()
        if post:
            c.ecospa_transpose_batch(post)
        return self

    def post_gather_items(self):
        """Transposing copies that complete a gather: the transposed copies for the backward pass, and - with the
        second matrix stored units-as-rows - its [d, kp] form for the forward pass out of the gathered rows."""
        items = []
        fused = self.gather_transposed
        if self.transposed and not fused:
            items.append(B.Context.transpose_item(self.w1_c, self.w1_t))
        if self.w2_rows:
            if not fused:
                items.append(B.Context.transpose_item(self.w2_t, self.w2_c))
        elif self.transposed:
            items.append(B.Context.transpose_item(self.w2_c, self.w2_t))
        return items

    def rebase(self):
        """Alg. 1's removal for good: the compact tensors become the block's own and what they were gathered from is
        let go (its memory is free once the caller drops its references too).  The next :meth:`compact` then takes
        indices into the present compact layout (positions 0 .. k-1 of the kept units, in order) and gathers into
        fresh buffers; padding units have zero weights, score zero and are never kept.  No write-back exists from here on."""
        kp = self.kp
        self.w1 = self.gate_rows(self.w1_c)
        self.w1b = self.up_rows(self.w1_c) if self.gated else None
        if self.b1 is not None:
            self.b1 = self.b1_c.view(kp, 2)[:, 0] if self.gated else self.b1_c
        self.w2 = self.w2_t if self.w2_rows else self.w2_c
        self.n = kp
        self.rebased = True
        return self

    def gate_rows(self, t: torch.Tensor) -> torch.Tensor:
        """The gate (or only) half of a tensor laid out like the compact first matrix or its bias: the gated block keeps
        gate unit i in row 2i and up unit i in row 2i + 1, so that one output tile of the first contraction holds whole
        (gate, up) pairs."""
        return t[0::2] if self.gated else t

    def up_rows(self, t: torch.Tensor) -> torch.Tensor:
        return t[1::2]

    def _map_items(self, scatter: int):
        """Descriptors between every full-size member and its compact counterpart: gathers (0) or scatters (1, 2)."""
        kp = self.kp
        fused = self.gather_transposed and not scatter      # gathers that write their transposed copies themselves
        # (full-size tensor, compact tensor, axis, transposed copy of the compact tensor, second interleaved source)
        if self.gated and fused and self.transposed:        # (gate, up) row pairs out of both matrices in one copy
            members = [(self.w1, self.w1_c, 0, self.w1_t, self.w1b)]
        else:
            members = [(self.w1, self.gate_rows(self.w1_c), 0, self.w1_t if fused and self.transposed and not self.gated else None, None)]
            if self.gated:
                members.append((self.w1b, self.up_rows(self.w1_c), 0, None, None))
        if self.b1 is not None:       # the up branch of a gated FFN has no bias: its slots stay zero
            if self.gated:            # every second slot: a [kp, 1] matrix with a row pitch of 2
                members.append((self.b1.view(-1, 1), self.b1_c.view(kp, 2)[:, :1], 0, None, None))
            else:
                members.append((self.b1, self.b1_c, 1, None, None))
        members.append((self.w2, self.w2_t, 0, self.w2_c if fused else None, None) if self.w2_rows else (self.w2, self.w2_c, 1, None, None))
        return [B.Context.map_item(c if scatter else f, f if scatter else c, self.idx, axis, 1, self.n, 1, kp,
                                   scatter=scatter, k_group=self.k_group, dst_t=ct, src_b=fb) for f, c, axis, ct, fb in members]

    def write_back_items(self):
        """Scatters of the compact tensors into the full-size ones that leave the pruned rows/columns as they are."""
        assert not self.rebased, "no full-size tensors to write back to"
        assert not self.w2_rows or self.transposed, "rows of the second matrix come from its transposed copy: keep it fresh (transposed=True)"
        return self._map_items(2)

    def transpose_items(self):
        """Transposed copies out of the compact matrices (after a parameter update)."""
        if not self.transposed:
            return []
        return [B.Context.transpose_item(self.w1_c, self.w1_t), B.Context.transpose_item(self.w2_c, self.w2_t)]

    def refresh_transposed(self):
        if self.transposed:
            self.ctx.ecospa_transpose_batch(self.transpose_items())

    def desc(self, Bsz: int, L: int) -> B.BlockDesc:
        d = B.BlockDesc()
        d.block, d.dtype, d.B, d.L, d.d_model = B.BLOCK_FFN, B.dtype_code(self.w1.dtype), Bsz, L, self.d
        d.kp_ff, d.act = self.kp, self.act
        if self.transposed:
            d.w_1_t, d.w_2_t, d.ld_w1t, d.ld_w2t = self.w1_t.data_ptr(), self.w2_t.data_ptr(), self.w1_t.stride(0), self.w2_t.stride(0)
        d.w_1, d.b_1 = self.w1_c.data_ptr(), B._ptr(self.b1_c)
        d.w_2, d.b_2 = self.w2_c.data_ptr(), B._ptr(self.b2)
        d.ld_w1, d.ld_w2 = self.w1_c.stride(0), self.w2_c.stride(0)
        return d

    def alloc(self, Bsz: int, L: int):
        T, dt, dev = Bsz * L, self.w1.dtype, self.w1.device
        nh = 2 * self.kp if self.gated else self.kp
        self._alloc_shape = (Bsz, L)
        self.hpre = torch.empty((T, nh), dtype=dt, device=dev)
        self.act_buf = torch.empty((T, self.kp), dtype=dt, device=dev)
        self.saved = B.Saved(None, None, None, self.hpre.data_ptr(), self.act_buf.data_ptr())
        self.y = torch.empty((T, self.d), dtype=dt, device=dev)
        self.dx = torch.empty((T, self.d), dtype=dt, device=dev)
        self.dw1_c = torch.empty_like(self.w1_c)
        self.dw2_c = torch.empty_like(self.w2_c)
        # bias gradients only for the biases the block has (a missing pointer tells the library to skip the sums)
        want1 = self.b1 is not None if self.bias_grads is None else self.bias_grads
        want2 = self.b2 is not None if self.bias_grads is None else self.bias_grads
        self.db1_c = torch.empty((nh,), dtype=dt, device=dev) if want1 else None
        self.db2 = torch.empty((self.d,), dtype=dt, device=dev) if want2 else None
        g = B.Grads()
        g.dw_1, g.db_1, g.dw_2, g.db_2 = (B._ptr(t) for t in (self.dw1_c, self.db1_c, self.dw2_c, self.db2))
        g.ld_dw1, g.ld_dw2 = self.dw1_c.stride(0), self.dw2_c.stride(0)
        self.grads = g
        self._desc = self.desc(Bsz, L)
        return self

    def fwd(self, x, save: bool = True):
        """save=False: forward only - the library keeps nothing for a backward pass (intermediates live in its
        workspace, the activation's input is not written at all)."""
        return self.ctx.ecospa_coupled_fwd(self._desc, x, self.y, self.saved if save else None)

    def bwd(self, x, dy):
        self.ctx.ecospa_coupled_bwd(self._desc, x, dy, self.saved, self.dx, self.grads)
        return self.dx


class AttnBlock:
    """Compacted attention block: per-head W_q/W_k pairs and W_v/W_o pairs (Eq. 4), optional RoPE.
    With h_kv < h (grouped-query attention, Eq. 5) W_k and W_v hold h_kv heads, and the h / h_kv query heads
    (and heads of W_o) of a group keep the inner dimensions of the key/value head they share."""

    def __init__(self, ctx: B.Context, wq, wk, wv, wo, bq, bk, bv, bo, h: int, d_h: int, *, rope: bool,
                 causal: bool = True, rope_base: float = 10000.0, h_kv: Optional[int] = None, transposed: bool = False,
                 bias_grads: Optional[bool] = None, wo_rows: bool = False, gather_transposed: bool = True):
        """bias_grads: ask the backward pass for the bias gradients (default: for the biases the block has).
        wo_rows: W_o is stored with its units as rows, [h * d_h, d]; gather_transposed: row gathers write their
        transposed copies themselves (see FfnBlock)."""
        self.ctx, self.h, self.d_h, self.rope, self.causal, self.rope_base = ctx, h, d_h, rope, causal, rope_base
        self.gather_transposed = gather_transposed
        self.bias_grads = bias_grads
        self.transposed = transposed      # transposed copies of the compact matrices for the backward pass
        self.h_kv = h if h_kv is None else h_kv
        assert h % self.h_kv == 0
        self.qpk = h // self.h_kv
        self.wq, self.wk, self.wv, self.wo = wq, wk, wv, wo
        self.wo_rows = wo_rows
        self.bq, self.bk, self.bv, self.bo = bq, bk, bv, bo
        self.d = wq.shape[1]
        self.unit = 2 if rope else 1
        self.n_qk = self.n_vo = d_h     # inner width per head of the tensors the block gathers from (d_h until rebase)
        self.rebased = False
        self.orig_qk = None             # rebased: original rotary block of every unit the block gathers from, int32 [h_kv, units]

    def pairs(self):
        mk = B.Context.make_pair
        return [mk(B.PAIR_QK, self.wq, self.wk, self.h_kv, self.n_qk, self.unit, rep1=self.qpk),
                mk(B.PAIR_VO, self.wv, self.wo, self.h_kv, self.n_vo, 1, rep2=self.qpk, w2_rows=self.wo_rows)]

    def track_rotary_blocks(self):
        """Before the first :meth:`compact` of a block that will be rebased: keep, beside the index lists, the original
        rotary block of every kept unit - the frequencies of Eq. 6 belong to the original positions, however often the
        block shrinks."""
        if self.rope and self.orig_qk is None:
            n_units = self.n_qk // self.unit
            self.orig_qk = torch.arange(n_units, dtype=torch.int32, device=self.wq.device).repeat(self.h_kv, 1).contiguous()
        return self

    def score(self):
        return self.ctx.ecospa_coupled_score(self.pairs())

    def compact(self, idx_qk: torch.Tensor, idx_vo: torch.Tensor, defer: bool = False,
                k_qk_group: Optional[torch.Tensor] = None, k_vo_group: Optional[torch.Tensor] = None,
                k_qk_max: Optional[int] = None, k_vo_max: Optional[int] = None):
        """Gather the kept dimensions.  With k_qk_group / k_vo_group (int32[h] on the device, the kept counts of the
        cumulative-threshold rule) every head keeps a count of its own: idx_* are then [h, n_units] lists whose first
        k_*_group[g] entries count, and all heads are padded with zeros to k_qk_max units / k_vo_max dimensions - upper
        bounds on the counts that the caller names (the counts stay on the device; units beyond the bound would be dropped).
        A call that changes a padded width after :meth:`alloc` allocates the block's buffers and tables again."""
        c, h, hk, u = self.ctx, self.h, self.h_kv, self.unit
        if (k_qk_group is not None and k_qk_max is None) or (k_vo_group is not None and k_vo_max is None):
            raise ValueError("ragged compaction needs k_qk_max / k_vo_max: the kept counts live on the device")
        self.idx_qk, self.idx_vo = idx_qk, idx_vo
        self.k_qk_group, self.k_vo_group = k_qk_group, k_vo_group
        self.k_qk_units = idx_qk.shape[1] if k_qk_group is None else int(k_qk_max)
        self.k_vo = idx_vo.shape[1] if k_vo_group is None else int(k_vo_max)
        self.kp_qk = B.round_up(self.k_qk_units * u, 16)
        self.kp_vo = B.round_up(self.k_vo, 16)
        # compact layout: the h query heads, then the h_kv key heads, then the h_kv value heads; W_o has h heads
        nq, nk, nv, no = h * self.kp_qk, hk * self.kp_qk, hk * self.kp_vo, h * self.kp_vo
        self.nq, self.nk = nq, nk
        dt, dev = self.wq.dtype, self.wq.device
        assert (k_qk_group is None and k_vo_group is None) or not self.rebased, "a block that was rebased shrinks by fixed counts"
        resized = (getattr(self, "wqkv_c", None) is None or self.wqkv_c.shape[0] != nq + nk + nv
                   or self.wo_c.shape[1] != no or self.rebased)
        if self.orig_qk is not None:    # original rotary blocks of the kept units: gathered like everything else
            self.rope_idx = torch.empty((hk, self.k_qk_units), dtype=torch.int32, device=dev)
        if resized:
            self.wqkv_c = torch.empty((nq + nk + nv, self.d), dtype=dt, device=dev)
            self.bqkv_c = None if self.bq is None else torch.empty((nq + nk + nv,), dtype=dt, device=dev)
            self.wo_c = torch.empty((self.d, no), dtype=dt, device=dev)
            if self.transposed:
                self.wqkv_t = torch.empty((self.d, nq + nk + nv), dtype=dt, device=dev)
            if self.transposed or self.wo_rows:
                self.wo_t = torch.empty((no, self.d), dtype=dt, device=dev)
        items = self._map_items(0)
        if not defer:
            c.ecospa_compact_batch(items)
            post = self.post_gather_items()
            if post:
                c.ecospa_transpose_batch(post)
        if getattr(self, "_alloc_shape", None) is not None:
            if resized:       # descriptors, saved activations, gradients and the rotary tables follow the new widths
                self.alloc(*self._alloc_shape)
            elif self.rope:   # same widths, but the kept blocks may have changed: new frequencies in place
                self._rope_table(self._L, out=(self.cos, self.sin))
        return items if defer else self

    def _map_items(self, scatter: int):
        """Descriptors between every full-size member and its compact counterpart: gathers (0) or scatters (1, 2)."""
        h, hk, u = self.h, self.h_kv, self.unit
        nq, nk, kpu = self.nq, self.nk, self.kp_qk // u

        fused = self.gather_transposed and not scatter      # gathers that write their transposed copies themselves

        def mq(full, cmp, axis, heads, cmp_t=None):      # heads that share an index list with (heads // h_kv - 1) others
            return B.Context.map_item(cmp if scatter else full, full if scatter else cmp, self.idx_qk, axis, heads, self.n_qk, u, kpu,
                                      scatter=scatter, k_group=self.k_qk_group, idx_div=heads // hk, dst_t=cmp_t)

        def mv(full, cmp, axis, heads, cmp_t=None):
            return B.Context.map_item(cmp if scatter else full, full if scatter else cmp, self.idx_vo, axis, heads, self.n_vo, 1,
                                      self.kp_vo, scatter=scatter, k_group=self.k_vo_group, idx_div=heads // hk, dst_t=cmp_t)

        qkv_t = self.wqkv_t if fused and self.transposed else None      # [d, nq + nk + nv]: every member writes its columns
        col = lambda a, b: None if qkv_t is None else qkv_t[:, a:b]
        items = [mq(self.wq, self.wqkv_c[:nq], 0, h, col(0, nq)), mq(self.wk, self.wqkv_c[nq:nq + nk], 0, hk, col(nq, nq + nk)),
                 mv(self.wv, self.wqkv_c[nq + nk:], 0, hk, col(nq + nk, None))]
        if self.bq is not None:
            items += [mq(self.bq, self.bqkv_c[:nq], 1, h), mq(self.bk, self.bqkv_c[nq:nq + nk], 1, hk),
                      mv(self.bv, self.bqkv_c[nq + nk:], 1, hk)]
        items.append(mv(self.wo, self.wo_t, 0, h, self.wo_c if fused else None) if self.wo_rows else mv(self.wo, self.wo_c, 1, h))
        if self.orig_qk is not None and not scatter:      # the int32 table moves as 4-byte words
            items.append(B.Context.map_item(self.orig_qk.view(torch.float32).view(-1), self.rope_idx.view(torch.float32).view(-1),
                                            self.idx_qk, 1, hk, self.orig_qk.shape[1], 1, self.k_qk_units))
        return items

    def write_back_items(self):
        """Scatters of the compact tensors into the full-size ones that leave the pruned rows/columns as they are."""
        assert not self.rebased, "no full-size tensors to write back to"
        assert not self.wo_rows or self.transposed, "rows of W_o come from its transposed copy: keep it fresh (transposed=True)"
        return self._map_items(2)

    def post_gather_items(self):
        """Transposing copies that complete a gather (see FfnBlock.post_gather_items)."""
        items = []
        fused = self.gather_transposed
        if self.transposed and not fused:
            items.append(B.Context.transpose_item(self.wqkv_c, self.wqkv_t))
        if self.wo_rows:
            if not fused:
                items.append(B.Context.transpose_item(self.wo_t, self.wo_c))
        elif self.transposed:
            items.append(B.Context.transpose_item(self.wo_c, self.wo_t))
        return items

    def rebase(self):
        """Alg. 1's removal for good: the compact tensors become the block's own and what they were gathered from is
        let go.  The next :meth:`compact` takes indices into the present compact layout of every head (positions
        0 .. k-1 of its kept units, in order) and gathers into fresh buffers; padding units have zero weights and are
        never kept.  The attention scale and the rotary frequencies stay those of the original head width and block
        positions (call :meth:`track_rotary_blocks` before the first compaction).  No write-back from here on."""
        assert self.k_qk_group is None and self.k_vo_group is None, "fixed kept counts only"
        assert not self.rope or self.orig_qk is not None, "track_rotary_blocks() before the first compaction"
        nq, nk = self.nq, self.nk
        self.wq, self.wk, self.wv = self.wqkv_c[:nq], self.wqkv_c[nq:nq + nk], self.wqkv_c[nq + nk:]
        self.wo = self.wo_t if self.wo_rows else self.wo_c
        if self.bq is not None:
            self.bq, self.bk, self.bv = self.bqkv_c[:nq], self.bqkv_c[nq:nq + nk], self.bqkv_c[nq + nk:]
        self.n_qk, self.n_vo = self.kp_qk, self.kp_vo
        if self.rope:
            self.orig_qk = self.rope_idx
        self.rebased = True
        return self

    def transpose_items(self):
        if not self.transposed:
            return []
        return [B.Context.transpose_item(self.wqkv_c, self.wqkv_t), B.Context.transpose_item(self.wo_c, self.wo_t)]

    def refresh_transposed(self):
        if self.transposed:
            self.ctx.ecospa_transpose_batch(self.transpose_items())

    def _rope_table(self, L: int, out=None):
        if self.k_qk_group is not None:
            return self.ctx.ecospa_rope_table_ragged(self.idx_qk, self.k_qk_group, L, self.kp_qk // 2, self.d_h,
                                                     self.rope_base, out=out)
        blocks = self.idx_qk if self.orig_qk is None else self.rope_idx      # original block positions of the kept units
        return self.ctx.ecospa_rope_table(blocks, self.h_kv, L, self.k_qk_units, self.kp_qk // 2, self.d_h,
                                          self.rope_base, out=out)

    def rope_item(self):
        """The block's rotary tables as a descriptor for :meth:`Context.ecospa_compact_batch` (after :meth:`alloc`): the
        gather launch of a re-compaction then refreshes them itself.  None for a block without rotary embedding."""
        if not self.rope:
            return None
        h, kp = self.cos.shape[0], self.cos.shape[2]
        if self.k_qk_group is not None:
            return B.Context.rope_item(self.idx_qk, h, self._L, 0, kp, self.d_h, self.rope_base, self.cos, self.sin,
                                       k_group=self.k_qk_group)
        blocks = self.idx_qk if self.orig_qk is None else self.rope_idx
        return B.Context.rope_item(blocks, h, self._L, self.k_qk_units, kp, self.d_h, self.rope_base, self.cos, self.sin)

    def alloc(self, Bsz: int, L: int):
        c, h = self.ctx, self.h
        T, dt, dev = Bsz * L, self.wq.dtype, self.wq.device
        nqkv, nv = self.wqkv_c.shape[0], h * self.kp_vo
        self.cos = self.sin = None
        self._L = L
        self._alloc_shape = (Bsz, L)
        if self.rope:
            self.cos, self.sin = self._rope_table(L)
        d = B.BlockDesc()
        d.block, d.dtype, d.B, d.L, d.d_model = B.BLOCK_ATTN, B.dtype_code(dt), Bsz, L, self.d
        d.h, d.kp_qk, d.kp_vo, d.causal = h, self.kp_qk, self.kp_vo, int(self.causal)
        d.h_kv = self.h_kv
        if self.transposed:
            d.w_qkv_t, d.w_o_t = self.wqkv_t.data_ptr(), self.wo_t.data_ptr()
            d.ld_wqkvt, d.ld_wot = self.wqkv_t.stride(0), self.wo_t.stride(0)
        d.scale = float(self.d_h) ** -0.5
        d.rope_cos, d.rope_sin = B._ptr(self.cos), B._ptr(self.sin)
        d.w_qkv, d.b_qkv, d.w_o, d.b_o = self.wqkv_c.data_ptr(), B._ptr(self.bqkv_c), self.wo_c.data_ptr(), B._ptr(self.bo)
        d.ld_wqkv, d.ld_wo = self.wqkv_c.stride(0), self.wo_c.stride(0)
        self._desc = d
        self.qkv = torch.empty((T, nqkv), dtype=dt, device=dev)
        self.o = torch.empty((T, nv), dtype=dt, device=dev)
        self.lse = torch.empty((Bsz * h * L,), dtype=torch.float32, device=dev)
        self.saved = B.Saved(self.qkv.data_ptr(), self.o.data_ptr(), self.lse.data_ptr(), None, None)
        self.y = torch.empty((T, self.d), dtype=dt, device=dev)
        self.dx = torch.empty((T, self.d), dtype=dt, device=dev)
        self.dwqkv_c = torch.empty_like(self.wqkv_c)
        want_qkv = self.bq is not None if self.bias_grads is None else self.bias_grads
        want_o = self.bo is not None if self.bias_grads is None else self.bias_grads
        self.dbqkv_c = torch.empty((nqkv,), dtype=dt, device=dev) if want_qkv else None
        self.dwo_c = torch.empty_like(self.wo_c)
        self.dbo = torch.empty((self.d,), dtype=dt, device=dev) if want_o else None
        g = B.Grads()
        g.dw_qkv, g.db_qkv, g.dw_o, g.db_o = (B._ptr(t) for t in (self.dwqkv_c, self.dbqkv_c, self.dwo_c, self.dbo))
        g.ld_dwqkv, g.ld_dwo = self.dwqkv_c.stride(0), self.dwo_c.stride(0)
        self.grads = g
        return self

    def fwd(self, x, save: bool = True):
        """save=False: forward only - Q, K, V, the attention output and the row statistics live in the workspace."""
        return self.ctx.ecospa_coupled_fwd(self._desc, x, self.y, self.saved if save else None)

    def bwd(self, x, dy):
        self.ctx.ecospa_coupled_bwd(self._desc, x, dy, self.saved, self.dx, self.grads)
        return self.dx
