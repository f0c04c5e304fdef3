"""ctypes binding of ``libecospa.so`` (see ``include/ecospa.h``).

Argument marshalling only: every step runs in the library's HIP kernels.  PyTorch supplies
device memory (tensors) and the HIP stream.  There is no fallback: if the built library is
missing, :func:`load` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libecospa.so")

OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_K, ERR_INDEX, ERR_WORKSPACE, ERR_ALIGN, ERR_HIP = range(9)
F32, BF16 = 0, 1
PAIR_QK, PAIR_VO, PAIR_FFN, PAIR_FFN_GATED = range(4)
BLOCK_ATTN, BLOCK_FFN = 0, 1
ACT_GELU_ERF, ACT_GELU_TANH, ACT_SWIGLU = range(3)

EXPORTS = (
    "ecospa_create", "ecospa_destroy", "ecospa_set_workspace", "ecospa_status_string", "ecospa_last_error",
    "ecospa_score_workspace_bytes", "ecospa_coupled_score", "ecospa_select_topk", "ecospa_compact",
    "ecospa_scatter", "ecospa_rope_table", "ecospa_block_workspace_bytes", "ecospa_coupled_fwd",
    "ecospa_coupled_bwd", "ecospa_profile_gemm", "ecospa_profile_gemm_read", "ecospa_contract",
    "ecospa_select_topk_batch", "ecospa_compact_batch", "ecospa_pair_fisher", "ecospa_select_theta",
    "ecospa_select_pairs", "ecospa_rope_table_ragged", "ecospa_adamw", "ecospa_transpose_batch",
    "ecospa_check_indices", "ecospa_contract_workspace_bytes", "ecospa_hbm_probe", "ecospa_contract_colsum", "ecospa_mfma_probe",
    "ecospa_coupled_score_static", "ecospa_coupled_score_static_max_bytes",
    "ecospa_score_select", "ecospa_compact_batch_rope",
    "ecospa_norm_fwd", "ecospa_norm_bwd", "ecospa_norm_bwd_workspace_bytes", "ecospa_embed_fwd", "ecospa_embed_bwd", "ecospa_xent",
)
NORM_RMS, NORM_LAYER = 0, 1


class EcospaError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: error {code} ({status_string(code)}) {detail}".strip())


class Pair(C.Structure):
    _fields_ = [("kind", C.c_int), ("dtype", C.c_int), ("groups", C.c_int), ("n", C.c_int), ("unit", C.c_int),
                ("d1", C.c_int), ("d2", C.c_int), ("w1", C.c_void_p), ("w1b", C.c_void_p), ("w2", C.c_void_p),
                ("ld1", C.c_longlong), ("ld1b", C.c_longlong), ("ld2", C.c_longlong), ("rep1", C.c_int), ("rep2", C.c_int),
                ("w2_rows", C.c_int)]


class BlockDesc(C.Structure):
    _fields_ = [("block", C.c_int), ("dtype", C.c_int), ("B", C.c_int), ("L", C.c_int), ("d_model", C.c_int),
                ("h", C.c_int), ("kp_qk", C.c_int), ("kp_vo", C.c_int), ("causal", C.c_int), ("scale", C.c_float),
                ("rope_cos", C.c_void_p), ("rope_sin", C.c_void_p),
                ("w_qkv", C.c_void_p), ("b_qkv", C.c_void_p), ("w_o", C.c_void_p), ("b_o", C.c_void_p),
                ("ld_wqkv", C.c_longlong), ("ld_wo", C.c_longlong),
                ("kp_ff", C.c_int), ("act", C.c_int),
                ("w_1", C.c_void_p), ("b_1", C.c_void_p), ("w_2", C.c_void_p), ("b_2", C.c_void_p),
                ("ld_w1", C.c_longlong), ("ld_w2", C.c_longlong), ("h_kv", C.c_int),
                ("w_qkv_t", C.c_void_p), ("w_o_t", C.c_void_p), ("w_1_t", C.c_void_p), ("w_2_t", C.c_void_p),
                ("ld_wqkvt", C.c_longlong), ("ld_wot", C.c_longlong), ("ld_w1t", C.c_longlong), ("ld_w2t", C.c_longlong)]


class SelectItem(C.Structure):
    _fields_ = [("scores", C.c_void_p), ("groups", C.c_int), ("n_units", C.c_int), ("k", C.c_int),
                ("idx", C.c_void_p)]


class MapItem(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("dtype", C.c_int), ("axis", C.c_int), ("groups", C.c_int),
                ("n", C.c_int), ("unit", C.c_int), ("k", C.c_int), ("kp", C.c_int), ("scatter", C.c_int),
                ("other_extent", C.c_longlong), ("ld_src", C.c_longlong), ("ld_dst", C.c_longlong),
                ("idx", C.c_void_p), ("k_group", C.c_void_p), ("ld_idx", C.c_int), ("idx_div", C.c_int),
                ("dst_t", C.c_void_p), ("ld_dst_t", C.c_longlong), ("src_b", C.c_void_p)]


class RopeItem(C.Structure):
    _fields_ = [("idx", C.c_void_p), ("k_group", C.c_void_p), ("h", C.c_int), ("L", C.c_int), ("k", C.c_int), ("kp", C.c_int),
                ("d_h", C.c_int), ("ld_idx", C.c_int), ("base", C.c_double), ("cos_out", C.c_void_p), ("sin_out", C.c_void_p)]


class TransposeItem(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("dtype", C.c_int), ("rows", C.c_int), ("cols", C.c_int),
                ("ld_src", C.c_longlong), ("ld_dst", C.c_longlong)]


class AdamwItem(C.Structure):
    _fields_ = [("w", C.c_void_p), ("w_lp", C.c_void_p), ("g", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("n", C.c_longlong), ("w_dtype", C.c_int), ("g_dtype", C.c_int), ("s_dtype", C.c_int)]


class AdamwHyper(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_int)]


class Saved(C.Structure):
    _fields_ = [("qkv", C.c_void_p), ("o", C.c_void_p), ("lse", C.c_void_p), ("hpre", C.c_void_p),
                ("act", C.c_void_p)]


class Grads(C.Structure):
    _fields_ = [("dw_qkv", C.c_void_p), ("db_qkv", C.c_void_p), ("dw_o", C.c_void_p), ("db_o", C.c_void_p),
                ("dw_1", C.c_void_p), ("db_1", C.c_void_p), ("dw_2", C.c_void_p), ("db_2", C.c_void_p),
                ("ld_dwqkv", C.c_longlong), ("ld_dwo", C.c_longlong), ("ld_dw1", C.c_longlong),
                ("ld_dw2", C.c_longlong)]


_lib = None


def load() -> C.CDLL:
    """Load the built library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_11641_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, ci, ll, sz = C.c_void_p, C.c_int, C.c_longlong, C.c_size_t
    lib.ecospa_create.argtypes = [C.POINTER(vp), vp]
    lib.ecospa_create.restype = ci
    lib.ecospa_destroy.argtypes = [vp]
    lib.ecospa_destroy.restype = None
    lib.ecospa_set_workspace.argtypes = [vp, vp, sz]
    lib.ecospa_set_workspace.restype = ci
    lib.ecospa_status_string.argtypes = [ci]
    lib.ecospa_status_string.restype = C.c_char_p
    lib.ecospa_last_error.argtypes = [vp]
    lib.ecospa_last_error.restype = C.c_char_p
    lib.ecospa_score_workspace_bytes.argtypes = [C.POINTER(Pair), ci]
    lib.ecospa_score_workspace_bytes.restype = sz
    lib.ecospa_coupled_score.argtypes = [vp, C.POINTER(Pair), ci, C.POINTER(vp)]
    lib.ecospa_coupled_score.restype = ci
    lib.ecospa_select_topk.argtypes = [vp, vp, ci, ci, ci, vp]
    lib.ecospa_select_topk.restype = ci
    lib.ecospa_pair_fisher.argtypes = [vp, C.POINTER(Pair), ci, C.c_float, C.POINTER(vp)]
    lib.ecospa_pair_fisher.restype = ci
    lib.ecospa_select_theta.argtypes = [vp, vp, ci, ci, C.c_float, vp, vp]
    lib.ecospa_select_theta.restype = ci
    lib.ecospa_select_pairs.argtypes = [vp, vp, ci, ci, vp]
    lib.ecospa_select_pairs.restype = ci
    for f in (lib.ecospa_compact, lib.ecospa_scatter):
        f.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ll, ll, ll, vp]
        f.restype = ci
    lib.ecospa_select_topk_batch.argtypes = [vp, C.POINTER(SelectItem), ci]
    lib.ecospa_select_topk_batch.restype = ci
    lib.ecospa_compact_batch.argtypes = [vp, C.POINTER(MapItem), ci]
    lib.ecospa_compact_batch.restype = ci
    lib.ecospa_compact_batch_rope.argtypes = [vp, C.POINTER(MapItem), ci, C.POINTER(RopeItem)]
    lib.ecospa_compact_batch_rope.restype = ci
    lib.ecospa_rope_table.argtypes = [vp, vp, ci, ci, ci, ci, ci, C.c_double, vp, vp]
    lib.ecospa_rope_table.restype = ci
    lib.ecospa_rope_table_ragged.argtypes = [vp, vp, ci, vp, ci, ci, ci, ci, C.c_double, vp, vp]
    lib.ecospa_rope_table_ragged.restype = ci
    lib.ecospa_transpose_batch.argtypes = [vp, C.POINTER(TransposeItem), ci]
    lib.ecospa_transpose_batch.restype = ci
    lib.ecospa_adamw.argtypes = [vp, C.POINTER(AdamwItem), ci, C.POINTER(AdamwHyper)]
    lib.ecospa_adamw.restype = ci
    lib.ecospa_block_workspace_bytes.argtypes = [C.POINTER(BlockDesc)]
    lib.ecospa_block_workspace_bytes.restype = sz
    lib.ecospa_coupled_fwd.argtypes = [vp, C.POINTER(BlockDesc), vp, vp, C.POINTER(Saved)]
    lib.ecospa_coupled_fwd.restype = ci
    lib.ecospa_coupled_bwd.argtypes = [vp, C.POINTER(BlockDesc), vp, vp, C.POINTER(Saved), vp, C.POINTER(Grads)]
    lib.ecospa_coupled_bwd.restype = ci
    lib.ecospa_profile_gemm.argtypes = [vp, ci]
    lib.ecospa_profile_gemm.restype = ci
    lib.ecospa_profile_gemm_read.argtypes = [vp, C.POINTER(ci), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.ecospa_profile_gemm_read.restype = ci
    lib.ecospa_contract.argtypes = [vp, ci, ci, ci, ci, vp, ll, ci, vp, ll, ci, vp, ll, vp, ci, ci]
    lib.ecospa_contract.restype = ci
    lib.ecospa_check_indices.argtypes = [vp, vp, ci, ci, ci, vp, ci]
    lib.ecospa_check_indices.restype = ci
    lib.ecospa_contract_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.ecospa_contract_workspace_bytes.restype = sz
    lib.ecospa_score_select.argtypes = [vp, C.POINTER(Pair), ci, C.POINTER(vp), C.POINTER(ci), C.POINTER(vp)]
    lib.ecospa_score_select.restype = ci
    lib.ecospa_coupled_score_static.argtypes = [vp, C.POINTER(Pair), ci, C.POINTER(vp)]
    lib.ecospa_coupled_score_static.restype = ci
    lib.ecospa_coupled_score_static_max_bytes.argtypes = []
    lib.ecospa_coupled_score_static_max_bytes.restype = sz
    lib.ecospa_contract_colsum.argtypes = [vp, ci, ci, ci, vp, ll, vp, ll, vp, ll, vp, ci, ci]
    lib.ecospa_contract_colsum.restype = ci
    lib.ecospa_mfma_probe.argtypes = [vp, vp, vp, ci, C.POINTER(C.c_double)]
    lib.ecospa_mfma_probe.restype = ci
    lib.ecospa_hbm_probe.argtypes = [vp, vp, vp, sz, ci]
    lib.ecospa_norm_fwd.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, C.c_float, vp, vp]
    lib.ecospa_norm_fwd.restype = ci
    lib.ecospa_norm_bwd.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ecospa_norm_bwd.restype = ci
    lib.ecospa_norm_bwd_workspace_bytes.argtypes = [ci, ci]
    lib.ecospa_norm_bwd_workspace_bytes.restype = sz
    lib.ecospa_embed_fwd.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, ci, vp]
    lib.ecospa_embed_fwd.restype = ci
    lib.ecospa_embed_bwd.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, ci]
    lib.ecospa_embed_bwd.restype = ci
    lib.ecospa_xent.argtypes = [vp, ci, ci, ci, vp, ll, vp, vp, ll, vp, vp]
    lib.ecospa_xent.restype = ci
    lib.ecospa_hbm_probe.restype = ci
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load().ecospa_status_string(int(code)).decode()


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


class Context:
    """One ecospa_ctx on the current torch stream, with a torch-owned workspace that grows on demand."""

    def __init__(self, device: str = "cuda:0", stream: Optional[torch.cuda.Stream] = None):
        self.lib = load()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        rc = self.lib.ecospa_create(C.byref(h), C.c_void_p(self.stream.cuda_stream))
        if rc:
            raise EcospaError(rc, "ecospa_create")
        self.h = h
        self._ws: Optional[torch.Tensor] = None

    def __del__(self):
        try:
            if getattr(self, "h", None):
                self.lib.ecospa_destroy(self.h)
                self.h = None
        except Exception:
            pass

    def _check(self, rc: int, where: str):
        if rc:
            raise EcospaError(rc, where, self.lib.ecospa_last_error(self.h).decode())

    def reserve(self, nbytes: int):
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=self.device)
            self._check(self.lib.ecospa_set_workspace(self.h, self._ws.data_ptr(), self._ws.numel()),
                        "ecospa_set_workspace")

    def ecospa_profile_gemm(self, enable: bool):
        self._check(self.lib.ecospa_profile_gemm(self.h, int(enable)), "ecospa_profile_gemm")

    def ecospa_profile_gemm_read(self):
        n, ms, fl = C.c_int(), C.c_double(), C.c_double()
        self._check(self.lib.ecospa_profile_gemm_read(self.h, C.byref(n), C.byref(ms), C.byref(fl)),
                    "ecospa_profile_gemm_read")
        return n.value, ms.value, fl.value

    def ecospa_hbm_probe(self, src: torch.Tensor, dst: torch.Tensor, copy: bool):
        """Measurement aid: read src once (copy=False; dst is a small sink) or copy it to dst."""
        nbytes = src.numel() * src.element_size()
        self._check(self.lib.ecospa_hbm_probe(self.h, src.data_ptr(), dst.data_ptr(), nbytes, int(copy)), "ecospa_hbm_probe")

    def ecospa_mfma_probe(self, src: torch.Tensor, sink: torch.Tensor, iters: int) -> float:
        """Measurement aid: launch the pure-MFMA loop on operand bits from src (>= 64 KiB); returns the flops of the launch."""
        assert src.numel() * src.element_size() >= 65536 and sink.dtype == torch.float32 and sink.numel() >= 65536
        fl = C.c_double()
        self._check(self.lib.ecospa_mfma_probe(self.h, src.data_ptr(), sink.data_ptr(), int(iters), C.byref(fl)), "ecospa_mfma_probe")
        return fl.value

    def ecospa_contract(self, A: torch.Tensor, trans_a: bool, Bm: torch.Tensor, trans_b: bool,
                        bias: Optional[torch.Tensor] = None, tile: int = 0, splits: int = 0,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """C[m,n] = sum_k A(m,k) B(n,k) (+ bias[n]); a transposed operand is stored [K, M] / [K, N]."""
        K, M = (A.shape if trans_a else A.shape[::-1])
        K2, N = (Bm.shape if trans_b else Bm.shape[::-1])
        assert K == K2
        if out is None:
            out = torch.empty((M, N), dtype=A.dtype, device=A.device)
        self.reserve(self.lib.ecospa_contract_workspace_bytes(dtype_code(A.dtype), M, N, K, splits))     # fp32 partials of a split contraction
        self._check(self.lib.ecospa_contract(self.h, dtype_code(A.dtype), M, N, K, A.data_ptr(), A.stride(0),
                                             int(trans_a), Bm.data_ptr(), Bm.stride(0), int(trans_b), out.data_ptr(),
                                             out.stride(0), _ptr(bias), tile, splits), "ecospa_contract")
        return out

    def ecospa_contract_colsum(self, A: torch.Tensor, Bm: torch.Tensor, tile: int = 0, splits: int = 0):
        """dY^T X form: A[K, M], Bm[K, N] (bf16) -> (C[M, N] bf16, colsum[M] fp32 = column sums of A)."""
        K, M = A.shape
        K2, N = Bm.shape
        assert K == K2 and A.dtype == torch.bfloat16
        out = torch.empty((M, N), dtype=A.dtype, device=A.device)
        cs = torch.empty((M,), dtype=torch.float32, device=A.device)
        sp = max(splits, 1) if splits else 8
        rows = sp * ((N + 127) // 128)          # at most one row of partial sums per split and 128-wide tile column
        self.reserve(round_up(rows * M * 4, 256) + self.lib.ecospa_contract_workspace_bytes(BF16, M, N, K, splits) + 256)
        self._check(self.lib.ecospa_contract_colsum(self.h, M, N, K, A.data_ptr(), A.stride(0), Bm.data_ptr(), Bm.stride(0),
                                                    out.data_ptr(), out.stride(0), cs.data_ptr(), tile, splits),
                    "ecospa_contract_colsum")
        return out, cs

    # ---- step 1 ------------------------------------------------------------------------------
    @staticmethod
    def make_pair(kind: int, w1: torch.Tensor, w2: torch.Tensor, groups: int, n: int, unit: int = 1,
                  w1b: Optional[torch.Tensor] = None, rep1: int = 1, rep2: int = 1, w2_rows: bool = False) -> Pair:
        """rep1 / rep2: heads of the first / second member that share one group's inner dimensions (Eq. 5).
        w2_rows: the second member of a VO / FFN pair is stored with its units as rows ([units, d])."""
        d1 = w1.shape[1]
        d2 = w2.shape[1] if (kind == PAIR_QK or w2_rows) else w2.shape[0]
        return Pair(kind, dtype_code(w1.dtype), groups, n, unit, d1, d2, _ptr(w1), _ptr(w1b), _ptr(w2),
                    w1.stride(0), 0 if w1b is None else w1b.stride(0), w2.stride(0), rep1, rep2, int(w2_rows))

    def ecospa_coupled_score(self, pairs: Sequence[Pair], out: Optional[Sequence[torch.Tensor]] = None) -> list[torch.Tensor]:
        """Scores of a batch of pairs, one float32 tensor [groups, n/unit] per pair (written into `out` if given)."""
        arr = pairs if isinstance(pairs, C.Array) else (Pair * len(pairs))(*pairs)
        need = self.lib.ecospa_score_workspace_bytes(arr, len(arr))
        self.reserve(need)
        if out is None:
            out = [torch.empty((p.groups, p.n // max(p.unit, 1)), dtype=torch.float32, device=self.device) for p in arr]
        ptrs = (C.c_void_p * len(arr))(*[o.data_ptr() for o in out])
        self._check(self.lib.ecospa_coupled_score(self.h, arr, len(arr), ptrs), "ecospa_coupled_score")
        return list(out)

    def ecospa_score_select(self, pairs: Sequence[Pair], k: Sequence[int], scores: Optional[Sequence[torch.Tensor]] = None,
                            idx: Optional[Sequence[torch.Tensor]] = None):
        """Steps 1 and 2 of a batch of pairs in two launches: (scores, idx) with scores[p] float32 [groups, n/unit] and
        idx[p] int32 [groups, k[p]] (written into the given tensors if any)."""
        arr = pairs if isinstance(pairs, C.Array) else (Pair * len(pairs))(*pairs)
        self.reserve(self.lib.ecospa_score_workspace_bytes(arr, len(arr)))
        if scores is None:
            scores = [torch.empty((p.groups, p.n // max(p.unit, 1)), dtype=torch.float32, device=self.device) for p in arr]
        if idx is None:
            idx = [torch.empty((p.groups, int(kk)), dtype=torch.int32, device=self.device) for p, kk in zip(arr, k)]
        sp = (C.c_void_p * len(arr))(*[o.data_ptr() for o in scores])
        ip = (C.c_void_p * len(arr))(*[o.data_ptr() for o in idx])
        ka = (C.c_int * len(arr))(*[int(kk) for kk in k])
        self._check(self.lib.ecospa_score_select(self.h, arr, len(arr), sp, ka, ip), "ecospa_score_select")
        return list(scores), list(idx)

    def ecospa_coupled_score_static(self, pairs: Sequence[Pair], out: Sequence[torch.Tensor]) -> list[torch.Tensor]:
        """ecospa_coupled_score for callers that cannot allocate: the caller brings the score tensors, the partial sums
        live in the library's own fixed device array (nothing is reserved or allocated here)."""
        arr = pairs if isinstance(pairs, C.Array) else (Pair * len(pairs))(*pairs)
        ptrs = (C.c_void_p * len(arr))(*[o.data_ptr() for o in out])
        self._check(self.lib.ecospa_coupled_score_static(self.h, arr, len(arr), ptrs), "ecospa_coupled_score_static")
        return list(out)

    def ecospa_pair_fisher(self, grads: Sequence[Pair], n_samples: float,
                           out: Optional[Sequence[torch.Tensor]] = None) -> list[torch.Tensor]:
        """Eq. 8 importance of each coupled pair from its gradient matrices (described like the weights): one
        float32 tensor [groups] per pair (written into `out` if given)."""
        arr = grads if isinstance(grads, C.Array) else (Pair * len(grads))(*grads)
        self.reserve(self.lib.ecospa_score_workspace_bytes(arr, len(arr)))
        if out is None:
            out = [torch.empty((p.groups,), dtype=torch.float32, device=self.device) for p in arr]
        ptrs = (C.c_void_p * len(arr))(*[o.data_ptr() for o in out])
        self._check(self.lib.ecospa_pair_fisher(self.h, arr, len(arr), float(n_samples), ptrs), "ecospa_pair_fisher")
        return list(out)

    def ecospa_select_theta(self, scores: torch.Tensor, theta: float):
        """Alg. 1's cumulative-threshold rule per row of scores[groups, n_units]: (idx[groups, n_units] int32 padded
        with -1, k[groups] int32)."""
        assert scores.dtype == torch.float32 and scores.dim() == 2 and scores.is_contiguous()
        groups, n = scores.shape
        idx = torch.empty((groups, n), dtype=torch.int32, device=scores.device)
        k = torch.empty((groups,), dtype=torch.int32, device=scores.device)
        self._check(self.lib.ecospa_select_theta(self.h, scores.data_ptr(), groups, n, float(theta), idx.data_ptr(),
                                                 k.data_ptr()), "ecospa_select_theta")
        return idx, k

    def ecospa_select_pairs(self, fisher: torch.Tensor, n_select: int) -> torch.Tensor:
        """Alg. 1's choice among the pairs: ascending indices (int32[n_select]) of the n_select smallest
        importance values of fisher[n_pairs]."""
        assert fisher.dtype == torch.float32 and fisher.dim() == 1 and fisher.is_contiguous()
        chosen = torch.empty((max(n_select, 1),), dtype=torch.int32, device=fisher.device)
        self._check(self.lib.ecospa_select_pairs(self.h, fisher.data_ptr(), fisher.numel(), n_select,
                                                 chosen.data_ptr()), "ecospa_select_pairs")
        return chosen[:n_select]

    # ---- step 2 ------------------------------------------------------------------------------
    def ecospa_select_topk(self, scores: torch.Tensor, k: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        groups, n_units = scores.shape
        assert scores.dtype == torch.float32 and scores.is_contiguous()
        idx = out if out is not None else torch.empty((groups, max(k, 0)), dtype=torch.int32, device=self.device)
        self._check(self.lib.ecospa_select_topk(self.h, scores.data_ptr(), groups, n_units, k, idx.data_ptr()),
                    "ecospa_select_topk")
        return idx

    def ecospa_select_topk_batch(self, items: Sequence[SelectItem]):
        """items: SelectItem structs (see :meth:`select_item`); one launch for all of them."""
        arr = items if isinstance(items, C.Array) else (SelectItem * len(items))(*items)
        self._check(self.lib.ecospa_select_topk_batch(self.h, arr, len(items)), "ecospa_select_topk_batch")

    @staticmethod
    def select_item(scores: torch.Tensor, k: int, idx: torch.Tensor) -> SelectItem:
        groups, n_units = scores.shape
        assert scores.dtype == torch.float32 and scores.is_contiguous() and idx.dtype == torch.int32
        return SelectItem(scores.data_ptr(), groups, n_units, k, idx.data_ptr())

    def ecospa_check_indices(self, idx: torch.Tensor, n_units: int, k_group: Optional[torch.Tensor] = None) -> bool:
        """Debugging aid (waits for the stream): True if every list idx[g, :k] (k = idx.shape[1], or k_group[g]) is
        strictly ascending with entries in [0, n_units)."""
        assert idx.dtype == torch.int32 and idx.dim() == 2 and idx.is_contiguous()
        self.reserve(256)
        rc = self.lib.ecospa_check_indices(self.h, idx.data_ptr(), idx.shape[0], idx.shape[1], idx.shape[1], _ptr(k_group),
                                           n_units)
        if rc == ERR_INDEX:
            return False
        self._check(rc, "ecospa_check_indices")
        return True

    # ---- step 3 ------------------------------------------------------------------------------
    @staticmethod
    def map_item(src: torch.Tensor, dst: torch.Tensor, idx: torch.Tensor, axis: int, groups: int, n: int,
                 unit: int = 1, kp: Optional[int] = None, scatter: int = 0,
                 k_group: Optional[torch.Tensor] = None, idx_div: int = 1,
                 dst_t: Optional[torch.Tensor] = None, src_b: Optional[torch.Tensor] = None) -> MapItem:
        """Descriptor of one gather (scatter = 0), scatter with zero fill (1) or scatter that leaves the pruned
        slots of dst untouched (2) for :meth:`ecospa_compact_batch`.  With k_group (int32[groups]
        on the device) group g keeps its first k_group[g] entries of idx[g, :] and kp must be given.  dst_t (row gathers
        only): the transposed copy of dst, [other, slots], written by the same launch.  src_b (row gathers only): a
        second source like src; dst then takes the kept rows of both, interleaved (row 2s from src, 2s + 1 from src_b)."""
        assert src_b is None or (src_b.shape == src.shape and src_b.stride(0) == src.stride(0) and src_b.dtype == src.dtype)
        if k_group is not None:
            assert kp is not None and k_group.dtype == torch.int32 and k_group.numel() == groups // idx_div
            assert idx.dtype == torch.int32 and idx.dim() == 2 and idx.is_contiguous() and idx.shape[0] == groups // idx_div
        k = idx.shape[1] if k_group is None else 0
        kp = k if kp is None else kp
        if src.dim() == 1:
            other, ld_s, ld_d, axis = 1, src.numel(), dst.numel(), 1
        else:
            other = src.shape[1] if axis == 0 else src.shape[0]
            ld_s, ld_d = src.stride(0), dst.stride(0)
        return MapItem(src.data_ptr(), dst.data_ptr(), dtype_code(src.dtype), axis, groups, n, unit, k, kp,
                       int(scatter), other, ld_s, ld_d, idx.data_ptr(), _ptr(k_group),
                       idx.shape[1] if k_group is not None else 0, idx_div,
                       _ptr(dst_t), 0 if dst_t is None else dst_t.stride(0), _ptr(src_b))

    def ecospa_compact_ragged(self, src: torch.Tensor, idx: torch.Tensor, k_group: torch.Tensor, axis: int, groups: int,
                              n: int, kp: int, unit: int = 1, scatter: int = 0,
                              out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Gather (or scatter: 1 zero fill, 2 into the contents of `out`) with ragged kept counts, all groups padded
        to kp slots."""
        slots = groups * n if scatter else groups * kp * unit
        if out is None:
            shape = (slots,) if src.dim() == 1 else ((slots, src.shape[1]) if axis == 0 else (src.shape[0], slots))
            out = torch.empty(shape, dtype=src.dtype, device=src.device)
        self.ecospa_compact_batch([self.map_item(src, out, idx, axis, groups, n, unit, kp, scatter, k_group)])
        return out

    def ecospa_compact_batch(self, items: Sequence[MapItem], rope: Optional[RopeItem] = None):
        """All gathers / scatters of `items` in one launch; with `rope` (see :meth:`rope_item`) the same launch also
        fills the cos/sin tables of the kept rotary blocks."""
        arr = items if isinstance(items, C.Array) else (MapItem * len(items))(*items)
        if rope is None:
            self._check(self.lib.ecospa_compact_batch(self.h, arr, len(items)), "ecospa_compact_batch")
        else:
            self._check(self.lib.ecospa_compact_batch_rope(self.h, arr, len(items), C.byref(rope)), "ecospa_compact_batch_rope")

    @staticmethod
    def rope_item(idx: Optional[torch.Tensor], h: int, L: int, k: int, kp: int, d_h: int, base: float, cos: torch.Tensor,
                  sin: torch.Tensor, k_group: Optional[torch.Tensor] = None) -> RopeItem:
        """Descriptor of the cos/sin tables [h, L, kp] of the kept rotary blocks for :meth:`ecospa_compact_batch`: as
        :meth:`ecospa_rope_table` (k blocks per head) or, with k_group, as :meth:`ecospa_rope_table_ragged`."""
        assert cos.shape == (h, L, kp) and sin.shape == (h, L, kp) and cos.dtype == torch.float32 and sin.dtype == torch.float32
        ld_idx = 0 if idx is None else idx.shape[1]
        return RopeItem(_ptr(idx), _ptr(k_group), h, L, 0 if k_group is not None else k, kp, d_h, ld_idx, float(base),
                        cos.data_ptr(), sin.data_ptr())

    def _mapped(self, fn, name, src, dst, axis, groups, n, unit, k, kp, idx):
        if src.dim() == 1:
            other, ld_s, ld_d = 1, src.numel(), dst.numel()
            axis = 1
        else:
            other = src.shape[1] if axis == 0 else src.shape[0]
            ld_s, ld_d = src.stride(0), dst.stride(0)
        self._check(fn(self.h, src.data_ptr(), dst.data_ptr(), dtype_code(src.dtype), axis, groups, n, unit, k, kp,
                       other, ld_s, ld_d, idx.data_ptr()), name)
        return dst

    def ecospa_compact(self, src: torch.Tensor, idx: torch.Tensor, axis: int, groups: int, n: int, unit: int = 1,
                       kp: Optional[int] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        k = idx.shape[1]
        kp = k if kp is None else kp
        slots = groups * kp * unit
        if out is None:
            shape = (slots,) if src.dim() == 1 else ((slots, src.shape[1]) if axis == 0 else (src.shape[0], slots))
            out = torch.empty(shape, dtype=src.dtype, device=src.device)
        return self._mapped(self.lib.ecospa_compact, "ecospa_compact", src, out, axis, groups, n, unit, k, kp, idx)

    def ecospa_scatter(self, src: torch.Tensor, idx: torch.Tensor, axis: int, groups: int, n: int, unit: int = 1,
                       kp: Optional[int] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        k = idx.shape[1]
        kp = k if kp is None else kp
        slots = groups * n
        if out is None:
            shape = (slots,) if src.dim() == 1 else ((slots, src.shape[1]) if axis == 0 else (src.shape[0], slots))
            out = torch.empty(shape, dtype=src.dtype, device=src.device)
        return self._mapped(self.lib.ecospa_scatter, "ecospa_scatter", src, out, axis, groups, n, unit, k, kp, idx)

    def ecospa_rope_table(self, idx: Optional[torch.Tensor], h: int, L: int, k: int, kp: int, d_h: int,
                          base: float = 10000.0, out=None):
        if out is not None:
            cos, sin = out
            assert cos.shape == (h, L, kp) and sin.shape == (h, L, kp) and cos.dtype == torch.float32
        else:
            cos = torch.empty((h, L, kp), dtype=torch.float32, device=self.device)
            sin = torch.empty_like(cos)
        self._check(self.lib.ecospa_rope_table(self.h, _ptr(idx), h, L, k, kp, d_h, float(base), cos.data_ptr(),
                                               sin.data_ptr()), "ecospa_rope_table")
        return cos, sin

    def ecospa_rope_table_ragged(self, idx: torch.Tensor, k_group: torch.Tensor, L: int, kp: int, d_h: int,
                                 base: float = 10000.0, out=None):
        h = idx.shape[0]
        assert idx.dtype == torch.int32 and idx.is_contiguous() and k_group.dtype == torch.int32 and k_group.numel() == h
        if out is not None:
            cos, sin = out
            assert cos.shape == (h, L, kp) and sin.shape == (h, L, kp) and cos.dtype == torch.float32
        else:
            cos = torch.empty((h, L, kp), dtype=torch.float32, device=self.device)
            sin = torch.empty_like(cos)
        self._check(self.lib.ecospa_rope_table_ragged(self.h, idx.data_ptr(), idx.shape[1], k_group.data_ptr(), h, L, kp,
                                                      d_h, float(base), cos.data_ptr(), sin.data_ptr()),
                    "ecospa_rope_table_ragged")
        return cos, sin

    @staticmethod
    def transpose_item(src: torch.Tensor, dst: torch.Tensor) -> TransposeItem:
        assert src.dim() == 2 and dst.shape == (src.shape[1], src.shape[0]) and src.dtype == dst.dtype
        return TransposeItem(src.data_ptr(), dst.data_ptr(), dtype_code(src.dtype), src.shape[0], src.shape[1],
                             src.stride(0), dst.stride(0))

    def ecospa_transpose_batch(self, items: Sequence[TransposeItem]):
        """dst = src^T for every item, one launch (see :meth:`transpose_item`)."""
        arr = items if isinstance(items, C.Array) else (TransposeItem * len(items))(*items)
        self._check(self.lib.ecospa_transpose_batch(self.h, arr, len(arr)), "ecospa_transpose_batch")

    # ---- layer glue ----------------------------------------------------------------------------
    def ecospa_norm_fwd(self, kind: int, x: torch.Tensor, gain: torch.Tensor, bias: Optional[torch.Tensor], eps: float,
                        y: torch.Tensor, res: Optional[torch.Tensor] = None, x_out: Optional[torch.Tensor] = None,
                        stat: Optional[torch.Tensor] = None):
        """y = norm(x + res); x + res -> x_out; the row statistics -> stat (float32 [T] for RMS, [T, 2] for LayerNorm).
        All [T, d] tensors contiguous bf16."""
        T, d = x.shape
        assert all(t is None or (t.is_contiguous() and t.shape == x.shape) for t in (x, y, res, x_out))
        self._check(self.lib.ecospa_norm_fwd(self.h, kind, T, d, dtype_code(x.dtype), x.data_ptr(), _ptr(res), _ptr(x_out),
                                             gain.data_ptr(), _ptr(bias), float(eps), y.data_ptr(), _ptr(stat)), "ecospa_norm_fwd")
        return y

    def ecospa_norm_bwd(self, kind: int, x: torch.Tensor, gain: torch.Tensor, stat: torch.Tensor, dy: torch.Tensor,
                        dx: torch.Tensor, dgain: torch.Tensor, dbias: Optional[torch.Tensor] = None,
                        dres: Optional[torch.Tensor] = None):
        """dx = dres + the gradient of the normalisation; dgain (and dbias) = the parameter gradients."""
        T, d = x.shape
        assert all(t is None or (t.is_contiguous() and t.shape == x.shape) for t in (x, dy, dx, dres))
        self.reserve(self.lib.ecospa_norm_bwd_workspace_bytes(T, d))
        self._check(self.lib.ecospa_norm_bwd(self.h, kind, T, d, dtype_code(x.dtype), x.data_ptr(), gain.data_ptr(), stat.data_ptr(),
                                             dy.data_ptr(), _ptr(dres), dx.data_ptr(), dgain.data_ptr(), _ptr(dbias)), "ecospa_norm_bwd")
        return dx

    def ecospa_embed_fwd(self, ids: torch.Tensor, table: torch.Tensor, out: torch.Tensor, pos: Optional[torch.Tensor] = None):
        """out[t] = table[ids[t]] (+ pos[t mod L]); ids int64."""
        assert ids.dtype == torch.int64 and ids.is_contiguous() and table.is_contiguous() and out.is_contiguous()
        T, (V, d) = ids.numel(), table.shape
        self._check(self.lib.ecospa_embed_fwd(self.h, T, d, V, dtype_code(table.dtype), ids.data_ptr(), table.data_ptr(), _ptr(pos),
                                              0 if pos is None else pos.shape[0], out.data_ptr()), "ecospa_embed_fwd")
        return out

    def ecospa_embed_bwd(self, ids: torch.Tensor, dx: torch.Tensor, dtable: torch.Tensor, dpos: Optional[torch.Tensor] = None):
        """dtable[v] = sum of dx[t] over ids[t] == v (the whole table is written); dpos[l] = sum over the sequences."""
        assert ids.dtype == torch.int64 and ids.is_contiguous() and dx.is_contiguous() and dtable.is_contiguous()
        T, (V, d) = ids.numel(), dtable.shape
        self._check(self.lib.ecospa_embed_bwd(self.h, T, d, V, dtype_code(dx.dtype), ids.data_ptr(), dx.data_ptr(), dtable.data_ptr(),
                                              _ptr(dpos), 0 if dpos is None else dpos.shape[0]), "ecospa_embed_bwd")

    def ecospa_xent(self, logits: torch.Tensor, targets: torch.Tensor, row_loss: torch.Tensor, loss: torch.Tensor,
                    dlogits: Optional[torch.Tensor] = None):
        """Mean cross-entropy of the rows of logits [T, V] (bf16, row stride free) against int64 targets: the row losses,
        the mean (a device float) and dlogits of the mean (may be logits itself)."""
        assert targets.dtype == torch.int64 and targets.is_contiguous() and logits.stride(1) == 1
        assert row_loss.dtype == torch.float32 and loss.dtype == torch.float32
        T, V = logits.shape
        self._check(self.lib.ecospa_xent(self.h, T, V, dtype_code(logits.dtype), logits.data_ptr(), logits.stride(0), targets.data_ptr(),
                                         _ptr(dlogits), 0 if dlogits is None else dlogits.stride(0), row_loss.data_ptr(),
                                         loss.data_ptr()), "ecospa_xent")
        return loss

    # ---- parameter update ----------------------------------------------------------------------
    @staticmethod
    def adamw_item(w: torch.Tensor, g: torch.Tensor, m: torch.Tensor, v: torch.Tensor,
                   w_lp: Optional[torch.Tensor] = None) -> AdamwItem:
        """Descriptor of one tensor for :meth:`ecospa_adamw` (all contiguous, same element count)."""
        n = w.numel()
        assert all(t.is_contiguous() and t.numel() == n for t in (w, g, m, v)) and m.dtype == v.dtype
        assert w_lp is None or (w_lp.is_contiguous() and w_lp.numel() == n and w_lp.dtype == torch.bfloat16)
        return AdamwItem(w.data_ptr(), _ptr(w_lp), g.data_ptr(), m.data_ptr(), v.data_ptr(), n, dtype_code(w.dtype),
                         dtype_code(g.dtype), dtype_code(m.dtype))

    def ecospa_adamw(self, items: Sequence[AdamwItem], step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999,
                     eps: float = 1e-8, weight_decay: float = 0.01):
        """One fused AdamW step over all tensors in `items` (one launch)."""
        arr = items if isinstance(items, C.Array) else (AdamwItem * len(items))(*items)
        hp = AdamwHyper(lr, beta1, beta2, eps, weight_decay, step)
        self._check(self.lib.ecospa_adamw(self.h, arr, len(arr), C.byref(hp)), "ecospa_adamw")

    # ---- steps 4-5 ---------------------------------------------------------------------------
    def ecospa_coupled_fwd(self, desc: BlockDesc, x: torch.Tensor, y: torch.Tensor, saved: Optional[Saved]):
        self.reserve(self.lib.ecospa_block_workspace_bytes(C.byref(desc)))
        self._check(self.lib.ecospa_coupled_fwd(self.h, C.byref(desc), x.data_ptr(), y.data_ptr(),
                                                None if saved is None else C.byref(saved)), "ecospa_coupled_fwd")
        return y

    def ecospa_coupled_bwd(self, desc: BlockDesc, x: torch.Tensor, dy: torch.Tensor, saved: Saved,
                           dx: Optional[torch.Tensor], grads: Grads):
        self.reserve(self.lib.ecospa_block_workspace_bytes(C.byref(desc)))
        self._check(self.lib.ecospa_coupled_bwd(self.h, C.byref(desc), x.data_ptr(), dy.data_ptr(), C.byref(saved),
                                                _ptr(dx), C.byref(grads)), "ecospa_coupled_bwd")
        return dx
