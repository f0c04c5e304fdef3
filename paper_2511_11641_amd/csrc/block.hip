// Steps 4-5: reduced forward/backward of one block on the compacted matrices.  This file holds
// the argument validation, the workspace layout, the FFN block (Eq. 3; gated form of the footnote
// to Eq. 8) and the dispatch of the C-ABI entry points; the attention block lives in attn.hip.
#include "block.h"
#include "gemm_epi.h"

static bool is_gated(const ecospa_block_desc& d) { return d.act == ECOSPA_ACT_SWIGLU; }

static int validate_block(const ecospa_block_desc* dp) {
  if (!dp) return ECOSPA_ERR_NULL;
  const ecospa_block_desc& d = *dp;
  if (!dtype_ok(d.dtype)) return ECOSPA_ERR_DTYPE;
  if (d.block != ECOSPA_BLOCK_ATTN && d.block != ECOSPA_BLOCK_FFN) return ECOSPA_ERR_DTYPE;
  if (d.B < 1 || d.L < 1 || d.d_model < 1) return ECOSPA_ERR_SHAPE;
  if (static_cast<long long>(d.B) * d.L > (1ll << 30)) return ECOSPA_ERR_SHAPE;
  if (d.d_model % 8) return ECOSPA_ERR_ALIGN;
  if (d.block == ECOSPA_BLOCK_FFN) {
    if (d.act < ECOSPA_ACT_GELU_ERF || d.act > ECOSPA_ACT_SWIGLU) return ECOSPA_ERR_DTYPE;
    if (d.kp_ff < 16 || d.kp_ff % 16) return ECOSPA_ERR_SHAPE;
    if (!d.w_1 || !d.w_2) return ECOSPA_ERR_NULL;
    if (d.ld_w1 < d.d_model || d.ld_w2 < d.kp_ff) return ECOSPA_ERR_SHAPE;
    if (d.ld_w1 % 8 || d.ld_w2 % 8 || !aligned16(d.w_1) || !aligned16(d.w_2)) return ECOSPA_ERR_ALIGN;
    const long long nh = static_cast<long long>(d.act == ECOSPA_ACT_SWIGLU ? 2 : 1) * d.kp_ff;
    if ((d.w_1_t && d.ld_w1t < nh) || (d.w_2_t && d.ld_w2t < d.d_model)) return ECOSPA_ERR_SHAPE;
    if ((d.w_1_t && (d.ld_w1t % 8 || !aligned16(d.w_1_t))) || (d.w_2_t && (d.ld_w2t % 8 || !aligned16(d.w_2_t)))) return ECOSPA_ERR_ALIGN;
  } else {
    // head widths: multiples of 16 up to 128 (the attention core is built for 32-, 64- and 128-wide padded heads)
    if (d.h < 1 || d.kp_qk < 16 || d.kp_vo < 16 || d.kp_qk % 16 || d.kp_vo % 16 || d.kp_qk > 128 || d.kp_vo > 128)
      return ECOSPA_ERR_SHAPE;
    if (d.h_kv < 0 || d.h % attn_h_kv(d)) return ECOSPA_ERR_SHAPE;
    if (!d.w_qkv || !d.w_o) return ECOSPA_ERR_NULL;
    if ((d.rope_cos == nullptr) != (d.rope_sin == nullptr)) return ECOSPA_ERR_NULL;
    if (d.ld_wqkv < d.d_model || d.ld_wo < static_cast<long long>(d.h) * d.kp_vo) return ECOSPA_ERR_SHAPE;
    if (d.ld_wqkv % 8 || d.ld_wo % 8 || !aligned16(d.w_qkv) || !aligned16(d.w_o)) return ECOSPA_ERR_ALIGN;
    if ((d.w_qkv_t && d.ld_wqkvt < attn_nqkv(d)) || (d.w_o_t && d.ld_wot < d.d_model)) return ECOSPA_ERR_SHAPE;
    if ((d.w_qkv_t && (d.ld_wqkvt % 8 || !aligned16(d.w_qkv_t))) || (d.w_o_t && (d.ld_wot % 8 || !aligned16(d.w_o_t)))) return ECOSPA_ERR_ALIGN;
    if (!(d.scale > 0.f)) return ECOSPA_ERR_SHAPE;
  }
  return ECOSPA_OK;
}

static size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

// Rows of partial column sums that the weight-gradient contraction dY^T X of this shape writes (library's own plan).
int block_colsum_rows(int dtype, int M, int N, int K) {
  GemmDesc g;
  memset(&g, 0, sizeof(g));
  g.dtype = dtype; g.M = M; g.N = N; g.K = K; g.lda = M; g.ldb = N; g.trans_a = g.trans_b = 1;
  g.splits = ecospa_gemm_splits(M, N, K);
  return ecospa_gemm_colsum_rows(g);
}

void block_ws_layout(const ecospa_block_desc& d, void* base, BlockWs& w) {
  memset(&w, 0, sizeof(w));
  WsCarver c(base ? base : reinterpret_cast<void*>(256), ~static_cast<size_t>(0) >> 1);
  const size_t T = static_cast<size_t>(d.B) * d.L, es = dtype_size(d.dtype);
  size_t part = 0, part2 = 0, cs = 0, cs2 = 0, px = 0;
  const int Ti = static_cast<int>(T);
  auto splitk_bytes = [&](int M, int N, int K) {
    const int s = ecospa_gemm_splits(M, N, K);
    return s > 1 ? static_cast<size_t>(s) * M * N * 4 : static_cast<size_t>(0);
  };
  auto colsum_bytes = [&](int M, int N, int K) { return static_cast<size_t>(block_colsum_rows(d.dtype, M, N, K)) * M * 4; };
  if (d.block == ECOSPA_BLOCK_FFN) {
    const size_t nh = static_cast<size_t>(is_gated(d) ? 2 : 1) * d.kp_ff;
    w.dh = c.take(T * nh * es);
    w.hpre_tmp = w.dh;                       // inference scratch aliases the backward scratch
    w.act_tmp = c.take(T * d.kp_ff * es);
    part = splitk_bytes(d.d_model, d.kp_ff, static_cast<int>(T));
    part2 = splitk_bytes(static_cast<int>(nh), d.d_model, static_cast<int>(T));
    cs = colsum_bytes(d.d_model, d.kp_ff, static_cast<int>(T));
    cs2 = colsum_bytes(static_cast<int>(nh), d.d_model, static_cast<int>(T));
    px = max_sz(max_sz(block_token_split_bytes(Ti, static_cast<int>(nh), d.d_model), block_token_split_bytes(Ti, d.d_model, d.kp_ff)),
                max_sz(block_token_split_bytes(Ti, d.kp_ff, d.d_model), block_token_split_bytes(Ti, d.d_model, static_cast<int>(nh))));
  } else {
    const size_t nqkv = attn_nqkv(d), nvo = static_cast<size_t>(d.h) * d.kp_vo;
    w.dqkv = c.take(T * nqkv * es);
    w.qkv_tmp = w.dqkv;
    w.d_o = c.take(T * nvo * es);
    w.o_tmp = w.d_o;
    w.delta = static_cast<float*>(c.take(static_cast<size_t>(d.B) * d.h * d.L * 4));
    w.lse_tmp = static_cast<float*>(c.take(static_cast<size_t>(d.B) * d.h * d.L * 4));
    part = splitk_bytes(d.d_model, static_cast<int>(nvo), static_cast<int>(T));
    part2 = splitk_bytes(static_cast<int>(nqkv), d.d_model, static_cast<int>(T));
    cs = colsum_bytes(d.d_model, static_cast<int>(nvo), static_cast<int>(T));
    cs2 = colsum_bytes(static_cast<int>(nqkv), d.d_model, static_cast<int>(T));
    px = max_sz(max_sz(block_token_split_bytes(Ti, static_cast<int>(nqkv), d.d_model), block_token_split_bytes(Ti, d.d_model, static_cast<int>(nvo))),
                max_sz(block_token_split_bytes(Ti, static_cast<int>(nvo), d.d_model), block_token_split_bytes(Ti, d.d_model, static_cast<int>(nqkv))));
  }
  w.partial_x = px ? static_cast<float*>(c.take(px)) : nullptr;
  w.partial = static_cast<float*>(c.take(part));
  w.partial2 = static_cast<float*>(c.take(part2));
  w.colsum = static_cast<float*>(c.take(cs));
  w.colsum2 = static_cast<float*>(c.take(cs2));
  w.total = c.off + 256;
  if (!base) memset(&w, 0, offsetof(BlockWs, total));
}

extern "C" size_t ecospa_block_workspace_bytes(const ecospa_block_desc* desc) {
  if (validate_block(desc) != ECOSPA_OK) return 0;
  BlockWs w;
  block_ws_layout(*desc, nullptr, w);
  return w.total;
}

// ---------------------------------------------------------------------------------------------
// FFN
// ---------------------------------------------------------------------------------------------
// Gated activation on pre-activations whose columns come in (gate, up) pairs (fp32 path; bf16 has it in the epilogue
// of the first contraction).
template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const T* __restrict__ hpre, long long ldh, T* __restrict__ act,
                                                     long long lda, long long rows, int kp) {
  const long long e = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= rows * kp) return;
  const long long m = e / kp;
  const int n = static_cast<int>(e % kp);
  const float g = load_f32<T>(hpre + m * ldh + 2 * n), u = load_f32<T>(hpre + m * ldh + 2 * n + 1);
  store_f32<T>(act + m * lda + n, g * act_sigmoid(g) * u);
}

static GemmDesc gemm_desc(int dtype, int M, int N, int K, const void* A, long long lda, int ta, const void* B,
                          long long ldb, int tb) {
  GemmDesc g;
  memset(&g, 0, sizeof(g));
  g.dtype = dtype; g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.trans_a = ta;
  g.B = B; g.ldb = ldb; g.trans_b = tb;
  g.splits = 1;
  return g;
}

static int ffn_forward(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x, void* y,
                       const ecospa_saved* saved) {
  const int T = d.B * d.L, kp = d.kp_ff, nh = is_gated(d) ? 2 * kp : kp;
  void* hpre = saved ? saved->hpre : w.hpre_tmp;
  void* act = saved ? saved->act : w.act_tmp;
  if (!hpre || !act) return ECOSPA_ERR_NULL;
  int rc;
  GemmDesc g = gemm_desc(d.dtype, T, nh, d.d_model, x, d.d_model, 0, d.w_1, d.ld_w1, 0);
  g.epi.c = hpre; g.epi.ldc = nh; g.epi.bias = d.b_1;
  block_token_split(g, w);
  if (is_gated(d) && d.dtype == ECOSPA_BF16) {
    // gate and up rows alternate in w_1, so every output tile holds whole (gate, up) pairs: the product is formed in
    // the epilogue; forward only (no saved activations) the pre-activations are not written at all
    g.epi.kind = EPI_SWIGLU;
    g.epi.c = saved ? hpre : nullptr;
    g.epi.c2 = act; g.epi.ldc2 = kp;
    if (!aligned16(hpre) || (reinterpret_cast<uintptr_t>(act) & 7u)) return ECOSPA_ERR_ALIGN;
    if ((rc = ecospa_gemm(ctx, g))) return rc;
  } else if (is_gated(d)) {
    g.epi.kind = EPI_STORE;
    if ((rc = ecospa_gemm(ctx, g))) return rc;
    const long long tot = static_cast<long long>(T) * kp;
    hipLaunchKernelGGL((swiglu_kernel<float>), dim3(static_cast<unsigned>((tot + 255) / 256)), dim3(256), 0, ctx->stream,
                       static_cast<const float*>(hpre), static_cast<long long>(nh), static_cast<float*>(act),
                       static_cast<long long>(kp), static_cast<long long>(T), kp);
    ECOSPA_CHECK_LAUNCH(ctx, "swiglu_kernel");
  } else if (!saved) {
    // forward only: nothing will ask for the activation's input, so it is not written
    g.epi.kind = EPI_ACT; g.epi.act = d.act;
    g.epi.c = act; g.epi.ldc = kp;
    if ((rc = ecospa_gemm(ctx, g))) return rc;
  } else {
    g.epi.kind = EPI_BIAS_ACT; g.epi.act = d.act;
    g.epi.c2 = act; g.epi.ldc2 = kp;
    if ((rc = ecospa_gemm(ctx, g))) return rc;
  }
  GemmDesc g2 = gemm_desc(d.dtype, T, d.d_model, kp, act, kp, 0, d.w_2, d.ld_w2, 0);
  g2.epi.kind = EPI_STORE; g2.epi.c = y; g2.epi.ldc = d.d_model; g2.epi.bias = d.b_2;
  block_token_split(g2, w);
  return ecospa_gemm(ctx, g2);
}

// Backward pass: dH, the two split-K weight gradients (partials only), dX, and then ONE launch for
// the reductions of the partials and the two bias-gradient column sums.
static int ffn_backward_body(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x, const void* dy,
                             const ecospa_saved& sv, void* dx, const ecospa_grads& gr) {
  const int T = d.B * d.L, kp = d.kp_ff, nh = is_gated(d) ? 2 * kp : kp, dm = d.d_model;
  int rc;
  // dH = (dY W_2) * act'(H)
  {
    GemmDesc g = d.w_2_t ? gemm_desc(d.dtype, T, kp, dm, dy, dm, 0, d.w_2_t, d.ld_w2t, 0)     // transposed copy [kp, d_model]
                         : gemm_desc(d.dtype, T, kp, dm, dy, dm, 0, d.w_2, d.ld_w2, 1);
    g.epi.c = w.dh; g.epi.ldc = nh; g.epi.h = sv.hpre; g.epi.ldh = nh; g.epi.act = d.act; g.epi.kp = kp;
    g.epi.kind = is_gated(d) ? EPI_DSWIGLU : EPI_DACT;
    block_token_split(g, w);
    if ((rc = ecospa_gemm(ctx, g))) return rc;
  }
  // dW_2 = dY^T A,  dW_1 = dH^T X
  GemmDesc g2 = gemm_desc(d.dtype, dm, kp, T, dy, dm, 1, sv.act, kp, 1);
  g2.splits = ecospa_gemm_splits(dm, kp, T); g2.partial = w.partial; g2.defer_reduce = 1;
  g2.epi.kind = EPI_STORE; g2.epi.c = gr.dw_2; g2.epi.ldc = gr.ld_dw2;
  // the bias gradients are column sums of dY and dH: the weight-gradient contractions read exactly these as
  // their K-slow operand and add them up on the way (bf16 kernels; otherwise a column-sum job below)
  const bool fused_db = d.dtype == ECOSPA_BF16;
  if (fused_db && gr.dw_2 && gr.db_2) g2.colsum = w.colsum;
  if (gr.dw_2 && (rc = ecospa_gemm(ctx, g2))) return rc;
  GemmDesc g1 = gemm_desc(d.dtype, nh, dm, T, w.dh, nh, 1, x, dm, 1);
  g1.splits = ecospa_gemm_splits(nh, dm, T); g1.partial = w.partial2; g1.defer_reduce = 1;
  g1.epi.kind = EPI_STORE; g1.epi.c = gr.dw_1; g1.epi.ldc = gr.ld_dw1;
  if (fused_db && gr.dw_1 && gr.db_1) g1.colsum = w.colsum2;
  if (gr.dw_1 && (rc = ecospa_gemm(ctx, g1))) return rc;

  // dX = dH W_1
  if (dx) {
    GemmDesc g = d.w_1_t ? gemm_desc(d.dtype, T, dm, nh, w.dh, nh, 0, d.w_1_t, d.ld_w1t, 0)   // transposed copy [d_model, nh]
                         : gemm_desc(d.dtype, T, dm, nh, w.dh, nh, 0, d.w_1, d.ld_w1, 1);
    g.epi.kind = EPI_STORE; g.epi.c = dx; g.epi.ldc = dm;
    block_token_split(g, w);
    if ((rc = ecospa_gemm(ctx, g))) return rc;
  }
  AuxBatch aux;
  memset(&aux, 0, sizeof(aux));
  if (gr.dw_2 && g2.splits > 1) aux.reduce[aux.n_reduce++] = g2;
  if (gr.dw_1 && g1.splits > 1) aux.reduce[aux.n_reduce++] = g1;
  if (gr.db_2) aux.colsum[aux.n_colsum++] = g2.colsum ? AuxColsum{g2.colsum, dm, ecospa_gemm_colsum_rows(g2), dm, ECOSPA_F32, gr.db_2, d.dtype}
                                                       : AuxColsum{dy, dm, T, dm, d.dtype, gr.db_2, 0};
  if (gr.db_1) aux.colsum[aux.n_colsum++] = g1.colsum ? AuxColsum{g1.colsum, nh, ecospa_gemm_colsum_rows(g1), nh, ECOSPA_F32, gr.db_1, d.dtype}
                                                       : AuxColsum{w.dh, nh, T, nh, d.dtype, gr.db_1, 0};
  return ecospa_aux_launch(ctx, aux);
}

static int ffn_backward(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x, const void* dy,
                        const ecospa_saved& sv, void* dx, const ecospa_grads& gr) {
  if (!sv.hpre || !sv.act) return ECOSPA_ERR_NULL;
  if (gr.dw_2 && gr.ld_dw2 < d.kp_ff) return ECOSPA_ERR_SHAPE;
  if (gr.dw_1 && gr.ld_dw1 < d.d_model) return ECOSPA_ERR_SHAPE;
  return ffn_backward_body(ctx, d, w, x, dy, sv, dx, gr);
}

// ---------------------------------------------------------------------------------------------
extern "C" int ecospa_coupled_fwd(ecospa_ctx* ctx, const ecospa_block_desc* desc, const void* x, void* y,
                                  const ecospa_saved* saved) {
  if (!ctx || !desc || !x || !y) return ECOSPA_ERR_NULL;
  int rc = validate_block(desc);
  if (rc) return rc;
  if (!aligned16(x) || !aligned16(y)) return ECOSPA_ERR_ALIGN;
  BlockWs w;
  block_ws_layout(*desc, nullptr, w);
  if (!ctx->ws || ctx->ws_bytes < w.total) return ECOSPA_ERR_WORKSPACE;
  block_ws_layout(*desc, ctx->ws, w);
  if (desc->block == ECOSPA_BLOCK_FFN) return ffn_forward(ctx, *desc, w, x, y, saved);
  return attn_forward(ctx, *desc, w, x, y, saved);
}

extern "C" int ecospa_coupled_bwd(ecospa_ctx* ctx, const ecospa_block_desc* desc, const void* x, const void* dy,
                                  const ecospa_saved* saved, void* dx, const ecospa_grads* grads) {
  if (!ctx || !desc || !x || !dy || !saved || !grads) return ECOSPA_ERR_NULL;
  int rc = validate_block(desc);
  if (rc) return rc;
  if (!aligned16(x) || !aligned16(dy) || (dx && !aligned16(dx))) return ECOSPA_ERR_ALIGN;
  BlockWs w;
  block_ws_layout(*desc, nullptr, w);
  if (!ctx->ws || ctx->ws_bytes < w.total) return ECOSPA_ERR_WORKSPACE;
  block_ws_layout(*desc, ctx->ws, w);
  if (desc->block == ECOSPA_BLOCK_FFN) return ffn_backward(ctx, *desc, w, x, dy, *saved, dx, *grads);
  return attn_backward(ctx, *desc, w, x, dy, *saved, dx, *grads);
}

// ---------------------------------------------------------------------------------------------
extern "C" size_t ecospa_contract_workspace_bytes(int dtype, int M, int N, int K, int splits) {
  if (!dtype_ok(dtype) || M < 1 || N < 1 || K < 1 || splits < 0 || splits > 64) return 0;
  const int s = splits == 0 ? ecospa_gemm_splits(M, N, K) : splits;
  return s > 1 ? static_cast<size_t>(s) * M * N * 4 : 0;
}

extern "C" int ecospa_contract(ecospa_ctx* ctx, int dtype, int M, int N, int K, const void* A, long long lda,
                               int trans_a, const void* B, long long ldb, int trans_b, void* C, long long ldc,
                               const void* bias, int tile, int splits) {
  if (!ctx || !A || !B || !C) return ECOSPA_ERR_NULL;
  if (!dtype_ok(dtype)) return ECOSPA_ERR_DTYPE;
  if (M < 1 || N < 1 || K < 1 || tile < 0 || tile > 38 || (tile > 21 && tile < 30) || splits < 0 || splits > 64) return ECOSPA_ERR_SHAPE;
  if (lda < (trans_a ? M : K) || ldb < (trans_b ? N : K) || ldc < N) return ECOSPA_ERR_SHAPE;
  GemmDesc g = gemm_desc(dtype, M, N, K, A, lda, trans_a ? 1 : 0, B, ldb, trans_b ? 1 : 0);
  g.tile = tile;
  g.splits = splits == 0 ? ecospa_gemm_splits(M, N, K) : splits;
  g.epi.kind = EPI_STORE; g.epi.c = C; g.epi.ldc = ldc; g.epi.bias = bias;
  if (g.splits > 1) {
    const size_t need = static_cast<size_t>(g.splits) * M * N * 4;
    if (!ctx->ws || ctx->ws_bytes < need) return ECOSPA_ERR_WORKSPACE;
    g.partial = static_cast<float*>(ctx->ws);
  }
  return ecospa_gemm(ctx, g);
}

// dY^T X with the column sums of its K-slow A operand (the bias gradient that belongs to the weight gradient), as the
// backward passes use it; exposed for tests of every tile shape.
extern "C" int ecospa_contract_colsum(ecospa_ctx* ctx, int M, int N, int K, const void* A, long long lda, const void* B,
                                      long long ldb, void* C, long long ldc, float* colsum, int tile, int splits) {
  if (!ctx || !A || !B || !C || !colsum) return ECOSPA_ERR_NULL;
  if (M < 1 || N < 1 || K < 1 || tile < 0 || tile > 38 || (tile > 21 && tile < 30) || splits < 0 || splits > 64) return ECOSPA_ERR_SHAPE;
  if (lda < M || ldb < N || ldc < N) return ECOSPA_ERR_SHAPE;
  GemmDesc g = gemm_desc(ECOSPA_BF16, M, N, K, A, lda, 1, B, ldb, 1);
  g.splits = splits == 0 ? ecospa_gemm_splits(M, N, K) : splits;
  const int sp = g.splits > 1 ? g.splits : 1;
  g.epi.kind = EPI_STORE; g.epi.c = C; g.epi.ldc = ldc;
  g.tile = tile;
  // workspace: [rows][M] partial column sums, then the fp32 partial products of a split contraction
  const int rows = ecospa_gemm_colsum_rows(g);
  const size_t cs_bytes = align_up(static_cast<size_t>(rows) * M * 4, 256);
  const size_t need = cs_bytes + (sp > 1 ? static_cast<size_t>(sp) * M * N * 4 : 0);
  if (!ctx->ws || ctx->ws_bytes < need) return ECOSPA_ERR_WORKSPACE;
  g.colsum = static_cast<float*>(ctx->ws);
  if (sp > 1) { g.partial = reinterpret_cast<float*>(static_cast<char*>(ctx->ws) + cs_bytes); g.defer_reduce = 1; }
  const int rc = ecospa_gemm(ctx, g);
  if (rc) return rc;
  AuxBatch aux;
  memset(&aux, 0, sizeof(aux));
  if (sp > 1) aux.reduce[aux.n_reduce++] = g;
  aux.colsum[aux.n_colsum++] = AuxColsum{g.colsum, M, rows, M, ECOSPA_F32, colsum, ECOSPA_F32};
  return ecospa_aux_launch(ctx, aux);
}
