// Internal: per-block orchestration shared by block.hip (FFN, dispatch) and attn.hip.
#pragma once
#include "common.h"
#include "gemm.h"

struct BlockWs {           // pieces carved from the caller's workspace
  // FFN
  void* dh;                // [T, (1|2)*kp_ff]
  void* hpre_tmp;          // inference only
  void* act_tmp;
  // ATTN
  void* qkv_tmp;           // inference only
  void* o_tmp;
  float* lse_tmp;
  void* dqkv;              // [T, nqkv]
  void* d_o;               // [T, h*kp_vo]
  float* delta;            // [B*h*L]
  // shared
  float* partial;          // split-K partials of the first weight-gradient contraction of a backward pass
  float* partial2;         // ... and of the second (both are reduced by the batched tail launch)
  float* colsum;           // [rows][M] partial operand column sums of the first weight-gradient contraction (bias gradient)
  float* colsum2;          // ... and of the second
  float* partial_x;        // split-K partials of a forward or input-gradient contraction (few tokens only), one at a time
  size_t total;
};

// K split of a contraction over few tokens (x W^T, dY W): partials from the workspace, reduced right after the launch.
static inline void block_token_split(GemmDesc& g, const BlockWs& w) {
  const int s = g.dtype == ECOSPA_BF16 ? ecospa_gemm_token_splits(g.M, g.N, g.K) : 1;
  if (s > 1 && w.partial_x) { g.splits = s; g.partial = w.partial_x; }
}
static inline size_t block_token_split_bytes(int M, int N, int K) {
  const int s = ecospa_gemm_token_splits(M, N, K);
  return s > 1 ? static_cast<size_t>(s) * M * N * 4 : 0;
}

int block_colsum_rows(int dtype, int M, int N, int K);

// Lay out the workspace for a validated descriptor; base may be NULL to only measure.
void block_ws_layout(const ecospa_block_desc& d, void* base, BlockWs& w);

int attn_forward(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x, void* y,
                 const ecospa_saved* saved);
int attn_backward(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x, const void* dy,
                  const ecospa_saved& saved, void* dx, const ecospa_grads& g);

// key/value heads: fewer than query heads under grouped-query attention (Eq. 5)
static inline int attn_h_kv(const ecospa_block_desc& d) { return d.h_kv > 0 ? d.h_kv : d.h; }
static inline int attn_nqkv(const ecospa_block_desc& d) { return (d.h + attn_h_kv(d)) * d.kp_qk + attn_h_kv(d) * d.kp_vo; }
