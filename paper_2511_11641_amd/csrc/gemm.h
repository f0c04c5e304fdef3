// Internal GEMM interface of the gfx950 library (not part of the C ABI).
//
//   C[m, n] = sum_k A(m, k) * B(n, k),   m < M, n < N, k < K
//   A(m, k) = A[m * lda + k]   (trans_a = 0, K contiguous)   or   A[k * lda + m]   (trans_a = 1)
//   B(n, k) = B[n * ldb + k]   (trans_b = 0, K contiguous)   or   B[k * ldb + n]   (trans_b = 1)
// so  X W^T  is (0, 0),  dY W  is (0, 1)  and  dY^T X  is (1, 1).
// Accumulation is fp32; the epilogue decides what is written.
#pragma once
#include "common.h"

enum {
  EPI_STORE = 0,     // c[m,n] = acc (+ bias[n])
  EPI_BIAS_ACT = 1,  // h = acc + bias[n]; c[m,n] = h; c2[m,n] = gelu(h)
  EPI_DACT = 2,      // c[m,n] = acc * gelu'(h[m,n])
  EPI_DSWIGLU = 3,   // unit n: g = h[m,2n], u = h[m,2n+1] (interleaved pairs); c[m,2n] = acc*u*dsilu(g); c[m,2n+1] = acc*silu(g)
  EPI_ACT = 4,       // c[m,n] = gelu(acc + bias[n]): forward only, the activation's input is not kept
  EPI_ROPE = 5,      // c[m,n] = acc + bias[n], with the adjacent column pairs (2i, 2i+1) of the first rope_cols columns
                     // turned by the angle of (row m % rope_L, pair) - the rotary form of the Q and K projections (bf16)
  EPI_SWIGLU = 6,    // columns come in (gate, up) pairs: h = acc (+ bias) is stored to c[m, n] (2 kp wide, when c is
                     // set) and silu(gate) * up to c2[m, n / 2] (kp wide) - the gated FFN's first contraction (bf16)
};

struct GemmEpi {
  int kind, act;
  void* c;
  long long ldc;
  const void* bias;
  void* c2;
  long long ldc2;
  const void* h;
  long long ldh;
  int kp;
  // EPI_ROPE: cos/sin tables float[rope_rows][rope_L][rope_kp / 2]; column n < rope_cols belongs to head n / rope_kp,
  // the query heads (the first rope_hq heads) share the table row of their key/value head: row head / rope_qpk for a
  // query head, head - rope_hq for a key head
  const float *rope_cos, *rope_sin;
  int rope_cols, rope_kp, rope_L, rope_hq, rope_qpk;
};

struct GemmDesc {
  int dtype;
  int M, N, K;
  const void* A;
  long long lda;
  int trans_a;
  const void* B;
  long long ldb;
  int trans_b;
  int tile;          // 0 = choose, 1 = 128x128 workgroup tiles, 2 = 256x256
  int splits;        // > 1: split K, fp32 partials in `partial`, reduced in a fixed order
  float* partial;    // [splits][M][N] when splits > 1
  int defer_reduce;  // splits > 1: only write the partials; the caller runs ecospa_gemm_reduce later
  float* colsum;     // optional, bf16 contractions with a K-slow A operand (dY^T X): [ecospa_gemm_colsum_rows(d)][M] partial
                     // column sums of A, sum_k A(m, k) over disjoint parts of K - the bias gradient that belongs to the
                     // weight gradient, taken from the operand on its way through the registers; the rows add up to the sums
  GemmEpi epi;
};

// Launch on ctx->stream.  bf16 runs on MFMA tiles; fp32 on a vector-ALU tile kernel.
int ecospa_gemm(ecospa_ctx* ctx, const GemmDesc& d);
// Rows (of M floats) of the partial column sums that the launch of d writes to d.colsum.
int ecospa_gemm_colsum_rows(const GemmDesc& d);
// Second half of a split-K contraction launched with defer_reduce: fixed-order sum of the partials,
// then the epilogue.  Same descriptor as the first half.
int ecospa_gemm_reduce(ecospa_ctx* ctx, const GemmDesc& d);
// How many K splits a (M, N, K) problem should use to fill the chip, and the bytes of partials.
int ecospa_gemm_splits(int M, int N, int K);
// The same question for the contractions whose M is the token count (x W^T and dY W): with few tokens (inference
// at batch 1) their output has too few tiles for the chip, and K is split until the 128x128 tiles reach a
// workgroup per compute unit, keeping at least 1024 of K per split (shorter splits lose more to the partial sums
// than they gain: measured on the batch-1 forward of the 24-layer stack); 1 for the training shapes.
int ecospa_gemm_token_splits(int M, int N, int K);

// Software-pipelined kernel for full K slabs (gemm_pipe.hip): configurations 0 .. GEMM_PIPE_CONFIGS-1
// differ in workgroup tile, slab depth and LDS ring length; d.tile = 10 + configuration forces one.
#define GEMM_PIPE_CONFIGS 11
bool gemm_pipe_ok(const GemmDesc& d, int cfg, int k_chunk);
hipError_t gemm_pipe_launch(ecospa_ctx* ctx, const GemmDesc& d, int cfg, int k_chunk);
int gemm_pipe_bk(int cfg);

// Register-staged kernel with a two-slab prefetch (gemm_rs.hip): bm x bn x 64 tiles, four wavefronts.
// 256 x 256: A K-contiguous with B either way, or both K-slow; the narrower shapes (bm, bn from 128, 192, 256)
// are built for dY^T X only.  d.tile = 20 forces 256 x 256, d.tile = 30 + i shape i of GEMM_RS_SHAPES.
bool gemm_rs_ok(const GemmDesc& d, int k_chunk);
bool gemm_rs_shape_ok(int bm, int bn);
hipError_t gemm_rs_launch(ecospa_ctx* ctx, const GemmDesc& d, int k_chunk, int bm, int bn);
#define GEMM_RS_NSHAPES 9
static const int GEMM_RS_SHAPES[GEMM_RS_NSHAPES][2] = {{256, 256}, {192, 256}, {256, 192}, {128, 256}, {256, 128},
                                                       {192, 192}, {128, 192}, {192, 128}, {128, 128}};
// Plan of a weight-gradient contraction dY^T X (M x N outputs, K = tokens): tile shape and number of K splits that
// finish soonest on 256 compute units by a cost model fitted to measurements; false if the problem does not suit
// the kernel (K not a multiple of 64, too short).
bool gemm_tt_plan(int M, int N, int K, int* bm, int* bn, int* splits);

// The small jobs that follow the contractions of a backward pass, batched into ONE launch (each of
// them alone would be bound by the fixed cost of a launch): fixed-order reductions of split-K
// partials (a GemmDesc launched with defer_reduce) and bias gradients out[n] = sum_m X[m, n].
// A column sum is done by one workgroup per strip of columns over all rows - no second pass.
#define AUX_MAX_JOBS 4
struct AuxColsum {
  const void* X;
  long long ldx;
  int M, N, dtype;
  void* out;
  int out_dtype;     // 0: as X; otherwise the type of `out` (fp32 partial sums reduced into a bf16 gradient)
};
struct AuxBatch {
  int n_reduce, n_colsum;
  GemmDesc reduce[AUX_MAX_JOBS];
  AuxColsum colsum[AUX_MAX_JOBS];
};
int ecospa_aux_launch(ecospa_ctx* ctx, const AuxBatch& b);

// Activation helpers shared by the epilogues and the elementwise kernels.
#ifdef __HIPCC__
// Standard normal CDF by the rational approximation 7.1.26 of Abramowitz & Stegun for erfc
// (absolute error about 3e-7 in Phi when evaluated in fp32: far below bf16 resolution, and a relative Frobenius error near 1e-7 on GELU outputs), written on the
// tail Phi(-|x|) so that negative arguments lose nothing to cancellation: one reciprocal, one
// exponential and a degree-5 Horner chain instead of the library erf.  `e` returns exp(-x^2 / 2),
// which the derivative needs as well.
__device__ __forceinline__ float act_norm_cdf(float x, float& e) {
  const float z = fabsf(x) * 0.7071067811865476f;
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, z, 1.f));
  float p = __builtin_fmaf(1.061405429f, t, -1.453152027f);
  p = __builtin_fmaf(p, t, 1.421413741f);
  p = __builtin_fmaf(p, t, -0.284496736f);
  p = __builtin_fmaf(p, t, 0.254829592f);
  e = __expf(-z * z);
  const float tail = 0.5f * p * t * e;   // Phi(-|x|)
  return x < 0.f ? tail : 1.f - tail;
}
__device__ __forceinline__ float act_gelu(float x, int act) {
  if (act == ECOSPA_ACT_GELU_TANH) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.f + tanhf(u));
  }
  float e;
  return x * act_norm_cdf(x, e);
}
__device__ __forceinline__ float act_gelu_grad(float x, int act) {
  if (act == ECOSPA_ACT_GELU_TANH) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    const float th = tanhf(u);
    return 0.5f * (1.f + th) + 0.5f * x * (1.f - th * th) * 0.7978845608028654f * (1.f + 0.134145f * x * x);
  }
  float e;
  const float cdf = act_norm_cdf(x, e);
  return cdf + x * (0.3989422804014327f * e);
}
__device__ __forceinline__ float act_sigmoid(float x) { return 1.f / (1.f + __expf(-x)); }
#endif
