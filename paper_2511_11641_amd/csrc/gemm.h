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
  EPI_DSWIGLU = 3,   // g = h[m,n], u = h[m,n+kp]; c[m,n] = acc*u*dsilu(g); c[m,n+kp] = acc*silu(g)
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
  GemmEpi epi;
};

// Launch on ctx->stream.  bf16 runs on MFMA tiles; fp32 on a vector-ALU tile kernel.
int ecospa_gemm(ecospa_ctx* ctx, const GemmDesc& d);
// How many K splits a (M, N, K) problem should use to fill the chip, and the bytes of partials.
int ecospa_gemm_splits(int M, int N, int K);

// out[n] = sum_m X[m, n] for n < N (bias gradients); deterministic two-stage reduction.
// partial: float[ecospa_colsum_chunks(M)][N].
int ecospa_colsum_chunks(int M);
int ecospa_colsum(ecospa_ctx* ctx, int dtype, const void* X, long long ldx, int M, int N, float* partial, void* out);

// Activation helpers shared by the epilogues and the elementwise kernels.
#ifdef __HIPCC__
__device__ __forceinline__ float act_gelu(float x, int act) {
  if (act == ECOSPA_ACT_GELU_TANH) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.f + tanhf(u));
  }
  return 0.5f * x * (1.f + erff(x * 0.7071067811865476f));
}
__device__ __forceinline__ float act_gelu_grad(float x, int act) {
  if (act == ECOSPA_ACT_GELU_TANH) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    const float th = tanhf(u);
    return 0.5f * (1.f + th) + 0.5f * x * (1.f - th * th) * 0.7978845608028654f * (1.f + 0.134145f * x * x);
  }
  const float cdf = 0.5f * (1.f + erff(x * 0.7071067811865476f));
  const float pdf = 0.3989422804014327f * __expf(-0.5f * x * x);
  return cdf + x * pdf;
}
__device__ __forceinline__ float act_sigmoid(float x) { return 1.f / (1.f + __expf(-x)); }
#endif
