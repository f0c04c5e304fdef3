// Step 2: deterministic block-wide top-k (Sec. 3.2 "rank upsilon_i"; Alg. 1 removal loop).
//
// One workgroup per group.  Scores are mapped to order-preserving 32-bit keys
// (-0 == +0, NaN below everything).  A 4-pass, 8-bit radix select finds the k-th largest key T
// and how many elements equal to T are still to be taken; a final pass in index order keeps
// every element above T plus the lowest-index ties, and writes the kept indices ascending with a
// block-wide prefix sum.  Only integer comparisons and integer LDS atomics: bit-exact.
#include "common.h"

#define SELECT_THREADS 256

__device__ __forceinline__ uint32_t score_key(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN: lowest
  if (u == 0x80000000u) u = 0u;                      // -0 -> +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix count of `flag` over the block's threads in thread order, and the block total.
__device__ __forceinline__ int block_prefix_count(bool flag, int* wave_tot, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long m = __ballot(flag);
  const int within = __popcll(m & ((1ull << lane) - 1ull));
  __syncthreads();   // protect wave_tot from the previous use
  if (lane == 0) wave_tot[wave] = __popcll(m);
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SELECT_THREADS / 64; ++w) {
    const int c = wave_tot[w];
    if (w < wave) before += c;
    tot += c;
  }
  total = tot;
  return before + within;
}

__global__ __launch_bounds__(SELECT_THREADS) void select_topk_kernel(const float* __restrict__ scores, int n, int k,
                                                                     int* __restrict__ idx) {
  __shared__ int hist[257];
  __shared__ int wave_tot[SELECT_THREADS / 64];
  __shared__ uint32_t s_prefix;
  __shared__ int s_krem;
  const int tid = threadIdx.x;
  const float* s = scores + static_cast<long long>(blockIdx.x) * n;
  int* out = idx + static_cast<long long>(blockIdx.x) * k;

  uint32_t prefix = 0u;   // high bits of the k-th largest key found so far
  int krem = k;           // rank (1-based) of the wanted key among keys matching the prefix
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    hist[tid] = 0;
    if (tid == 0) hist[256] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += SELECT_THREADS) {
      const uint32_t key = score_key(s[i]);
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    // suffix sums: hist[t] = number of matching keys with digit >= t
    for (int off = 1; off < 256; off <<= 1) {
      const int v = (tid + off < 256) ? hist[tid + off] : 0;
      __syncthreads();
      hist[tid] += v;
      __syncthreads();
    }
    if (hist[tid] >= krem && hist[tid + 1] < krem) {   // exactly one thread
      s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
      s_krem = krem - hist[tid + 1];
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    __syncthreads();
  }
  const uint32_t T = prefix;   // k-th largest key; take `krem` of the elements equal to it

  int eq_seen = 0, taken = 0;
  for (int base = 0; base < n; base += SELECT_THREADS) {
    const int i = base + tid;
    const uint32_t key = i < n ? score_key(s[i]) : 0u;
    const bool eq = i < n && key == T;
    const bool gt = i < n && key > T;
    int eq_tot, take_tot;
    const int eq_rank = eq_seen + block_prefix_count(eq, wave_tot, eq_tot);
    const bool take = gt || (eq && eq_rank < krem);
    const int pos = taken + block_prefix_count(take, wave_tot, take_tot);
    if (take && pos < k) out[pos] = i;
    eq_seen += eq_tot;
    taken += take_tot;
  }
}

extern "C" int ecospa_select_topk(ecospa_ctx* ctx, const float* scores, int groups, int n_units, int k, int* idx) {
  if (!ctx || !scores || !idx) return ECOSPA_ERR_NULL;
  if (groups < 1 || n_units < 1) return ECOSPA_ERR_SHAPE;
  if (k < 1 || k > n_units) return ECOSPA_ERR_K;
  hipLaunchKernelGGL(select_topk_kernel, dim3(groups), dim3(SELECT_THREADS), 0, ctx->stream, scores, n_units, k, idx);
  ECOSPA_CHECK_LAUNCH(ctx, "select_topk_kernel");
  return ECOSPA_OK;
}
