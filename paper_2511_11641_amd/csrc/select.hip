// Step 2: deterministic block-wide top-k (Sec. 3.2 "rank upsilon_i"; Alg. 1 removal loop).
//
// One workgroup per group; all groups of a batch of score arrays share one launch.  Scores are
// mapped to order-preserving 32-bit keys (-0 == +0, NaN below everything).  A 4-pass, 8-bit radix
// select with LDS integer histograms finds the k-th largest key T and how many elements equal to T
// are still to be taken.  Then every thread walks its own contiguous run of indices: two block-wide
// exclusive scans (ties seen before the run, elements kept before the run) give the output position
// of everything it keeps, so the kept indices come out ascending and ties go to the lower index.
// Only integer comparisons, integer LDS atomics and integer scans: bit-exact.
#include "common.h"

#define SELECT_THREADS 1024
#define SELECT_MAX_ITEMS 96    // descriptors travel as kernel arguments

struct SelectItemDev {
  const float* scores;
  int* idx;
  int n, k;
  int blk_begin;   // first workgroup (= group) of this item
};
struct SelectBatch {
  int n_items;
  SelectItemDev it[SELECT_MAX_ITEMS];
};

__device__ __forceinline__ uint32_t score_key(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN: lowest
  if (u == 0x80000000u) u = 0u;                      // -0 -> +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum of `v` over the block's threads in thread order, and the block total.
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(inc, off, 64);
    if (lane >= off) inc += up;
  }
  __syncthreads();   // protect wave_tot from the previous use
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SELECT_THREADS / 64; ++w) {
    const int c = wave_tot[w];
    if (w < wave) before += c;
    tot += c;
  }
  total = tot;
  return before + inc - v;
}

__global__ __launch_bounds__(SELECT_THREADS) void select_topk_kernel(const SelectBatch b) {
  __shared__ int hist[257];
  __shared__ int wave_tot[SELECT_THREADS / 64];
  __shared__ uint32_t s_prefix;
  __shared__ int s_krem;
  const int tid = threadIdx.x;
  int item = 0, hi = b.n_items - 1;       // last item whose first block is <= blockIdx.x
  while (item < hi) {
    const int mid = (item + hi + 1) >> 1;
    if (b.it[mid].blk_begin <= static_cast<int>(blockIdx.x)) item = mid; else hi = mid - 1;
  }
  const SelectItemDev& t = b.it[item];
  const int n = t.n, k = t.k, g = blockIdx.x - t.blk_begin;
  const float* s = t.scores + static_cast<long long>(g) * n;
  int* out = t.idx + static_cast<long long>(g) * k;

  uint32_t prefix = 0u;   // high bits of the k-th largest key found so far
  int krem = k;           // rank (1-based) of the wanted key among keys matching the prefix
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    if (tid <= 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += SELECT_THREADS) {
      const uint32_t key = score_key(s[i]);
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    // suffix sums: hist[d] = number of matching keys with digit >= d
    for (int off = 1; off < 256; off <<= 1) {
      const int v = (tid < 256 && tid + off < 256) ? hist[tid + off] : 0;
      __syncthreads();
      if (tid < 256) hist[tid] += v;
      __syncthreads();
    }
    if (tid < 256 && hist[tid] >= krem && hist[tid + 1] < krem) {   // exactly one thread
      s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
      s_krem = krem - hist[tid + 1];
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    __syncthreads();
  }
  const uint32_t T = prefix;   // k-th largest key; take `krem` of the elements equal to it

  // this thread's contiguous run of indices
  const int per = (n + SELECT_THREADS - 1) / SELECT_THREADS;
  const int i0 = min(tid * per, n), i1 = min(i0 + per, n);
  int n_eq = 0, n_gt = 0;
  for (int i = i0; i < i1; ++i) {
    const uint32_t key = score_key(s[i]);
    n_eq += key == T;
    n_gt += key > T;
  }
  int tot;
  const int eq_before = block_exclusive_scan(n_eq, wave_tot, tot);
  const int eq_take = max(0, min(n_eq, krem - eq_before));       // ties of this run that are kept
  int pos = block_exclusive_scan(n_gt + eq_take, wave_tot, tot);
  int eq_left = eq_take;
  for (int i = i0; i < i1; ++i) {
    const uint32_t key = score_key(s[i]);
    bool take = key > T;
    if (key == T && eq_left > 0) { take = true; --eq_left; }
    if (take && pos < k) out[pos++] = i;
  }
}

static int validate_select(const ecospa_select_item& q) {
  if (!q.scores || !q.idx) return ECOSPA_ERR_NULL;
  if (q.groups < 1 || q.n_units < 1) return ECOSPA_ERR_SHAPE;
  if (q.k < 1 || q.k > q.n_units) return ECOSPA_ERR_K;
  return ECOSPA_OK;
}

extern "C" int ecospa_select_topk_batch(ecospa_ctx* ctx, const ecospa_select_item* items, int n_items) {
  if (!ctx || !items) return ECOSPA_ERR_NULL;
  if (n_items < 1) return ECOSPA_ERR_SHAPE;
  for (int i = 0; i < n_items; ++i) {
    const int rc = validate_select(items[i]);
    if (rc) return rc;
  }
  for (int first = 0; first < n_items; first += SELECT_MAX_ITEMS) {
    SelectBatch b;
    memset(&b, 0, sizeof(b));
    b.n_items = n_items - first < SELECT_MAX_ITEMS ? n_items - first : SELECT_MAX_ITEMS;
    long long blk = 0;
    for (int i = 0; i < b.n_items; ++i) {
      const ecospa_select_item& q = items[first + i];
      b.it[i] = SelectItemDev{q.scores, q.idx, q.n_units, q.k, static_cast<int>(blk)};
      blk += q.groups;
      if (blk > (1ll << 30)) return ECOSPA_ERR_SHAPE;
    }
    hipLaunchKernelGGL(select_topk_kernel, dim3(static_cast<unsigned>(blk)), dim3(SELECT_THREADS), 0, ctx->stream, b);
    ECOSPA_CHECK_LAUNCH(ctx, "select_topk_kernel");
  }
  return ECOSPA_OK;
}

extern "C" int ecospa_select_topk(ecospa_ctx* ctx, const float* scores, int groups, int n_units, int k, int* idx) {
  if (!ctx) return ECOSPA_ERR_NULL;
  const ecospa_select_item q{scores, groups, n_units, k, idx};
  return ecospa_select_topk_batch(ctx, &q, 1);
}
