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

#include "select_dev.h"

#define SELECT_CACHE 8          // scores a thread of the threshold kernel keeps in registers

__global__ __launch_bounds__(SELECT_THREADS) void select_topk_kernel(const SelectBatch b) {
  __shared__ SelectShared sh;
  int item = 0, hi = b.n_items - 1;       // last item whose first block is <= blockIdx.x
  while (item < hi) {
    const int mid = (item + hi + 1) >> 1;
    if (b.first_blk[mid] <= static_cast<int>(blockIdx.x)) item = mid; else hi = mid - 1;
  }
  const SelectItemDev& t = b.it[item];
  select_item_block(t, static_cast<int>(blockIdx.x) - t.blk_begin, sh);
}


// ---------------------------------------------------------------------------------------------
// Cumulative-threshold rule (Alg. 1's inner loop): how many units of a group stay when the smallest
// scores are removed for as long as the rest still holds the fraction theta of the group's total.
// Scores become integer masses (floor(clip(s, 0, 1) * 2^32), NaN -> 0), so every sum is exact and the
// count does not depend on the order of summation.  The removable mass R = total - ceil(theta * total)
// is spent in ascending key order: a 4-pass, 8-bit radix descent over (count, mass) histograms finds the
// first key that cannot be removed entirely; of the units with exactly that key (equal masses) as many go
// as R still covers.  The kept set is then the top-k of the same ordering, written by select_topk_kernel.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long theta_mass(float x) {
  if (!(x > 0.f)) return 0ull;                       // negative, zero, NaN
  const double v = fmin(static_cast<double>(x), 1.0) * 4294967296.0;
  return static_cast<unsigned long long>(v);         // exact: a float times 2^32, truncated
}
struct ThetaItemDev {
  const float* scores;
  int* k_out;
  int n;
  float theta;
};
__global__ __launch_bounds__(SELECT_THREADS) void select_theta_count_kernel(const ThetaItemDev t) {
  __shared__ unsigned long long wsum[SELECT_THREADS / 64][256];   // per wavefront: see select_topk_kernel
  __shared__ int wcnt[SELECT_THREADS / 64][256];
  __shared__ unsigned long long hsum[256], csum[256];
  __shared__ int hcnt[256], ccnt[256];
  __shared__ unsigned long long s_total, s_rem;
  __shared__ uint32_t s_prefix;
  __shared__ int s_below, s_digit;
  const int tid = threadIdx.x, g = blockIdx.x, n = t.n;
  const float* s = t.scores + static_cast<long long>(g) * n;
  const int per = (n + SELECT_THREADS - 1) / SELECT_THREADS;
  const int i0 = min(tid * per, n), i1 = min(i0 + per, n);
  const bool cached = per <= SELECT_CACHE;
  float vc[SELECT_CACHE];
  if (cached) {
#pragma unroll
    for (int j = 0; j < SELECT_CACHE; ++j) vc[j] = i0 + j < i1 ? s[i0 + j] : 0.f;
  }
  if (tid == 0) s_total = 0ull;
  __syncthreads();
  unsigned long long mine = 0ull;
  if (cached) {
#pragma unroll
    for (int j = 0; j < SELECT_CACHE; ++j) mine += i0 + j < i1 ? theta_mass(vc[j]) : 0ull;
  } else {
    for (int i = i0; i < i1; ++i) mine += theta_mass(s[i]);
  }
  if (mine) atomicAdd(&s_total, mine);
  __syncthreads();
  const unsigned long long total = s_total;
  const double bound_d = ceil(static_cast<double>(t.theta) * static_cast<double>(total));
  const unsigned long long bound = bound_d <= 0.0 ? 0ull : static_cast<unsigned long long>(bound_d);
  unsigned long long rem = bound >= total ? 0ull : total - bound;   // mass that may be removed
  uint32_t prefix = 0u;
  int below = 0;             // units removed so far (keys below the range being refined)
  int digit = 0;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int i = tid; i < (SELECT_THREADS / 64) * 256; i += SELECT_THREADS) {
      (&wsum[0][0])[i] = 0ull;
      (&wcnt[0][0])[i] = 0;
    }
    __syncthreads();
#pragma unroll 1
    for (int i = i0; i < i1; ++i) {
      float x;
      if (cached) {
        x = vc[0];
#pragma unroll
        for (int j = 1; j < SELECT_CACHE; ++j) x = (i - i0 == j) ? vc[j] : x;
      } else {
        x = s[i];
      }
      const uint32_t key = score_key(x);
      if ((key & hi_mask) == prefix) {
        const int d = (key >> shift) & 255u;
        atomicAdd(&wcnt[tid >> 6][d], 1);
        const unsigned long long q = theta_mass(x);
        if (q) atomicAdd(&wsum[tid >> 6][d], q);
      }
    }
    __syncthreads();
    if (tid < 256) {
      unsigned long long m = 0ull;
      int c = 0;
#pragma unroll
      for (int w = 0; w < SELECT_THREADS / 64; ++w) { m += wsum[w][tid]; c += wcnt[w][tid]; }
      hsum[tid] = m;
      hcnt[tid] = c;
    }
    __syncthreads();
    // inclusive prefix sums over the digits (ascending keys); the first digit whose cumulative mass
    // exceeds what may still be removed is the one that cannot go entirely
    if (tid < 256) { csum[tid] = hsum[tid]; ccnt[tid] = hcnt[tid]; }
    if (tid == 0) s_digit = 256;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
      unsigned long long vm = 0ull;
      int vc = 0;
      if (tid < 256 && tid >= off) { vm = csum[tid - off]; vc = ccnt[tid - off]; }
      __syncthreads();
      if (tid < 256) { csum[tid] += vm; ccnt[tid] += vc; }
      __syncthreads();
    }
    if (tid < 256) {
      const unsigned long long incl = csum[tid], excl = incl - hsum[tid];
      if (incl > rem && excl <= rem) {      // exactly one digit, if any
        s_digit = tid;
        s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
        s_rem = rem - excl;
        s_below = below + ccnt[tid] - hcnt[tid];
      }
    }
    __syncthreads();
    digit = s_digit;
    prefix = s_prefix;
    rem = s_rem;
    below = s_below;
    if (digit == 256) break;      // (first pass only) everything may go: uniform, no barrier follows
  }
  if (tid == 0) {
    int removed;
    if (digit == 256) {
      removed = n;
    } else {
      // units whose key equals `prefix` share one mass
      const int c_eq = hcnt[digit];
      const unsigned long long qk = c_eq > 0 ? hsum[digit] / static_cast<unsigned long long>(c_eq) : 0ull;
      const unsigned long long can = qk == 0ull ? static_cast<unsigned long long>(c_eq) : rem / qk;
      removed = below + static_cast<int>(can < static_cast<unsigned long long>(c_eq) ? can : c_eq);
    }
    const int k = n - removed;
    t.k_out[g] = k < 1 ? 1 : k;
  }
}

// Workgroups of an item: one per group, or one per SELECT_THREADS / 64 small groups (a wavefront each).
static int select_blocks(int groups, int n_units) {
  return n_units <= 64 ? (groups + SELECT_THREADS / 64 - 1) / (SELECT_THREADS / 64) : groups;
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
      b.it[i] = SelectItemDev{q.scores, q.idx, q.n_units, q.k, static_cast<int>(blk), q.groups, nullptr, 0, 0};
      b.first_blk[i] = static_cast<int>(blk);
      blk += select_blocks(q.groups, q.n_units);
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

extern "C" int ecospa_select_theta(ecospa_ctx* ctx, const float* scores, int groups, int n_units, float theta, int* idx,
                                   int* k_out) {
  if (!ctx || !scores || !idx || !k_out) return ECOSPA_ERR_NULL;
  if (groups < 1 || n_units < 1 || groups > (1 << 30)) return ECOSPA_ERR_SHAPE;
  if (!(theta >= 0.f && theta <= 1.f)) return ECOSPA_ERR_K;
  hipLaunchKernelGGL(select_theta_count_kernel, dim3(groups), dim3(SELECT_THREADS), 0, ctx->stream,
                     ThetaItemDev{scores, k_out, n_units, theta});
  ECOSPA_CHECK_LAUNCH(ctx, "select_theta_count_kernel");
  SelectBatch b;
  memset(&b, 0, sizeof(b));
  b.n_items = 1;
  b.it[0] = SelectItemDev{scores, idx, n_units, 0, 0, groups, k_out, n_units, 0};
  hipLaunchKernelGGL(select_topk_kernel, dim3(select_blocks(groups, n_units)), dim3(SELECT_THREADS), 0, ctx->stream, b);
  ECOSPA_CHECK_LAUNCH(ctx, "select_topk_kernel");
  return ECOSPA_OK;
}

// Alg. 1's choice among the coupled pairs: the n_select pairs with the smallest importance (Eq. 8).
extern "C" int ecospa_select_pairs(ecospa_ctx* ctx, const float* fisher, int n_pairs, int n_select, int* chosen) {
  if (!ctx || !fisher || !chosen) return ECOSPA_ERR_NULL;
  if (n_pairs < 1) return ECOSPA_ERR_SHAPE;
  if (n_select < 1 || n_select > n_pairs) return ECOSPA_ERR_K;
  SelectBatch b;
  memset(&b, 0, sizeof(b));
  b.n_items = 1;
  b.it[0] = SelectItemDev{fisher, chosen, n_pairs, n_select, 0, 1, nullptr, 0, 1};
  hipLaunchKernelGGL(select_topk_kernel, dim3(1), dim3(SELECT_THREADS), 0, ctx->stream, b);
  ECOSPA_CHECK_LAUNCH(ctx, "select_topk_kernel");
  return ECOSPA_OK;
}
