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
#define SELECT_CACHE 8          // score keys a thread keeps in registers
#define SELECT_MAX_ITEMS 96    // descriptors travel as kernel arguments

struct SelectItemDev {
  const float* scores;
  int* idx;
  int n, k;
  int blk_begin;   // first workgroup (= group) of this item
  int groups;        // groups of this item (n <= 64: SELECT_THREADS / 64 of them share a workgroup)
  const int* k_dev;  // optional: per-group kept counts in device memory (then k is unused, the rows of idx
  int ld_idx;        //           are ld_idx apart and the slots behind the kept indices are set to -1)
  int smallest;      // take the k smallest scores instead (the order of the keys reversed, ties still to the lower index)
};
struct SelectBatch {
  int n_items;
  int first_blk[SELECT_MAX_ITEMS];   // blk_begin of every item, side by side: the search for a group's item stays in a few cache lines
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

#define ITEM_KEY(x) (score_key(x) ^ flip)
__global__ __launch_bounds__(SELECT_THREADS) void select_topk_kernel(const SelectBatch b) {
  // one histogram per wavefront: normalised scores share their top key bits, so a single histogram
  // would serialise nearly every atomic of the first pass on a few counters
  __shared__ int whist[SELECT_THREADS / 64][256];
  __shared__ int hist[257];
  __shared__ int wave_tot[SELECT_THREADS / 64];
  __shared__ uint32_t s_prefix;
  __shared__ int s_krem;
  const int tid = threadIdx.x, wave = tid >> 6;
  int item = 0, hi = b.n_items - 1;       // last item whose first block is <= blockIdx.x
  while (item < hi) {
    const int mid = (item + hi + 1) >> 1;
    if (b.first_blk[mid] <= static_cast<int>(blockIdx.x)) item = mid; else hi = mid - 1;
  }
  const SelectItemDev& t = b.it[item];
  const uint32_t flip = t.smallest ? 0xffffffffu : 0u;
  if (t.n <= 64) {
    // Small groups (the units of one head): a wavefront ranks a group by direct comparison - the rank of
    // a unit is the number of units that come before it in the order (larger key, or equal key and lower
    // index) - and the lanes whose rank is below k write their indices, ascending.  One group per wavefront.
    const int g = (static_cast<int>(blockIdx.x) - t.blk_begin) * (SELECT_THREADS / 64) + wave;
    if (g >= t.groups) return;
    const int lane = tid & 63, n = t.n;
    const int k = t.k_dev ? t.k_dev[g] : t.k;
    const uint32_t key = lane < n ? ITEM_KEY(t.scores[static_cast<long long>(g) * n + lane]) : 0u;
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const uint32_t kj = __shfl(key, j, 64);
      rank += (kj > key) || (kj == key && j < lane);
    }
    const bool take = lane < n && rank < k;
    const unsigned long long mask = __ballot(take);
    int* out = t.idx + static_cast<long long>(g) * (t.k_dev ? t.ld_idx : k);
    if (take) out[__popcll(mask & ((1ull << lane) - 1ull))] = lane;
    if (t.k_dev)
      for (int i = k + lane; i < t.ld_idx; i += 64) out[i] = -1;
    return;
  }
  const int n = t.n, g = blockIdx.x - t.blk_begin;
  const int k = t.k_dev ? t.k_dev[g] : t.k;
  const float* s = t.scores + static_cast<long long>(g) * n;
  int* out = t.idx + static_cast<long long>(g) * (t.k_dev ? t.ld_idx : k);

  // this thread's contiguous run of indices; runs of up to SELECT_CACHE elements (groups of up to
  // SELECT_THREADS * SELECT_CACHE units) are read once and kept in registers for all passes
  const int per = (n + SELECT_THREADS - 1) / SELECT_THREADS;
  const int i0 = min(tid * per, n), i1 = min(i0 + per, n);
  const bool cached = per <= SELECT_CACHE;
  uint32_t kc[SELECT_CACHE];
  if (cached) {
#pragma unroll
    for (int j = 0; j < SELECT_CACHE; ++j) kc[j] = i0 + j < i1 ? ITEM_KEY(s[i0 + j]) : 0u;
  }

  uint32_t prefix = 0u;   // high bits of the k-th largest key found so far
  int krem = k;           // rank (1-based) of the wanted key among keys matching the prefix
  for (int i = tid; i < (SELECT_THREADS / 64) * 256; i += SELECT_THREADS) (&whist[0][0])[i] = 0;
  __syncthreads();
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    if (cached) {
#pragma unroll
      for (int j = 0; j < SELECT_CACHE; ++j)
        if (i0 + j < i1 && (kc[j] & hi_mask) == prefix) atomicAdd(&whist[wave][(kc[j] >> shift) & 255u], 1);
    } else {
      for (int i = i0; i < i1; ++i) {
        const uint32_t key = ITEM_KEY(s[i]);
        if ((key & hi_mask) == prefix) atomicAdd(&whist[wave][(key >> shift) & 255u], 1);
      }
    }
    __syncthreads();
    // suffix sums hist[d] = number of matching keys with digit >= d: the first four wavefronts own 64 digits
    // each, add the per-wavefront histograms, scan inside the wavefront, then add the totals of the digits above
    int suf = 0;
    if (tid < 256) {
#pragma unroll
      for (int w = 0; w < SELECT_THREADS / 64; ++w) suf += whist[w][tid];
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_down(suf, off, 64);
        if ((tid & 63) + off < 64) suf += v;
      }
      if ((tid & 63) == 0) wave_tot[wave] = suf;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = wave + 1; w < 4; ++w) suf += wave_tot[w];
      hist[tid] = suf;
    } else if (tid == 256) {
      hist[256] = 0;
    }
    for (int i = tid; i < (SELECT_THREADS / 64) * 256; i += SELECT_THREADS) (&whist[0][0])[i] = 0;   // for the next pass
    __syncthreads();
    if (tid < 256 && hist[tid] >= krem && hist[tid + 1] < krem) {   // exactly one thread
      s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
      s_krem = krem - hist[tid + 1];
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
  }
  const uint32_t T = prefix;   // k-th largest key; take `krem` of the elements equal to it

  int n_eq = 0, n_gt = 0;
  if (cached) {
#pragma unroll
    for (int j = 0; j < SELECT_CACHE; ++j)
      if (i0 + j < i1) { n_eq += kc[j] == T; n_gt += kc[j] > T; }
  } else {
    for (int i = i0; i < i1; ++i) {
      const uint32_t key = ITEM_KEY(s[i]);
      n_eq += key == T;
      n_gt += key > T;
    }
  }
  int tot;
  const int eq_before = block_exclusive_scan(n_eq, wave_tot, tot);
  const int eq_take = max(0, min(n_eq, krem - eq_before));       // ties of this run that are kept
  int pos = block_exclusive_scan(n_gt + eq_take, wave_tot, tot);
  int eq_left = eq_take;
  if (cached) {
#pragma unroll
    for (int j = 0; j < SELECT_CACHE; ++j) {
      if (i0 + j >= i1) continue;
      bool take = kc[j] > T;
      if (kc[j] == T && eq_left > 0) { take = true; --eq_left; }
      if (take && pos < k) out[pos++] = i0 + j;
    }
  } else {
    for (int i = i0; i < i1; ++i) {
      const uint32_t key = ITEM_KEY(s[i]);
      bool take = key > T;
      if (key == T && eq_left > 0) { take = true; --eq_left; }
      if (take && pos < k) out[pos++] = i;
    }
  }
  if (t.k_dev)
    for (int i = k + tid; i < t.ld_idx; i += SELECT_THREADS) out[i] = -1;
}

// ---------------------------------------------------------------------------------------------
#undef ITEM_KEY

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
