// Device side of the deterministic block-wide top-k (step 2), shared by the selection launches and by the launch that
// finishes the scores and selects in one go (not part of the C ABI).
#pragma once
#include "common.h"

#define SELECT_THREADS 1024
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

// Inclusive prefix sum over the lanes of a wavefront by lane-permutation (DPP) adds: inside the rows of 16, then the last
// lane of rows 0 and 2 into rows 1 and 3, then lane 31 into the upper half - nothing goes through LDS.
#define ECOSPA_DPP_IADD(v, ctrl, rows) ((v) + __builtin_amdgcn_update_dpp(0, (v), (ctrl), (rows), 0xF, false))
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1, lanes without a source add 0
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
  v = ECOSPA_DPP_IADD(v, 0x142, 0xA);                              // row_bcast:15 into rows 1 and 3
  v = ECOSPA_DPP_IADD(v, 0x143, 0xC);                              // row_bcast:31 into rows 2 and 3
  return v;
}

// Exclusive prefix sums of `a` and of `b` over the block's threads in thread order (one pass for both).
// `wave_tot` holds 2 x (SELECT_THREADS / 64) ints and must not be in use by another scan one barrier earlier.
__device__ __forceinline__ void block_exclusive_scan2(int a, int b, int* wave_tot, int& a_before, int& b_before) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ia = wave_inclusive_scan(a), ib = wave_inclusive_scan(b);
  if (lane == 63) { wave_tot[2 * wave] = ia; wave_tot[2 * wave + 1] = ib; }
  __syncthreads();
  int ba = 0, bb = 0;
#pragma unroll
  for (int w = 0; w < SELECT_THREADS / 64; ++w) {
    const int ca = wave_tot[2 * w], cb = wave_tot[2 * w + 1];
    if (w < wave) { ba += ca; bb += cb; }
  }
  a_before = ba + ia - a;
  b_before = bb + ib - b;
}

// LDS of one selecting workgroup.  One histogram per wavefront: normalised scores share their top key bits, so a
// single histogram would serialise nearly every atomic of the first pass on a few counters.
struct SelectShared {
  int whist[SELECT_THREADS / 64][256];
  int wave_tot[2 * (SELECT_THREADS / 64)];
  uint32_t s_prefix;
  int s_krem;
};
#define ITEM_KEY(x) (score_key(x) ^ flip)
// A group of more than 64 units by one workgroup.  CACHE: score keys a thread keeps in registers (its contiguous run of
// indices is read once for all passes); 0: longer runs are read again in every pass.
template <int CACHE>
__device__ __forceinline__ void select_large_group(const SelectItemDev& t, int blk, SelectShared& sh) {
  auto& whist = sh.whist;
  auto& wave_tot = sh.wave_tot;
  uint32_t& s_prefix = sh.s_prefix;
  int& s_krem = sh.s_krem;
  const int tid = threadIdx.x, wave = tid >> 6;
  const uint32_t flip = t.smallest ? 0xffffffffu : 0u;
  constexpr bool cached = CACHE > 0;
  constexpr int NC = CACHE > 0 ? CACHE : 1;
  const int n = t.n, g = blk;
  const int k = t.k_dev ? t.k_dev[g] : t.k;
  const float* s = t.scores + static_cast<long long>(g) * n;
  int* out = t.idx + static_cast<long long>(g) * (t.k_dev ? t.ld_idx : k);

  // this thread's contiguous run of indices
  const int per = (n + SELECT_THREADS - 1) / SELECT_THREADS;
  const int i0 = min(tid * per, n), i1 = min(i0 + per, n);
  uint32_t kc[NC];
  if (cached) {
#pragma unroll
    for (int j = 0; j < NC; ++j) kc[j] = i0 + j < i1 ? ITEM_KEY(s[i0 + j]) : 0u;
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
      for (int j = 0; j < NC; ++j)
        if (i0 + j < i1 && (kc[j] & hi_mask) == prefix) atomicAdd(&whist[wave][(kc[j] >> shift) & 255u], 1);
    } else {
      for (int i = i0; i < i1; ++i) {
        const uint32_t key = ITEM_KEY(s[i]);
        if ((key & hi_mask) == prefix) atomicAdd(&whist[wave][(key >> shift) & 255u], 1);
      }
    }
    __syncthreads();
    // suffix sums suf[d] = number of matching keys with digit >= d: the first four wavefronts own 64 digits each, add
    // the per-wavefront histograms (and clear them for the next pass), scan inside the wavefront by lane permutations,
    // then add the totals of the digits above.  Exactly one digit has suf[d] >= krem > suf[d + 1] = suf[d] - cnt[d].
    int cnt = 0, suf = 0;
    if (tid < 256) {
#pragma unroll
      for (int w = 0; w < SELECT_THREADS / 64; ++w) { cnt += whist[w][tid]; whist[w][tid] = 0; }
      const int inc = wave_inclusive_scan(cnt);
      const int tot = __builtin_amdgcn_readlane(inc, 63);
      suf = tot - inc + cnt;
      if ((tid & 63) == 0) wave_tot[wave] = tot;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = wave + 1; w < 4; ++w) suf += wave_tot[w];
      if (suf >= krem && suf - cnt < krem) {
        s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
        s_krem = krem - (suf - cnt);
      }
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
  }
  const uint32_t T = prefix;   // k-th largest key; take `krem` of the elements equal to it

  int n_eq = 0, n_gt = 0;
  if (cached) {
#pragma unroll
    for (int j = 0; j < NC; ++j)
      if (i0 + j < i1) { n_eq += kc[j] == T; n_gt += kc[j] > T; }
  } else {
    for (int i = i0; i < i1; ++i) {
      const uint32_t key = ITEM_KEY(s[i]);
      n_eq += key == T;
      n_gt += key > T;
    }
  }
  // the ties are kept in index order until `krem` of them are: min(ties before this run, krem) of those before it
  int eq_before, gt_before;
  block_exclusive_scan2(n_eq, n_gt, wave_tot, eq_before, gt_before);
  int eq_left = max(0, min(n_eq, krem - eq_before));       // ties of this run that are kept
  int pos = gt_before + min(eq_before, krem);
  if (cached) {
#pragma unroll
    for (int j = 0; j < NC; ++j) {
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

// The work of workgroup number `blk` of item t (all SELECT_THREADS threads of the workgroup call it).
__device__ __forceinline__ void select_item_block(const SelectItemDev& t, int blk, SelectShared& sh) {
  const int tid = threadIdx.x, wave = tid >> 6;
  const uint32_t flip = t.smallest ? 0xffffffffu : 0u;
  if (t.n <= 64) {
    // Small groups (the units of one head): a wavefront ranks a group by direct comparison - the rank of
    // a unit is the number of units that come before it in the order (larger key, or equal key and lower
    // index) - and the lanes whose rank is below k write their indices, ascending.  One group per wavefront.
    const int g = blk * (SELECT_THREADS / 64) + wave;
    if (g >= t.groups) return;
    const int lane = tid & 63, n = t.n;
    const int k = t.k_dev ? t.k_dev[g] : t.k;
    const uint32_t key = lane < n ? ITEM_KEY(t.scores[static_cast<long long>(g) * n + lane]) : 0u;
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const uint32_t kj = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(key), j));   // j is uniform: no LDS crossbar
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
  // runs of up to 8 units per thread (groups of up to 8192) or of up to 32 (32768) stay in registers
  const int per = (t.n + SELECT_THREADS - 1) / SELECT_THREADS;
  if (per <= 8) select_large_group<8>(t, blk, sh);
  else if (per <= 32) select_large_group<32>(t, blk, sh);
  else select_large_group<0>(t, blk, sh);
}

#undef ITEM_KEY
