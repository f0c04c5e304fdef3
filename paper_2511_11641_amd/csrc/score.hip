// Step 1: per-dimension coupled importance score (paper Eq. 10, criterion of Eq. 12).
//
// HBM-bound: every weight element of every pair in the batch is read exactly once with
// 16-byte loads, by one launch per SCORE_MAX_PAIRS pairs:
//   * squared row norms: a wavefront takes four rows at a time, all their loads in flight, then
//     lane-permutation sums;
//   * squared column norms of the [d, n] member: a workgroup takes a strip of one 128-byte line
//     (8 lanes x 16 bytes) over a range of rows, eight loads in flight per lane, and writes one
//     partial sum per column and row range;
// and a short finishing launch (score_finish_kernel) that adds the partial sums in order and writes the
// scores: r = |a||b|, group L2 norm, normalised scores (or the weighted sums of Eq. 8).
// No floating-point atomics; all reduction orders are fixed.
#include "common.h"
#include "select_dev.h"

#define SCORE_MAX_PAIRS 96         // descriptors travel as kernel arguments (about 15 KB)
#define SCORE_ROWS_PER_BLOCK 16   // row-norm blocks: 4 waves x 4 rows
#define SCORE_COL_ROWS 256             // rows of a column-norm workgroup (up to SCORE_MAX_PARTS ranges per matrix)
#define SCORE_COL_LDS (256 * 8 + 32)   // floats: slots x (strip width + 1) for every split of 256 threads into lanes x slots

struct ScorePairDev {
  const void* w1;
  const void* w1b;
  const void* w2;
  long long ld1, ld1b, ld2;
  float* a_sq;     // [rows]            squared norms of a_j
  float* b_sq;     // [rows]            squared norms of b_j (rows of W_k, or columns of w2)
  int rows1, rows2;  // rows of w1 (groups * rep1 * n) and rows (QK) or columns of w2 (groups * rep2 * n)
  int rep1, rep2;    // heads of each member that share one group's inner dimensions (grouped-query attention, Eq. 5); 1 otherwise
  int groups, n, unit;
  int d1, d2;
  int kind, dtype;
  int fisher;      // 1: squared gradient sums for Eq. 8 (w1 and w1b are added, not multiplied)
  int col_lanes;   // column norms: lanes (16 bytes each) side by side on a row; 256 / col_lanes row slots per workgroup
  int col_strips;  //               strips of col_lanes * 16 bytes that cover the columns
  int col_parts;   //               row ranges; part q writes its partial sums to b_sq + q * rows
  int blk_row1, blk_row2, blk_col, blk_end;   // first block index of each phase of this pair
  // finishing launch
  int fin_blocks;       // workgroups of this pair in the finishing launch
  float* scores;       // Eq. 10: [groups, n / unit]; Eq. 8: [groups]
  float fw1, fw2;      // Eq. 8: weights 1 / (2 |W_k| |D|) of the two members' squared sums
};
struct ScoreBatch {
  int n_pairs;
  int first_blk[SCORE_MAX_PAIRS];   // blk_row1 of every pair, side by side: the search for a block's pair stays in a few cache lines
  ScorePairDev p[SCORE_MAX_PAIRS];
};
static_assert(sizeof(ScoreBatch) <= 16384, "kernel arguments of one launch");

template <typename T> struct Vec16;
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16_t> { static constexpr int N = 8; };

template <typename T>
__device__ __forceinline__ void load_vec(const T* p, float (&out)[Vec16<T>::N]);
template <>
__device__ __forceinline__ void load_vec<float>(const float* p, float (&out)[4]) {
  float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <>
__device__ __forceinline__ void load_vec<bf16_t>(const bf16_t* p, float (&out)[8]) {
  uint4 v = *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

// Squared norms of NR consecutive rows (optionally of the elementwise products with the rows of a
// second matrix) by one wavefront: the loads of all NR rows are in flight together, the cross-lane
// sums come last.  Rows >= rows_valid are skipped (their slot returns 0).
template <typename T, int NR>
__device__ __forceinline__ void rows_sumsq(const T* r, const T* rb, long long ld, long long ldb, int len, int rows_valid,
                                           bool vec_ok, bool add_rb, int lane, float (&out)[NR]) {
  constexpr int V = Vec16<T>::N;
  float acc[NR];
#pragma unroll
  for (int j = 0; j < NR; ++j) acc[j] = 0.f;
  if (vec_ok) {
#pragma unroll 2
    for (int c = lane * V; c < len; c += 64 * V) {
      float a[NR][V], b[NR][V];
#pragma unroll
      for (int j = 0; j < NR; ++j) {
        const int jj = j < rows_valid ? j : 0;       // clamped: always a valid row
        load_vec<T>(r + jj * ld + c, a[j]);
        if (rb) load_vec<T>(rb + jj * ldb + c, b[j]);
      }
#pragma unroll
      for (int j = 0; j < NR; ++j) {
        if (rb && add_rb) {
#pragma unroll
          for (int i = 0; i < V; ++i) acc[j] += a[j][i] * a[j][i] + b[j][i] * b[j][i];
        } else if (rb) {
#pragma unroll
          for (int i = 0; i < V; ++i) { const float t = a[j][i] * b[j][i]; acc[j] += t * t; }
        } else {
#pragma unroll
          for (int i = 0; i < V; ++i) acc[j] += a[j][i] * a[j][i];
        }
      }
    }
  } else {
    for (int j = 0; j < NR && j < rows_valid; ++j)
      for (int c = lane; c < len; c += 64) {
        float a = load_f32<T>(r + j * ld + c);
        if (rb && add_rb) {
          const float b = load_f32<T>(rb + j * ldb + c);
          acc[j] += a * a + b * b;
        } else {
          if (rb) a *= load_f32<T>(rb + j * ldb + c);
          acc[j] += a * a;
        }
      }
  }
#pragma unroll
  for (int j = 0; j < NR; ++j) out[j] = j < rows_valid ? wave_sum(acc[j]) : 0.f;
}

// ---- finishing step of a pair --------------------------------------------------------------------
// r of unit u of group g: |a| |b| over the unit's UR rows (Eq. 10), or the weighted squared sums (Eq. 8).
// The partial column sums of a row are added in order of their row ranges.  No load sits behind a branch
// or in a loop of unknown length (an index out of range is clamped and its value dropped), so that the
// loads of all units a thread holds can be in flight together.
#define SCORE_MAX_PARTS 4
template <int UR>
__device__ __forceinline__ float pair_unit_value(const ScorePairDev& p, int g, int u, int unit_rows) {
  float a = 0.f, b = 0.f;
  if (UR > 0) {        // one head per group on both sides
#pragma unroll
    for (int j = 0; j < UR; ++j) {
      const int row = g * p.n + u * UR + j;
      a += p.a_sq[row];
#pragma unroll
      for (int q = 0; q < SCORE_MAX_PARTS; ++q) {
        const float v = p.b_sq[static_cast<long long>(q < p.col_parts ? q : 0) * p.rows2 + row];
        b += q < p.col_parts ? v : 0.f;
      }
    }
  } else {             // any unit, any number of heads sharing the group (Eq. 5): heads, then rows, then row ranges, in order
    for (int h = 0; h < p.rep1; ++h)
      for (int j = 0; j < unit_rows; ++j) a += p.a_sq[(g * p.rep1 + h) * p.n + u * unit_rows + j];
    for (int h = 0; h < p.rep2; ++h)
      for (int j = 0; j < unit_rows; ++j) {
        const int row = (g * p.rep2 + h) * p.n + u * unit_rows + j;
        for (int q = 0; q < p.col_parts; ++q) b += p.b_sq[static_cast<long long>(q) * p.rows2 + row];
      }
  }
  return p.fisher ? p.fw1 * a + p.fw2 * b : sqrtf(a) * sqrtf(b);
}

// Finishing launch: scores of the groups of every pair from the finished squared sums.  A pair with
// SCORE_FIN_WAVES groups or more (attention heads) gives every wavefront a group of its own and needs no
// workgroup barriers; otherwise (the FFN pair) a whole workgroup works on one group.  A thread keeps up to
// SCORE_FIN_KEEP units in registers: their loads are all in flight together, and nothing is re-read.
#define SCORE_FIN_THREADS 1024
#define SCORE_FIN_WAVES (SCORE_FIN_THREADS / 64)
#define SCORE_FIN_KEEP 8
// One group by `stride` threads of which this is number `t`; `total(x)` adds x over those threads in a fixed order.
template <int UR, int KEEP, typename Total>
__device__ __forceinline__ void score_finish_group_k(const ScorePairDev& p, int g, int t, int stride, Total total) {
  const int nu = p.fisher ? p.n : p.n / p.unit;      // Eq. 8 sums over single rows
  const int unit_rows = p.fisher ? 1 : p.unit;
  float* out = p.scores + static_cast<long long>(g) * nu;
  float acc = 0.f;
  if (nu <= KEEP * stride) {
    float r[KEEP];
#pragma unroll
    for (int k = 0; k < KEEP; ++k) {
      const int u = t + k * stride;
      const float v = pair_unit_value<UR>(p, g, u < nu ? u : nu - 1, unit_rows);
      r[k] = u < nu ? v : 0.f;
    }
#pragma unroll
    for (int k = 0; k < KEEP; ++k) acc += p.fisher ? r[k] : r[k] * r[k];
    acc = total(acc);
    if (p.fisher) {
      if (t == 0) p.scores[g] = acc;
      return;
    }
    const float nrm = sqrtf(acc);
#pragma unroll
    for (int k = 0; k < KEEP; ++k) {
      const int u = t + k * stride;
      if (u < nu) out[u] = nrm > 0.f ? r[k] / nrm : 0.f;
    }
    return;
  }
  for (int u = t; u < nu; u += stride) {
    const float r = pair_unit_value<UR>(p, g, u, unit_rows);
    if (p.fisher) acc += r;
    else { acc += r * r; out[u] = r; }
  }
  acc = total(acc);
  if (p.fisher) {
    if (t == 0) p.scores[g] = acc;
    return;
  }
  const float nrm = sqrtf(acc);
  for (int u = t; u < nu; u += stride) out[u] = nrm > 0.f ? out[u] / nrm : 0.f;   // re-read by the thread that wrote it
}

template <typename T>
__device__ void score_block(const ScorePairDev& p, int blk, float* lds) {
  constexpr int V = Vec16<T>::N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (blk < p.blk_col) {
    // ---- row norms: phase 1 = w1 (x w1b), phase 2 = rows of w2 (QK) ----
    const bool second = blk >= p.blk_row2;
    const int local = blk - (second ? p.blk_row2 : p.blk_row1);
    const T* w = static_cast<const T*>(second ? p.w2 : p.w1);
    const T* wb = second ? nullptr : static_cast<const T*>(p.w1b);
    const long long ld = second ? p.ld2 : p.ld1;
    const int len = second ? p.d2 : p.d1;
    float* out = second ? p.b_sq : p.a_sq;
    bool vec_ok = (len % V == 0) && (ld % V == 0) && ((reinterpret_cast<uintptr_t>(w) & 15u) == 0);
    if (wb) vec_ok = vec_ok && (p.ld1b % V == 0) && ((reinterpret_cast<uintptr_t>(wb) & 15u) == 0);
    constexpr int NR = SCORE_ROWS_PER_BLOCK / 4;
    const int row0 = local * SCORE_ROWS_PER_BLOCK + wave * NR;
    const int rows = second ? p.rows2 : p.rows1;
    if (row0 < rows) {
      float sums[NR];
      rows_sumsq<T, NR>(w + row0 * ld, wb ? wb + row0 * p.ld1b : nullptr, ld, p.ld1b, len, rows - row0, vec_ok, p.fisher != 0, lane, sums);
      if (lane == 0) {
#pragma unroll
        for (int j = 0; j < NR; ++j)
          if (row0 + j < rows) out[row0 + j] = sums[j];
      }
    }
    return;
  }
  // ---- squared column norms of w2 [d2, rows]: one strip of col_lanes x V columns, one range of rows ----
  const int local = blk - p.blk_col;
  const int L = p.col_lanes, S = 256 / L, W = L * V;
  const int strip = local % p.col_strips, part = local / p.col_strips;   // neighbours in the grid: neighbours on the rows
  const int slot = tid / L, ln = tid % L;
  const T* w = static_cast<const T*>(p.w2);
  const int col0 = strip * W + ln * V;
  const int per = (p.d2 + p.col_parts - 1) / p.col_parts;
  const int r_begin = part * per, r_end = min(p.d2, r_begin + per);
  const bool vec_ok = (p.ld2 % V == 0) && ((reinterpret_cast<uintptr_t>(w) & 15u) == 0);
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.f;
  if (vec_ok && col0 + V <= p.rows2) {
    for (int r0 = r_begin + slot; r0 < r_end; r0 += 8 * S) {     // 8 independent loads in flight
      float a[8][V];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int r = r0 + q * S;
        load_vec<T>(w + static_cast<long long>(r < r_end ? r : r0) * p.ld2 + col0, a[q]);
        if (r >= r_end) {
#pragma unroll
          for (int i = 0; i < V; ++i) a[q][i] = 0.f;
        }
      }
#pragma unroll
      for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += a[q][i] * a[q][i];
    }
  } else {
    for (int r = r_begin + slot; r < r_end; r += S) {
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (col0 + i < p.rows2) {
          float a = load_f32<T>(w + static_cast<long long>(r) * p.ld2 + col0 + i);
          acc[i] += a * a;
        }
    }
  }
  // the row slots of a column are added in slot order by one thread
#pragma unroll
  for (int i = 0; i < V; ++i) lds[slot * (W + 1) + ln * V + i] = acc[i];
  __syncthreads();
  float* out = p.b_sq + static_cast<long long>(part) * p.rows2;
  for (int c = tid; c < W; c += 256) {
    float tot = 0.f;
    for (int k = 0; k < S; ++k) tot += lds[k * (W + 1) + c];
    const int col = strip * W + c;
    if (col < p.rows2) out[col] = tot;
  }
}

__global__ __launch_bounds__(256) void score_sumsq_kernel(const ScoreBatch b) {
  __shared__ float lds[SCORE_COL_LDS];
  const int blk = blockIdx.x;
  int lo = 0, hi = b.n_pairs - 1;          // last pair whose first block is <= blk
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (b.first_blk[mid] <= blk) lo = mid; else hi = mid - 1;
  }
  const ScorePairDev& p = b.p[lo];
  if (p.dtype == ECOSPA_BF16) score_block<bf16_t>(p, blk, lds);
  else score_block<float>(p, blk, lds);
}

// The number of units a thread holds follows the size of the group, so that small groups issue no idle loads.
template <int UR, typename Total>
__device__ __forceinline__ void score_finish_group(const ScorePairDev& p, int g, int t, int stride, Total total) {
  const int nu = p.fisher ? p.n : p.n / p.unit;
  if (nu <= stride) score_finish_group_k<UR, 1>(p, g, t, stride, total);
  else if (nu <= 4 * stride) score_finish_group_k<UR, 4>(p, g, t, stride, total);
  else score_finish_group_k<UR, SCORE_FIN_KEEP>(p, g, t, stride, total);
}

__global__ __launch_bounds__(SCORE_FIN_THREADS) void score_finish_kernel(const ScoreBatch b) {
  __shared__ float red[SCORE_FIN_WAVES];
  // grid: (workgroups of the pair that needs most, pairs) - the pair is named directly, a search through the
  // descriptors would cost a chain of dependent loads that is longer than the work itself
  const ScorePairDev& p = b.p[blockIdx.y];
  const int local = blockIdx.x, tid = threadIdx.x;
  if (local >= p.fin_blocks) return;
  // rows per unit: 1, 2 (rotary blocks), or the general form (other units, heads sharing a group)
  const int ur = (p.rep1 > 1 || p.rep2 > 1) ? 0 : (p.fisher ? 1 : p.unit);
  if (p.groups >= SCORE_FIN_WAVES) {
    const int g = local * SCORE_FIN_WAVES + (tid >> 6);
    if (g >= p.groups) return;
    auto total = [](float v) { return wave_sum(v); };
    if (ur == 1) score_finish_group<1>(p, g, tid & 63, 64, total);
    else if (ur == 2) score_finish_group<2>(p, g, tid & 63, 64, total);
    else score_finish_group<0>(p, g, tid & 63, 64, total);
    return;
  }
  auto total = [&](float v) {
    v = wave_sum(v);
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < SCORE_FIN_WAVES; ++w) tot += red[w];
    return tot;
  };
  if (ur == 1) score_finish_group<1>(p, local, tid, SCORE_FIN_THREADS, total);
  else if (ur == 2) score_finish_group<2>(p, local, tid, SCORE_FIN_THREADS, total);
  else score_finish_group<0>(p, local, tid, SCORE_FIN_THREADS, total);
}

// Steps 1 and 2 in one finishing launch: the workgroup (or wavefront) that has written a group's scores goes on to
// select the group's k best units - the scores are still in its cache, and one launch and its start-up are gone.
// The team of a group follows the selection's rule (a wavefront for groups of up to 64 units, else a workgroup).
#define SCORE_SEL_PAIRS 48        // pairs per launch of the combined form: both argument structs stay inside 16 KB
struct ScoreSelect {
  int k[SCORE_SEL_PAIRS];
  int* idx[SCORE_SEL_PAIRS];
};
static_assert(sizeof(ScoreBatch) + sizeof(ScoreSelect) <= 16384, "kernel arguments of one launch");
static_assert(SCORE_FIN_THREADS == SELECT_THREADS, "one team shape for both halves");

__global__ __launch_bounds__(SCORE_FIN_THREADS) void score_finish_select_kernel(const ScoreBatch b, const ScoreSelect s) {
  __shared__ SelectShared sh;
  __shared__ float red[SCORE_FIN_WAVES];
  const ScorePairDev& p = b.p[blockIdx.y];
  const int local = blockIdx.x, tid = threadIdx.x;
  const int nu = p.n / p.unit;
  const bool wave_team = nu <= 64;
  const int blocks = wave_team ? (p.groups + SCORE_FIN_WAVES - 1) / SCORE_FIN_WAVES : p.groups;
  if (local >= blocks) return;      // the whole workgroup leaves together
  const int ur = (p.rep1 > 1 || p.rep2 > 1) ? 0 : p.unit;
  if (wave_team) {
    const int g = local * SCORE_FIN_WAVES + (tid >> 6);
    if (g < p.groups) {
      auto total = [](float v) { return wave_sum(v); };
      if (ur == 1) score_finish_group<1>(p, g, tid & 63, 64, total);
      else if (ur == 2) score_finish_group<2>(p, g, tid & 63, 64, total);
      else score_finish_group<0>(p, g, tid & 63, 64, total);
    }
  } else {
    auto total = [&](float v) {
      v = wave_sum(v);
      if ((tid & 63) == 0) red[tid >> 6] = v;
      __syncthreads();
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < SCORE_FIN_WAVES; ++w) tot += red[w];
      return tot;
    };
    if (ur == 1) score_finish_group<1>(p, local, tid, SCORE_FIN_THREADS, total);
    else if (ur == 2) score_finish_group<2>(p, local, tid, SCORE_FIN_THREADS, total);
    else score_finish_group<0>(p, local, tid, SCORE_FIN_THREADS, total);
  }
  __threadfence_block();      // the scores were written by other threads of this team
  __syncthreads();
  SelectItemDev t;
  t.scores = p.scores; t.idx = s.idx[blockIdx.y];
  t.n = nu; t.k = s.k[blockIdx.y];
  t.blk_begin = 0; t.groups = p.groups; t.k_dev = nullptr; t.ld_idx = t.k; t.smallest = 0;
  select_item_block(t, local, sh);
}

// ------------------------------------------------------------------------------------------
static inline int pair_rep1(const ecospa_pair& q) { return q.rep1 > 0 ? q.rep1 : 1; }
static inline int pair_rep2(const ecospa_pair& q) { return q.rep2 > 0 ? q.rep2 : 1; }

// the second member's units are rows (W_k always; W_o / W_out / W_down when the caller stores them that way)
static inline bool pair_w2_rows(const ecospa_pair& q) { return q.kind == ECOSPA_PAIR_QK || q.w2_rows != 0; }

static int validate_pair(const ecospa_pair& q) {
  if (q.kind < ECOSPA_PAIR_QK || q.kind > ECOSPA_PAIR_FFN_GATED || !dtype_ok(q.dtype)) return ECOSPA_ERR_DTYPE;
  if (!q.w1 || !q.w2 || (q.kind == ECOSPA_PAIR_FFN_GATED && !q.w1b)) return ECOSPA_ERR_NULL;
  if (q.groups < 1 || q.n < 1 || q.unit < 1 || q.d1 < 1 || q.d2 < 1 || q.n % q.unit) return ECOSPA_ERR_SHAPE;
  if (q.rep1 < 0 || q.rep2 < 0) return ECOSPA_ERR_SHAPE;
  if ((pair_rep1(q) > 1 || pair_rep2(q) > 1) && q.kind != ECOSPA_PAIR_QK && q.kind != ECOSPA_PAIR_VO) return ECOSPA_ERR_SHAPE;
  const long long rows1 = static_cast<long long>(q.groups) * pair_rep1(q) * q.n;
  const long long rows2 = static_cast<long long>(q.groups) * pair_rep2(q) * q.n;
  if (rows1 > (1ll << 30) || rows2 > (1ll << 30)) return ECOSPA_ERR_SHAPE;
  if (q.ld1 < q.d1) return ECOSPA_ERR_SHAPE;
  if (q.kind == ECOSPA_PAIR_FFN_GATED && q.ld1b < q.d1) return ECOSPA_ERR_SHAPE;
  if (pair_w2_rows(q) ? q.ld2 < q.d2 : q.ld2 < rows2) return ECOSPA_ERR_SHAPE;
  return ECOSPA_OK;
}

// Shape of the column-norm phase of a pair: lanes side by side on a row (strip width), strips, and row ranges.
struct ColShape { int lanes, strips, parts; };
static ColShape col_shape(const ecospa_pair& q) {
  const int V = q.dtype == ECOSPA_BF16 ? 8 : 4;
  const long long rows = static_cast<long long>(q.groups) * pair_rep2(q) * q.n;
  ColShape c;
  c.lanes = 8;        // one 128-byte line per row: wider strips measured slower (fewer, longer workgroups)
  c.strips = static_cast<int>((rows + c.lanes * V - 1) / (c.lanes * V));
  c.parts = (q.d2 + SCORE_COL_ROWS - 1) / SCORE_COL_ROWS;
  if (c.parts > SCORE_MAX_PARTS) c.parts = SCORE_MAX_PARTS;
  return c;
}

static size_t pair_ws_bytes(const ecospa_pair& q) {
  const size_t rows1 = static_cast<size_t>(q.groups) * pair_rep1(q) * q.n, rows2 = static_cast<size_t>(q.groups) * pair_rep2(q) * q.n;
  const size_t parts = pair_w2_rows(q) ? 1 : col_shape(q).parts;
  return align_up(rows1 * 4, 256) + align_up(parts * rows2 * 4, 256);   // a_sq, b_sq (partial sums)
}

extern "C" size_t ecospa_score_workspace_bytes(const ecospa_pair* pairs, int n_pairs) {
  if (!pairs || n_pairs < 1) return 0;
  size_t tot = 0;
  for (int i = 0; i < n_pairs; ++i) {
    if (validate_pair(pairs[i]) != ECOSPA_OK) return 0;
    tot += pair_ws_bytes(pairs[i]);
  }
  return tot + 256;
}

// Shared driver of Eq. 10 (fisher = 0: `pairs` are weights) and Eq. 8 (fisher = 1: `pairs` are gradients).
static int score_validate(ecospa_ctx* ctx, const ecospa_pair* pairs, int n_pairs, float* const* scores) {
  if (!ctx || !pairs || !scores) return ECOSPA_ERR_NULL;
  if (n_pairs < 1) return ECOSPA_ERR_SHAPE;
  for (int i = 0; i < n_pairs; ++i) {
    int rc = validate_pair(pairs[i]);
    if (rc) return rc;
    if (!scores[i]) return ECOSPA_ERR_NULL;
  }
  return ECOSPA_OK;
}

// `scratch` / `scratch_bytes`: device memory for the partial squared sums (the caller's workspace, or the library's
// own fixed array); the arguments have been validated.
// With `sel_k` / `sel_idx` (host arrays, one entry per pair) the finishing launch also selects (step 2).
static int score_run(ecospa_ctx* ctx, const ecospa_pair* pairs, int n_pairs, float* const* scores, int fisher,
                     float n_samples, void* scratch, size_t scratch_bytes, const int* sel_k = nullptr,
                     int* const* sel_idx = nullptr) {
  const size_t need = ecospa_score_workspace_bytes(pairs, n_pairs);
  if (!scratch || scratch_bytes < need) return ECOSPA_ERR_WORKSPACE;
  WsCarver ws(scratch, scratch_bytes);

  const int chunk = sel_k ? SCORE_SEL_PAIRS : SCORE_MAX_PAIRS;
  for (int first = 0; first < n_pairs; first += chunk) {
    ScoreBatch b;
    memset(&b, 0, sizeof(b));
    b.n_pairs = (n_pairs - first < chunk) ? n_pairs - first : chunk;
    int blk = 0, fin = 0, fin_sel = 0;
    ScoreSelect sel;
    for (int i = 0; i < b.n_pairs; ++i) {
      const ecospa_pair& q = pairs[first + i];
      ScorePairDev& p = b.p[i];
      if (sel_k) {
        sel.k[i] = sel_k[first + i];
        sel.idx[i] = sel_idx[first + i];
        const int team_blocks = q.n / q.unit <= 64 ? (q.groups + SCORE_FIN_WAVES - 1) / SCORE_FIN_WAVES : q.groups;
        if (team_blocks > fin_sel) fin_sel = team_blocks;
      }
      p.w1 = q.w1; p.w1b = (q.kind == ECOSPA_PAIR_FFN_GATED) ? q.w1b : nullptr; p.w2 = q.w2;
      p.ld1 = q.ld1; p.ld1b = q.ld1b; p.ld2 = q.ld2;
      p.rep1 = pair_rep1(q); p.rep2 = pair_rep2(q);
      p.rows1 = q.groups * p.rep1 * q.n; p.rows2 = q.groups * p.rep2 * q.n;
      p.groups = q.groups; p.n = q.n; p.unit = q.unit;
      p.d1 = q.d1; p.d2 = q.d2; p.kind = q.kind; p.dtype = q.dtype; p.fisher = fisher;
      p.a_sq = static_cast<float*>(ws.take(static_cast<size_t>(p.rows1) * 4));
      const int row_blocks = (p.rows1 + SCORE_ROWS_PER_BLOCK - 1) / SCORE_ROWS_PER_BLOCK;
      p.blk_row1 = blk;
      b.first_blk[i] = blk;
      blk += row_blocks;
      p.blk_row2 = blk;
      p.col_lanes = 8; p.col_strips = 1; p.col_parts = 1;
      if (pair_w2_rows(q)) {
        p.b_sq = static_cast<float*>(ws.take(static_cast<size_t>(p.rows2) * 4));
        blk += (p.rows2 + SCORE_ROWS_PER_BLOCK - 1) / SCORE_ROWS_PER_BLOCK;
        p.blk_col = blk;
      } else {
        const ColShape c = col_shape(q);
        p.col_lanes = c.lanes; p.col_strips = c.strips; p.col_parts = c.parts;
        p.b_sq = static_cast<float*>(ws.take(static_cast<size_t>(c.parts) * p.rows2 * 4));
        p.blk_col = blk;
        blk += c.strips * c.parts;
      }
      p.blk_end = blk;
      p.fin_blocks = q.groups >= SCORE_FIN_WAVES ? (q.groups + SCORE_FIN_WAVES - 1) / SCORE_FIN_WAVES : q.groups;
      if (p.fin_blocks > fin) fin = p.fin_blocks;
      p.scores = scores[first + i];
      const double members = q.kind == ECOSPA_PAIR_FFN_GATED ? 2.0 : 1.0;   // W_gate and W_up form the first member
      p.fw1 = fisher ? static_cast<float>(0.5 / (members * p.rep1 * q.n * static_cast<double>(q.d1) * n_samples)) : 0.f;
      p.fw2 = fisher ? static_cast<float>(0.5 / (static_cast<double>(p.rep2) * q.n * static_cast<double>(q.d2) * n_samples)) : 0.f;
    }
    if (!ws.ok()) return ECOSPA_ERR_WORKSPACE;
    hipLaunchKernelGGL(score_sumsq_kernel, dim3(blk), dim3(256), 0, ctx->stream, b);
    ECOSPA_CHECK_LAUNCH(ctx, "score_sumsq_kernel");
    if (sel_k) {
      hipLaunchKernelGGL(score_finish_select_kernel, dim3(fin_sel, b.n_pairs), dim3(SCORE_FIN_THREADS), 0, ctx->stream, b, sel);
      ECOSPA_CHECK_LAUNCH(ctx, "score_finish_select_kernel");
    } else {
      hipLaunchKernelGGL(score_finish_kernel, dim3(fin, b.n_pairs), dim3(SCORE_FIN_THREADS), 0, ctx->stream, b);
      ECOSPA_CHECK_LAUNCH(ctx, "score_finish_kernel");
    }
  }
  return ECOSPA_OK;
}

extern "C" int ecospa_coupled_score(ecospa_ctx* ctx, const ecospa_pair* pairs, int n_pairs, float* const* scores) {
  const int rc = score_validate(ctx, pairs, n_pairs, scores);
  if (rc) return rc;
  return score_run(ctx, pairs, n_pairs, scores, 0, 1.f, ctx->ws, ctx->ws_bytes);
}

extern "C" int ecospa_score_select(ecospa_ctx* ctx, const ecospa_pair* pairs, int n_pairs, float* const* scores,
                                   const int* k, int* const* idx) {
  const int rc = score_validate(ctx, pairs, n_pairs, scores);
  if (rc) return rc;
  if (!k || !idx) return ECOSPA_ERR_NULL;
  for (int i = 0; i < n_pairs; ++i) {
    if (!idx[i]) return ECOSPA_ERR_NULL;
    if (k[i] < 1 || k[i] > pairs[i].n / pairs[i].unit) return ECOSPA_ERR_K;
    if (static_cast<long long>(pairs[i].groups) * (pairs[i].n / pairs[i].unit) > (1ll << 31) - 1) return ECOSPA_ERR_SHAPE;
  }
  return score_run(ctx, pairs, n_pairs, scores, 0, 1.f, ctx->ws, ctx->ws_bytes, k, idx);
}

extern "C" int ecospa_pair_fisher(ecospa_ctx* ctx, const ecospa_pair* grads, int n_pairs, float n_samples,
                                  float* const* fisher) {
  if (!(n_samples > 0.f)) return ECOSPA_ERR_SHAPE;
  const int rc = score_validate(ctx, grads, n_pairs, fisher);
  if (rc) return rc;
  return score_run(ctx, grads, n_pairs, fisher, 1, n_samples, ctx->ws, ctx->ws_bytes);
}

// ------------------------------------------------------------------------------------------
// The same scores for callers that can neither allocate device memory nor hand over a workspace: the partial
// squared sums live in a fixed array in the library's own device image.  Host code never uses the array's name
// as an address: the device address is asked for once per device and kept.
#define SCORE_STATIC_BYTES (2u << 20)
static __device__ __align__(256) unsigned char scratch[SCORE_STATIC_BYTES];

#define SCORE_MAX_DEVICES 64
static void* scratch_dev_ptr[SCORE_MAX_DEVICES];       // per device ordinal; written once, under the lock
static std::atomic<unsigned long long> scratch_known{0};
static std::atomic_flag scratch_lock = ATOMIC_FLAG_INIT;

// Device address of `scratch` on the current device (asked for on the first call there).
static hipError_t score_static_ptr(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= SCORE_MAX_DEVICES) return hipErrorInvalidDevice;
  const unsigned long long bit = 1ull << dev;
  if (!(scratch_known.load(std::memory_order_acquire) & bit)) {
    while (scratch_lock.test_and_set(std::memory_order_acquire)) {}
    if (!(scratch_known.load(std::memory_order_relaxed) & bit)) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e == hipSuccess) {
        scratch_dev_ptr[dev] = p;
        scratch_known.fetch_or(bit, std::memory_order_release);
      }
    }
    scratch_lock.clear(std::memory_order_release);
    if (e != hipSuccess) return e;
  }
  *out = scratch_dev_ptr[dev];
  return hipSuccess;
}

extern "C" size_t ecospa_coupled_score_static_max_bytes(void) { return SCORE_STATIC_BYTES; }

extern "C" int ecospa_coupled_score_static(ecospa_ctx* ctx, const ecospa_pair* pairs, int n_pairs, float* const* scores) {
  const int rc = score_validate(ctx, pairs, n_pairs, scores);
  if (rc) return rc;
  if (ecospa_score_workspace_bytes(pairs, n_pairs) > SCORE_STATIC_BYTES) return ECOSPA_ERR_WORKSPACE;
  void* p = nullptr;
  const hipError_t e = score_static_ptr(&p);
  if (e != hipSuccess) return hip_fail(ctx, e, "hipGetSymbolAddress(scratch)");
  // every slot of the partial sums that the finishing launch reads is written by the first launch of the same call,
  // so nothing has to be cleared between calls
  return score_run(ctx, pairs, n_pairs, scores, 0, 1.f, p, SCORE_STATIC_BYTES);
}
