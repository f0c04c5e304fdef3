// Step 1: per-dimension coupled importance score (paper Eq. 10, criterion of Eq. 12).
//
// HBM-bound: every weight element of every pair in the batch is read exactly once with
// 16-byte loads.
//   1. score_sumsq_kernel  - one launch per SCORE_MAX_PAIRS pairs: squared row norms (a wavefront
//                            takes four rows at a time, all their loads in flight, then lane-
//                            permutation sums) and squared column norms of the [d, n] member (one
//                            workgroup per strip of one 128-byte line = 8 lanes x 16 bytes, over
//                            all d rows, eight loads in flight per lane)
//   2. score_finish_kernel - one launch per SCORE_FIN_MAX_PAIRS pairs, one workgroup per (pair,
//                            group): r = |a||b|, group L2 norm, normalised scores
// No floating-point atomics; all reduction orders are fixed.
#include "common.h"

#define SCORE_MAX_PAIRS 96         // descriptors travel as kernel arguments (about 10 KB)
#define SCORE_ROWS_PER_BLOCK 16   // row-norm blocks: 4 waves x 4 rows
#define SCORE_COL_LANES 8         // column-norm blocks: 8 lanes (128 bytes of columns) x 32 row slots
#define SCORE_COL_SLOTS (256 / SCORE_COL_LANES)

struct ScorePairDev {
  const void* w1;
  const void* w1b;
  const void* w2;
  long long ld1, ld1b, ld2;
  float* a_sq;     // [rows]            squared norms of a_j
  float* b_sq;     // [rows]            squared norms of b_j (rows of W_k, or columns of w2)
  int rows;        // groups * n
  int groups, n, unit;
  int d1, d2;
  int kind, dtype;
  int fisher;      // 1: squared gradient sums for Eq. 8 (w1 and w1b are added, not multiplied)
  int blk_row1, blk_row2, blk_col, blk_end;   // first block index of each phase in launch 1
};
struct ScoreBatch {
  int n_pairs;
  ScorePairDev p[SCORE_MAX_PAIRS];
};

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
    if (row0 < p.rows) {
      float sums[NR];
      rows_sumsq<T, NR>(w + row0 * ld, wb ? wb + row0 * p.ld1b : nullptr, ld, p.ld1b, len, p.rows - row0, vec_ok, p.fisher != 0, lane, sums);
      if (lane == 0) {
#pragma unroll
        for (int j = 0; j < NR; ++j)
          if (row0 + j < p.rows) out[row0 + j] = sums[j];
      }
    }
    return;
  }
  // ---- squared column norms of w2 [d2, rows]: one strip of SCORE_COL_LANES x V columns, all rows ----
  const int local = blk - p.blk_col;
  constexpr int W = SCORE_COL_LANES * V;
  if (local * W >= p.rows) return;                 // padding of the range (whole workgroup)
  const int slot = tid / SCORE_COL_LANES, ln = tid % SCORE_COL_LANES;
  const T* w = static_cast<const T*>(p.w2);
  const int col0 = local * W + ln * V;
  const bool vec_ok = (p.ld2 % V == 0) && ((reinterpret_cast<uintptr_t>(w) & 15u) == 0);
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.f;
  if (vec_ok && col0 + V <= p.rows) {
    for (int r0 = slot; r0 < p.d2; r0 += 8 * SCORE_COL_SLOTS) {     // 8 independent loads in flight
      float a[8][V];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int r = r0 + q * SCORE_COL_SLOTS;
        load_vec<T>(w + static_cast<long long>(r < p.d2 ? r : r0) * p.ld2 + col0, a[q]);
        if (r >= p.d2) {
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
    for (int r = slot; r < p.d2; r += SCORE_COL_SLOTS) {
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (col0 + i < p.rows) {
          float a = load_f32<T>(w + static_cast<long long>(r) * p.ld2 + col0 + i);
          acc[i] += a * a;
        }
    }
  }
  // reduce the row slots in a fixed order: thread (column c, part q) adds slots q, q + PARTS, ...;
  // then the PARTS partial sums of a column are added in order
#pragma unroll
  for (int i = 0; i < V; ++i) lds[slot * (W + 1) + ln * V + i] = acc[i];
  __syncthreads();
  constexpr int PARTS = 256 / W;                    // threads per column
  const int c = tid / PARTS, q = tid % PARTS;
  float s = 0.f;
  for (int k = q; k < SCORE_COL_SLOTS; k += PARTS) s += lds[k * (W + 1) + c];
  __syncthreads();
  lds[c * PARTS + q] = s;
  __syncthreads();
  if (tid < W) {
    float tot = 0.f;
    for (int k = 0; k < PARTS; ++k) tot += lds[tid * PARTS + k];
    const int col = local * W + tid;
    if (col < p.rows) p.b_sq[col] = tot;
  }
}

__global__ __launch_bounds__(256) void score_sumsq_kernel(const ScoreBatch b) {
  __shared__ float lds[SCORE_COL_SLOTS * (SCORE_COL_LANES * 8 + 1)];
  const int blk = blockIdx.x;
  int lo = 0, hi = b.n_pairs - 1;          // last pair whose first block is <= blk
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (b.p[mid].blk_row1 <= blk) lo = mid; else hi = mid - 1;
  }
  const ScorePairDev& p = b.p[lo];
  if (p.dtype == ECOSPA_BF16) score_block<bf16_t>(p, blk, lds);
  else score_block<float>(p, blk, lds);
}

// Finishing launch: one workgroup per (pair, group).  Every thread finishes its units (r = |a| |b|),
// the group's L2 norm of r is reduced in a fixed order, and the normalised scores are written.  It
// needs little per pair, so one launch serves up to SCORE_FIN_MAX_PAIRS pairs (several batches of the
// first launch).
#define SCORE_FIN_THREADS 1024
#define SCORE_FIN_MAX_PAIRS 96
struct ScoreFinPair {
  const float* a_sq;
  const float* b_sq;
  float* scores;
  int n, unit;
  int fin_begin;
  int fisher;          // 1: Eq. 8 instead of Eq. 10: scores[g] = w1 * sum(a_sq of group g) + w2 * sum(b_sq of group g)
  float w1, w2;        //    with w_k = 1 / (2 |W_k| |D|)
};
struct ScoreFinBatch {
  int n_pairs;
  ScoreFinPair p[SCORE_FIN_MAX_PAIRS];
};
__global__ __launch_bounds__(SCORE_FIN_THREADS) void score_finish_kernel(const ScoreFinBatch b) {
  __shared__ float red[SCORE_FIN_THREADS / 64];
  const int blk = blockIdx.x;
  int lo = 0, hi = b.n_pairs - 1;          // last pair whose first workgroup is <= blk
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (b.p[mid].fin_begin <= blk) lo = mid; else hi = mid - 1;
  }
  const ScoreFinPair& p = b.p[lo];
  const int g = blk - p.fin_begin;
  const int nu = p.n / p.unit;
  const int tid = threadIdx.x;
  if (p.fisher) {
    float part = 0.f;
    for (int j = tid; j < p.n; j += SCORE_FIN_THREADS) part += p.w1 * p.a_sq[g * p.n + j] + p.w2 * p.b_sq[g * p.n + j];
    part = wave_sum(part);
    if ((tid & 63) == 0) red[tid >> 6] = part;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
      for (int w = 0; w < SCORE_FIN_THREADS / 64; ++w) tot += red[w];
      p.scores[g] = tot;
    }
    return;
  }
  float* out = p.scores + static_cast<long long>(g) * nu;
  float sq = 0.f;
  for (int u = tid; u < nu; u += SCORE_FIN_THREADS) {
    float a = 0.f, bsum = 0.f;
    for (int j = 0; j < p.unit; ++j) {
      const int row = (g * nu + u) * p.unit + j;
      a += p.a_sq[row];
      bsum += p.b_sq[row];
    }
    const float r = sqrtf(a) * sqrtf(bsum);
    out[u] = r;          // re-read below by the same thread
    sq += r * r;
  }
  sq = wave_sum(sq);
  if ((tid & 63) == 0) red[tid >> 6] = sq;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < SCORE_FIN_THREADS / 64; ++w) tot += red[w];
  const float nrm = sqrtf(tot);
  for (int u = tid; u < nu; u += SCORE_FIN_THREADS) out[u] = nrm > 0.f ? out[u] / nrm : 0.f;
}

// ------------------------------------------------------------------------------------------
static int validate_pair(const ecospa_pair& q) {
  if (q.kind < ECOSPA_PAIR_QK || q.kind > ECOSPA_PAIR_FFN_GATED || !dtype_ok(q.dtype)) return ECOSPA_ERR_DTYPE;
  if (!q.w1 || !q.w2 || (q.kind == ECOSPA_PAIR_FFN_GATED && !q.w1b)) return ECOSPA_ERR_NULL;
  if (q.groups < 1 || q.n < 1 || q.unit < 1 || q.d1 < 1 || q.d2 < 1 || q.n % q.unit) return ECOSPA_ERR_SHAPE;
  const long long rows = static_cast<long long>(q.groups) * q.n;
  if (rows > (1ll << 30)) return ECOSPA_ERR_SHAPE;
  if (q.ld1 < q.d1) return ECOSPA_ERR_SHAPE;
  if (q.kind == ECOSPA_PAIR_FFN_GATED && q.ld1b < q.d1) return ECOSPA_ERR_SHAPE;
  if (q.kind == ECOSPA_PAIR_QK ? q.ld2 < q.d2 : q.ld2 < rows) return ECOSPA_ERR_SHAPE;
  return ECOSPA_OK;
}

static size_t pair_ws_bytes(const ecospa_pair& q) {
  const size_t rows = static_cast<size_t>(q.groups) * q.n;
  return 2 * align_up(rows * 4, 256);   // a_sq, b_sq
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
static int score_run(ecospa_ctx* ctx, const ecospa_pair* pairs, int n_pairs, float* const* scores, int fisher,
                     float n_samples) {
  if (!ctx || !pairs || !scores) return ECOSPA_ERR_NULL;
  if (n_pairs < 1) return ECOSPA_ERR_SHAPE;
  for (int i = 0; i < n_pairs; ++i) {
    int rc = validate_pair(pairs[i]);
    if (rc) return rc;
    if (!scores[i]) return ECOSPA_ERR_NULL;
  }
  const size_t need = ecospa_score_workspace_bytes(pairs, n_pairs);
  if (!ctx->ws || ctx->ws_bytes < need) return ECOSPA_ERR_WORKSPACE;
  WsCarver ws(ctx->ws, ctx->ws_bytes);

  ScoreFinBatch fb;
  fb.n_pairs = 0;
  int fin = 0;
  for (int first = 0; first < n_pairs; first += SCORE_MAX_PAIRS) {
    ScoreBatch b;
    memset(&b, 0, sizeof(b));
    b.n_pairs = (n_pairs - first < SCORE_MAX_PAIRS) ? n_pairs - first : SCORE_MAX_PAIRS;
    int blk = 0;
    for (int i = 0; i < b.n_pairs; ++i) {
      const ecospa_pair& q = pairs[first + i];
      ScorePairDev& p = b.p[i];
      p.w1 = q.w1; p.w1b = (q.kind == ECOSPA_PAIR_FFN_GATED) ? q.w1b : nullptr; p.w2 = q.w2;
      p.ld1 = q.ld1; p.ld1b = q.ld1b; p.ld2 = q.ld2;
      p.rows = q.groups * q.n;
      p.groups = q.groups; p.n = q.n; p.unit = q.unit;
      p.d1 = q.d1; p.d2 = q.d2; p.kind = q.kind; p.dtype = q.dtype; p.fisher = fisher;
      p.a_sq = static_cast<float*>(ws.take(static_cast<size_t>(p.rows) * 4));
      const int row_blocks = (p.rows + SCORE_ROWS_PER_BLOCK - 1) / SCORE_ROWS_PER_BLOCK;
      p.blk_row1 = blk;
      blk += row_blocks;
      p.blk_row2 = blk;
      p.b_sq = static_cast<float*>(ws.take(static_cast<size_t>(p.rows) * 4));
      if (q.kind == ECOSPA_PAIR_QK) {
        blk += row_blocks;
        p.blk_col = blk;
      } else {
        p.blk_col = blk;
        const int strip = SCORE_COL_LANES * (q.dtype == ECOSPA_BF16 ? 8 : 4);
        blk += (p.rows + strip - 1) / strip;
      }
      p.blk_end = blk;
    }
    if (!ws.ok()) return ECOSPA_ERR_WORKSPACE;
    hipLaunchKernelGGL(score_sumsq_kernel, dim3(blk), dim3(256), 0, ctx->stream, b);
    ECOSPA_CHECK_LAUNCH(ctx, "score_sumsq_kernel");
    // queue the finishing work of this batch; launch it when the queue is full or the batches are done
    for (int i = 0; i < b.n_pairs; ++i) {
      if (fb.n_pairs == SCORE_FIN_MAX_PAIRS) {
        hipLaunchKernelGGL(score_finish_kernel, dim3(fin), dim3(SCORE_FIN_THREADS), 0, ctx->stream, fb);
        ECOSPA_CHECK_LAUNCH(ctx, "score_finish_kernel");
        fb.n_pairs = 0;
        fin = 0;
      }
      ScoreFinPair& f = fb.p[fb.n_pairs++];
      f.a_sq = b.p[i].a_sq; f.b_sq = b.p[i].b_sq; f.scores = scores[first + i];
      f.n = b.p[i].n; f.unit = b.p[i].unit; f.fin_begin = fin; f.fisher = fisher;
      const double members = b.p[i].kind == ECOSPA_PAIR_FFN_GATED ? 2.0 : 1.0;   // W_gate and W_up form the first member
      f.w1 = fisher ? static_cast<float>(0.5 / (members * b.p[i].n * static_cast<double>(b.p[i].d1) * n_samples)) : 0.f;
      f.w2 = fisher ? static_cast<float>(0.5 / (b.p[i].n * static_cast<double>(b.p[i].d2) * n_samples)) : 0.f;
      fin += b.p[i].groups;
    }
  }
  if (fb.n_pairs > 0) {
    hipLaunchKernelGGL(score_finish_kernel, dim3(fin), dim3(SCORE_FIN_THREADS), 0, ctx->stream, fb);
    ECOSPA_CHECK_LAUNCH(ctx, "score_finish_kernel");
  }
  return ECOSPA_OK;
}

extern "C" int ecospa_coupled_score(ecospa_ctx* ctx, const ecospa_pair* pairs, int n_pairs, float* const* scores) {
  return score_run(ctx, pairs, n_pairs, scores, 0, 1.f);
}

extern "C" int ecospa_pair_fisher(ecospa_ctx* ctx, const ecospa_pair* grads, int n_pairs, float n_samples,
                                  float* const* fisher) {
  if (!(n_samples > 0.f)) return ECOSPA_ERR_SHAPE;
  return score_run(ctx, grads, n_pairs, fisher, 1, n_samples);
}
