// Step 3: aligned gather of kept inner dimensions into compact dense matrices and the inverse
// scatter with zero fill (Def. 1 / Alg. 1 removal; gradients written back to the full layout).
//
// Pure data movement, HBM-bound.  Both directions are one "mapped copy": destination slot s
// along the inner axis takes source slot map(s), or zeros when map(s) < 0 (the merging scatter leaves
// such slots as they are: compact parameters and moments written back into their full-size arrays).
//   gather : s = g*kp*unit + i*unit + u  ->  g*n + idx[g,i]*unit + u   (i < k), else -1 (padding)
//   scatter: s = g*n + q*unit + u        ->  g*kp*unit + i*unit + u    where idx[g,i] == q (binary
//            search in the ascending index list), else -1 (pruned)
// Rows (axis 0) are copied two at a time by a wavefront with 16-byte accesses (four loads in flight per lane; more rows
// per wavefront - fewer, longer-lived workgroups - measured slower, one row too); for columns (axis 1)
// each thread owns a fixed set of destination columns, resolves their sources once and then
// walks down the rows, so that the stores are full 16-byte coalesced writes.  A batch of copies
// (all matrices, biases and tables of a layer) runs as ONE launch: launches of this size are
// bound by their fixed cost, not by the bytes they move.
#include "common.h"

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // 16 bytes held in registers

struct MapArgs {
  const int* idx;
  int groups, n, unit, k, kp;
  int scatter;          // 0 gather, 1 scatter with zero fill, 2 scatter that leaves pruned slots untouched
  const int* k_group;   // ragged kept counts (one per group, device memory) or null: every group keeps k
  int ld_idx;           // distance between the index lists of consecutive groups
  int idx_div;          // heads that share one index list (grouped-query attention): group g uses list g / idx_div
};

// Kept count of group g: the ragged count is clamped to what the destination and the index list hold.
__device__ __forceinline__ int map_kept(const MapArgs& m, int g) {
  if (!m.k_group) return m.k;
  const int kg = m.k_group[g / m.idx_div], cap = m.kp < m.ld_idx ? m.kp : m.ld_idx;
  return kg < 0 ? 0 : (kg < cap ? kg : cap);
}

__device__ __forceinline__ long long map_slot(const MapArgs& m, long long s) {
  if (!m.scatter) {
    const int per = m.kp * m.unit;
    const int g = static_cast<int>(s / per), rem = static_cast<int>(s % per);
    const int i = rem / m.unit, u = rem % m.unit;
    if (i >= map_kept(m, g)) return -1;
    return static_cast<long long>(g) * m.n +
           static_cast<long long>(m.idx[static_cast<long long>(g / m.idx_div) * m.ld_idx + i]) * m.unit + u;
  }
  const int g = static_cast<int>(s / m.n), rem = static_cast<int>(s % m.n);
  const int q = rem / m.unit, u = rem % m.unit;
  const int* list = m.idx + static_cast<long long>(g / m.idx_div) * m.ld_idx;
  const int kg = map_kept(m, g);
  int lo = 0, hi = kg;   // first position with list[pos] >= q
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (list[mid] < q) lo = mid + 1; else hi = mid;
  }
  if (lo >= kg || list[lo] != q) return -1;
  return static_cast<long long>(g) * m.kp * m.unit + static_cast<long long>(lo) * m.unit + u;
}

// One mapped copy of a batch; all items of a batch share one launch (block ranges in `blk_begin`).
#define MAP_MAX_ITEMS 120    // descriptors travel as kernel arguments (about 15.5 KB)
#define MAP_COL_ROWS 4      // rows a column-copy thread keeps in flight
struct MapItemDev {
  const void* src;
  void* dst;
  void* dst_t;    // axis 0 gather: also the transposed copy of dst, [other, dst_slots] (null: none)
  const void* src_b;   // axis 0 gather: second source, its rows interleaved with those of src (null: none)
  MapArgs m;
  long long ld_src, ld_dst, ld_dst_t;
  int other;
  int dst_slots;
  int gx;         // axis 1: blocks along the destination columns; with dst_t: 64-wide tiles along the columns
  int rpb;        // axis 1: rows per workgroup
  int blk_begin;  // first block of this item
  unsigned char esize;      // 2 or 4 bytes per element
  unsigned char axis;
  unsigned char vec;        // 16-byte accesses are legal
  unsigned char lds_path;   // axis 1 gather with aligned rows: source window staged through LDS
};
static_assert(sizeof(MapItemDev) == 128, "descriptor size");
// cos/sin tables of the kept rotary blocks (Eq. 6): one element per thread.  The same code serves the launch of its
// own and the workgroups that a gather launch carries along (the tables follow from the same index lists as the
// gathers, so a layer's compaction needs no second launch for them).
struct RopeArgs {
  const int* idx;        // kept blocks per head, or null (block i at slot i)
  const int* k_group;    // ragged kept counts per head, or null
  float* cos_out;
  float* sin_out;
  double base;
  int h, L, k, kp, d_h, ld_idx;
};
__device__ __forceinline__ void rope_table_element(const RopeArgs& r, long long e) {
  const long long tot = static_cast<long long>(r.h) * r.L * r.kp;
  if (e >= tot) return;
  const int i = static_cast<int>(e % r.kp);
  const int t = static_cast<int>((e / r.kp) % r.L);
  const int g = static_cast<int>(e / (static_cast<long long>(r.kp) * r.L));
  float c = 1.f, s = 0.f;
  int kg = r.k;
  if (r.k_group) {
    const int cap = r.kp < r.ld_idx ? r.kp : r.ld_idx;
    kg = r.k_group[g] < 0 ? 0 : (r.k_group[g] < cap ? r.k_group[g] : cap);
  }
  if (i < kg) {
    const int p = r.idx ? r.idx[static_cast<long long>(g) * r.ld_idx + i] : i;
    const double theta = exp(-2.0 * static_cast<double>(p) / static_cast<double>(r.d_h) * log(r.base));
    const double ang = static_cast<double>(t) * theta;
    c = static_cast<float>(cos(ang));
    s = static_cast<float>(sin(ang));
  }
  r.cos_out[e] = c;
  r.sin_out[e] = s;
}

struct MapBatch {
  int n_items;
  int rope_blk0;                  // first of the workgroups that fill the rotary tables (behind the copies), -1: none
  int first_blk[MAP_MAX_ITEMS];   // blk_begin of every item, side by side: the search for a block's item stays in a few cache lines
  MapItemDev it[MAP_MAX_ITEMS];
  RopeArgs rope;
};
static_assert(sizeof(MapBatch) <= 16384, "kernel arguments of one launch");

// ---- axis 0: a wavefront copies MAP_ROW_PER_WAVE destination rows at a time, the loads of all of them in flight
#define MAP_ROW_PER_WAVE 2
#define MAP_ROWS_PER_BLOCK (4 * MAP_ROW_PER_WAVE)
template <typename E>
__device__ __forceinline__ void map_rows_block(const MapItemDev& t, int blk) {
  const E* __restrict__ src = static_cast<const E*>(t.src);
  E* __restrict__ dst = static_cast<E*>(t.dst);
  const int lane = threadIdx.x & 63;
  const long long row0 = static_cast<long long>(blk) * MAP_ROWS_PER_BLOCK + (threadIdx.x >> 6) * MAP_ROW_PER_WAVE;
  if (row0 >= t.dst_slots) return;
  const long long cols = t.other;
  long long srow[MAP_ROW_PER_WAVE];   // source row, -1: zeros (padding / pruned), -2: no such destination row
  if (t.src_b) {      // two sources interleaved row by row: MAP_ROW_PER_WAVE == 2, one destination row from each
    static_assert(MAP_ROW_PER_WAVE == 2, "a wavefront's two rows are one interleaved pair");
    const E* __restrict__ srcs[2] = {src, static_cast<const E*>(t.src_b)};
    const long long sr = row0 < t.dst_slots ? map_slot(t.m, row0 >> 1) : -2;
    if (sr == -2) return;
    for (int j = 0; j < 2; ++j)
      for (long long c = lane; c < cols; c += 64)      // rare shape (no transposed copy wanted): plain element copies
        dst[(row0 + j) * t.ld_dst + c] = sr >= 0 ? srcs[j][sr * t.ld_src + c] : E(0);
    return;
  }
#pragma unroll
  for (int j = 0; j < MAP_ROW_PER_WAVE; ++j) {
    srow[j] = row0 + j < t.dst_slots ? map_slot(t.m, row0 + j) : -2;
    if (t.m.scatter == 2 && srow[j] == -1) srow[j] = -2;     // merging scatter: a pruned row keeps its contents
  }
  if (t.vec) {
    constexpr int V = 16 / sizeof(E);
    const u32x4_t zero = {0u, 0u, 0u, 0u};
    const long long nv = cols / V;
    for (long long c0 = 0; c0 < nv; c0 += 128) {         // two 16-byte pieces per lane and row
      u32x4_t x[MAP_ROW_PER_WAVE][2];
#pragma unroll
      for (int j = 0; j < MAP_ROW_PER_WAVE; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const long long c = c0 + lane + 64 * i;          // out of range: a valid piece is loaded and dropped
          const u32x4_t v = reinterpret_cast<const u32x4_t*>(src + (srow[j] >= 0 ? srow[j] : 0) * t.ld_src)[c < nv ? c : nv - 1];
          x[j][i] = srow[j] >= 0 ? v : zero;
        }
#pragma unroll
      for (int j = 0; j < MAP_ROW_PER_WAVE; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const long long c = c0 + lane + 64 * i;
          if (srow[j] > -2 && c < nv) reinterpret_cast<u32x4_t*>(dst + (row0 + j) * t.ld_dst)[c] = x[j][i];
        }
    }
    for (int j = 0; j < MAP_ROW_PER_WAVE; ++j)
      if (srow[j] > -2)
        for (long long c = nv * V + lane; c < cols; c += 64)
          dst[(row0 + j) * t.ld_dst + c] = srow[j] >= 0 ? src[srow[j] * t.ld_src + c] : E(0);
  } else {
    for (int j = 0; j < MAP_ROW_PER_WAVE; ++j)
      if (srow[j] > -2)
        for (long long c = lane; c < cols; c += 64)
          dst[(row0 + j) * t.ld_dst + c] = srow[j] >= 0 ? src[srow[j] * t.ld_src + c] : E(0);
  }
}

// ---- axis 0 with a transposed copy: a workgroup gathers a tile of 64 destination rows x 64 columns, stores it as it
// is and, through a padded LDS tile, transposed - the transposed copies the contractions want beside a compact matrix
// come out of the gather itself instead of a second pass that reads the compact matrix again.
template <typename E>
__device__ __forceinline__ void map_rows_tr_block(const MapItemDev& t, int blk, unsigned char* lds_raw) {
  E* tile = reinterpret_cast<E*>(lds_raw);                                   // [64][65]
  long long* srow = reinterpret_cast<long long*>(lds_raw + 64 * 65 * 4);     // [64]: source row, -1: zeros
  const E* __restrict__ src = static_cast<const E*>(t.src);
  E* __restrict__ dst = static_cast<E*>(t.dst);
  E* __restrict__ dst_t = static_cast<E*>(t.dst_t);
  const int tid = threadIdx.x;
  const int r0 = (blk / t.gx) * 64, c0 = (blk % t.gx) * 64;
  const int rows = t.dst_slots, cols = t.other;
  const E* __restrict__ src_b = t.src_b ? static_cast<const E*>(t.src_b) : src;
  // two sources interleaved row by row (src_b): destination row s is row map(s / 2) of src (s even) or of src_b
  if (tid < 64) srow[tid] = r0 + tid < rows ? map_slot(t.m, t.src_b ? (r0 + tid) >> 1 : r0 + tid) : -1;
  __syncthreads();
  constexpr int V = 16 / sizeof(E), CH = 64 / V;            // elements per 16 bytes, 16-byte pieces per tile row
  if (t.vec) {
    const u32x4_t zero = {0u, 0u, 0u, 0u};
    for (int p = tid; p < 64 * CH; p += 256) {
      const int r = p / CH, c = (p % CH) * V;
      const long long sr = srow[r];
      const bool inside = r0 + r < rows && c0 + c < cols;   // cols % V == 0: a piece is inside or outside as a whole
      union { u32x4_t v; E e[V]; } x;
      x.v = zero;
      if (inside && sr >= 0) x.v = *reinterpret_cast<const u32x4_t*>(((r & 1) ? src_b : src) + sr * t.ld_src + c0 + c);
      if (inside) *reinterpret_cast<u32x4_t*>(dst + static_cast<long long>(r0 + r) * t.ld_dst + c0 + c) = x.v;
#pragma unroll
      for (int v = 0; v < V; ++v) tile[(c + v) * 65 + r] = x.e[v];
    }
    __syncthreads();
    for (int p = tid; p < 64 * CH; p += 256) {
      const int c = p / CH, r = (p % CH) * V;                 // row c of dst_t, V consecutive destination rows
      if (c0 + c < cols && r0 + r < rows) {
        union { u32x4_t v; E e[V]; } x;
#pragma unroll
        for (int v = 0; v < V; ++v) x.e[v] = tile[c * 65 + r + v];
        *reinterpret_cast<u32x4_t*>(dst_t + static_cast<long long>(c0 + c) * t.ld_dst_t + r0 + r) = x.v;
      }
    }
  } else {
    for (int p = tid; p < 64 * 64; p += 256) {
      const int r = p / 64, c = p % 64;
      const bool inside = r0 + r < rows && c0 + c < cols;
      const E x = (inside && srow[r] >= 0) ? ((r & 1) ? src_b : src)[srow[r] * t.ld_src + c0 + c] : E(0);
      if (inside) dst[static_cast<long long>(r0 + r) * t.ld_dst + c0 + c] = x;
      tile[c * 65 + r] = x;
    }
    __syncthreads();
    for (int p = tid; p < 64 * 64; p += 256) {
      const int c = p / 64, r = p % 64;
      if (c0 + c < cols && r0 + r < rows) dst_t[static_cast<long long>(c0 + c) * t.ld_dst_t + r0 + r] = tile[c * 65 + r];
    }
  }
}

// ---- axis 1: a thread owns V destination columns, resolves their sources once and walks down its
// rows MAP_COL_ROWS at a time (that many independent gathers in flight) ---------------------------
template <typename E, bool VEC>
__device__ __forceinline__ void map_cols_block(const MapItemDev& t, int blk) {
  constexpr int V = VEC ? 16 / sizeof(E) : 1;
  const E* __restrict__ src = static_cast<const E*>(t.src);
  E* __restrict__ dst = static_cast<E*>(t.dst);
  const int bx = blk % t.gx, by = blk / t.gx;
  const long long c0 = (static_cast<long long>(bx) * 256 + threadIdx.x) * V;
  if (c0 >= t.dst_slots) return;
  long long sc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) sc[v] = (c0 + v < t.dst_slots) ? map_slot(t.m, c0 + v) : -1;
  const long long r0 = static_cast<long long>(by) * t.rpb;
  const long long r1 = (r0 + t.rpb < t.other) ? r0 + t.rpb : t.other;
  const bool merge = t.m.scatter == 2;          // merging scatter: slots without a source are not written
  const bool full = c0 + V <= t.dst_slots && !merge;
  for (long long rb = r0; rb < r1; rb += MAP_COL_ROWS) {
    alignas(16) E vals[MAP_COL_ROWS][V];
#pragma unroll
    for (int q = 0; q < MAP_COL_ROWS; ++q) {
      const long long r = (rb + q < r1) ? rb + q : r1 - 1;
      const E* s = src + r * t.ld_src;
#pragma unroll
      for (int v = 0; v < V; ++v) vals[q][v] = sc[v] >= 0 ? s[sc[v]] : E(0);
    }
#pragma unroll
    for (int q = 0; q < MAP_COL_ROWS; ++q) {
      if (rb + q >= r1) break;
      E* d = dst + (rb + q) * t.ld_dst + c0;
      if (VEC && full) {
        *reinterpret_cast<uint4*>(d) = *reinterpret_cast<const uint4*>(vals[q]);
      } else {
#pragma unroll
        for (int v = 0; v < V; ++v)
          if (c0 + v < t.dst_slots && (sc[v] >= 0 || !merge)) d[v] = vals[q][v];
      }
    }
  }
}

// ---- axis 1 through LDS (gather and scatter): a workgroup owns MAP_LDS_GROUPS x V destination columns
// and MAP_LDS_ROWS_TOTAL rows.  The source columns of its destination range are ascending, so they lie
// in one window of the source row; the window is fetched with coalesced 16-byte loads into LDS, MAP_LDS_ROWS rows
// at a time, and every thread picks the V columns of its 16-byte store from there.  If the window is
// wider than the LDS tile (kept indices far apart: below a quarter kept) the region falls back to element-wise
// gathers.  Measured: 16 column groups x 16 rows per pass beat 32 x 8 (1.5 % on a 24-layer launch, 12 % on a
// single layer's) and 8 x 32; 64 x 4 is a third slower.
#define MAP_LDS_GROUPS 16          // 16-byte column groups per workgroup
#define MAP_LDS_ROWS (256 / MAP_LDS_GROUPS)   // rows per pass (MAP_LDS_GROUPS * MAP_LDS_ROWS = 256 threads)
#define MAP_LDS_ROWS_TOTAL 64      // rows per workgroup
#define MAP_LDS_CHUNKS 64          // 16-byte chunks of the source window per row
template <typename E>
__device__ __forceinline__ void map_cols_lds_block(const MapItemDev& t, int blk, unsigned char* lds_raw) {
  constexpr int V = 16 / sizeof(E);
  constexpr int CB = MAP_LDS_GROUPS * V;
  E* tile = reinterpret_cast<E*>(lds_raw);                                   // [MAP_LDS_ROWS][MAP_LDS_CHUNKS * V]
  int* smap = reinterpret_cast<int*>(lds_raw + MAP_LDS_ROWS * MAP_LDS_CHUNKS * 16);   // [CB]
  int* lim = smap + CB;                                                      // [2]: min, max source column
  const E* __restrict__ src = static_cast<const E*>(t.src);
  E* __restrict__ dst = static_cast<E*>(t.dst);
  const int tid = threadIdx.x;
  const int bx = blk % t.gx, by = blk / t.gx;
  const long long c0 = static_cast<long long>(bx) * CB;
  const long long r_begin = static_cast<long long>(by) * t.rpb;
  const long long r_end = r_begin + t.rpb < t.other ? r_begin + t.rpb : t.other;
  if (tid == 0) { lim[0] = 0x7fffffff; lim[1] = -1; }
  __syncthreads();
  for (int c = tid; c < CB; c += 256) {
    const long long sc = (c0 + c < t.dst_slots) ? map_slot(t.m, c0 + c) : -1;
    smap[c] = static_cast<int>(sc);
    if (sc >= 0) { atomicMin(&lim[0], static_cast<int>(sc)); atomicMax(&lim[1], static_cast<int>(sc)); }
  }
  __syncthreads();
  const int smin = lim[0], smax = lim[1];
  const int w0 = smin & ~(V - 1);                            // window start, 16-byte aligned
  const int chunks = smax >= 0 ? (smax - w0) / V + 1 : 0;    // 16-byte chunks per row
  const int grp = tid % MAP_LDS_GROUPS, rr = tid / MAP_LDS_GROUPS;   // this thread's column group and row slot
  const long long dc = c0 + static_cast<long long>(grp) * V;  // its first destination column
  const bool full = dc + V <= t.dst_slots;
  if (chunks > MAP_LDS_CHUNKS || chunks == 0) {
    // window too wide for the tile (or no source column at all: padding only): element by element
    for (long long r = r_begin + rr; r < r_end; r += MAP_LDS_ROWS) {
      alignas(16) E vals[V];
#pragma unroll
      for (int v = 0; v < V; ++v) vals[v] = smap[grp * V + v] >= 0 ? src[r * t.ld_src + smap[grp * V + v]] : E(0);
      E* d = dst + r * t.ld_dst + dc;
      if (full) *reinterpret_cast<uint4*>(d) = *reinterpret_cast<const uint4*>(vals);
      else
        for (int v = 0; v < V; ++v)
          if (dc + v < t.dst_slots) d[v] = vals[v];
    }
    return;
  }
  int off[V];   // this thread's V source columns relative to the window (-1 = padding slot)
#pragma unroll
  for (int v = 0; v < V; ++v) off[v] = smap[grp * V + v] >= 0 ? smap[grp * V + v] - w0 : -1;
  // From here on every wavefront works alone on its own rows of each pass (its own part of the
  // tile): lane = (row, 16-byte column group), for the loads as for the stores, so only
  // wavefront-level ordering is needed between the LDS writes and reads - no workgroup barriers.
  static_assert(MAP_LDS_GROUPS * MAP_LDS_ROWS == 256 && 64 % MAP_LDS_GROUPS == 0, "a row's groups lie in one wavefront");
  constexpr int RPW = 64 / MAP_LDS_GROUPS;     // rows per wavefront and pass
  const int lane = tid & 63, wave = tid >> 6;
  const int wrow = wave * RPW + lane / MAP_LDS_GROUPS, l16 = lane % MAP_LDS_GROUPS;
  E* wtile = tile + wrow * MAP_LDS_CHUNKS * V;
  // the windows of the next two passes are fetched into registers while this pass is gathered and stored; a
  // lane whose chunk lies beyond the window fetches the window's last chunk instead and drops it
  constexpr int PC = MAP_LDS_CHUNKS / MAP_LDS_GROUPS;   // 16-byte chunks a lane fetches per pass
  u32x4_t pre_a[PC], pre_b[PC];
#define MAP_FETCH(PRE, RB)                                                                          \
  if ((RB) < r_end) {                                                                               \
    const long long rn_ = (RB) + wrow;                                                              \
    const E* sp_ = src + (rn_ < r_end ? rn_ : r_end - 1) * t.ld_src + w0;                           \
    _Pragma("unroll") for (int i = 0; i < PC; ++i) {                                                \
      const int ch_ = l16 + i * MAP_LDS_GROUPS;                                                     \
      PRE[i] = *reinterpret_cast<const u32x4_t*>(sp_ + (ch_ < chunks ? ch_ : chunks - 1) * V);      \
    }                                                                                               \
  }
#define MAP_PASS(PRE, RB)                                                                           \
  {                                                                                                 \
    const long long r_ = (RB) + wrow;                                                               \
    _Pragma("unroll") for (int i = 0; i < PC; ++i) {                                                \
      const int ch_ = l16 + i * MAP_LDS_GROUPS;                                                     \
      if (ch_ < chunks) *reinterpret_cast<u32x4_t*>(wtile + ch_ * V) = PRE[i];                      \
    }                                                                                               \
    MAP_FETCH(PRE, (RB) + 2 * MAP_LDS_ROWS)                                                         \
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");                                          \
    __builtin_amdgcn_wave_barrier();                                                                \
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");                                          \
    if (r_ < r_end && dc < t.dst_slots) {                                                           \
      alignas(16) E vals[V];                                                                        \
      _Pragma("unroll") for (int v = 0; v < V; ++v) vals[v] = off[v] >= 0 ? wtile[off[v]] : E(0);   \
      E* d = dst + r_ * t.ld_dst + dc;                                                              \
      if (full) *reinterpret_cast<uint4*>(d) = *reinterpret_cast<const uint4*>(vals);               \
      else                                                                                          \
        for (int v = 0; v < V; ++v)                                                                 \
          if (dc + v < t.dst_slots) d[v] = vals[v];                                                 \
    }                                                                                               \
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");                                          \
    __builtin_amdgcn_wave_barrier();                                                                \
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");                                          \
  }
  MAP_FETCH(pre_a, r_begin)
  MAP_FETCH(pre_b, r_begin + MAP_LDS_ROWS)
  for (long long rb = r_begin; rb < r_end; rb += 2 * MAP_LDS_ROWS) {
    MAP_PASS(pre_a, rb)
    if (rb + MAP_LDS_ROWS < r_end) MAP_PASS(pre_b, rb + MAP_LDS_ROWS)
  }
#undef MAP_PASS
#undef MAP_FETCH
}

__global__ __launch_bounds__(256) void map_batch_kernel(const MapBatch b) {
  constexpr int LDS_COLS = MAP_LDS_ROWS * MAP_LDS_CHUNKS * 16 + (MAP_LDS_GROUPS * 8 + 2) * 4, LDS_TR = 64 * 65 * 4 + 64 * 8;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[LDS_COLS > LDS_TR ? LDS_COLS : LDS_TR];
  const int blk = blockIdx.x;
  if (b.rope_blk0 >= 0 && blk >= b.rope_blk0) {
    rope_table_element(b.rope, static_cast<long long>(blk - b.rope_blk0) * 256 + threadIdx.x);
    return;
  }
  int i = 0, hi = b.n_items - 1;          // last item whose first block is <= blk
  while (i < hi) {
    const int mid = (i + hi + 1) >> 1;
    if (b.first_blk[mid] <= blk) i = mid; else hi = mid - 1;
  }
  const MapItemDev& t = b.it[i];
  const int local = blk - t.blk_begin;
  if (t.dst_t) {
    if (t.esize == 2) map_rows_tr_block<bf16_t>(t, local, lds_raw);
    else map_rows_tr_block<float>(t, local, lds_raw);
  } else if (t.axis == 0) {
    if (t.esize == 2) map_rows_block<bf16_t>(t, local);
    else map_rows_block<float>(t, local);
  } else if (t.lds_path) {
    if (t.esize == 2) map_cols_lds_block<bf16_t>(t, local, lds_raw);
    else map_cols_lds_block<float>(t, local, lds_raw);
  } else if (t.esize == 2) {
    if (t.vec) map_cols_block<bf16_t, true>(t, local);
    else map_cols_block<bf16_t, false>(t, local);
  } else {
    if (t.vec) map_cols_block<float, true>(t, local);
    else map_cols_block<float, false>(t, local);
  }
}

static int validate_map(const ecospa_map_item& q) {
  if (!q.src || !q.dst || !q.idx) return ECOSPA_ERR_NULL;
  if (!dtype_ok(q.dtype)) return ECOSPA_ERR_DTYPE;
  if (q.axis != 0 && q.axis != 1) return ECOSPA_ERR_SHAPE;
  if (q.scatter < 0 || q.scatter > 2) return ECOSPA_ERR_SHAPE;
  if (q.groups < 1 || q.n < 1 || q.unit < 1 || q.n % q.unit || q.other_extent < 1) return ECOSPA_ERR_SHAPE;
  if (q.idx_div < 0 || (q.idx_div > 1 && q.groups % q.idx_div)) return ECOSPA_ERR_SHAPE;
  if (q.k_group) {      // ragged: the counts live on the device, only the capacities can be checked here
    if (q.kp < 1 || q.ld_idx < 1) return ECOSPA_ERR_K;
  } else if (q.k < 1 || q.k > q.n / q.unit || q.kp < q.k || (q.ld_idx != 0 && q.ld_idx < q.k)) {
    return ECOSPA_ERR_K;
  }
  const long long full_slots = static_cast<long long>(q.groups) * q.n;
  const long long cmp_slots = static_cast<long long>(q.groups) * q.kp * q.unit;
  if (full_slots > (1ll << 31) - 1 || cmp_slots > (1ll << 31) - 1) return ECOSPA_ERR_SHAPE;
  const long long src_slots = q.scatter ? cmp_slots : full_slots;
  const long long dst_slots = q.scatter ? full_slots : cmp_slots;
  if (q.other_extent > (1ll << 31) - 1) return ECOSPA_ERR_SHAPE;
  if (q.src_b) {      // interleaved sources: row gathers of single rows
    if (q.axis != 0 || q.scatter != 0 || q.unit != 1 || 2 * cmp_slots > (1ll << 31) - 1) return ECOSPA_ERR_SHAPE;
  }
  if (q.dst_t) {      // the transposed copy comes out of row gathers only
    if (q.axis != 0 || q.scatter != 0 || q.ld_dst_t < (q.src_b ? 2 : 1) * dst_slots) return ECOSPA_ERR_SHAPE;
  }
  if (q.axis == 0) {
    if (q.ld_src < q.other_extent || q.ld_dst < q.other_extent) return ECOSPA_ERR_SHAPE;
  } else {
    if (q.ld_src < src_slots || q.ld_dst < dst_slots) return ECOSPA_ERR_SHAPE;
  }
  return ECOSPA_OK;
}

static int validate_rope(const ecospa_rope_item& r) {
  if (!r.cos_out || !r.sin_out) return ECOSPA_ERR_NULL;
  if (r.h < 1 || r.L < 1 || r.d_h < 2 || !(r.base > 1.0)) return ECOSPA_ERR_SHAPE;
  if (r.k_group) {
    if (!r.idx) return ECOSPA_ERR_NULL;
    if (r.kp < 1 || r.ld_idx < 1) return ECOSPA_ERR_K;
  } else if (r.k < 1 || r.kp < r.k || r.k > r.d_h / 2 || (r.ld_idx != 0 && r.ld_idx < r.k)) {
    return ECOSPA_ERR_K;
  }
  if (static_cast<long long>(r.h) * r.L * r.kp > (1ll << 31) - 1) return ECOSPA_ERR_SHAPE;
  return ECOSPA_OK;
}
static RopeArgs rope_args(const ecospa_rope_item& r) {
  RopeArgs a;
  a.idx = r.idx; a.k_group = r.k_group; a.cos_out = r.cos_out; a.sin_out = r.sin_out; a.base = r.base;
  a.h = r.h; a.L = r.L; a.k = r.k; a.kp = r.kp; a.d_h = r.d_h; a.ld_idx = r.ld_idx ? r.ld_idx : r.k;
  return a;
}

extern "C" int ecospa_compact_batch_rope(ecospa_ctx* ctx, const ecospa_map_item* items, int n_items, const ecospa_rope_item* rope) {
  if (!ctx || !items) return ECOSPA_ERR_NULL;
  if (n_items < 1) return ECOSPA_ERR_SHAPE;
  for (int i = 0; i < n_items; ++i) {
    const int rc = validate_map(items[i]);
    if (rc) return rc;
  }
  if (rope) {
    const int rc = validate_rope(*rope);
    if (rc) return rc;
  }
  for (int first = 0; first < n_items; first += MAP_MAX_ITEMS) {
    MapBatch b;
    memset(&b, 0, sizeof(b));
    b.rope_blk0 = -1;
    b.n_items = n_items - first < MAP_MAX_ITEMS ? n_items - first : MAP_MAX_ITEMS;
    // workgroups the launch has with the most rows per workgroup: only a launch that would leave the
    // chip short of work at that size (a single layer's matrices) takes fewer rows per workgroup
    long long coarse = 0;
    for (int i = 0; i < b.n_items; ++i) {
      const ecospa_map_item& q = items[first + i];
      const long long slots = static_cast<long long>(q.groups) * (q.scatter ? q.n : q.kp * q.unit);
      const int V = 16 / static_cast<int>(dtype_size(q.dtype));
      coarse += q.axis == 0 ? (slots + MAP_ROWS_PER_BLOCK - 1) / MAP_ROWS_PER_BLOCK
                            : (q.other_extent + MAP_LDS_ROWS_TOTAL - 1) / MAP_LDS_ROWS_TOTAL *
                                  ((slots + MAP_LDS_GROUPS * V - 1) / (MAP_LDS_GROUPS * V));
    }
    const bool short_launch = coarse < 4096;
    long long blk = 0;
    for (int i = 0; i < b.n_items; ++i) {
      const ecospa_map_item& q = items[first + i];
      MapItemDev& t = b.it[i];
      t.src = q.src; t.dst = q.dst;
      t.m = MapArgs{q.idx, q.groups, q.n, q.unit, q.k, q.kp, q.scatter, q.k_group, q.ld_idx ? q.ld_idx : q.k, q.idx_div > 0 ? q.idx_div : 1};
      const long long full_slots = static_cast<long long>(q.groups) * q.n;
      const long long cmp_slots = static_cast<long long>(q.groups) * q.kp * q.unit;
      t.dst_slots = static_cast<int>(q.scatter ? full_slots : (q.src_b ? 2 : 1) * cmp_slots);
      t.other = static_cast<int>(q.other_extent); t.ld_src = q.ld_src; t.ld_dst = q.ld_dst;
      t.dst_t = q.dst_t; t.ld_dst_t = q.ld_dst_t; t.src_b = q.src_b;
      t.esize = static_cast<unsigned char>(dtype_size(q.dtype));
      t.axis = static_cast<unsigned char>(q.axis);
      const int V = 16 / t.esize;
      t.blk_begin = static_cast<int>(blk);
      b.first_blk[i] = t.blk_begin;
      if (q.dst_t) {
        t.vec = aligned16(q.src) && aligned16(q.src_b) && aligned16(q.dst) && aligned16(q.dst_t) && q.ld_src % V == 0 && q.ld_dst % V == 0 &&
                q.ld_dst_t % V == 0 && t.dst_slots % V == 0 && q.other_extent % V == 0;
        t.gx = static_cast<int>((q.other_extent + 63) / 64);
        blk += static_cast<long long>((t.dst_slots + 63) / 64) * t.gx;
      } else if (q.axis == 0) {
        t.vec = aligned16(q.src) && aligned16(q.dst) && q.ld_src % V == 0 && q.ld_dst % V == 0;
        blk += (t.dst_slots + MAP_ROWS_PER_BLOCK - 1) / MAP_ROWS_PER_BLOCK;
      } else {
        t.vec = aligned16(q.dst) && q.ld_dst % V == 0;
        // the LDS path reads whole 16-byte chunks of the source rows, up to the end of the last kept chunk: the row's
        // storage (its leading dimension) must reach that far
        const long long src_slots = q.scatter ? cmp_slots : full_slots;
        t.lds_path = t.vec && q.scatter != 2 && aligned16(q.src) && q.ld_src % V == 0 && q.ld_src >= (src_slots + V - 1) / V * V;
        if (t.lds_path) {
          t.gx = static_cast<int>((t.dst_slots + MAP_LDS_GROUPS * V - 1) / (MAP_LDS_GROUPS * V));
          int rpb = MAP_LDS_ROWS_TOTAL;
          while (short_launch && rpb > 2 * MAP_LDS_ROWS && (q.other_extent + rpb - 1) / rpb * t.gx < 1024) rpb /= 2;
          t.rpb = rpb;
          blk += (q.other_extent + rpb - 1) / rpb * t.gx;
        } else {
          const int vv = t.vec ? V : 1;
          t.gx = static_cast<int>((t.dst_slots + 256ll * vv - 1) / (256ll * vv));
          // enough row chunks to fill the chip, at least MAP_COL_ROWS rows each
          int rpb = MAP_COL_ROWS;
          while (rpb < 64 && (q.other_extent + rpb - 1) / rpb * t.gx > 4096) rpb *= 2;
          t.rpb = rpb;
          blk += (q.other_extent + rpb - 1) / rpb * t.gx;
        }
      }
      if (blk > (1ll << 30)) return ECOSPA_ERR_SHAPE;
    }
    if (rope && first + MAP_MAX_ITEMS >= n_items) {      // the tables ride on the last launch of the batch
      b.rope = rope_args(*rope);
      b.rope_blk0 = static_cast<int>(blk);
      blk += (static_cast<long long>(rope->h) * rope->L * rope->kp + 255) / 256;
      if (blk > (1ll << 30)) return ECOSPA_ERR_SHAPE;
    }
    hipLaunchKernelGGL(map_batch_kernel, dim3(static_cast<unsigned>(blk)), dim3(256), 0, ctx->stream, b);
    ECOSPA_CHECK_LAUNCH(ctx, "map_batch_kernel");
  }
  return ECOSPA_OK;
}

extern "C" int ecospa_compact_batch(ecospa_ctx* ctx, const ecospa_map_item* items, int n_items) {
  return ecospa_compact_batch_rope(ctx, items, n_items, nullptr);
}

static int mapped_copy(ecospa_ctx* ctx, const void* src, void* dst, int dtype, int axis, int groups, int n, int unit,
                       int k, int kp, long long other, long long ld_src, long long ld_dst, const int* idx,
                       int scatter) {
  ecospa_map_item q;
  q.src = src; q.dst = dst; q.dtype = dtype; q.axis = axis; q.groups = groups; q.n = n; q.unit = unit; q.k = k;
  q.kp = kp; q.other_extent = other; q.ld_src = ld_src; q.ld_dst = ld_dst; q.idx = idx; q.scatter = scatter;
  q.k_group = nullptr; q.ld_idx = 0; q.idx_div = 0; q.dst_t = nullptr; q.ld_dst_t = 0; q.src_b = nullptr;
  return ecospa_compact_batch(ctx, &q, 1);
}

extern "C" int ecospa_compact(ecospa_ctx* ctx, const void* src, void* dst, int dtype, int axis, int groups, int n,
                              int unit, int k, int kp, long long other_extent, long long ld_src, long long ld_dst,
                              const int* idx) {
  return mapped_copy(ctx, src, dst, dtype, axis, groups, n, unit, k, kp, other_extent, ld_src, ld_dst, idx, 0);
}

extern "C" int ecospa_scatter(ecospa_ctx* ctx, const void* src, void* dst, int dtype, int axis, int groups, int n,
                              int unit, int k, int kp, long long other_extent, long long ld_src, long long ld_dst,
                              const int* idx) {
  return mapped_copy(ctx, src, dst, dtype, axis, groups, n, unit, k, kp, other_extent, ld_src, ld_dst, idx, 1);
}

// ---- debugging aid: the caller's contract on index lists, checked on the device -------------------------------
__global__ __launch_bounds__(256) void idx_flag_clear_kernel(int* flag) { if (threadIdx.x == 0) *flag = 0; }
__global__ __launch_bounds__(256) void idx_check_kernel(const int* __restrict__ idx, int groups, int ld_idx, int k,
                                                        const int* __restrict__ k_group, int n_units, int* flag) {
  const long long e = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= static_cast<long long>(groups) * ld_idx) return;
  const int g = static_cast<int>(e / ld_idx), i = static_cast<int>(e % ld_idx);
  int kg = k;
  if (k_group) {
    kg = k_group[g];
    if (kg < 0 || kg > ld_idx) { *flag = 1; return; }     // a count the list cannot hold
  }
  if (i >= kg) return;
  const int v = idx[e];
  const bool bad = v < 0 || v >= n_units || (i > 0 && idx[e - 1] >= v);
  if (bad) *flag = 1;       // every writer stores the same value
}

extern "C" int ecospa_check_indices(ecospa_ctx* ctx, const int* idx, int groups, int ld_idx, int k, const int* k_group,
                                    int n_units) {
  if (!ctx || !idx) return ECOSPA_ERR_NULL;
  if (groups < 1 || n_units < 1 || ld_idx < 1 || static_cast<long long>(groups) * ld_idx > (1ll << 31) - 1) return ECOSPA_ERR_SHAPE;
  if (!k_group && (k < 1 || k > ld_idx || k > n_units)) return ECOSPA_ERR_K;
  if (!ctx->ws || ctx->ws_bytes < sizeof(int)) return ECOSPA_ERR_WORKSPACE;
  int* flag = static_cast<int*>(ctx->ws);
  hipLaunchKernelGGL(idx_flag_clear_kernel, dim3(1), dim3(64), 0, ctx->stream, flag);
  ECOSPA_CHECK_LAUNCH(ctx, "idx_flag_clear_kernel");
  const long long tot = static_cast<long long>(groups) * ld_idx;
  hipLaunchKernelGGL(idx_check_kernel, dim3(static_cast<unsigned>((tot + 255) / 256)), dim3(256), 0, ctx->stream, idx, groups,
                     ld_idx, k, k_group, n_units, flag);
  ECOSPA_CHECK_LAUNCH(ctx, "idx_check_kernel");
  int host_flag = 0;
  hipError_t e = hipMemcpyAsync(&host_flag, flag, sizeof(int), hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "ecospa_check_indices");
  return host_flag ? ECOSPA_ERR_INDEX : ECOSPA_OK;
}

// ---- transposed copies of compact matrices ------------------------------------------------------------
// The input-gradient contractions dY W read W with its contraction index slow; with a transposed copy of
// the (small, compact) matrix beside it they become x W^T contractions like the forward ones, which the
// matrix-core kernels run faster.  Plain HBM-bound data movement: 64 x 64 tiles through LDS, 16-byte
// accesses on both sides when the shapes allow; all matrices of a layer in one launch.
#define TR_MAX_ITEMS 64
struct TrItemDev {
  const void* src;
  void* dst;
  long long ld_src, ld_dst;
  int rows, cols;      // of src; dst is [cols, rows]
  int esize, vec;
  int tiles_c;         // 64-wide tiles along the columns of src
  int blk_begin;
};
struct TrBatch {
  int n_items;
  int first_blk[TR_MAX_ITEMS];
  TrItemDev it[TR_MAX_ITEMS];
};

template <typename E>
__device__ __forceinline__ void transpose_tile(const TrItemDev& t, int local, E* tile /* [64][65] */) {
  const E* __restrict__ src = static_cast<const E*>(t.src);
  E* __restrict__ dst = static_cast<E*>(t.dst);
  const int r0 = (local / t.tiles_c) * 64, c0 = (local % t.tiles_c) * 64;
  const int tid = threadIdx.x;
  constexpr int V = 16 / sizeof(E), CH = 64 / V;            // elements per 16 bytes, 16-byte pieces per tile row
  if (t.vec) {
    for (int p = tid; p < 64 * CH; p += 256) {
      const int r = p / CH, c = (p % CH) * V;
      alignas(16) E x[V];
      if (r0 + r < t.rows && c0 + c < t.cols)                // cols % V == 0: a piece is inside or outside as a whole
        *reinterpret_cast<u32x4_t*>(x) = *reinterpret_cast<const u32x4_t*>(src + static_cast<long long>(r0 + r) * t.ld_src + c0 + c);
      else
        for (int v = 0; v < V; ++v) x[v] = E(0);
#pragma unroll
      for (int v = 0; v < V; ++v) tile[(c + v) * 65 + r] = x[v];
    }
    __syncthreads();
    for (int p = tid; p < 64 * CH; p += 256) {
      const int c = p / CH, r = (p % CH) * V;                 // row c of dst, V consecutive source rows
      if (c0 + c < t.cols && r0 + r < t.rows) {
        alignas(16) E x[V];
#pragma unroll
        for (int v = 0; v < V; ++v) x[v] = tile[c * 65 + r + v];
        *reinterpret_cast<u32x4_t*>(dst + static_cast<long long>(c0 + c) * t.ld_dst + r0 + r) = *reinterpret_cast<const u32x4_t*>(x);
      }
    }
  } else {
    for (int p = tid; p < 64 * 64; p += 256) {
      const int r = p / 64, c = p % 64;
      tile[c * 65 + r] = (r0 + r < t.rows && c0 + c < t.cols) ? src[static_cast<long long>(r0 + r) * t.ld_src + c0 + c] : E(0);
    }
    __syncthreads();
    for (int p = tid; p < 64 * 64; p += 256) {
      const int c = p / 64, r = p % 64;
      if (c0 + c < t.cols && r0 + r < t.rows) dst[static_cast<long long>(c0 + c) * t.ld_dst + r0 + r] = tile[c * 65 + r];
    }
  }
}

__global__ __launch_bounds__(256) void transpose_batch_kernel(const TrBatch b) {
  __shared__ __attribute__((aligned(16))) unsigned char tile_raw[64 * 65 * 4];
  const int blk = blockIdx.x;
  int i = 0, hi = b.n_items - 1;          // last item whose first block is <= blk
  while (i < hi) {
    const int mid = (i + hi + 1) >> 1;
    if (b.first_blk[mid] <= blk) i = mid; else hi = mid - 1;
  }
  const TrItemDev& t = b.it[i];
  if (t.esize == 2) transpose_tile<bf16_t>(t, blk - t.blk_begin, reinterpret_cast<bf16_t*>(tile_raw));
  else transpose_tile<float>(t, blk - t.blk_begin, reinterpret_cast<float*>(tile_raw));
}

extern "C" int ecospa_transpose_batch(ecospa_ctx* ctx, const ecospa_transpose_item* items, int n_items) {
  if (!ctx || !items) return ECOSPA_ERR_NULL;
  if (n_items < 1) return ECOSPA_ERR_SHAPE;
  for (int i = 0; i < n_items; ++i) {
    const ecospa_transpose_item& q = items[i];
    if (!q.src || !q.dst) return ECOSPA_ERR_NULL;
    if (!dtype_ok(q.dtype)) return ECOSPA_ERR_DTYPE;
    if (q.rows < 1 || q.cols < 1 || q.ld_src < q.cols || q.ld_dst < q.rows) return ECOSPA_ERR_SHAPE;
  }
  for (int first = 0; first < n_items; first += TR_MAX_ITEMS) {
    TrBatch b;
    memset(&b, 0, sizeof(b));
    b.n_items = n_items - first < TR_MAX_ITEMS ? n_items - first : TR_MAX_ITEMS;
    long long blk = 0;
    for (int i = 0; i < b.n_items; ++i) {
      const ecospa_transpose_item& q = items[first + i];
      TrItemDev& t = b.it[i];
      t.src = q.src; t.dst = q.dst; t.ld_src = q.ld_src; t.ld_dst = q.ld_dst; t.rows = q.rows; t.cols = q.cols;
      t.esize = static_cast<int>(dtype_size(q.dtype));
      const int V = 16 / t.esize;
      t.vec = aligned16(q.src) && aligned16(q.dst) && q.ld_src % V == 0 && q.ld_dst % V == 0 && q.rows % V == 0 && q.cols % V == 0;
      t.tiles_c = (q.cols + 63) / 64;
      t.blk_begin = static_cast<int>(blk);
      b.first_blk[i] = t.blk_begin;
      blk += static_cast<long long>((q.rows + 63) / 64) * t.tiles_c;
      if (blk > (1ll << 30)) return ECOSPA_ERR_SHAPE;
    }
    hipLaunchKernelGGL(transpose_batch_kernel, dim3(static_cast<unsigned>(blk)), dim3(256), 0, ctx->stream, b);
    ECOSPA_CHECK_LAUNCH(ctx, "transpose_batch_kernel");
  }
  return ECOSPA_OK;
}

// ---- cos/sin tables of the kept rotary blocks (Eq. 6) -------------------------------------------
__global__ void rope_table_kernel(const RopeArgs r) {
  rope_table_element(r, static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x);
}

static int rope_launch(ecospa_ctx* ctx, const ecospa_rope_item& r) {
  const int rc = validate_rope(r);
  if (rc) return rc;
  const long long tot = static_cast<long long>(r.h) * r.L * r.kp;
  hipLaunchKernelGGL(rope_table_kernel, dim3(static_cast<unsigned>((tot + 255) / 256)), dim3(256), 0, ctx->stream, rope_args(r));
  ECOSPA_CHECK_LAUNCH(ctx, "rope_table_kernel");
  return ECOSPA_OK;
}

extern "C" int ecospa_rope_table(ecospa_ctx* ctx, const int* idx, int h, int L, int k, int kp, int d_h, double base,
                                 float* cos_out, float* sin_out) {
  if (!ctx) return ECOSPA_ERR_NULL;
  const ecospa_rope_item r{idx, nullptr, h, L, k, kp, d_h, 0, base, cos_out, sin_out};
  return rope_launch(ctx, r);
}

extern "C" int ecospa_rope_table_ragged(ecospa_ctx* ctx, const int* idx, int ld_idx, const int* k_group, int h, int L,
                                        int kp, int d_h, double base, float* cos_out, float* sin_out) {
  if (!ctx || !idx || !k_group) return ECOSPA_ERR_NULL;
  const ecospa_rope_item r{idx, k_group, h, L, 0, kp, d_h, ld_idx, base, cos_out, sin_out};
  return rope_launch(ctx, r);
}
