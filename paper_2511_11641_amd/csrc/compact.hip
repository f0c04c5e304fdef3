// Step 3: aligned gather of kept inner dimensions into compact dense matrices and the inverse
// scatter with zero fill (Def. 1 / Alg. 1 removal; gradients written back to the full layout).
//
// Pure data movement, HBM-bound.  Both directions are one "mapped copy": destination slot s
// along the inner axis takes source slot map(s), or zeros when map(s) < 0.
//   gather : s = g*kp*unit + i*unit + u  ->  g*n + idx[g,i]*unit + u   (i < k), else -1 (padding)
//   scatter: s = g*n + q*unit + u        ->  g*kp*unit + i*unit + u    where idx[g,i] == q (binary
//            search in the ascending index list), else -1 (pruned)
// Rows (axis 0) are copied by one wavefront each with 16-byte accesses; for columns (axis 1)
// each thread owns a fixed set of destination columns, resolves their sources once and then
// walks down the rows, so that the stores are full 16-byte coalesced writes.
#include "common.h"

struct MapArgs {
  const int* idx;
  int groups, n, unit, k, kp;
  int scatter;
};

__device__ __forceinline__ long long map_slot(const MapArgs& m, long long s) {
  if (!m.scatter) {
    const int per = m.kp * m.unit;
    const int g = static_cast<int>(s / per), rem = static_cast<int>(s % per);
    const int i = rem / m.unit, u = rem % m.unit;
    if (i >= m.k) return -1;
    return static_cast<long long>(g) * m.n + static_cast<long long>(m.idx[g * m.k + i]) * m.unit + u;
  }
  const int g = static_cast<int>(s / m.n), rem = static_cast<int>(s % m.n);
  const int q = rem / m.unit, u = rem % m.unit;
  const int* list = m.idx + static_cast<long long>(g) * m.k;
  int lo = 0, hi = m.k;   // first position with list[pos] >= q
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (list[mid] < q) lo = mid + 1; else hi = mid;
  }
  if (lo >= m.k || list[lo] != q) return -1;
  return static_cast<long long>(g) * m.kp * m.unit + static_cast<long long>(lo) * m.unit + u;
}

// ---- axis 0: one wavefront per destination row ------------------------------------------------
template <typename E, bool VEC>
__global__ __launch_bounds__(256) void map_rows_kernel(const E* __restrict__ src, E* __restrict__ dst, MapArgs m,
                                                       long long dst_rows, long long cols, long long ld_src,
                                                       long long ld_dst) {
  const int lane = threadIdx.x & 63;
  const long long row = static_cast<long long>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= dst_rows) return;
  const long long srow = map_slot(m, row);
  E* d = dst + row * ld_dst;
  if (VEC) {
    constexpr int V = 16 / sizeof(E);
    const uint4 zero = make_uint4(0, 0, 0, 0);
    const long long nv = cols / V;
    const uint4* s4 = srow >= 0 ? reinterpret_cast<const uint4*>(src + srow * ld_src) : nullptr;
    uint4* d4 = reinterpret_cast<uint4*>(d);
    for (long long c = lane; c < nv; c += 64) d4[c] = s4 ? s4[c] : zero;
    for (long long c = nv * V + lane; c < cols; c += 64) d[c] = srow >= 0 ? src[srow * ld_src + c] : E(0);
  } else {
    for (long long c = lane; c < cols; c += 64) d[c] = srow >= 0 ? src[srow * ld_src + c] : E(0);
  }
}

// ---- axis 1: thread owns V destination columns, loops over a chunk of rows ----------------------
template <typename E, bool VEC>
__global__ __launch_bounds__(256) void map_cols_kernel(const E* __restrict__ src, E* __restrict__ dst, MapArgs m,
                                                       long long rows, long long dst_cols, long long ld_src,
                                                       long long ld_dst, int rows_per_block) {
  constexpr int V = VEC ? 16 / sizeof(E) : 1;
  const long long c0 = (static_cast<long long>(blockIdx.x) * 256 + threadIdx.x) * V;
  if (c0 >= dst_cols) return;
  long long sc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) sc[v] = (c0 + v < dst_cols) ? map_slot(m, c0 + v) : -1;
  const long long r0 = static_cast<long long>(blockIdx.y) * rows_per_block;
  const long long r1 = (r0 + rows_per_block < rows) ? r0 + rows_per_block : rows;
  const bool full = c0 + V <= dst_cols;
  for (long long r = r0; r < r1; ++r) {
    const E* s = src + r * ld_src;
    alignas(16) E vals[V];
#pragma unroll
    for (int v = 0; v < V; ++v) vals[v] = sc[v] >= 0 ? s[sc[v]] : E(0);
    E* d = dst + r * ld_dst + c0;
    if (VEC && full) {
      *reinterpret_cast<uint4*>(d) = *reinterpret_cast<const uint4*>(vals);
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v)
        if (c0 + v < dst_cols) d[v] = vals[v];
    }
  }
}

template <typename E>
static int launch_map(ecospa_ctx* ctx, const void* src, void* dst, int axis, const MapArgs& m, long long dst_slots,
                      long long other, long long ld_src, long long ld_dst) {
  const E* s = static_cast<const E*>(src);
  E* d = static_cast<E*>(dst);
  constexpr int V = 16 / sizeof(E);
  if (axis == 0) {
    const bool vec = aligned16(src) && aligned16(dst) && ld_src % V == 0 && ld_dst % V == 0;
    const unsigned grid = static_cast<unsigned>((dst_slots + 3) / 4);
    if (vec)
      hipLaunchKernelGGL((map_rows_kernel<E, true>), dim3(grid), dim3(256), 0, ctx->stream, s, d, m, dst_slots, other,
                         ld_src, ld_dst);
    else
      hipLaunchKernelGGL((map_rows_kernel<E, false>), dim3(grid), dim3(256), 0, ctx->stream, s, d, m, dst_slots, other,
                         ld_src, ld_dst);
  } else {
    const bool vec = aligned16(dst) && ld_dst % V == 0;
    const int vv = vec ? V : 1;
    const unsigned gx = static_cast<unsigned>((dst_slots + 256ll * vv - 1) / (256ll * vv));
    // enough row chunks to fill the chip, at least 8 rows each
    int rpb = 8;
    while (rpb < 64 && (other + rpb - 1) / rpb * gx > 4096) rpb *= 2;
    const unsigned gy = static_cast<unsigned>((other + rpb - 1) / rpb);
    if (vec)
      hipLaunchKernelGGL((map_cols_kernel<E, true>), dim3(gx, gy), dim3(256), 0, ctx->stream, s, d, m, other, dst_slots,
                         ld_src, ld_dst, rpb);
    else
      hipLaunchKernelGGL((map_cols_kernel<E, false>), dim3(gx, gy), dim3(256), 0, ctx->stream, s, d, m, other,
                         dst_slots, ld_src, ld_dst, rpb);
  }
  ECOSPA_CHECK_LAUNCH(ctx, "map kernel");
  return ECOSPA_OK;
}

static int mapped_copy(ecospa_ctx* ctx, const void* src, void* dst, int dtype, int axis, int groups, int n, int unit,
                       int k, int kp, long long other, long long ld_src, long long ld_dst, const int* idx,
                       int scatter) {
  if (!ctx || !src || !dst || !idx) return ECOSPA_ERR_NULL;
  if (!dtype_ok(dtype)) return ECOSPA_ERR_DTYPE;
  if (axis != 0 && axis != 1) return ECOSPA_ERR_SHAPE;
  if (groups < 1 || n < 1 || unit < 1 || n % unit || other < 1) return ECOSPA_ERR_SHAPE;
  if (k < 1 || k > n / unit || kp < k) return ECOSPA_ERR_K;
  const long long full_slots = static_cast<long long>(groups) * n;
  const long long cmp_slots = static_cast<long long>(groups) * kp * unit;
  if (full_slots > (1ll << 31) - 1 || cmp_slots > (1ll << 31) - 1) return ECOSPA_ERR_SHAPE;
  const long long src_slots = scatter ? cmp_slots : full_slots;
  const long long dst_slots = scatter ? full_slots : cmp_slots;
  if (axis == 0) {
    if (ld_src < other || ld_dst < other) return ECOSPA_ERR_SHAPE;
  } else {
    if (ld_src < src_slots || ld_dst < dst_slots) return ECOSPA_ERR_SHAPE;
  }
  MapArgs m{idx, groups, n, unit, k, kp, scatter};
  if (dtype == ECOSPA_BF16) return launch_map<bf16_t>(ctx, src, dst, axis, m, dst_slots, other, ld_src, ld_dst);
  return launch_map<float>(ctx, src, dst, axis, m, dst_slots, other, ld_src, ld_dst);
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

// ---- cos/sin tables of the kept rotary blocks (Eq. 6) -------------------------------------------
__global__ void rope_table_kernel(const int* __restrict__ idx, int h, int L, int k, int kp, int d_h, double base,
                                  float* __restrict__ cos_out, float* __restrict__ sin_out) {
  const long long tot = static_cast<long long>(h) * L * kp;
  const long long e = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (e >= tot) return;
  const int i = static_cast<int>(e % kp);
  const int t = static_cast<int>((e / kp) % L);
  const int g = static_cast<int>(e / (static_cast<long long>(kp) * L));
  float c = 1.f, s = 0.f;
  if (i < k) {
    const int p = idx ? idx[g * k + i] : i;
    const double theta = exp(-2.0 * static_cast<double>(p) / static_cast<double>(d_h) * log(base));
    const double ang = static_cast<double>(t) * theta;
    c = static_cast<float>(cos(ang));
    s = static_cast<float>(sin(ang));
  }
  cos_out[e] = c;
  sin_out[e] = s;
}

extern "C" int ecospa_rope_table(ecospa_ctx* ctx, const int* idx, int h, int L, int k, int kp, int d_h, double base,
                                 float* cos_out, float* sin_out) {
  if (!ctx || !cos_out || !sin_out) return ECOSPA_ERR_NULL;
  if (h < 1 || L < 1 || d_h < 2 || !(base > 1.0)) return ECOSPA_ERR_SHAPE;
  if (k < 1 || kp < k || k > d_h / 2) return ECOSPA_ERR_K;
  const long long tot = static_cast<long long>(h) * L * kp;
  hipLaunchKernelGGL(rope_table_kernel, dim3(static_cast<unsigned>((tot + 255) / 256)), dim3(256), 0, ctx->stream, idx,
                     h, L, k, kp, d_h, base, cos_out, sin_out);
  ECOSPA_CHECK_LAUNCH(ctx, "rope_table_kernel");
  return ECOSPA_OK;
}
