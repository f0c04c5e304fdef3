// Parameter update on the compact tensors (Alg. 1 "Update W"): fused multi-tensor AdamW.
//
// Alg. 1 removes the optimizer moments of a removed row/column together with the row/column itself, so
// after compaction the parameters, their fp32 master copies and both moments all live in the compact
// layout and one elementwise pass updates them.  The pass is pure streaming: per element it reads the
// gradient, both moments and the parameter and writes both moments and the parameter (and, for fp32
// master weights, the bf16 working copy the contractions read) - HBM-bound, nothing is read twice.
// All tensors of a model share one launch; each workgroup owns a contiguous slice of one tensor.
#include "common.h"

#define ADAMW_MAX_ITEMS 192       // descriptors travel as kernel arguments
#define ADAMW_THREADS 256
#define ADAMW_VEC 8               // elements per thread and pass
#define ADAMW_PASSES 2            // passes per workgroup: ADAMW_THREADS * ADAMW_VEC * ADAMW_PASSES elements
#define ADAMW_CHUNK (ADAMW_THREADS * ADAMW_VEC * ADAMW_PASSES)

struct AdamwItemDev {
  void* w;
  bf16_t* w_lp;
  const void* g;
  void* m;
  void* v;
  long long n;
  int w_bf16, g_bf16, s_bf16;   // element types: 1 = bf16, 0 = fp32
  int vec;                      // every pointer is 16-byte aligned: 8 elements per access
  int blk_begin;
};
struct AdamwBatch {
  int n_items;
  float lr, beta1, beta2, omb1, omb2, eps, wd, inv_bc1, inv_bc2;
  int first_blk[ADAMW_MAX_ITEMS];   // blk_begin of every item, side by side: the search for a block's item stays in a few cache lines
  AdamwItemDev it[ADAMW_MAX_ITEMS];
};
static_assert(sizeof(AdamwBatch) <= 16384, "kernel arguments of one launch");

template <typename T> __device__ __forceinline__ void load8(const T* p, float (&x)[ADAMW_VEC]);
template <> __device__ __forceinline__ void load8<float>(const float* p, float (&x)[ADAMW_VEC]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float (&x)[ADAMW_VEC]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  const uint32_t u[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(u[i] << 16);
    x[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
  }
}
template <typename T> __device__ __forceinline__ void store8(T* p, const float (&x)[ADAMW_VEC]);
template <> __device__ __forceinline__ void store8<float>(float* p, const float (&x)[ADAMW_VEC]) {
  *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
}
template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t* p, const float (&x)[ADAMW_VEC]) {
  uint32_t u[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    u[i] = static_cast<uint32_t>(f32_to_bf16(x[2 * i])) | (static_cast<uint32_t>(f32_to_bf16(x[2 * i + 1])) << 16);
  *reinterpret_cast<uint4*>(p) = make_uint4(u[0], u[1], u[2], u[3]);
}

__device__ __forceinline__ void adamw_element(const AdamwBatch& b, float g, float& w, float& m, float& v) {
  m = b.beta1 * m + b.omb1 * g;
  v = b.beta2 * v + b.omb2 * g * g;
  const float denom = sqrtf(v * b.inv_bc2) + b.eps;
  w = w - b.lr * ((m * b.inv_bc1) / denom + b.wd * w);
}

template <typename WT, typename GT, typename ST>
__device__ __forceinline__ void adamw_slice(const AdamwBatch& b, const AdamwItemDev& t, long long e0) {
  WT* __restrict__ w = static_cast<WT*>(t.w);
  const GT* __restrict__ g = static_cast<const GT*>(t.g);
  ST* __restrict__ m = static_cast<ST*>(t.m);
  ST* __restrict__ v = static_cast<ST*>(t.v);
  bf16_t* __restrict__ lp = t.w_lp;
  const long long e1 = e0 + ADAMW_CHUNK < t.n ? e0 + ADAMW_CHUNK : t.n;
  if (t.vec && e1 - e0 == ADAMW_CHUNK) {
    // all loads of the slice first (2 passes x 4 streams in flight per thread), then the arithmetic and the stores
    float xg[ADAMW_PASSES][ADAMW_VEC], xw[ADAMW_PASSES][ADAMW_VEC], xm[ADAMW_PASSES][ADAMW_VEC], xv[ADAMW_PASSES][ADAMW_VEC];
#pragma unroll
    for (int p = 0; p < ADAMW_PASSES; ++p) {
      const long long e = e0 + (static_cast<long long>(p) * ADAMW_THREADS + threadIdx.x) * ADAMW_VEC;
      load8<GT>(g + e, xg[p]);
      load8<ST>(m + e, xm[p]);
      load8<ST>(v + e, xv[p]);
      load8<WT>(w + e, xw[p]);
    }
#pragma unroll
    for (int p = 0; p < ADAMW_PASSES; ++p) {
      const long long e = e0 + (static_cast<long long>(p) * ADAMW_THREADS + threadIdx.x) * ADAMW_VEC;
#pragma unroll
      for (int i = 0; i < ADAMW_VEC; ++i) adamw_element(b, xg[p][i], xw[p][i], xm[p][i], xv[p][i]);
      store8<ST>(m + e, xm[p]);
      store8<ST>(v + e, xv[p]);
      store8<WT>(w + e, xw[p]);
      if (lp) store8<bf16_t>(lp + e, xw[p]);
    }
    return;
  }
  for (long long e = e0 + threadIdx.x; e < e1; e += ADAMW_THREADS) {
    float xw = load_f32<WT>(w + e), xm = load_f32<ST>(m + e), xv = load_f32<ST>(v + e);
    adamw_element(b, load_f32<GT>(g + e), xw, xm, xv);
    store_f32<ST>(m + e, xm);
    store_f32<ST>(v + e, xv);
    store_f32<WT>(w + e, xw);
    if (lp) lp[e] = f32_to_bf16(xw);
  }
}

__global__ __launch_bounds__(ADAMW_THREADS) void adamw_kernel(const AdamwBatch b) {
  const int blk = blockIdx.x;
  int i = 0, hi = b.n_items - 1;          // last item whose first block is <= blk
  while (i < hi) {
    const int mid = (i + hi + 1) >> 1;
    if (b.first_blk[mid] <= blk) i = mid; else hi = mid - 1;
  }
  const AdamwItemDev& t = b.it[i];
  const long long e0 = static_cast<long long>(blk - t.blk_begin) * ADAMW_CHUNK;
  const int code = (t.w_bf16 << 2) | (t.g_bf16 << 1) | t.s_bf16;
  switch (code) {
    case 0: adamw_slice<float, float, float>(b, t, e0); break;
    case 1: adamw_slice<float, float, bf16_t>(b, t, e0); break;
    case 2: adamw_slice<float, bf16_t, float>(b, t, e0); break;
    case 3: adamw_slice<float, bf16_t, bf16_t>(b, t, e0); break;
    case 4: adamw_slice<bf16_t, float, float>(b, t, e0); break;
    case 5: adamw_slice<bf16_t, float, bf16_t>(b, t, e0); break;
    case 6: adamw_slice<bf16_t, bf16_t, float>(b, t, e0); break;
    default: adamw_slice<bf16_t, bf16_t, bf16_t>(b, t, e0); break;
  }
}

static int validate_adamw(const ecospa_adamw_item& q) {
  if (!q.w || !q.g || !q.m || !q.v) return ECOSPA_ERR_NULL;
  if (!dtype_ok(q.w_dtype) || !dtype_ok(q.g_dtype) || !dtype_ok(q.s_dtype)) return ECOSPA_ERR_DTYPE;
  if (q.w_lp && q.w_dtype != ECOSPA_F32) return ECOSPA_ERR_DTYPE;   // a working copy belongs to fp32 master weights
  if (q.n < 1) return ECOSPA_ERR_SHAPE;
  return ECOSPA_OK;
}

extern "C" int ecospa_adamw(ecospa_ctx* ctx, const ecospa_adamw_item* items, int n_items, const ecospa_adamw_hyper* hp) {
  if (!ctx || !items || !hp) return ECOSPA_ERR_NULL;
  if (n_items < 1) return ECOSPA_ERR_SHAPE;
  if (hp->step < 1 || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) ||
      !(hp->eps >= 0.f) || !(hp->lr >= 0.f) || !(hp->weight_decay >= 0.f))
    return ECOSPA_ERR_SHAPE;
  for (int i = 0; i < n_items; ++i) {
    const int rc = validate_adamw(items[i]);
    if (rc) return rc;
  }
  AdamwBatch b;
  memset(&b, 0, sizeof(b));
  b.lr = hp->lr; b.beta1 = hp->beta1; b.beta2 = hp->beta2; b.eps = hp->eps; b.wd = hp->weight_decay;
  const double b1 = hp->beta1, b2 = hp->beta2;     // the float values, so both sides use the same betas
  b.omb1 = static_cast<float>(1.0 - b1);
  b.omb2 = static_cast<float>(1.0 - b2);
  b.inv_bc1 = static_cast<float>(1.0 / (1.0 - pow(b1, hp->step)));
  b.inv_bc2 = static_cast<float>(1.0 / (1.0 - pow(b2, hp->step)));
  for (int first = 0; first < n_items; first += ADAMW_MAX_ITEMS) {
    b.n_items = n_items - first < ADAMW_MAX_ITEMS ? n_items - first : ADAMW_MAX_ITEMS;
    long long blk = 0;
    for (int i = 0; i < b.n_items; ++i) {
      const ecospa_adamw_item& q = items[first + i];
      AdamwItemDev& t = b.it[i];
      t.w = q.w; t.w_lp = static_cast<bf16_t*>(q.w_lp); t.g = q.g; t.m = q.m; t.v = q.v; t.n = q.n;
      t.w_bf16 = q.w_dtype == ECOSPA_BF16; t.g_bf16 = q.g_dtype == ECOSPA_BF16; t.s_bf16 = q.s_dtype == ECOSPA_BF16;
      t.vec = aligned16(q.w) && aligned16(q.g) && aligned16(q.m) && aligned16(q.v) && (!q.w_lp || aligned16(q.w_lp));
      t.blk_begin = static_cast<int>(blk);
      b.first_blk[i] = t.blk_begin;
      blk += (q.n + ADAMW_CHUNK - 1) / ADAMW_CHUNK;
      if (blk > (1ll << 30)) return ECOSPA_ERR_SHAPE;
    }
    hipLaunchKernelGGL(adamw_kernel, dim3(static_cast<unsigned>(blk)), dim3(ADAMW_THREADS), 0, ctx->stream, b);
    ECOSPA_CHECK_LAUNCH(ctx, "adamw_kernel");
  }
  return ECOSPA_OK;
}
