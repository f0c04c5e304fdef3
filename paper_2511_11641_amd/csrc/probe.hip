// Measurement aids: a plain streaming read and a plain 1:1 copy of a buffer.  What they reach on a given GPU is the
// ceiling that the HBM-bound steps (score: read only; compaction: read and write) are priced against.
#include "common.h"

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
#define PROBE_U 4      // 16-byte pieces per thread, all in flight together

// Each workgroup takes 256 * PROBE_U consecutive pieces; a thread's pieces are 256 apart (coalesced).
template <bool COPY>
__global__ __launch_bounds__(256) void hbm_probe_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst,
                                                        long long n16, unsigned* __restrict__ sink) {
  const long long base = static_cast<long long>(blockIdx.x) * (256 * PROBE_U) + threadIdx.x;
  u32x4_t v[PROBE_U];
#pragma unroll
  for (int i = 0; i < PROBE_U; ++i) {
    const long long p = base + i * 256;
    v[i] = src[p < n16 ? p : n16 - 1];
  }
  if (COPY) {
#pragma unroll
    for (int i = 0; i < PROBE_U; ++i) {
      const long long p = base + i * 256;
      if (p < n16) dst[p] = v[i];
    }
  } else {
    // the loads must not be dropped: fold them and store on a condition no ordinary buffer content meets
    unsigned acc = 0u;
#pragma unroll
    for (int i = 0; i < PROBE_U; ++i) acc ^= (v[i].x + 0x9e3779b9u) ^ (v[i].y * 0x85ebca6bu) ^ (v[i].z + v[i].w);
    if (acc == 0x5bd1e995u && (v[0].x ^ v[0].w) == 0x1b873593u) *sink = acc;
  }
}

extern "C" int ecospa_hbm_probe(ecospa_ctx* ctx, const void* src, void* dst, size_t bytes, int mode) {
  if (!ctx || !src || !dst) return ECOSPA_ERR_NULL;
  if (mode != 0 && mode != 1) return ECOSPA_ERR_SHAPE;
  if (bytes < 16 || bytes % 16 || bytes > (static_cast<size_t>(1) << 40)) return ECOSPA_ERR_SHAPE;
  if (!aligned16(src) || (mode == 1 && !aligned16(dst)) || (reinterpret_cast<uintptr_t>(dst) & 3u)) return ECOSPA_ERR_ALIGN;
  const long long n16 = static_cast<long long>(bytes / 16);
  const long long blocks = (n16 + 256 * PROBE_U - 1) / (256 * PROBE_U);
  if (blocks > (1ll << 30)) return ECOSPA_ERR_SHAPE;
  if (mode == 1)
    hipLaunchKernelGGL((hbm_probe_kernel<true>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, ctx->stream,
                       static_cast<const u32x4_t*>(src), static_cast<u32x4_t*>(dst), n16, nullptr);
  else
    hipLaunchKernelGGL((hbm_probe_kernel<false>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, ctx->stream,
                       static_cast<const u32x4_t*>(src), nullptr, n16, static_cast<unsigned*>(dst));
  ECOSPA_CHECK_LAUNCH(ctx, "hbm_probe_kernel");
  return ECOSPA_OK;
}
