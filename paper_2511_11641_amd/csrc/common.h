// Shared host/device helpers of the gfx950 library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <atomic>

#include "../../include/ecospa.h"

#define ECOSPA_PROF_MAX 4096   // GEMM launches that one profiling window can hold

struct ecospa_ctx {
  hipStream_t stream;
  void* ws;
  size_t ws_bytes;
  char err[256];
  // optional timing of the GEMM launches with events on `stream` (ecospa_profile_gemm)
  int prof_on, prof_n, prof_cap;
  hipEvent_t* prof_ev;      // 2 events per launch
  double* prof_flop;
};

typedef unsigned short bf16_t;  // raw bfloat16 bits

static inline size_t dtype_size(int dtype) { return dtype == ECOSPA_BF16 ? 2 : 4; }
static inline bool dtype_ok(int dtype) { return dtype == ECOSPA_F32 || dtype == ECOSPA_BF16; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Record a HIP failure on the context and return ERR_HIP.
static inline int hip_fail(ecospa_ctx* ctx, hipError_t e, const char* where) {
  if (ctx) snprintf(ctx->err, sizeof(ctx->err), "%s: %s", where, hipGetErrorString(e));
  return ECOSPA_ERR_HIP;
}
#define ECOSPA_CHECK_LAUNCH(ctx, where)                         \
  do {                                                          \
    hipError_t e__ = hipGetLastError();                         \
    if (e__ != hipSuccess) return hip_fail(ctx, e__, where);    \
  } while (0)

// A kernel that needs more than 64 KB of dynamic LDS has its limit raised once per device before its first launch
// there.  One object per kernel (a function-local static of the launch code); safe to use from several host threads:
// the attribute call is idempotent, so two threads that race only set the same value twice.
struct LdsAttrOnce {
  std::atomic<unsigned long long> done{0};     // one bit per device ordinal (mod 64)
  hipError_t ensure(const void* kern, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
  }
};

// Carve 256-byte aligned pieces out of the caller's workspace.
struct WsCarver {
  char* base;
  size_t off, cap;
  WsCarver(void* p, size_t bytes) : base(static_cast<char*>(p)), off(0), cap(bytes) {}
  void* take(size_t bytes) {
    size_t o = align_up(off, 256);
    off = o + bytes;
    return (base && off <= cap) ? base + o : nullptr;
  }
  bool ok() const { return base != nullptr && off <= cap; }
};

#ifdef __HIPCC__
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}
template <typename T> __device__ __forceinline__ float load_f32(const T* p);
template <> __device__ __forceinline__ float load_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void store_f32(T* p, float v);
template <> __device__ __forceinline__ void store_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_f32<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// Sum over the 64 lanes of a wavefront; every lane gets the total (fixed order: deterministic).
// Inside each row of 16 lanes the partners come through DPP lane permutations (swap neighbours, swap
// pairs, mirror halves of 8, mirror the row: after each step the lanes of the growing group agree), so
// nothing goes through LDS; the four row sums are then read out and added in order.
#define ECOSPA_DPP_ADD(v, ctrl) ((v) + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (v)), (ctrl), 0xF, 0xF, true)))
__device__ __forceinline__ float row16_sum(float v) {
  v = ECOSPA_DPP_ADD(v, 0xB1);    // quad_perm [1,0,3,2]
  v = ECOSPA_DPP_ADD(v, 0x4E);    // quad_perm [2,3,0,1]
  v = ECOSPA_DPP_ADD(v, 0x141);   // row_half_mirror
  v = ECOSPA_DPP_ADD(v, 0x140);   // row_mirror
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
#endif
