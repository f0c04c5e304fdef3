// Device-side epilogues shared by the contraction kernels (not part of the C ABI).
#pragma once
#include "gemm.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------------------
// epilogue
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void epi_apply(const GemmEpi& e, int m, int n, float acc) {
  T* c = static_cast<T*>(e.c);
  const long long off = static_cast<long long>(m) * e.ldc + n;
  switch (e.kind) {
    case EPI_STORE: {
      if (e.bias) acc += load_f32<T>(static_cast<const T*>(e.bias) + n);
      store_f32<T>(c + off, acc);
    } break;
    case EPI_BIAS_ACT: {
      if (e.bias) acc += load_f32<T>(static_cast<const T*>(e.bias) + n);
      store_f32<T>(c + off, acc);
      store_f32<T>(static_cast<T*>(e.c2) + static_cast<long long>(m) * e.ldc2 + n, act_gelu(acc, e.act));
    } break;
    case EPI_ACT: {
      if (e.bias) acc += load_f32<T>(static_cast<const T*>(e.bias) + n);
      store_f32<T>(c + off, act_gelu(acc, e.act));
    } break;
    case EPI_DACT: {
      const float h = load_f32<T>(static_cast<const T*>(e.h) + static_cast<long long>(m) * e.ldh + n);
      store_f32<T>(c + off, acc * act_gelu_grad(h, e.act));
    } break;
    case EPI_DSWIGLU: {
      const T* hp = static_cast<const T*>(e.h) + static_cast<long long>(m) * e.ldh + n;
      const float g = load_f32<T>(hp), u = load_f32<T>(hp + e.kp);
      const float sg = act_sigmoid(g);
      store_f32<T>(c + off, acc * u * sg * (1.f + g * (1.f - sg)));
      store_f32<T>(c + off + e.kp, acc * g * sg);
    } break;
  }
}

// 8 consecutive columns of one row, bf16 storage, 16-byte aligned (N, ld* multiples of 8)
__device__ __forceinline__ void unpack8(const uint4& u, float (&f)[8]) {
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  typedef float floatx8 __attribute__((ext_vector_type(8)));
  floatx8 v;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = f[i];
  const bf16x8_t b = __builtin_convertvector(v, bf16x8_t);   // round to nearest even (v_cvt_pk_bf16_f32)
  return __builtin_bit_cast(uint4, b);
}
__device__ __forceinline__ void epi_apply_vec8(const GemmEpi& e, int m, int n, float (&v)[8]) {
  bf16_t* c = static_cast<bf16_t*>(e.c) + static_cast<long long>(m) * e.ldc + n;
  if (e.kind == EPI_STORE || e.kind == EPI_BIAS_ACT) {
    if (e.bias) {
      float b[8];
      unpack8(*reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(e.bias) + n), b);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += b[i];
    }
    *reinterpret_cast<uint4*>(c) = pack8(v);
    if (e.kind == EPI_BIAS_ACT) {
      float a[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = act_gelu(v[i], e.act);
      *reinterpret_cast<uint4*>(static_cast<bf16_t*>(e.c2) + static_cast<long long>(m) * e.ldc2 + n) = pack8(a);
    }
  } else if (e.kind == EPI_ACT) {
    if (e.bias) {
      float b[8];
      unpack8(*reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(e.bias) + n), b);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += b[i];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = act_gelu(v[i], e.act);
    *reinterpret_cast<uint4*>(c) = pack8(v);
  } else if (e.kind == EPI_DACT) {
    float h[8];
    unpack8(*reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(e.h) + static_cast<long long>(m) * e.ldh + n), h);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= act_gelu_grad(h[i], e.act);
    *reinterpret_cast<uint4*>(c) = pack8(v);
  } else {  // EPI_DSWIGLU
    const bf16_t* hp = static_cast<const bf16_t*>(e.h) + static_cast<long long>(m) * e.ldh + n;
    float g[8], u[8], dg[8], du[8];
    unpack8(*reinterpret_cast<const uint4*>(hp), g);
    unpack8(*reinterpret_cast<const uint4*>(hp + e.kp), u);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float sg = act_sigmoid(g[i]);
      dg[i] = v[i] * u[i] * sg * (1.f + g[i] * (1.f - sg));
      du[i] = v[i] * g[i] * sg;
    }
    *reinterpret_cast<uint4*>(c) = pack8(dg);
    *reinterpret_cast<uint4*>(c + e.kp) = pack8(du);
  }
}

