// Device-side epilogues shared by the contraction kernels (not part of the C ABI).
#pragma once
#include <type_traits>
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
    case EPI_DSWIGLU: {      // unit n: gate and up pre-activations in columns 2n and 2n + 1 of h, their gradients likewise in c
      const T* hp = static_cast<const T*>(e.h) + static_cast<long long>(m) * e.ldh + 2 * n;
      const float g = load_f32<T>(hp), u = load_f32<T>(hp + 1);
      const float sg = act_sigmoid(g);
      T* cp = c + static_cast<long long>(m) * e.ldc + 2 * n;
      store_f32<T>(cp, acc * u * sg * (1.f + g * (1.f - sg)));
      store_f32<T>(cp + 1, acc * g * sg);
    } break;
    default: break;          // EPI_ROPE, EPI_SWIGLU: bf16 only (vector epilogue)
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
// Rotary turn of the four adjacent pairs in v (columns n .. n+7 of row m), sign = +1 forward, -1 for gradients.
__device__ __forceinline__ void rope_turn8(const float4& c4, const float4& s4, float sign, float (&v)[8]) {
  const float cv[4] = {c4.x, c4.y, c4.z, c4.w}, sv[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float x0 = v[2 * i], x1 = v[2 * i + 1], s = sign * sv[i];
    v[2 * i] = x0 * cv[i] - x1 * s;
    v[2 * i + 1] = x0 * s + x1 * cv[i];
  }
}

// What an epilogue reads from global memory for one group of 8 columns besides the accumulators: the saved
// pre-activations (EPI_DACT: one 16-byte word, EPI_DSWIGLU: two) or the rotation table entries (EPI_ROPE: four
// cosines, four sines).  A kernel that loads them rows ahead of their use keeps their latency off the path of every
// row (on this target a wait for a load also waits for the stores issued before it).
// The epilogue kind is a template argument of the *_k functions, so that a kernel that branches on it once gets
// straight-line code per kind; the functions without the suffix branch per call.
struct EpiSide { uint4 a, b; };
__device__ __forceinline__ constexpr bool epi_has_side(int kind) { return kind == EPI_DACT || kind == EPI_DSWIGLU || kind == EPI_ROPE; }
template <int KIND>
__device__ __forceinline__ void epi_side_load_k(const GemmEpi& e, int m, int n, EpiSide& s) {
  if constexpr (KIND == EPI_ROPE) {
    if (n < e.rope_cols) {
      const int head = n / e.rope_kp, row = head < e.rope_hq ? head / e.rope_qpk : head - e.rope_hq;
      const long long tab = (static_cast<long long>(row) * e.rope_L + m % e.rope_L) * (e.rope_kp / 2) + (n % e.rope_kp) / 2;
      s.a = *reinterpret_cast<const uint4*>(e.rope_cos + tab);
      s.b = *reinterpret_cast<const uint4*>(e.rope_sin + tab);
    }
  } else if constexpr (KIND == EPI_DACT) {
    s.a = *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(e.h) + static_cast<long long>(m) * e.ldh + n);
  } else if constexpr (KIND == EPI_DSWIGLU) {
    const bf16_t* hp = static_cast<const bf16_t*>(e.h) + static_cast<long long>(m) * e.ldh + 2 * n;
    s.a = *reinterpret_cast<const uint4*>(hp);
    s.b = *reinterpret_cast<const uint4*>(hp + 8);
  }
}
// The bias of columns n .. n+7 for the epilogues that add one (the same for every row a lane handles).
__device__ __forceinline__ bool epi_bias_load(const GemmEpi& e, int n, float (&b)[8]) {
  if (!e.bias || e.kind == EPI_DACT || e.kind == EPI_DSWIGLU) return false;
  unpack8(*reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(e.bias) + n), b);
  return true;
}
// Columns n .. n+7 of row m with the bias and the side inputs already in registers.
template <int KIND>
__device__ __forceinline__ void epi_apply_vec8_k(const GemmEpi& e, int m, int n, float (&v)[8], bool has_bias, const float (&b)[8],
                                                 const EpiSide& sd) {
  bf16_t* c = static_cast<bf16_t*>(e.c) + static_cast<long long>(m) * e.ldc + n;
  if constexpr (KIND != EPI_DACT && KIND != EPI_DSWIGLU) {
    if (has_bias) {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += b[i];
    }
  }
  if constexpr (KIND == EPI_ROPE) {
    if (n < e.rope_cols) rope_turn8(__builtin_bit_cast(float4, sd.a), __builtin_bit_cast(float4, sd.b), 1.f, v);
    *reinterpret_cast<uint4*>(c) = pack8(v);
  } else if constexpr (KIND == EPI_STORE) {
    *reinterpret_cast<uint4*>(c) = pack8(v);
  } else if constexpr (KIND == EPI_BIAS_ACT) {
    *reinterpret_cast<uint4*>(c) = pack8(v);
    float a[8];
    if (e.act == ECOSPA_ACT_GELU_TANH) {
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = act_gelu(v[i], ECOSPA_ACT_GELU_TANH);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = act_gelu(v[i], ECOSPA_ACT_GELU_ERF);
    }
    *reinterpret_cast<uint4*>(static_cast<bf16_t*>(e.c2) + static_cast<long long>(m) * e.ldc2 + n) = pack8(a);
  } else if constexpr (KIND == EPI_ACT) {
    if (e.act == ECOSPA_ACT_GELU_TANH) {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = act_gelu(v[i], ECOSPA_ACT_GELU_TANH);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = act_gelu(v[i], ECOSPA_ACT_GELU_ERF);
    }
    *reinterpret_cast<uint4*>(c) = pack8(v);
  } else if constexpr (KIND == EPI_DACT) {
    float h[8];
    unpack8(sd.a, h);
    if (e.act == ECOSPA_ACT_GELU_TANH) {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] *= act_gelu_grad(h[i], ECOSPA_ACT_GELU_TANH);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] *= act_gelu_grad(h[i], ECOSPA_ACT_GELU_ERF);
    }
    *reinterpret_cast<uint4*>(c) = pack8(v);
  } else if constexpr (KIND == EPI_SWIGLU) {
    // columns n .. n+7 are four (gate, up) pairs: units n/2 .. n/2+3
    if (e.c) *reinterpret_cast<uint4*>(c) = pack8(v);
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    floatx4 a;
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = v[2 * i] * act_sigmoid(v[2 * i]) * v[2 * i + 1];
    *reinterpret_cast<bf16x4_t*>(static_cast<bf16_t*>(e.c2) + static_cast<long long>(m) * e.ldc2 + (n >> 1)) = __builtin_convertvector(a, bf16x4_t);
  } else {  // EPI_DSWIGLU: units n .. n+7, their (gate, up) pairs in columns 2n .. 2n+15 of h and of c
    static_assert(KIND == EPI_DSWIGLU, "epilogue kind");
    bf16_t* cp = static_cast<bf16_t*>(e.c) + static_cast<long long>(m) * e.ldc + 2 * n;
    float p[2][8], o[2][8];
    unpack8(sd.a, p[0]);
    unpack8(sd.b, p[1]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float g = p[i >> 2][2 * (i & 3)], u = p[i >> 2][2 * (i & 3) + 1];
      const float sg = act_sigmoid(g);
      o[i >> 2][2 * (i & 3)] = v[i] * u * sg * (1.f + g * (1.f - sg));
      o[i >> 2][2 * (i & 3) + 1] = v[i] * g * sg;
    }
    *reinterpret_cast<uint4*>(cp) = pack8(o[0]);
    *reinterpret_cast<uint4*>(cp + 8) = pack8(o[1]);
  }
}
// Calls f with the epilogue kind as a compile-time constant (std::integral_constant).
template <typename F>
__device__ __forceinline__ void epi_dispatch(int kind, F&& f) {
  switch (kind) {
    case EPI_STORE: f(std::integral_constant<int, EPI_STORE>{}); break;
    case EPI_BIAS_ACT: f(std::integral_constant<int, EPI_BIAS_ACT>{}); break;
    case EPI_ACT: f(std::integral_constant<int, EPI_ACT>{}); break;
    case EPI_DACT: f(std::integral_constant<int, EPI_DACT>{}); break;
    case EPI_DSWIGLU: f(std::integral_constant<int, EPI_DSWIGLU>{}); break;
    case EPI_ROPE: f(std::integral_constant<int, EPI_ROPE>{}); break;
    case EPI_SWIGLU: f(std::integral_constant<int, EPI_SWIGLU>{}); break;
    default: break;
  }
}
__device__ __forceinline__ void epi_apply_vec8(const GemmEpi& e, int m, int n, float (&v)[8]) {
  float b[8];
  const bool has_bias = epi_bias_load(e, n, b);
  epi_dispatch(e.kind, [&](auto k_) __attribute__((always_inline)) {
    constexpr int KIND = decltype(k_)::value;
    EpiSide sd;
    epi_side_load_k<KIND>(e, m, n, sd);
    epi_apply_vec8_k<KIND>(e, m, n, v, has_bias, b, sd);
  });
}
