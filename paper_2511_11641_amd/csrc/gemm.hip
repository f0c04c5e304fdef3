// Dense contractions of the reduced forward/backward pass.
//
// bf16: 128x128x64 workgroup tiles, 4 wavefronts of 64x64, v_mfma_f32_32x32x16_bf16, operands
//       staged through XOR-swizzled LDS with register double buffering; operands whose K index
//       is the slow storage axis (dY W, dY^T X) are transposed in registers on the way to LDS.
// fp32: 64x64x16 vector-ALU tiles (the fp32 configuration is small and launch bound).
// Split-K writes fp32 partials that a second kernel adds in a fixed order (deterministic dW).
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
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = static_cast<uint32_t>(f32_to_bf16(f[2 * i])) | (static_cast<uint32_t>(f32_to_bf16(f[2 * i + 1])) << 16);
  return make_uint4(w[0], w[1], w[2], w[3]);
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

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ---------------------------------------------------------------------------------------------
#define GB_M 128
#define GB_N 128
#define GB_K 64

// 16-byte chunk swizzle of a 64-element (128-byte) LDS row
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// K-contiguous operand: thread moves 4 chunks of 8 elements (row = c / 8, k-chunk = c % 8)
__device__ __forceinline__ void gload_kc(const bf16_t* __restrict__ base, long long ld, int row0, int R, int k0,
                                         int k_end, uint4 (&reg)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + i * 256;
    const int gr = row0 + (c >> 3), gk = k0 + (c & 7) * 8;
    reg[i] = (gr < R && gk < k_end) ? *reinterpret_cast<const uint4*>(base + static_cast<long long>(gr) * ld + gk)
                                    : make_uint4(0, 0, 0, 0);
  }
}
__device__ __forceinline__ void sstore_kc(bf16_t* lds, const uint4 (&reg)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + i * 256;
    const int row = c >> 3, kc = c & 7;
    *reinterpret_cast<uint4*>(lds + row * GB_K + ((kc ^ swz(row)) << 3)) = reg[i];
  }
}
// K-slow operand (storage [K][R]): thread owns a 4(k) x 8(r) block, transposed in registers
__device__ __forceinline__ void gload_tr(const bf16_t* __restrict__ base, long long ld, int row0, int R, int k0,
                                         int k_end, uint4 (&reg)[4]) {
  const int rblk = threadIdx.x & 15, kblk = threadIdx.x >> 4;
  const int gr = row0 + rblk * 8;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gk = k0 + kblk * 4 + i;
    reg[i] = (gr < R && gk < k_end) ? *reinterpret_cast<const uint4*>(base + static_cast<long long>(gk) * ld + gr)
                                    : make_uint4(0, 0, 0, 0);
  }
}
__device__ __forceinline__ uint32_t half16(const uint4& v, int j) {
  const uint32_t w = (j >> 1) == 0 ? v.x : (j >> 1) == 1 ? v.y : (j >> 1) == 2 ? v.z : v.w;
  return (j & 1) ? (w >> 16) : (w & 0xffffu);
}
__device__ __forceinline__ void sstore_tr(bf16_t* lds, const uint4 (&reg)[4]) {
  const int rblk = threadIdx.x & 15, kblk = threadIdx.x >> 4;
  const int kc = kblk >> 1, half = kblk & 1;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int r = rblk * 8 + j;
    uint2 v;
    v.x = half16(reg[0], j) | (half16(reg[1], j) << 16);
    v.y = half16(reg[2], j) | (half16(reg[3], j) << 16);
    *reinterpret_cast<uint2*>(lds + r * GB_K + ((kc ^ swz(r)) << 3) + half * 4) = v;
  }
}

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_bf16_mfma_kernel(const GemmDesc d, int tiles_n, int k_chunk) {
  __shared__ __attribute__((aligned(16))) bf16_t lds[2][2][GB_M * GB_K];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs, so give each XCD a
  // contiguous range of tiles (neighbouring tiles share operand rows in that XCD's L2).
  int id = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) id = (id & 7) * (nb >> 3) + (id >> 3);
  const int m0 = (id / tiles_n) * GB_M, n0 = (id % tiles_n) * GB_N;
  const int k_begin = blockIdx.z * k_chunk;
  const int k_end = min(d.K, k_begin + k_chunk);
  const int nk = (k_end - k_begin + GB_K - 1) / GB_K;

  const bf16_t* A = static_cast<const bf16_t*>(d.A);
  const bf16_t* B = static_cast<const bf16_t*>(d.B);
  uint4 ra[4], rb[4];
  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  auto gload = [&](int k0) {
    if (TA) gload_tr(A, d.lda, m0, d.M, k0, k_end, ra); else gload_kc(A, d.lda, m0, d.M, k0, k_end, ra);
    if (TB) gload_tr(B, d.ldb, n0, d.N, k0, k_end, rb); else gload_kc(B, d.ldb, n0, d.N, k0, k_end, rb);
  };
  auto sstore = [&](int buf) {
    if (TA) sstore_tr(lds[buf][0], ra); else sstore_kc(lds[buf][0], ra);
    if (TB) sstore_tr(lds[buf][1], rb); else sstore_kc(lds[buf][1], rb);
  };

  if (nk > 0) {
    gload(k_begin);
    sstore(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload(k_begin + (kt + 1) * GB_K);
    const bf16_t* As = lds[cur][0];
    const bf16_t* Bs = lds[cur][1];
#pragma unroll
    for (int s = 0; s < GB_K / 16; ++s) {
      bf16x8_t a[2], b[2];
      const int kc = s * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = wm * 64 + i * 32 + (lane & 31);
        a[i] = *reinterpret_cast<const bf16x8_t*>(As + row * GB_K + ((kc ^ swz(row)) << 3));
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row = wn * 64 + j * 32 + (lane & 31);
        b[j] = *reinterpret_cast<const bf16x8_t*>(Bs + row * GB_K + ((kc ^ swz(row)) << 3));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(cur ^ 1);
    __syncthreads();
  }

  // Epilogue through LDS: each wavefront parks its 64x64 fp32 tile in its own 16 KB quarter of
  // the (now idle) operand buffers, then every lane handles 8 consecutive columns of a row, so
  // global traffic is 16-byte vectors.  Accumulator layout of a 32x32 MFMA tile:
  // column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4.
  float* cs = reinterpret_cast<float*>(&lds[0][0][0]) + wave * (64 * 64);
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        cs[(i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * 64 + j * 32 + (lane & 31)] = acc[i][j][r];
  __syncthreads();
  const bool split = d.splits > 1;
  float* part = split ? d.partial + static_cast<long long>(blockIdx.z) * d.M * d.N : nullptr;
  const int n = n0 + wn * 64 + (lane & 7) * 8;
#pragma unroll 1
  for (int it = 0; it < 8; ++it) {
    const int row = it * 8 + (lane >> 3);
    const int m = m0 + wm * 64 + row;
    if (m >= d.M || n >= d.N) continue;
    float v[8];
    const float4 lo = *reinterpret_cast<const float4*>(cs + row * 64 + (lane & 7) * 8);
    const float4 hi = *reinterpret_cast<const float4*>(cs + row * 64 + (lane & 7) * 8 + 4);
    v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    if (split) {
      float* p = part + static_cast<long long>(m) * d.N + n;
      *reinterpret_cast<float4*>(p) = lo;
      *reinterpret_cast<float4*>(p + 4) = hi;
    } else {
      epi_apply_vec8(d.epi, m, n, v);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// fp32 (and generic fallback) vector-ALU kernel: 64x64 tile, 16x16 threads, 4x4 per thread
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gemm_valu_kernel(const GemmDesc d, int tiles_n, int k_chunk) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = (blockIdx.x / tiles_n) * 64, n0 = (blockIdx.x % tiles_n) * 64;
  const int k_begin = blockIdx.z * k_chunk;
  const int k_end = min(d.K, k_begin + k_chunk);
  const T* A = static_cast<const T*>(d.A);
  const T* B = static_cast<const T*>(d.B);
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = k_begin; k0 < k_end; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      {
        const int kk = d.trans_a ? e >> 6 : e & 15, r = d.trans_a ? e & 63 : e >> 4;
        const int gm = m0 + r, gk = k0 + kk;
        float v = 0.f;
        if (gm < d.M && gk < k_end)
          v = load_f32<T>(A + (d.trans_a ? static_cast<long long>(gk) * d.lda + gm : static_cast<long long>(gm) * d.lda + gk));
        As[kk][r] = v;
      }
      {
        const int kk = d.trans_b ? e >> 6 : e & 15, r = d.trans_b ? e & 63 : e >> 4;
        const int gn = n0 + r, gk = k0 + kk;
        float v = 0.f;
        if (gn < d.N && gk < k_end)
          v = load_f32<T>(B + (d.trans_b ? static_cast<long long>(gk) * d.ldb + gn : static_cast<long long>(gn) * d.ldb + gk));
        Bs[kk][r] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  const bool split = d.splits > 1;
  float* part = split ? d.partial + static_cast<long long>(blockIdx.z) * d.M * d.N : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= d.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= d.N) continue;
      if (split) part[static_cast<long long>(m) * d.N + n] = acc[i][j];
      else epi_apply<T>(d.epi, m, n, acc[i][j]);
    }
  }
}

// fixed-order sum of the K-split partials, then the epilogue
template <typename T>
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const GemmDesc d) {
  const long long tot = static_cast<long long>(d.M) * d.N;
  const long long e = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= tot) return;
  float s = 0.f;
  for (int z = 0; z < d.splits; ++z) s += d.partial[z * tot + e];
  epi_apply<T>(d.epi, static_cast<int>(e / d.N), static_cast<int>(e % d.N), s);
}

// ---------------------------------------------------------------------------------------------
int ecospa_gemm_splits(int M, int N, int K) {
  const long long tiles = static_cast<long long>((M + GB_M - 1) / GB_M) * ((N + GB_N - 1) / GB_N);
  int s = 1;
  // fill ~2 waves of the 256 CUs while every split keeps at least 512 of K
  while (tiles * s < 512 && K / (s * 2) >= 512 && s < 32) s *= 2;
  return s;
}

int ecospa_gemm(ecospa_ctx* ctx, const GemmDesc& d) {
  if (d.M < 1 || d.N < 1 || d.K < 1) return ECOSPA_ERR_SHAPE;
  if (!d.A || !d.B || !d.epi.c) return ECOSPA_ERR_NULL;
  if (d.splits > 1 && !d.partial) return ECOSPA_ERR_WORKSPACE;
  const int splits = d.splits > 1 ? d.splits : 1;
  if (d.dtype == ECOSPA_BF16) {
    // 16-byte vector loads along the contiguous axis of each operand
    const int ca = d.trans_a ? d.M : d.K, cb = d.trans_b ? d.N : d.K;
    if (ca % 8 || cb % 8 || d.lda % 8 || d.ldb % 8) return ECOSPA_ERR_ALIGN;
    if (!aligned16(d.A) || !aligned16(d.B)) return ECOSPA_ERR_ALIGN;
    // the epilogue moves 8 columns at a time
    if (d.N % 8 || d.epi.ldc % 8 || !aligned16(d.epi.c)) return ECOSPA_ERR_ALIGN;
    if (d.epi.bias && !aligned16(d.epi.bias)) return ECOSPA_ERR_ALIGN;
    if (d.epi.kind == EPI_BIAS_ACT && (!d.epi.c2 || d.epi.ldc2 % 8 || !aligned16(d.epi.c2))) return ECOSPA_ERR_ALIGN;
    if ((d.epi.kind == EPI_DACT || d.epi.kind == EPI_DSWIGLU) && (!d.epi.h || d.epi.ldh % 8 || !aligned16(d.epi.h)))
      return ECOSPA_ERR_ALIGN;
    if (d.epi.kind == EPI_DSWIGLU && d.epi.kp % 8) return ECOSPA_ERR_ALIGN;
    if (d.splits > 1 && !aligned16(d.partial)) return ECOSPA_ERR_ALIGN;
    const int tm = (d.M + GB_M - 1) / GB_M, tn = (d.N + GB_N - 1) / GB_N;
    int k_chunk = (d.K + splits - 1) / splits;
    k_chunk = (k_chunk + GB_K - 1) / GB_K * GB_K;
    dim3 grid(tm * tn, 1, splits);
    const bool prof = ctx->prof_on && ctx->prof_n < ctx->prof_cap;
    if (prof) (void)hipEventRecord(ctx->prof_ev[2 * ctx->prof_n], ctx->stream);
    if (!d.trans_a && !d.trans_b)
      hipLaunchKernelGGL((gemm_bf16_mfma_kernel<false, false>), grid, dim3(256), 0, ctx->stream, d, tn, k_chunk);
    else if (!d.trans_a && d.trans_b)
      hipLaunchKernelGGL((gemm_bf16_mfma_kernel<false, true>), grid, dim3(256), 0, ctx->stream, d, tn, k_chunk);
    else if (d.trans_a && d.trans_b)
      hipLaunchKernelGGL((gemm_bf16_mfma_kernel<true, true>), grid, dim3(256), 0, ctx->stream, d, tn, k_chunk);
    else
      hipLaunchKernelGGL((gemm_bf16_mfma_kernel<true, false>), grid, dim3(256), 0, ctx->stream, d, tn, k_chunk);
    if (prof) {
      (void)hipEventRecord(ctx->prof_ev[2 * ctx->prof_n + 1], ctx->stream);
      ctx->prof_flop[ctx->prof_n++] = 2.0 * d.M * d.N * d.K;
    }
    ECOSPA_CHECK_LAUNCH(ctx, "gemm_bf16_mfma_kernel");
  } else if (d.dtype == ECOSPA_F32) {
    const int tm = (d.M + 63) / 64, tn = (d.N + 63) / 64;
    int k_chunk = (d.K + splits - 1) / splits;
    k_chunk = (k_chunk + 15) / 16 * 16;
    hipLaunchKernelGGL((gemm_valu_kernel<float>), dim3(tm * tn, 1, splits), dim3(256), 0, ctx->stream, d, tn, k_chunk);
    ECOSPA_CHECK_LAUNCH(ctx, "gemm_valu_kernel");
  } else {
    return ECOSPA_ERR_DTYPE;
  }
  if (splits > 1) {
    const long long tot = static_cast<long long>(d.M) * d.N;
    const unsigned grid = static_cast<unsigned>((tot + 255) / 256);
    if (d.dtype == ECOSPA_BF16)
      hipLaunchKernelGGL((gemm_splitk_reduce_kernel<bf16_t>), dim3(grid), dim3(256), 0, ctx->stream, d);
    else
      hipLaunchKernelGGL((gemm_splitk_reduce_kernel<float>), dim3(grid), dim3(256), 0, ctx->stream, d);
    ECOSPA_CHECK_LAUNCH(ctx, "gemm_splitk_reduce_kernel");
  }
  return ECOSPA_OK;
}

// ---------------------------------------------------------------------------------------------
// column sums (bias gradients): 16-lane x 16-row-slot tiles, then a fixed-order second stage
// ---------------------------------------------------------------------------------------------
#define CS_ROWS 256   // rows per first-stage block

int ecospa_colsum_chunks(int M) { return (M + CS_ROWS - 1) / CS_ROWS; }

template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ X, long long ldx, int M, int N,
                                                             float* __restrict__ partial) {
  __shared__ float lds[16][64 + 1];
  const int slot = threadIdx.x >> 6, lane = threadIdx.x & 63;   // 4 row slots x 64 columns
  const int col = blockIdx.x * 64 + lane;
  const int r0 = blockIdx.y * CS_ROWS, r1 = min(M, r0 + CS_ROWS);
  float acc = 0.f;
  if (col < N)
    for (int r = r0 + slot; r < r1; r += 4) acc += load_f32<T>(X + static_cast<long long>(r) * ldx + col);
  lds[slot][lane] = acc;
  __syncthreads();
  if (threadIdx.x < 64 && col < N)
    partial[static_cast<long long>(blockIdx.y) * N + col] = (lds[0][lane] + lds[1][lane]) + (lds[2][lane] + lds[3][lane]);
}

template <typename T>
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ partial, int chunks, int N,
                                                           T* __restrict__ out) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= N) return;
  float s = 0.f;
  for (int c = 0; c < chunks; ++c) s += partial[static_cast<long long>(c) * N + col];
  store_f32<T>(out + col, s);
}

int ecospa_colsum(ecospa_ctx* ctx, int dtype, const void* X, long long ldx, int M, int N, float* partial, void* out) {
  if (!X || !partial || !out) return ECOSPA_ERR_NULL;
  const int chunks = ecospa_colsum_chunks(M);
  dim3 g1((N + 63) / 64, chunks), g2((N + 255) / 256);
  if (dtype == ECOSPA_BF16) {
    hipLaunchKernelGGL((colsum_partial_kernel<bf16_t>), g1, dim3(256), 0, ctx->stream, static_cast<const bf16_t*>(X), ldx,
                       M, N, partial);
    hipLaunchKernelGGL((colsum_final_kernel<bf16_t>), g2, dim3(256), 0, ctx->stream, partial, chunks, N,
                       static_cast<bf16_t*>(out));
  } else {
    hipLaunchKernelGGL((colsum_partial_kernel<float>), g1, dim3(256), 0, ctx->stream, static_cast<const float*>(X), ldx, M,
                       N, partial);
    hipLaunchKernelGGL((colsum_final_kernel<float>), g2, dim3(256), 0, ctx->stream, partial, chunks, N,
                       static_cast<float*>(out));
  }
  ECOSPA_CHECK_LAUNCH(ctx, "colsum kernels");
  return ECOSPA_OK;
}
