// bf16 contraction with a register-staged, two-slab-deep prefetch: 256x256x64 workgroup tiles, four
// wavefronts of 128x128 (one per SIMD, accumulators in the AGPR half of the register file).
//
// Operand slabs travel global -> VGPR -> LDS.  The loads of slab t+2 are issued while slab t is
// multiplied and sit in registers for a whole slab before they are written to the LDS buffer that
// slab t-1 has just freed, so a load has more than one slab time (about 1.3 us) to come back from
// L2 or HBM - with two 64 KB LDS buffers a direct global->LDS load can only be issued one slab
// ahead.  Four wavefronts of 128x128 read (128+128) x 64 operand elements from LDS per slab each,
// a third less than eight wavefronts of 128x64.
//
// Per slab and wavefront: 64 MFMAs in four 16-wide k steps.  Behind each MFMA goes one small piece of
// the other work, in a fixed order (sched_barrier keeps the compiler from regrouping it):
//   k step 0: the 16 global loads of slab t+2, fragment reads of k step 1
//   k step 1: LDS writes of the A part of slab t+1, fragment reads of k step 2
//   k step 2: LDS writes of the B part of slab t+1, fragment reads of k step 3
//   k step 3: barrier (slab t+1 complete in LDS, slab t no longer read), fragment reads of slab t+1
// K-contiguous operands sit in LDS as [rows][64] (ds_read_b128), K-slow ones as [64][rows]
// (transposing reads), with the swizzles of gemm_lds.h applied by the LDS writes.
#include "gemm_lds.h"

#include <type_traits>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int I, int N, typename F>
__device__ __forceinline__ void rs_static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    rs_static_for<I + 1, N>(f);
  }
}

// The eight 16-byte pieces of one operand slab that a thread moves: where they come from and where
// they go in the LDS tile.
template <int ROWS, bool KSLOW>
struct RsOperand {
  const bf16_t* src[8];
  long long step;     // elements per slab
  int dst[2];         // LDS element offset of piece 0 and piece 1; piece i sits at dst[i & 1] + (i / 2) * 1024
  __device__ __forceinline__ void init(const bf16_t* base, long long ld, int r0, int R, int k0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (!KSLOW) {
      // piece i: tile rows (wave * 8 + i) * 8 + lane / 8, 16-byte chunk lane % 8 of the 64-wide slab row
      const int rl = lane >> 3, kc = lane & 7;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = (wave * 8 + i) * 8 + rl;
        src[i] = base + static_cast<long long>(min(r0 + row, R - 1)) * ld + k0 + kc * 8;
      }
      dst[0] = kc_off<64>(wave * 64 + rl, kc);
      dst[1] = kc_off<64>(wave * 64 + 8 + rl, kc);
      step = 64;
    } else {
      // piece i: slab rows k = (wave * 8 + i) * 2 + lane / 32, 16-byte chunk lane % 32 of the ROWS-wide row
      static_assert(ROWS == 256, "one K-slow slab row = 32 chunks");
      const int kl = lane >> 5, c = lane & 31;
      const int col = min(r0 + c * 8, R - 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) src[i] = base + static_cast<long long>(k0 + (wave * 8 + i) * 2 + kl) * ld + col;
      dst[0] = ks_off<ROWS>(wave * 16 + kl, c);
      dst[1] = ks_off<ROWS>(wave * 16 + 2 + kl, c);
      step = 64 * ld;
    }
  }
  __device__ __forceinline__ u32x4 load(int i, long long adv) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(src[i]);
    src[i] += adv;
    return v;
  }
  __device__ __forceinline__ void store(bf16_t* tile, int i, const u32x4& v) const {
    // pieces i and i + 2 are 16 tile rows (K-contiguous: 16 * 64 elements) or 4 slab rows (K-slow:
    // 4 * 256 elements) apart: 1024 elements either way, and the swizzle repeats with that period
    *reinterpret_cast<u32x4*>(tile + dst[i & 1] + (i >> 1) * 1024) = v;
  }
};

template <bool TA, bool TB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_bf16_rs_kernel(const GemmDesc d, int tiles_n, int k_chunk) {
  constexpr int BM = 256, BN = 256, BK = 64, WGN = 2;
  constexpr int WTM = 128, WTN = 128, FM = 4, FN = 4, KS = 4, NM = FM * FN;
  constexpr int STAGE = (BM + BN) * BK;
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // tile order: a contiguous id range per XCD, bands of four tile rows walked column by column
  int id, zsplit;
  const int nsplit = d.splits > 1 ? d.splits : 1;
  gemm_work_item(nsplit, id, zsplit);
  constexpr int GROUP_M = 4;
  const int tiles_m = static_cast<int>(gridDim.x) / nsplit / tiles_n;
  const int band = id / (GROUP_M * tiles_n), in_band = id - band * (GROUP_M * tiles_n);
  const int band_rows = min(GROUP_M, tiles_m - band * GROUP_M);
  const int m0 = (band * GROUP_M + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BN;
  const int k_begin = zsplit * k_chunk;
  const int k_end = min(d.K, k_begin + k_chunk);
  const int nk = (k_end - k_begin) / BK;               // full slabs only (checked on the host)

  RsOperand<BM, TA> oa;
  RsOperand<BN, TB> ob;
  oa.init(static_cast<const bf16_t*>(d.A), d.lda, m0, d.M, k_begin);
  ob.init(static_cast<const bf16_t*>(d.B), d.ldb, n0, d.N, k_begin);

  // Column sums of a K-slow A (dY^T X: the bias gradient is the column sum of dY): the first tile column adds up
  // the pieces it moves anyway.  A thread's pieces all cover the same 8 columns, m0 + (lane % 32) * 8 ...
  constexpr bool CS = TA && TB;
  const bool do_cs = CS && d.colsum && n0 == 0;
  float cs_acc[CS ? 8 : 1];
  if constexpr (CS) {
#pragma unroll
    for (int j = 0; j < 8; ++j) cs_acc[j] = 0.f;
  }
  auto cs_add = [&](const u32x4& v) {
    if constexpr (CS) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        cs_acc[2 * q] += __uint_as_float(v[q] << 16);
        cs_acc[2 * q + 1] += __uint_as_float(v[q] & 0xffff0000u);
      }
    }
  };

  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // prologue: slabs 0 and 1 into registers (a slab beyond the last repeats it), slab 0 on into LDS
  u32x4 ra[2][8], rb[2][8];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const bool adv = p + 1 < nk;
#pragma unroll
    for (int i = 0; i < 8; ++i) ra[p][i] = oa.load(i, adv ? oa.step : 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) rb[p][i] = ob.load(i, adv ? ob.step : 0);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) oa.store(lds, i, ra[0][i]);
  if (do_cs) {
#pragma unroll
    for (int i = 0; i < 8; ++i) cs_add(ra[0][i]);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) ob.store(lds + BM * BK, i, rb[0][i]);
  __syncthreads();
  bf16x8_t fa[2][FM], fb[2][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) fa[0][i] = read_frag<BM, BK, TA>(lds, wm * WTM + i * 32, 0);
#pragma unroll
  for (int j = 0; j < FN; ++j) fb[0][j] = read_frag<BN, BK, TB>(lds + BM * BK, wn * WTN + j * 32, 0);

  // One slab.  P = t % 2: LDS buffer of slab t, register set that receives slab t+2; the other register
  // set holds slab t+1 and goes to the other LDS buffer.
  auto slab = [&](auto p_, int t) {
    constexpr int P = decltype(p_)::value, Q = P ^ 1;
    const bf16_t* as_cur = lds + P * STAGE;
    const bf16_t* bs_cur = as_cur + BM * BK;
    bf16_t* as_nxt = lds + Q * STAGE;
    bf16_t* bs_nxt = as_nxt + BM * BK;
    const bool adv = t + 3 < nk;                       // the slab after the one loaded now exists
    const long long adv_a = adv ? oa.step : 0, adv_b = adv ? ob.step : 0;
    const bool cs_now = do_cs && t + 1 < nk;           // the slab written to LDS here is a real one, not the repeat past the end
    rs_static_for<0, KS>([&](auto s_) {
      constexpr int s = decltype(s_)::value;
      constexpr int cur = s & 1, nxt = cur ^ 1;
      constexpr bool last = s + 1 == KS;
      if constexpr (last) {
        // slab t+1 is complete in LDS (everyone's writes) and slab t is read no more from here on; only
        // the LDS counter is waited for - the global loads of slab t+2 stay in flight
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, true));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
      }
      const bf16_t* fa_src = last ? as_nxt : as_cur;
      const bf16_t* fb_src = last ? bs_nxt : bs_cur;
      constexpr int sn = last ? 0 : s + 1;
      rs_static_for<0, NM>([&](auto m_) {
        constexpr int m = decltype(m_)::value;
        constexpr int i = m / FN, j = m % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (m < FM) fa[nxt][m] = read_frag<BM, BK, TA>(fa_src, wm * WTM + m * 32, sn);
        else if constexpr (m < FM + FN) fb[nxt][m - FM] = read_frag<BN, BK, TB>(fb_src, wn * WTN + (m - FM) * 32, sn);
        if constexpr (s == 0) {
          if constexpr (m < 8) ra[P][m] = oa.load(m, adv_a);
          else rb[P][m - 8] = ob.load(m - 8, adv_b);
        } else if constexpr (s == 1 && (m & 1)) {
          oa.store(as_nxt, m >> 1, ra[Q][m >> 1]);
          if (cs_now) cs_add(ra[Q][m >> 1]);
        } else if constexpr (s == 2 && (m & 1)) {
          ob.store(bs_nxt, m >> 1, rb[Q][m >> 1]);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    });
  };
  int t = 0;
  for (; t + 1 < nk; t += 2) {
    slab(std::integral_constant<int, 0>{}, t);
    slab(std::integral_constant<int, 1>{}, t + 1);
  }
  if (t < nk) slab(std::integral_constant<int, 0>{}, t);
  __syncthreads();   // operand buffers are idle from here on

  if constexpr (CS) {
    if (do_cs) {     // the same for the whole workgroup
      // eight partial sums per column (two slab-row halves in each of the four wavefronts), added in a fixed order
      float* red = reinterpret_cast<float*>(lds);
      const int part_id = wave * 2 + (lane >> 5), c = lane & 31;
      const bool own = m0 + c * 8 + 8 <= d.M;      // beyond the ragged edge the loads were clamped onto another thread's columns
#pragma unroll
      for (int j = 0; j < 8; ++j) red[part_id * BM + c * 8 + j] = own ? cs_acc[j] : 0.f;
      __syncthreads();
      const int r = threadIdx.x;
      if (m0 + r < d.M) {
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) sum += red[q * BM + r];
        d.colsum[static_cast<long long>(zsplit) * d.M + m0 + r] = sum;
      }
      __syncthreads();
    }
  }

  // Epilogue through LDS: each wavefront parks 32 rows x 128 columns of fp32 at a time in its own
  // slice of the operand buffers, then every lane handles 8 consecutive columns of a row (16-byte
  // global accesses).  Accumulator layout of a 32x32 tile: column = lane % 32,
  // row = 8 * (r / 4) + 4 * (lane / 32) + r % 4.
  float* cs = reinterpret_cast<float*>(lds) + wave * (32 * WTN);
  const bool split = d.splits > 1;
  float* part = split ? d.partial + static_cast<long long>(zsplit) * d.M * d.N : nullptr;
  constexpr int LPR = WTN / 8;          // lanes per row
  constexpr int RPI = 64 / LPR;         // rows per pass
  const int n = n0 + wn * WTN + (lane % LPR) * 8;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        cs[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * WTN + j * 32 + (lane & 31)] = acc[i][j][r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll 1
    for (int it = 0; it < 32 / RPI; ++it) {
      const int row = it * RPI + lane / LPR;
      const int m = m0 + wm * WTM + i * 32 + row;
      if (m >= d.M || n >= d.N) continue;
      float v[8];
      const float4 lo = *reinterpret_cast<const float4*>(cs + row * WTN + (lane % LPR) * 8);
      const float4 hi = *reinterpret_cast<const float4*>(cs + row * WTN + (lane % LPR) * 8 + 4);
      v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
      if (split) {
        float* p = part + static_cast<long long>(m) * d.N + n;
        *reinterpret_cast<float4*>(p) = lo;
        *reinterpret_cast<float4*>(p + 4) = hi;
      } else {
        epi_apply_vec8(d.epi, m, n, v);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// instantiated explicitly (see gemm_pipe.hip)
template __global__ void gemm_bf16_rs_kernel<false, false>(const GemmDesc, int, int);
template __global__ void gemm_bf16_rs_kernel<false, true>(const GemmDesc, int, int);
template __global__ void gemm_bf16_rs_kernel<true, true>(const GemmDesc, int, int);

// ---------------------------------------------------------------------------------------------
bool gemm_rs_ok(const GemmDesc& d, int k_chunk) {
  if (d.trans_a && !d.trans_b) return false;            // combination not used by the layers
  if (d.K % 64 || k_chunk % 64) return false;           // full slabs only
  return d.M >= 8 && d.N >= 8;
}

hipError_t gemm_rs_launch(ecospa_ctx* ctx, const GemmDesc& d, int k_chunk) {
  const int tm = (d.M + 255) / 256, tn = (d.N + 255) / 256;
  const int splits = d.splits > 1 ? d.splits : 1;
  const dim3 grid(tm * tn * splits), block(256);
  const int lds_bytes = 2 * (256 + 256) * 64 * static_cast<int>(sizeof(bf16_t));   // also covers the epilogue staging
#define RS_LAUNCH(TA, TB)                                                                                      \
  do {                                                                                                         \
    auto kern = gemm_bf16_rs_kernel<TA, TB>;                                                                   \
    static LdsAttrOnce attr_once;                                                                              \
    {                                                                                                          \
      hipError_t e = attr_once.ensure(reinterpret_cast<const void*>(kern), lds_bytes);                         \
      if (e != hipSuccess) return e;                                                                           \
    }                                                                                                          \
    hipLaunchKernelGGL(kern, grid, block, lds_bytes, ctx->stream, d, tn, k_chunk);                             \
  } while (0)
  if (d.trans_a) RS_LAUNCH(true, true);
  else if (d.trans_b) RS_LAUNCH(false, true);
  else RS_LAUNCH(false, false);
#undef RS_LAUNCH
  return hipGetLastError();
}
