// bf16 contraction with a register-staged, two-slab-deep prefetch: BM x BN x 64 workgroup tiles (BM, BN from
// 128, 192, 256), four wavefronts of (BM/2) x (BN/2) (one per SIMD, accumulators in the AGPR half of the
// register file).
//
// Operand slabs travel global -> VGPR -> LDS.  The loads of slab t+2 are issued while slab t is
// multiplied and sit in registers for a whole slab before they are written to the LDS buffer that
// slab t-1 has just freed, so a load has more than one slab time (about 1.3 us) to come back from
// L2 or HBM - with two LDS buffers a direct global->LDS load can only be issued one slab
// ahead.  Four wavefronts of 128x128 read (128+128) x 64 operand elements from LDS per slab each,
// a third less than eight wavefronts of 128x64.
//
// The narrower tiles exist for the weight-gradient contractions dY^T X: few output tiles and a long K, so the
// tile shape and the number of K splits are chosen to fill the 256 compute units (gemm_tt_plan in gemm.hip).
//
// Per slab and wavefront: FM*FN MFMAs in each of four 16-wide k steps.  Behind each MFMA goes a share of
// the other work, in a fixed order (sched_barrier keeps the compiler from regrouping it):
//   k step 0: the global loads of slab t+2, fragment reads of k step 1
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

// The ROWS / 32 16-byte pieces of one operand slab that a thread moves: where they come from and where
// they go in the LDS tile.  Piece i of a thread is number (wave * PER + i) * 64 + lane of the slab's pieces.
template <int ROWS, bool KSLOW>
struct RsOperand {
  static constexpr int PER = ROWS / 32;
  // LDS offsets repeat with a period of NDST pieces (the swizzles repeat every 16 tile rows / 4 slab rows):
  // piece i sits at dst[i % NDST] + (i / NDST) * STRIDE
  static constexpr int NDST = !KSLOW ? 2 : (ROWS == 256 ? 2 : (ROWS == 128 ? 1 : 3));
  static constexpr int STRIDE = NDST * 512;
  static_assert(ROWS == 128 || ROWS == 192 || ROWS == 256, "tile extents that are built");
  static_assert(PER % NDST == 0, "whole periods");
  // Addresses: a wavefront-uniform base (the current slab; scalar registers, advanced by scalar adds) plus a per-lane
  // byte offset that never changes - a wavefront that is alone on its SIMD pays MFMA time for every vector instruction.
  const char* base;
  unsigned off[PER];
  long long step;     // bytes per slab
  int dst[NDST];
  __device__ __forceinline__ void init(const bf16_t* mat, long long ld, int r0, int R, int k0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if constexpr (!KSLOW) {
      // piece i: tile rows (wave * PER + i) * 8 + lane / 8, 16-byte chunk lane % 8 of the 64-wide slab row
      const int rl = lane >> 3, kc = lane & 7;
      base = reinterpret_cast<const char*>(mat + static_cast<long long>(r0) * ld + k0);
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int row = (wave * PER + i) * 8 + rl;
        off[i] = static_cast<unsigned>((static_cast<long long>(min(r0 + row, R - 1) - r0) * ld + kc * 8) * 2);
      }
      dst[0] = kc_off<64>(wave * PER * 8 + rl, kc);
      dst[1] = kc_off<64>(wave * PER * 8 + 8 + rl, kc);
      step = 64 * 2;
    } else {
      // piece i: slab row k = p / (ROWS / 8), chunk c = p % (ROWS / 8) of the ROWS-wide row, p its number
      constexpr int CPR = ROWS / 8;
      base = reinterpret_cast<const char*>(mat + static_cast<long long>(k0) * ld + r0);
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int p = (wave * PER + i) * 64 + lane;
        const int k = p / CPR, c = p - k * CPR;
        const int col = min(r0 + c * 8, R - 8) - r0;
        off[i] = static_cast<unsigned>((static_cast<long long>(k) * ld + col) * 2);
        if (i < NDST) dst[i] = ks_off<ROWS>(k, c);
      }
      step = 64 * ld * 2;
    }
  }
  // piece i of the current slab; the last piece of a slab moves the base on by `adv` (the step, or 0 past the end)
  __device__ __forceinline__ u32x4 load(int i, long long adv) {
    asm volatile("" : "+v"(off[i]));   // keeps the offset a 32-bit register at the load: address = scalar base + lane offset
    const u32x4 v = *reinterpret_cast<const u32x4*>(base + off[i]);
    if (i == PER - 1) base += adv;
    return v;
  }
  __device__ __forceinline__ void store(bf16_t* tile, int i, const u32x4& v) const {
    *reinterpret_cast<u32x4*>(tile + dst[i % NDST] + (i / NDST) * STRIDE) = v;
  }
};

template <int BM, int BN, bool TA, bool TB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_bf16_rs_kernel(const GemmDesc d, int tiles_n, int k_chunk) {
  constexpr int BK = 64, WGN = 2;
  constexpr int WTM = BM / 2, WTN = BN / 2, FM = WTM / 32, FN = WTN / 32, KS = 4, NM = FM * FN;
  constexpr int STAGE = (BM + BN) * BK;
  constexpr int PA = BM / 32, PB = BN / 32;            // 16-byte pieces per thread and slab
  static_assert(FM + FN <= NM, "a fragment slot per MFMA");
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

  // Column sums of a K-slow A (dY^T X: the bias gradient is the column sum of dY), added up from the pieces a thread
  // moves anyway.  A wavefront that is alone on its SIMD pays for every vector instruction, so the work is shared out:
  // the workgroup of tile column j takes the slabs whose number is j modulo the tile columns, and writes row
  // (split * tile columns + j) of the partial sums.  Piece i of a thread covers the same 8 columns as piece i + NDST.
  constexpr bool CS = TA && TB;
  constexpr int NCS = CS ? RsOperand<BM, TA>::NDST : 1;
  const bool do_cs = CS && d.colsum;
  const int tile_col = in_band / band_rows;
  int cs_next = tile_col;                              // next slab of this split whose pieces are added
  float cs_acc[NCS][CS ? 8 : 1];
  if constexpr (CS) {
#pragma unroll
    for (int q = 0; q < NCS; ++q)
#pragma unroll
      for (int j = 0; j < 8; ++j) cs_acc[q][j] = 0.f;
  }
  auto cs_add = [&](auto i_, const u32x4& v) {
    if constexpr (CS) {
      constexpr int q0 = decltype(i_)::value % NCS;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        cs_acc[q0][2 * q] += __uint_as_float(v[q] << 16);
        cs_acc[q0][2 * q + 1] += __uint_as_float(v[q] & 0xffff0000u);
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
  u32x4 ra[2][PA], rb[2][PB];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const bool adv = p + 1 < nk;
#pragma unroll
    for (int i = 0; i < PA; ++i) ra[p][i] = oa.load(i, adv ? oa.step : 0);
#pragma unroll
    for (int i = 0; i < PB; ++i) rb[p][i] = ob.load(i, adv ? ob.step : 0);
  }
#pragma unroll
  for (int i = 0; i < PA; ++i) oa.store(lds, i, ra[0][i]);
  if (do_cs && cs_next == 0) {
    rs_static_for<0, PA>([&](auto i_) { cs_add(i_, ra[0][decltype(i_)::value]); });
    cs_next += tiles_n;
  }
#pragma unroll
  for (int i = 0; i < PB; ++i) ob.store(lds + BM * BK, i, rb[0][i]);
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
    const bool cs_now = do_cs && t + 1 < nk && t + 1 == cs_next;   // slab t+1 (a real one, not the repeat past the end) is this workgroup's
    if (cs_now) cs_next += tiles_n;
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
      // the other work of this k step, dealt evenly over the MFMA slots
      constexpr int NOPS = s == 0 ? PA + PB : (s == 1 ? PA : (s == 2 ? PB : 0));
      rs_static_for<0, NM>([&](auto m_) {
        constexpr int m = decltype(m_)::value;
        constexpr int i = m / FN, j = m % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (m < FM) fa[nxt][m] = read_frag<BM, BK, TA>(fa_src, wm * WTM + m * 32, sn);
        else if constexpr (m < FM + FN) fb[nxt][m - FM] = read_frag<BN, BK, TB>(fb_src, wn * WTN + (m - FM) * 32, sn);
        constexpr int O0 = m * NOPS / NM, O1 = (m + 1) * NOPS / NM;
        rs_static_for<O0, O1>([&](auto o_) {
          constexpr int o = decltype(o_)::value;
          if constexpr (s == 0) {
            if constexpr (o < PA) ra[P][o] = oa.load(o, adv_a);
            else rb[P][o - PA] = ob.load(o - PA, adv_b);
          } else if constexpr (s == 1) {
            oa.store(as_nxt, o, ra[Q][o]);
            if (cs_now) cs_add(o_, ra[Q][o]);
          } else if constexpr (s == 2) {
            ob.store(bs_nxt, o, rb[Q][o]);
          }
        });
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
      // Every thread parks its partial sums; column r then adds those of the threads that moved its 8-column chunk, in
      // a fixed order.  Piece q of thread (wave, lane) covers chunk (q * 64 + lane) % CPR (a wave's pieces start at a
      // multiple of CPR), so the threads of chunk c are the lanes congruent to c - 64 q modulo CPR of every wavefront.
      constexpr int CPR = BM / 8;
      float* red = reinterpret_cast<float*>(lds);                          // [256][NCS][8]
#pragma unroll
      for (int q = 0; q < NCS; ++q)
#pragma unroll
        for (int j = 0; j < 8; ++j) red[(threadIdx.x * NCS + q) * 8 + j] = cs_acc[q][j];
      __syncthreads();
      const int r = threadIdx.x;
      if (r < BM && m0 + r < d.M) {
        float sum = 0.f;
        const int c = r >> 3, j = r & 7;
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int q = 0; q < NCS; ++q) {
            const int l0 = ((c - q * 64) % CPR + CPR) % CPR;
            for (int l = l0; l < 64; l += CPR) sum += red[((w * 64 + l) * NCS + q) * 8 + j];
          }
        d.colsum[(static_cast<long long>(zsplit) * tiles_n + tile_col) * d.M + m0 + r] = sum;
      }
      __syncthreads();
    }
  }

  // Epilogue through LDS: each wavefront parks 32 rows x WTN columns of fp32 at a time in its own
  // slice of the operand buffers, then every lane handles 8 consecutive columns of a row (16-byte
  // global accesses).  Accumulator layout of a 32x32 tile: column = lane % 32,
  // row = 8 * (r / 4) + 4 * (lane / 32) + r % 4.
  float* cs = reinterpret_cast<float*>(lds) + wave * (32 * WTN);
  const bool split = d.splits > 1;
  float* part = split ? d.partial + static_cast<long long>(zsplit) * d.M * d.N : nullptr;
  constexpr int LPR = WTN / 8;          // lanes per row
  constexpr int RPI = 64 / LPR;         // rows per pass (96 columns: 5 rows, four lanes idle)
  constexpr int NIT = (32 + RPI - 1) / RPI;
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
    for (int it = 0; it < NIT; ++it) {
      const int row = it * RPI + lane / LPR;
      const int m = m0 + wm * WTM + i * 32 + row;
      if (lane / LPR >= RPI || row >= 32 || m >= d.M || n >= d.N) continue;
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

// The shapes that are built, instantiated explicitly (see gemm_pipe.hip): 256 x 256 for all three operand forms,
// the narrower ones for dY^T X.
#define RS_TT_SHAPES(X) X(256, 256) X(192, 256) X(256, 192) X(128, 256) X(256, 128) X(192, 192) X(128, 192) X(192, 128) X(128, 128)
template __global__ void gemm_bf16_rs_kernel<256, 256, false, false>(const GemmDesc, int, int);
template __global__ void gemm_bf16_rs_kernel<256, 256, false, true>(const GemmDesc, int, int);
#define RS_INSTANTIATE_TT(BM, BN) template __global__ void gemm_bf16_rs_kernel<BM, BN, true, true>(const GemmDesc, int, int);
RS_TT_SHAPES(RS_INSTANTIATE_TT)
#undef RS_INSTANTIATE_TT

// ---------------------------------------------------------------------------------------------
bool gemm_rs_ok(const GemmDesc& d, int k_chunk) {
  if (d.trans_a && !d.trans_b) return false;            // combination not used by the layers
  if (d.K % 64 || k_chunk % 64) return false;           // full slabs only
  return d.M >= 8 && d.N >= 8;
}

template <int BM, int BN, bool TA, bool TB>
static hipError_t rs_launch_shape(ecospa_ctx* ctx, const GemmDesc& d, int k_chunk) {
  const int tm = (d.M + BM - 1) / BM, tn = (d.N + BN - 1) / BN;
  const int splits = d.splits > 1 ? d.splits : 1;
  const dim3 grid(tm * tn * splits), block(256);
  // two operand buffers; they also cover the epilogue staging (4 x 32 x BN/2 floats) and the column-sum scratch
  // (256 x 3 x 9 words at most)
  constexpr int operand_bytes = 2 * (BM + BN) * 64 * static_cast<int>(sizeof(bf16_t));
  constexpr int lds_bytes = operand_bytes > 32768 ? operand_bytes : 32768;
  auto kern = gemm_bf16_rs_kernel<BM, BN, TA, TB>;
  static LdsAttrOnce attr_once;
  if (lds_bytes > 64 * 1024) {
    hipError_t e = attr_once.ensure(reinterpret_cast<const void*>(kern), lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, grid, block, lds_bytes, ctx->stream, d, tn, k_chunk);
  return hipGetLastError();
}

bool gemm_rs_shape_ok(int bm, int bn) {
#define RS_SHAPE_CHECK(BM, BN) if (bm == BM && bn == BN) return true;
  RS_TT_SHAPES(RS_SHAPE_CHECK)
#undef RS_SHAPE_CHECK
  return false;
}

hipError_t gemm_rs_launch(ecospa_ctx* ctx, const GemmDesc& d, int k_chunk, int bm, int bn) {
  if (d.trans_a) {
#define RS_SHAPE_LAUNCH(BM, BN) if (bm == BM && bn == BN) return rs_launch_shape<BM, BN, true, true>(ctx, d, k_chunk);
    RS_TT_SHAPES(RS_SHAPE_LAUNCH)
#undef RS_SHAPE_LAUNCH
    return hipErrorInvalidValue;
  }
  if (bm != 256 || bn != 256) return hipErrorInvalidValue;
  if (d.trans_b) return rs_launch_shape<256, 256, false, true>(ctx, d, k_chunk);
  return rs_launch_shape<256, 256, false, false>(ctx, d, k_chunk);
}
