// Dense contractions of the reduced forward/backward pass.
//
// bf16: 128x128x64 workgroup tiles, 4 wavefronts of 64x64, v_mfma_f32_32x32x16_bf16, operands
//       staged through XOR-swizzled LDS with register double buffering; operands whose K index
//       is the slow storage axis (dY W, dY^T X) are transposed in registers on the way to LDS.
// fp32: 64x64x16 vector-ALU tiles (the fp32 configuration is small and launch bound).
// Split-K writes fp32 partials that a second kernel adds in a fixed order (deterministic dW).
#include "gemm_lds.h"

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel, parametrised by the workgroup tile BM x BN and the WGM x WGN grid of wavefronts
// ---------------------------------------------------------------------------------------------
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// LDS operand tiles are [rows][BK] bf16 with the 16-byte chunks of a row XOR-swizzled by the row
// index, so that the 32 lanes that read one k-chunk of 32 consecutive rows spread over the banks.
template <int BK>
__device__ __forceinline__ int lds_off(int row, int chunk) {
  constexpr int CPR = BK / 8;                       // chunks per row (8 for BK = 64, 4 for BK = 32)
  const int f = BK == 64 ? (row ^ (row >> 3)) : ((row >> 1) ^ (row >> 3));
  return row * BK + ((chunk ^ (f & (CPR - 1))) << 3);
}

// Loads are unconditional (straight-line code that the scheduler can interleave with MFMAs): row
// indices beyond the matrix are clamped - such rows only feed outputs that are never stored - and
// only a K slab that crosses k_end (FULL = false) zero-fills its out-of-range chunks.
// K-contiguous operand: the tile is ROWS x BK/8 chunks of 8 elements.
template <int ROWS, int BK, int THREADS, bool FULL>
__device__ __forceinline__ void gload_kc(const bf16_t* __restrict__ base, long long ld, int row0, int R, int k0,
                                         int k_end, u32x4 (&reg)[(ROWS * BK / 8 / THREADS < 4 ? 4 : ROWS * BK / 8 / THREADS)]) {
  constexpr int CPR = BK / 8;
#pragma unroll
  for (int i = 0; i < ROWS * CPR / THREADS; ++i) {
    const int c = threadIdx.x + i * THREADS;
    const int gr = min(row0 + c / CPR, R - 1), gk = k0 + (c % CPR) * 8;
    if (FULL) {
      reg[i] = *reinterpret_cast<const u32x4*>(base + static_cast<long long>(gr) * ld + gk);
    } else {
      const u32x4 v = *reinterpret_cast<const u32x4*>(base + static_cast<long long>(gr) * ld + min(gk, k_end - 8));
      reg[i] = gk < k_end ? v : u32x4{0u, 0u, 0u, 0u};
    }
  }
}
template <int ROWS, int BK, int THREADS>
__device__ __forceinline__ void sstore_kc(bf16_t* lds, const u32x4 (&reg)[(ROWS * BK / 8 / THREADS < 4 ? 4 : ROWS * BK / 8 / THREADS)]) {
  constexpr int CPR = BK / 8;
#pragma unroll
  for (int i = 0; i < ROWS * CPR / THREADS; ++i) {
    const int c = threadIdx.x + i * THREADS;
    *reinterpret_cast<u32x4*>(lds + lds_off<BK>(c / CPR, c % CPR)) = reg[i];
  }
}
// K-contiguous operand, full K slab, BK = 64: global -> LDS without passing through registers.
// One global_load_lds_dwordx4 of a wavefront fills 64 consecutive 16-byte chunks of LDS (lane i
// writes chunk i of the 1 KB block the wave-uniform base points at) = 8 tile rows.  The swizzle is
// applied on the global side: the lane that owns physical chunk pc of row r fetches the logical
// k-chunk that lds_off() maps there.
template <int ROWS, int THREADS>
__device__ __forceinline__ void dload_kc(const bf16_t* __restrict__ base, long long ld, int row0, int R, int k0,
                                         lds_bf16_t* tile) {
  constexpr int PER = ROWS / 8 / (THREADS / 64);     // 8-row groups per wavefront
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane >> 3, pc = lane & 7;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int group = wave * PER + i;
    const int row = group * 8 + r;
    const int kc = pc ^ ((row ^ (row >> 3)) & 7);
    const int gr = min(row0 + row, R - 1);
    __builtin_amdgcn_global_load_lds(base + static_cast<long long>(gr) * ld + k0 + kc * 8, tile + group * 8 * 64, 16, 0, 0);
  }
}
// K-slow operand (storage [K][R]): 4(k) x 8(r) blocks, transposed in registers on the way to LDS
template <int ROWS, int BK, int THREADS, bool FULL>
__device__ __forceinline__ void gload_tr(const bf16_t* __restrict__ base, long long ld, int row0, int R, int k0,
                                         int k_end, u32x4 (&reg)[(ROWS * BK / 8 / THREADS < 4 ? 4 : ROWS * BK / 8 / THREADS)]) {
  constexpr int NSUB = ROWS * BK / 32;            // 4 x 8 sub-blocks in the tile
#pragma unroll
  for (int b = 0; b < (NSUB + THREADS - 1) / THREADS; ++b) {
    const int sb = threadIdx.x + b * THREADS;
    if (NSUB % THREADS != 0 && sb >= NSUB) break;
    const int rblk = sb % (ROWS / 8), kblk = sb / (ROWS / 8);
    const int gr = min(row0 + rblk * 8, R - 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int gk = k0 + kblk * 4 + i;
      if (FULL) {
        reg[b * 4 + i] = *reinterpret_cast<const u32x4*>(base + static_cast<long long>(gk) * ld + gr);
      } else {
        const u32x4 v = *reinterpret_cast<const u32x4*>(base + static_cast<long long>(min(gk, k_end - 1)) * ld + gr);
        reg[b * 4 + i] = gk < k_end ? v : u32x4{0u, 0u, 0u, 0u};
      }
    }
  }
}
template <int ROWS, int BK, int THREADS>
__device__ __forceinline__ void sstore_tr(bf16_t* lds, const u32x4 (&reg)[(ROWS * BK / 8 / THREADS < 4 ? 4 : ROWS * BK / 8 / THREADS)]) {
  constexpr int NSUB = ROWS * BK / 32;
#pragma unroll
  for (int b = 0; b < (NSUB + THREADS - 1) / THREADS; ++b) {
    const int sb = threadIdx.x + b * THREADS;
    if (NSUB % THREADS != 0 && sb >= NSUB) break;
    const int rblk = sb % (ROWS / 8), kblk = sb / (ROWS / 8);
    const int kc = kblk >> 1, half = kblk & 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int r = rblk * 8 + j;
      uint32_t e[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) e[i] = (j & 1) ? (reg[b * 4 + i][j >> 1] >> 16) : (reg[b * 4 + i][j >> 1] & 0xffffu);
      u32x2 v;
      v.x = e[0] | (e[1] << 16);
      v.y = e[2] | (e[3] << 16);
      *reinterpret_cast<u32x2*>(lds + lds_off<BK>(r, kc) + half * 4) = v;
    }
  }
}

// K-slow operand kept as it lies in memory, [BK][ROWS] (fragments then come from transposing LDS
// reads): the four 16-byte pieces of a thread's 4(k) x 8(r) block go to four k rows - no shuffling.
template <int ROWS, int BK, int THREADS>
__device__ __forceinline__ void sstore_ks(bf16_t* lds, const u32x4 (&reg)[(ROWS * BK / 8 / THREADS < 4 ? 4 : ROWS * BK / 8 / THREADS)]) {
  constexpr int NSUB = ROWS * BK / 32;
#pragma unroll
  for (int b = 0; b < (NSUB + THREADS - 1) / THREADS; ++b) {
    const int sb = threadIdx.x + b * THREADS;
    if (NSUB % THREADS != 0 && sb >= NSUB) break;
    const int rblk = sb % (ROWS / 8), kblk = sb / (ROWS / 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(lds + ks_off<ROWS>(kblk * 4 + i, rblk)) = reg[b * 4 + i];
  }
}

// LDS traffic of one wavefront with itself (its private staging area): order only, no s_barrier
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup tile BM x BN x BK, WGM x WGN wavefronts; WPE = wavefronts per SIMD the register
// allocation is tuned for (occupancy hides the LDS and global latencies between MFMAs).
// TRR: K-slow operands stay untransposed in LDS and are read with ds_read_b64_tr_b16.
template <int BM, int BN, int BK, int WGM, int WGN, int WPE, bool TA, bool TB, bool TRR>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemm_bf16_mfma_kernel(const GemmDesc d, int tiles_n, int k_chunk) {
  constexpr int THREADS = 64 * WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, FM = WTM / 32, FN = WTN / 32;
  constexpr int STAGE = (BM + BN) * BK;            // elements of one LDS buffer (A tile then B tile)
  constexpr int NA = BM * BK / 8 / THREADS < 4 ? 4 : BM * BK / 8 / THREADS;
  constexpr int NB = BN * BK / 8 / THREADS < 4 ? 4 : BN * BK / 8 / THREADS;
  static_assert(WTN == 64 || WTN == 128, "epilogue handles 64 or 128 columns per wavefront");
  static_assert((BM * BK / 8) % THREADS == 0 && (BN * BK / 8) % THREADS == 0, "loader shape");
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs, so give each XCD a
  // contiguous range of tiles (neighbouring tiles share operand rows in that XCD's L2).
  int id, zsplit;
  gemm_work_item(d.splits > 1 ? d.splits : 1, id, zsplit);
  const int m0 = (id / tiles_n) * BM, n0 = (id % tiles_n) * BN;
  const int k_begin = zsplit * k_chunk;
  const int k_end = min(d.K, k_begin + k_chunk);
  const int nk = (k_end - k_begin + BK - 1) / BK;

  const bf16_t* A = static_cast<const bf16_t*>(d.A);
  const bf16_t* B = static_cast<const bf16_t*>(d.B);
  u32x4 ra[NA], rb[NB];
  // Column sums of a K-slow A operand (bias gradient, GemmDesc::colsum): a thread's 4(k) x 8(m) sub-blocks keep their
  // m across the K loop, so it adds up its own eight columns; only the first tile column of the grid does it.
  constexpr bool CS = TA && TB;                      // the dY^T X form, the only one that asks for it
  constexpr int NCS = CS ? NA / 4 : 1;
  const bool do_cs = CS && d.colsum != nullptr && n0 == 0;
  float cs_acc[NCS][8];
#pragma unroll
  for (int b = 0; b < NCS; ++b)
#pragma unroll
    for (int j = 0; j < 8; ++j) cs_acc[b][j] = 0.f;
  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Operand staging for K slab k0 into LDS buffer `buf`.  K-contiguous operands whose slab lies
  // fully inside [k_begin, k_end) go straight to LDS (BK = 64 only); K-slow operands and the ragged
  // last slab travel through registers (FETCH now, STORE after the MFMAs of the current slab).
  constexpr bool DIRECT_OK = BK == 64;
  lds_bf16_t* lds3 = (lds_bf16_t*)lds;   // same array, LDS address space for the direct loads
#define GEMM_FETCH(k0, buf)                                                                        \
  do {                                                                                             \
    const bool full_ = (k0) + BK <= k_end;                                                         \
    if (!TA && DIRECT_OK && full_) dload_kc<BM, THREADS>(A, d.lda, m0, d.M, (k0), lds3 + (buf) * STAGE);          \
    else if (TA) { if (full_) gload_tr<BM, BK, THREADS, true>(A, d.lda, m0, d.M, (k0), k_end, ra);                \
                   else gload_tr<BM, BK, THREADS, false>(A, d.lda, m0, d.M, (k0), k_end, ra); }                   \
    else { if (full_) gload_kc<BM, BK, THREADS, true>(A, d.lda, m0, d.M, (k0), k_end, ra);                        \
           else gload_kc<BM, BK, THREADS, false>(A, d.lda, m0, d.M, (k0), k_end, ra); }                           \
    if (!TB && DIRECT_OK && full_) dload_kc<BN, THREADS>(B, d.ldb, n0, d.N, (k0), lds3 + (buf) * STAGE + BM * BK); \
    else if (TB) { if (full_) gload_tr<BN, BK, THREADS, true>(B, d.ldb, n0, d.N, (k0), k_end, rb);                \
                   else gload_tr<BN, BK, THREADS, false>(B, d.ldb, n0, d.N, (k0), k_end, rb); }                   \
    else { if (full_) gload_kc<BN, BK, THREADS, true>(B, d.ldb, n0, d.N, (k0), k_end, rb);                        \
           else gload_kc<BN, BK, THREADS, false>(B, d.ldb, n0, d.N, (k0), k_end, rb); }                           \
  } while (0)
#define GEMM_STORE(k0, buf)                                                                        \
  do {                                                                                             \
    const bool full_ = (k0) + BK <= k_end;                                                         \
    bf16_t* as_ = lds + (buf) * STAGE;                                                             \
    if (CS && do_cs) {                                                                             \
      _Pragma("unroll") for (int q_ = 0; q_ < NCS * 4; ++q_) {                                     \
        const uint32_t w_[4] = {ra[q_].x, ra[q_].y, ra[q_].z, ra[q_].w};                           \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                                         \
          cs_acc[q_ / 4][2 * i_] += __uint_as_float(w_[i_] << 16);                                 \
          cs_acc[q_ / 4][2 * i_ + 1] += __uint_as_float(w_[i_] & 0xffff0000u);                     \
        }                                                                                          \
      }                                                                                            \
    }                                                                                              \
    if (TA && TRR) sstore_ks<BM, BK, THREADS>(as_, ra);                                            \
    else if (TA) sstore_tr<BM, BK, THREADS>(as_, ra);                                              \
    else if (!(DIRECT_OK && full_)) sstore_kc<BM, BK, THREADS>(as_, ra);                           \
    if (TB && TRR) sstore_ks<BN, BK, THREADS>(as_ + BM * BK, rb);                                  \
    else if (TB) sstore_tr<BN, BK, THREADS>(as_ + BM * BK, rb);                                    \
    else if (!(DIRECT_OK && full_)) sstore_kc<BN, BK, THREADS>(as_ + BM * BK, rb);                 \
  } while (0)

  if (nk > 0) {
    GEMM_FETCH(k_begin, 0);
    GEMM_STORE(k_begin, 0);
  }
  __builtin_amdgcn_s_waitcnt(0);     // direct-to-LDS loads are counted by vmcnt
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const int k_next = k_begin + (kt + 1) * BK;
    if (kt + 1 < nk) GEMM_FETCH(k_next, cur ^ 1);
    const bf16_t* As = lds + cur * STAGE;
    const bf16_t* Bs = As + BM * BK;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      bf16x8_t a[FM], b[FN];
      const int kc = s * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < FM; ++i)
        a[i] = (TA && TRR) ? read_frag<BM, BK, true>(As, wm * WTM + i * 32, s)
                           : *reinterpret_cast<const bf16x8_t*>(As + lds_off<BK>(wm * WTM + i * 32 + (lane & 31), kc));
#pragma unroll
      for (int j = 0; j < FN; ++j)
        b[j] = (TB && TRR) ? read_frag<BN, BK, true>(Bs, wn * WTN + j * 32, s)
                           : *reinterpret_cast<const bf16x8_t*>(Bs + lds_off<BK>(wn * WTN + j * 32 + (lane & 31), kc));
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) GEMM_STORE(k_next, cur ^ 1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  }
#undef GEMM_FETCH
#undef GEMM_STORE

  if (CS && d.colsum != nullptr) {       // uniform over the grid; the operand buffers are idle now
    float* red = reinterpret_cast<float*>(lds);      // [BK / 4 k-blocks][BM]
    if (do_cs) {
#pragma unroll
      for (int b = 0; b < NCS; ++b) {
        const int sb = tid + b * THREADS;
        const int rblk = sb % (BM / 8), kblk = sb / (BM / 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) red[kblk * BM + rblk * 8 + j] = cs_acc[b][j];
      }
    }
    __syncthreads();
    if (do_cs)
      for (int r = tid; r < BM; r += THREADS) {
        float s = 0.f;
#pragma unroll
        for (int kb = 0; kb < BK / 4; ++kb) s += red[kb * BM + r];     // fixed order
        if (m0 + r < d.M) d.colsum[static_cast<long long>(zsplit) * d.M + m0 + r] = s;
      }
    __syncthreads();
  }

  // Epilogue through LDS: each wavefront parks 32 rows x WTN columns of fp32 at a time in its own
  // slice of the (now idle) operand buffers, then every lane handles 8 consecutive columns of a
  // row, so global traffic is 16-byte vectors.  Accumulator layout of a 32x32 MFMA tile:
  // column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4.
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
    wave_lds_sync();
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
    wave_lds_sync();
  }
}

// ---------------------------------------------------------------------------------------------
// fp32 (and generic fallback) vector-ALU kernel: 64x64 tile, 16x16 threads, 4x4 per thread
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gemm_valu_kernel(const GemmDesc d, int tiles_n, int k_chunk) {
  // 64 x 64 tile, 32-deep slabs; the 16 operand elements a thread moves per slab are fetched one slab ahead with
  // unconditional loads from clamped addresses (all in flight together, none behind a branch) and dropped by a
  // select where they lie outside the problem: these problems are small, so nothing but the loads' own
  // parallelism hides their latency.
  constexpr int BK = 32, NL = 64 * BK / 256;
  __shared__ float As[BK][64 + 4];
  __shared__ float Bs[BK][64 + 4];
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

  float ra[NL], rb[NL];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int e = tid + i * 256;
      {
        const int kk = d.trans_a ? e >> 6 : e & (BK - 1), r = d.trans_a ? e & 63 : e / BK;
        const int gm = m0 + r, gk = k0 + kk;
        const long long cm = min(gm, d.M - 1), ck = min(gk, k_end - 1);
        const float v = load_f32<T>(A + (d.trans_a ? ck * d.lda + cm : cm * d.lda + ck));
        ra[i] = (gm < d.M && gk < k_end) ? v : 0.f;
      }
      {
        const int kk = d.trans_b ? e >> 6 : e & (BK - 1), r = d.trans_b ? e & 63 : e / BK;
        const int gn = n0 + r, gk = k0 + kk;
        const long long cn = min(gn, d.N - 1), ck = min(gk, k_end - 1);
        const float v = load_f32<T>(B + (d.trans_b ? ck * d.ldb + cn : cn * d.ldb + ck));
        rb[i] = (gn < d.N && gk < k_end) ? v : 0.f;
      }
    }
  };
  if (k_begin < k_end) fetch(k_begin);
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int e = tid + i * 256;
      As[d.trans_a ? e >> 6 : e & (BK - 1)][d.trans_a ? e & 63 : e / BK] = ra[i];
      Bs[d.trans_b ? e >> 6 : e & (BK - 1)][d.trans_b ? e & 63 : e / BK] = rb[i];
    }
    __syncthreads();
    if (k0 + BK < k_end) fetch(k0 + BK);      // the same for the whole workgroup
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
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
// bf16: 8 consecutive columns per thread (N is a multiple of 8)
__global__ __launch_bounds__(256) void gemm_splitk_reduce_vec8_kernel(const GemmDesc d) {
  const long long tot = static_cast<long long>(d.M) * d.N;
  const long long e = (static_cast<long long>(blockIdx.x) * 256 + threadIdx.x) * 8;
  if (e >= tot) return;
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = 0.f;
  for (int z = 0; z < d.splits; ++z) {
    const float4 lo = *reinterpret_cast<const float4*>(d.partial + z * tot + e);
    const float4 hi = *reinterpret_cast<const float4*>(d.partial + z * tot + e + 4);
    v[0] += lo.x; v[1] += lo.y; v[2] += lo.z; v[3] += lo.w; v[4] += hi.x; v[5] += hi.y; v[6] += hi.z; v[7] += hi.w;
  }
  epi_apply_vec8(d.epi, static_cast<int>(e / d.N), static_cast<int>(e % d.N), v);
}

// ---------------------------------------------------------------------------------------------
// Tile choice: 256x256 tiles (8 wavefronts, 128 KB LDS, one workgroup per CU) need about twice
// fewer operand bytes per flop than 128x128 tiles (4 wavefronts, two workgroups per CU), but only
// pay off when there are enough of them to occupy the 256 CUs.
static bool gemm_prefers_big_tile(int M, int N, int splits) {
  const long long big = static_cast<long long>((M + 255) / 256) * ((N + 255) / 256) * splits;
  const long long small = static_cast<long long>((M + 127) / 128) * ((N + 127) / 128) * splits;
  // 256x256 tiles when they fill three quarters of the compute units - or two thirds, if the 128x128 tiles
  // would need more than one round of 512
  return big >= 192 || (big >= 168 && small > 512);
}

// Which configuration of the software-pipelined kernel (gemm_pipe.hip) suits a problem, or -1 for the
// register-staged kernel above.  Measured on the layer shapes (M = tokens = 8192, N and K between 512
// and 4096) inside the layer step: for K-contiguous operands (x W^T) the largest workgroup tile that
// still yields about one tile per compute unit wins; with a K-slow B operand (dY W) that holds only
// for the 256x256 configuration (its two wavefronts per SIMD cover the transposing reads); dY^T X
// stays on the register-staged kernel.
static int gemm_pipe_choice(const GemmDesc& d) {
  if (d.trans_a) return -1;
  const long long tm256 = (d.M + 255) / 256, t256 = tm256 * ((d.N + 255) / 256), t256x128 = tm256 * ((d.N + 127) / 128);
  if (t256 >= 192) {
    // 256x256 with 8 wavefronts - unless its tiles fill the last round over the 256 compute units so badly that
    // narrower tiles finish sooner.  Cost of a choice: rounds of work times the area of a tile, the 256x128 tiles
    // taken as 7 % and the 256x192 tiles (two ring slots only) as 17 % less efficient per flop (fitted to cold-cache
    // timings of the layer shapes); 256x192 serves the widths that are multiples of 192 (the fused Q|K|V
    // projections of both layers) and K-contiguous operands only.
    if (!d.trans_b) {
      const long long t256x192 = tm256 * ((d.N + 191) / 192);
      const long long c256 = (t256 + 255) / 256 * 256 * 100, c192 = (t256x192 + 255) / 256 * 192 * 117,
                      c128 = (t256x128 + 255) / 256 * 128 * 107;
      if (c192 < c256 && c192 <= c128) return 10;
      if (c128 < c256) return 9;
    }
    return 5;
  }
  if (d.trans_b) return -1;
  if (t256x128 >= 192) {
    // 256x128 (8 wavefronts, 3-deep ring) - or 256x192 when its tiles fit one round where the narrower ones need
    // two (output widths a little above a multiple of 256: what an FFN keeps at a keep ratio like 3/10)
    const long long t256x192 = tm256 * ((d.N + 191) / 192);
    const long long c192 = (t256x192 + 255) / 256 * 192 * 117, c128 = (t256x128 + 255) / 256 * 128 * 107;
    return c192 < c128 ? 10 : 9;
  }
  return 6;                       // 128x128 with 32-deep slabs in a ring of four: more loads in flight than two 64-deep slabs, which
                                  // matters when a compute unit holds one such workgroup (measured on the few-token shapes)
}
// Long contractions with a K-slow B operand (K of several thousand, at least a tile per compute unit)
// run fastest on the two-slab register prefetch of gemm_rs.hip.
static bool gemm_prefers_rs_nt(const GemmDesc& d) {
  const long long t256 = static_cast<long long>((d.M + 255) / 256) * ((d.N + 255) / 256);
  return !d.trans_a && d.trans_b && d.splits <= 1 && d.K >= 4096 && t256 >= 192;
}

template <int BM, int BN, int BK, int WGM, int WGN, int WPE, bool TRR>
static hipError_t launch_tile(ecospa_ctx* ctx, const GemmDesc& d, int k_chunk) {
  const int tm = (d.M + BM - 1) / BM, tn = (d.N + BN - 1) / BN;
  const int splits = d.splits > 1 ? d.splits : 1;
  const dim3 grid(tm * tn * splits), block(64 * WGM * WGN);
  const size_t operand_bytes = 2ull * (BM + BN) * BK * sizeof(bf16_t);
  const size_t staging_bytes = static_cast<size_t>(WGM) * WGN * 32 * (BN / WGN) * 4;   // epilogue tiles
  const size_t lds_bytes = operand_bytes > staging_bytes ? operand_bytes : staging_bytes;
#define LAUNCH_TT(TA, TB)                                                                                      \
  do {                                                                                                         \
    auto kern = gemm_bf16_mfma_kernel<BM, BN, BK, WGM, WGN, WPE, TA, TB, (TRR && (TA || TB))>;                         \
    static LdsAttrOnce attr_once;                                                                              \
    if (lds_bytes > 64 * 1024) {                                                                               \
      hipError_t e = attr_once.ensure(reinterpret_cast<const void*>(kern), static_cast<int>(lds_bytes));       \
      if (e != hipSuccess) return e;                                                                           \
    }                                                                                                          \
    hipLaunchKernelGGL(kern, grid, block, lds_bytes, ctx->stream, d, tn, k_chunk);                             \
  } while (0)
  if (!d.trans_a && !d.trans_b) LAUNCH_TT(false, false);
  else if (!d.trans_a && d.trans_b) LAUNCH_TT(false, true);
  else if (d.trans_a && d.trans_b) LAUNCH_TT(true, true);
  else LAUNCH_TT(true, false);
#undef LAUNCH_TT
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Weight-gradient contractions (dY^T X: K = tokens, few output tiles) on the register-prefetch kernel of
// gemm_rs.hip: one workgroup per compute unit, so the tile shape (bm, bn from 128, 192, 256) and the number of K
// splits are chosen together to finish soonest on 256 compute units.  Cost of a choice, in microseconds, fitted to
// per-workgroup timings of every shape on this GPU (both operands K-slow; the loop is bound by moving the operands,
// hence the term in bm + bn beside the one in bm * bn):
//   slab (64 of K)  = 0.05 + 0.9 (bm + bn) / 512 + 0.73 bm bn / 256^2
//   epilogue        = 0.3 + 8.1 bm bn / 256^2          (all workgroups of a round write at once)
//   rounds          = ceil(tiles * splits / 256), each round = slabs per split * slab + epilogue
//   split K         = a later pass over the partial sums: 3 + (splits * M * N * 4 + M * N * 2) bytes at 4 TB/s
// A split keeps at least 512 of K.
bool gemm_tt_plan(int M, int N, int K, int* bm_out, int* bn_out, int* splits_out) {
  if (K % 64 || K < 1024 || M < 8 || N < 8) return false;
  const int slabs = K / 64;
  double best = 0.0;
  bool found = false;
  for (int q = 0; q < GEMM_RS_NSHAPES; ++q) {
    const int bm = GEMM_RS_SHAPES[q][0], bn = GEMM_RS_SHAPES[q][1];
    const long long tiles = static_cast<long long>((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    const double area = static_cast<double>(bm) * bn / 65536.0;
    const double slab = 0.05 + 0.9 * (bm + bn) / 512.0 + 0.73 * area, epi = 0.3 + 8.1 * area;
    for (int sp = 1; sp <= 8; ++sp) {
      const int per = (slabs + sp - 1) / sp;                 // slabs of the first splits; the last one takes the rest
      if (per * (sp - 1) >= slabs || (sp > 1 && per < 8)) continue;
      const long long wg = tiles * sp, rounds = (wg + 255) / 256;
      const double mn = static_cast<double>(M) * N;
      const double red = sp > 1 ? 3.0 + (sp * mn * 4.0 + mn * 2.0) / 4.0e6 : 0.0;
      const double t = 3.0 + rounds * (per * slab + epi) + red;
      if (!found || t < best) {
        found = true;
        best = t;
        *bm_out = bm; *bn_out = bn; *splits_out = sp;
      }
    }
  }
  return found;
}

int ecospa_gemm_splits(int M, int N, int K) {
  int bm, bn, sp;
  if (gemm_tt_plan(M, N, K, &bm, &bn, &sp)) return sp;
  const long long tiles = static_cast<long long>((M + 127) / 128) * ((N + 127) / 128);
  int s = 1;
  // Two 128x128 workgroups fit a compute unit, so 512 of them run at once: split K while all splits still fit
  // that one round and every split keeps at least 512 of K, eight ways at most.  More splits than that only add
  // partial sums to write and reduce (measured on the weight-gradient shapes of both layers, inside their steps).
  while (tiles * s * 2 <= 512 && K / (s * 2) >= 512 && s < 8) s *= 2;
  return s;
}

int ecospa_gemm_token_splits(int M, int N, int K) {
  const long long tiles = static_cast<long long>((M + 127) / 128) * ((N + 127) / 128);
  int s = 1;
  while (tiles * s * 2 <= 256 && K / (s * 2) >= 1024 && s < 8) s *= 2;
  return s;
}

// Which kernel a bf16 contraction goes to: the register-prefetch kernel with tile rs_bm x rs_bn (rs_bm = 0: not that
// one), else configuration cfg of the pipelined kernel (cfg < 0: neither - the register-staged kernel).
// tile codes: 10-19 and 21 name the configurations 0-9 and 10 of the pipelined kernel, 20 the register-prefetch
// kernel with 256 x 256 tiles, 30 + i the same kernel with shape i of GEMM_RS_SHAPES (dY^T X only).
static void gemm_route(const GemmDesc& d, int splits, int* k_split_out, int* cfg_out, int* rs_bm_out, int* rs_bn_out) {
  // K range of a split: whole 64-deep slabs, the first splits take one slab more when the slabs do not divide
  const int k_split = d.K % 64 == 0 ? (d.K / 64 + splits - 1) / splits * 64 : (d.K + splits - 1) / splits;
  const bool no_empty_split = static_cast<long long>(k_split) * (splits - 1) < d.K;
  int cfg = d.tile >= 10 && d.tile < 20 ? d.tile - 10 : (d.tile == 21 ? 10 : (d.tile == 0 ? gemm_pipe_choice(d) : -1));
  int rs_bm = 0, rs_bn = 0;
  if (d.tile == 20) { rs_bm = rs_bn = 256; }
  else if (d.tile >= 30 && d.tile < 30 + GEMM_RS_NSHAPES && d.trans_a && d.trans_b) { rs_bm = GEMM_RS_SHAPES[d.tile - 30][0]; rs_bn = GEMM_RS_SHAPES[d.tile - 30][1]; }
  else if (d.tile == 0 && d.trans_a && d.trans_b) {
    int sp;      // dY^T X: the planned shape, when the caller split K as planned
    if (!(gemm_tt_plan(d.M, d.N, d.K, &rs_bm, &rs_bn, &sp) && sp == splits)) rs_bm = rs_bn = 0;
  } else if (d.tile == 0 && gemm_prefers_rs_nt(d)) { rs_bm = rs_bn = 256; }
  if (!(rs_bm && gemm_rs_ok(d, k_split) && no_empty_split)) rs_bm = rs_bn = 0;
  if (!(cfg >= 0 && gemm_pipe_ok(d, cfg, k_split) && no_empty_split)) cfg = -1;
  *k_split_out = k_split; *cfg_out = cfg; *rs_bm_out = rs_bm; *rs_bn_out = rs_bn;
}

// Rows of the partial column-sum matrix (GemmDesc::colsum) that the launch of d writes, M floats each: one per K split,
// times the tile columns when the register-prefetch kernel runs it (there every tile column adds up its share of the
// slabs).  The caller sizes the buffer with it and adds the rows up in order.
int ecospa_gemm_colsum_rows(const GemmDesc& d) {
  const int splits = d.splits > 1 ? d.splits : 1;
  if (d.dtype != ECOSPA_BF16) return splits;
  int k_split, cfg, rs_bm, rs_bn;
  gemm_route(d, splits, &k_split, &cfg, &rs_bm, &rs_bn);
  return rs_bm ? splits * ((d.N + rs_bn - 1) / rs_bn) : splits;
}

int ecospa_gemm(ecospa_ctx* ctx, const GemmDesc& d) {
  if (d.M < 1 || d.N < 1 || d.K < 1) return ECOSPA_ERR_SHAPE;
  if (!d.A || !d.B || (!d.epi.c && d.epi.kind != EPI_SWIGLU)) return ECOSPA_ERR_NULL;      // the gated epilogue may skip its first output
  if (d.splits > 1 && !d.partial) return ECOSPA_ERR_WORKSPACE;
  // column sums of the A operand: the dY^T X form on the kernels that stage A through registers (not the pipelined one)
  if (d.colsum && !(d.dtype == ECOSPA_BF16 && d.trans_a && d.trans_b && (d.tile <= 4 || d.tile == 20 || d.tile >= 30))) return ECOSPA_ERR_SHAPE;
  const int splits = d.splits > 1 ? d.splits : 1;
  if (d.dtype == ECOSPA_BF16) {
    // 16-byte vector loads along the contiguous axis of each operand
    const int ca = d.trans_a ? d.M : d.K, cb = d.trans_b ? d.N : d.K;
    if (ca % 8 || cb % 8 || d.lda % 8 || d.ldb % 8) return ECOSPA_ERR_ALIGN;
    if (!aligned16(d.A) || !aligned16(d.B)) return ECOSPA_ERR_ALIGN;
    // the epilogue moves 8 columns at a time
    if (d.N % 8 || d.epi.ldc % 8 || !aligned16(d.epi.c)) return ECOSPA_ERR_ALIGN;
    if (d.epi.kind == EPI_SWIGLU && (!d.epi.c2 || d.epi.ldc2 % 4 || (reinterpret_cast<uintptr_t>(d.epi.c2) & 7u))) return ECOSPA_ERR_ALIGN;
    if (d.epi.kind == EPI_ROPE && (!d.epi.rope_cos || !d.epi.rope_sin || !aligned16(d.epi.rope_cos) || !aligned16(d.epi.rope_sin) ||
                                   d.epi.rope_kp % 8 || d.epi.rope_cols % 8 || d.epi.rope_L < 1 || d.epi.rope_qpk < 1)) return ECOSPA_ERR_ALIGN;
    if (d.epi.bias && !aligned16(d.epi.bias)) return ECOSPA_ERR_ALIGN;
    if (d.epi.kind == EPI_BIAS_ACT && (!d.epi.c2 || d.epi.ldc2 % 8 || !aligned16(d.epi.c2))) return ECOSPA_ERR_ALIGN;
    if ((d.epi.kind == EPI_DACT || d.epi.kind == EPI_DSWIGLU) && (!d.epi.h || d.epi.ldh % 8 || !aligned16(d.epi.h)))
      return ECOSPA_ERR_ALIGN;
    if (d.epi.kind == EPI_DSWIGLU && d.epi.kp % 8) return ECOSPA_ERR_ALIGN;
    if (d.splits > 1 && !aligned16(d.partial)) return ECOSPA_ERR_ALIGN;
    int k_chunk = (d.K + splits - 1) / splits;
    k_chunk = (k_chunk + 63) / 64 * 64;
    const bool big = d.tile == 2 || (d.tile == 0 && gemm_prefers_big_tile(d.M, d.N, splits));
    const bool prof = ctx->prof_on && ctx->prof_n < ctx->prof_cap;
    if (prof) (void)hipEventRecord(ctx->prof_ev[2 * ctx->prof_n], ctx->stream);
    hipError_t le;
    int k_split, cfg, rs_bm, rs_bn;
    gemm_route(d, splits, &k_split, &cfg, &rs_bm, &rs_bn);
    if (rs_bm) le = gemm_rs_launch(ctx, d, k_split, rs_bm, rs_bn);
    else if (cfg >= 0) le = gemm_pipe_launch(ctx, d, cfg, k_split);
    else {
      // register-staged kernel; tile 1/2 = 128/256 tiles with K-slow operands transposed on the way to
      // LDS, 3/4 = the same tiles with K-slow operands read by transposing LDS reads.  Measured: the
      // transposing reads win only when BOTH operands are K-slow (dY^T X).
      int t = d.tile >= 1 && d.tile <= 4 ? d.tile : (big ? 2 : 1);
      if (d.tile == 0 && d.trans_a && d.trans_b) t += 2;
      if (t == 4) le = launch_tile<256, 256, 64, 2, 4, 2, true>(ctx, d, k_chunk);
      else if (t == 3) le = launch_tile<128, 128, 64, 2, 2, 2, true>(ctx, d, k_chunk);
      else if (t == 2) le = launch_tile<256, 256, 64, 2, 4, 2, false>(ctx, d, k_chunk);
      else le = launch_tile<128, 128, 64, 2, 2, 2, false>(ctx, d, k_chunk);
    }
    if (le != hipSuccess) return hip_fail(ctx, le, "gemm launch");
    if (prof) {
      (void)hipEventRecord(ctx->prof_ev[2 * ctx->prof_n + 1], ctx->stream);
      ctx->prof_flop[ctx->prof_n++] = 2.0 * d.M * d.N * d.K;
    }
    ECOSPA_CHECK_LAUNCH(ctx, "gemm_bf16_mfma_kernel");
  } else if (d.dtype == ECOSPA_F32) {
    if (d.epi.kind == EPI_ROPE || d.epi.kind == EPI_SWIGLU) return ECOSPA_ERR_DTYPE;
    const int tm = (d.M + 63) / 64, tn = (d.N + 63) / 64;
    int k_chunk = (d.K + splits - 1) / splits;
    k_chunk = (k_chunk + 31) / 32 * 32;
    hipLaunchKernelGGL((gemm_valu_kernel<float>), dim3(tm * tn, 1, splits), dim3(256), 0, ctx->stream, d, tn, k_chunk);
    ECOSPA_CHECK_LAUNCH(ctx, "gemm_valu_kernel");
  } else {
    return ECOSPA_ERR_DTYPE;
  }
  if (splits > 1 && !d.defer_reduce) return ecospa_gemm_reduce(ctx, d);
  return ECOSPA_OK;
}

int ecospa_gemm_reduce(ecospa_ctx* ctx, const GemmDesc& d) {
  if (d.splits <= 1) return ECOSPA_OK;
  if (!d.partial || (!d.epi.c && d.epi.kind != EPI_SWIGLU)) return ECOSPA_ERR_NULL;
  const long long tot = static_cast<long long>(d.M) * d.N;
  if (d.dtype == ECOSPA_BF16)
    hipLaunchKernelGGL(gemm_splitk_reduce_vec8_kernel, dim3(static_cast<unsigned>((tot / 8 + 255) / 256)), dim3(256), 0,
                       ctx->stream, d);
  else
    hipLaunchKernelGGL((gemm_splitk_reduce_kernel<float>), dim3(static_cast<unsigned>((tot + 255) / 256)), dim3(256), 0,
                       ctx->stream, d);
  ECOSPA_CHECK_LAUNCH(ctx, "gemm_splitk_reduce_kernel");
  return ECOSPA_OK;
}

// ---------------------------------------------------------------------------------------------
// batched tail of a backward pass: split-K reductions and bias-gradient column sums in one launch
// ---------------------------------------------------------------------------------------------
#define AUX_THREADS 1024

struct AuxBatchDev {
  AuxBatch b;
  int blk_begin[2 * AUX_MAX_JOBS + 1];   // column sums first (long dependent chains), then reductions
};

template <typename T>
__device__ __forceinline__ void aux_reduce_block(const GemmDesc& d, int blk) {
  const long long tot = static_cast<long long>(d.M) * d.N;
  if (sizeof(T) == 2) {      // 8 consecutive columns per thread (N is a multiple of 8)
    const long long e = (static_cast<long long>(blk) * AUX_THREADS + threadIdx.x) * 8;
    if (e >= tot) return;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = 0.f;
    for (int z0 = 0; z0 < d.splits; z0 += 4) {     // four partials in flight, added in split order
      float4 lo[4], hi[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const bool on = z0 + q < d.splits;
        const float* p = d.partial + (on ? z0 + q : z0) * tot + e;
        lo[q] = *reinterpret_cast<const float4*>(p);
        hi[q] = *reinterpret_cast<const float4*>(p + 4);
        if (!on) lo[q] = hi[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        v[0] += lo[q].x; v[1] += lo[q].y; v[2] += lo[q].z; v[3] += lo[q].w;
        v[4] += hi[q].x; v[5] += hi[q].y; v[6] += hi[q].z; v[7] += hi[q].w;
      }
    }
    epi_apply_vec8(d.epi, static_cast<int>(e / d.N), static_cast<int>(e % d.N), v);
  } else {
    const long long e = static_cast<long long>(blk) * AUX_THREADS + threadIdx.x;
    if (e >= tot) return;
    float s = 0.f;
    for (int z = 0; z < d.splits; ++z) s += d.partial[z * tot + e];
    epi_apply<T>(d.epi, static_cast<int>(e / d.N), static_cast<int>(e % d.N), s);
  }
}

// One workgroup sums a strip of AUX_LANES x (16 bytes of columns) over all M rows: the row slots
// (AUX_THREADS / AUX_LANES of them) walk down the rows with 16-byte loads, several in flight, then
// the slots are added in a fixed order.  Narrow strips (a quarter of a 128-byte line) give enough
// workgroups to hide the latency; the four strips of a line are mapped to workgroup ids that differ
// by 8, 16 and 24, i.e. to the same XCD, so that the line is fetched into one L2 only.
#define AUX_LANES 2
template <typename T, typename TO>
__device__ __forceinline__ void aux_colsum_block(const AuxColsum& c, int blk, float* lds) {
  static_assert(AUX_LANES == 2, "four strips of AUX_LANES x 16 bytes make one 128-byte line");
  constexpr int V = 16 / sizeof(T);          // columns per lane
  constexpr int W = AUX_LANES * V;           // strip width
  constexpr int SLOTS = AUX_THREADS / AUX_LANES;
  const T* __restrict__ X = static_cast<const T*>(c.X);
  const int slot = threadIdx.x / AUX_LANES, ln = threadIdx.x % AUX_LANES;
  {   // blk -> strip: workgroup ids are dealt round-robin to the 8 XCDs (job ranges start at multiples of 8)
    const int xcd = blk & 7, t = blk >> 3;
    blk = (((t >> 2) * 8 + xcd) << 2) + (t & 3);
  }
  if (blk * W >= c.N) return;     // padding of the range (whole workgroup)
  const int col0 = blk * W + ln * V;
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.f;
  const bool vec_ok = (c.ldx % V == 0) && ((reinterpret_cast<uintptr_t>(X) & 15u) == 0) && col0 + V <= c.N;
  if (vec_ok) {
    for (int r0 = slot; r0 < c.M; r0 += 8 * SLOTS) {
      uint4 u[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int r = r0 + q * SLOTS;
        u[q] = r < c.M ? *reinterpret_cast<const uint4*>(X + static_cast<long long>(r) * c.ldx + col0) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        if (sizeof(T) == 2) {
          const uint32_t w[4] = {u[q].x, u[q].y, u[q].z, u[q].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[(2 * i) % V] += __uint_as_float(w[i] << 16);
            acc[(2 * i + 1) % V] += __uint_as_float(w[i] & 0xffff0000u);
          }
        } else {
          acc[0] += __uint_as_float(u[q].x); acc[1 % V] += __uint_as_float(u[q].y);
          acc[2 % V] += __uint_as_float(u[q].z); acc[3 % V] += __uint_as_float(u[q].w);
        }
      }
    }
  } else {
    for (int r = slot; r < c.M; r += SLOTS)
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (col0 + i < c.N) acc[i] += load_f32<T>(X + static_cast<long long>(r) * c.ldx + col0 + i);
  }
#pragma unroll
  for (int i = 0; i < V; ++i) lds[slot * (W + 1) + ln * V + i] = acc[i];
  __syncthreads();
  // W columns x 64 groups of SLOTS / 64 slots, then the 64 group sums by one wavefront per column
  constexpr int GROUPS = 64, PER = SLOTS / GROUPS;
  float part = 0.f;
  const int colw = threadIdx.x / GROUPS, grp = threadIdx.x % GROUPS;     // AUX_THREADS == W * 64 for bf16
  if (colw < W) {
    for (int k = 0; k < PER; ++k) part += lds[(grp * PER + k) * (W + 1) + colw];
  }
  part = wave_sum(part);     // lanes of a wavefront = the 64 groups of one column; fixed order
  if (colw < W && grp == 0) {
    const int col = blk * W + colw;
    if (col < c.N) store_f32<TO>(static_cast<TO*>(c.out) + col, part);
  }
}

__global__ __launch_bounds__(AUX_THREADS) void bwd_aux_kernel(const AuxBatchDev a) {
  __shared__ float lds[(AUX_THREADS / AUX_LANES) * (AUX_LANES * 8 + 1)];
  const int blk = blockIdx.x;
  int j = 0;
  while (blk >= a.blk_begin[j + 1]) ++j;     // blk_begin[n_jobs] = grid size
  const int local = blk - a.blk_begin[j];
  if (j < a.b.n_colsum) {
    const AuxColsum& c = a.b.colsum[j];
    const int od = c.out_dtype ? c.out_dtype : c.dtype;
    if (c.dtype == ECOSPA_BF16) aux_colsum_block<bf16_t, bf16_t>(c, local, lds);
    else if (od == ECOSPA_BF16) aux_colsum_block<float, bf16_t>(c, local, lds);
    else aux_colsum_block<float, float>(c, local, lds);
  } else {
    const GemmDesc& d = a.b.reduce[j - a.b.n_colsum];
    if (d.dtype == ECOSPA_BF16) aux_reduce_block<bf16_t>(d, local);
    else aux_reduce_block<float>(d, local);
  }
}

int ecospa_aux_launch(ecospa_ctx* ctx, const AuxBatch& b) {
  if (b.n_reduce < 0 || b.n_reduce > AUX_MAX_JOBS || b.n_colsum < 0 || b.n_colsum > AUX_MAX_JOBS) return ECOSPA_ERR_SHAPE;
  AuxBatchDev a;
  memset(&a, 0, sizeof(a));
  a.b = b;
  long long blk = 0;
  int j = 0;
  for (int i = 0; i < b.n_colsum; ++i, ++j) {
    const AuxColsum& c = b.colsum[i];
    if (!c.X || !c.out) return ECOSPA_ERR_NULL;
    if (!dtype_ok(c.dtype) || c.M < 1 || c.N < 1) return ECOSPA_ERR_SHAPE;
    const int line = 4 * AUX_LANES * (c.dtype == ECOSPA_BF16 ? 8 : 4);   // columns of four strips
    a.blk_begin[j] = static_cast<int>(blk);                               // a multiple of 32: starts on XCD 0
    blk += ((c.N + line - 1) / line + 7) / 8 * 32;                        // 8 lines x 4 strips at a time
  }
  for (int i = 0; i < b.n_reduce; ++i, ++j) {
    const GemmDesc& d = b.reduce[i];
    if (d.splits <= 1 || !d.partial || (!d.epi.c && d.epi.kind != EPI_SWIGLU)) return ECOSPA_ERR_NULL;
    if (!dtype_ok(d.dtype)) return ECOSPA_ERR_DTYPE;
    a.blk_begin[j] = static_cast<int>(blk);
    const long long items = static_cast<long long>(d.M) * d.N / (d.dtype == ECOSPA_BF16 ? 8 : 1);
    blk += (items + AUX_THREADS - 1) / AUX_THREADS;
  }
  if (j == 0) return ECOSPA_OK;
  if (blk > (1ll << 30)) return ECOSPA_ERR_SHAPE;
  for (int q = j; q <= 2 * AUX_MAX_JOBS; ++q) a.blk_begin[q] = static_cast<int>(blk);
  hipLaunchKernelGGL(bwd_aux_kernel, dim3(static_cast<unsigned>(blk)), dim3(AUX_THREADS), 0, ctx->stream, a);
  ECOSPA_CHECK_LAUNCH(ctx, "bwd_aux_kernel");
  return ECOSPA_OK;
}
