// Software-pipelined bf16 contraction for full K slabs (the shapes of the reduced layers).
//
// Every operand tile goes global -> LDS with global_load_lds_dwordx4 (no register staging) into a
// ring of NS buffers, issued NS-1 slabs ahead and waited for with a vmcnt that leaves the younger
// slabs in flight.  K-contiguous operands sit in LDS as [rows][BK] and are read with ds_read_b128;
// K-slow operands (dY W, dY^T X) sit as [BK][rows], exactly as they lie in memory, and are read with
// ds_read_b64_tr_b16, which hands every lane four consecutive k of its own row - no transposition
// in registers.  Fragments of the next 16-wide k step are fetched while the MFMAs of the current one
// run (register double buffer); one s_barrier per slab.
//
// Bank layout: 16-byte chunks are XOR-swizzled on the GLOBAL side of the direct load (the lane that
// owns physical chunk pc of an LDS row fetches the logical chunk that maps there):
//   [rows][BK]:   pc = kc ^ f(row), f periodic in 16 rows, so the 16 rows one ds_read_b128 pass
//                 touches fall on 16 different 16-byte bank groups;
//   [BK][rows]:   pc = c ^ ((k & 3) << 2), so the four k rows that one transposing read gathers fall
//                 on four different 64-byte bank groups.
#include "gemm_lds.h"

#include <type_traits>

// Per-wave description of the direct loads of one operand tile: PER instructions per slab, each
// moving 1 KB (64 lanes x 16 bytes) to LDS offset dst[i] (elements, relative to the tile).
template <int RT, int BK, int NW, bool KSLOW>
struct TileLoads {
  static constexpr int PER = RT * BK * 2 / 1024 / NW;
  // Addresses are a wavefront-uniform base (the tile's current slab; lives in scalar registers and is advanced by
  // scalar adds) plus a per-lane byte offset that never changes: no vector instruction is spent on addressing in
  // the main loop (on this target a vector instruction of a wavefront takes issue time from its own MFMAs).
  const char* base;
  unsigned off[PER];        // this lane's byte offset of instruction i inside the slab
  long long step;           // bytes to advance per slab
  __device__ __forceinline__ void init(const bf16_t* mat, long long ld, int r0, int R, int k0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (!KSLOW) {
      constexpr int CPR = BK / 8, RPI = 64 / CPR;
      const int r = lane / CPR, pc = lane % CPR;
      base = reinterpret_cast<const char*>(mat + static_cast<long long>(r0) * ld + k0);
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int row = (wave * PER + i) * RPI + r;
        const int kc = pc ^ kc_swz<BK>(row);
        const int gr = min(r0 + row, R - 1) - r0;          // rows past the end repeat the last one
        off[i] = static_cast<unsigned>((static_cast<long long>(gr) * ld + kc * 8) * 2);
      }
      step = BK * 2;
    } else {
      constexpr int CPR = RT / 8, KPI = 64 / CPR;
      const int kl = lane / CPR, pc = lane % CPR;
      base = reinterpret_cast<const char*>(mat + static_cast<long long>(k0) * ld + r0);
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int k = (wave * PER + i) * KPI + kl;
        const int c = pc ^ ((k & 3) << 2);
        const int col = min(r0 + c * 8, R - 8) - r0;
        off[i] = static_cast<unsigned>((static_cast<long long>(k) * ld + col) * 2);
      }
      step = static_cast<long long>(BK) * ld * 2;
    }
  }
  // issue instruction i of the current slab into `tile` (LDS, start of this operand's tile); the last one of a
  // slab moves the base on.  `adv` is `step` while a further slab exists and 0 afterwards: the loads of the last slab
  // are then simply repeated (into ring buffers nobody reads any more), which keeps the main loop branch free.
  __device__ __forceinline__ void issue(int i, lds_bf16_t* tile, long long adv) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    asm volatile("" : "+v"(off[i]));   // keeps the offset a 32-bit register at the load: address = scalar base + lane offset
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const void*>(base + off[i]), tile + (wave * PER + i) * 512, 16, 0, 0);
    if (i == PER - 1) base += adv;
  }
};

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

template <int BM, int BN, int BK, int NS, int WGM, int WGN, int WPE, bool TA, bool TB>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemm_bf16_pipe_kernel(const GemmDesc d, int tiles_n, int k_chunk) {
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, FM = WTM / 32, FN = WTN / 32, KS = BK / 16;
  constexpr int STAGE = (BM + BN) * BK;
  static_assert(WTN == 64 || WTN == 96 || WTN == 128, "epilogue: 8 columns per lane, whole rows per pass");
  static_assert(KS >= 2 && KS % 2 == 0, "fragment double buffer needs an even number of k steps");
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  lds_bf16_t* lds3 = (lds_bf16_t*)lds;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // Workgroups go round-robin to the 8 XCDs, each with an L2 of its own: give every XCD a contiguous
  // range of tile ids, and order the ids in bands of GROUP_M tile rows, column by column inside a
  // band, so that the ~32 tiles an XCD works on at a time form a near-square block of C and share
  // their operand rows in that L2.
  int id, zsplit;
  const int nsplit = d.splits > 1 ? d.splits : 1;
  gemm_work_item(nsplit, id, zsplit);
  constexpr int GROUP_M = BM >= 256 ? 4 : 8;
  const int tiles_m = static_cast<int>(gridDim.x) / nsplit / tiles_n;
  const int band = id / (GROUP_M * tiles_n), in_band = id - band * (GROUP_M * tiles_n);
  const int band_rows = min(GROUP_M, tiles_m - band * GROUP_M);
  const int m0 = (band * GROUP_M + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BN;
  const int k_begin = zsplit * k_chunk;
  const int k_end = min(d.K, k_begin + k_chunk);
  const int nk = (k_end - k_begin) / BK;               // full slabs only (checked on the host)

  TileLoads<BM, BK, NW, TA> la;
  TileLoads<BN, BK, NW, TB> lb;
  la.init(static_cast<const bf16_t*>(d.A), d.lda, m0, d.M, k_begin);
  lb.init(static_cast<const bf16_t*>(d.B), d.ldb, n0, d.N, k_begin);
  constexpr int PA = TileLoads<BM, BK, NW, TA>::PER, PB = TileLoads<BN, BK, NW, TB>::PER, LPW = PA + PB;
  static_assert(LPW * (NS - 1) < 64, "vmcnt range");

  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // load instruction q (0 .. LPW-1) of the next slab to issue, into ring buffer `buf`
#define PIPE_ISSUE(q, buf, adv_a, adv_b)                                            \
  do {                                                                              \
    if ((q) < PA) la.issue((q), lds3 + (buf) * STAGE, (adv_a));                     \
    else lb.issue((q) - PA, lds3 + (buf) * STAGE + BM * BK, (adv_b));               \
  } while (0)
#define PIPE_FRAGS(set, buf, s)                                                                             \
  do {                                                                                                      \
    const bf16_t* as_ = lds + (buf) * STAGE;                                                                \
    const bf16_t* bs_ = as_ + BM * BK;                                                                      \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) fa[set][i] = read_frag<BM, BK, TA>(as_, wm * WTM + i * 32, (s)); \
    _Pragma("unroll") for (int j = 0; j < FN; ++j) fb[set][j] = read_frag<BN, BK, TB>(bs_, wn * WTN + j * 32, (s)); \
  } while (0)

  // prologue: slabs 0 .. NS-2 in flight (slabs beyond the last repeat it), slab 0 landed, its first
  // fragments in registers
#pragma unroll
  for (int p = 0; p < NS - 1; ++p) {
    const bool adv = p + 1 < nk;
#pragma unroll
    for (int q = 0; q < LPW; ++q) PIPE_ISSUE(q, p, adv ? la.step : 0, adv ? lb.step : 0);
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(waitcnt_imm((NS - 2) * LPW, false));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  bf16x8_t fa[2][FM], fb[2][FN];
  PIPE_FRAGS(0, 0, 0);

  // a short ring (NS = 2) needs its loads out at once; a long one spreads them over the slab
  constexpr int LSTEPS = NS == 2 ? 1 : KS - 1;         // k steps that issue loads
  constexpr int LPS = (LPW + LSTEPS - 1) / LSTEPS;
  static_assert(FM + FN <= FM * FN, "a fragment slot per MFMA");
  // One slab.  The ring position of slab t is a compile-time constant (the loop below walks NS slabs per round), so
  // every LDS address is a per-lane base plus an immediate: nothing is added up in vector registers per slab.
  auto slab = [&](auto buf_, int t) __attribute__((always_inline)) {
    constexpr int buf = decltype(buf_)::value;          // t % NS
    constexpr int buf_issue = buf == 0 ? NS - 1 : buf - 1;   // (t + NS - 1) % NS
    constexpr int buf_next = buf + 1 == NS ? 0 : buf + 1;
    const bool adv = t + NS < nk;                      // the slab after the one issued now exists
    const long long adv_a = adv ? la.step : 0, adv_b = adv ? lb.step : 0;
    // One k step = FM*FN MFMAs in source order; behind MFMA m go fragment m of the next k step (FM
    // A fragments, then FN B fragments) and this step's share of the global->LDS loads, fenced with
    // sched_barrier so that a wavefront that is alone on its SIMD keeps the matrix pipe fed while it
    // issues everything else.
    auto kstep = [&](auto s_) __attribute__((always_inline)) {
      constexpr int s = decltype(s_)::value;
      constexpr int cur = s & 1, nxt = cur ^ 1;
      constexpr bool last = s + 1 == KS;
      constexpr int NM = FM * FN;
      constexpr int Q0 = s * LPS, Q1 = (s + 1) * LPS < LPW ? (s + 1) * LPS : LPW;
      constexpr int NVM = (s < LSTEPS && Q1 > Q0) ? Q1 - Q0 : 0;
      constexpr int LPM = (NVM + NM - 1) / NM;          // loads per MFMA slot
      if constexpr (last) {
        // slab t+1 must have landed (own loads: vmcnt; everyone's: barrier); the barrier also tells
        // that every wavefront holds its last fragments of slab t, whose buffer is refilled next
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_imm((NS - 2) * LPW, true));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
      }
      const bf16_t* as_ = lds + (last ? buf_next : buf) * STAGE;
      const bf16_t* bs_ = as_ + BM * BK;
      constexpr int sn = last ? 0 : s + 1;
      static_for<0, NM>([&](auto m_) __attribute__((always_inline)) {
        constexpr int m = decltype(m_)::value;
        constexpr int i = m / FN, j = m % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (m < FM) fa[nxt][m] = read_frag<BM, BK, TA>(as_, wm * WTM + m * 32, sn);
        else if constexpr (m < FM + FN) fb[nxt][m - FM] = read_frag<BN, BK, TB>(bs_, wn * WTN + (m - FM) * 32, sn);
        if constexpr (LPM > 0) {
#pragma unroll
          for (int q = Q0 + m * LPM; q < Q0 + (m + 1) * LPM && q < Q1; ++q) PIPE_ISSUE(q, buf_issue, adv_a, adv_b);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    kstep(std::integral_constant<int, 0>{});
    kstep(std::integral_constant<int, 1>{});
    if constexpr (KS > 2) {
      kstep(std::integral_constant<int, 2>{});
      kstep(std::integral_constant<int, 3>{});
    }
    static_assert(KS == 2 || KS == 4, "k steps per slab");
  };
  int t = 0;
  for (; t + NS <= nk; t += NS)
    static_for<0, NS>([&](auto b_) __attribute__((always_inline)) { slab(b_, t + decltype(b_)::value); });
  static_for<0, NS - 1>([&](auto b_) __attribute__((always_inline)) {      // the last nk % NS slabs (t is a multiple of NS here)
    if (t + decltype(b_)::value < nk) slab(b_, t + decltype(b_)::value);
  });
#undef PIPE_ISSUE
#undef PIPE_FRAGS
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
  __syncthreads();   // operand buffers are idle from here on

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
  const bool lane_on = lane / LPR < RPI && n < d.N;
  const int mw = m0 + wm * WTM;
  auto park = [&](auto i_) __attribute__((always_inline)) {   // accumulators of row block i -> this wavefront's LDS slice
    constexpr int i = decltype(i_)::value;
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        cs[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * WTN + j * 32 + (lane & 31)] = acc[i][j][r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  auto unpark = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  if (split) {
    static_for<0, FM>([&](auto i_) __attribute__((always_inline)) {
      park(i_);
#pragma unroll 1
      for (int it = 0; it < NIT; ++it) {
        const int row = it * RPI + lane / LPR;
        const int m = mw + decltype(i_)::value * 32 + row;
        if (!lane_on || row >= 32 || m >= d.M) continue;
        float* p = part + static_cast<long long>(m) * d.N + n;
        *reinterpret_cast<float4*>(p) = *reinterpret_cast<const float4*>(cs + row * WTN + (lane % LPR) * 8);
        *reinterpret_cast<float4*>(p + 4) = *reinterpret_cast<const float4*>(cs + row * WTN + (lane % LPR) * 8 + 4);
      }
      unpark();
    });
    return;
  }
  // A lane keeps its 8 columns for every row: their bias is loaded once.  The epilogue kind is branched on once, here,
  // so that each kind runs straight-line code.
  float bias[8];
  const bool has_bias = lane_on && epi_bias_load(d.epi, n, bias);
  epi_dispatch(d.epi.kind, [&](auto kind_) __attribute__((always_inline)) {
    constexpr int KIND = decltype(kind_)::value;
    auto one_row = [&](int m, int row, const EpiSide sd) __attribute__((always_inline)) {
      float v[8];
      const float4 lo = *reinterpret_cast<const float4*>(cs + row * WTN + (lane % LPR) * 8);
      const float4 hi = *reinterpret_cast<const float4*>(cs + row * WTN + (lane % LPR) * 8 + 4);
      v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
      epi_apply_vec8_k<KIND>(d.epi, m, n, v, has_bias, bias, sd);
    };
    if constexpr (epi_has_side(KIND)) {
      // The inputs read beside the accumulators (saved pre-activations, rotation tables) run one 32-row block ahead:
      // those of block 0 are requested before anything else, and as soon as a row is done the same registers request
      // that row's inputs of the next block - so a load has a block's worth of work to land behind.
      EpiSide sd[NIT];
      auto request = [&](auto i_, auto it_) __attribute__((always_inline)) {
        constexpr int i = decltype(i_)::value, it = decltype(it_)::value;
        const int row = it * RPI + lane / LPR, m = mw + i * 32 + row;
        if (lane_on && row < 32 && m < d.M) epi_side_load_k<KIND>(d.epi, m, n, sd[it]);
      };
      static_for<0, NIT>([&](auto it_) __attribute__((always_inline)) { request(std::integral_constant<int, 0>{}, it_); });
      static_for<0, FM>([&](auto i_) __attribute__((always_inline)) {
        constexpr int i = decltype(i_)::value;
        park(i_);
        static_for<0, NIT>([&](auto it_) __attribute__((always_inline)) {
          constexpr int it = decltype(it_)::value;
          const int row = it * RPI + lane / LPR, m = mw + i * 32 + row;
          if (lane_on && row < 32 && m < d.M) one_row(m, row, sd[it]);
          if constexpr (i + 1 < FM) request(std::integral_constant<int, i + 1>{}, it_);
        });
        unpark();
      });
    } else {
      static_for<0, FM>([&](auto i_) __attribute__((always_inline)) {
        park(i_);
#pragma unroll 1
        for (int it = 0; it < NIT; ++it) {
          const int row = it * RPI + lane / LPR, m = mw + decltype(i_)::value * 32 + row;
          if (lane_on && row < 32 && m < d.M) one_row(m, row, EpiSide{});
        }
        unpark();
      });
    }
  });
}

// The configurations that are built.  They are instantiated explicitly: left to implicit
// instantiation from the launch code, the host side of this compiler drops some of the stubs.
#define PIPE_CONFIGS(X)          \
  X(256, 256, 64, 2, 2, 2, 1)    \
  X(256, 256, 32, 4, 2, 2, 1)    \
  X(256, 128, 64, 3, 2, 2, 1)    \
  X(128, 256, 64, 3, 2, 2, 1)    \
  X(128, 128, 64, 2, 2, 2, 2)    \
  X(256, 256, 64, 2, 2, 4, 2)    \
  X(128, 128, 32, 4, 2, 2, 2)    \
  X(256, 256, 32, 4, 2, 4, 2)    \
  X(256, 256, 32, 5, 2, 4, 2)    \
  X(256, 128, 64, 3, 4, 2, 2)    \
  X(256, 192, 64, 2, 4, 2, 2)
#define PIPE_INSTANTIATE(BM, BN, BK, NS, WGM, WGN, WPE)                                                             \
  template __global__ void gemm_bf16_pipe_kernel<BM, BN, BK, NS, WGM, WGN, WPE, false, false>(const GemmDesc, int, int); \
  template __global__ void gemm_bf16_pipe_kernel<BM, BN, BK, NS, WGM, WGN, WPE, false, true>(const GemmDesc, int, int);  \
  template __global__ void gemm_bf16_pipe_kernel<BM, BN, BK, NS, WGM, WGN, WPE, true, true>(const GemmDesc, int, int);
PIPE_CONFIGS(PIPE_INSTANTIATE)
#undef PIPE_INSTANTIATE

// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int NS, int WGM, int WGN, int WPE>
static hipError_t launch_pipe(ecospa_ctx* ctx, const GemmDesc& d, int k_chunk) {
  const int tm = (d.M + BM - 1) / BM, tn = (d.N + BN - 1) / BN;
  const int splits = d.splits > 1 ? d.splits : 1;
  const dim3 grid(tm * tn * splits), block(64 * WGM * WGN);
  const size_t operand_bytes = static_cast<size_t>(NS) * (BM + BN) * BK * sizeof(bf16_t);
  const size_t staging_bytes = static_cast<size_t>(WGM) * WGN * 32 * (BN / WGN) * 4;
  const size_t lds_bytes = operand_bytes > staging_bytes ? operand_bytes : staging_bytes;
#define LAUNCH_TT(TA, TB)                                                                                      \
  do {                                                                                                         \
    auto kern = gemm_bf16_pipe_kernel<BM, BN, BK, NS, WGM, WGN, WPE, TA, TB>;                                  \
    static LdsAttrOnce attr_once;                                                                              \
    if (lds_bytes > 64 * 1024) {                                                                               \
      hipError_t e = attr_once.ensure(reinterpret_cast<const void*>(kern), static_cast<int>(lds_bytes));       \
      if (e != hipSuccess) return e;                                                                           \
    }                                                                                                          \
    hipLaunchKernelGGL(kern, grid, block, lds_bytes, ctx->stream, d, tn, k_chunk);                             \
  } while (0)
  if (!d.trans_a && !d.trans_b) LAUNCH_TT(false, false);
  else if (!d.trans_a && d.trans_b) LAUNCH_TT(false, true);
  else LAUNCH_TT(true, true);
#undef LAUNCH_TT
  return hipGetLastError();
}

int gemm_pipe_bk(int cfg) {
  switch (cfg) {
    case 1: case 6: case 7: case 8: return 32;
    default: return 64;
  }
}

bool gemm_pipe_ok(const GemmDesc& d, int cfg, int k_chunk) {
  if (cfg < 0 || cfg >= GEMM_PIPE_CONFIGS) return false;
  if (d.trans_a && !d.trans_b) return false;           // combination not used by the layers
  if (cfg == 10 && (d.trans_a || d.trans_b)) return false;   // 192 rows do not divide into the K-slow load pattern
  const int bk = gemm_pipe_bk(cfg);
  if (d.K % bk || k_chunk % bk) return false;           // full slabs only
  return d.M >= 8 && d.N >= 8;
}

hipError_t gemm_pipe_launch(ecospa_ctx* ctx, const GemmDesc& d, int cfg, int k_chunk) {
  switch (cfg) {
    case 0: return launch_pipe<256, 256, 64, 2, 2, 2, 1>(ctx, d, k_chunk);
    case 1: return launch_pipe<256, 256, 32, 4, 2, 2, 1>(ctx, d, k_chunk);
    case 2: return launch_pipe<256, 128, 64, 3, 2, 2, 1>(ctx, d, k_chunk);
    case 3: return launch_pipe<128, 256, 64, 3, 2, 2, 1>(ctx, d, k_chunk);
    case 4: return launch_pipe<128, 128, 64, 2, 2, 2, 2>(ctx, d, k_chunk);
    case 5: return launch_pipe<256, 256, 64, 2, 2, 4, 2>(ctx, d, k_chunk);
    case 6: return launch_pipe<128, 128, 32, 4, 2, 2, 2>(ctx, d, k_chunk);
    case 7: return launch_pipe<256, 256, 32, 4, 2, 4, 2>(ctx, d, k_chunk);
    case 8: return launch_pipe<256, 256, 32, 5, 2, 4, 2>(ctx, d, k_chunk);
    case 9: return launch_pipe<256, 128, 64, 3, 4, 2, 2>(ctx, d, k_chunk);
    case 10: return launch_pipe<256, 192, 64, 2, 4, 2, 2>(ctx, d, k_chunk);
    default: return hipErrorInvalidValue;
  }
}
