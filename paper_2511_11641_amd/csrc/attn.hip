// Attention block on compacted heads (paper Eq. 1-2 rewritten per head as Eq. 4; rotary form
// Eq. 6): projections and W_o run on the GEMM kernels, this file holds the attention core
// (tiled over keys, never materialising the L x L matrix) and its backward pass, all on
// v_mfma_f32_32x32x16_bf16.
//
// Layout trick used by all three kernels: the score tile is computed "transposed" so that the
// softmax row index sits in the lane (column of the MFMA result) and the contraction index of
// the NEXT matmul sits in the accumulator registers.  Eight consecutive accumulator registers
// then are, after conversion to bf16, directly the B operand of that next matmul - the
// probabilities never go through LDS.  The matching A operand is read from a transposed LDS
// copy of V (or K, Q, dO) with the same register->index permutation:
//   registers r = 8*(s%2) .. +7 of 32-row tile s/2, lane half hh  <->  rows 16*s + 8*(j/4) + 4*hh + j%4.
// Determinism: dQ and dK/dV come from two kernels (one loops over keys, one over queries), so no
// floating-point atomics are needed.
#include "block.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define LOG2E 1.4426950408889634f
#define LN2 0.6931471805599453f
#define RESCALE_LOG2 8.0f   // forward softmax: growth of a row maximum (in binades) that triggers a rescale

struct AttnArgs {
  const bf16_t* qkv;   // [T, nqkv]: Q | K | V column blocks, head-major inside each
  long long ld_qkv;
  bf16_t* o;           // [T, h*kp_vo]
  const bf16_t* d_o;   // backward: gradient of o
  long long ld_o;
  float* lse;          // [B, h, L] natural-log sum-exp of the scaled, masked scores
  float* delta;        // [B, h, L] rowsum(dO * O)
  bf16_t* dqkv;        // backward output, same layout as qkv
  int B, L, h, kp_qk, kp_vo, causal;
  float scale;
  int h_kv;            // key/value heads (grouped-query attention, Eq. 5: query head i uses key/value head i / qpk)
  int qpk;             // query heads per key/value head, h / h_kv (1: multi-head attention)
  const float *rope_cos, *rope_sin;   // backward: tables [h_kv, L, kp_qk / 2] of the rotary form (Eq. 6), or null - the gradients
                                      // of the rotated Q and K are turned back (angle -t theta) as they are written
};
// Column offsets inside a row of the qkv buffer: Q heads, then the key heads, then the value heads.
__device__ __forceinline__ int k_col(const AttnArgs& a, int kv_head) { return a.h * a.kp_qk + kv_head * a.kp_qk; }
__device__ __forceinline__ int v_col(const AttnArgs& a, int kv_head) { return (a.h + a.h_kv) * a.kp_qk + kv_head * a.kp_vo; }

// ---------------------------------------------------------------------------------------------
// LDS tile addressing (element offsets).  Tiles are [rows][D] (D = 32, 64 or 128 dims, 16-byte chunks
// XOR-swizzled by row) and are read two ways:
//   frag_nat: ds_read_b128, lane (l32, hh) takes chunk 2s+hh of row l32 - sixteen consecutive rows
//             of one chunk column must fall on sixteen different 16-byte bank groups;
//   frag_trn: ds_read_b64_tr_b16, a 16-lane group takes 4 rows x 16 dims - the four rows must fall
//             on four different 64-byte bank groups.
// D = 64 (128-byte rows): swizzle (row % 8) ^ bit 3 of row ^ (bit 1 of row) << 2 serves both;
// D = 32 (64-byte rows, a transposing read covers whole rows): (row / 4) % 4;
// D = 128 (256-byte rows): the swizzle of D = 64 on the low three bits of the chunk number - a bijection of the row's
// sixteen chunks that leaves two-way conflicts on the direct reads (the 128-wide kernels are the rare, wide shapes).
// ---------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) bf16_t lds_bf16_t;
typedef short shortx4_t __attribute__((ext_vector_type(4)));
typedef short shortx8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) shortx4_t lds_shortx4_t;

template <int D>
__device__ __forceinline__ int nat_swz(int row) {
  return D >= 64 ? ((row & 7) ^ ((row >> 3) & 1) ^ (((row >> 1) & 1) << 2)) : ((row >> 2) & 3);
}
template <int D>
__device__ __forceinline__ int nat_off(int row, int chunk) {   // [rows][D], D in {32, 64, 128}
  return row * D + ((chunk ^ nat_swz<D>(row)) << 3);
}
template <int D>
__device__ __forceinline__ bf16x8_t frag_nat(const bf16_t* tile, int row, int s, int hh) {
  return *reinterpret_cast<const bf16x8_t*>(tile + nat_off<D>(row, 2 * s + hh));
}
// Operand taken transposed from a natural tile with ds_read_b64_tr_b16: lane (l32, hh) gets dim
// dim0 + l32 of the rows {16s + 4hh + 0..3, 16s + 8 + 4hh + 0..3} - the order in which acc_to_frag()
// lays out the contraction index.  Within a 16-lane group, lane i addresses (row i / 4, dims
// 4 * (i % 4) ..+3) and receives dim i of the group's four rows.
// The reads are issued through inline assembly: the compiler would hold the builtin form back until
// every direct global->LDS load in flight has landed (it cannot tell the stream buffers apart), which
// would undo the prefetch.  trn_issue() starts the two reads of a fragment, trn_wait() waits for all LDS
// reads issued so far, trn_frag() then hands a fragment over (its empty asm statements keep the uses
// behind the wait).
struct TrnRegs { shortx4_t lo, hi; };
template <int D>
__device__ __forceinline__ void trn_issue(TrnRegs& r, const bf16_t* tile, int dim0, int s) {
  const int lane = threadIdx.x & 63, g = lane >> 4, i = lane & 15;
  const int row = 16 * s + 4 * (g >> 1) + (i >> 2);
  const int col = dim0 + 16 * (g & 1) + 4 * (i & 3);
  const lds_bf16_t* t3 = (const lds_bf16_t*)tile;
  const unsigned a0 = static_cast<unsigned>(reinterpret_cast<uintptr_t>(t3 + nat_off<D>(row, col >> 3) + (col & 7)));
  const unsigned a1 = static_cast<unsigned>(reinterpret_cast<uintptr_t>(t3 + nat_off<D>(row + 8, col >> 3) + (col & 7)));
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r.lo) : "v"(a0) : "memory");
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r.hi) : "v"(a1) : "memory");
}
__device__ __forceinline__ void trn_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ bf16x8_t trn_frag(TrnRegs& r) {
  asm volatile("" : "+v"(r.lo), "+v"(r.hi));
  const shortx8_t v = {r.lo[0], r.lo[1], r.lo[2], r.lo[3], r.hi[0], r.hi[1], r.hi[2], r.hi[3]};
  return __builtin_bit_cast(bf16x8_t, v);
}

// Stream of [64 rows][D] tiles of a row-major matrix into LDS with direct global->LDS loads (no
// registers in between): each of the workgroup's 4 wavefronts moves PER kilobytes per tile; an
// instruction fills RPI consecutive tile rows, lane by lane, so the swizzle is applied on the
// global side (the lane that owns physical chunk pc of a row fetches the logical chunk that maps
// there).  Rows beyond the end of the sequence repeat its last row and dims beyond the kept width
// repeat the last kept chunk: finite stand-ins that the callers keep out of every result (masked
// scores; a zero-padded partner operand; output columns that are never stored).
template <int D>
struct TileStream {
  static constexpr int CPR = D / 8, RPI = 64 / CPR, PER = (64 / RPI) / 4;
  const bf16_t* base;
  long long ld;
  const bf16_t* p0[PER];   // this lane's source in a tile that starts at row 0
  int row[PER], col[PER];
  __device__ __forceinline__ void init(const bf16_t* b, long long l, int kp) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    base = b;
    ld = l;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int r = (wave * PER + i) * RPI + lane / CPR, pc = lane % CPR;
      row[i] = r;
      col[i] = min((pc ^ nat_swz<D>(r)) * 8, kp - 8);
      p0[i] = b + r * l + col[i];
    }
  }
  // rows g0 .. g0 + 63 of the matrix, of which the first rows_valid (>= 1) exist
  __device__ __forceinline__ void issue(bf16_t* tile, long long g0, int rows_valid) const {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (rows_valid >= 64) {      // uniform: one scalar product, one add per load
      const long long adv = g0 * ld;
#pragma unroll
      for (int i = 0; i < PER; ++i)
        __builtin_amdgcn_global_load_lds(p0[i] + adv, (lds_bf16_t*)tile + (wave * PER + i) * 512, 16, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const bf16_t* src = base + (g0 + min(row[i], rows_valid - 1)) * ld + col[i];
        __builtin_amdgcn_global_load_lds(src, (lds_bf16_t*)tile + (wave * PER + i) * 512, 16, 0, 0);
      }
    }
  }
};
// own direct loads have landed (then a barrier tells the same of everyone's)
__device__ __forceinline__ void stream_wait() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0);   // vmcnt(0) lgkmcnt(0) expcnt(0)
  asm volatile("" ::: "memory");
}
// accumulator registers 8*half .. 8*half+7 as a bf16 B operand
__device__ __forceinline__ bf16x8_t acc_to_frag(const floatx16& a, int half) {
  floatx8 f;
#pragma unroll
  for (int i = 0; i < 8; ++i) f[i] = a[8 * half + i];
  return __builtin_convertvector(f, bf16x8_t);
}

// The MFMA fragments of a lane's own row of a row-major matrix, straight from memory: fragment s of lane (l32, hh) is
// the 16-byte chunk 2s + hh of row l32 of the wavefront's 32 rows - what frag_nat() would read from an LDS copy of
// the tile, without the copy and its barrier.  Unconditional loads from clamped (always valid) addresses; rows beyond
// the sequence end (`row_ok` false; `row` is then any valid row) and dims beyond the kept width come out as zeros.
template <int D>
__device__ __forceinline__ void own_row_load(u32x4 (&v)[D / 16], const bf16_t* __restrict__ base, long long ld, long long row,
                                             int kp, int hh) {
#pragma unroll
  for (int s = 0; s < D / 16; ++s) v[s] = *reinterpret_cast<const u32x4*>(base + row * ld + min(16 * s + 8 * hh, kp - 8));
}
template <int D>
__device__ __forceinline__ void own_row_frags(bf16x8_t (&f)[D / 16], const u32x4 (&v)[D / 16], bool row_ok, int kp, int hh) {
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    f[s] = __builtin_bit_cast(bf16x8_t, (row_ok && 16 * s + 8 * hh < kp) ? v[s] : u32x4{0u, 0u, 0u, 0u});
}

// Write a [ROWS][D] natural LDS tile to global rows row0.. (only rows < rows_valid, dims < kp).
template <int D>
__device__ __forceinline__ void tile_to_global(const bf16_t* tile, int rows, bf16_t* __restrict__ base, long long ld,
                                               long long row0, int rows_valid, int kp) {
  for (int c = threadIdx.x; c < rows * (D / 8); c += 256) {
    const int r = c / (D / 8), ch = c % (D / 8);
    if (r < rows_valid && ch * 8 < kp)
      *reinterpret_cast<u32x4*>(base + (row0 + r) * ld + ch * 8) = *reinterpret_cast<const u32x4*>(tile + nat_off<D>(r, ch));
  }
}
// The same for gradients of rotated queries or keys: every adjacent pair (2i, 2i+1) of token t is turned by -angle(t, i)
// on the way out (Eq. 6: the forward pass turned Q and K by +angle).  tab: the head's rows of the tables, [L][kp / 2];
// pos0: position in the sequence of tile row 0.
template <int D>
__device__ __forceinline__ void tile_to_global_unrope(const bf16_t* tile, int rows, bf16_t* __restrict__ base, long long ld,
                                                      long long row0, int rows_valid, int kp, const float* __restrict__ cs,
                                                      const float* __restrict__ sn, int pos0) {
  for (int c = threadIdx.x; c < rows * (D / 8); c += 256) {
    const int r = c / (D / 8), ch = c % (D / 8);
    if (r < rows_valid && ch * 8 < kp) {
      const u32x4 x = *reinterpret_cast<const u32x4*>(tile + nat_off<D>(r, ch));
      const long long tab = static_cast<long long>(pos0 + r) * (kp / 2) + ch * 4;
      const float4 c4 = *reinterpret_cast<const float4*>(cs + tab);
      const float4 s4 = *reinterpret_cast<const float4*>(sn + tab);
      const float cv[4] = {c4.x, c4.y, c4.z, c4.w}, sv[4] = {s4.x, s4.y, s4.z, s4.w};
      const uint32_t w[4] = {x.x, x.y, x.z, x.w};
      typedef float floatx8 __attribute__((ext_vector_type(8)));
      floatx8 y;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x0 = __uint_as_float(w[i] << 16), x1 = __uint_as_float(w[i] & 0xffff0000u);
        y[2 * i] = x0 * cv[i] + x1 * sv[i];
        y[2 * i + 1] = x1 * cv[i] - x0 * sv[i];
      }
      const bf16x8_t b = __builtin_convertvector(y, bf16x8_t);
      *reinterpret_cast<u32x4*>(base + (row0 + r) * ld + ch * 8) = __builtin_bit_cast(u32x4, b);
    }
  }
}
// Park a transposed accumulator (column = token lane%32, rows = dims) in a natural LDS tile.
template <int D>
__device__ __forceinline__ void acc_to_tile(bf16_t* tile, int tok_row, int dim_tile, const floatx16& a, float mul,
                                            int hh) {
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    floatx4 f;
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = a[4 * g + i] * mul;
    const bf16x4_t b = __builtin_convertvector(f, bf16x4_t);
    *reinterpret_cast<bf16x4_t*>(tile + nat_off<D>(tok_row, dim_tile * 4 + g) + 4 * hh) = b;
  }
}

// Work item of a workgroup: (128-row tile, head, batch element) from a 1-D grid of n_tiles * h * B.
// With a causal mask the work of a tile grows linearly with its index (query tiles) or falls with it
// (key tiles), all workgroups of the layer's shapes are resident at once, and the hardware deals
// workgroups round-robin to the 8 XCDs - so a mapping with the tile index fastest would hand one
// XCD all the heavy tiles.  Here tiles are taken in zigzag order (last, first, last-1, second, ...:
// any run of 2 or 4 neighbours carries average work), all tiles of one (head, batch element) go to
// one XCD (its L2 then holds that head's K and V for all of them), and the starting point of the
// zigzag moves on every 32 workgroups of an XCD, so that both neighbouring workgroups and workgroups
// 32 apart - the likely co-residents of a compute unit - differ in weight.
__device__ __forceinline__ void attn_work_item(const AttnArgs& a, int heads, int n_tiles, int& tile, int& head, int& b) {
  const int id = blockIdx.x, n_bh = heads * a.B;
  int bh, z;
  if ((n_bh & 7) == 0) {
    const int x = id & 7, l = id >> 3;            // XCD, index inside the XCD's share
    const int blk = l / n_tiles, r = l - blk * n_tiles;
    z = (r + (blk * n_tiles) / 32) % n_tiles;
    bh = x * (n_bh >> 3) + blk;
  } else {
    bh = id / n_tiles;
    z = id - bh * n_tiles;
  }
  tile = (z & 1) ? (z >> 1) : n_tiles - 1 - (z >> 1);
  head = bh % heads;
  b = bh / heads;
}

// Wavefronts per SIMD the register allocation aims at: the narrow (32, 32) heads of a half-kept
// layer need few registers, and more resident workgroups hide their barrier and LDS latencies.
#define ATTN_WPE(DQ, DV, narrow) ((DQ) + (DV) <= 64 ? (narrow) : ((DQ) > 64 || (DV) > 64 ? 1 : 2))

// ---------------------------------------------------------------------------------------------
// forward: one workgroup per (128 queries, head, batch); 4 wavefronts x 32 queries
// ---------------------------------------------------------------------------------------------
template <int DQ, int DV>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(ATTN_WPE(DQ, DV, 4), ATTN_WPE(DQ, DV, 4))))
void attn_fwd_kernel(const AttnArgs a) {
  constexpr int DMAX = DQ > DV ? DQ : DV;
  // One LDS object per kernel, carved by hand: with several, the compiler tags every LDS access with the
  // object it touches and then holds each read of a stream buffer back until the direct loads into the
  // other half of that buffer have landed.
  extern __shared__ __attribute__((aligned(16))) bf16_t lds_all[];     // attn_lds_bytes<DQ, DV>(0)
  bf16_t* const Qs = lds_all;                                      // O staging tile
  bf16_t* const Ks0 = Qs + 128 * DMAX;        // [2][64 * DQ]
  bf16_t* const Vs0 = Ks0 + 2 * 64 * DQ;      // [2][64 * DV]
#define Ks(buf) (Ks0 + (buf) * (64 * DQ))
#define Vs(buf) (Vs0 + (buf) * (64 * DV))
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hh = lane >> 5, l32 = lane & 31;
  int qt, head, b;
  attn_work_item(a, a.h, (a.L + 127) / 128, qt, head, b);
  const int q0 = qt * 128;
  const long long tok0 = static_cast<long long>(b) * a.L;
  const bf16_t* Qg = a.qkv + head * a.kp_qk;

  // key/value tiles stream straight into LDS, one tile ahead of the one being used
  TileStream<DQ> ks;
  TileStream<DV> vs;
  ks.init(a.qkv + k_col(a, head / a.qpk), a.ld_qkv, a.kp_qk);
  vs.init(a.qkv + v_col(a, head / a.qpk), a.ld_qkv, a.kp_vo);
  ks.issue(Ks(0), tok0, a.L);
  vs.issue(Vs(0), tok0, a.L);

  // Q: every lane takes the fragments of its own query row straight from memory (rows and dims outside are zeroed)
  const int kv_end = a.causal ? min(a.L, q0 + 128) : a.L;
  const int n_kv = (kv_end + 63) / 64;
  bf16x8_t qf[DQ / 16];
  {
    const int qrow = q0 + wave * 32 + l32;
    u32x4 qraw[DQ / 16];
    own_row_load<DQ>(qraw, Qg, a.ld_qkv, tok0 + min(qrow, a.L - 1), a.kp_qk, hh);
    own_row_frags<DQ>(qf, qraw, qrow < a.L, a.kp_qk, hh);
  }

  // oacc: O^T (dims x queries); lacc: the softmax denominators, accumulated by the matrix unit from
  // the same rounded probabilities as the numerator (an all-ones operand in place of V^T, so every
  // row of lacc holds the row sums)
  floatx16 oacc[DV / 32], lacc;
#pragma unroll
  for (int u = 0; u < DV / 32; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[u][r] = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) lacc[r] = 0.f;
  bf16x8_t ones;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones[i] = static_cast<__bf16>(1.0f);
  float m_run = -INFINITY;
  const float sc = a.scale * LOG2E;
  const int qw0 = q0 + wave * 32, q_idx = qw0 + l32;

  for (int j = 0; j < n_kv; ++j) {
    const int cur = j & 1, kv0 = j * 64;
    stream_wait();
    __syncthreads();    // tile j is in LDS; every wavefront is done with tile j-1, whose buffer is refilled now
    if (j + 1 < n_kv) {
      ks.issue(Ks(cur ^ 1), tok0 + kv0 + 64, a.L - kv0 - 64);
      vs.issue(Vs(cur ^ 1), tok0 + kv0 + 64, a.L - kv0 - 64);
    }
    if (a.causal && kv0 > qw0 + 31) continue;   // no query of this wavefront sees the tile
    floatx16 sacc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[t][r] = 0.f;
#pragma unroll
      for (int s = 0; s < DQ / 16; ++s)
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat<DQ>(Ks(cur), t * 32 + l32, s, hh), qf[s], sacc[t], 0, 0, 0);
    }
    // Softmax on raw scores: the scale is folded into the exponent's FMA.  Masking is a
    // wave-uniform special case (tiles on the diagonal or at the end of the sequence) done
    // with selects, never with divergent branches.
    if ((a.causal && kv0 + 63 > qw0) || (kv0 + 64 > a.L)) {
      const int lim = a.causal ? min(q_idx, a.L - 1) : a.L - 1;   // last visible key of this query
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + t * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
          sacc[t][r] = key > lim ? -INFINITY : sacc[t][r];
        }
    }
    float mx = sacc[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // Running reference maximum (raw, unscaled).  It only has to keep the exponentials in range, so it
    // moves - and the accumulators are rescaled - only when some query's maximum has grown by more than
    // RESCALE_LOG2 binades since the reference was set (wave-uniform test); until then probabilities
    // up to 2^RESCALE_LOG2 are accumulated against the old reference.
    const float m_new = fmaxf(m_run, mx);
    if (__builtin_amdgcn_ballot_w64((m_new - m_run) * sc > RESCALE_LOG2 || (m_new > m_run && m_run == -INFINITY)) != 0ull) {
      const float msc_new = (m_new == -INFINITY ? 0.f : m_new) * sc;
      const float alpha = __builtin_amdgcn_exp2f(__builtin_fmaf(m_run, sc, -msc_new));
#pragma unroll
      for (int r = 0; r < 16; ++r) lacc[r] *= alpha;
#pragma unroll
      for (int u = 0; u < DV / 32; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[u][r] *= alpha;
      m_run = m_new;
    }
    const float msc = (m_run == -INFINITY ? 0.f : m_run) * sc;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[t][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[t][r], sc, -msc));
    TrnRegs vr[4][DV / 32];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int u = 0; u < DV / 32; ++u) trn_issue<DV>(vr[s][u], Vs(cur), u * 32, s);
    trn_wait();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const bf16x8_t pf = acc_to_frag(sacc[s >> 1], s & 1);
      lacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, pf, lacc, 0, 0, 0);
#pragma unroll
      for (int u = 0; u < DV / 32; ++u)
        oacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trn_frag(vr[s][u]), pf, oacc[u], 0, 0, 0);
    }
  }
  const float l_tot = lacc[0];
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (hh == 0 && q_idx < a.L)
    a.lse[(static_cast<long long>(b) * a.h + head) * a.L + q_idx] = (m_run * sc + __log2f(l_tot)) * LN2;
  // O staging
#pragma unroll
  for (int u = 0; u < DV / 32; ++u) acc_to_tile<DV>(Qs, wave * 32 + l32, u, oacc[u], inv, hh);
  __syncthreads();
  tile_to_global<DV>(Qs, 128, a.o + head * a.kp_vo, a.ld_o, tok0 + q0, a.L - q0, a.kp_vo);
#undef Ks
#undef Vs
}

// ---------------------------------------------------------------------------------------------
// backward, dQ: one workgroup per (128 queries, head, batch), loop over key tiles
//   S^T = K Q^T, dP^T = V dO^T, dS^T = P^T * (dP^T - delta), dQ^T += K^T dS^T
// ---------------------------------------------------------------------------------------------
template <int DQ, int DV>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(ATTN_WPE(DQ, DV, 4), ATTN_WPE(DQ, DV, 4))))
void attn_bwd_dq_kernel(const AttnArgs a) {
  constexpr int DMAX = DQ > DV ? DQ : DV;
  extern __shared__ __attribute__((aligned(16))) bf16_t lds_all[];     // one object: see attn_fwd_kernel; attn_lds_bytes<DQ, DV>(1)
  bf16_t* const Qs = lds_all;                                      // dQ staging tile
  bf16_t* const Ks0 = Qs + 128 * DMAX;        // [2][64 * DQ]
  bf16_t* const Vs0 = Ks0 + 2 * 64 * DQ;      // [2][64 * DV]
#define Ks(buf) (Ks0 + (buf) * (64 * DQ))
#define Vs(buf) (Vs0 + (buf) * (64 * DV))
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hh = lane >> 5, l32 = lane & 31;
  int qt, head, b;
  attn_work_item(a, a.h, (a.L + 127) / 128, qt, head, b);
  const int q0 = qt * 128;
  const long long tok0 = static_cast<long long>(b) * a.L;
  const bf16_t* Qg = a.qkv + head * a.kp_qk;
  const bf16_t* dOg = a.d_o + head * a.kp_vo;

  // key/value tiles stream straight into LDS, one tile ahead of the one being used
  TileStream<DQ> ks;
  TileStream<DV> vs;
  ks.init(a.qkv + k_col(a, head / a.qpk), a.ld_qkv, a.kp_qk);
  vs.init(a.qkv + v_col(a, head / a.qpk), a.ld_qkv, a.kp_vo);
  ks.issue(Ks(0), tok0, a.L);
  vs.issue(Vs(0), tok0, a.L);

  // Nothing of the prologue goes through LDS: every lane takes the fragments of its own query row of Q and of dO, its
  // pieces of the O row and the row's log-sum-exp straight from memory, all requested before the first wait.
  const int qw0 = q0 + wave * 32, q_idx = qw0 + l32;
  const long long stat = (static_cast<long long>(b) * a.h + head) * a.L;
  const long long qrow = tok0 + min(q_idx, a.L - 1);
  bf16x8_t qf[DQ / 16], dof[DV / 16];
  u32x4 qraw[DQ / 16], doraw[DV / 16], ov[DV / 16];
  own_row_load<DQ>(qraw, Qg, a.ld_qkv, qrow, a.kp_qk, hh);
  own_row_load<DV>(doraw, dOg, a.ld_o, qrow, a.kp_vo, hh);
  own_row_load<DV>(ov, a.o + head * a.kp_vo, a.ld_o, qrow, a.kp_vo, hh);
  const float lse_raw = a.lse[stat + min(q_idx, a.L - 1)];
  own_row_frags<DQ>(qf, qraw, q_idx < a.L, a.kp_qk, hh);
  own_row_frags<DV>(dof, doraw, q_idx < a.L, a.kp_vo, hh);
  const float lse2 = q_idx < a.L ? lse_raw * LOG2E : 0.f;
  // delta = rowsum(dO * O) of this lane's query from its half of the two rows; the other half sits in lane ^ 32.  The
  // kernel over key tiles reads the sums from memory.  (dO is zero beyond the kept width, so O's stand-in there drops out.)
  float dlt = 0.f;
  {
#pragma unroll
    for (int s = 0; s < DV / 16; ++s) {
      const u32x4 gv = __builtin_bit_cast(u32x4, dof[s]);
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        part += __uint_as_float(ov[s][i] << 16) * __uint_as_float(gv[i] << 16);
        part += __uint_as_float(ov[s][i] & 0xffff0000u) * __uint_as_float(gv[i] & 0xffff0000u);
      }
      dlt += 16 * s + 8 * hh < a.kp_vo ? part : 0.f;
    }
    dlt += __shfl_xor(dlt, 32, 64);
    if (hh == 0 && q_idx < a.L) a.delta[stat + q_idx] = dlt;
  }
  const float sc = a.scale * LOG2E;

  floatx16 dq[DQ / 32];
#pragma unroll
  for (int u = 0; u < DQ / 32; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[u][r] = 0.f;

  const int kv_end = a.causal ? min(a.L, q0 + 128) : a.L;
  const int n_kv = (kv_end + 63) / 64;
  for (int j = 0; j < n_kv; ++j) {
    const int cur = j & 1, kv0 = j * 64;
    stream_wait();
    __syncthreads();    // tile j is in LDS; every wavefront is done with tile j-1, whose buffer is refilled now
    if (j + 1 < n_kv) {
      ks.issue(Ks(cur ^ 1), tok0 + kv0 + 64, a.L - kv0 - 64);
      vs.issue(Vs(cur ^ 1), tok0 + kv0 + 64, a.L - kv0 - 64);
    }
    if (a.causal && kv0 > qw0 + 31) continue;
    const bool need_mask = (a.causal && kv0 + 63 > qw0) || (kv0 + 64 > a.L);
    const int lim = a.causal ? min(q_idx, a.L - 1) : a.L - 1;       // last visible key of this query
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      floatx16 sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
#pragma unroll
      for (int s = 0; s < DQ / 16; ++s)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat<DQ>(Ks(cur), t * 32 + l32, s, hh), qf[s], sacc, 0, 0, 0);
#pragma unroll
      for (int s = 0; s < DV / 16; ++s)
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat<DV>(Vs(cur), t * 32 + l32, s, hh), dof[s], pacc, 0, 0, 0);
      if (need_mask) {        // wave-uniform; selects only
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + t * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
          sacc[r] = key > lim ? -INFINITY : sacc[r];
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[r], sc, -lse2));
        sacc[r] = p * (pacc[r] - dlt);
      }
      TrnRegs kr[2][DQ / 32];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int u = 0; u < DQ / 32; ++u) trn_issue<DQ>(kr[s2][u], Ks(cur), u * 32, t * 2 + s2);
      trn_wait();
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8_t df = acc_to_frag(sacc, s2);
#pragma unroll
        for (int u = 0; u < DQ / 32; ++u)
          dq[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trn_frag(kr[s2][u]), df, dq[u], 0, 0, 0);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < DQ / 32; ++u) acc_to_tile<DQ>(Qs, wave * 32 + l32, u, dq[u], a.scale, hh);
  __syncthreads();
  if (a.rope_cos) {
    const long long tb = static_cast<long long>(head / a.qpk) * a.L * (a.kp_qk / 2);
    tile_to_global_unrope<DQ>(Qs, 128, a.dqkv + head * a.kp_qk, a.ld_qkv, tok0 + q0, a.L - q0, a.kp_qk, a.rope_cos + tb, a.rope_sin + tb, q0);
  } else {
    tile_to_global<DQ>(Qs, 128, a.dqkv + head * a.kp_qk, a.ld_qkv, tok0 + q0, a.L - q0, a.kp_qk);
  }
#undef Ks
#undef Vs
}

// ---------------------------------------------------------------------------------------------
// backward, dK and dV: one workgroup per (128 keys, head, batch), loop over query tiles
//   S = Q K^T, dP = dO V^T, dS = P * (dP - delta), dV^T += dO^T P, dK^T += Q^T dS
// ---------------------------------------------------------------------------------------------
template <int DQ, int DV>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(ATTN_WPE(DQ, DV, 3), ATTN_WPE(DQ, DV, 3)))) void attn_bwd_dkdv_kernel(const AttnArgs a) {
  constexpr int DMAX = DQ > DV ? DQ : DV;
  extern __shared__ __attribute__((aligned(16))) bf16_t lds_all[];     // one object: see attn_fwd_kernel; attn_lds_bytes<DQ, DV>(2)
  bf16_t* const KVs = lds_all;                                     // output staging tile
  bf16_t* const Qs0 = KVs + 128 * DMAX;       // [2][64 * DQ]
  bf16_t* const dOs0 = Qs0 + 2 * 64 * DQ;     // [2][64 * DV]
  float* const stats = reinterpret_cast<float*>(dOs0 + 2 * 64 * DV);   // [2][64] log-sum-exp, [2][64] delta
#define Qs(buf) (Qs0 + (buf) * (64 * DQ))
#define dOs(buf) (dOs0 + (buf) * (64 * DV))
#define lse_s(buf) (stats + (buf) * 64)
#define dlt_s(buf) (stats + 128 + (buf) * 64)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hh = lane >> 5, l32 = lane & 31;
  // one workgroup per (128 keys, key/value head, batch element); the query heads that share the key/value head
  // (Eq. 5) are walked one after the other, their contributions adding up in the same accumulators
  int kt, kvh, b;
  attn_work_item(a, a.h_kv, (a.L + 127) / 128, kt, kvh, b);
  const int k0 = kt * 128, head0 = kvh * a.qpk;
  const long long tok0 = static_cast<long long>(b) * a.L;
  const bf16_t* Kg = a.qkv + k_col(a, kvh);
  const bf16_t* Vg = a.qkv + v_col(a, kvh);

  // every lane takes the fragments of its own key row of K and of V straight from memory (nothing through LDS)
  bf16x8_t kf[DQ / 16], vf[DV / 16];
  {
    const int krow = k0 + wave * 32 + l32;
    u32x4 kraw[DQ / 16], vraw[DV / 16];
    own_row_load<DQ>(kraw, Kg, a.ld_qkv, tok0 + min(krow, a.L - 1), a.kp_qk, hh);
    own_row_load<DV>(vraw, Vg, a.ld_qkv, tok0 + min(krow, a.L - 1), a.kp_vo, hh);
    own_row_frags<DQ>(kf, kraw, krow < a.L, a.kp_qk, hh);
    own_row_frags<DV>(vf, vraw, krow < a.L, a.kp_vo, hh);
  }
  const int kw0 = k0 + wave * 32, key_idx = kw0 + l32;
  const float sc = a.scale * LOG2E;

  floatx16 dk[DQ / 32], dv[DV / 32];
#pragma unroll
  for (int u = 0; u < DQ / 32; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[u][r] = 0.f;
#pragma unroll
  for (int u = 0; u < DV / 32; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) dv[u][r] = 0.f;

  const int n_q = (a.L + 63) / 64;
  const int j0 = a.causal ? k0 / 64 : 0;     // first query tile that can see a key of this tile
  // Query tiles (Q and dO) stream straight into LDS, one tile ahead; the tile's 64 log-sum-exp and
  // delta values travel through a register of threads 0..127 and are parked in LDS one iteration later.
  TileStream<DQ> qs;
  TileStream<DV> ds;
  float st = 0.f;
  const int cnt = n_q - j0, n_it = cnt > 0 ? cnt * a.qpk : 0;   // iterations: query heads of the group x their query tiles
  // iteration `it` is query tile j0 + it % cnt of query head head0 + it / cnt; a new head re-aims the streams
#define KV_ISSUE(it, buf)                                                                              \
  do {                                                                                                 \
    const int hq_ = head0 + (it) / cnt, j_ = j0 + (it) % cnt;                                          \
    if ((it) % cnt == 0) {                                                                             \
      qs.init(a.qkv + hq_ * a.kp_qk, a.ld_qkv, a.kp_qk);                                               \
      ds.init(a.d_o + hq_ * a.kp_vo, a.ld_o, a.kp_vo);                                                 \
    }                                                                                                  \
    qs.issue(Qs(buf), tok0 + j_ * 64, a.L - j_ * 64);                                                  \
    ds.issue(dOs(buf), tok0 + j_ * 64, a.L - j_ * 64);                                                 \
    if (tid < 128)                                                                                     \
      st = (tid < 64 ? a.lse : a.delta)[(static_cast<long long>(b) * a.h + hq_) * a.L +                \
                                        min(j_ * 64 + (tid & 63), a.L - 1)];                           \
  } while (0)
  if (n_it > 0) KV_ISSUE(0, 0);
  for (int it = 0; it < n_it; ++it) {
    const int j = j0 + it % cnt;
    const int qb0 = j * 64, cur = it & 1;
    if (tid < 64) lse_s(cur)[tid] = st * LOG2E;
    else if (tid < 128) dlt_s(cur)[tid - 64] = st;
    stream_wait();
    __syncthreads();    // this tile is in LDS; every wavefront is done with the one before, whose buffers are refilled now
    if (it + 1 < n_it) KV_ISSUE(it + 1, cur ^ 1);
    if (a.causal && qb0 + 63 < kw0) continue;          // every query of the tile precedes this wave's keys
    const bool need_mask = (a.causal && qb0 < kw0 + 31) || (qb0 + 64 > a.L) || (kw0 + 32 > a.L);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      floatx16 sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
#pragma unroll
      for (int s = 0; s < DQ / 16; ++s)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat<DQ>(Qs(cur), t * 32 + l32, s, hh), kf[s], sacc, 0, 0, 0);
#pragma unroll
      for (int s = 0; s < DV / 16; ++s)
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat<DV>(dOs(cur), t * 32 + l32, s, hh), vf[s], pacc, 0, 0, 0);
      floatx16 pr;
      if (need_mask) {        // wave-uniform: only tiles on the diagonal or at the end of the sequence pay for the selects
        // a query sees this lane's key if key <= q (causal) and both are inside the sequence
        const int q_min = key_idx >= a.L ? 0x7fffffff : (a.causal ? key_idx : 0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int q = qb0 + t * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
          sacc[r] = (q < q_min || q >= a.L) ? -INFINITY : sacc[r];
        }
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int qrow = t * 32 + g * 8 + hh * 4;
        const float4 ls = *reinterpret_cast<const float4*>(lse_s(cur) + qrow);
        const float4 dl = *reinterpret_cast<const float4*>(dlt_s(cur) + qrow);
        const float lsv[4] = {ls.x, ls.y, ls.z, ls.w}, dlv[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = g * 4 + i;
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[r], sc, -lsv[i]));
          pr[r] = p;
          sacc[r] = p * (pacc[r] - dlv[i]);
        }
      }
      if constexpr (DQ + DV <= 192) {
        TrnRegs dor[2][DV / 32], qr[2][DQ / 32];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
          for (int u = 0; u < DV / 32; ++u) trn_issue<DV>(dor[s2][u], dOs(cur), u * 32, t * 2 + s2);
#pragma unroll
          for (int u = 0; u < DQ / 32; ++u) trn_issue<DQ>(qr[s2][u], Qs(cur), u * 32, t * 2 + s2);
        }
        trn_wait();
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8_t pf = acc_to_frag(pr, s2), df = acc_to_frag(sacc, s2);
#pragma unroll
          for (int u = 0; u < DV / 32; ++u)
            dv[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trn_frag(dor[s2][u]), pf, dv[u], 0, 0, 0);
#pragma unroll
          for (int u = 0; u < DQ / 32; ++u)
            dk[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trn_frag(qr[s2][u]), df, dk[u], 0, 0, 0);
        }
      } else {
        // two 128-wide sides: the transposed fragments of one operand and one 16-query step at a time, or they would
        // not fit the registers
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          {
            TrnRegs dor[DV / 32];
#pragma unroll
            for (int u = 0; u < DV / 32; ++u) trn_issue<DV>(dor[u], dOs(cur), u * 32, t * 2 + s2);
            trn_wait();
            const bf16x8_t pf = acc_to_frag(pr, s2);
#pragma unroll
            for (int u = 0; u < DV / 32; ++u)
              dv[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trn_frag(dor[u]), pf, dv[u], 0, 0, 0);
          }
          {
            TrnRegs qr[DQ / 32];
#pragma unroll
            for (int u = 0; u < DQ / 32; ++u) trn_issue<DQ>(qr[u], Qs(cur), u * 32, t * 2 + s2);
            trn_wait();
            const bf16x8_t df = acc_to_frag(sacc, s2);
#pragma unroll
            for (int u = 0; u < DQ / 32; ++u)
              dk[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trn_frag(qr[u]), df, dk[u], 0, 0, 0);
          }
        }
      }
    }
  }
#undef KV_ISSUE
#undef Qs
#undef dOs
#undef lse_s
#undef dlt_s
  __syncthreads();
#pragma unroll
  for (int u = 0; u < DQ / 32; ++u) acc_to_tile<DQ>(KVs, wave * 32 + l32, u, dk[u], a.scale, hh);
  __syncthreads();
  if (a.rope_cos) {
    const long long tb = static_cast<long long>(kvh) * a.L * (a.kp_qk / 2);
    tile_to_global_unrope<DQ>(KVs, 128, a.dqkv + k_col(a, kvh), a.ld_qkv, tok0 + k0, a.L - k0, a.kp_qk, a.rope_cos + tb, a.rope_sin + tb, k0);
  } else {
    tile_to_global<DQ>(KVs, 128, a.dqkv + k_col(a, kvh), a.ld_qkv, tok0 + k0, a.L - k0, a.kp_qk);
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < DV / 32; ++u) acc_to_tile<DV>(KVs, wave * 32 + l32, u, dv[u], 1.f, hh);
  __syncthreads();
  tile_to_global<DV>(KVs, 128, a.dqkv + v_col(a, kvh), a.ld_qkv, tok0 + k0, a.L - k0, a.kp_vo);
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

// The head-width combinations that are built, instantiated explicitly (left to implicit instantiation
// from the launch code, the host side of this compiler can drop some of the kernel stubs).
#define ATTN_INSTANTIATE(DQ, DV)                                              \
  template __global__ void attn_fwd_kernel<DQ, DV>(const AttnArgs);           \
  template __global__ void attn_bwd_dq_kernel<DQ, DV>(const AttnArgs);        \
  template __global__ void attn_bwd_dkdv_kernel<DQ, DV>(const AttnArgs);
ATTN_INSTANTIATE(32, 32)
ATTN_INSTANTIATE(32, 64)
ATTN_INSTANTIATE(64, 32)
ATTN_INSTANTIATE(64, 64)
ATTN_INSTANTIATE(32, 128)
ATTN_INSTANTIATE(64, 128)
ATTN_INSTANTIATE(128, 32)
ATTN_INSTANTIATE(128, 64)
ATTN_INSTANTIATE(128, 128)
#undef ATTN_INSTANTIATE

// LDS of a kernel (which: 0 forward, 1 dQ, 2 dK/dV): the staging tile, the two double-buffered stream tiles, and for
// dK/dV the row statistics of two query tiles.
template <int DQ, int DV>
static constexpr int attn_lds_bytes(int which) {
  return (128 * (DQ > DV ? DQ : DV) + 2 * 64 * DQ + 2 * 64 * DV + (which == 2 ? 512 : 0)) * 2;
}

template <int DQ, int DV>
static hipError_t launch_core(int which, const AttnArgs& a, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((a.L + 127) / 128);
  const dim3 grid(tiles * a.h * a.B), grid_kv(tiles * a.h_kv * a.B);
  const int lds = attn_lds_bytes<DQ, DV>(which);
#define ATTN_LAUNCH(kern, g)                                                                      \
  do {                                                                                            \
    static LdsAttrOnce attr_once;                                                                 \
    if (lds > 64 * 1024) {                                                                        \
      const hipError_t e = attr_once.ensure(reinterpret_cast<const void*>(kern), lds);            \
      if (e != hipSuccess) return e;                                                              \
    }                                                                                             \
    hipLaunchKernelGGL(kern, g, dim3(256), lds, st, a);                                           \
  } while (0)
  if (which == 0) ATTN_LAUNCH((attn_fwd_kernel<DQ, DV>), grid);
  else if (which == 1) ATTN_LAUNCH((attn_bwd_dq_kernel<DQ, DV>), grid);
  else ATTN_LAUNCH((attn_bwd_dkdv_kernel<DQ, DV>), grid_kv);
#undef ATTN_LAUNCH
  return hipGetLastError();
}
// Kernel width of a padded head width: 32, 64 or 128 dims (a 96-wide head runs in the 128-wide kernel: the swizzle
// of the LDS tiles wants a power of two).
static int attn_width(int kp) { return kp <= 32 ? 32 : (kp <= 64 ? 64 : 128); }
static int dispatch_core(ecospa_ctx* ctx, int which, const AttnArgs& a) {
  if (a.kp_qk > 128 || a.kp_vo > 128) return ECOSPA_ERR_SHAPE;   // rejected by the block validation before anything is launched
  const int dq = attn_width(a.kp_qk), dv = attn_width(a.kp_vo);
  hipError_t e = hipSuccess;
#define ATTN_CASE(Q, V) if (dq == Q && dv == V) e = launch_core<Q, V>(which, a, ctx->stream);
  ATTN_CASE(32, 32) else ATTN_CASE(32, 64) else ATTN_CASE(64, 32) else ATTN_CASE(64, 64)
  else ATTN_CASE(32, 128) else ATTN_CASE(64, 128) else ATTN_CASE(128, 32) else ATTN_CASE(128, 64) else ATTN_CASE(128, 128)
#undef ATTN_CASE
  if (e != hipSuccess) return hip_fail(ctx, e, "attention core kernel");
  return ECOSPA_OK;
}

static GemmDesc mk_gemm(int dtype, int M, int N, int K, const void* A, long long lda, int ta, const void* B,
                        long long ldb, int tb, void* C, long long ldc, const void* bias) {
  GemmDesc g;
  memset(&g, 0, sizeof(g));
  g.dtype = dtype; g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.trans_a = ta;
  g.B = B; g.ldb = ldb; g.trans_b = tb;
  g.splits = 1;
  g.epi.kind = EPI_STORE; g.epi.c = C; g.epi.ldc = ldc; g.epi.bias = bias;
  return g;
}

// a contraction whose rows are the tokens: K is split when there are too few of them to fill the chip
static int token_gemm(ecospa_ctx* ctx, const BlockWs& w, GemmDesc g) {
  block_token_split(g, w);
  return ecospa_gemm(ctx, g);
}

int attn_forward(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x, void* y,
                 const ecospa_saved* saved) {
  if (d.dtype != ECOSPA_BF16) return ECOSPA_ERR_DTYPE;   // the attention core is bf16 MFMA only
  const int T = d.B * d.L, nqkv = attn_nqkv(d), nvo = d.h * d.kp_vo;
  void* qkv = saved ? saved->qkv : w.qkv_tmp;
  void* o = saved ? saved->o : w.o_tmp;
  float* lse = saved ? saved->lse : w.lse_tmp;
  if (!qkv || !o || !lse) return ECOSPA_ERR_NULL;
  if (!aligned16(qkv) || !aligned16(o)) return ECOSPA_ERR_ALIGN;
  int rc;
  {
    GemmDesc g = mk_gemm(d.dtype, T, nqkv, d.d_model, x, d.d_model, 0, d.w_qkv, d.ld_wqkv, 0, qkv, nqkv, d.b_qkv);
    if (d.rope_cos) {      // the rotation of Q and K (Eq. 6) rides on the projection's epilogue
      const int hkv = attn_h_kv(d);
      g.epi.kind = EPI_ROPE;
      g.epi.rope_cos = d.rope_cos; g.epi.rope_sin = d.rope_sin;
      g.epi.rope_cols = (d.h + hkv) * d.kp_qk; g.epi.rope_kp = d.kp_qk; g.epi.rope_L = d.L;
      g.epi.rope_hq = d.h; g.epi.rope_qpk = d.h / hkv;
    }
    if ((rc = token_gemm(ctx, w, g))) return rc;
  }
  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.qkv = static_cast<const bf16_t*>(qkv); a.ld_qkv = nqkv;
  a.o = static_cast<bf16_t*>(o); a.ld_o = nvo; a.lse = lse;
  a.B = d.B; a.L = d.L; a.h = d.h; a.kp_qk = d.kp_qk; a.kp_vo = d.kp_vo; a.causal = d.causal; a.scale = d.scale;
  a.h_kv = attn_h_kv(d); a.qpk = d.h / a.h_kv;
  if ((rc = dispatch_core(ctx, 0, a))) return rc;
  return token_gemm(ctx, w, mk_gemm(d.dtype, T, d.d_model, nvo, o, nvo, 0, d.w_o, d.ld_wo, 0, y, d.d_model, d.b_o));
}

// dW_o and dW_qkv are split-K contractions whose partials are reduced, together with the two
// bias-gradient column sums, by one batched launch at the end.
static int attn_backward_body(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x,
                              const void* dy, const ecospa_saved& sv, void* dx, const ecospa_grads& gr) {
  const int T = d.B * d.L, nqkv = attn_nqkv(d), nvo = d.h * d.kp_vo, dm = d.d_model;
  int rc;
  // dW_o = dY^T O (partials),  dO = dY W_o
  GemmDesc go = mk_gemm(d.dtype, dm, nvo, T, dy, dm, 1, sv.o, nvo, 1, gr.dw_o, gr.ld_dwo, nullptr);
  go.splits = ecospa_gemm_splits(dm, nvo, T); go.partial = w.partial; go.defer_reduce = 1;
  // the bias gradients are column sums of dY and dQKV, the K-slow operands of the two weight-gradient
  // contractions: those add them up on the way
  if (gr.dw_o && gr.db_o) go.colsum = w.colsum;
  if (gr.dw_o && (rc = ecospa_gemm(ctx, go))) return rc;
  if ((rc = token_gemm(ctx, w, d.w_o_t ? mk_gemm(d.dtype, T, nvo, dm, dy, dm, 0, d.w_o_t, d.ld_wot, 0, w.d_o, nvo, nullptr)   // transposed copy [nvo, d_model]
                                     : mk_gemm(d.dtype, T, nvo, dm, dy, dm, 0, d.w_o, d.ld_wo, 1, w.d_o, nvo, nullptr))))
    return rc;

  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.qkv = static_cast<const bf16_t*>(sv.qkv); a.ld_qkv = nqkv;
  a.o = static_cast<bf16_t*>(sv.o); a.d_o = static_cast<const bf16_t*>(w.d_o); a.ld_o = nvo;
  a.lse = sv.lse; a.delta = w.delta; a.dqkv = static_cast<bf16_t*>(w.dqkv);
  a.B = d.B; a.L = d.L; a.h = d.h; a.kp_qk = d.kp_qk; a.kp_vo = d.kp_vo; a.causal = d.causal; a.scale = d.scale;
  a.h_kv = attn_h_kv(d); a.qpk = d.h / a.h_kv;
  a.rope_cos = d.rope_cos; a.rope_sin = d.rope_sin;
  // the kernel over query tiles also leaves delta = rowsum(dO * O) for the kernel over key tiles
  if ((rc = dispatch_core(ctx, 1, a))) return rc;
  if ((rc = dispatch_core(ctx, 2, a))) return rc;

  // dW_qkv = dQKV^T X (partials)
  GemmDesc gq = mk_gemm(d.dtype, nqkv, dm, T, w.dqkv, nqkv, 1, x, dm, 1, gr.dw_qkv, gr.ld_dwqkv, nullptr);
  gq.splits = ecospa_gemm_splits(nqkv, dm, T); gq.partial = w.partial2; gq.defer_reduce = 1;
  if (gr.dw_qkv && gr.db_qkv) gq.colsum = w.colsum2;
  if (gr.dw_qkv && (rc = ecospa_gemm(ctx, gq))) return rc;

  // dX = dQKV W_qkv
  if (dx && (rc = token_gemm(ctx, w, d.w_qkv_t ? mk_gemm(d.dtype, T, dm, nqkv, w.dqkv, nqkv, 0, d.w_qkv_t, d.ld_wqkvt, 0, dx, dm, nullptr)   // [d_model, nqkv]
                                             : mk_gemm(d.dtype, T, dm, nqkv, w.dqkv, nqkv, 0, d.w_qkv, d.ld_wqkv, 1, dx, dm, nullptr))))
    return rc;
  AuxBatch aux;
  memset(&aux, 0, sizeof(aux));
  if (gr.dw_o && go.splits > 1) aux.reduce[aux.n_reduce++] = go;
  if (gr.dw_qkv && gq.splits > 1) aux.reduce[aux.n_reduce++] = gq;
  if (gr.db_o) aux.colsum[aux.n_colsum++] = go.colsum ? AuxColsum{go.colsum, dm, ecospa_gemm_colsum_rows(go), dm, ECOSPA_F32, gr.db_o, d.dtype}
                                                       : AuxColsum{dy, dm, T, dm, d.dtype, gr.db_o, 0};
  if (gr.db_qkv) aux.colsum[aux.n_colsum++] = gq.colsum ? AuxColsum{gq.colsum, nqkv, ecospa_gemm_colsum_rows(gq), nqkv, ECOSPA_F32, gr.db_qkv, d.dtype}
                                                         : AuxColsum{w.dqkv, nqkv, T, nqkv, d.dtype, gr.db_qkv, 0};
  return ecospa_aux_launch(ctx, aux);
}

int attn_backward(ecospa_ctx* ctx, const ecospa_block_desc& d, const BlockWs& w, const void* x, const void* dy,
                  const ecospa_saved& sv, void* dx, const ecospa_grads& gr) {
  if (d.dtype != ECOSPA_BF16) return ECOSPA_ERR_DTYPE;
  if (!sv.qkv || !sv.o || !sv.lse) return ECOSPA_ERR_NULL;
  if (!aligned16(sv.qkv) || !aligned16(sv.o)) return ECOSPA_ERR_ALIGN;
  if (gr.dw_o && gr.ld_dwo < static_cast<long long>(d.h) * d.kp_vo) return ECOSPA_ERR_SHAPE;
  if (gr.dw_qkv && gr.ld_dwqkv < d.d_model) return ECOSPA_ERR_SHAPE;
  return attn_backward_body(ctx, d, w, x, dy, sv, dx, gr);
}
