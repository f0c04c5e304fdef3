// LDS operand-tile layouts and fragment reads shared by the contraction kernels (not part of the C ABI).
//
// 16-byte chunks are XOR-swizzled so that the lanes of one LDS access fall on different bank groups:
//   K-contiguous tile [rows][BK]:  pc = kc ^ f(row), f periodic in 16 rows (the 16 rows one
//                                  ds_read_b128 pass touches land on 16 different 16-byte groups);
//   K-slow tile [BK][rows]:        pc = c ^ ((k & 3) << 2) (the four k rows that one transposing
//                                  read gathers land on four different 64-byte groups); rows of 192
//                                  elements rotate the chunk index instead (see ks_off).
#pragma once
#include "gemm_epi.h"

typedef __attribute__((address_space(3))) bf16_t lds_bf16_t;
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short shortx4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) shortx4_t lds_shortx4_t;

// s_waitcnt immediates: vmcnt <= N with lgkmcnt either untouched or 0
__host__ __device__ constexpr int waitcnt_imm(int vm, bool lgkm0) {
  return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm0 ? 0 : 15) << 8);
}

// ---- K-contiguous tile [ROWS][BK] ---------------------------------------------------------------
template <int BK>
__device__ __forceinline__ int kc_swz(int row) {
  return BK == 64 ? ((row & 7) ^ ((row >> 3) & 1)) : ((row >> 2) & 3);
}
template <int BK>
__device__ __forceinline__ int kc_off(int row, int kc) {
  return row * BK + ((kc ^ kc_swz<BK>(row)) << 3);
}
// ---- K-slow tile [BK][RT] -------------------------------------------------------------------------
template <int RT>
__device__ __forceinline__ int ks_off(int k, int c) {
  if constexpr (RT % 128 == 0) {
    return k * RT + ((c ^ ((k & 3) << 2)) << 3);
  } else {
    // 192-element rows (384 bytes) hold 24 chunks: an XOR would leave the row, so the chunk index is rotated by
    // 4 * (k % 4) instead; with the row pitch of 96 banks the four k rows of a transposing read then start at
    // banks 0, 48, 32 and 16 (mod 64)
    constexpr int CPR = RT / 8;
    const int pc = c + ((k & 3) << 2);
    return k * RT + ((pc >= CPR ? pc - CPR : pc) << 3);
  }
}

// Fragment of a 32-row block for k step s (16 wide): lane l holds row l % 32, k = 8 * (l / 32) + 0..7.
template <int RT, int BK, bool KSLOW>
__device__ __forceinline__ bf16x8_t read_frag(const bf16_t* tile, int row0, int s) {
  const int lane = threadIdx.x & 63;
  if (!KSLOW) {
    return *reinterpret_cast<const bf16x8_t*>(tile + kc_off<BK>(row0 + (lane & 31), 2 * s + (lane >> 5)));
  } else {
    // two transposing reads; within a 16-lane group lane i addresses (k = kb + i / 4, r = rb + 4 * (i % 4))
    // and receives (r = rb + i, k = kb .. kb + 3)
    const int g = lane >> 4, i = lane & 15;
    const int r = row0 + 16 * (g & 1) + 4 * (i & 3);
    const int kb = 16 * s + 8 * (g >> 1) + (i >> 2);
    const lds_bf16_t* t3 = (const lds_bf16_t*)tile;
    const shortx4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t*)(t3 + ks_off<RT>(kb, r >> 3) + (r & 7)));
    const shortx4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t*)(t3 + ks_off<RT>(kb + 4, r >> 3) + (r & 7)));
    typedef short shortx8_t __attribute__((ext_vector_type(8)));
    const shortx8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, v);
  }
}

// Work item of a workgroup on a 1-D grid of tiles * splits: which output tile and which K split.
// Workgroups are dealt round-robin to the 8 XCDs, each with an L2 of its own.  Every XCD gets a contiguous
// range of tile ids, and with split K the splits are spread over the XCDs first (8 / splits XCDs per split,
// or splits / 8 splits per XCD): the tiles of one split read one K range of both operands, so an XCD's L2
// then holds that range once instead of every XCD fetching all of K for its share of the tiles.
__device__ __forceinline__ void gemm_work_item(int splits, int& tile, int& z) {
  const int id = blockIdx.x, nb = gridDim.x, tiles = nb / splits;
  if (nb & 7) {                                   // no even deal: plain order
    z = id / tiles;
    tile = id - z * tiles;
    return;
  }
  const int xcd = id & 7, j = id >> 3;            // j: index inside the XCD's share of nb / 8 workgroups
  if (splits <= 8 && (8 % splits) == 0 && tiles % (8 / splits) == 0) {
    const int p = 8 / splits;                     // XCDs per split
    z = xcd / p;
    tile = (xcd % p) * (tiles / p) + j;
  } else if ((splits & 7) == 0) {
    const int q = splits >> 3;                    // splits per XCD
    z = xcd * q + j / tiles;
    tile = j % tiles;
  } else {
    const int lin = xcd * (nb >> 3) + j;          // contiguous range per XCD over (split, tile)
    z = lin / tiles;
    tile = lin - z * tiles;
  }
}
