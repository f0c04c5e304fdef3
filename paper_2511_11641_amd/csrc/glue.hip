// Layer glue: the operators between the blocks of a pre-norm decoder layer (RMSNorm / LayerNorm with the residual
// addition in front, embedding lookup and its gradient, mean cross-entropy over the vocabulary).  They are the same for
// a dense and a sparse model - the method prunes the coupled pairs only (Sec. 3.1) - and are here so that a whole
// training step of a stack runs in this library.  All of them are bound by memory traffic: every row is read once
// into registers, 16 bytes per lane and load, and all reductions have a fixed order (no floating-point atomics), so
// results repeat bit for bit.
#include "common.h"

#define GLUE_MAXC 8                 // 16-byte chunks of a row that a lane holds: rows of up to 64 * 8 * 8 = 4096 bf16 elements
#define GLUE_NORM_THREADS 256       // 4 wavefronts, a row each
#define GLUE_XENT_THREADS 1024
#define GLUE_XENT_MAXC 8            // vocabulary up to 1024 * 8 * 8 = 65536

__device__ __forceinline__ void glue_unpack8(const uint4& u, float (&f)[8]) {
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 glue_pack8(const float (&f)[8]) {
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = static_cast<uint32_t>(f32_to_bf16(f[2 * i])) | (static_cast<uint32_t>(f32_to_bf16(f[2 * i + 1])) << 16);
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// ---------------------------------------------------------------------------------------------
// Normalisation, forward.  One wavefront per row: x (+ res) -> registers (the sum rounded to bf16 is what the residual
// stream holds, so the statistics are taken of the rounded values - what a later pass would read), mean and variance
// around the mean in two register passes, y and the row statistics out.
// ---------------------------------------------------------------------------------------------
struct NormFwdArgs {
  const bf16_t *x, *res, *gain, *bias;
  bf16_t *x_out, *y;
  float* stat;
  int T, d, layer;
  float eps;
};
template <int MAXC>
__global__ __launch_bounds__(GLUE_NORM_THREADS) void norm_fwd_kernel(const NormFwdArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * (GLUE_NORM_THREADS / 64) + wave;
  if (row >= a.T) return;
  const int nc = a.d >> 3;                          // 16-byte chunks per row
  const long long base = static_cast<long long>(row) * a.d;
  float v[MAXC][8];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int ch = c * 64 + lane;
    if (ch < nc) {
      glue_unpack8(*reinterpret_cast<const uint4*>(a.x + base + ch * 8), v[c]);
      if (a.res) {
        float r[8];
        glue_unpack8(*reinterpret_cast<const uint4*>(a.res + base + ch * 8), r);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[c][i] += r[i];
        const uint4 packed = glue_pack8(v[c]);
        *reinterpret_cast<uint4*>(a.x_out + base + ch * 8) = packed;
        glue_unpack8(packed, v[c]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) s += v[c][i];
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[c][i] = 0.f;
    }
  }
  const float inv_d = 1.f / static_cast<float>(a.d);
  const float mean = a.layer ? wave_sum(s) * inv_d : 0.f;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    if (c * 64 + lane < nc) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float t = v[c][i] - mean;
        q += t * t;
      }
    }
  }
  const float rstd = rsqrtf(wave_sum(q) * inv_d + a.eps);
  if (a.stat && lane == 0) {
    if (a.layer) { a.stat[2 * row] = mean; a.stat[2 * row + 1] = rstd; }
    else a.stat[row] = rstd;
  }
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int ch = c * 64 + lane;
    if (ch < nc) {
      float g[8], o[8];
      glue_unpack8(*reinterpret_cast<const uint4*>(a.gain + ch * 8), g);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = (v[c][i] - mean) * rstd * g[i];
      if (a.bias) {
        float b[8];
        glue_unpack8(*reinterpret_cast<const uint4*>(a.bias + ch * 8), b);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] += b[i];
      }
      *reinterpret_cast<uint4*>(a.y + base + ch * 8) = glue_pack8(o);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Normalisation, backward.  A workgroup takes a contiguous range of rows, a wavefront a row at a time; with
// u = dy * gain and xhat = (x - mean) * rstd:   dx = rstd * (u - mean(u) - xhat * mean(u * xhat))  (RMSNorm: mean = 0 and no
// mean(u) term), plus the gradient that reaches the same rows through the residual connection.  Every lane also adds up
// dy * xhat (and dy) of its own columns over the rows of its wavefront; the four wavefronts' sums are added in order
// through LDS and written as one partial row per workgroup; norm_bwd_finish_kernel adds the partial rows in order.
// ---------------------------------------------------------------------------------------------
struct NormBwdArgs {
  const bf16_t *x, *gain, *dy, *dres;
  const float* stat;
  bf16_t* dx;
  float* part;          // [blocks][2][d]: sums of dy * xhat, sums of dy
  int T, d, layer, rows_per_block;
};
template <int MAXC, bool LAYER>
__global__ __launch_bounds__(GLUE_NORM_THREADS) void norm_bwd_kernel(const NormBwdArgs a) {
  __shared__ float red[GLUE_NORM_THREADS / 64 - 1][2 * 8 * 64];   // two chunks of every lane at a time
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nc = a.d >> 3;
  const int r0 = blockIdx.x * a.rows_per_block, r1 = min(a.T, r0 + a.rows_per_block);
  float gacc[MAXC][8], bacc[LAYER ? MAXC : 1][8];
#pragma unroll
  for (int c = 0; c < MAXC; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) { gacc[c][i] = 0.f; if (LAYER) bacc[c][i] = 0.f; }
  const float inv_d = 1.f / static_cast<float>(a.d);
  for (int row = r0 + wave; row < r1; row += GLUE_NORM_THREADS / 64) {
    const long long base = static_cast<long long>(row) * a.d;
    const float mean = LAYER ? a.stat[2 * row] : 0.f;
    const float rstd = LAYER ? a.stat[2 * row + 1] : a.stat[row];
    uint4 xr[MAXC], dr[MAXC], gr[MAXC];     // the gain comes from the cache again for every row: registers go to the sums
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      const int ch = c * 64 + lane;
      if (ch < nc) {
        xr[c] = *reinterpret_cast<const uint4*>(a.x + base + ch * 8);
        dr[c] = *reinterpret_cast<const uint4*>(a.dy + base + ch * 8);
        gr[c] = *reinterpret_cast<const uint4*>(a.gain + ch * 8);
      }
    }
    float su = 0.f, sux = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      if (c * 64 + lane < nc) {
        float xv[8], dv[8], g[8];
        glue_unpack8(xr[c], xv);
        glue_unpack8(dr[c], dv);
        glue_unpack8(gr[c], g);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xh = (xv[i] - mean) * rstd, u = dv[i] * g[i];
          su += u;
          sux += u * xh;
          gacc[c][i] += dv[i] * xh;
          if (LAYER) bacc[c][i] += dv[i];
        }
      }
    }
    const float mu = LAYER ? wave_sum(su) * inv_d : 0.f;
    const float mux = wave_sum(sux) * inv_d;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      const int ch = c * 64 + lane;
      if (ch < nc) {
        float xv[8], dv[8], g[8], o[8];
        glue_unpack8(xr[c], xv);
        glue_unpack8(dr[c], dv);
        glue_unpack8(gr[c], g);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xh = (xv[i] - mean) * rstd;
          o[i] = rstd * (dv[i] * g[i] - mu - xh * mux);
        }
        if (a.dres) {
          float r[8];
          glue_unpack8(*reinterpret_cast<const uint4*>(a.dres + base + ch * 8), r);
#pragma unroll
          for (int i = 0; i < 8; ++i) o[i] += r[i];
        }
        *reinterpret_cast<uint4*>(a.dx + base + ch * 8) = glue_pack8(o);
      }
    }
  }
  // the four wavefronts' column sums, added in wavefront order, two chunks of every lane per round through LDS
  float* prow = a.part + static_cast<long long>(blockIdx.x) * 2 * a.d;
  constexpr int STEP = MAXC >= 2 ? 2 : 1;
#pragma unroll
  for (int which = 0; which < (LAYER ? 2 : 1); ++which) {
#pragma unroll
    for (int c0 = 0; c0 < MAXC; c0 += STEP) {
      __syncthreads();
      if (wave > 0) {
#pragma unroll
        for (int cc = 0; cc < STEP; ++cc)
#pragma unroll
          for (int i = 0; i < 8; ++i) red[wave - 1][(cc * 8 + i) * 64 + lane] = which ? bacc[LAYER ? c0 + cc : 0][i] : gacc[c0 + cc][i];
      }
      __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int cc = 0; cc < STEP; ++cc) {
          const int ch = (c0 + cc) * 64 + lane;
          if (ch < nc) {
            float o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              float t = which ? bacc[LAYER ? c0 + cc : 0][i] : gacc[c0 + cc][i];
#pragma unroll
              for (int w = 0; w < GLUE_NORM_THREADS / 64 - 1; ++w) t += red[w][(cc * 8 + i) * 64 + lane];
              o[i] = t;
            }
            float* p = prow + which * a.d + ch * 8;
            *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
            *reinterpret_cast<float4*>(p + 4) = make_float4(o[4], o[5], o[6], o[7]);
          }
        }
      }
    }
  }
}
// dgain[c] (and dbias[c]) = the partial rows of all workgroups, rounded once.  A workgroup takes 64 columns: its 16
// wavefronts each add a contiguous sixteenth of the partial rows (eight loads in flight per lane), then the sixteen
// sums are added in order - a fixed order altogether.
#define GLUE_FIN_SLICES 16
__global__ __launch_bounds__(64 * GLUE_FIN_SLICES) void norm_bwd_finish_kernel(const float* part, int blocks, int d, int layer,
                                                                               bf16_t* dgain, bf16_t* dbias) {
  __shared__ float red[2][GLUE_FIN_SLICES][64];
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  const int per = (blocks + GLUE_FIN_SLICES - 1) / GLUE_FIN_SLICES;
  const int b0 = slice * per, b1 = min(blocks, b0 + per);
  float sg = 0.f, sb = 0.f;
  if (c < d) {
#pragma unroll 8
    for (int b = b0; b < b1; ++b) {
      sg += part[(static_cast<long long>(b) * 2) * d + c];
      if (layer) sb += part[(static_cast<long long>(b) * 2 + 1) * d + c];
    }
  }
  red[0][slice][lane] = sg;
  red[1][slice][lane] = sb;
  __syncthreads();
  if (slice == 0 && c < d) {
    float tg = 0.f, tb = 0.f;
#pragma unroll
    for (int q = 0; q < GLUE_FIN_SLICES; ++q) { tg += red[0][q][lane]; tb += red[1][q][lane]; }
    dgain[c] = f32_to_bf16(tg);
    if (layer && dbias) dbias[c] = f32_to_bf16(tb);
  }
}

// ---------------------------------------------------------------------------------------------
// Embedding lookup (+ learned position table) and its gradient.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void embed_fwd_kernel(const long long* ids, const bf16_t* table, const bf16_t* pos, int L, int T, int d,
                                                        int vocab, bf16_t* out) {
  const int nc = d >> 3;
  const long long e = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= static_cast<long long>(T) * nc) return;
  const int t = static_cast<int>(e / nc), ch = static_cast<int>(e % nc);
  const long long id = ids[t];
  uint4 v = make_uint4(0u, 0u, 0u, 0u);        // an id outside the table reads as a zero row
  if (id >= 0 && id < vocab) v = *reinterpret_cast<const uint4*>(table + id * d + ch * 8);
  if (pos) {
    float a[8], b[8];
    glue_unpack8(v, a);
    glue_unpack8(*reinterpret_cast<const uint4*>(pos + static_cast<long long>(t % L) * d + ch * 8), b);
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] += b[i];
    v = glue_pack8(a);
  }
  *reinterpret_cast<uint4*>(out + static_cast<long long>(t) * d + ch * 8) = v;
}
__global__ __launch_bounds__(256) void glue_zero_kernel(uint4* p, long long n16) {
  const long long i = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}
// Gradient of the table: one workgroup per token position t.  The workgroup of the first position that holds a token id
// adds the rows of all positions with that id, in position order, in fp32, and writes the table row once; the other
// workgroups find an earlier position with their id and leave.  No atomics: the order of every sum is fixed.
__global__ __launch_bounds__(256) void embed_bwd_kernel(const long long* ids, const bf16_t* dx, int T, int d, int vocab, bf16_t* dtable) {
  __shared__ int list[256];
  __shared__ int wcount[4];
  const int t0 = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long id = ids[t0];
  if (id < 0 || id >= vocab) return;           // outside the table: no row to add to (uniform over the workgroup)
  int earlier = 0;
  for (int t = tid; t < t0; t += 256) earlier |= ids[t] == id;
  if (__syncthreads_or(earlier)) return;
  const int nc = d >> 3;
  float acc[GLUE_MAXC / 4][8];       // a thread owns chunks tid, tid + 256: rows of up to 4096 elements
#pragma unroll
  for (int c = 0; c < GLUE_MAXC / 4; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[c][i] = 0.f;
  for (int base = t0; base < T; base += 256) {
    const int t = base + tid;
    const bool hit = t < T && ids[t] == id;
    const unsigned long long m = __ballot(hit);
    __syncthreads();                 // the list of the previous round has been read
    if (lane == 0) wcount[wave] = __popcll(m);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) { if (w < wave) before += wcount[w]; total += wcount[w]; }
    if (hit) list[before + __popcll(m & ((1ull << lane) - 1ull))] = t;
    __syncthreads();
    for (int j = 0; j < total; ++j) {
      const long long row = static_cast<long long>(list[j]) * d;
#pragma unroll
      for (int c = 0; c < GLUE_MAXC / 4; ++c) {
        const int ch = c * 256 + tid;
        if (ch < nc) {
          float v[8];
          glue_unpack8(*reinterpret_cast<const uint4*>(dx + row + ch * 8), v);
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[c][i] += v[i];
        }
      }
    }
  }
#pragma unroll
  for (int c = 0; c < GLUE_MAXC / 4; ++c) {
    const int ch = c * 256 + tid;
    if (ch < nc) *reinterpret_cast<uint4*>(dtable + id * d + ch * 8) = glue_pack8(acc[c]);
  }
}
// Gradient of the position table: dpos[l] = sum over the sequences of dx[b * L + l], in order of b.
__global__ __launch_bounds__(256) void pos_bwd_kernel(const bf16_t* dx, int Bsz, int L, int d, bf16_t* dpos) {
  const int nc = d >> 3;
  const long long e = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= static_cast<long long>(L) * nc) return;
  const int l = static_cast<int>(e / nc), ch = static_cast<int>(e % nc);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int b = 0; b < Bsz; ++b) {
    float v[8];
    glue_unpack8(*reinterpret_cast<const uint4*>(dx + (static_cast<long long>(b) * L + l) * d + ch * 8), v);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += v[i];
  }
  *reinterpret_cast<uint4*>(dpos + static_cast<long long>(l) * d + ch * 8) = glue_pack8(acc);
}

// ---------------------------------------------------------------------------------------------
// Mean cross-entropy over the vocabulary.  One workgroup per row: the row goes into registers once (raw bf16), maximum,
// sum of exponentials (base-2 domain), then the row loss lse - logit[target] and dlogits = (softmax - onehot) * scale
// in one pass over the registers.  xent_finish_kernel adds the row losses in a fixed order.
// ---------------------------------------------------------------------------------------------
struct XentArgs {
  const bf16_t* logits;
  const long long* targets;
  bf16_t* dlogits;
  float* row_loss;
  long long ldl, ldd;
  int T, V;
  float scale;
};
__device__ __forceinline__ float xent_block_reduce(float v, bool is_max, float* red) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < GLUE_XENT_THREADS / 64; ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
  return r;
}
__global__ __launch_bounds__(GLUE_XENT_THREADS) void xent_kernel(const XentArgs a) {
  __shared__ float red[GLUE_XENT_THREADS / 64];
  const int row = blockIdx.x, tid = threadIdx.x;
  const bf16_t* lg = a.logits + static_cast<long long>(row) * a.ldl;
  const int nfull = a.V >> 3;        // whole 16-byte chunks; the tail (V % 8 elements) is handled by thread 0's scalar loop
  uint4 raw[GLUE_XENT_MAXC];
  float mx = -INFINITY;
#pragma unroll
  for (int c = 0; c < GLUE_XENT_MAXC; ++c) {
    const int ch = c * GLUE_XENT_THREADS + tid;
    if (ch < nfull) {
      raw[c] = *reinterpret_cast<const uint4*>(lg + ch * 8);
      float v[8];
      glue_unpack8(raw[c], v);
#pragma unroll
      for (int i = 0; i < 8; ++i) mx = fmaxf(mx, v[i]);
    }
  }
  if (tid == 0)
    for (int j = nfull * 8; j < a.V; ++j) mx = fmaxf(mx, bf16_to_f32(lg[j]));
  mx = xent_block_reduce(mx, true, red);
  constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
  const float mx2 = mx * LOG2E;
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < GLUE_XENT_MAXC; ++c) {
    if (c * GLUE_XENT_THREADS + tid < nfull) {
      float v[8];
      glue_unpack8(raw[c], v);
#pragma unroll
      for (int i = 0; i < 8; ++i) s += __builtin_amdgcn_exp2f(__builtin_fmaf(v[i], LOG2E, -mx2));
    }
  }
  if (tid == 0)
    for (int j = nfull * 8; j < a.V; ++j) s += __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_to_f32(lg[j]), LOG2E, -mx2));
  s = xent_block_reduce(s, false, red);
  const float lse2 = mx2 + __builtin_amdgcn_logf(s);          // log2 of the sum of exponentials
  const long long tgt = a.targets[row];
  const bool counted = tgt >= 0 && tgt < a.V;      // a target outside the vocabulary: the row adds nothing to the loss
  if (tid == 0) a.row_loss[row] = counted ? (lse2 - bf16_to_f32(lg[tgt]) * LOG2E) * LN2 : 0.f;
  if (!a.dlogits) return;
  bf16_t* dl = a.dlogits + static_cast<long long>(row) * a.ldd;
#pragma unroll
  for (int c = 0; c < GLUE_XENT_MAXC; ++c) {
    const int ch = c * GLUE_XENT_THREADS + tid;
    if (ch < nfull) {
      float v[8], o[8];
      glue_unpack8(raw[c], v);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(v[i], LOG2E, -lse2));
        o[i] = counted ? (p - (ch * 8 + i == tgt ? 1.f : 0.f)) * a.scale : 0.f;
      }
      *reinterpret_cast<uint4*>(dl + ch * 8) = glue_pack8(o);
    }
  }
  if (tid == 0)
    for (int j = nfull * 8; j < a.V; ++j) {
      const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_to_f32(lg[j]), LOG2E, -lse2));
      dl[j] = f32_to_bf16(counted ? (p - (j == tgt ? 1.f : 0.f)) * a.scale : 0.f);
    }
}
// loss = scale * sum of the row losses: 1024 strided partial sums, then a fixed tree.
__global__ __launch_bounds__(1024) void xent_finish_kernel(const float* row_loss, int T, float scale, float* loss) {
  __shared__ float red[1024];
  float s = 0.f;
  for (int t = threadIdx.x; t < T; t += 1024) s += row_loss[t];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (static_cast<int>(threadIdx.x) < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = red[0] * scale;
}

// ---------------------------------------------------------------------------------------------
// entry points
// ---------------------------------------------------------------------------------------------
static int norm_check(int kind, int T, int d, int dtype) {
  if (kind != ECOSPA_NORM_RMS && kind != ECOSPA_NORM_LAYER) return ECOSPA_ERR_SHAPE;
  if (dtype != ECOSPA_BF16) return ECOSPA_ERR_DTYPE;
  if (T < 1 || d < 8 || d % 8 || d > 64 * GLUE_MAXC * 8) return ECOSPA_ERR_SHAPE;
  return ECOSPA_OK;
}

extern "C" int ecospa_norm_fwd(ecospa_ctx* ctx, int kind, int T, int d, int dtype, const void* x, const void* res, void* x_out,
                               const void* gain, const void* bias, float eps, void* y, float* stat) {
  if (!ctx || !x || !gain || !y || (res && !x_out)) return ECOSPA_ERR_NULL;
  const int rc = norm_check(kind, T, d, dtype);
  if (rc != ECOSPA_OK) return rc;
  if (!(eps >= 0.f)) return ECOSPA_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(y) || !aligned16(gain) || (res && (!aligned16(res) || !aligned16(x_out))) || (bias && !aligned16(bias)))
    return ECOSPA_ERR_ALIGN;
  NormFwdArgs a;
  a.x = static_cast<const bf16_t*>(x); a.res = static_cast<const bf16_t*>(res); a.gain = static_cast<const bf16_t*>(gain);
  a.bias = kind == ECOSPA_NORM_LAYER ? static_cast<const bf16_t*>(bias) : nullptr;
  a.x_out = static_cast<bf16_t*>(x_out); a.y = static_cast<bf16_t*>(y); a.stat = stat;
  a.T = T; a.d = d; a.layer = kind == ECOSPA_NORM_LAYER; a.eps = eps;
  const int per = GLUE_NORM_THREADS / 64;
  const dim3 grid((T + per - 1) / per), block(GLUE_NORM_THREADS);
  if (d <= 1024) hipLaunchKernelGGL(norm_fwd_kernel<2>, grid, block, 0, ctx->stream, a);
  else if (d <= 2048) hipLaunchKernelGGL(norm_fwd_kernel<4>, grid, block, 0, ctx->stream, a);
  else hipLaunchKernelGGL(norm_fwd_kernel<GLUE_MAXC>, grid, block, 0, ctx->stream, a);
  ECOSPA_CHECK_LAUNCH(ctx, "norm_fwd_kernel");
  return ECOSPA_OK;
}

static int norm_bwd_blocks(int T) { return T < 1024 ? (T + 3) / 4 : 512; }
extern "C" size_t ecospa_norm_bwd_workspace_bytes(int T, int d) {
  if (T < 1 || d < 1) return 0;
  return static_cast<size_t>(norm_bwd_blocks(T)) * 2 * d * sizeof(float) + 256;
}
extern "C" int ecospa_norm_bwd(ecospa_ctx* ctx, int kind, int T, int d, int dtype, const void* x, const void* gain, const float* stat,
                               const void* dy, const void* dres, void* dx, void* dgain, void* dbias) {
  if (!ctx || !x || !gain || !stat || !dy || !dx || !dgain) return ECOSPA_ERR_NULL;
  const int rc = norm_check(kind, T, d, dtype);
  if (rc != ECOSPA_OK) return rc;
  if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(gain) || (dres && !aligned16(dres))) return ECOSPA_ERR_ALIGN;
  const int blocks = norm_bwd_blocks(T);
  WsCarver ws(ctx->ws, ctx->ws_bytes);
  float* part = static_cast<float*>(ws.take(static_cast<size_t>(blocks) * 2 * d * sizeof(float)));
  if (!ws.ok()) return ECOSPA_ERR_WORKSPACE;
  NormBwdArgs a;
  a.x = static_cast<const bf16_t*>(x); a.gain = static_cast<const bf16_t*>(gain); a.dy = static_cast<const bf16_t*>(dy);
  a.dres = static_cast<const bf16_t*>(dres); a.stat = stat; a.dx = static_cast<bf16_t*>(dx); a.part = part;
  a.T = T; a.d = d; a.layer = kind == ECOSPA_NORM_LAYER; a.rows_per_block = (T + blocks - 1) / blocks;
  const dim3 grid(blocks), block(GLUE_NORM_THREADS);
#define NORM_BWD_LAUNCH(MAXC)                                                                                   \
  do {                                                                                                          \
    if (a.layer) hipLaunchKernelGGL((norm_bwd_kernel<MAXC, true>), grid, block, 0, ctx->stream, a);              \
    else hipLaunchKernelGGL((norm_bwd_kernel<MAXC, false>), grid, block, 0, ctx->stream, a);                     \
  } while (0)
  if (d <= 1024) NORM_BWD_LAUNCH(2);
  else if (d <= 2048) NORM_BWD_LAUNCH(4);
  else NORM_BWD_LAUNCH(GLUE_MAXC);
#undef NORM_BWD_LAUNCH
  ECOSPA_CHECK_LAUNCH(ctx, "norm_bwd_kernel");
  hipLaunchKernelGGL(norm_bwd_finish_kernel, dim3((d + 63) / 64), dim3(64 * GLUE_FIN_SLICES), 0, ctx->stream, part, blocks, d, a.layer,
                     static_cast<bf16_t*>(dgain), static_cast<bf16_t*>(dbias));
  ECOSPA_CHECK_LAUNCH(ctx, "norm_bwd_finish_kernel");
  return ECOSPA_OK;
}

extern "C" int ecospa_embed_fwd(ecospa_ctx* ctx, int T, int d, int vocab, int dtype, const long long* ids, const void* table,
                                const void* pos, int L, void* out) {
  if (!ctx || !ids || !table || !out) return ECOSPA_ERR_NULL;
  if (dtype != ECOSPA_BF16) return ECOSPA_ERR_DTYPE;
  if (T < 1 || vocab < 1 || d < 8 || d % 8 || (pos && (L < 1 || T % L))) return ECOSPA_ERR_SHAPE;
  if (!aligned16(table) || !aligned16(out) || (pos && !aligned16(pos))) return ECOSPA_ERR_ALIGN;
  const long long n = static_cast<long long>(T) * (d / 8);
  hipLaunchKernelGGL(embed_fwd_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, ctx->stream, ids,
                     static_cast<const bf16_t*>(table), static_cast<const bf16_t*>(pos), L, T, d, vocab, static_cast<bf16_t*>(out));
  ECOSPA_CHECK_LAUNCH(ctx, "embed_fwd_kernel");
  return ECOSPA_OK;
}

extern "C" int ecospa_embed_bwd(ecospa_ctx* ctx, int T, int d, int vocab, int dtype, const long long* ids, const void* dx, void* dtable,
                                void* dpos, int L) {
  if (!ctx || !ids || !dx || !dtable) return ECOSPA_ERR_NULL;
  if (dtype != ECOSPA_BF16) return ECOSPA_ERR_DTYPE;
  if (T < 1 || vocab < 1 || d < 8 || d % 8 || d > 64 * GLUE_MAXC * 8 || (dpos && (L < 1 || T % L))) return ECOSPA_ERR_SHAPE;
  if (!aligned16(dx) || !aligned16(dtable) || (dpos && !aligned16(dpos))) return ECOSPA_ERR_ALIGN;
  const long long n16 = static_cast<long long>(vocab) * d / 8;
  hipLaunchKernelGGL(glue_zero_kernel, dim3(static_cast<unsigned>((n16 + 255) / 256)), dim3(256), 0, ctx->stream,
                     static_cast<uint4*>(dtable), n16);
  ECOSPA_CHECK_LAUNCH(ctx, "glue_zero_kernel");
  hipLaunchKernelGGL(embed_bwd_kernel, dim3(T), dim3(256), 0, ctx->stream, ids, static_cast<const bf16_t*>(dx), T, d,
                     vocab, static_cast<bf16_t*>(dtable));
  ECOSPA_CHECK_LAUNCH(ctx, "embed_bwd_kernel");
  if (dpos) {
    const long long n = static_cast<long long>(L) * (d / 8);
    hipLaunchKernelGGL(pos_bwd_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, ctx->stream,
                       static_cast<const bf16_t*>(dx), T / L, L, d, static_cast<bf16_t*>(dpos));
    ECOSPA_CHECK_LAUNCH(ctx, "pos_bwd_kernel");
  }
  return ECOSPA_OK;
}

extern "C" int ecospa_xent(ecospa_ctx* ctx, int T, int V, int dtype, const void* logits, long long ldl, const long long* targets,
                           void* dlogits, long long ldd, float* row_loss, float* loss) {
  if (!ctx || !logits || !targets || !row_loss || !loss) return ECOSPA_ERR_NULL;
  if (dtype != ECOSPA_BF16) return ECOSPA_ERR_DTYPE;
  if (T < 1 || V < 1 || V > GLUE_XENT_THREADS * GLUE_XENT_MAXC * 8 || ldl < V || (dlogits && ldd < V)) return ECOSPA_ERR_SHAPE;
  if (!aligned16(logits) || ldl % 8 || (dlogits && (!aligned16(dlogits) || ldd % 8))) return ECOSPA_ERR_ALIGN;
  XentArgs a;
  a.logits = static_cast<const bf16_t*>(logits); a.targets = targets; a.dlogits = static_cast<bf16_t*>(dlogits);
  a.row_loss = row_loss; a.ldl = ldl; a.ldd = ldd; a.T = T; a.V = V; a.scale = 1.f / static_cast<float>(T);
  hipLaunchKernelGGL(xent_kernel, dim3(T), dim3(GLUE_XENT_THREADS), 0, ctx->stream, a);
  ECOSPA_CHECK_LAUNCH(ctx, "xent_kernel");
  hipLaunchKernelGGL(xent_finish_kernel, dim3(1), dim3(1024), 0, ctx->stream, row_loss, T, a.scale, loss);
  ECOSPA_CHECK_LAUNCH(ctx, "xent_finish_kernel");
  return ECOSPA_OK;
}
