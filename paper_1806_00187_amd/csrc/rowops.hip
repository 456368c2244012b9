// HBM-bound row kernels of the training step: embedding (+positions, dropout), fused
// residual + dropout + LayerNorm forward / backward (one wavefront per token row), column sums
// for bias gradients, fused vocabulary softmax + label-smoothed cross-entropy + gradient, and the
// deterministic embedding-gradient reduction.
#include <math.h>

#include <mutex>

#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;

__device__ __forceinline__ void unpack8(const half8_t h, float (&f)[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = (float)h[e];
}
__device__ __forceinline__ half8_t pack8(const float (&f)[8]) {
  half8_t h;
#pragma unroll
  for (int e = 0; e < 8; ++e) h[e] = (half_t)f[e];
  return h;
}

// ------------------------------------------------------------------------------------------------
// Embedding forward: x = dropout(sqrt(d) * E[id] + PE(pos)); PE[t,2i] = sin(t / 10000^(2i/d)),
// PE[t,2i+1] = cos(same).  One thread per 8 columns.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) embed_fwd_kernel(const int32_t* __restrict__ ids, const half_t* __restrict__ E,
                                                             half_t* __restrict__ x, int rows, int d, int vocab,
                                                             DropDev drop) {
  const int chunks = d >> 3;
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (gid >= (int64_t)rows * chunks) return;
  const int row = (int)(gid / chunks), c = (int)(gid % chunks);
  int id = ids[row];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  float v[8];
  unpack8(ld_half8(E + (size_t)id * d + c * 8), v);
  const float pos = (float)drop_row_pos(drop, (uint32_t)row);
  const float sq = sqrtf((float)d);
  const float k = -logf(10000.f) / (float)d;
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const float ang = pos * expf(k * (float)(c * 8 + e));
    v[e] = v[e] * sq + sinf(ang);
    v[e + 1] = v[e + 1] * sq + cosf(ang);
  }
  if (drop.thr) {
    const uint32_t bits = drop_keep8(drop, (uint32_t)row, (uint32_t)c);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = ((bits >> e) & 1u) ? v[e] * drop.scale : 0.f;
  }
  st_half8(x + (size_t)row * d + c * 8, pack8(v));
}

// ------------------------------------------------------------------------------------------------
// out = LayerNorm(resid + dropout(sub)); one wavefront per row, NCH chunks of 8 columns per lane.
// ------------------------------------------------------------------------------------------------
template <int NCH>
__device__ __forceinline__ void load_presum(float (&y)[NCH][8], const half_t* __restrict__ sub,
                                            const half_t* __restrict__ resid, int row, int d, int lane,
                                            const DropDev& drop, uint32_t (&bits)[NCH]) {
  const int chunks = d >> 3;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + kWave * i;
    bits[i] = 0xFFu;
    if (c < chunks) {
      float s[8], r[8];
      unpack8(ld_half8_nt(sub + (size_t)row * d + c * 8), s);
      unpack8(ld_half8_nt(resid + (size_t)row * d + c * 8), r);
      if (drop.thr) bits[i] = drop_keep8(drop, (uint32_t)row, (uint32_t)c);
#pragma unroll
      for (int e = 0; e < 8; ++e) y[i][e] = r[e] + (((bits[i] >> e) & 1u) ? s[e] * drop.scale : 0.f);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) y[i][e] = 0.f;
    }
  }
}

template <int NCH>
__global__ void __launch_bounds__(kThreads) res_ln_fwd_kernel(const half_t* __restrict__ sub, const half_t* __restrict__ resid,
                                                              const half_t* __restrict__ gamma, const half_t* __restrict__ beta,
                                                              half_t* __restrict__ out, float* __restrict__ stats, int rows,
                                                              int d, float eps, DropDev drop) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int chunks = d >> 3;
  float y[NCH][8];
  uint32_t bits[NCH];
  load_presum<NCH>(y, sub, resid, row, d, lane, drop, bits);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) s += y[i][e];
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
    if (lane + kWave * i < chunks) {
#pragma unroll
      for (int e = 0; e < 8; ++e) q += (y[i][e] - mean) * (y[i][e] - mean);
    }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + kWave * i;
    if (c < chunks) {
      float g[8], b[8], o[8];
      unpack8(ld_half8(gamma + c * 8), g);
      unpack8(ld_half8(beta + c * 8), b);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (y[i][e] - mean) * rstd * g[e] + b[e];
      st_half8_nt(out + (size_t)row * d + c * 8, pack8(o));
    }
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
}

// Backward.  Each wavefront walks groups of kLnRows rows (their loads are all issued before anything is
// computed), keeps per-lane column sums for dgamma, dbeta and the bias gradient in registers, and the block
// writes one partial row per quantity (pitch NCH*512 floats, column-indexed).  The three inputs of a row stay in
// registers as the fp16 values they were loaded as and are widened where they are used (twice: row statistics,
// then the result), which keeps the kernel at four wavefronts per SIMD.
constexpr int kLnBwdMaxBlocks = 1024;
constexpr int kLnRows = 2;

template <int NCH>
__global__ void __launch_bounds__(kThreads) res_ln_bwd_kernel(const half_t* __restrict__ dout, const half_t* __restrict__ sub,
                                                              const half_t* __restrict__ resid, const half_t* __restrict__ gamma,
                                                              const float* __restrict__ stats, half_t* __restrict__ dy_out,
                                                              half_t* __restrict__ dym_out, float* __restrict__ partial, int rows,
                                                              int d, DropDev drop) {
  extern __shared__ __align__(16) float red[];  // [3][NCH][64 lanes][8] = [3][NCH*512]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunks = d >> 3;
  float sg[NCH][8], sb[NCH][8], sbias[NCH][8];
  half8_t gam[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    gam[i] = lane + kWave * i < chunks ? ld_half8(gamma + (lane + kWave * i) * 8) : zero_half8();
#pragma unroll
    for (int e = 0; e < 8; ++e) sg[i][e] = sb[i][e] = sbias[i][e] = 0.f;
  }
  for (int row0 = (blockIdx.x * kWavesPerBlock + wave) * kLnRows; row0 < rows; row0 += gridDim.x * kWavesPerBlock * kLnRows) {
    half8_t hs[kLnRows][NCH], hr[kLnRows][NCH], hg[kLnRows][NCH];
    uint32_t bits[kLnRows][NCH];
    float mean[kLnRows], rstd[kLnRows], s1[kLnRows], s2[kLnRows];
#pragma unroll
    for (int u = 0; u < kLnRows; ++u) {
      const int row = min(row0 + u, rows - 1);  // a row past the end repeats the last one and is not written
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + kWave * i;
        const bool in = c < chunks;
        hs[u][i] = in ? ld_half8_nt(sub + (size_t)row * d + c * 8) : zero_half8();
        hr[u][i] = in ? ld_half8_nt(resid + (size_t)row * d + c * 8) : zero_half8();
        hg[u][i] = in ? ld_half8_nt(dout + (size_t)row * d + c * 8) : zero_half8();
      }
      mean[u] = stats[2 * row];
      rstd[u] = stats[2 * row + 1];
    }
#pragma unroll
    for (int u = 0; u < kLnRows; ++u) {
      const int row = min(row0 + u, rows - 1);
#pragma unroll
      for (int i = 0; i < NCH; ++i)
        bits[u][i] = (drop.thr && lane + kWave * i < chunks) ? drop_keep8(drop, (uint32_t)row, (uint32_t)(lane + kWave * i)) : 0xFFu;
    }
    // normalised value of element e of chunk i of row u (the pre-normalisation sum is formed in fp32, as in the forward pass)
    auto xhat = [&](int u, int i, int e) {
      const float y = (float)hr[u][i][e] + (((bits[u][i] >> e) & 1u) ? (float)hs[u][i][e] * drop.scale : 0.f);
      return (y - mean[u]) * rstd[u];
    };
#pragma unroll
    for (int u = 0; u < kLnRows; ++u) {
      const bool live = row0 + u < rows;
      s1[u] = s2[u] = 0.f;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        if (lane + kWave * i < chunks) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float xh = xhat(u, i, e), go = (float)hg[u][i][e];
            const float g = go * (float)gam[i][e];
            s1[u] += g;
            s2[u] += g * xh;
            if (live) {
              sg[i][e] += go * xh;
              sb[i][e] += go;
            }
          }
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
#pragma unroll
      for (int u = 0; u < kLnRows; ++u) {
        s1[u] += __shfl_xor(s1[u], o, kWave);
        s2[u] += __shfl_xor(s2[u], o, kWave);
      }
    }
    // (the widened copies of the first pass are not kept: the inputs are widened again from their fp16 registers)
#pragma unroll
    for (int u = 0; u < kLnRows; ++u)
#pragma unroll
      for (int i = 0; i < NCH; ++i) asm volatile("" : "+v"(hs[u][i]), "+v"(hr[u][i]), "+v"(hg[u][i]));
#pragma unroll
    for (int u = 0; u < kLnRows; ++u) {
      const int row = row0 + u;
      if (row >= rows) break;
      const float m1 = s1[u] / (float)d, m2 = s2[u] / (float)d;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + kWave * i;
        if (c < chunks) {
          float dy[8], dm[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            dy[e] = rstd[u] * ((float)hg[u][i][e] * (float)gam[i][e] - m1 - xhat(u, i, e) * m2);
            dm[e] = ((bits[u][i] >> e) & 1u) ? dy[e] * drop.scale : 0.f;
            sbias[i][e] += dm[e];
          }
          st_half8_nt(dy_out + (size_t)row * d + c * 8, pack8(dy));
          if (dym_out) st_half8_nt(dym_out + (size_t)row * d + c * 8, pack8(dm));
        }
      }
    }
  }
  // block reduction, wave after wave (fixed order), 16-byte LDS accesses
  floatx4* red4 = reinterpret_cast<floatx4*>(red);
  for (int w = 0; w < kWavesPerBlock; ++w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          const float(&src)[8] = q == 0 ? sg[i] : (q == 1 ? sb[i] : sbias[i]);
          const int idx = ((q * NCH + i) * kWave + lane) * 2;
          floatx4 lo = {src[0], src[1], src[2], src[3]}, hi = {src[4], src[5], src[6], src[7]};
          if (w) {
            lo += red4[idx];
            hi += red4[idx + 1];
          }
          red4[idx] = lo;
          red4[idx + 1] = hi;
        }
      }
    }
    __syncthreads();
  }
  floatx4* dst = reinterpret_cast<floatx4*>(partial + (size_t)blockIdx.x * 3 * NCH * 512);
  for (int i = threadIdx.x; i < 3 * NCH * 128; i += kThreads) dst[i] = red4[i];
}

// dst_k[col] = fp16(sum_b partial[b][k][col]), k = 0..nq-1.  A block of 1024 threads owns 32 columns of
// one quantity; its 32 row-lanes stride over the partial rows (independent loads, several in
// flight) and are combined in a fixed order.
constexpr int kFinThreads = 1024;
__global__ void __launch_bounds__(kFinThreads) finalize_partials_kernel(const float* __restrict__ partial, int nblk, int nq,
                                                                        int cols, int pitch, half_t* d0, half_t* d1, half_t* d2,
                                                                        float scale) {
  __shared__ float red[32][33];
  const int cx = threadIdx.x & 31, ry = threadIdx.x >> 5;
  const int cblocks = (cols + 31) / 32;
  const int k = blockIdx.x / cblocks, col = (blockIdx.x % cblocks) * 32 + cx;
  float s = 0.f;
  if (col < cols) {
    const float* p = partial + (size_t)k * pitch + col;
    const size_t step = (size_t)nq * pitch;
    int b = ry;
    for (; b + 96 < nblk; b += 128)
      s += (p[b * step] + p[(b + 32) * step]) + (p[(b + 64) * step] + p[(b + 96) * step]);
    for (; b < nblk; b += 32) s += p[b * step];
  }
  red[ry][cx] = s;
  __syncthreads();
  if (ry == 0 && col < cols) {
    float t = red[0][cx];
#pragma unroll
    for (int r = 1; r < 32; ++r) t += red[r][cx];
    half_t* dst = k == 0 ? d0 : (k == 1 ? d1 : d2);
    if (dst) dst[col] = (half_t)(t * scale);
  }
}

// ------------------------------------------------------------------------------------------------
// Column sums of an fp16 matrix (bias gradients): grid (column blocks of 512, row splits).
// ------------------------------------------------------------------------------------------------
constexpr int kColsumMaxSplits = 512;

__global__ void __launch_bounds__(kThreads) colsum_kernel(const half_t* __restrict__ src, int ld, float* __restrict__ partial,
                                                          int rows, int cols) {
  __shared__ float red[kWavesPerBlock][512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = blockIdx.x * 512 + lane * 8;
  const int nsplit = gridDim.y;
  const int per = (rows + nsplit - 1) / nsplit;
  const int r0 = blockIdx.y * per, r1 = min(rows, r0 + per);
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < cols) {
    int r = r0 + wave;
    for (; r + 3 * kWavesPerBlock < r1; r += 4 * kWavesPerBlock) {  // four independent loads in flight
      half8_t h[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) h[u] = ld_half8_nt(src + (size_t)(r + u * kWavesPerBlock) * ld + col);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float v[8];
        unpack8(h[u], v);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += v[e];
      }
    }
    for (; r < r1; r += kWavesPerBlock) {
      float v[8];
      unpack8(ld_half8(src + (size_t)r * ld + col), v);
#pragma unroll
      for (int e = 0; e < 8; ++e) s[e] += v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[wave][lane * 8 + e] = s[e];
  __syncthreads();
  if (wave == 0 && col < cols) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      partial[(size_t)blockIdx.y * cols + col + e] = red[0][lane * 8 + e] + red[1][lane * 8 + e] + red[2][lane * 8 + e] + red[3][lane * 8 + e];
  }
}

// ------------------------------------------------------------------------------------------------
// Fused softmax + label-smoothed cross-entropy + gradient; one block per row, the row held in
// registers (NCH chunks of 8 logits per thread).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_reduce(float v, bool is_max, float* sh) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  float r = sh[0];
#pragma unroll
  for (int w = 1; w < kWavesPerBlock; ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
  return r;
}

template <int NCH>
__global__ void __launch_bounds__(kThreads) softmax_xent_kernel(half_t* __restrict__ logits, const int32_t* __restrict__ targets,
                                                                float* __restrict__ row_loss, int V, int pad_id, float eps_ls,
                                                                float loss_scale) {
  __shared__ float sh[kWavesPerBlock];
  const int row = blockIdx.x;
  const int chunks = V >> 3;
  half_t* z = logits + (size_t)row * V;
  const int y = targets[row];
  if (y == pad_id) {  // padding positions contribute neither loss nor gradient
    for (int c = threadIdx.x; c < chunks; c += kThreads) st_half8(z + c * 8, zero_half8());
    if (threadIdx.x == 0) row_loss[row] = 0.f;
    return;
  }
  // The row stays in registers as fp16.  Pass 1 (maximum, plain sum) runs on pairs of halfs; the two
  // exponential passes fold the shift and the scale into one fused multiply-add in front of the base-2
  // exponential: exp(z - m) = 2^(z log2e - m log2e), loss_scale * exp(z - lse) = 2^(z log2e - lse log2e + log2 loss_scale).
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  struct Pairs { half2_t p[4]; };
  constexpr float kLog2e = 1.4426950408889634f;
  half8_t reg[NCH];
  half2_t mx2 = {(_Float16)-INFINITY, (_Float16)-INFINITY};
  const half2_t ones = {(_Float16)1.f, (_Float16)1.f};
  float sz = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = threadIdx.x + kThreads * i;
    if (c < chunks) {
      reg[i] = ld_half8_nt(z + c * 8);
      const Pairs h = __builtin_bit_cast(Pairs, reg[i]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        mx2 = __builtin_elementwise_max(mx2, h.p[e]);
        sz = __builtin_amdgcn_fdot2(h.p[e], ones, sz, false);
      }
    }
  }
  const int yc = min(max(y, 0), V - 1);
  const float zy = (float)z[yc];
  const float mx = block_reduce(fmaxf((float)mx2[0], (float)mx2[1]), true, sh);
  const float shift = -mx * kLog2e;
  float se = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    if (threadIdx.x + kThreads * i < chunks) {
#pragma unroll
      for (int e = 0; e < 8; ++e) se += __builtin_amdgcn_exp2f(fmaf((float)reg[i][e], kLog2e, shift));
    }
  }
  se = block_reduce(se, false, sh);
  sz = block_reduce(sz, false, sh);
  const float lse = mx + logf(se);
  if (threadIdx.x == 0) row_loss[row] = lse - (1.f - eps_ls) * zy - (eps_ls / (float)V) * sz;
  const float q_scaled = loss_scale * eps_ls / (float)V, hit = loss_scale * (1.f - eps_ls);
  const float shift2 = -lse * kLog2e + log2f(loss_scale);
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = threadIdx.x + kThreads * i;
    if (c < chunks) {
      float g[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) g[e] = __builtin_amdgcn_exp2f(fmaf((float)reg[i][e], kLog2e, shift2)) - q_scaled;
      if (c == (yc >> 3)) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (e == (yc & 7)) g[e] -= hit;
      }
      half8_t o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (half_t)g[e];
      st_half8_nt(z + c * 8, o);
    }
  }
}

// loss_sum = sum of row losses (fixed order), ntok = number of non-pad targets; single block.
__global__ void __launch_bounds__(1024) loss_reduce_kernel(const float* __restrict__ row_loss, const int32_t* __restrict__ targets,
                                                           int rows, int pad_id, float* loss_sum, int32_t* ntok) {
  __shared__ float sl[1024];
  __shared__ int sn[1024];
  float s = 0.f;
  int n = 0;
  for (int r = threadIdx.x; r < rows; r += 1024) {
    s += row_loss[r];
    n += targets[r] != pad_id;
  }
  sl[threadIdx.x] = s;
  sn[threadIdx.x] = n;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      sl[threadIdx.x] += sl[threadIdx.x + o];
      sn[threadIdx.x] += sn[threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *loss_sum = sl[0];
    *ntok = sn[0];
  }
}

// ------------------------------------------------------------------------------------------------
// Embedding backward.  The token positions of both id streams are sorted by id with a stable two-pass
// radix sort (8 bits per pass), so every vocabulary row's positions are contiguous and in increasing
// order.  The sorted list is cut into segments of kEmbSeg entries; one block per segment sums the
// gradient rows of each run of equal ids.  A run that holds all positions of its id is added to the
// row of the shared matrix at once; runs of ids that spill over segment borders leave fp32 partial
// sums, which a second kernel adds up in segment order.  The order of every sum is fixed, so results
// do not depend on scheduling.
// ------------------------------------------------------------------------------------------------
constexpr int kEmbSeg = 64;        // sorted entries per block of the row-summing kernel
constexpr int kSortPerBlock = 1024;  // entries per block of a radix pass

__global__ void fill_int_kernel(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__device__ __forceinline__ int clamp_id(int id, int vocab) { return id < 0 ? 0 : (id >= vocab ? vocab - 1 : id); }
__device__ __forceinline__ int id_at(const int32_t* a, int na, const int32_t* b, int i, int vocab) {
  return clamp_id(i < na ? a[i] : b[i - na], vocab);
}
// Histogram of the ids.  A frequent id (the end-of-sentence symbol, the most common word) would serialise one global
// atomic per occurrence; each block therefore counts its contiguous share of the positions in LDS first, two 16-bit
// counters per word (a block takes at most 65535 positions, so a counter cannot carry into its neighbour), and then
// adds its non-zero counts to the global ones: one global atomic per (block, id that occurs in it).  Integer sums:
// the result does not depend on the order.
constexpr int kHistThreads = 1024;
constexpr int kHistMaxPerBlock = 32768;
__global__ void __launch_bounds__(kHistThreads) emb_hist_kernel(const int32_t* a, int na, const int32_t* b, int nb, int vocab, int per_block,
                                                                int32_t* cnt) {
  extern __shared__ uint32_t hist[];  // (vocab + 1) / 2 words
  const int words = (vocab + 1) >> 1;
  for (int w = threadIdx.x; w < words; w += kHistThreads) hist[w] = 0u;
  __syncthreads();
  const int n = na + nb, lo = min(n, (int)blockIdx.x * per_block), hi = min(n, lo + per_block);
  for (int i = lo + (int)threadIdx.x; i < hi; i += kHistThreads) {
    const int id = id_at(a, na, b, i, vocab);  // clamped to [0, vocab)
    atomicAdd(&hist[id >> 1], 1u << (16 * (id & 1)));
  }
  __syncthreads();
  for (int w = threadIdx.x; w < words; w += kHistThreads) {
    const uint32_t v = hist[w];
    if (v & 0xFFFFu) atomicAdd(&cnt[2 * w], (int32_t)(v & 0xFFFFu));
    if ((v >> 16) && 2 * w + 1 < vocab) atomicAdd(&cnt[2 * w + 1], (int32_t)(v >> 16));
  }
}
// exclusive scan of cnt[0..V) into start[0..V]; single block of 1024 threads
// (start may be cnt itself)
__global__ void __launch_bounds__(1024) emb_scan_kernel(const int32_t* cnt, int32_t* start, int V) {
  __shared__ int sh[1024];
  const int per = (V + 1023) / 1024;
  const int lo = min(V, (int)threadIdx.x * per), hi = min(V, lo + per);
  int s = 0;
  for (int i = lo; i < hi; ++i) s += cnt[i];
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int v = (int)threadIdx.x >= o ? sh[threadIdx.x - o] : 0;
    __syncthreads();
    sh[threadIdx.x] += v;
    __syncthreads();
  }
  int run = sh[threadIdx.x] - s;
  for (int i = lo; i < hi; ++i) {
    const int c = cnt[i];
    start[i] = run;
    run += c;
  }
  if (threadIdx.x == 1023) start[V] = sh[1023];
}

// One radix pass over (key, value) pairs; pass 0 takes key = id of position i, value = i.
// Histogram: hist[digit * nblk + block] = number of the block's entries with that digit, so that an
// exclusive scan of the whole array gives each (digit, block) its first output slot.
__global__ void __launch_bounds__(kThreads) radix_hist_kernel(const int32_t* a, int na, const int32_t* b, int vocab,
                                                              const int32_t* __restrict__ keys, int n, int shift, int nblk,
                                                              int32_t* __restrict__ hist) {
  __shared__ int h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int base = blockIdx.x * kSortPerBlock;
  for (int r = 0; r < kSortPerBlock / kThreads; ++r) {
    const int i = base + r * kThreads + threadIdx.x;
    if (i < n) atomicAdd(&h[((keys ? keys[i] : id_at(a, na, b, i, vocab)) >> shift) & 255], 1);
  }
  __syncthreads();
  hist[threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}
// Stable scatter: entries keep their order within a digit.  The block's four wavefronts take turns;
// within a wavefront the lanes holding the same digit are found with eight ballots.
__global__ void __launch_bounds__(kThreads) radix_scatter_kernel(const int32_t* a, int na, const int32_t* b, int vocab,
                                                                 const int32_t* __restrict__ keys, const int32_t* __restrict__ vals,
                                                                 int n, int shift, int nblk, const int32_t* __restrict__ offs,
                                                                 int32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out) {
  __shared__ int next[256];
  next[threadIdx.x] = offs[threadIdx.x * nblk + blockIdx.x];
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int base = blockIdx.x * kSortPerBlock;
  for (int r = 0; r < kSortPerBlock / kThreads; ++r) {
    const int i = base + r * kThreads + threadIdx.x;
    const bool valid = i < n;
    const int key = valid ? (keys ? keys[i] : id_at(a, na, b, i, vocab)) : 0;
    const int val = valid ? (vals ? vals[i] : i) : 0;
    const int digit = (key >> shift) & 255;
    for (int w = 0; w < kThreads / kWave; ++w) {
      if (wave == w) {
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
          const unsigned long long set = __ballot((digit >> bit) & 1);
          peers &= ((digit >> bit) & 1) ? set : ~set;
        }
        if (valid) {
          const int rank = __popcll(peers & ((1ull << lane) - 1ull));
          const int slot = next[digit] + rank;
          keys_out[slot] = key;
          vals_out[slot] = val;
          if (rank == 0) next[digit] += __popcll(peers);   // every peer has read next[digit] (lock-step) before this write
        }
      }
      __syncthreads();
    }
  }
}

// dropout-masked, unscaled gradient chunk (8 columns) of sorted entry `pos`
__device__ __forceinline__ void emb_row_chunk(int pos, int c, int d, const half_t* __restrict__ dxa, int na, const DropDev& da,
                                              const half_t* __restrict__ dxb, const DropDev& db, float (&acc)[8]) {
  const bool in_a = pos < na;
  const int row = in_a ? pos : pos - na;
  const DropDev& dd = in_a ? da : db;
  float x[8];
  unpack8(ld_half8((in_a ? dxa : dxb) + (size_t)row * d + c * 8), x);
  uint32_t bits = 0xFFu;
  float sc = 1.f;
  if (dd.thr) {
    bits = drop_keep8(dd, (uint32_t)row, (uint32_t)c);
    sc = dd.scale;
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] += ((bits >> e) & 1u) ? x[e] * sc : 0.f;
}
__device__ __forceinline__ void emb_add_to_row(half_t* __restrict__ gE, int v, int c, int d, const float (&tot)[8], float scale) {
  half_t* dst = gE + (size_t)v * d + c * 8;
  float cur[8];
  unpack8(ld_half8(dst), cur);
  const float sq = sqrtf((float)d) * scale;
#pragma unroll
  for (int e = 0; e < 8; ++e) cur[e] += sq * tot[e];
  st_half8(dst, pack8(cur));
}

// One block per segment of kEmbSeg sorted entries, one thread per 8 columns.
// part[(2 * seg + 0) * d ..]: sum of the segment's first run if that run began in an earlier segment;
// part[(2 * seg + 1) * d ..]: sum of its last run if that run began here and goes on in the next one.
__global__ void __launch_bounds__(kThreads) emb_segment_kernel(const int32_t* a, const half_t* __restrict__ dxa, int na, DropDev da,
                                                               const int32_t* b, const half_t* __restrict__ dxb, int nb, DropDev db,
                                                               half_t* __restrict__ gE, int d, int vocab,
                                                               const int32_t* __restrict__ start, const int32_t* __restrict__ perm,
                                                               float* __restrict__ part, float scale) {
  __shared__ int s_pos[kEmbSeg], s_id[kEmbSeg];
  const int n = na + nb, e0 = blockIdx.x * kEmbSeg, cnt = min(kEmbSeg, n - e0);
  if ((int)threadIdx.x < cnt) {
    const int pos = perm[e0 + threadIdx.x];
    s_pos[threadIdx.x] = pos;
    s_id[threadIdx.x] = id_at(a, na, b, pos, vocab);
  }
  __syncthreads();
  const int c = threadIdx.x;
  if (c >= (d >> 3)) return;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int run_begin = 0;
  for (int k = 0; k < cnt; ++k) {
    emb_row_chunk(s_pos[k], c, d, dxa, na, da, dxb, db, acc);
    const int v = s_id[k];
    if (k + 1 < cnt && s_id[k + 1] == v) continue;
    const int g_begin = start[v], g_end = start[v + 1];  // where id v's positions lie in the sorted list
    if (g_begin == e0 + run_begin && g_end == e0 + k + 1) {
      emb_add_to_row(gE, v, c, d, acc, scale);
    } else {
      float* dst = part + ((size_t)2 * blockIdx.x + (g_begin < e0 ? 0 : 1)) * d + c * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[e] = acc[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    run_begin = k + 1;
  }
}
// Block s finishes the id whose run began in an earlier segment and ends in segment s.
__global__ void __launch_bounds__(kThreads) emb_finish_kernel(const int32_t* a, int na, const int32_t* b, int nb, half_t* __restrict__ gE,
                                                              int d, int vocab, const int32_t* __restrict__ start,
                                                              const int32_t* __restrict__ perm, const float* __restrict__ part,
                                                              float scale) {
  const int e0 = blockIdx.x * kEmbSeg;
  const int v = id_at(a, na, b, perm[e0], vocab);
  const int g_begin = start[v], g_end = start[v + 1];
  if (g_begin >= e0 || g_end > e0 + kEmbSeg) return;  // no run carried in, or it goes on: a later block finishes it
  const int c = threadIdx.x;
  if (c >= (d >> 3)) return;
  const int first = g_begin / kEmbSeg;
  float tot[8];
  const float* p = part + ((size_t)2 * first + 1) * d + c * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) tot[e] = p[e];
  for (int sg = first + 1; sg <= (int)blockIdx.x; ++sg) {
    p = part + (size_t)2 * sg * d + c * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) tot[e] += p[e];
  }
  emb_add_to_row(gE, v, c, d, tot, scale);
}

__global__ void __launch_bounds__(kThreads) dropout_mask_kernel(uint8_t* keep, int rows, int n_cols, DropDev drop) {
  const int groups = (n_cols + 7) >> 3;
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (gid >= (int64_t)rows * groups) return;
  const int row = (int)(gid / groups), grp = (int)(gid % groups);
  const uint32_t bits = drop.thr ? drop_keep8(drop, (uint32_t)row, (uint32_t)grp) : 0xFFu;
  for (int e = 0; e < 8; ++e) {
    const int col = grp * 8 + e;
    if (col < n_cols) keep[(size_t)row * n_cols + col] = (bits >> e) & 1u;
  }
}

int ln_nch(int d) { return d <= 512 ? 1 : (d <= 1024 ? 2 : 4); }

}  // namespace

// ------------------------------------------------------------------------------------------------
// Row keys and sentence tables of a group of sub-batches: one thread per sentence.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) build_tables_kernel(const SegmentList sl, int n_sent, const uint32_t* __restrict__ uid,
                                                               uint2* __restrict__ rk_src, uint2* __restrict__ rk_tgt,
                                                               int4* __restrict__ tab_ss, int4* __restrict__ tab_tt,
                                                               int4* __restrict__ tab_ts) {
  const int sb = blockIdx.x * kThreads + threadIdx.x;
  if (sb >= n_sent) return;
  int seg = 0, first = 0, src0 = 0, tgt0 = 0;  // first sentence / source row / target row of the segment
  while (seg + 1 < sl.n && sb >= first + sl.B[seg]) {
    first += sl.B[seg];
    src0 += sl.B[seg] * sl.S[seg];
    tgt0 += sl.B[seg] * sl.T[seg];
    ++seg;
  }
  const int b = sb - first, S = sl.S[seg], T = sl.T[seg];
  const int srow = src0 + b * S, trow = tgt0 + b * T;
  const uint32_t id = uid ? uid[sb] : (uint32_t)b;
  const uint32_t hi = sl.micro[seg] << 16;
  tab_ss[sb] = make_int4(srow, srow, S, S);
  tab_tt[sb] = make_int4(trow, trow, T, T);
  tab_ts[sb] = make_int4(trow, srow, T, S);
  for (int t = 0; t < S; ++t) rk_src[srow + t] = make_uint2(id, hi | (uint32_t)t);
  for (int t = 0; t < T; ++t) rk_tgt[trow + t] = make_uint2(id, hi | (uint32_t)t);
}

// Packed sentences: exclusive prefix sums of the clamped lengths (one block of 1024 threads) ...
__global__ void __launch_bounds__(1024) packed_rows_kernel(const nmt_sentence* __restrict__ sent, int n_sent, int max_src, int max_tgt,
                                                           int32_t* __restrict__ rows) {
  __shared__ int sh_s[1024], sh_t[1024];
  const int per = (n_sent + 1023) / 1024;
  const int lo = min(n_sent, (int)threadIdx.x * per), hi = min(n_sent, lo + per);
  int ss = 0, tt = 0;
  for (int i = lo; i < hi; ++i) {
    ss += min(max(sent[i].src_len, 1), max_src);
    tt += min(max(sent[i].tgt_len, 1), max_tgt);
  }
  sh_s[threadIdx.x] = ss;
  sh_t[threadIdx.x] = tt;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int vs = (int)threadIdx.x >= o ? sh_s[threadIdx.x - o] : 0, vt = (int)threadIdx.x >= o ? sh_t[threadIdx.x - o] : 0;
    __syncthreads();
    sh_s[threadIdx.x] += vs;
    sh_t[threadIdx.x] += vt;
    __syncthreads();
  }
  int rs = sh_s[threadIdx.x] - ss, rt = sh_t[threadIdx.x] - tt;
  for (int i = lo; i < hi; ++i) {
    rows[2 * i] = rs;
    rows[2 * i + 1] = rt;
    rs += min(max(sent[i].src_len, 1), max_src);
    rt += min(max(sent[i].tgt_len, 1), max_tgt);
  }
}
// ... then one thread per sentence writes its table entries and row keys.
__global__ void __launch_bounds__(kThreads) packed_tables_kernel(const nmt_sentence* __restrict__ sent, int n_sent, int n_src, int n_tgt,
                                                                int max_src, int max_tgt, const int32_t* __restrict__ rows,
                                                                uint2* __restrict__ rk_src, uint2* __restrict__ rk_tgt,
                                                                int4* __restrict__ tab_ss, int4* __restrict__ tab_tt,
                                                                int4* __restrict__ tab_ts) {
  const int sb = blockIdx.x * kThreads + threadIdx.x;
  if (sb >= n_sent) return;
  const nmt_sentence se = sent[sb];
  // rows past the totals the host sized everything for do not exist: a sentence is cut there
  const int srow = min(rows[2 * sb], n_src - 1), trow = min(rows[2 * sb + 1], n_tgt - 1);
  const int S = min(min(max(se.src_len, 1), max_src), n_src - srow), T = min(min(max(se.tgt_len, 1), max_tgt), n_tgt - trow);
  const uint32_t hi = (se.micro_idx & 0xFFu) << 16;
  tab_ss[sb] = make_int4(srow, srow, S, S);
  tab_tt[sb] = make_int4(trow, trow, T, T);
  tab_ts[sb] = make_int4(trow, srow, T, S);
  for (int t = 0; t < S; ++t) rk_src[srow + t] = make_uint2(se.uid, hi | (uint32_t)t);
  for (int t = 0; t < T; ++t) rk_tgt[trow + t] = make_uint2(se.uid, hi | (uint32_t)t);
}

// ================================================================================================
// launchers
// ================================================================================================
int launch_embed_fwd(const int32_t* ids, const half_t* E, half_t* x, int rows, int d, int vocab, const DropDev& drop,
                     hipStream_t stream) {
  NMT_REQUIRE(rows > 0 && d > 0 && d % 8 == 0 && vocab > 0, "embed_fwd: bad shape rows=%d d=%d", rows, d);
  NMT_REQUIRE(ids && E && x && aligned16(E) && aligned16(x), "embed_fwd: null or misaligned pointer");
  NMT_REQUIRE(drop.n_pos > 0, "embed_fwd: positions per sentence must be positive");
  const int64_t n = (int64_t)rows * (d / 8);
  hipLaunchKernelGGL(embed_fwd_kernel, dim3(ceil_div(n, kThreads)), dim3(kThreads), 0, stream, ids, E, x, rows, d, vocab, drop);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_residual_layernorm_fwd(const half_t* sub, const half_t* resid, const half_t* gamma, const half_t* beta,
                                  half_t* out, float* stats, int rows, int d, float eps, const DropDev& drop,
                                  hipStream_t stream) {
  NMT_REQUIRE(rows > 0 && d >= 8 && d % 8 == 0 && d <= 2048, "layernorm: d=%d must be a multiple of 8 in [8, 2048]", d);
  NMT_REQUIRE(sub && resid && gamma && beta && out && stats, "layernorm: null pointer");
  NMT_REQUIRE(aligned16(sub) && aligned16(resid) && aligned16(gamma) && aligned16(beta) && aligned16(out), "layernorm: misaligned pointer");
  NMT_REQUIRE(!drop.thr || drop.n_pos > 0, "layernorm: positions per sentence must be positive");
  const dim3 grid(ceil_div(rows, kWavesPerBlock)), block(kThreads);
  switch (ln_nch(d)) {
    case 1: hipLaunchKernelGGL(res_ln_fwd_kernel<1>, grid, block, 0, stream, sub, resid, gamma, beta, out, stats, rows, d, eps, drop); break;
    case 2: hipLaunchKernelGGL(res_ln_fwd_kernel<2>, grid, block, 0, stream, sub, resid, gamma, beta, out, stats, rows, d, eps, drop); break;
    default: hipLaunchKernelGGL(res_ln_fwd_kernel<4>, grid, block, 0, stream, sub, resid, gamma, beta, out, stats, rows, d, eps, drop); break;
  }
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int64_t layernorm_bwd_scratch_floats(int d) { return (int64_t)kLnBwdMaxBlocks * 3 * ln_nch(d) * 512; }

int launch_residual_layernorm_bwd(const half_t* dout, const half_t* sub, const half_t* resid, const half_t* gamma,
                                  const float* stats, half_t* dy, half_t* dym, half_t* dgamma, half_t* dbeta,
                                  half_t* dbias, float* partial, int rows, int d, const DropDev& drop,
                                  hipStream_t stream, float vec_scale) {
  NMT_REQUIRE(rows > 0 && d >= 8 && d % 8 == 0 && d <= 2048, "layernorm_bwd: d=%d must be a multiple of 8 in [8, 2048]", d);
  NMT_REQUIRE(dout && sub && resid && gamma && stats && dy && partial, "layernorm_bwd: null pointer");
  NMT_REQUIRE(aligned16(dout) && aligned16(sub) && aligned16(resid) && aligned16(gamma) && aligned16(dy) && aligned16(dym),
              "layernorm_bwd: misaligned pointer");
  NMT_REQUIRE(!drop.thr || (drop.n_pos > 0 && dym), "layernorm_bwd: dropout needs the masked output and positions per sentence");
  const int nch = ln_nch(d);
  // a grid that is resident at once (3 or 4 work-groups per compute unit fit, by registers): no second, partly filled round
  const int resident = (nch >= 2 ? 3 : 4) * device_info().cus;
  const int nblk = min(min(kLnBwdMaxBlocks, resident), ceil_div(rows, kWavesPerBlock * kLnRows));
  const dim3 grid(nblk), block(kThreads);
  const size_t smem = (size_t)3 * nch * 512 * sizeof(float);
  switch (nch) {
    case 1: hipLaunchKernelGGL(res_ln_bwd_kernel<1>, grid, block, smem, stream, dout, sub, resid, gamma, stats, dy, dym, partial, rows, d, drop); break;
    case 2: hipLaunchKernelGGL(res_ln_bwd_kernel<2>, grid, block, smem, stream, dout, sub, resid, gamma, stats, dy, dym, partial, rows, d, drop); break;
    default: hipLaunchKernelGGL(res_ln_bwd_kernel<4>, grid, block, smem, stream, dout, sub, resid, gamma, stats, dy, dym, partial, rows, d, drop); break;
  }
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(finalize_partials_kernel, dim3(3 * ceil_div(d, 32)), dim3(kFinThreads), 0, stream, partial, nblk, 3, d,
                     nch * 512, dgamma, dbeta, dbias, vec_scale);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int64_t colsum_scratch_floats(int cols) { return (int64_t)kColsumMaxSplits * cols; }

// ------------------------------------------------------------------------------------------------
// Column sums for callers that cannot allocate (code under graph capture, serving loops): the partial
// sums live in a fixed device array instead of a caller-provided buffer.  Each GPU holds its own copy of
// the array at its own address, looked up once per device; every call on a GPU shares that copy.
// ------------------------------------------------------------------------------------------------
constexpr int kStaticColsumMaxCols = 4096;
static __device__ __align__(256) float scratch[(size_t)kColsumMaxSplits * kStaticColsumMaxCols];  // 8 MiB per GPU

namespace {
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;
// Device address of `scratch` on the current device (its name is only a host-side stand-in for it).
int static_scratch(float** out) {
  int dev = 0;
  NMT_HIP_CHECK(hipGetDevice(&dev));
  NMT_REQUIRE(dev >= 0 && dev < kMaxDevices, "colsum_static: device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    NMT_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    NMT_REQUIRE(p, "colsum_static: the scratch array has no device address");
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return NMT_OK;
}
}  // namespace

int launch_colsum_static(const half_t* src, int ld, half_t* dst, int rows, int cols, hipStream_t stream) {
  NMT_REQUIRE(cols > 0 && cols <= kStaticColsumMaxCols, "colsum_static: cols=%d outside [1, %d], the width the fixed scratch array holds", cols,
              kStaticColsumMaxCols);
  float* partial = nullptr;
  if (int rc = static_scratch(&partial)) return rc;
  // every partial sum the second kernel reads is written by the first one of the same call: nothing to clear
  return launch_colsum(src, ld, dst, partial, rows, cols, stream, 1.f);
}

int launch_colsum(const half_t* src, int ld, half_t* dst, float* partial, int rows, int cols, hipStream_t stream, float scale) {
  NMT_REQUIRE(rows > 0 && cols > 0 && cols % 8 == 0 && ld % 8 == 0 && ld >= cols, "colsum: bad shape rows=%d cols=%d ld=%d", rows, cols, ld);
  NMT_REQUIRE(src && dst && partial && aligned16(src), "colsum: null or misaligned pointer");
  const int cb = ceil_div(cols, 512);
  int splits = 2048 / cb;  // enough blocks to keep every compute unit streaming
  splits = splits > kColsumMaxSplits ? kColsumMaxSplits : splits;
  splits = splits > rows / 16 ? rows / 16 : splits;
  splits = splits < 1 ? 1 : splits;
  hipLaunchKernelGGL(colsum_kernel, dim3(cb, splits), dim3(kThreads), 0, stream, src, ld, partial, rows, cols);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(finalize_partials_kernel, dim3(ceil_div(cols, 32)), dim3(kFinThreads), 0, stream, partial, splits, 1, cols,
                     cols, dst, (half_t*)nullptr, (half_t*)nullptr, scale);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_softmax_xent(half_t* logits, const int32_t* targets, float* row_loss, int rows, int V, int pad_id, float eps_ls,
                        float loss_scale, float* loss_sum, int32_t* ntok, hipStream_t stream) {
  NMT_REQUIRE(rows > 0 && V >= 8 && V % 8 == 0 && V <= 65536, "softmax_xent: V=%d must be a multiple of 8 in [8, 65536]", V);
  NMT_REQUIRE(logits && targets && row_loss && loss_sum && ntok && aligned16(logits), "softmax_xent: null or misaligned pointer");
  const dim3 grid(rows), block(kThreads);
  const int nch = ceil_div(V / 8, kThreads);
#define NMT_XENT(N) hipLaunchKernelGGL(softmax_xent_kernel<N>, grid, block, 0, stream, logits, targets, row_loss, V, pad_id, eps_ls, loss_scale)
  if (nch <= 1) NMT_XENT(1);
  else if (nch <= 4) NMT_XENT(4);
  else if (nch <= 16) NMT_XENT(16);
  else if (nch <= 20) NMT_XENT(20);
  else NMT_XENT(32);
#undef NMT_XENT
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, stream, row_loss, targets, rows, pad_id, loss_sum, ntok);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

namespace {
struct EmbScratch {
  int64_t cnt, start, k1, v1, k2, perm, hist, part, total;  // offsets in int32 units
  int nblk, nseg;
};
EmbScratch emb_scratch(int vocab, int n, int d) {
  EmbScratch e;
  e.nblk = ceil_div(n, kSortPerBlock);
  e.nseg = ceil_div(n, kEmbSeg);
  int64_t cur = 0;
  auto take = [&](int64_t ints) {
    const int64_t off = cur;
    cur += round_up(ints, 4);
    return off;
  };
  e.cnt = take(vocab);
  e.start = take(vocab + 1);
  e.k1 = take(n);
  e.v1 = take(n);
  e.k2 = take(n);
  e.perm = take(n);
  e.hist = take((int64_t)256 * e.nblk + 1);
  e.part = take((int64_t)2 * e.nseg * d);
  e.total = cur;
  return e;
}
}  // namespace

int64_t embed_bwd_scratch_ints(int vocab, int rows_total, int d) { return emb_scratch(vocab, rows_total, d).total; }

int launch_embed_bwd(const int32_t* ids_a, const half_t* dx_a, int rows_a, const DropDev& drop_a, const int32_t* ids_b,
                     const half_t* dx_b, int rows_b, const DropDev& drop_b, half_t* gE, int d, int vocab, int32_t* scratch,
                     hipStream_t stream, float scale) {
  NMT_REQUIRE(rows_a >= 0 && rows_b >= 0 && rows_a + rows_b > 0, "embed_bwd: no rows");
  NMT_REQUIRE(d >= 8 && d % 8 == 0 && d / 8 <= kThreads && vocab > 0 && vocab <= 65536, "embed_bwd: bad d=%d or vocab=%d", d, vocab);
  NMT_REQUIRE((rows_a == 0 || (ids_a && dx_a && aligned16(dx_a))) && (rows_b == 0 || (ids_b && dx_b && aligned16(dx_b))) && gE &&
                  aligned16(gE) && scratch && aligned16(scratch),
              "embed_bwd: null or misaligned pointer");
  NMT_REQUIRE((!drop_a.thr || drop_a.n_pos > 0) && (!drop_b.thr || drop_b.n_pos > 0), "embed_bwd: positions per sentence must be positive");
  const int n = rows_a + rows_b;
  const EmbScratch e = emb_scratch(vocab, n, d);
  int32_t *cnt = scratch + e.cnt, *start = scratch + e.start, *k1 = scratch + e.k1, *v1 = scratch + e.v1, *k2 = scratch + e.k2;
  int32_t *perm = scratch + e.perm, *hist = scratch + e.hist;
  float* part = reinterpret_cast<float*>(scratch + e.part);
  hipLaunchKernelGGL(fill_int_kernel, dim3(ceil_div(vocab, kThreads)), dim3(kThreads), 0, stream, cnt, vocab, 0);
  NMT_LAUNCH_CHECK();
  {
    // one block per compute unit, more if a block's share would exceed what its 16-bit counters hold
    int blocks = device_info().cus;
    if (ceil_div(n, blocks) > kHistMaxPerBlock) blocks = ceil_div(n, kHistMaxPerBlock);
    const int per_block = ceil_div(n, blocks);
    const size_t hist_bytes = (size_t)((vocab + 1) / 2) * sizeof(uint32_t);
    if (hist_bytes > 64 * 1024)
      NMT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(emb_hist_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)hist_bytes));
    hipLaunchKernelGGL(emb_hist_kernel, dim3(blocks), dim3(kHistThreads), hist_bytes, stream, ids_a, rows_a, ids_b, rows_b, vocab, per_block, cnt);
    NMT_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(emb_scan_kernel, dim3(1), dim3(1024), 0, stream, cnt, start, vocab);
  NMT_LAUNCH_CHECK();
  // stable sort of the positions by id: low byte, then high byte
  const int nh = 256 * e.nblk;
  hipLaunchKernelGGL(radix_hist_kernel, dim3(e.nblk), dim3(kThreads), 0, stream, ids_a, rows_a, ids_b, vocab, (const int32_t*)nullptr, n, 0,
                     e.nblk, hist);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(emb_scan_kernel, dim3(1), dim3(1024), 0, stream, hist, hist, nh);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(radix_scatter_kernel, dim3(e.nblk), dim3(kThreads), 0, stream, ids_a, rows_a, ids_b, vocab, (const int32_t*)nullptr,
                     (const int32_t*)nullptr, n, 0, e.nblk, hist, k1, v1);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(radix_hist_kernel, dim3(e.nblk), dim3(kThreads), 0, stream, ids_a, rows_a, ids_b, vocab, k1, n, 8, e.nblk, hist);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(emb_scan_kernel, dim3(1), dim3(1024), 0, stream, hist, hist, nh);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(radix_scatter_kernel, dim3(e.nblk), dim3(kThreads), 0, stream, ids_a, rows_a, ids_b, vocab, k1, v1, n, 8, e.nblk, hist,
                     k2, perm);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(emb_segment_kernel, dim3(e.nseg), dim3(kThreads), 0, stream, ids_a, dx_a, rows_a, drop_a, ids_b, dx_b, rows_b, drop_b, gE,
                     d, vocab, start, perm, part, scale);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(emb_finish_kernel, dim3(e.nseg), dim3(kThreads), 0, stream, ids_a, rows_a, ids_b, rows_b, gE, d, vocab, start, perm, part, scale);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_dropout_mask(uint8_t* keep, int rows, int n_cols, const DropDev& drop, hipStream_t stream) {
  NMT_REQUIRE(keep && rows > 0 && n_cols > 0, "dropout_mask: bad arguments");
  NMT_REQUIRE(!drop.thr || drop.n_pos > 0, "dropout_mask: positions per sentence must be positive");
  const int64_t n = (int64_t)rows * ((n_cols + 7) / 8);
  hipLaunchKernelGGL(dropout_mask_kernel, dim3(ceil_div(n, kThreads)), dim3(kThreads), 0, stream, keep, rows, n_cols, drop);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_build_tables(const SegmentList& segs, int n_sent, const uint32_t* uid, uint2* rk_src, uint2* rk_tgt, int4* tab_ss,
                        int4* tab_tt, int4* tab_ts, hipStream_t stream) {
  NMT_REQUIRE(segs.n >= 1 && segs.n <= NMT_MAX_SEGMENTS && n_sent > 0, "build_tables: bad segment list");
  NMT_REQUIRE(rk_src && rk_tgt && tab_ss && tab_tt && tab_ts, "build_tables: null pointer");
  hipLaunchKernelGGL(build_tables_kernel, dim3(ceil_div(n_sent, kThreads)), dim3(kThreads), 0, stream, segs, n_sent, uid, rk_src, rk_tgt,
                     tab_ss, tab_tt, tab_ts);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_build_tables_packed(const nmt_sentence* sentences, int n_sent, int n_src, int n_tgt, int max_src, int max_tgt,
                               int32_t* sent_rows, uint2* rk_src, uint2* rk_tgt, int4* tab_ss, int4* tab_tt, int4* tab_ts,
                               hipStream_t stream) {
  NMT_REQUIRE(sentences && n_sent > 0 && n_src >= n_sent && n_tgt >= n_sent && max_src > 0 && max_tgt > 0, "build_tables: bad packed batch");
  NMT_REQUIRE(sent_rows && rk_src && rk_tgt && tab_ss && tab_tt && tab_ts, "build_tables: null pointer");
  hipLaunchKernelGGL(packed_rows_kernel, dim3(1), dim3(1024), 0, stream, sentences, n_sent, max_src, max_tgt, sent_rows);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(packed_tables_kernel, dim3(ceil_div(n_sent, kThreads)), dim3(kThreads), 0, stream, sentences, n_sent, n_src, n_tgt,
                     max_src, max_tgt, sent_rows, rk_src, rk_tgt, tab_ss, tab_tt, tab_ts);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}
