// Fused masked multi-head attention for gfx950: forward with online softmax, and backward as two
// kernels (dK/dV: a wavefront owns 32 keys and sweeps the queries; dQ: a wavefront owns 32 queries
// and sweeps the keys).  K/V (or Q/dO) tiles of one (sentence, head) live in LDS; scores never go
// to memory.  All products run on 32x32x16 fp16 MFMAs.
//
// Register layouts (v_mfma_f32_32x32x16_f16, D = A x B): A lane l holds row l%32, k = 8*(l/32)+j;
// B lane l holds column l%32, same k; D lane l holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4
// for r = 0..15.  Scores are produced transposed where that puts the softmax row (the query) on a
// lane, so that row statistics are per-lane scalars; probabilities are fed to the second product
// straight from registers: the contraction index may be permuted freely as long as both operands
// use the same permutation, so slot j of k-step s2 stands for row 16*s2 + 8*(j/4) + 4*(l/32) + j%4.
#include <math.h>

#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kQC = 64;   // queries staged per pass of the dK/dV kernel
constexpr int kKC = 128;  // keys staged per pass of the dQ kernel

struct AttnArgs {
  const half_t *Q, *K, *V, *O, *dO;
  half_t *Out, *dQ, *dK, *dV;
  float* lse;
  const int32_t* key_ids;
  int ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv;
  int pad_id, causal, B, H, Tq, Tk;  // with a sentence table: Tq, Tk are the largest lengths in it
  const int4* tab;                   // per sentence (first query row, first key row, Tq, Tk), or nullptr
  int Nq;                            // query rows in total: lse is [H, Nq]
};

// Rows and lengths of sentence b: from the table when several batches of different shapes are
// stacked row-wise, else sentence b of one rectangular batch.
struct Sent {
  int q0, k0, Tq, Tk;
};
__device__ __forceinline__ Sent sentence(const AttnArgs& a, int b) {
  if (a.tab) {
    const int4 t = a.tab[b];
    return Sent{t.x, t.y, t.z, t.w};
  }
  return Sent{b * a.Tq, b * a.Tk, a.Tq, a.Tk};
}

__device__ __forceinline__ half8_t join4(half4_t a, half4_t b) {
  half8_t r;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    r[e] = a[e];
    r[4 + e] = b[e];
  }
  return r;
}
__device__ __forceinline__ floatx16 zero16() {
  floatx16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef short short8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) short4_t* lds_short4_ptr;

// A-operand fragment of X^T taken from a row-major LDS tile X[k][DH] (pitch in halfs) with the gfx950
// transposing read: MFMA tile t covers columns 32t..32t+31 of X (rows of X^T); slot j of the lane
// stands for k row kbase + 8*(j/4) + j%4, where kbase already contains 4*(lane/32).
template <int DH>
__device__ __forceinline__ half8_t tr_frag(const half_t* x, int pitch, int kbase, int t, int lane) {
  const int q = lane >> 4, i = lane & 15;
  const bool live = DH >= 32 || !(q & 1);   // head sizes below 32 fill only half of the MFMA rows
  const int col = live ? t * 32 + 16 * (q & 1) + 4 * (i & 3) : 0;
  const half_t* p = x + (kbase + (i >> 2)) * pitch + col;
  short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p));
  short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p + 8 * pitch));
  if (!live) {
    lo = short4_t{0, 0, 0, 0};
    hi = lo;
  }
  const short8_t r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(half8_t, r);
}

// Stage rows [r_begin, r_begin + nrows_pad) of a [*, DH] head slice into LDS, row-major (pitch DH+8);
// rows >= r_end are zero.
template <int DH>
__device__ __forceinline__ void stage_rows(const half_t* __restrict__ src, int ld, int r_begin, int r_end, int nrows_pad,
                                           half_t* row_major) {
  constexpr int CH = DH / 8, PR = DH + 8;
  for (int idx = threadIdx.x; idx < nrows_pad * CH; idx += kThreads) {
    const int rl = idx / CH, c = idx % CH;
    const int r = r_begin + rl;
    st_half8(row_major + rl * PR + c * 8, r < r_end ? ld_half8(src + (size_t)r * ld + c * 8) : zero_half8());
  }
}

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ void __launch_bounds__(kThreads) attn_fwd_kernel(const AttnArgs a) {
  constexpr int DHP = DH < 32 ? 32 : DH, KS = DH / 16, DT = DHP / 32, PR = DH + 8;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
  const Sent se = sentence(a, b);
  if ((int)blockIdx.y * 128 >= se.Tq) return;
  const int KP = (se.Tk + 31) & ~31;
  half_t* Ks = reinterpret_cast<half_t*>(smem_raw);
  half_t* Vs = Ks + KP * PR;
  uint8_t* hidk = reinterpret_cast<uint8_t*>(Vs + KP * PR);

  stage_rows<DH>(a.K + (size_t)se.k0 * a.ldk + h * DH, a.ldk, 0, se.Tk, KP, Ks);
  stage_rows<DH>(a.V + (size_t)se.k0 * a.ldv + h * DH, a.ldv, 0, se.Tk, KP, Vs);
  for (int k = threadIdx.x; k < KP; k += kThreads) hidk[k] = (k >= se.Tk) || (a.key_ids && a.key_ids[se.k0 + k] == a.pad_id);
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int q0 = blockIdx.y * 128 + wave * 32;
  if (q0 >= se.Tq) return;
  const int q = q0 + (lane & 31);
  const bool qvalid = q < se.Tq;
  half8_t qf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s)
    qf[s] = qvalid ? ld_half8(a.Q + (size_t)(se.q0 + q) * a.ldq + h * DH + s * 16 + g * 8) : zero_half8();

  const float sc = rsqrtf((float)DH) * kLog2e;
  float m = -1e30f, l = 0.f;
  floatx16 oacc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) oacc[t] = zero16();
  int nkt = KP / 32;
  if (a.causal) nkt = min(nkt, (q0 + 31) / 32 + 1);
  for (int kt = 0; kt < nkt; ++kt) {
    floatx16 s = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s = MFMA(ld_half8(Ks + (kt * 32 + (lane & 31)) * PR + ks * 16 + g * 8), qf[ks], s);
    float tmax = -1e30f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = kt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
      const bool hid = hidk[key] || (a.causal && key > q);
      s[r] = hid ? -INFINITY : s[r] * sc;
      tmax = fmaxf(tmax, s[r]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m, tmax);
    const float alpha = exp2f(m - m_new);
    m = m_new;
    float psum = 0.f;
    half8_t pf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = exp2f(s[r] - m_new);
      psum += p;
      pf[r >> 3][r & 7] = (half_t)p;
    }
    l = l * alpha + psum;
#pragma unroll
    for (int t = 0; t < DT; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[t][r] *= alpha;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        oacc[t] = MFMA(tr_frag<DH>(Vs, PR, kt * 32 + 16 * s2 + 4 * g, t, lane), pf[s2], oacc[t]);
      }
    }
  }
  l += __shfl_xor(l, 32, kWave);
  if (!qvalid) return;
  const float inv = 1.f / l;
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int dh0 = t * 32 + 8 * rq + 4 * g;
      if (dh0 < DH) {
        half4_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (half_t)(oacc[t][4 * rq + e] * inv);
        *reinterpret_cast<half4_t*>(a.Out + (size_t)(se.q0 + q) * a.ldo + h * DH + dh0) = o;
      }
    }
  if (g == 0) a.lse[(size_t)h * a.Nq + se.q0 + q] = (m + log2f(l)) * kLn2;
}

// ------------------------------------------------------------------------------------------------
// backward, dK and dV
// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ void __launch_bounds__(kThreads) attn_bwd_dkv_kernel(const AttnArgs a) {
  constexpr int DHP = DH < 32 ? 32 : DH, KS = DH / 16, DT = DHP / 32, PR = DH + 8, CH = DH / 8;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  half_t* Qs = reinterpret_cast<half_t*>(smem_raw);
  half_t* dOs = Qs + kQC * PR;
  float* lse_s = reinterpret_cast<float*>(dOs + kQC * PR);
  float* D_s = lse_s + kQC;

  const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
  const Sent se = sentence(a, b);
  if ((int)blockIdx.y * 128 >= se.Tk) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int k0 = blockIdx.y * 128 + wave * 32;
  const int key = k0 + (lane & 31);
  const bool kvalid = key < se.Tk;
  const bool khid = !kvalid || (a.key_ids && a.key_ids[se.k0 + key] == a.pad_id);
  half8_t kf[KS], vf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    kf[s] = kvalid ? ld_half8(a.K + (size_t)(se.k0 + key) * a.ldk + h * DH + s * 16 + g * 8) : zero_half8();
    vf[s] = kvalid ? ld_half8(a.V + (size_t)(se.k0 + key) * a.ldv + h * DH + s * 16 + g * 8) : zero_half8();
  }
  floatx16 dKt[DT], dVt[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) {
    dKt[t] = zero16();
    dVt[t] = zero16();
  }
  const float scale = rsqrtf((float)DH), sc = scale * kLog2e;
  const half_t* Qb = a.Q + (size_t)se.q0 * a.ldq + h * DH;
  const half_t* dOb = a.dO + (size_t)se.q0 * a.lddo + h * DH;
  const half_t* Ob = a.O + (size_t)se.q0 * a.ldo + h * DH;

  for (int qc = 0; qc < se.Tq; qc += kQC) {
    __syncthreads();
    stage_rows<DH>(Qb, a.ldq, qc, se.Tq, kQC, Qs);
    stage_rows<DH>(dOb, a.lddo, qc, se.Tq, kQC, dOs);
    // D[q] = sum_dh dO[q,dh] * O[q,dh]: CH consecutive lanes share a row
    for (int idx = threadIdx.x; idx < kQC * CH; idx += kThreads) {
      const int rl = idx / CH, c = idx % CH, q = qc + rl;
      float part = 0.f;
      if (q < se.Tq) {
        const half8_t dv = ld_half8(dOb + (size_t)q * a.lddo + c * 8), ov = ld_half8(Ob + (size_t)q * a.ldo + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) part += (float)dv[e] * (float)ov[e];
      }
#pragma unroll
      for (int o = CH / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, kWave);
      if (c == 0) {
        D_s[rl] = part;
        lse_s[rl] = q < se.Tq ? a.lse[(size_t)h * a.Nq + se.q0 + q] : 0.f;
      }
    }
    __syncthreads();
    if (k0 >= se.Tk) continue;
    const int nqt = (min(kQC, se.Tq - qc) + 31) / 32;
    for (int qt = 0; qt < nqt; ++qt) {
      if (a.causal && qc + qt * 32 + 31 < k0) continue;  // every query of the tile precedes every key
      floatx16 s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = (qt * 32 + (lane & 31)) * PR + ks * 16 + g * 8;
        s = MFMA(ld_half8(Qs + off), kf[ks], s);
        dp = MFMA(ld_half8(dOs + off), vf[ks], dp);
      }
      half8_t pf[2], dsf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ql = qt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        const int q = qc + ql;
        const bool hid = khid || q >= se.Tq || (a.causal && key > q);
        const float p = hid ? 0.f : exp2f(s[r] * sc - lse_s[ql] * kLog2e);
        pf[r >> 3][r & 7] = (half_t)p;
        dsf[r >> 3][r & 7] = (half_t)(p * (dp[r] - D_s[ql]) * scale);
      }
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const int kb = qt * 32 + 16 * s2 + 4 * g;
          dVt[t] = MFMA(tr_frag<DH>(dOs, PR, kb, t, lane), pf[s2], dVt[t]);
          dKt[t] = MFMA(tr_frag<DH>(Qs, PR, kb, t, lane), dsf[s2], dKt[t]);
        }
    }
  }
  if (!kvalid) return;
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int dh0 = t * 32 + 8 * rq + 4 * g;
      if (dh0 < DH) {
        half4_t ok, ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ok[e] = (half_t)dKt[t][4 * rq + e];
          ov[e] = (half_t)dVt[t][4 * rq + e];
        }
        *reinterpret_cast<half4_t*>(a.dK + (size_t)(se.k0 + key) * a.lddk + h * DH + dh0) = ok;
        *reinterpret_cast<half4_t*>(a.dV + (size_t)(se.k0 + key) * a.lddv + h * DH + dh0) = ov;
      }
    }
}

// ------------------------------------------------------------------------------------------------
// backward, dQ
// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ void __launch_bounds__(kThreads) attn_bwd_dq_kernel(const AttnArgs a) {
  constexpr int DHP = DH < 32 ? 32 : DH, KS = DH / 16, DT = DHP / 32, PR = DH + 8;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  half_t* Ks = reinterpret_cast<half_t*>(smem_raw);
  half_t* Vs = Ks + kKC * PR;
  uint8_t* hidk = reinterpret_cast<uint8_t*>(Vs + kKC * PR);

  const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
  const Sent se = sentence(a, b);
  if ((int)blockIdx.y * 128 >= se.Tq) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int q0 = blockIdx.y * 128 + wave * 32;
  const int q = q0 + (lane & 31);
  const bool qvalid = q < se.Tq;
  half8_t qf[KS], dof[KS];
  float Dq = 0.f;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    const int col = h * DH + s * 16 + g * 8;
    qf[s] = qvalid ? ld_half8(a.Q + (size_t)(se.q0 + q) * a.ldq + col) : zero_half8();
    dof[s] = qvalid ? ld_half8(a.dO + (size_t)(se.q0 + q) * a.lddo + col) : zero_half8();
    const half8_t ov = qvalid ? ld_half8(a.O + (size_t)(se.q0 + q) * a.ldo + col) : zero_half8();
#pragma unroll
    for (int e = 0; e < 8; ++e) Dq += (float)dof[s][e] * (float)ov[e];
  }
  Dq += __shfl_xor(Dq, 32, kWave);
  const float lse_q = qvalid ? a.lse[(size_t)h * a.Nq + se.q0 + q] * kLog2e : 0.f;
  const float scale = rsqrtf((float)DH), sc = scale * kLog2e;
  floatx16 dQt[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) dQt[t] = zero16();
  const half_t* Kb = a.K + (size_t)se.k0 * a.ldk + h * DH;
  const half_t* Vb = a.V + (size_t)se.k0 * a.ldv + h * DH;

  for (int kc = 0; kc < se.Tk; kc += kKC) {
    __syncthreads();
    stage_rows<DH>(Kb, a.ldk, kc, se.Tk, kKC, Ks);
    stage_rows<DH>(Vb, a.ldv, kc, se.Tk, kKC, Vs);
    for (int k = threadIdx.x; k < kKC; k += kThreads)
      hidk[k] = (kc + k >= se.Tk) || (a.key_ids && a.key_ids[se.k0 + kc + k] == a.pad_id);
    __syncthreads();
    if (q0 >= se.Tq) continue;
    const int nkt = (min(kKC, se.Tk - kc) + 31) / 32;
    for (int kt = 0; kt < nkt; ++kt) {
      if (a.causal && kc + kt * 32 > q0 + 31) break;  // every key of the tile follows every query
      floatx16 s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = (kt * 32 + (lane & 31)) * PR + ks * 16 + g * 8;
        s = MFMA(ld_half8(Ks + off), qf[ks], s);
        dp = MFMA(ld_half8(Vs + off), dof[ks], dp);
      }
      half8_t dsf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kl = kt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        const bool hid = hidk[kl] || (a.causal && kc + kl > q);
        const float p = hid ? 0.f : exp2f(s[r] * sc - lse_q);
        dsf[r >> 3][r & 7] = (half_t)(p * (dp[r] - Dq) * scale);
      }
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          dQt[t] = MFMA(tr_frag<DH>(Ks, PR, kt * 32 + 16 * s2 + 4 * g, t, lane), dsf[s2], dQt[t]);
        }
    }
  }
  if (!qvalid) return;
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int dh0 = t * 32 + 8 * rq + 4 * g;
      if (dh0 < DH) {
        half4_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (half_t)dQt[t][4 * rq + e];
        *reinterpret_cast<half4_t*>(a.dQ + (size_t)(se.q0 + q) * a.lddq + h * DH + dh0) = o;
      }
    }
}

template <int DH>
size_t fwd_smem(int Tk) {
  const int KP = (Tk + 31) & ~31;
  return (size_t)(2 * KP * (DH + 8)) * sizeof(half_t) + KP;
}
template <int DH>
size_t dkv_smem() {
  return (size_t)(2 * kQC * (DH + 8)) * sizeof(half_t) + 2 * kQC * sizeof(float);
}
template <int DH>
size_t dq_smem() {
  return (size_t)(2 * kKC * (DH + 8)) * sizeof(half_t) + kKC;
}

template <typename Kern>
int allow_big_lds(Kern kern, size_t bytes) {
  if (bytes > 64 * 1024)
    NMT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return NMT_OK;
}

template <int DH>
int fwd_launch(const AttnArgs& a, hipStream_t stream) {
  const size_t smem = fwd_smem<DH>(a.Tk);
  NMT_REQUIRE(smem <= 160 * 1024, "attention: Tk=%d needs %zu bytes of LDS", a.Tk, smem);
  if (int rc = allow_big_lds(attn_fwd_kernel<DH>, smem)) return rc;
  hipLaunchKernelGGL(attn_fwd_kernel<DH>, dim3(a.B * a.H, ceil_div(a.Tq, 128)), dim3(kThreads), smem, stream, a);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}
template <int DH>
int bwd_launch(const AttnArgs& a, hipStream_t stream) {
  if (int rc = allow_big_lds(attn_bwd_dkv_kernel<DH>, dkv_smem<DH>())) return rc;
  if (int rc = allow_big_lds(attn_bwd_dq_kernel<DH>, dq_smem<DH>())) return rc;
  hipLaunchKernelGGL(attn_bwd_dkv_kernel<DH>, dim3(a.B * a.H, ceil_div(a.Tk, 128)), dim3(kThreads), dkv_smem<DH>(), stream, a);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(attn_bwd_dq_kernel<DH>, dim3(a.B * a.H, ceil_div(a.Tq, 128)), dim3(kThreads), dq_smem<DH>(), stream, a);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int check_common(const AttnArgs& a, int dh) {
  NMT_REQUIRE(a.B > 0 && a.H > 0 && a.Tq > 0 && a.Tk > 0, "attention: empty problem");
  NMT_REQUIRE(dh == 16 || dh == 32 || dh == 64 || dh == 128, "attention: head size %d not in {16,32,64,128}", dh);
  NMT_REQUIRE(a.Tk <= 1024 && a.Tq <= 65535 && (int64_t)a.B * a.H < (1ll << 31), "attention: Tk=%d / B*H out of range", a.Tk);
  NMT_REQUIRE(a.tab ? a.Nq > 0 : a.Nq == a.B * a.Tq, "attention: inconsistent number of query rows");
  NMT_REQUIRE(a.ldq % 8 == 0 && a.ldk % 8 == 0 && a.ldv % 8 == 0 && a.ldo % 8 == 0, "attention: row strides must be multiples of 8");
  NMT_REQUIRE(a.ldq >= a.H * dh && a.ldk >= a.H * dh && a.ldv >= a.H * dh && a.ldo >= a.H * dh, "attention: row stride smaller than H*dh");
  NMT_REQUIRE(aligned16(a.Q) && aligned16(a.K) && aligned16(a.V), "attention: Q/K/V must be 16-byte aligned");
  return NMT_OK;
}

}  // namespace

int launch_attention_fwd(const half_t* Q, int ldq, const half_t* K, int ldk, const half_t* V, int ldv, half_t* O, int ldo,
                         float* lse, const int32_t* key_ids, int pad_id, int causal, int B, int H, int dh, int Tq, int Tk,
                         const int4* sent_tab, int n_q_rows, hipStream_t stream) {
  AttnArgs a = {};
  a.tab = sent_tab; a.Nq = sent_tab ? n_q_rows : B * Tq;
  a.Q = Q; a.K = K; a.V = V; a.Out = O; a.lse = lse; a.key_ids = key_ids;
  a.ldq = ldq; a.ldk = ldk; a.ldv = ldv; a.ldo = ldo;
  a.pad_id = pad_id; a.causal = causal; a.B = B; a.H = H; a.Tq = Tq; a.Tk = Tk;
  NMT_REQUIRE(Q && K && V && O && lse, "attention_fwd: null pointer");
  if (int rc = check_common(a, dh)) return rc;
  NMT_REQUIRE(aligned16(O), "attention_fwd: O must be 16-byte aligned");
  NMT_REQUIRE(!causal || Tq == Tk, "attention_fwd: the causal mask needs Tq == Tk");  // (per sentence, with a table)
  switch (dh) {
    case 16: return fwd_launch<16>(a, stream);
    case 32: return fwd_launch<32>(a, stream);
    case 64: return fwd_launch<64>(a, stream);
    default: return fwd_launch<128>(a, stream);
  }
}

int launch_attention_bwd(const half_t* Q, int ldq, const half_t* K, int ldk, const half_t* V, int ldv, const half_t* O, int ldo,
                         const half_t* dO, int lddo, const float* lse, half_t* dQ, int lddq, half_t* dK, int lddk, half_t* dV,
                         int lddv, const int32_t* key_ids, int pad_id, int causal, int B, int H, int dh, int Tq, int Tk,
                         const int4* sent_tab, int n_q_rows, hipStream_t stream) {
  AttnArgs a = {};
  a.tab = sent_tab; a.Nq = sent_tab ? n_q_rows : B * Tq;
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.dO = dO; a.lse = const_cast<float*>(lse); a.key_ids = key_ids;
  a.dQ = dQ; a.dK = dK; a.dV = dV;
  a.ldq = ldq; a.ldk = ldk; a.ldv = ldv; a.ldo = ldo; a.lddo = lddo; a.lddq = lddq; a.lddk = lddk; a.lddv = lddv;
  a.pad_id = pad_id; a.causal = causal; a.B = B; a.H = H; a.Tq = Tq; a.Tk = Tk;
  NMT_REQUIRE(Q && K && V && O && dO && lse && dQ && dK && dV, "attention_bwd: null pointer");
  if (int rc = check_common(a, dh)) return rc;
  NMT_REQUIRE(lddo % 8 == 0 && lddq % 8 == 0 && lddk % 8 == 0 && lddv % 8 == 0, "attention_bwd: row strides must be multiples of 8");
  NMT_REQUIRE(lddo >= H * dh && lddq >= H * dh && lddk >= H * dh && lddv >= H * dh, "attention_bwd: row stride smaller than H*dh");
  NMT_REQUIRE(aligned16(O) && aligned16(dO) && aligned16(dQ) && aligned16(dK) && aligned16(dV), "attention_bwd: misaligned pointer");
  NMT_REQUIRE(!causal || Tq == Tk, "attention_bwd: the causal mask needs Tq == Tk");
  switch (dh) {
    case 16: return bwd_launch<16>(a, stream);
    case 32: return bwd_launch<32>(a, stream);
    case 64: return bwd_launch<64>(a, stream);
    default: return bwd_launch<128>(a, stream);
  }
}
