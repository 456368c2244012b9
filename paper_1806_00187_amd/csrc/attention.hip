// Fused masked multi-head attention for gfx950: forward with online softmax, and backward as two
// kernels (dK/dV: a wavefront owns 32 keys and sweeps the queries; dQ: a wavefront owns 32 queries
// and sweeps the keys).  Scores never go to memory.  All products run on 32x32x16 fp16 MFMAs.
//
// Sentences here are short (tens of positions), so the unit of work is small: ONE WAVEFRONT per
// (sentence, head, 32-row tile), four heads of a sentence per work-group, and no work-group
// barrier anywhere.  Operands whose contraction index is contiguous in memory (Q, K, V, dO rows
// against the head dimension) are loaded from global memory straight into MFMA operand registers,
// 16 bytes per lane.  An operand that is contracted over its row index (V in P V, K in dS K, Q and
// dO in dS^T Q and P^T dO) passes through a wavefront-private 32-row LDS tile and comes back through
// the transposing LDS read.
//
// Register layouts (v_mfma_f32_32x32x16_f16, D = A x B): A lane l holds row l%32, k = 8*(l/32)+j;
// B lane l holds column l%32, same k; D lane l holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4
// for r = 0..15.  Scores are produced transposed where that puts the softmax row (the query) on a
// lane, so that row statistics are per-lane scalars; probabilities are fed to the second product
// straight from registers: the contraction index may be permuted freely as long as both operands
// use the same permutation, so slot j of k-step s2 stands for row 16*s2 + 8*(j/4) + 4*(l/32) + j%4.
#include <math.h>
#include <stdlib.h>

#include "common.h"

#include <atomic>
#include <mutex>
#include <unordered_map>

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
  const half_t *Q, *K, *V, *O, *dO;
  half_t *Out, *dQ, *dK, *dV;
  float* lse;
  const int32_t* key_ids;
  int ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv;
  int pad_id, causal, B, H, Tq, Tk;  // with a sentence table: Tq, Tk are the largest lengths in it
  const int4* tab;                   // per sentence (first query row, first key row, Tq, Tk), or nullptr
  int Nq;                            // query rows in total: lse is [H, Nq]
  int fused_max;                     // backward: sentences with max(Tq, Tk) <= this are left to the fused kernel
  // work lists over the table (or nullptr: every (sentence, tile) of the grid is looked at)
  const int32_t* wl_counts;          // [0..3] sentences by tiles of the longer side, [4] longer ones, [5] query tiles
  const int4* wl_sent;               // [4][B] table entries of the sentences of each class
  const int4* wl_qsent;              // per query tile: its sentence's table entry ...
  const int32_t* wl_qtile;           // ... and its tile number
  int vgx, vgy;                      // persistent kernels: the grid of work items their work-groups walk through
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

// The wavefront's own work item: a sentence, head h, 32-row tile `tile`.
struct Item {
  Sent se;
  int h, tile;
  bool live;
};
// LIST 0: the grid enumerates (sentence, tile); 1: entry bx / hg of the query-tile list;
// 2: entry bx / hg of the list of sentences of class `cls` (tile = 0).  List entries carry
// the sentence's table entry, so a work item costs one dependent load, not two.
// (bx, by): the work-group's place in the grid of work items -- blockIdx for a kernel that takes one item
// per work-group, the loop position for a persistent one.
template <int LIST>
__device__ __forceinline__ Item work_item(const AttnArgs& a, int bx, int by, int cls = 0) {
  const int wpb = blockDim.x >> 6;            // heads per work-group (one wavefront each)
  const int hg = (a.H + wpb - 1) / wpb;
  const int idx = bx / hg;
  Item it;
  it.h = (bx % hg) * wpb + (threadIdx.x >> 6);
  it.tile = by;
  it.live = it.h < a.H;
  if (LIST == 1 && a.wl_qsent) {
    it.live = it.live && idx < a.wl_counts[5];
    const int4 t = it.live ? a.wl_qsent[idx] : make_int4(0, 0, 0, 0);
    it.tile = it.live ? a.wl_qtile[idx] : 0;
    it.se = Sent{t.x, t.y, t.z, t.w};
  } else if (LIST == 2 && a.wl_sent) {
    it.live = it.live && idx < a.wl_counts[cls];
    const int4 t = it.live ? a.wl_sent[(size_t)cls * a.B + idx] : make_int4(0, 0, 0, 0);
    it.se = Sent{t.x, t.y, t.z, t.w};
  } else {
    it.se = it.live ? sentence(a, idx) : Sent{0, 0, 0, 0};
  }
  return it;
}

// 32 rows of a [*, DH] head slice as MFMA operand registers: lane l gets row row0 + l%32, columns
// 16*s + 8*(l/32) .. +7 for every k-step s; rows >= row_end are zero.
template <int DH>
__device__ __forceinline__ void load_rows(const half_t* __restrict__ base, int ld, int row0, int row_end, int lane, half8_t (&f)[DH / 16]) {
  const int row = row0 + (lane & 31);
  const half_t* p = base + (size_t)row * ld + 8 * (lane >> 5);
#pragma unroll
  for (int s = 0; s < DH / 16; ++s) f[s] = row < row_end ? ld_half8(p + s * 16) : zero_half8();
}
// The same registers written to the wavefront's LDS tile in row-major order (pitch DH+8 halfs).
template <int DH>
__device__ __forceinline__ void put_rows(half_t* tile, int lane, const half8_t (&f)[DH / 16]) {
  half_t* p = tile + (lane & 31) * (DH + 8) + 8 * (lane >> 5);
#pragma unroll
  for (int s = 0; s < DH / 16; ++s) st_half8(p + s * 16, f[s]);
}
// Orders the wavefront's LDS accesses: what other lanes wrote before is visible after (LDS
// instructions of one wavefront execute in order; this keeps the compiler from reordering them).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// Bit k of the result: key row0 + k (k < 32) is hidden from every query (padding or past the end).
__device__ __forceinline__ uint32_t hidden_keys(const AttnArgs& a, const Sent& se, int row0, int lane) {
  const int key = row0 + (lane & 31);
  const bool hid = key >= se.Tk || (a.key_ids && a.key_ids[se.k0 + key] == a.pad_id);
  return (uint32_t)__ballot(hid);
}

// Writes a transposed result tile (MFMA layout: lane = row l%32 of the output, registers = groups of
// four consecutive columns) to global memory through the wavefront's LDS tile, so that every store
// instruction covers whole 2*DH-byte rows instead of 16-byte pieces of 32 rows.
template <int DH>
__device__ __forceinline__ void store_rows(half_t* tile, const floatx16 (&acc)[(DH < 32 ? 32 : DH) / 32], float scale, half_t* dst, int ld,
                                           int row0, int row_end, int lane) {
  constexpr int PR = DH + 8, DT = (DH < 32 ? 32 : DH) / 32, CH = DH / 8;
  const int g = lane >> 5;
  wave_sync();  // earlier reads of the tile are done
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int dh0 = t * 32 + 8 * rq + 4 * g;
      if (dh0 < DH) {
        half4_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (half_t)(acc[t][4 * rq + e] * scale);
        *reinterpret_cast<half4_t*>(tile + (lane & 31) * PR + dh0) = o;
      }
    }
  wave_sync();
#pragma unroll
  for (int it = 0; it < (32 * CH + 63) / 64; ++it) {
    const int idx = it * 64 + lane, r = idx / CH, c = idx % CH;
    if (r < 32 && row0 + r < row_end) st_half8(dst + (size_t)(row0 + r) * ld + c * 8, ld_half8(tile + r * PR + c * 8));
  }
}

// ------------------------------------------------------------------------------------------------
// forward: the wavefront owns 32 queries
// ------------------------------------------------------------------------------------------------
template <int DH>
__device__ __forceinline__ void attn_fwd_item(const AttnArgs& a, int bx, int by, unsigned char* smem_raw) {
  constexpr int DHP = DH < 32 ? 32 : DH, KS = DH / 16, DT = DHP / 32, PR = DH + 8;
  const Item it = work_item<1>(a, bx, by);
  if (!it.live) return;
  const Sent se = it.se;
  const int q0 = it.tile * 32;
  if (q0 >= se.Tq) return;
  const int lane = threadIdx.x & 63, g = lane >> 5, h = it.h;
  half_t* Vs = reinterpret_cast<half_t*>(smem_raw) + (threadIdx.x >> 6) * (32 * PR);
  const half_t* Kb = a.K + (size_t)se.k0 * a.ldk + h * DH;
  const half_t* Vb = a.V + (size_t)se.k0 * a.ldv + h * DH;

  const int q = q0 + (lane & 31);
  const bool qvalid = q < se.Tq;
  half8_t qf[KS];
  load_rows<DH>(a.Q + (size_t)se.q0 * a.ldq + h * DH, a.ldq, q0, se.Tq, lane, qf);

  const float sc = rsqrtf((float)DH) * kLog2e;
  float m = -1e30f, l = 0.f;
  floatx16 oacc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) oacc[t] = zero16();
  int nkt = (se.Tk + 31) >> 5;
  if (a.causal) nkt = min(nkt, (q0 + 31) / 32 + 1);
  for (int kt = 0; kt < nkt; ++kt) {
    half8_t kf[KS], vf[KS];
    load_rows<DH>(Kb, a.ldk, kt * 32, se.Tk, lane, kf);
    load_rows<DH>(Vb, a.ldv, kt * 32, se.Tk, lane, vf);
    const uint32_t hm = hidden_keys(a, se, kt * 32, lane);
    wave_sync();  // the previous tile's reads are done
    put_rows<DH>(Vs, lane, vf);
    floatx16 s = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s = MFMA(kf[ks], qf[ks], s);
    float tmax = -1e30f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kl = 8 * (r >> 2) + 4 * g + (r & 3);
      const bool hid = ((hm >> kl) & 1u) || (a.causal && kt * 32 + kl > q);
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
    wave_sync();  // the V tile is in LDS
#pragma unroll
    for (int t = 0; t < DT; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[t][r] *= alpha;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) oacc[t] = MFMA(tr_frag<DH>(Vs, PR, 16 * s2 + 4 * g, t, lane), pf[s2], oacc[t]);
    }
  }
  l += __shfl_xor(l, 32, kWave);
  store_rows<DH>(Vs, oacc, 1.f / l, a.Out + (size_t)se.q0 * a.ldo + h * DH, a.ldo, q0, se.Tq, lane);
  if (!qvalid) return;
  if (g == 0) a.lse[(size_t)h * a.Nq + se.q0 + q] = (m + log2f(l)) * kLn2;
}
// Persistent: the launch fills the chip once and every work-group walks through the work items with the
// grid's stride.  A wavefront that ended after each item would first wait for its stores to land; here the
// next item's loads go out right behind them.
template <int DH>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(DH <= 64 ? 3 : 1, DH <= 64 ? 3 : 1)))
attn_fwd_kernel(const AttnArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int total = a.vgx * a.vgy;
  for (int v = blockIdx.x; v < total; v += gridDim.x) attn_fwd_item<DH>(a, v % a.vgx, v / a.vgx, smem_raw);
}

// ------------------------------------------------------------------------------------------------
// backward, dK and dV: the wavefront owns 32 keys
// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ void __launch_bounds__(kThreads) attn_bwd_dkv_kernel(const AttnArgs a) {
  constexpr int DHP = DH < 32 ? 32 : DH, KS = DH / 16, DT = DHP / 32, PR = DH + 8;
  constexpr int WAVE_LDS = 2 * 32 * PR * 2 + 2 * 32 * 4;  // Q and dO tiles, lse and D of the tile's queries
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const Item it = work_item<0>(a, blockIdx.x, blockIdx.y);
  if (!it.live) return;
  const Sent se = it.se;
  const int k0 = it.tile * 32;
  if (k0 >= se.Tk || max(se.Tq, se.Tk) <= a.fused_max) return;
  const int lane = threadIdx.x & 63, g = lane >> 5, h = it.h;
  unsigned char* mine = smem_raw + (threadIdx.x >> 6) * WAVE_LDS;
  half_t* Qs = reinterpret_cast<half_t*>(mine);
  half_t* dOs = Qs + 32 * PR;
  float* lse_s = reinterpret_cast<float*>(dOs + 32 * PR);
  float* D_s = lse_s + 32;

  const int key = k0 + (lane & 31);
  const bool kvalid = key < se.Tk;
  const bool khid = !kvalid || (a.key_ids && a.key_ids[se.k0 + key] == a.pad_id);
  half8_t kf[KS], vf[KS];
  load_rows<DH>(a.K + (size_t)se.k0 * a.ldk + h * DH, a.ldk, k0, se.Tk, lane, kf);
  load_rows<DH>(a.V + (size_t)se.k0 * a.ldv + h * DH, a.ldv, k0, se.Tk, lane, vf);
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
  const float* lse_b = a.lse + (size_t)h * a.Nq + se.q0;

  const int nqt = (se.Tq + 31) >> 5;
  for (int qt = a.causal ? k0 >> 5 : 0; qt < nqt; ++qt) {  // causal: earlier query tiles precede every key of this tile
    half8_t qf[KS], dof[KS], of[KS];
    load_rows<DH>(Qb, a.ldq, qt * 32, se.Tq, lane, qf);
    load_rows<DH>(dOb, a.lddo, qt * 32, se.Tq, lane, dof);
    load_rows<DH>(Ob, a.ldo, qt * 32, se.Tq, lane, of);
    const int ql = qt * 32 + (lane & 31);
    const float lse_q = ql < se.Tq ? lse_b[ql] * kLog2e : 0.f;
    // D[q] = sum_dh dO[q,dh] * O[q,dh]: lanes l and l+32 hold the two halves of row q
    float Dq = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) Dq += (float)dof[s][e] * (float)of[s][e];
    Dq += __shfl_xor(Dq, 32, kWave);
    wave_sync();  // the previous tile's reads are done
    put_rows<DH>(Qs, lane, qf);
    put_rows<DH>(dOs, lane, dof);
    if (g == 0) {
      lse_s[lane] = lse_q;
      D_s[lane] = Dq;
    }
    floatx16 s = zero16(), dp = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      s = MFMA(qf[ks], kf[ks], s);
      dp = MFMA(dof[ks], vf[ks], dp);
    }
    wave_sync();  // tiles and row statistics are in LDS
    half8_t pf[2], dsf[2];
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const floatx4 l4 = *reinterpret_cast<const floatx4*>(lse_s + 8 * rq + 4 * g);
      const floatx4 d4 = *reinterpret_cast<const floatx4*>(D_s + 8 * rq + 4 * g);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = 4 * rq + e;
        const int qq = qt * 32 + 8 * rq + 4 * g + e;
        const bool hid = khid || qq >= se.Tq || (a.causal && key > qq);
        const float p = hid ? 0.f : exp2f(s[r] * sc - l4[e]);
        pf[r >> 3][r & 7] = (half_t)p;
        dsf[r >> 3][r & 7] = (half_t)(p * (dp[r] - d4[e]) * scale);
      }
    }
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const int kb = 16 * s2 + 4 * g;
        dVt[t] = MFMA(tr_frag<DH>(dOs, PR, kb, t, lane), pf[s2], dVt[t]);
        dKt[t] = MFMA(tr_frag<DH>(Qs, PR, kb, t, lane), dsf[s2], dKt[t]);
      }
  }
  store_rows<DH>(Qs, dKt, 1.f, a.dK + (size_t)se.k0 * a.lddk + h * DH, a.lddk, k0, se.Tk, lane);
  store_rows<DH>(dOs, dVt, 1.f, a.dV + (size_t)se.k0 * a.lddv + h * DH, a.lddv, k0, se.Tk, lane);
}

// ------------------------------------------------------------------------------------------------
// backward, dQ: the wavefront owns 32 queries
// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ void __launch_bounds__(kThreads) attn_bwd_dq_kernel(const AttnArgs a) {
  constexpr int DHP = DH < 32 ? 32 : DH, KS = DH / 16, DT = DHP / 32, PR = DH + 8;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const Item it = work_item<0>(a, blockIdx.x, blockIdx.y);
  if (!it.live) return;
  const Sent se = it.se;
  const int q0 = it.tile * 32;
  if (q0 >= se.Tq || max(se.Tq, se.Tk) <= a.fused_max) return;
  const int lane = threadIdx.x & 63, g = lane >> 5, h = it.h;
  half_t* Ks = reinterpret_cast<half_t*>(smem_raw) + (threadIdx.x >> 6) * (32 * PR);

  const int q = q0 + (lane & 31);
  const bool qvalid = q < se.Tq;
  half8_t qf[KS], dof[KS], of[KS];
  load_rows<DH>(a.Q + (size_t)se.q0 * a.ldq + h * DH, a.ldq, q0, se.Tq, lane, qf);
  load_rows<DH>(a.dO + (size_t)se.q0 * a.lddo + h * DH, a.lddo, q0, se.Tq, lane, dof);
  load_rows<DH>(a.O + (size_t)se.q0 * a.ldo + h * DH, a.ldo, q0, se.Tq, lane, of);
  float Dq = 0.f;
#pragma unroll
  for (int s = 0; s < KS; ++s)
#pragma unroll
    for (int e = 0; e < 8; ++e) Dq += (float)dof[s][e] * (float)of[s][e];
  Dq += __shfl_xor(Dq, 32, kWave);
  const float lse_q = qvalid ? a.lse[(size_t)h * a.Nq + se.q0 + q] * kLog2e : 0.f;
  const float scale = rsqrtf((float)DH), sc = scale * kLog2e;
  floatx16 dQt[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) dQt[t] = zero16();
  const half_t* Kb = a.K + (size_t)se.k0 * a.ldk + h * DH;
  const half_t* Vb = a.V + (size_t)se.k0 * a.ldv + h * DH;

  int nkt = (se.Tk + 31) >> 5;
  if (a.causal) nkt = min(nkt, (q0 + 31) / 32 + 1);  // later key tiles follow every query of this tile
  for (int kt = 0; kt < nkt; ++kt) {
    half8_t kf[KS], vf[KS];
    load_rows<DH>(Kb, a.ldk, kt * 32, se.Tk, lane, kf);
    load_rows<DH>(Vb, a.ldv, kt * 32, se.Tk, lane, vf);
    const uint32_t hm = hidden_keys(a, se, kt * 32, lane);
    wave_sync();  // the previous tile's reads are done
    put_rows<DH>(Ks, lane, kf);
    floatx16 s = zero16(), dp = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      s = MFMA(kf[ks], qf[ks], s);
      dp = MFMA(vf[ks], dof[ks], dp);
    }
    half8_t dsf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kl = 8 * (r >> 2) + 4 * g + (r & 3);
      const bool hid = ((hm >> kl) & 1u) || (a.causal && kt * 32 + kl > q);
      const float p = hid ? 0.f : exp2f(s[r] * sc - lse_q);
      dsf[r >> 3][r & 7] = (half_t)(p * (dp[r] - Dq) * scale);
    }
    wave_sync();  // the K tile is in LDS
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) dQt[t] = MFMA(tr_frag<DH>(Ks, PR, 16 * s2 + 4 * g, t, lane), dsf[s2], dQt[t]);
  }
  store_rows<DH>(Ks, dQt, 1.f, a.dQ + (size_t)se.q0 * a.lddq + h * DH, a.lddq, q0, se.Tq, lane);
}

// ------------------------------------------------------------------------------------------------
// backward, fused: one wavefront owns a whole (sentence, head) whose queries and keys fit NT 32-row
// tiles each, reads Q, K, V, O, dO once and writes dQ, dK, dV once.  Scores are formed with the key on
// the lane (as in the dK/dV kernel); for dQ the dS tile is turned around through a small LDS tile
// and the transposing read.
// ------------------------------------------------------------------------------------------------
constexpr int kDsPitch = 40;  // halfs per row of the 32 x 32 dS tile in LDS
template <int DH, int NT>
constexpr int fused_wave_lds() {
  return (2 * NT + 1) * 32 * (DH + 8) * 2 + 32 * kDsPitch * 2 + 2 * 32 * NT * 4;  // Q and dO tiles, one K tile, dS, lse and D
}
template <int DH, int NT>
__device__ __forceinline__ void attn_bwd_fused_item(const AttnArgs& a, int bx, unsigned char* smem_raw) {
  constexpr int DHP = DH < 32 ? 32 : DH, KS = DH / 16, DT = DHP / 32, PR = DH + 8, TILE = 32 * PR;
  const Item it = work_item<2>(a, bx, 0, NT - 1);
  if (!it.live) return;
  const Sent se = it.se;
  const int tmax = max(se.Tq, se.Tk);
  if (tmax > 32 * NT || tmax <= 32 * (NT - 1)) return;  // longer: other kernels; shorter: the instance with fewer tiles
  const int lane = threadIdx.x & 63, g = lane >> 5, h = it.h;
  unsigned char* mine = smem_raw + (threadIdx.x >> 6) * fused_wave_lds<DH, NT>();
  half_t* Qs = reinterpret_cast<half_t*>(mine);
  half_t* dOs = Qs + NT * TILE;
  half_t* Ks = dOs + NT * TILE;
  half_t* dSs = Ks + TILE;
  float* lse_s = reinterpret_cast<float*>(dSs + 32 * kDsPitch);
  float* D_s = lse_s + 32 * NT;

  const half_t* Qb = a.Q + (size_t)se.q0 * a.ldq + h * DH;
  const half_t* dOb = a.dO + (size_t)se.q0 * a.lddo + h * DH;
  const half_t* Ob = a.O + (size_t)se.q0 * a.ldo + h * DH;
  const half_t* Kb = a.K + (size_t)se.k0 * a.ldk + h * DH;
  const half_t* Vb = a.V + (size_t)se.k0 * a.ldv + h * DH;
  const float* lse_b = a.lse + (size_t)h * a.Nq + se.q0;
  const int nqt = (se.Tq + 31) >> 5, nkt = (se.Tk + 31) >> 5;

  // queries: Q and dO tiles to LDS, D[q] = sum_dh dO[q,dh] * O[q,dh] and the log-sum-exp beside them
#pragma unroll
  for (int qt = 0; qt < NT; ++qt) {
    if (qt < nqt) {
      half8_t qf[KS], dof[KS], of[KS];
      load_rows<DH>(Qb, a.ldq, qt * 32, se.Tq, lane, qf);
      load_rows<DH>(dOb, a.lddo, qt * 32, se.Tq, lane, dof);
      load_rows<DH>(Ob, a.ldo, qt * 32, se.Tq, lane, of);
      const int ql = qt * 32 + (lane & 31);
      const float lse_q = ql < se.Tq ? lse_b[ql] * kLog2e : 0.f;
      float Dq = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) Dq += (float)dof[s][e] * (float)of[s][e];
      Dq += __shfl_xor(Dq, 32, kWave);
      put_rows<DH>(Qs + qt * TILE, lane, qf);
      put_rows<DH>(dOs + qt * TILE, lane, dof);
      if (g == 0) {
        lse_s[ql] = lse_q;
        D_s[ql] = Dq;
      }
    }
  }
  const float scale = rsqrtf((float)DH), sc = scale * kLog2e;
  floatx16 dQt[NT][DT];
#pragma unroll
  for (int qt = 0; qt < NT; ++qt)
#pragma unroll
    for (int t = 0; t < DT; ++t) dQt[qt][t] = zero16();

#pragma unroll
  for (int kt = 0; kt < NT; ++kt) {
    if (kt < nkt) {
      const int k0 = kt * 32, key = k0 + (lane & 31);
      const bool khid = key >= se.Tk || (a.key_ids && a.key_ids[se.k0 + key] == a.pad_id);
      half8_t kf[KS], vf[KS];
      load_rows<DH>(Kb, a.ldk, k0, se.Tk, lane, kf);
      load_rows<DH>(Vb, a.ldv, k0, se.Tk, lane, vf);
      wave_sync();  // whatever read the K tile before is done
      put_rows<DH>(Ks, lane, kf);
      floatx16 dKt[DT], dVt[DT];
#pragma unroll
      for (int t = 0; t < DT; ++t) {
        dKt[t] = zero16();
        dVt[t] = zero16();
      }
#pragma unroll
      for (int qt = 0; qt < NT; ++qt) {
        if (qt < nqt && !(a.causal && qt < kt)) {  // causal: earlier query tiles precede every key of this tile
          wave_sync();  // Q, dO, K tiles and the row statistics are in LDS; the previous dS tile has been read
          floatx16 s = zero16(), dp = zero16();
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const int off = qt * TILE + (lane & 31) * PR + ks * 16 + g * 8;
            s = MFMA(ld_half8(Qs + off), kf[ks], s);
            dp = MFMA(ld_half8(dOs + off), vf[ks], dp);
          }
          half8_t pf[2], dsf[2];
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const floatx4 l4 = *reinterpret_cast<const floatx4*>(lse_s + qt * 32 + 8 * rq + 4 * g);
            const floatx4 d4 = *reinterpret_cast<const floatx4*>(D_s + qt * 32 + 8 * rq + 4 * g);
            half4_t ds4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int r = 4 * rq + e;
              const int qq = qt * 32 + 8 * rq + 4 * g + e;
              const bool hid = khid || qq >= se.Tq || (a.causal && key > qq);
              const float p = hid ? 0.f : exp2f(s[r] * sc - l4[e]);
              pf[r >> 3][r & 7] = (half_t)p;
              ds4[e] = (half_t)(p * (dp[r] - d4[e]) * scale);
              dsf[r >> 3][r & 7] = ds4[e];
            }
            // dS[key][query]: this lane's key row, four consecutive queries
            *reinterpret_cast<half4_t*>(dSs + (lane & 31) * kDsPitch + 8 * rq + 4 * g) = ds4;
          }
#pragma unroll
          for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
              const int kb = 16 * s2 + 4 * g;
              dVt[t] = MFMA(tr_frag<DH>(dOs + qt * TILE, PR, kb, t, lane), pf[s2], dVt[t]);
              dKt[t] = MFMA(tr_frag<DH>(Qs + qt * TILE, PR, kb, t, lane), dsf[s2], dKt[t]);
            }
          wave_sync();  // the dS tile is complete
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            const half8_t dst = tr_frag<32>(dSs, kDsPitch, 16 * s2 + 4 * g, 0, lane);  // lane = query, slots = keys
#pragma unroll
            for (int t = 0; t < DT; ++t) dQt[qt][t] = MFMA(tr_frag<DH>(Ks, PR, 16 * s2 + 4 * g, t, lane), dst, dQt[qt][t]);
          }
        }
      }
      store_rows<DH>(Ks, dKt, 1.f, a.dK + (size_t)se.k0 * a.lddk + h * DH, a.lddk, k0, se.Tk, lane);
      store_rows<DH>(Ks, dVt, 1.f, a.dV + (size_t)se.k0 * a.lddv + h * DH, a.lddv, k0, se.Tk, lane);
    }
  }
#pragma unroll
  for (int qt = 0; qt < NT; ++qt)
    if (qt < nqt) store_rows<DH>(Qs + qt * TILE, dQt[qt], 1.f, a.dQ + (size_t)se.q0 * a.lddq + h * DH, a.lddq, qt * 32, se.Tq, lane);
}
// Persistent, as the forward kernel, for sentences of up to 64 positions; the instances for longer ones need
// every register for one item (the loop form spills) and take one item per work-group.
template <int DH, int NT>
__global__ void __launch_bounds__(kThreads) attn_bwd_fused_kernel(const AttnArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  if constexpr (NT <= 2) {
    for (int v = blockIdx.x; v < a.vgx; v += gridDim.x) {
      wave_sync();  // the wavefront's LDS tiles are free again
      attn_bwd_fused_item<DH, NT>(a, v, smem_raw);
    }
  } else {
    attn_bwd_fused_item<DH, NT>(a, blockIdx.x, smem_raw);
  }
}

template <int DH>
constexpr size_t tile_smem() { return (size_t)4 * 32 * (DH + 8) * sizeof(half_t); }   // one 32-row tile per wavefront
template <int DH>
constexpr size_t dkv_smem() { return (size_t)4 * (2 * 32 * (DH + 8) * sizeof(half_t) + 2 * 32 * sizeof(float)); }

template <typename Kern>
int allow_big_lds(Kern kern, size_t bytes) {
  if (bytes <= 64 * 1024) return NMT_OK;
  // asked of the runtime once per kernel and size, not once per launch (callers may launch from several threads)
  static std::mutex mu;
  static std::unordered_map<const void*, size_t> allowed;
  const void* key = reinterpret_cast<const void*>(kern);
  std::lock_guard<std::mutex> lock(mu);
  auto it = allowed.find(key);
  if (it != allowed.end() && it->second >= bytes) return NMT_OK;
  NMT_HIP_CHECK(hipFuncSetAttribute(key, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  allowed[key] = bytes;
  return NMT_OK;
}

// Upper bounds of the list lengths, from what the host knows (the lists themselves are made on the device).
// Query tiles: sum_b ceil(Tq_b / 32) <= (sum_b Tq_b) / 32 + B, and sum_b Tq_b <= Nq + B (a table made from
// lengths that exceed the host's totals cuts sentences down to one row, which they may share).
int64_t qtile_capacity(int n_sent, int n_q_rows) { return ((int64_t)n_q_rows + n_sent) / 32 + n_sent + 1; }
int64_t qtile_bound(int n_sent, int n_q_rows, int max_tq) {
  const int64_t a = (int64_t)n_sent * ceil_div(max_tq, 32), b = qtile_capacity(n_sent, n_q_rows);
  return a < b ? a : b;
}
// Sentences whose longer side has more than 32 c positions: each takes that many of the Nq query rows or of
// the Nk key rows (n_k_rows == 0: self-attention, the keys are the queries' rows).
int64_t class_bound(int n_sent, int n_q_rows, int n_k_rows, int c) {
  if (c == 0) return n_sent;
  const int64_t b = n_q_rows / (32 * c + 1) + n_k_rows / (32 * c + 1);
  return b < n_sent ? b : n_sent;
}

// Work-groups of `kern` that the device holds at once (occupancy x compute units): the grid of a persistent launch.
template <typename Kern>
int resident_blocks(Kern kern, int threads, size_t smem, int* out) {
  int per_cu = 0;
  NMT_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern), threads, smem));
  *out = (per_cu > 0 ? per_cu : 1) * device_info().cus;
  return NMT_OK;
}

template <int DH>
int fwd_launch(const AttnArgs& a0, hipStream_t stream) {
  AttnArgs a = a0;
  a.vgx = a.B * ((a.H + 3) / 4);
  a.vgy = ceil_div(a.Tq, 32);
  if (a.wl_qsent) {
    a.vgx = (int)(qtile_bound(a.B, a.Nq, a.Tq) * ((a.H + 3) / 4));
    a.vgy = 1;
  }
  static std::atomic<int> resident_once{0};  // (per head size: the function is a template)
  int resident = resident_once.load(std::memory_order_relaxed);
  if (!resident) {
    if (int rc = resident_blocks(attn_fwd_kernel<DH>, kThreads, tile_smem<DH>(), &resident)) return rc;
    resident_once.store(resident, std::memory_order_relaxed);
  }
  const int64_t total = (int64_t)a.vgx * a.vgy;
  NMT_REQUIRE(total < (1ll << 31), "attention_fwd: too many work items");
  const int64_t grid = (total < resident || !tuning().attn_persist) ? total : resident;  // (not persistent: one work item per work-group)
  hipLaunchKernelGGL(attn_fwd_kernel<DH>, dim3((unsigned)grid), dim3(kThreads), tile_smem<DH>(), stream, a);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}
template <int DH, int NT>
int fused_launch(const AttnArgs& a, int n_k_rows, hipStream_t stream) {
  constexpr int kWaves = NT == 1 ? 4 : (NT == 2 ? 2 : 1);   // wavefronts (heads) per work-group: bounded by LDS
  const size_t smem = (size_t)kWaves * fused_wave_lds<DH, NT>();
  if (int rc = allow_big_lds(attn_bwd_fused_kernel<DH, NT>, smem)) return rc;
  const int64_t n = a.wl_sent ? class_bound(a.B, a.Nq, n_k_rows, NT - 1) : a.B;
  if (n == 0) return NMT_OK;
  AttnArgs b = a;
  b.vgx = (int)(n * ((a.H + kWaves - 1) / kWaves));
  b.vgy = 1;
  static std::atomic<int> resident_once{0};
  int resident = resident_once.load(std::memory_order_relaxed);
  if (NT <= 2 && !resident) {
    if (int rc = resident_blocks(attn_bwd_fused_kernel<DH, NT>, 64 * kWaves, smem, &resident)) return rc;
    resident_once.store(resident, std::memory_order_relaxed);
  }
  // (the instances for longer sentences, and everything with the persistent form switched off: one item per work-group)
  const int grid = (NT > 2 || b.vgx < resident || !tuning().attn_persist) ? b.vgx : resident;
  hipLaunchKernelGGL((attn_bwd_fused_kernel<DH, NT>), dim3((unsigned)grid), dim3(64 * kWaves), smem, stream, b);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}
template <int DH>
int bwd_launch(const AttnArgs& a0, int n_k_rows, hipStream_t stream) {
  AttnArgs a = a0;
  const int tmax = a.Tq > a.Tk ? a.Tq : a.Tk, nt_max = ceil_div(tmax, 32);
  // sentences of up to 128 positions on both sides (64 for the largest head size, whose accumulators would not
  // fit the register file): everything in one kernel, one wavefront per (sentence, head).  One instance per
  // number of 32-position tiles; without a table all sentences have the same lengths and need just one.
  a.fused_max = DH <= 64 ? 128 : 64;
  auto wanted = [&](int nt) { return nt <= nt_max && (a.tab || nt == nt_max); };
  if (wanted(1))
    if (int rc = fused_launch<DH, 1>(a, n_k_rows, stream)) return rc;
  if (wanted(2))
    if (int rc = fused_launch<DH, 2>(a, n_k_rows, stream)) return rc;
  if constexpr (DH <= 64) {
    if (wanted(3))
      if (int rc = fused_launch<DH, 3>(a, n_k_rows, stream)) return rc;
    if (wanted(4))
      if (int rc = fused_launch<DH, 4>(a, n_k_rows, stream)) return rc;
  }
  if (tmax <= a.fused_max) return NMT_OK;
  // longer ones: a wavefront per 32 queries for dQ, a wavefront per 32 keys for dK and dV
  if (int rc = allow_big_lds(attn_bwd_dkv_kernel<DH>, dkv_smem<DH>())) return rc;
  const int groups = a.B * ((a.H + 3) / 4);
  hipLaunchKernelGGL(attn_bwd_dq_kernel<DH>, dim3(groups, ceil_div(a.Tq, 32)), dim3(kThreads), tile_smem<DH>(), stream, a);
  NMT_LAUNCH_CHECK();
  hipLaunchKernelGGL(attn_bwd_dkv_kernel<DH>, dim3(groups, ceil_div(a.Tk, 32)), dim3(kThreads), dkv_smem<DH>(), stream, a);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int check_common(const AttnArgs& a, int dh) {
  NMT_REQUIRE(a.B > 0 && a.H > 0 && a.Tq > 0 && a.Tk > 0, "attention: empty problem");
  NMT_REQUIRE(dh == 16 || dh == 32 || dh == 64 || dh == 128, "attention: head size %d not in {16,32,64,128}", dh);
  NMT_REQUIRE(a.Tk <= (1 << 20) && a.Tq <= (1 << 20) && (int64_t)a.B * a.H < (1ll << 31), "attention: Tq=%d / Tk=%d / B*H out of range", a.Tq, a.Tk);
  NMT_REQUIRE(a.tab ? a.Nq > 0 : a.Nq == a.B * a.Tq, "attention: inconsistent number of query rows");
  NMT_REQUIRE(a.ldq % 8 == 0 && a.ldk % 8 == 0 && a.ldv % 8 == 0 && a.ldo % 8 == 0, "attention: row strides must be multiples of 8");
  NMT_REQUIRE(a.ldq >= a.H * dh && a.ldk >= a.H * dh && a.ldv >= a.H * dh && a.ldo >= a.H * dh, "attention: row stride smaller than H*dh");
  NMT_REQUIRE(aligned16(a.Q) && aligned16(a.K) && aligned16(a.V), "attention: Q/K/V must be 16-byte aligned");
  return NMT_OK;
}

}  // namespace

int launch_attention_fwd(const half_t* Q, int ldq, const half_t* K, int ldk, const half_t* V, int ldv, half_t* O, int ldo,
                         float* lse, const int32_t* key_ids, int pad_id, int causal, int B, int H, int dh, int Tq, int Tk,
                         const int4* sent_tab, int n_q_rows, const AttnWork* work, hipStream_t stream) {
  AttnArgs a = {};
  a.tab = sent_tab; a.Nq = sent_tab ? n_q_rows : B * Tq;
  if (sent_tab && work && tuning().worklists) { a.wl_counts = work->counts; a.wl_sent = work->by_tiles; a.wl_qsent = work->qsent; a.wl_qtile = work->qtile; }
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
                         const int4* sent_tab, int n_q_rows, const AttnWork* work, hipStream_t stream) {
  AttnArgs a = {};
  a.tab = sent_tab; a.Nq = sent_tab ? n_q_rows : B * Tq;
  if (sent_tab && work && tuning().worklists) { a.wl_counts = work->counts; a.wl_sent = work->by_tiles; a.wl_qsent = work->qsent; a.wl_qtile = work->qtile; }
  const int n_k_rows = work ? work->n_k_rows : 0;
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
    case 16: return bwd_launch<16>(a, n_k_rows, stream);
    case 32: return bwd_launch<32>(a, n_k_rows, stream);
    case 64: return bwd_launch<64>(a, n_k_rows, stream);
    default: return bwd_launch<128>(a, n_k_rows, stream);
  }
}

// ------------------------------------------------------------------------------------------------
// Work lists of one attention kind over a sentence table.  One block; thread t takes a contiguous run of
// sentences, so every list is in sentence order (and so the same from run to run).
// storage (int32 words): [0..7] counts, then [4][n_sent] int4 table entries by class, then bound_q int4
// table entries and bound_q tile numbers of the query tiles.
// ------------------------------------------------------------------------------------------------
namespace {
__global__ void __launch_bounds__(1024) attn_worklists_kernel(const int4* __restrict__ tab, int n_sent, int bound_q,
                                                              int32_t* __restrict__ st) {
  __shared__ int sh[6][1024];
  const int t = threadIdx.x, per = (n_sent + 1023) / 1024;
  const int lo = min(n_sent, t * per), hi = min(n_sent, lo + per);
  int cnt[6] = {0, 0, 0, 0, 0, 0};
  for (int i = lo; i < hi; ++i) {
    const int4 e = tab[i];
    const int nt = max(1, (max(e.z, e.w) + 31) >> 5);
    ++cnt[nt <= 4 ? nt - 1 : 4];
    cnt[5] += (e.z + 31) >> 5;
  }
#pragma unroll
  for (int c = 0; c < 6; ++c) sh[c][t] = cnt[c];
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    int v[6];
#pragma unroll
    for (int c = 0; c < 6; ++c) v[c] = t >= o ? sh[c][t - o] : 0;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 6; ++c) sh[c][t] += v[c];
    __syncthreads();
  }
  int at[6];
#pragma unroll
  for (int c = 0; c < 6; ++c) at[c] = sh[c][t] - cnt[c];
  int4* by_tiles = reinterpret_cast<int4*>(st + 8);
  int4* qsent = by_tiles + 4 * (size_t)n_sent;
  int32_t* qtile = reinterpret_cast<int32_t*>(qsent + bound_q);
  for (int i = lo; i < hi; ++i) {
    const int4 e = tab[i];
    const int nt = max(1, (max(e.z, e.w) + 31) >> 5);
    if (nt <= 4) by_tiles[(size_t)(nt - 1) * n_sent + at[nt - 1]++] = e;
    for (int q = 0; q < (e.z + 31) >> 5; ++q, ++at[5])
      if (at[5] < bound_q) {
        qsent[at[5]] = e;
        qtile[at[5]] = q;
      }
  }
  if (t == 1023) {
#pragma unroll
    for (int c = 0; c < 5; ++c) st[c] = sh[c][1023];
    st[5] = min(sh[5][1023], bound_q);
  }
}
}  // namespace

int64_t attention_worklist_ints(int n_sent, int n_q_rows) {
  return 8 + 16 * (int64_t)n_sent + 5 * qtile_capacity(n_sent, n_q_rows);
}

AttnWork attention_work(const int32_t* storage, int n_sent, int n_q_rows, int n_k_rows) {
  AttnWork w;
  w.counts = storage;
  w.by_tiles = reinterpret_cast<const int4*>(storage + 8);
  w.qsent = w.by_tiles + 4 * (size_t)n_sent;
  w.qtile = reinterpret_cast<const int32_t*>(w.qsent + qtile_capacity(n_sent, n_q_rows));
  w.n_k_rows = n_k_rows;
  return w;
}

int launch_attention_worklists(const int4* tab, int n_sent, int n_q_rows, int32_t* storage, hipStream_t stream) {
  NMT_REQUIRE(tab && storage && n_sent > 0 && n_q_rows > 0, "attention work lists: null pointer or empty table");
  NMT_REQUIRE((reinterpret_cast<uintptr_t>(storage) & 15u) == 0, "attention work lists: storage must be 16-byte aligned");
  hipLaunchKernelGGL(attn_worklists_kernel, dim3(1), dim3(1024), 0, stream, tab, n_sent, (int)qtile_capacity(n_sent, n_q_rows), storage);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}
