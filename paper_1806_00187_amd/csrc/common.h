// Internal helpers shared by the gfx950 kernels of the NMT training-step library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "nmt.h"

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---- error handling --------------------------------------------------------------------------
void nmt_set_error(const char* fmt, ...);

#define NMT_HIP_CHECK(expr)                                                                  \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) {                                                                  \
      nmt_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return NMT_EHIP;                                                                       \
    }                                                                                        \
  } while (0)

#define NMT_REQUIRE(cond, ...)   \
  do {                           \
    if (!(cond)) {               \
      nmt_set_error(__VA_ARGS__); \
      return NMT_EINVAL;         \
    }                            \
  } while (0)

#define NMT_LAUNCH_CHECK() NMT_HIP_CHECK(hipGetLastError())

// ---- the device and the launch-form switches ------------------------------------------------------
// Compute units and XCDs (dies with an L2 of their own) of the current device, asked of the runtime once.
struct DeviceInfo {
  int cus = 256, xcds = 8;
};
const DeviceInfo& device_info();
// Process-wide switches of launch forms (nmt_tuning): which work-group computes what, never what is computed.
struct Tuning {
  int gemm_group = 4;     // tile rows swept column by column before the next rows
  int gemm_persist = 1;   // 0: never the persistent GEMM form, 1: where it applies (large products whose epilogue loads nothing per element)
  int attn_persist = 1;   // 0: one attention work item per work-group
  int worklists = 1;      // 0: attention kernels enumerate every (sentence, tile) instead of taking work lists
  int one_stream = 0;     // 1: the backward pass's weight-gradient kernels run on the caller's stream, not beside it
  int gemm_share = 1;     // products expected to run side by side (callers that keep several passes in flight): large tiles
                          // are chosen as if each product had 1/gemm_share of the compute units
  int gemm_tile = 0;      // experiments: 0 = chosen per product; 1..5 force 256x256, 128x128, 128x64, 64x128, 64x64 tiles (products not cut along k)
  int gemm_timing = 0;    // 1: every GEMM product is bracketed by HIP events on its launch stream (nmt_gemm_timing reads them)
};
Tuning& tuning();

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
static inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ---- wavefront reductions (64 lanes) --------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// ---- Philox4x32-10 counter-based generator (Salmon et al., SC'11) ----------------------------
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    // one 32 x 32 -> 64 bit multiply per product (a single quarter-rate instruction instead of a high / low pair)
    const uint64_t p0 = (uint64_t)0xD2511F53u * c.x, p1 = (uint64_t)0xCD9E8D57u * c.z;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0, hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    c = make_uint4(hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0);
  }
  return c;
}

// Device-side dropout description (built on the host from nmt_dropout).  Row r of an activation
// belongs to sentence `uid` at position `pos` of sub-batch `micro`: either r / n_pos, r % n_pos and
// the micro index in c3 (one rectangular batch), or, when `rowkey` is set, rowkey[r] =
// (uid, pos | micro << 16) (several batches of different shapes stacked row-wise).
struct DropDev {
  uint32_t k0, k1;      // Philox key = seed
  uint32_t c3;          // step << 8 | micro
  uint32_t site_hi;     // site << 16
  uint32_t thr;         // keep iff 16-bit uniform >= thr; 0 = dropout off
  float scale;          // 1 / (1 - p)
  int32_t n_pos;        // rows per sentence
  const uint32_t* uid;  // per-sentence ids or nullptr
  const uint2* rowkey;  // per-row (uid, pos | micro << 16) or nullptr
};

DropDev make_drop(const nmt_dropout* d);  // host; d == nullptr or p <= 0 gives thr = 0

// Position within its sentence of row `row`.
__device__ __forceinline__ uint32_t drop_row_pos(const DropDev& dd, uint32_t row) {
  return dd.rowkey ? (dd.rowkey[row].y & 0xFFFFu) : row % (uint32_t)dd.n_pos;
}

// Keep decisions of the 8 columns [8*grp, 8*grp+8) of row `row`: bit i set = column 8*grp+i kept.
__device__ __forceinline__ uint32_t drop_keep8(const DropDev& dd, uint32_t row, uint32_t grp) {
  uint32_t uid, pos, c3 = dd.c3;
  if (dd.rowkey) {
    const uint2 rk = dd.rowkey[row];
    uid = rk.x;
    pos = rk.y & 0xFFFFu;
    c3 = (c3 & 0xFFFFFF00u) | (rk.y >> 16);
  } else {
    const uint32_t sent = row / (uint32_t)dd.n_pos;
    pos = row - sent * (uint32_t)dd.n_pos;
    uid = dd.uid ? dd.uid[sent] : sent;
  }
  const uint4 w = philox4x32_10(make_uint4(grp, uid, dd.site_hi | pos, c3), dd.k0, dd.k1);
  const uint32_t words[4] = {w.x, w.y, w.z, w.w};
  uint32_t bits = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    bits |= ((words[i] & 0xFFFFu) >= dd.thr ? 1u : 0u) << (2 * i);
    bits |= ((words[i] >> 16) >= dd.thr ? 1u : 0u) << (2 * i + 1);
  }
  return bits;
}

// ---- small vector helpers ---------------------------------------------------------------------
__device__ __forceinline__ half8_t ld_half8(const half_t* p) { return *reinterpret_cast<const half8_t*>(p); }
__device__ __forceinline__ void st_half8(half_t* p, half8_t v) { *reinterpret_cast<half8_t*>(p) = v; }
// Streaming forms for data that is touched once per kernel and is larger than the caches: no retention asked for.
__device__ __forceinline__ half8_t ld_half8_nt(const half_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(p)); }
__device__ __forceinline__ void st_half8_nt(half_t* p, half8_t v) { __builtin_nontemporal_store(v, reinterpret_cast<half8_t*>(p)); }
__device__ __forceinline__ floatx4 ld_float4_nt(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p)); }
__device__ __forceinline__ void st_float4_nt(float* p, floatx4 v) { __builtin_nontemporal_store(v, reinterpret_cast<floatx4*>(p)); }
__device__ __forceinline__ half8_t zero_half8() {
  half8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
  return z;
}

// ---- internal launchers (all enqueue on `stream`, return NMT_* codes) -------------------------
struct GemmEpilogue {
  const half_t* bias = nullptr;
  int relu = 0;
  DropDev drop = {};
  const half_t* add = nullptr;
  const half_t* relu_src = nullptr;
  float mask_scale = 1.f;
  int row0 = 0;  // row of the whole activation that row 0 of this product is (dropout counters)
  float out_scale = 1.f;  // the accumulated product is multiplied by this first (weight gradients of a large pass)
};
// partial: optional fp32 scratch of partial_floats floats for cutting the contraction into `splits`
// pieces summed by a second kernel (splits == 0: the launcher decides; needs an empty epilogue).
int launch_gemm(const half_t* A, bool a_t, int lda, const half_t* B, bool b_t, int ldb, half_t* C, int ldc,
                int M, int N, int K, const GemmEpilogue& ep, hipStream_t stream, float* partial = nullptr,
                int64_t partial_floats = 0, int splits = 1);

// fp32 product on the matrix cores, for the benchmark's fp32 comparison leg (not used by the training step)
int launch_gemm_f32(const float* A, bool a_t, int lda, const float* B, bool b_t, int ldb, float* C, int ldc, int M, int N, int K,
                    int splits, hipStream_t stream);

// Sum of the event-bracketed durations of the products launched since the last call (tuning().gemm_timing), their
// number and their algorithmic FLOPs; waits for them to finish.
int gemm_timing_read(double* ms, int64_t* products, double* flops);

// Work lists of one attention kind over a sentence table, made on the device (launch_attention_worklists)
// so that the attention kernels start no work-group for a (sentence, tile) that does not exist:
// counts[c], c = 0..3: sentences whose longer side takes c + 1 tiles of 32 positions, [4]: longer ones,
// [5]: query tiles; by_tiles [4][n_sent]: the table entries of the sentences of each class; qsent / qtile:
// per query tile its sentence's table entry and its tile number (entries are copies, so that a work
// item needs one dependent load).
struct AttnWork {
  const int32_t* counts = nullptr;
  const int4* by_tiles = nullptr;
  const int4* qsent = nullptr;
  const int32_t* qtile = nullptr;
  int n_k_rows = 0;  // key rows in total; 0 for self-attention (the keys are the queries' rows)
};
int64_t attention_worklist_ints(int n_sent, int n_q_rows);  // int32 words of storage behind one AttnWork (16-byte aligned)
AttnWork attention_work(const int32_t* storage, int n_sent, int n_q_rows, int n_k_rows);
int launch_attention_worklists(const int4* tab, int n_sent, int n_q_rows, int32_t* storage, hipStream_t stream);

int launch_attention_fwd(const half_t* Q, int ldq, const half_t* K, int ldk, const half_t* V, int ldv, half_t* O,
                         int ldo, float* lse, const int32_t* key_ids, int pad_id, int causal, int B, int H,
                         int dh, int Tq, int Tk, const int4* sent_tab, int n_q_rows, const AttnWork* work,
                         hipStream_t stream);
int launch_attention_bwd(const half_t* Q, int ldq, const half_t* K, int ldk, const half_t* V, int ldv,
                         const half_t* O, int ldo, const half_t* dO, int lddo, const float* lse, half_t* dQ,
                         int lddq, half_t* dK, int lddk, half_t* dV, int lddv, const int32_t* key_ids, int pad_id,
                         int causal, int B, int H, int dh, int Tq, int Tk, const int4* sent_tab, int n_q_rows,
                         const AttnWork* work, hipStream_t stream);

int launch_residual_layernorm_fwd(const half_t* sub, const half_t* resid, const half_t* gamma, const half_t* beta,
                                  half_t* out, float* stats, int rows, int d, float eps, const DropDev& drop,
                                  hipStream_t stream);
int64_t layernorm_bwd_scratch_floats(int d);
int launch_residual_layernorm_bwd(const half_t* dout, const half_t* sub, const half_t* resid, const half_t* gamma,
                                  const float* stats, half_t* dy, half_t* dym, half_t* dgamma, half_t* dbeta,
                                  half_t* dbias, float* partial, int rows, int d, const DropDev& drop,
                                  hipStream_t stream, float vec_scale = 1.f);  // vec_scale: factor on dgamma, dbeta, dbias
int launch_embed_fwd(const int32_t* ids, const half_t* E, half_t* x, int rows, int d, int vocab, const DropDev& drop,
                     hipStream_t stream);
int launch_softmax_xent(half_t* logits, const int32_t* targets, float* row_loss, int rows, int V, int pad_id,
                        float eps_ls, float loss_scale, float* loss_sum, int32_t* ntok, hipStream_t stream);
int64_t colsum_scratch_floats(int cols);
int launch_colsum(const half_t* src, int ld, half_t* dst, float* partial, int rows, int cols, hipStream_t stream, float scale = 1.f);
int launch_colsum_static(const half_t* src, int ld, half_t* dst, int rows, int cols, hipStream_t stream);  // partial sums in a fixed device array
int64_t embed_bwd_scratch_ints(int vocab, int rows_total, int d);
int launch_embed_bwd(const int32_t* ids_a, const half_t* dx_a, int rows_a, const DropDev& drop_a,
                     const int32_t* ids_b, const half_t* dx_b, int rows_b, const DropDev& drop_b, half_t* gE, int d,
                     int vocab, int32_t* scratch, hipStream_t stream, float scale = 1.f);
int launch_accumulate(const half_t* g16, float* acc, int64_t n, int first, hipStream_t stream, float mult = 1.f);
// in_place: acc *= inv_scale in the same pass; otherwise acc is only read
int launch_check_overflow(float* acc, int64_t n, float inv_scale, int32_t* flag, hipStream_t stream, bool in_place = true);
// *loss_total (+)= *loss, *ntok_total (+)= *ntok (first: overwrite)
int launch_add_scalars(const float* loss, const int32_t* ntok, float* loss_total, int32_t* ntok_total, int first, hipStream_t stream);
int launch_adam(float* master, float* m, float* v, const float* g, half_t* w16, int64_t n, float lr, float b1,
                float b2, float eps, int t, const int32_t* flag, hipStream_t stream, float grad_scale = 1.f);  // the update uses g * grad_scale
// Shapes of the sub-batches stacked row-wise in one pass (passed to the table kernel by value).
struct SegmentList {
  int n;
  int B[NMT_MAX_SEGMENTS], S[NMT_MAX_SEGMENTS], T[NMT_MAX_SEGMENTS];
  uint32_t micro[NMT_MAX_SEGMENTS];
};
// Row keys (uid, pos | micro << 16) of all source / target rows and the per-sentence attention
// tables (first query row, first key row, Tq, Tk) for encoder self-, decoder self- and
// encoder-decoder attention.  uid == nullptr: a sentence's id is its index within its sub-batch.
int launch_build_tables(const SegmentList& segs, int n_sent, const uint32_t* uid, uint2* rk_src, uint2* rk_tgt, int4* tab_ss,
                        int4* tab_tt, int4* tab_ts, hipStream_t stream);
// The same for sentences packed back to back (no padding): first rows come from a prefix sum of the
// lengths in `sentences`; lengths are clamped to [1, max] and to the row totals, so no table entry
// ever points outside [0, n_src) / [0, n_tgt).  sent_rows: scratch of 2 * n_sent ints.
int launch_build_tables_packed(const nmt_sentence* sentences, int n_sent, int n_src, int n_tgt, int max_src, int max_tgt,
                               int32_t* sent_rows, uint2* rk_src, uint2* rk_tgt, int4* tab_ss, int4* tab_tt, int4* tab_ts,
                               hipStream_t stream);
int launch_dropout_mask(uint8_t* keep, int rows, int n_cols, const DropDev& drop, hipStream_t stream);
