// fp16-in / fp32-accumulate MFMA GEMM with LDS-staged tiles and a fused epilogue
// (bias, ReLU, dropout, residual/gradient add, ReLU-backward mask) for gfx950.
//
// C[M,N] = epilogue(sum_k A(m,k) * B(n,k)).  Either operand may be stored with the contraction
// index contiguous ("direct": [rows][K]) or with its other index contiguous ("transposed":
// [K][rows]).  This covers the three products of a linear layer: forward x W^T (both direct),
// input gradient dy W (B transposed) and weight gradient dy^T x (both transposed).
//
// Data path, chosen so that the main loop carries (almost) no vector-ALU work besides the MFMAs:
//  * global -> registers with raw buffer loads: the per-thread byte offset is fixed at kernel
//    start, the k advance is one add, and out-of-range rows / k read as zero in hardware
//    (invalid elements get an offset beyond the buffer's extent), so there are no branches, no
//    64-bit address arithmetic and no selects;
//  * registers -> LDS with 16-byte stores, both layouts kept exactly as they are in memory;
//  * LDS -> MFMA fragments: a direct tile [row][k] gives a lane its 8 consecutive k with one
//    ds_read_b128; a transposed tile [k][row] gives them with two ds_read_b64_tr_b16 (the
//    gfx950 transposing LDS read: within 16 lanes, lane L receives element L%4 of the 8-byte
//    words addressed by lanes 4j + L/4, j = 0..3), so no register shuffling is needed;
//  * all LDS addresses are one per-lane base plus compile-time offsets; row pitches are padded
//    (not XOR-swizzled) to keep them additive and bank-conflict free;
//  * two register sets keep two k-tiles of global loads in flight behind the tile being
//    multiplied.
#include <stdlib.h>

#include <type_traits>

#include "common.h"

namespace {

constexpr int BK = 64;         // k extent of one LDS stage
constexpr int kThreads = 256;  // 4 wavefronts, arranged 2 x 2 over the block tile
constexpr uint32_t kOob = 0x80000000u;  // byte offset no operand reaches: such loads return 0

typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4_t* lds_short4_ptr;

struct GemmArgs {
  const half_t* A;
  const half_t* B;
  half_t* C;
  int lda, ldb, ldc, M, N, K;
  int tiles_m, tiles_n, tm_fast;
  GemmEpilogue ep;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const half_t* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(p), 0, (int)bytes, 0x00020000);
}
// The whole byte offset travels in the per-lane offset, which is what the hardware range-checks.
__device__ __forceinline__ half8_t buf_load(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff) {
  return __builtin_bit_cast(half8_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, 0, 0));
}

// ---- direct operand: memory [rows][K] (k contiguous), LDS tile [R][BK] with padded row pitch ----
template <int R>
struct DirectOp {
  static constexpr int NV = R / 32;              // 16-byte chunks moved per thread and k-tile
  static constexpr int PITCH = (BK + 8) * 2;     // bytes per tile row (144: conflict-free ds_read_b128)
  static constexpr int BYTES = R * PITCH;
  uint32_t voff[NV];
  uint32_t lds_st;   // this thread's store address within the tile (bytes)
  int c8;
  __device__ __forceinline__ static uint32_t extent(int rmax, int ld, int K) { return ((uint32_t)(rmax - 1) * ld + K) * 2u; }
  __device__ __forceinline__ void init(int ld, int r0, int rmax, int tid) {
    const int row = tid >> 3;
    c8 = (tid & 7) << 3;
#pragma unroll
    for (int it = 0; it < NV; ++it)
      voff[it] = (r0 + row + 32 * it < rmax) ? ((uint32_t)(r0 + row + 32 * it) * (uint32_t)ld + (uint32_t)c8) * 2u : kOob;
    lds_st = row * PITCH + (tid & 7) * 16;
  }
  __device__ __forceinline__ void load(half8_t (&v)[NV], __amdgpu_buffer_rsrc_t rsrc, int ld, int k0, int K) const {
    const bool kv = k0 + c8 < K;  // only the last k-tile can fail this
#pragma unroll
    for (int it = 0; it < NV; ++it) v[it] = buf_load(rsrc, kv ? voff[it] + (uint32_t)k0 * 2u : kOob);
  }
  __device__ __forceinline__ void store(const half8_t (&v)[NV], unsigned char* tile) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) *reinterpret_cast<half8_t*>(tile + lds_st + it * 32 * PITCH) = v[it];
  }
  // fragment base for the wave's rows starting at `row0`: lane -> row lane%32, k-half lane/32
  __device__ __forceinline__ static uint32_t frag_base(int row0, int lane) { return (row0 + (lane & 31)) * PITCH + (lane >> 5) * 16; }
  // 8 consecutive k of MFMA tile i, k-step s
  __device__ __forceinline__ static half8_t frag(const unsigned char* tile, uint32_t base, int i, int s) {
    return *reinterpret_cast<const half8_t*>(tile + base + i * 32 * PITCH + s * 32);
  }
};

// ---- transposed operand: memory [K][rows] (rows contiguous), LDS tile [BK][R] as in memory -------
template <int R>
struct TransOp {
  static constexpr int NV = R / 32;
  static constexpr int PITCH = (R + 16) * 2;     // bytes per k row of the tile
  static constexpr int BYTES = BK * PITCH;
  static constexpr int CPR = R / 8;              // 16-byte chunks per k row
  uint32_t voff[NV];
  uint32_t lds_st;
  __device__ __forceinline__ static uint32_t extent(int rmax, int ld, int K) { return ((uint32_t)(K - 1) * ld + rmax) * 2u; }
  __device__ __forceinline__ void init(int ld, int r0, int rmax, int tid) {
    const int k = tid / CPR, ch = tid % CPR;
    const bool ok = r0 + ch * 8 < rmax;
#pragma unroll
    for (int it = 0; it < NV; ++it)
      voff[it] = ok ? ((uint32_t)(k + it * (kThreads / CPR)) * (uint32_t)ld + (uint32_t)(r0 + ch * 8)) * 2u : kOob;
    lds_st = k * PITCH + ch * 16;
  }
  // rows k >= K lie beyond the buffer's extent and read as zero
  __device__ __forceinline__ void load(half8_t (&v)[NV], __amdgpu_buffer_rsrc_t rsrc, int ld, int k0, int K) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) v[it] = buf_load(rsrc, voff[it] + (uint32_t)k0 * (uint32_t)ld * 2u);
  }
  __device__ __forceinline__ void store(const half8_t (&v)[NV], unsigned char* tile) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) *reinterpret_cast<half8_t*>(tile + lds_st + it * (kThreads / CPR) * PITCH) = v[it];
  }
  // 16-lane group q = lane/16 serves rows 16*(q&1).. of the MFMA tile and k-half q/2; lane i of the group
  // addresses k row i/4, row offset 4*(i%4) of its 4(k) x 16(row) block.
  __device__ __forceinline__ static uint32_t frag_base(int row0, int lane) {
    const int q = lane >> 4, i = lane & 15;
    return (8 * (q >> 1) + (i >> 2)) * PITCH + (row0 + 16 * (q & 1) + 4 * (i & 3)) * 2;
  }
  __device__ __forceinline__ static half8_t frag(const unsigned char* tile, uint32_t base, int i, int s) {
    const unsigned char* p = tile + base + s * 16 * PITCH + i * 64;
    typedef short short8_t __attribute__((ext_vector_type(8)));
    const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p));
    const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p + 4 * PITCH));
    const short8_t r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(half8_t, r);
  }
};

template <int BM, int BN, bool AT, bool BT>
struct Tile {
  using OpA = typename std::conditional<AT, TransOp<BM>, DirectOp<BM>>::type;
  using OpB = typename std::conditional<BT, TransOp<BN>, DirectOp<BN>>::type;
  static constexpr int STAGE = OpA::BYTES + OpB::BYTES;
  static constexpr int WN = BN / 2;
  static constexpr int STAGING = 4 * 32 * (WN + 4) * 4;
  static constexpr int SMEM = 2 * STAGE > STAGING ? 2 * STAGE : STAGING;
};

template <int BM, int BN, bool AT, bool BT>
__global__ void __launch_bounds__(kThreads) gemm_kernel(const GemmArgs g) {
  extern __shared__ __align__(16) unsigned char smem[];
  using T = Tile<BM, BN, AT, BT>;
  using OpA = typename T::OpA;
  using OpB = typename T::OpB;
  constexpr int STAGE = T::STAGE;
  constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // Work-group -> tile.  Consecutive work-group ids go round-robin over the 8 XCDs; undo that so
  // each XCD (own L2) gets a contiguous run of tiles, then sweep the smaller operand fastest.
  int pid = blockIdx.x;
  {
    const int nt = g.tiles_m * g.tiles_n, xcd = pid & 7, idx = pid >> 3;
    const int base = nt >> 3, rem = nt & 7;
    pid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  int tm, tn;
  if (g.tm_fast) {
    tm = pid % g.tiles_m;
    tn = pid / g.tiles_m;
  } else {
    tn = pid % g.tiles_n;
    tm = pid / g.tiles_n;
  }
  const int m0 = tm * BM, n0 = tn * BN;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  OpA opa;
  OpB opb;
  opa.init(g.lda, m0, g.M, tid);
  opb.init(g.ldb, n0, g.N, tid);
  const __amdgpu_buffer_rsrc_t ra_src = make_rsrc(g.A, OpA::extent(g.M, g.lda, g.K));
  const __amdgpu_buffer_rsrc_t rb_src = make_rsrc(g.B, OpB::extent(g.N, g.ldb, g.K));
  const uint32_t fa = OpA::frag_base(wm * WM, lane), fb = OpB::frag_base(wn * WN, lane);
  half8_t ra0[OpA::NV], rb0[OpB::NV], ra1[OpA::NV], rb1[OpB::NV];

  auto g2r = [&](half8_t (&ra)[OpA::NV], half8_t (&rb)[OpB::NV], int k0) {
    opa.load(ra, ra_src, g.lda, k0, g.K);
    opb.load(rb, rb_src, g.ldb, k0, g.K);
  };
  auto r2s = [&](const half8_t (&ra)[OpA::NV], const half8_t (&rb)[OpB::NV], int stage) {
    opa.store(ra, smem + stage * STAGE);
    opb.store(rb, smem + stage * STAGE + OpA::BYTES);
  };
  auto compute = [&](int stage) {
    const unsigned char* As = smem + stage * STAGE;
    const unsigned char* Bs = As + OpA::BYTES;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      half8_t af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = OpA::frag(As, fa, i, s);
#pragma unroll
      for (int j = 0; j < TN; ++j) bf[j] = OpB::frag(Bs, fb, j, s);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
  };

  // Software pipeline: LDS holds tile kt, registers hold tile kt+1 and (in flight) tile kt+2, so a
  // global load has two tile computations to land.  The loop body is written twice so that the
  // two register sets and the two LDS stages are addressed statically.
  const int nk = (g.K + BK - 1) / BK;
  g2r(ra0, rb0, 0);
  if (nk > 1) g2r(ra1, rb1, BK);
  r2s(ra0, rb0, 0);
  __syncthreads();
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    if (kt + 2 < nk) g2r(ra0, rb0, (kt + 2) * BK);
    compute(0);
    r2s(ra1, rb1, 1);
    __syncthreads();
    if (kt + 3 < nk) g2r(ra1, rb1, (kt + 3) * BK);
    compute(1);
    if (kt + 2 < nk) r2s(ra0, rb0, 0);
    __syncthreads();
  }
  if (kt < nk) compute(0);  // odd number of k tiles: the last one sits in stage 0
  __syncthreads();

  // ---- epilogue: accumulators -> per-wave LDS staging (fp32) -> row-wise 16-byte stores -------
  constexpr int SP = WN + 4;  // staging row pitch in floats
  float* stg = reinterpret_cast<float*>(smem) + wave * (32 * SP);
  constexpr int CH = WN / 8;  // 8-column chunks per staged row
  const GemmEpilogue& ep = g.ep;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (i) __syncthreads();
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);  // MFMA 32x32 result layout
        stg[row * SP + j * 32 + (lane & 31)] = acc[i][j][r];
      }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < CH / 2; ++it) {
      const int q = it * 64 + lane;
      const int rl = q / CH, c8 = q % CH;
      const int gr = m0 + wm * WM + i * 32 + rl, gc = n0 + wn * WN + c8 * 8;
      if (gr < g.M && gc < g.N) {
        float v[8];
        const floatx4 lo = *reinterpret_cast<const floatx4*>(stg + rl * SP + c8 * 8);
        const floatx4 hi = *reinterpret_cast<const floatx4*>(stg + rl * SP + c8 * 8 + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = lo[e];
          v[4 + e] = hi[e];
        }
        if (ep.bias) {
          const half8_t b = ld_half8(ep.bias + gc);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += (float)b[e];
        }
        if (ep.relu) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
        }
        if (ep.drop.thr) {
          const uint32_t bits = drop_keep8(ep.drop, (uint32_t)gr, (uint32_t)gc >> 3);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = ((bits >> e) & 1u) ? v[e] * ep.drop.scale : 0.f;
        }
        const size_t off = (size_t)gr * g.ldc + gc;
        if (ep.add) {
          const half8_t a = ld_half8(ep.add + off);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += (float)a[e];
        }
        if (ep.relu_src) {
          const half8_t h = ld_half8(ep.relu_src + off);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = ((float)h[e] > 0.f) ? v[e] * ep.mask_scale : 0.f;
        }
        half8_t o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (half_t)v[e];
        st_half8(g.C + off, o);
      }
    }
  }
}

template <int BM, int BN, bool AT, bool BT>
int launch_variant(const GemmArgs& g, hipStream_t stream) {
  constexpr int smem = Tile<BM, BN, AT, BT>::SMEM;
  static bool big_lds_enabled = false;  // dynamic LDS beyond 64 KB has to be allowed once per kernel
  if (smem > 64 * 1024 && !big_lds_enabled) {
    NMT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<BM, BN, AT, BT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, smem));
    big_lds_enabled = true;
  }
  hipLaunchKernelGGL((gemm_kernel<BM, BN, AT, BT>), dim3(g.tiles_m * g.tiles_n), dim3(kThreads), smem, stream, g);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

template <int BM, int BN>
int launch_tile(const GemmArgs& a, bool a_t, bool b_t, hipStream_t stream) {
  GemmArgs g = a;
  g.tiles_m = ceil_div(g.M, BM);
  g.tiles_n = ceil_div(g.N, BN);
  g.tm_fast = g.M <= g.N;
  if (!a_t && !b_t) return launch_variant<BM, BN, false, false>(g, stream);
  if (!a_t && b_t) return launch_variant<BM, BN, false, true>(g, stream);
  if (a_t && b_t) return launch_variant<BM, BN, true, true>(g, stream);
  return launch_variant<BM, BN, true, false>(g, stream);
}

// Estimated efficiency of a tile shape on a (M, N) problem: useful fraction of the padded tiles,
// times how well the tile count fills whole rounds of the 256 CUs, times a per-shape factor (small
// tiles re-read LDS more often per MFMA).
double tile_score(int M, int N, int bm, int bn, int per_cu, double shape_eff) {
  const double tiles = (double)ceil_div(M, bm) * ceil_div(N, bn);
  const double useful = ((double)M * N) / (tiles * bm * bn);
  const double slots = 256.0 * per_cu;
  const double rounds = (tiles + slots - 1) / slots;
  const double fill = tiles / (double)((int64_t)rounds * slots);
  return useful * fill * shape_eff;
}

}  // namespace

int launch_gemm(const half_t* A, bool a_t, int lda, const half_t* B, bool b_t, int ldb, half_t* C, int ldc, int M,
                int N, int K, const GemmEpilogue& ep, hipStream_t stream) {
  NMT_REQUIRE(M > 0 && N > 0 && K > 0, "gemm: empty problem M=%d N=%d K=%d", M, N, K);
  NMT_REQUIRE(A && B && C, "gemm: null operand");
  NMT_REQUIRE(aligned16(A) && aligned16(B) && aligned16(C), "gemm: operands must be 16-byte aligned");
  NMT_REQUIRE(lda % 8 == 0 && ldb % 8 == 0 && ldc % 8 == 0 && N % 8 == 0, "gemm: lda/ldb/ldc/N must be multiples of 8");
  NMT_REQUIRE((a_t ? M : K) % 8 == 0 && (b_t ? N : K) % 8 == 0, "gemm: contiguous operand dimension must be a multiple of 8");
  NMT_REQUIRE(lda >= (a_t ? M : K) && ldb >= (b_t ? N : K) && ldc >= N, "gemm: leading dimension too small");
  NMT_REQUIRE((int64_t)(a_t ? K : M) * lda < (1ll << 30) && (int64_t)(b_t ? K : N) * ldb < (1ll << 30),
              "gemm: operands of 2^30 or more elements are not supported");
  NMT_REQUIRE(!ep.bias || aligned16(ep.bias), "gemm: bias must be 16-byte aligned");
  NMT_REQUIRE((!ep.add || aligned16(ep.add)) && (!ep.relu_src || aligned16(ep.relu_src)), "gemm: epilogue operand misaligned");
  GemmArgs g{A, B, C, lda, ldb, ldc, M, N, K, 0, 0, 0, ep};
  if (const char* force = getenv("NMT_GEMM_TILE")) {  // tuning aid: force one tile shape
    if (!strcmp(force, "128x128")) return launch_tile<128, 128>(g, a_t, b_t, stream);
    if (!strcmp(force, "128x64")) return launch_tile<128, 64>(g, a_t, b_t, stream);
    if (!strcmp(force, "64x128")) return launch_tile<64, 128>(g, a_t, b_t, stream);
    if (!strcmp(force, "64x64")) return launch_tile<64, 64>(g, a_t, b_t, stream);
  }
  const double s128 = tile_score(M, N, 128, 128, 2, 1.0);
  const double s12864 = tile_score(M, N, 128, 64, 2, 0.85);
  const double s64128 = tile_score(M, N, 64, 128, 2, 0.85);
  const double s64 = tile_score(M, N, 64, 64, 4, 0.65);
  if (s128 >= s12864 && s128 >= s64128 && s128 >= s64) return launch_tile<128, 128>(g, a_t, b_t, stream);
  if (s12864 >= s64128 && s12864 >= s64) return launch_tile<128, 64>(g, a_t, b_t, stream);
  if (s64128 >= s64) return launch_tile<64, 128>(g, a_t, b_t, stream);
  return launch_tile<64, 64>(g, a_t, b_t, stream);
}
