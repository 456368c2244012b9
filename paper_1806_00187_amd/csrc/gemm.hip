// fp16-in / fp32-accumulate MFMA GEMM with LDS-staged tiles and a fused epilogue
// (bias, ReLU, dropout, residual/gradient add, ReLU-backward mask) for gfx950.
//
// C[M,N] = epilogue(sum_k A(m,k) * B(n,k)).  Either operand may be stored with the contraction
// index contiguous ("direct": [rows][K]) or with its other index contiguous ("transposed":
// [K][rows]).  This covers the three products of a linear layer: forward x W^T (both direct),
// input gradient dy W (B transposed) and weight gradient dy^T x (both transposed).
//
// The kernel is bound by LDS instruction throughput, not by the matrix cores: measured on this
// chip a wave's ds_read_b128 streams ~64 B/clk per CU and ds_write_b128 half of that, against
// 4096 MFMA flop/clk.  The data path therefore avoids every LDS instruction it can:
//  * global -> LDS directly (buffer_load ... lds, 16 bytes per lane, 1 KB contiguous per wave
//    instruction): no ds_write, no staging registers.  Out-of-range rows / k (offset beyond the
//    buffer's extent) arrive as zeros, so ragged edges need no branches;
//  * both tile layouts are kept as they are in memory (direct [row][64 k], transposed
//    [64 k][row]) and made bank-conflict free by permuting, on the global-address side, which
//    16-byte chunk lands in which slot (XOR swizzles chosen so that every LDS address is one
//    per-lane base plus compile-time offsets);
//  * LDS -> MFMA fragments: one ds_read_b128 per fragment for a direct tile; two
//    ds_read_b64_tr_b16 (the gfx950 transposing read: within 16 lanes, lane L receives element
//    L%4 of the 8-byte words addressed by lanes 4j + L/4, j = 0..3) for a transposed tile, so
//    no register shuffling is needed;
//  * two LDS stages: the k-tile after the one being multiplied streams in meanwhile.
#include <stdlib.h>

#include <type_traits>

#include "common.h"

namespace {

constexpr int BK = 64;         // k extent of one LDS stage
constexpr int kThreads = 256;  // 4 wavefronts, arranged 2 x 2 over the block tile
constexpr uint32_t kOob = 0x80000000u;  // byte offset no operand reaches: such loads return 0

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef short short8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) short4_t* lds_short4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

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
// One wave instruction: lane L's 16 bytes at byte offset `voff` of the buffer land at lds + 16 L.
// The whole offset travels in the per-lane operand, which is what the hardware range-checks.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned char* lds_wave_base, uint32_t voff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)lds_wave_base, 16, (int)voff, 0, 0, 0);
}

// ---- direct operand: memory [rows][K] (k contiguous), LDS tile [R][64 k], 128 bytes per row ------
// Slot p (16 bytes) of tile row r holds chunk p ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 1).
template <int R>
struct DirectOp {
  static constexpr int NV = R / 32;   // wave instructions (8 rows each) per wave and k-tile
  static constexpr int BYTES = R * 128;
  uint32_t voff[NV];
  int c8, wave;
  __device__ __forceinline__ static uint32_t extent(int rmax, int ld, int K) { return ((uint32_t)(rmax - 1) * ld + K) * 2u; }
  __device__ __forceinline__ void init(int ld, int r0, int rmax, int tid) {
    wave = tid >> 6;
    const int L = tid & 63, rowl = L >> 3, p = L & 7;
    c8 = (p ^ rowl ^ (wave & 1)) << 3;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int row = r0 + 8 * (wave + 4 * it) + rowl;
      voff[it] = row < rmax ? ((uint32_t)row * (uint32_t)ld + (uint32_t)c8) * 2u : kOob;
    }
  }
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, unsigned char* tile, int ld, int k0, int K) const {
    const bool kv = k0 + c8 < K;  // only the last k-tile can fail this
#pragma unroll
    for (int it = 0; it < NV; ++it) dma16(rsrc, tile + (wave + 4 * it) * 1024, kv ? voff[it] + (uint32_t)k0 * 2u : kOob);
  }
  // per-lane fragment addresses, one per k-step (the swizzle is an XOR in the k-step bits)
  struct Frag { uint32_t a[BK / 16]; };
  __device__ __forceinline__ static Frag frag_init(int row0, int lane) {
    Frag f;
    const int h = (lane >> 5) ^ (lane & 7) ^ ((lane >> 3) & 1);
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) f.a[s] = (row0 + (lane & 31)) * 128 + (((h ^ (2 * s)) & 7) << 4);
    return f;
  }
  __device__ __forceinline__ static half8_t frag(const unsigned char* tile, const Frag& f, int i, int s) {
    return *reinterpret_cast<const half8_t*>(tile + f.a[s] + i * 32 * 128);
  }
};

// ---- transposed operand: memory [K][rows] (rows contiguous), LDS tile [64 k][R] -------------------
// Within k row k, slot q (16 bytes) holds chunk q ^ (y(k) << 1): the four k rows a 16-lane group of
// the transposing read touches then lie in four different 32-byte bank segments.
template <int R>
struct TransOp {
  static constexpr int NV = R / 32;
  static constexpr int ROWB = R * 2;        // bytes per k row
  static constexpr int BYTES = BK * ROWB;
  static constexpr int CPR = R / 8;         // 16-byte chunks per k row
  static constexpr int KPI = 64 / CPR;      // k rows per wave instruction
  uint32_t voff[NV];
  int wave;
  __device__ __forceinline__ static int ysw(int k2) { return R == 128 ? ((k2 & 1) | ((k2 & 2) << 1)) : (k2 & 3); }
  __device__ __forceinline__ static uint32_t extent(int rmax, int ld, int K) { return ((uint32_t)(K - 1) * ld + rmax) * 2u; }
  __device__ __forceinline__ void init(int ld, int r0, int rmax, int tid) {
    wave = tid >> 6;
    const int L = tid & 63, kl = L / CPR, slot = L % CPR;
    const int cc = slot ^ (ysw(kl & 3) << 1);
    const bool ok = r0 + cc * 8 < rmax;
#pragma unroll
    for (int it = 0; it < NV; ++it)
      voff[it] = ok ? ((uint32_t)(KPI * (wave + 4 * it) + kl) * (uint32_t)ld + (uint32_t)(r0 + cc * 8)) * 2u : kOob;
  }
  // k rows >= K lie beyond the buffer's extent and arrive as zeros
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, unsigned char* tile, int ld, int k0, int K) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) dma16(rsrc, tile + (wave + 4 * it) * 1024, voff[it] + (uint32_t)k0 * (uint32_t)ld * 2u);
  }
  struct Frag { uint32_t a; };
  // 16-lane group q = lane/16 serves rows 16*(q&1).. of the MFMA tile and k-half q/2; lane i of the group
  // addresses k row i/4, row offset 4*(i%4) of its 4(k) x 16(row) block.
  __device__ __forceinline__ static Frag frag_init(int row0, int lane) {
    const int q = lane >> 4, i = lane & 15;
    const int kk = 8 * (q >> 1) + (i >> 2);
    const int r = row0 + 16 * (q & 1) + 4 * (i & 3);
    const int cc = (r >> 3) ^ (ysw((i >> 2) & 3) << 1);
    return Frag{(uint32_t)(kk * ROWB + cc * 16 + (r & 7) * 2)};
  }
  __device__ __forceinline__ static half8_t frag(const unsigned char* tile, const Frag& f, int i, int s) {
    const unsigned char* p = tile + f.a + s * 16 * ROWB + i * 64;
    const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p));
    const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p + 4 * ROWB));
    const short8_t r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(half8_t, r);
  }
};

template <int BM, int BN, bool AT, bool BT>
struct Tile {
  using OpA = typename std::conditional<AT, TransOp<BM>, DirectOp<BM>>::type;
  using OpB = typename std::conditional<BT, TransOp<BN>, DirectOp<BN>>::type;
  static constexpr int STAGE = OpA::BYTES + OpB::BYTES;   // (BM + BN) * 128 bytes
};

template <int BM, int BN, bool AT, bool BT>
__global__ void __launch_bounds__(kThreads) gemm_kernel(const GemmArgs g) {
  using T = Tile<BM, BN, AT, BT>;
  using OpA = typename T::OpA;
  using OpB = typename T::OpB;
  // two separate arrays, so that the compiler can tell that fragment reads of one stage do not
  // depend on the loads in flight into the other
  __shared__ __align__(1024) unsigned char stage0[T::STAGE];
  __shared__ __align__(1024) unsigned char stage1[T::STAGE];
  constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // Work-group -> tile.  Consecutive work-group ids go round-robin over the 8 XCDs; undo that so
  // each XCD (own L2) gets a contiguous run of tiles.
  int pid = blockIdx.x;
  {
    const int nt = g.tiles_m * g.tiles_n, xcd = pid & 7, idx = pid >> 3;
    const int base = nt >> 3, rem = nt & 7;
    pid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  // Grouped order: 8 tile rows are swept column by column, so the ~64 work-groups an XCD runs at a
  // time form an 8 x 8 patch of tiles and each A / B panel they stream is shared by 8 of them in L2.
  int tm, tn;
  {
    constexpr int GROUP = 8;
    const int per_group = GROUP * g.tiles_n;
    const int first = (pid / per_group) * GROUP;
    const int rows = min(g.tiles_m - first, GROUP);
    tm = first + (pid % per_group) % rows;
    tn = (pid % per_group) / rows;
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
  const typename OpA::Frag fa = OpA::frag_init(wm * WM, lane);
  const typename OpB::Frag fb = OpB::frag_init(wn * WN, lane);

  auto request = [&](unsigned char* stage, int k0) {  // asynchronous: tile k0 streams into `stage`
    opa.load(ra_src, stage, g.lda, k0, g.K);
    opb.load(rb_src, stage + OpA::BYTES, g.ldb, k0, g.K);
    __builtin_amdgcn_sched_barrier(0);  // keep the requests ahead of the products they overlap with
  };
  auto compute = [&](const unsigned char* stage) {
    const unsigned char* As = stage;
    const unsigned char* Bs = stage + OpA::BYTES;
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
  // all of this wave's loads into LDS have landed (vmcnt(0)); the barrier then publishes every wave's part
  auto landed = [&]() {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  };

  // A k-tile past the end reads zeros (its offsets are out of range) and multiplying it changes
  // nothing, so the loop always runs in pairs and carries no edge conditions.
  const int nk = (g.K + BK - 1) / BK;
  request(stage0, 0);
  landed();
  for (int kt = 0; kt < nk; kt += 2) {
    request(stage1, (kt + 1) * BK);
    compute(stage0);
    landed();
    request(stage0, (kt + 2) * BK);
    compute(stage1);
    landed();
  }

  // ---- epilogue: accumulators -> per-wave LDS staging (fp32) -> row-wise 16-byte stores -------
  // staging width per pass: the wave's whole width if 4 waves x 32 rows of it fit one stage, else 32
  constexpr int SW = (4 * 32 * WN * 4 <= T::STAGE) ? WN : 32;
  static_assert(4 * 32 * SW * 4 <= T::STAGE, "epilogue staging does not fit");
  float* stg = reinterpret_cast<float*>(stage1) + wave * (32 * SW);
  constexpr int CH = SW / 8;  // 8-column chunks per staged row
  const GemmEpilogue& ep = g.ep;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int jg = 0; jg < WN / SW; ++jg) {
      if (i || jg) __syncthreads();
#pragma unroll
      for (int jj = 0; jj < SW / 32; ++jj)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);  // MFMA 32x32 result layout
          stg[row * SW + jj * 32 + (lane & 31)] = acc[i][jg * (SW / 32) + jj][r];
        }
      __syncthreads();
#pragma unroll
      for (int it = 0; it < CH / 2; ++it) {
        const int q = it * 64 + lane;
        const int rl = q / CH, c8 = q % CH;
        const int gr = m0 + wm * WM + i * 32 + rl, gc = n0 + wn * WN + jg * SW + c8 * 8;
        if (gr < g.M && gc < g.N) {
          float v[8];
          const floatx4 lo = *reinterpret_cast<const floatx4*>(stg + rl * SW + c8 * 8);
          const floatx4 hi = *reinterpret_cast<const floatx4*>(stg + rl * SW + c8 * 8 + 4);
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
}

template <int BM, int BN, bool AT, bool BT>
int launch_variant(const GemmArgs& g, hipStream_t stream) {
  hipLaunchKernelGGL((gemm_kernel<BM, BN, AT, BT>), dim3(g.tiles_m * g.tiles_n), dim3(kThreads), 0, stream, g);
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
