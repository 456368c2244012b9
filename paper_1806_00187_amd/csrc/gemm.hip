// fp16-in / fp32-accumulate MFMA GEMM with LDS-staged tiles and a fused epilogue
// (bias, ReLU, dropout, residual/gradient add, ReLU-backward mask) for gfx950.
//
// C[M,N] = epilogue(sum_k A(m,k) * B(n,k)).  Either operand may be stored with the contraction
// index contiguous ("direct") or with its other index contiguous ("transposed"); transposed
// operands are turned around in registers (8x8 blocks) on their way into LDS, so the LDS tiles
// always hold 8 consecutive k per 16-byte chunk, which is what one MFMA lane consumes.
// This covers the three products of a linear layer: forward x W^T (both direct), input gradient
// dy W (B transposed) and weight gradient dy^T x (both transposed).
#include "common.h"

namespace {

constexpr int BK = 64;        // k extent of one LDS stage (8 chunks of 8 halfs per row)
constexpr int kThreads = 256; // 4 wavefronts, arranged 2 x 2 over the block tile

struct GemmArgs {
  const half_t* A;
  const half_t* B;
  half_t* C;
  int lda, ldb, ldc, M, N, K;
  int tiles_m, tiles_n, tm_fast;
  GemmEpilogue ep;
};

// Offset (in halfs) of chunk `c` (8 halfs) of tile row `row`.  The XOR swizzle makes the three
// access patterns conflict-free: MFMA fragment reads (32 consecutive rows, one chunk), direct
// stores (one row, 8 chunks) and transposed stores (rows 8 apart, one chunk).
__device__ __forceinline__ int lds_off(int row, int c) { return row * BK + (((c ^ row ^ (row >> 3)) & 7) << 3); }

template <int R>
__device__ __forceinline__ void load_direct(half8_t (&v)[R / 32], const half_t* __restrict__ base, int ld, int r0,
                                            int rmax, int k0, int K, int tid) {
#pragma unroll
  for (int it = 0; it < R / 32; ++it) {
    const int q = it * kThreads + tid;
    const int gr = r0 + (q >> 3), gk = k0 + ((q & 7) << 3);
    v[it] = (gr < rmax && gk < K) ? ld_half8(base + (size_t)gr * ld + gk) : zero_half8();
  }
}
template <int R>
__device__ __forceinline__ void store_direct(const half8_t (&v)[R / 32], half_t* tile, int tid) {
#pragma unroll
  for (int it = 0; it < R / 32; ++it) {
    const int q = it * kThreads + tid;
    st_half8(tile + lds_off(q >> 3, q & 7), v[it]);
  }
}
// Transposed operand: stored [K][R] with R contiguous.  Thread slot t < R owns the 8(k) x 8(r) block
// (kb = t / (R/8), rb = t % (R/8)).
template <int R>
__device__ __forceinline__ void load_trans(half8_t (&v)[8], const half_t* __restrict__ base, int ld, int r0, int rmax,
                                           int k0, int K, int t) {
  if (t < R) {
    const int rb = t % (R / 8), kb = t / (R / 8);
    const int gr = r0 + rb * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int gk = k0 + kb * 8 + j;
      v[j] = (gk < K && gr < rmax) ? ld_half8(base + (size_t)gk * ld + gr) : zero_half8();
    }
  }
}
template <int R>
__device__ __forceinline__ void store_trans(const half8_t (&v)[8], half_t* tile, int t) {
  if (t < R) {
    const int rb = t % (R / 8), kb = t / (R / 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      half8_t o;
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = v[j][i];
      st_half8(tile + lds_off(rb * 8 + i, kb), o);
    }
  }
}

template <int BM, int BN, bool AT, bool BT>
__global__ void __launch_bounds__(kThreads) gemm_kernel(const GemmArgs g) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  half_t* smem = reinterpret_cast<half_t*>(smem_raw);
  constexpr int A_ELEMS = BM * BK, B_ELEMS = BN * BK, STAGE = A_ELEMS + B_ELEMS;
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

  half8_t ra[AT ? 8 : BM / 32];
  half8_t rb[BT ? 8 : BN / 32];
  const int tb = (BN <= 128) ? ((tid + 128) & 255) : tid;  // spread transposed-B work over the idle half

  auto g2r = [&](int k0) {
    if constexpr (AT) load_trans<BM>(ra, g.A, g.lda, m0, g.M, k0, g.K, tid);
    else load_direct<BM>(ra, g.A, g.lda, m0, g.M, k0, g.K, tid);
    if constexpr (BT) load_trans<BN>(rb, g.B, g.ldb, n0, g.N, k0, g.K, tb);
    else load_direct<BN>(rb, g.B, g.ldb, n0, g.N, k0, g.K, tid);
  };
  auto r2s = [&](int stage) {
    half_t* As = smem + stage * STAGE;
    half_t* Bs = As + A_ELEMS;
    if constexpr (AT) store_trans<BM>(ra, As, tid);
    else store_direct<BM>(ra, As, tid);
    if constexpr (BT) store_trans<BN>(rb, Bs, tb);
    else store_direct<BN>(rb, Bs, tid);
  };

  const int nk = (g.K + BK - 1) / BK;
  g2r(0);
  r2s(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) g2r((kt + 1) * BK);  // global loads for the next stage fly during the MFMAs
    const half_t* As = smem + (kt & 1) * STAGE;
    const half_t* Bs = As + A_ELEMS;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      half8_t af[TM], bf[TN];
      const int c = s * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = ld_half8(As + lds_off(wm * WM + i * 32 + (lane & 31), c));
#pragma unroll
      for (int j = 0; j < TN; ++j) bf[j] = ld_half8(Bs + lds_off(wn * WN + j * 32 + (lane & 31), c));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) r2s((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: accumulators -> per-wave LDS staging (fp32) -> row-wise 16-byte stores -------
  constexpr int SP = WN + 4;  // staging row pitch in floats
  float* stg = reinterpret_cast<float*>(smem_raw) + wave * (32 * SP);
  constexpr int CH = WN / 8;  // 8-column chunks per staged row
  const GemmEpilogue& ep = g.ep;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    __syncthreads();
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

template <int BM, int BN>
int launch_tile(const GemmArgs& a, bool a_t, bool b_t, hipStream_t stream) {
  GemmArgs g = a;
  g.tiles_m = ceil_div(g.M, BM);
  g.tiles_n = ceil_div(g.N, BN);
  g.tm_fast = g.M <= g.N;
  const dim3 grid(g.tiles_m * g.tiles_n), block(kThreads);
  const size_t smem = 2 * (BM + BN) * BK * sizeof(half_t);
  if (!a_t && !b_t) hipLaunchKernelGGL((gemm_kernel<BM, BN, false, false>), grid, block, smem, stream, g);
  else if (!a_t && b_t) hipLaunchKernelGGL((gemm_kernel<BM, BN, false, true>), grid, block, smem, stream, g);
  else if (a_t && b_t) hipLaunchKernelGGL((gemm_kernel<BM, BN, true, true>), grid, block, smem, stream, g);
  else hipLaunchKernelGGL((gemm_kernel<BM, BN, true, false>), grid, block, smem, stream, g);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
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
  NMT_REQUIRE(!ep.bias || aligned16(ep.bias), "gemm: bias must be 16-byte aligned");
  NMT_REQUIRE((!ep.add || aligned16(ep.add)) && (!ep.relu_src || aligned16(ep.relu_src)), "gemm: epilogue operand misaligned");
  GemmArgs g{A, B, C, lda, ldb, ldc, M, N, K, 0, 0, 0, ep};
  const double s128 = tile_score(M, N, 128, 128, 2, 1.0);
  const double s12864 = tile_score(M, N, 128, 64, 2, 0.85);
  const double s64128 = tile_score(M, N, 64, 128, 2, 0.85);
  const double s64 = tile_score(M, N, 64, 64, 4, 0.65);
  if (s128 >= s12864 && s128 >= s64128 && s128 >= s64) return launch_tile<128, 128>(g, a_t, b_t, stream);
  if (s12864 >= s64128 && s12864 >= s64) return launch_tile<128, 64>(g, a_t, b_t, stream);
  if (s64128 >= s64) return launch_tile<64, 128>(g, a_t, b_t, stream);
  return launch_tile<64, 64>(g, a_t, b_t, stream);
}
