// fp32 GEMM on the matrix cores (v_mfma_f32_32x32x2_f32), for the benchmark's comparison leg only: the step's
// products with fp32 operands, i.e. what the same update costs without half precision ("Half-Precision
// Training": the paper's own first measurement is fp32 against fp16 training at equal settings).  Not part of
// the training step; the step never calls it.
//
// C[M,N] = sum_k A(m,k) B(n,k), fp32 in, fp32 out.  Block tile 128 x 128 x 16, four wavefronts (2 x 2) of 64 x 64;
// both operand tiles are kept k-major in LDS ([k][row], padded) so that a wavefront's fragment reads (lane = row
// within the 32 x 32 product, k = lane / 32) are conflict-free whichever way the operand is stored in memory.
#include "common.h"

namespace {

constexpr int BM = 128, BN = 128, BK = 16, PITCH = 128 + 4;  // floats per k row of a tile in LDS

// A [128 rows][16 k] operand tile on its way into LDS as [k][row]: fetch() brings each thread's two float4 from
// global memory into registers, put() writes them to LDS.  direct: memory [rows][K] (k contiguous); transposed:
// memory [K][rows].  Splitting the two lets the global latency pass behind the products of the current tile.
template <bool TRANS>
struct TileLoad {
  floatx4 v[2];
  __device__ __forceinline__ void fetch(const float* __restrict__ p, int ld, int r0, int rows, int k0, int K, int tid) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      v[it] = floatx4{0.f, 0.f, 0.f, 0.f};
      if (!TRANS) {  // 512 float4 along k; thread t: row t / 4 (+64), k chunk t % 4
        const int gr = r0 + (tid >> 2) + 64 * it, gk = k0 + (tid & 3) * 4;
        if (gr < rows) {
          const float* src = p + (size_t)gr * ld + gk;
          if (gk + 3 < K) v[it] = *reinterpret_cast<const floatx4*>(src);
          else
#pragma unroll
            for (int e = 0; e < 4; ++e) if (gk + e < K) v[it][e] = src[e];
        }
      } else {       // 512 float4 along rows; thread t: k t / 32 (+8), row chunk t % 32
        const int gk = k0 + (tid >> 5) + 8 * it, gr = r0 + (tid & 31) * 4;
        if (gk < K) {
          const float* src = p + (size_t)gk * ld + gr;
          if (gr + 3 < rows) v[it] = *reinterpret_cast<const floatx4*>(src);
          else
#pragma unroll
            for (int e = 0; e < 4; ++e) if (gr + e < rows) v[it][e] = src[e];
        }
      }
    }
  }
  __device__ __forceinline__ void put(float* lds, int tid) const {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      if (!TRANS) {
        const int row = (tid >> 2) + 64 * it, kc = (tid & 3) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) lds[(kc + e) * PITCH + row] = v[it][e];
      } else {
        const int k = (tid >> 5) + 8 * it, rc = (tid & 31) * 4;
        *reinterpret_cast<floatx4*>(lds + k * PITCH + rc) = v[it];
      }
    }
  }
};

template <bool AT, bool BT>
__global__ void __launch_bounds__(256) gemm_f32_kernel(const float* __restrict__ A, int lda, const float* __restrict__ B, int ldb,
                                                       float* __restrict__ C, int ldc, int M, int N, int K, int k_chunk) {
  __shared__ __align__(16) float As[2][BK * PITCH];
  __shared__ __align__(16) float Bs[2][BK * PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  // piece blockIdx.z of the contraction: k in [z * k_chunk, min(K, (z + 1) * k_chunk)), partial product to block z of C
  const int kb = blockIdx.z * k_chunk;
  if (AT) A += (size_t)kb * lda; else A += kb;
  if (BT) B += (size_t)kb * ldb; else B += kb;
  C += (size_t)blockIdx.z * M * ldc;
  K = min(K - kb, k_chunk);
  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int nk = (K + BK - 1) / BK;
  TileLoad<AT> la;
  TileLoad<BT> lb;
  la.fetch(A, lda, m0, M, 0, K, tid);
  lb.fetch(B, ldb, n0, N, 0, K, tid);
  la.put(As[0], tid);
  lb.put(Bs[0], tid);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {  // the next tile is requested now and written to the other buffer after this one's products
      la.fetch(A, lda, m0, M, (kt + 1) * BK, K, tid);
      lb.fetch(B, ldb, n0, N, (kt + 1) * BK, K, tid);
    }
    const float* a = As[cur] + (lane >> 5) * PITCH + wm * 64 + (lane & 31);
    const float* b = Bs[cur] + (lane >> 5) * PITCH + wn * 64 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < BK / 2; ++ks) {
      float af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) af[i] = a[2 * ks * PITCH + 32 * i];
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[j] = b[2 * ks * PITCH + 32 * j];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)  // B first: lane = row of C, registers = columns (as in the fp16 kernel)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bf[j], af[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      la.put(As[cur ^ 1], tid);
      lb.put(Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }
  // result layout: lane l holds row l % 32 of the 32 x 32 product and, in registers 4q..4q+3, columns 8q + 4(l/32) .. +3
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int gr = m0 + wm * 64 + 32 * i + (lane & 31), gc = n0 + wn * 64 + 32 * j + 8 * q + 4 * (lane >> 5);
        if (gr < M) {
          float* dst = C + (size_t)gr * ldc + gc;
          if (gc + 3 < N) *reinterpret_cast<floatx4*>(dst) = floatx4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          else
#pragma unroll
            for (int e = 0; e < 4; ++e) if (gc + e < N) dst[e] = acc[i][j][4 * q + e];
        }
      }
}

}  // namespace

int launch_gemm_f32(const float* A, bool a_t, int lda, const float* B, bool b_t, int ldb, float* C, int ldc, int M, int N, int K,
                    int splits, hipStream_t stream) {
  NMT_REQUIRE(M > 0 && N > 0 && K > 0 && A && B && C, "gemm_f32: empty problem or null operand");
  NMT_REQUIRE(aligned16(A) && aligned16(B) && aligned16(C) && lda % 4 == 0 && ldb % 4 == 0 && ldc % 4 == 0, "gemm_f32: operands must be 16-byte aligned, leading dimensions multiples of 4");
  NMT_REQUIRE(lda >= (a_t ? M : K) && ldb >= (b_t ? N : K) && ldc >= N, "gemm_f32: leading dimension too small");
  NMT_REQUIRE(splits >= 1 && splits <= 64, "gemm_f32: splits %d outside [1, 64]", splits);
  const int k_chunk = (int)round_up(ceil_div(K, splits), 4);   // (pieces start 16-byte aligned)
  splits = ceil_div(K, k_chunk);
  const dim3 grid(ceil_div(N, BN), ceil_div(M, BM), splits), block(256);
  if (!a_t && !b_t) hipLaunchKernelGGL((gemm_f32_kernel<false, false>), grid, block, 0, stream, A, lda, B, ldb, C, ldc, M, N, K, k_chunk);
  else if (!a_t && b_t) hipLaunchKernelGGL((gemm_f32_kernel<false, true>), grid, block, 0, stream, A, lda, B, ldb, C, ldc, M, N, K, k_chunk);
  else if (a_t && b_t) hipLaunchKernelGGL((gemm_f32_kernel<true, true>), grid, block, 0, stream, A, lda, B, ldb, C, ldc, M, N, K, k_chunk);
  else hipLaunchKernelGGL((gemm_f32_kernel<true, false>), grid, block, 0, stream, A, lda, B, ldb, C, ldc, M, N, K, k_chunk);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}
