// fp16-in / fp32-accumulate MFMA GEMM with LDS-staged tiles and a fused epilogue
// (bias, ReLU, dropout, residual/gradient add, ReLU-backward mask) for gfx950.
//
// C[M,N] = epilogue(sum_k A(m,k) * B(n,k)).  Either operand may be stored with the contraction
// index contiguous ("direct": [rows][K]) or with its other index contiguous ("transposed":
// [K][rows]).  This covers the three products of a linear layer: forward x W^T (both direct),
// input gradient dy W (B transposed) and weight gradient dy^T x (both transposed).
//
// Measured on this chip: ds_read_b128 streams ~200 B/clk per CU (the 8-byte transposing read half
// of that), global -> LDS loads ~50 B/clk per CU, and with fp16 data of full entropy the sustained
// rate of LDS reads + MFMAs alone is ~1.2-1.35 PFLOP/s (clocks drop under that load).  The loop is
// therefore organised around the load path and around keeping the matrix pipe fed:
//  * global -> LDS directly (buffer_load ... lds, 16 bytes per lane, 1 KB contiguous per wave
//    instruction): no ds_write, no staging registers.  Every k-tile gets a buffer descriptor that
//    starts at the tile's first element and ends at its last, so out-of-range rows / k arrive as
//    zeros, ragged edges need no branches, and operands may be larger than 4 GB;
//  * both tile layouts are kept as they are in memory (direct [row][k], transposed [k][row]) and
//    made bank-conflict free by permuting, on the global-address side, which 16-byte chunk lands
//    in which slot (XOR swizzles chosen so that every LDS address is one per-lane base plus
//    compile-time offsets);
//  * LDS -> MFMA fragments: one ds_read_b128 per fragment for a direct tile; two
//    ds_read_b64_tr_b16 (the gfx950 transposing read: within 16 lanes, lane L receives element
//    L%4 of the 8-byte words addressed by lanes 4j + L/4, j = 0..3) for a transposed tile, so
//    no register shuffling is needed;
//  * the fragments of k-step s+1 are read while the MFMAs of step s issue (two register sets,
//    instruction order pinned with scheduling groups);
//  * a ring of 2 or 4 LDS stages: the next 1 or 3 k-tiles stream in while one is multiplied; one
//    barrier per k-tile both publishes the next tile and frees the current one for refilling.
#include <stdlib.h>

#include <mutex>
#include <type_traits>
#include <vector>

#include "common.h"

namespace {

constexpr int kThreads = 256;  // threads of the split-k reduction kernel
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
  int tiles_m, tiles_n, group_m;
  int xcds;  // dies with their own L2: consecutive work-group ids go round-robin over them
  GemmEpilogue ep;
  // split-K: work-group (tile, z) contracts k in [z * k_chunk, min(K, (z + 1) * k_chunk)) and writes its
  // fp32 tile to partial[z][M][N]; partial == nullptr: one work-group per tile, epilogue, fp16 result
  float* partial;
  int k_chunk;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const half_t* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(p), 0, (int)bytes, 0x00020000);
}
// One wave instruction: lane L's 16 bytes at byte offset `voff` of the buffer land at lds + 16 L.
// The whole offset travels in the per-lane operand, which is what the hardware range-checks.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned char* lds_wave_base, uint32_t voff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)lds_wave_base, 16, (int)voff, 0, 0, 0);
}

// ---- direct operand: memory [rows][K] (k contiguous), LDS tile [R][BK k] -------------------------
// BK = 64: 128 bytes per row; slot p (16 bytes) of row r holds chunk p ^ (r & 7) ^ ((r >> 3) & 1).
// BK = 32:  64 bytes per row; slot p of row r holds chunk p ^ ((r >> 2) & 3).
// Either way a wavefront's ds_read_b128 of 32 rows x 2 chunks touches every bank equally often.
// All offsets are relative to the first element of the block's current k-tile, so operands of any
// size work with 32-bit offsets.
template <int R, int BK, int NW>
struct DirectOp {
  static constexpr int ROWB = BK * 2;             // bytes per tile row
  static constexpr int CPR = BK / 8;              // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;            // rows per wave instruction (1 KB)
  static constexpr int BYTES = R * ROWB;
  static constexpr int NV = BYTES / (1024 * NW);  // wave instructions per wave and k-tile
  static_assert(NV >= 1 && BYTES % (1024 * NW) == 0, "tile too small for the work-group's waves");
  uint32_t voff[NV];
  int c8, wave;
  __device__ __forceinline__ static int swz(int row) { return BK == 64 ? ((row & 7) ^ ((row >> 3) & 1)) : ((row >> 2) & 3); }
  // first element of the k-tile at k0 of the block whose first row is r0
  __device__ __forceinline__ static const half_t* origin(const half_t* p, int ld, int r0, int k0) { return p + (size_t)r0 * ld + k0; }
  // bytes from there to the end of the tile's last row (0 if the k-tile lies past K)
  __device__ __forceinline__ static uint32_t extent(int rows_in, int ld, int kleft) {
    return kleft > 0 ? ((uint32_t)(rows_in - 1) * ld + (uint32_t)min(kleft, BK)) * 2u : 0u;
  }
  __device__ __forceinline__ void init(int ld, int rows_in, int tid) {
    wave = tid >> 6;
    const int L = tid & 63, rowl = L / CPR, p = L % CPR;
    // RPI * (wave + NW it) adds nothing to the swizzle bits except, for BK = 64, bit 3 of the row (= wave & 1)
    c8 = (p ^ swz(RPI * wave + rowl)) << 3;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int row = RPI * (wave + NW * it) + rowl;
      voff[it] = row < rows_in ? ((uint32_t)row * (uint32_t)ld + (uint32_t)c8) * 2u : kOob;
    }
  }
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, unsigned char* tile, int kleft) const {
    const bool kv = c8 < kleft;  // only the last k-tile can fail this
#pragma unroll
    for (int it = 0; it < NV; ++it) dma16(rsrc, tile + (wave + NW * it) * 1024, kv ? voff[it] : kOob);
  }
  // per-lane fragment addresses, one per k-step (the swizzle is an XOR in the k-step bits)
  struct Frag { uint32_t a[BK / 16]; };
  __device__ __forceinline__ static Frag frag_init(int row0, int lane) {
    Frag f;
    const int row = row0 + (lane & 31);  // row0 and the 32-row steps between MFMA tiles leave the swizzle bits alone
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) f.a[s] = row * ROWB + (((((lane >> 5) | (2 * s)) ^ swz(lane & 31)) & (CPR - 1)) << 4);
    return f;
  }
  static constexpr int READS = 1;  // LDS instructions per fragment
  __device__ __forceinline__ static half8_t frag(const unsigned char* tile, const Frag& f, int i, int s) {
    return *reinterpret_cast<const half8_t*>(tile + f.a[s] + i * 32 * ROWB);
  }
};

// ---- transposed operand: memory [K][rows] (rows contiguous), LDS tile [BK k][R] -------------------
// Within k row k, slot q (16 bytes) holds chunk q ^ sw(k & 3).  A transposing read serves 32 lanes at a
// time: two 16-lane groups (MFMA rows 0..15 and 16..31), each touching four k rows x two chunks.  With
// sw(k) = k << 2 (chunk bits 2 and 3; bit 0 counts the two chunks of a group, bit 1 the group) those
// sixteen chunks are all different, i.e. the 32 lanes cover every bank of a 256-byte row segment once.
// (A 64-wide tile has only 8 chunks per k row: there sw(k) = k << 1 and the two groups share banks.)
template <int R, int BK, int NW>
struct TransOp {
  static constexpr int ROWB = R * 2;        // bytes per k row
  static constexpr int BYTES = BK * ROWB;
  static constexpr int NV = BYTES / (1024 * NW);
  static constexpr int CPR = R / 8;         // 16-byte chunks per k row
  static constexpr int KPI = 64 / CPR;      // k rows per wave instruction
  static_assert(NV >= 1 && BYTES % (1024 * NW) == 0, "tile too small for the work-group's waves");
  uint32_t voff[NV];
  int wave;
  __device__ __forceinline__ static int sw(int k) { return (k & 3) << (R == 64 ? 1 : 2); }
  __device__ __forceinline__ static const half_t* origin(const half_t* p, int ld, int r0, int k0) { return p + (size_t)k0 * ld + r0; }
  // k rows >= K lie beyond the extent and arrive as zeros
  __device__ __forceinline__ static uint32_t extent(int rows_in, int ld, int kleft) {
    return kleft > 0 ? ((uint32_t)(min(kleft, BK) - 1) * ld + (uint32_t)rows_in) * 2u : 0u;
  }
  __device__ __forceinline__ void init(int ld, int rows_in, int tid) {
    wave = tid >> 6;
    const int L = tid & 63, kl = L / CPR, slot = L % CPR;
    const int cc = slot ^ sw(KPI * wave + kl);  // k row of instruction `it` is KPI * (wave + NW it) + kl: same k & 3 for every it
    const bool ok = cc * 8 < rows_in;
#pragma unroll
    for (int it = 0; it < NV; ++it)
      voff[it] = ok ? ((uint32_t)(KPI * (wave + NW * it) + kl) * (uint32_t)ld + (uint32_t)(cc * 8)) * 2u : kOob;
  }
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, unsigned char* tile, int /*kleft*/) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) dma16(rsrc, tile + (wave + NW * it) * 1024, voff[it]);
  }
  static constexpr int READS = 2;
  struct Frag { uint32_t a[4]; };  // one address per MFMA tile of the wave (the swizzle reaches the bits a tile step changes)
  // 16-lane group q = lane/16 serves rows 16*(q&1).. of the MFMA tile and k-half q/2; lane i of the group
  // addresses k row i/4, row offset 4*(i%4) of its 4(k) x 16(row) block.
  __device__ __forceinline__ static Frag frag_init(int row0, int lane) {
    const int q = lane >> 4, i = lane & 15;
    const int kk = 8 * (q >> 1) + (i >> 2);
    Frag f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int r = row0 + 32 * t + 16 * (q & 1) + 4 * (i & 3);
      const int cc = ((r >> 3) ^ sw(i >> 2)) & (CPR - 1);   // (tiles past the wave's share are never read)
      f.a[t] = (uint32_t)(kk * ROWB + cc * 16 + (r & 7) * 2);
    }
    return f;
  }
  __device__ __forceinline__ static half8_t frag(const unsigned char* tile, const Frag& f, int i, int s) {
    const unsigned char* p = tile + f.a[i] + s * 16 * ROWB;
    const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p));
    const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p + 4 * ROWB));
    const short8_t r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(half8_t, r);
  }
};

// Instruction order of one k-step: the NR LDS reads of the next step's fragments go between the
// first three quarters of this step's MF matrix instructions, so that every read has returned
// before the next step starts.
template <int M, int MF, int NR>
struct Interleave {
  static constexpr int SLOTS = MF - MF / 4, PER = (NR + SLOTS - 1) / SLOTS;
  static constexpr int DONE = M * PER < NR ? M * PER : NR, NOW = NR - DONE < PER ? NR - DONE : PER;
  __device__ __forceinline__ static void run() {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
    if (NOW > 0) __builtin_amdgcn_sched_group_barrier(0x100, NOW, 0);
    Interleave<M + 1, MF, NR>::run();
  }
};
template <int MF, int NR>
struct Interleave<MF, MF, NR> {
  __device__ __forceinline__ static void run() {}
};

template <int BM, int BN, bool AT, bool BT, int BK, int NW>
struct Tile {
  using OpA = typename std::conditional<AT, TransOp<BM, BK, NW>, DirectOp<BM, BK, NW>>::type;
  using OpB = typename std::conditional<BT, TransOp<BN, BK, NW>, DirectOp<BN, BK, NW>>::type;
  static constexpr int STAGE = OpA::BYTES + OpB::BYTES;   // (BM + BN) * BK * 2 bytes
};

// Orders one wavefront's LDS accesses: what its other lanes wrote before is visible after (LDS
// instructions of a wavefront execute in order; this keeps the compiler from reordering them).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// s_waitcnt immediates (gfx9 encoding): at most n vector-memory operations outstanding, with or
// without also waiting for every LDS operation
constexpr int wait_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
constexpr int wait_vm_lds(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070; }

// NS stages of BK k each form a ring: while k-tile t is multiplied, tiles t+1 .. t+NS-1 are in LDS
// or on their way.
template <int BM, int BN, bool AT, bool BT, int BK, int NS, int NW>
__global__ void __launch_bounds__(64 * NW) gemm_kernel(const GemmArgs g) {
  using T = Tile<BM, BN, AT, BT, BK, NW>;
  using OpA = typename T::OpA;
  using OpB = typename T::OpB;
  static_assert(NS >= 2 && NS <= 4, "two to four stages");
  // separate arrays, so that the compiler can tell that fragment reads of one stage do not depend
  // on the loads in flight into the others
  __shared__ __align__(1024) unsigned char stage0[T::STAGE];
  __shared__ __align__(1024) unsigned char stage1[T::STAGE];
  __shared__ __align__(1024) unsigned char stage2[NS > 2 ? T::STAGE : 16];
  __shared__ __align__(1024) unsigned char stage3[NS > 3 ? T::STAGE : 16];
  constexpr int WGN = NW / 2;  // the waves form a 2 x WGN grid over the block tile
  constexpr int WM = BM / 2, WN = BN / WGN, TM = WM / 32, TN = WN / 32, KS = BK / 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // Work-group -> (k-split, tile).  Consecutive work-group ids go round-robin over the XCDs; undo
  // that so each XCD (own L2) gets a contiguous run of tiles of as few k-splits as possible: the
  // tiles of one split read the same k-range of A and B and share those panels in L2.
  int pid, split;
  {
    const int nt = g.tiles_m * g.tiles_n, total = nt * (int)gridDim.y;
    const int lin = (int)blockIdx.x + (int)blockIdx.y * nt, xcd = lin % g.xcds, idx = lin / g.xcds;
    const int base = total / g.xcds, rem = total % g.xcds;
    const int at = xcd * base + (xcd < rem ? xcd : rem) + idx;
    split = at / nt;
    pid = at - split * nt;
  }
  // Grouped order: group_m tile rows are swept column by column, so the work-groups an XCD runs at a
  // time form a patch of tiles and each A / B panel they stream is shared by several of them in L2.
  int tm, tn;
  {
    const int per_group = g.group_m * g.tiles_n;
    const int first = (pid / per_group) * g.group_m;
    const int rows = min(g.tiles_m - first, g.group_m);
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
  const int rows_a = min(g.M - m0, BM), rows_b = min(g.N - n0, BN);
  opa.init(g.lda, rows_a, tid);
  opb.init(g.ldb, rows_b, tid);
  const typename OpA::Frag fa = OpA::frag_init(wm * WM, lane);
  const typename OpB::Frag fb = OpB::frag_init(wn * WN, lane);

  const int k_base = g.partial ? split * g.k_chunk : 0;
  const int k_end = g.partial ? min(g.K, k_base + g.k_chunk) : g.K;
  auto request = [&](unsigned char* stage, int k0) {  // asynchronous: tile k0 streams into `stage`
    const int kleft = k_end - k0;
    opa.load(make_rsrc(OpA::origin(g.A, g.lda, m0, k0), OpA::extent(rows_a, g.lda, kleft)), stage, kleft);
    opb.load(make_rsrc(OpB::origin(g.B, g.ldb, n0, k0), OpB::extent(rows_b, g.ldb, kleft)), stage + OpA::BYTES, kleft);
    __builtin_amdgcn_sched_barrier(0);  // keep the requests ahead of the products they overlap with
  };
  constexpr int kPerTile = OpA::NV + OpB::NV;  // vector-memory instructions of one request, per wave
  half8_t af[2][TM], bf[2][TN];  // fragments of two consecutive k-steps
  auto fetch = [&](const unsigned char* stage, int s, int set) {
#pragma unroll
    for (int i = 0; i < TM; ++i) af[set][i] = OpA::frag(stage, fa, i, s);
#pragma unroll
    for (int j = 0; j < TN; ++j) bf[set][j] = OpB::frag(stage + OpA::BYTES, fb, j, s);
  };
  auto multiply = [&](int set) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)  // B first: the result tile is transposed, lane = row of C, registers = columns
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[set][j], af[set][i], acc[i][j], 0, 0, 0);
  };
  auto interleave = [&]() { Interleave<0, TM * TN, OpA::READS * TM + OpB::READS * TN>::run(); };
  // One k-tile.  On entry the fragments of k-step 0 of `cur` are in registers and the next NS-1
  // tiles have been requested.  Before the last k-step every wave holds its last fragments of `cur`
  // in registers and has seen its own part of `nxt` land (the requests of the NS-2 tiles behind it
  // may still be in flight); the barrier then publishes `nxt` and frees `cur`, which is refilled at
  // once with the tile NS ahead.
  auto k_tile = [&](unsigned char* cur, const unsigned char* nxt, int k_refill) {
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s == KS - 1) {
        __builtin_amdgcn_s_waitcnt(wait_vm_lds((NS - 2) * kPerTile));
        __builtin_amdgcn_s_barrier();
        request(cur, k_refill);
      }
      fetch(s == KS - 1 ? nxt : cur, (s + 1) % KS, (s + 1) & 1);
      multiply(s & 1);
      interleave();
    }
  };

  // A k-tile past the end reads zeros (it lies outside the extent of its buffer descriptor) and
  // multiplying it changes nothing, so the loop always runs whole rings and carries no edge conditions.
  const int nk = (k_end - k_base + BK - 1) / BK;
  request(stage0, k_base);
  request(stage1, k_base + BK);
  if constexpr (NS >= 3) request(stage2, k_base + 2 * BK);
  if constexpr (NS == 4) request(stage3, k_base + 3 * BK);
  __builtin_amdgcn_s_waitcnt(wait_vm((NS - 1) * kPerTile));
  __builtin_amdgcn_s_barrier();
  fetch(stage0, 0, 0);
  if constexpr (NS == 2) {
    for (int kt = 0; kt < nk; kt += 2) {
      k_tile(stage0, stage1, k_base + (kt + 2) * BK);
      k_tile(stage1, stage0, k_base + (kt + 3) * BK);
    }
  } else if constexpr (NS == 3) {
    for (int kt = 0; kt < nk; kt += 3) {
      k_tile(stage0, stage1, k_base + (kt + 3) * BK);
      k_tile(stage1, stage2, k_base + (kt + 4) * BK);
      k_tile(stage2, stage0, k_base + (kt + 5) * BK);
    }
  } else {
    for (int kt = 0; kt < nk; kt += 4) {
      k_tile(stage0, stage1, k_base + (kt + 4) * BK);
      k_tile(stage1, stage2, k_base + (kt + 5) * BK);
      k_tile(stage2, stage3, k_base + (kt + 6) * BK);
      k_tile(stage3, stage0, k_base + (kt + 7) * BK);
    }
  }
  __builtin_amdgcn_s_waitcnt(wait_vm_lds(0));  // the last refills (all zeros) must land before the stages are reused
  __syncthreads();

  // ---- epilogue: accumulators -> per-wave LDS staging (fp32) -> row-wise 16-byte stores -------
  // The products were formed as (B tile) x (A tile)^T, so in the MFMA result layout lane l holds row
  // l%32 of the C tile and, in registers 4q..4q+3, the four consecutive columns 8q + 4(l/32) .. +3:
  // one 16-byte LDS write per register quad.  A staged row is SW floats; its 16-byte chunks are
  // XOR-swizzled with the row so that 16 lanes (16 rows, same logical chunk) hit every bank once.
  // staging width per pass: the wave's whole width if NW waves x 32 rows of it fit one stage, else less
  // (half of the waves stage in stage0, the other half in stage1, so that a staged row can be 64 columns
  //  = whole 128-byte lines of fp16 output even when a stage is small)
  constexpr int HW = NW / 2;
  constexpr int SW = (HW * 32 * WN * 4 <= T::STAGE) ? WN : (HW * 32 * 64 * 4 <= T::STAGE && WN % 64 == 0) ? 64 : 32;
  static_assert(HW * 32 * SW * 4 <= T::STAGE, "epilogue staging does not fit");
  float* stg = reinterpret_cast<float*>(wave < HW ? stage0 : stage1) + (wave % HW) * (32 * SW);
  constexpr int CH = SW / 8;    // 8-column chunks per staged row
  constexpr int QC = SW / 4;    // 16-byte chunks per staged row (8, 16 or 32)
  auto swz = [](int row, int chunk) { return QC >= 16 ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7)); };
  const GemmEpilogue& ep = g.ep;
  // The addend (or the ReLU mask source) of the wave's whole share is requested up front, into registers
  // the fragments no longer need, so that its latency is paid once and behind the staging of the first rows
  // rather than once per 32 rows.  (Reading it all before any store is also what lets it alias C.)
  constexpr int kPre = TM * (WN / SW) * (CH / 2);
  constexpr bool PRELOAD = kPre <= 16;
  const half_t* pre_src = ep.add ? ep.add : ep.relu_src;
  half8_t pre[PRELOAD ? kPre : 1];
  if constexpr (PRELOAD) {
    if (pre_src && !g.partial) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jg = 0; jg < WN / SW; ++jg)
#pragma unroll
          for (int it = 0; it < CH / 2; ++it) {
            const int q = it * 64 + lane;
            const int gr = m0 + wm * WM + i * 32 + q / CH, gc = n0 + wn * WN + jg * SW + (q % CH) * 8;
            pre[(i * (WN / SW) + jg) * (CH / 2) + it] = (gr < g.M && gc < g.N) ? ld_half8(pre_src + (size_t)gr * g.ldc + gc) : zero_half8();
          }
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int jg = 0; jg < WN / SW; ++jg) {
      if (i || jg) wave_sync();  // the staging area is the wave's own: no work-group barrier needed
#pragma unroll
      for (int jj = 0; jj < SW / 32; ++jj)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const floatx16& a = acc[i][jg * (SW / 32) + jj];
          const floatx4 v4 = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
          const int row = lane & 31, chunk = jj * 8 + 2 * q + (lane >> 5);
          *reinterpret_cast<floatx4*>(stg + row * SW + swz(row, chunk) * 4) = v4;
        }
      wave_sync();
#pragma unroll
      for (int it = 0; it < CH / 2; ++it) {
        const int q = it * 64 + lane;
        const int rl = q / CH, c8 = q % CH;
        const int gr = m0 + wm * WM + i * 32 + rl, gc = n0 + wn * WN + jg * SW + c8 * 8;
        if (gr < g.M && gc < g.N) {
          float v[8];
          const floatx4 lo = *reinterpret_cast<const floatx4*>(stg + rl * SW + swz(rl, 2 * c8) * 4);
          const floatx4 hi = *reinterpret_cast<const floatx4*>(stg + rl * SW + swz(rl, 2 * c8 + 1) * 4);
          if (g.partial) {
            float* dst = g.partial + ((size_t)split * g.M + gr) * g.N + gc;
            *reinterpret_cast<floatx4*>(dst) = lo;
            *reinterpret_cast<floatx4*>(dst + 4) = hi;
            continue;
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = lo[e] * ep.out_scale;
            v[4 + e] = hi[e] * ep.out_scale;
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
            const uint32_t bits = drop_keep8(ep.drop, (uint32_t)(gr + ep.row0), (uint32_t)gc >> 3);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = ((bits >> e) & 1u) ? v[e] * ep.drop.scale : 0.f;
          }
          const size_t off = (size_t)gr * g.ldc + gc;
          if (ep.add) {
            half8_t a;
            if constexpr (PRELOAD) a = pre[(i * (WN / SW) + jg) * (CH / 2) + it];
            else a = ld_half8(ep.add + off);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += (float)a[e];
          }
          if (ep.relu_src) {
            half8_t h;
            if (PRELOAD && !ep.add) h = pre[(i * (WN / SW) + jg) * (CH / 2) + it];
            else h = ld_half8(ep.relu_src + off);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = ((float)h[e] > 0.f) ? v[e] * ep.mask_scale : 0.f;
          }
          half8_t o;
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (half_t)v[e];
          // streaming store: a result tile is not read again by this product, and letting it stay in L2 pushes out
          // the operand panels the XCD's other tiles are reading (products with wide results: +5-7 %)
          __builtin_nontemporal_store(o, reinterpret_cast<half8_t*>(g.C + off));
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Persistent form of the 256 x 256, 8-wave kernel for products whose epilogue loads nothing per
// element (bias, ReLU and the output scale only): one work-group per compute unit walks its tiles
// (the same tile -> XCD assignment as above) and asks for the first k-tiles of its next tile -- the
// whole stage ring -- BEFORE it stores the current one, so that their latency passes behind the
// epilogue and the next main loop starts with its ring full.  Vector-memory operations retire in
// issue order on one counter: the wait for the first of those k-tiles is "at most as many operations
// outstanding as were issued after it" (the other requests and the epilogue's stores), which does not
// wait for the stores.  The epilogue leaves the stages alone: bias, ReLU and scale are applied to the
// accumulators where they are (MFMA layout), the fp16 results pass through the 32 KB of LDS the stage
// ring leaves free (32 rows x 64 columns per wave, wave-private, so no work-group barrier) and leave
// as whole 128-byte rows.
// ------------------------------------------------------------------------------------------------
// LDS accesses of the staging rows, written as instructions: while requests into the stages are in
// flight the compiler would otherwise put a wait for ALL of them in front of any LDS access it
// cannot tell apart from their targets.
__device__ __forceinline__ uint32_t lds_addr(const void* p) { return (uint32_t)(uintptr_t)(lds_void_ptr)p; }
typedef _Float16 half4v_t __attribute__((ext_vector_type(4)));
// eight 8-byte writes: one 32 x 64 slab of results (the lane's four consecutive columns of each of its eight column groups)
__device__ __forceinline__ void out_write_slab(const uint32_t (&a)[8], const half4v_t (&v)[8]) {
  asm volatile(
      "ds_write_b64 %0, %8\n\tds_write_b64 %1, %9\n\tds_write_b64 %2, %10\n\tds_write_b64 %3, %11\n\t"
      "ds_write_b64 %4, %12\n\tds_write_b64 %5, %13\n\tds_write_b64 %6, %14\n\tds_write_b64 %7, %15"
      :
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]), "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]),
        "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7])
      : "memory");
}
// the slab back as rows: four 16-byte reads, returned once all have arrived (LDS operations of a wave complete in
// order, so the writes above are done too); one instruction sequence, so that nothing touches the registers between
// the reads and the wait
__device__ __forceinline__ void out_read_slab(const uint32_t (&a)[4], half8_t (&d)[4]) {
  asm volatile(
      "ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(d[0]), "=&v"(d[1]), "=&v"(d[2]), "=&v"(d[3])
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3])
      : "memory");
}

template <bool AT, bool BT, int BK, int NS>
__global__ void __launch_bounds__(512) gemm_persistent_kernel(const GemmArgs g) {
  constexpr int BM = 256, BN = 256, NW = 8;
  using T = Tile<BM, BN, AT, BT, BK, NW>;
  using OpA = typename T::OpA;
  using OpB = typename T::OpB;
  static_assert(NS == 2 || NS == 4, "two or four stages");
  static_assert(NS * T::STAGE == 128 * 1024, "the ring takes 128 KB; the staging rows take the 32 KB that are left");
  // separate arrays (see gemm_kernel); the third and fourth exist only in the four-stage form
  __shared__ __align__(1024) unsigned char stage0[T::STAGE];
  __shared__ __align__(1024) unsigned char stage1[T::STAGE];
  unsigned char *stage2 = nullptr, *stage3 = nullptr;
  if constexpr (NS == 4) {
    __shared__ __align__(1024) unsigned char stage2_[T::STAGE];
    __shared__ __align__(1024) unsigned char stage3_[T::STAGE];
    stage2 = stage2_;
    stage3 = stage3_;
  }
  constexpr int WGN = 4, WM = 128, WN = 64, TM = 4, TN = 2, KS = BK / 16;
  constexpr int kOutPitch = WN * 2;                       // bytes per staged row: 64 fp16
  __shared__ __align__(16) unsigned char out_rows[NW * 32 * kOutPitch];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int nt = g.tiles_m * g.tiles_n;

  auto decode = [&](int lin, int& m0, int& n0) {
    const int xcd = lin % g.xcds, idx = lin / g.xcds, base = nt / g.xcds, rem = nt % g.xcds;
    const int pid = xcd * base + (xcd < rem ? xcd : rem) + idx;
    const int per_group = g.group_m * g.tiles_n;
    const int first = (pid / per_group) * g.group_m;
    const int rows = min(g.tiles_m - first, g.group_m);
    m0 = (first + (pid % per_group) % rows) * BM;
    n0 = ((pid % per_group) / rows) * BN;
  };

  OpA opa;
  OpB opb;
  int m0, n0, rows_a, rows_b;  // the tile the operand descriptors are set up for
  // Per-lane offsets are recomputed where they are needed rather than kept in registers across the
  // epilogue (the register file is full there); the empty asm keeps the compiler from merging the copies.
  auto setup = [&]() {
    int t = tid;
    asm volatile("" : "+v"(t));
    rows_a = min(g.M - m0, BM);
    rows_b = min(g.N - n0, BN);
    opa.init(g.lda, rows_a, t);
    opb.init(g.ldb, rows_b, t);
  };
  typename OpA::Frag fa;
  typename OpB::Frag fb;
  auto frag_setup = [&]() {
    int l = lane;
    asm volatile("" : "+v"(l));
    fa = OpA::frag_init(wm * WM, l);
    fb = OpB::frag_init(wn * WN, l);
  };
  auto request = [&](unsigned char* stage, int k0) {
    const int kleft = g.K - k0;
    opa.load(make_rsrc(OpA::origin(g.A, g.lda, m0, k0), OpA::extent(rows_a, g.lda, kleft)), stage, kleft);
    opb.load(make_rsrc(OpB::origin(g.B, g.ldb, n0, k0), OpB::extent(rows_b, g.ldb, kleft)), stage + OpA::BYTES, kleft);
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr int kPerTile = OpA::NV + OpB::NV;
  floatx16 acc[TM][TN];
  half8_t af[2][TM], bf[2][TN];
  auto fetch = [&](const unsigned char* stage, int s, int set) {
#pragma unroll
    for (int i = 0; i < TM; ++i) af[set][i] = OpA::frag(stage, fa, i, s);
#pragma unroll
    for (int j = 0; j < TN; ++j) bf[set][j] = OpB::frag(stage + OpA::BYTES, fb, j, s);
  };
  auto multiply = [&](int set) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[set][j], af[set][i], acc[i][j], 0, 0, 0);
  };
  auto interleave = [&]() { Interleave<0, TM * TN, OpA::READS * TM + OpB::READS * TN>::run(); };
  auto k_tile = [&](unsigned char* cur, const unsigned char* nxt, int k_refill) {
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s == KS - 1) {
        __builtin_amdgcn_s_waitcnt(wait_vm_lds((NS - 2) * kPerTile));
        __builtin_amdgcn_s_barrier();
        request(cur, k_refill);
      }
      fetch(s == KS - 1 ? nxt : cur, (s + 1) % KS, (s + 1) & 1);
      multiply(s & 1);
      interleave();
    }
  };
  const int nk = (g.K + BK - 1) / BK;
  const GemmEpilogue& ep = g.ep;
  // staged rows of this wave: row r, 16-byte chunk c (eight columns) at r * pitch + (c ^ (r & 7)) * 16, so that the
  // eight lanes that read a row back cover its 128 bytes and sixteen lanes cover every bank once
  const uint32_t out = lds_addr(out_rows) + wave * (32 * kOutPitch);
  constexpr int kStores = TM * 4;  // global stores of one wave's epilogue on a tile that lies wholly inside C

  int lin = blockIdx.x;
  decode(lin, m0, n0);
  setup();
  request(stage0, 0);
  request(stage1, BK);
  if constexpr (NS == 4) {
    request(stage2, 2 * BK);
    request(stage3, 3 * BK);
  }
  __builtin_amdgcn_s_waitcnt(wait_vm((NS - 1) * kPerTile));
  __builtin_amdgcn_s_barrier();
  frag_setup();
  fetch(stage0, 0, 0);
  for (;;) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    if constexpr (NS == 2) {
      for (int kt = 0; kt < nk; kt += 2) {
        k_tile(stage0, stage1, (kt + 2) * BK);
        k_tile(stage1, stage0, (kt + 3) * BK);
      }
    } else {
      for (int kt = 0; kt < nk; kt += 4) {
        k_tile(stage0, stage1, (kt + 4) * BK);
        k_tile(stage1, stage2, (kt + 5) * BK);
        k_tile(stage2, stage3, (kt + 6) * BK);
        k_tile(stage3, stage0, (kt + 7) * BK);
      }
    }
    // What the epilogue needs of the current tile.  The bias of the lane's columns in the MFMA layout (column group
    // cg = 4 jj + q holds columns 32 jj + 8 q + 4 (lane / 32) .. + 3 of the wave's 64) is fetched here, ahead of the
    // requests below, and waited for together with the last refills (zeros past k), so that no wait of the epilogue
    // has to pass those requests.
    const int m0c = m0, n0c = n0;
    const int g32 = lane >> 5, row = lane & 31;
    const int col0 = n0c + wn * WN + 4 * g32;
    half4v_t bias4[8];
#pragma unroll
    for (int cg = 0; cg < 8; ++cg) {
      const int col = col0 + 8 * cg;   // (N is a multiple of 8 and col of 4: the four columns are inside C or all outside)
      bias4[cg] = half4v_t{0, 0, 0, 0};
      if (ep.bias && col < g.N) bias4[cg] = *reinterpret_cast<const half4v_t*>(ep.bias + col);
    }
    __builtin_amdgcn_s_waitcnt(wait_vm_lds(0));
    __syncthreads();
    const int next = lin + (int)gridDim.x;
    const bool more = next < nt;
    if (more) {
      decode(next, m0, n0);
      setup();
      request(stage0, 0);
      request(stage1, BK);
      if constexpr (NS == 4) {
        request(stage2, 2 * BK);
        request(stage3, 3 * BK);
      }
    }
    // ---- epilogue of (m0c, n0c): accumulators -> fp16 -> the wave's staging rows -> 16-byte pieces of whole rows ----
    const int c8 = lane & 7;
    const int gc = n0c + wn * WN + c8 * 8;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      uint32_t wa[8];
      half4v_t wv[8];
#pragma unroll
      for (int cg = 0; cg < 8; ++cg) {
        const floatx16& a = acc[i][cg >> 2];
        const int q = cg & 3;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float v = a[4 * q + e] * ep.out_scale + (float)bias4[cg][e];
          if (ep.relu) v = fmaxf(v, 0.f);
          wv[cg][e] = (_Float16)v;
        }
        wa[cg] = out + row * kOutPitch + ((cg ^ (row & 7)) << 4) + (g32 << 3);
      }
      out_write_slab(wa, wv);   // (the reads of the previous slab have returned: out_read_slab waits for them)
      uint32_t ra[4];
      half8_t rv[4];
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int rl = it * 8 + (lane >> 3);
        ra[it] = out + rl * kOutPitch + ((c8 ^ (rl & 7)) << 4);
      }
      out_read_slab(ra, rv);
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int gr = m0c + wm * WM + i * 32 + it * 8 + (lane >> 3);
        // streaming store: a result tile is not read again by this product, and letting it stay in L2 pushes out
        // the operand panels the XCD's other tiles are reading (products with wide results: +5-7 %)
        if (gr < g.M && gc < g.N) __builtin_nontemporal_store(rv[it], reinterpret_cast<half8_t*>(g.C + (size_t)gr * g.ldc + gc));
      }
    }
    if (!more) break;
    // wait for the first k-tile of the new tile: everything issued after it may stay outstanding (the other early
    // requests and the stores of a full tile); a tile at the edge of C stores fewer rows or columns, so there the
    // wait is for everything
    const bool whole = m0c + BM <= g.M && n0c + BN <= g.N;
    constexpr int kLater = (NS - 1) * kPerTile + kStores;
    static_assert(kLater < 64, "s_waitcnt vmcnt holds six bits");
    if (whole) __builtin_amdgcn_s_waitcnt(wait_vm(kLater));
    else __builtin_amdgcn_s_waitcnt(wait_vm(0));
    __builtin_amdgcn_s_barrier();
    frag_setup();
    fetch(stage0, 0, 0);
    lin = next;
  }
}

// C[m, n] = fp16(sum_z partial[z][m][n]), 8 columns per thread, splits summed in increasing order
__global__ void __launch_bounds__(kThreads) splitk_reduce_kernel(const float* __restrict__ partial, int splits, int M, int N,
                                                                half_t* __restrict__ C, int ldc, float scale) {
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int chunks = N >> 3;
  if (gid >= (int64_t)M * chunks) return;
  const int row = (int)(gid / chunks), c8 = (int)(gid % chunks);
  const size_t off = (size_t)row * N + c8 * 8, plane = (size_t)M * N;
  floatx4 lo = *reinterpret_cast<const floatx4*>(partial + off), hi = *reinterpret_cast<const floatx4*>(partial + off + 4);
  for (int z = 1; z < splits; ++z) {
    lo += *reinterpret_cast<const floatx4*>(partial + z * plane + off);
    hi += *reinterpret_cast<const floatx4*>(partial + z * plane + off + 4);
  }
  half8_t o;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    o[e] = (half_t)(lo[e] * scale);
    o[4 + e] = (half_t)(hi[e] * scale);
  }
  st_half8(C + (size_t)row * ldc + c8 * 8, o);
}

template <int BM, int BN, bool AT, bool BT, int BK, int NS, int NW>
int launch_variant(const GemmArgs& g, int splits, hipStream_t stream) {
  hipLaunchKernelGGL((gemm_kernel<BM, BN, AT, BT, BK, NS, NW>), dim3(g.tiles_m * g.tiles_n, splits), dim3(64 * NW), 0, stream, g);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

template <int BM, int BN, int BK, int NS, int NW = 4>
int launch_tile(const GemmArgs& a, bool a_t, bool b_t, int splits, hipStream_t stream) {
  GemmArgs g = a;
  g.tiles_m = ceil_div(g.M, BM);
  g.tiles_n = ceil_div(g.N, BN);
  // tile rows per sweep: the 32 tiles an XCD works on at a time form a patch of 4 rows x 8 columns (or
  // the result's whole width); between 2 and 8 the whole update is flat within 0.5 %, 4 measured best and
  // fetches least past L2, 12 and more cost 2 %
  g.group_m = tuning().gemm_group;
  g.xcds = device_info().xcds;
  if (splits > 1) {
    static_assert(64 % BK == 0, "the k range of a split is a multiple of 64 whatever the tile, so that the tile shape changes no bit");
    g.k_chunk = (int)round_up(ceil_div(g.K, splits), 64);
    splits = ceil_div(g.K, g.k_chunk);  // no empty split
  }
  if (splits <= 1) {
    g.partial = nullptr;
    splits = 1;
  }
  int rc;
  if (!a_t && !b_t) rc = launch_variant<BM, BN, false, false, BK, NS, NW>(g, splits, stream);
  else if (!a_t && b_t) rc = launch_variant<BM, BN, false, true, BK, NS, NW>(g, splits, stream);
  else if (a_t && b_t) rc = launch_variant<BM, BN, true, true, BK, NS, NW>(g, splits, stream);
  else rc = launch_variant<BM, BN, true, false, BK, NS, NW>(g, splits, stream);
  if (rc != NMT_OK || splits == 1) return rc;
  const int64_t n = (int64_t)g.M * (g.N / 8);
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3(ceil_div(n, kThreads)), dim3(kThreads), 0, stream, g.partial, splits, g.M, g.N, g.C, g.ldc, g.ep.out_scale);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

// Estimated efficiency of a tile shape on a (M, N) problem: useful fraction of the padded tiles,
// times how well the tile count fills whole rounds of the compute units, times a per-shape factor (small
// tiles re-read LDS more often per MFMA).
double tile_score(int M, int N, int bm, int bn, int per_cu, double shape_eff) {
  const double tiles = (double)ceil_div(M, bm) * ceil_div(N, bn);
  const double useful = ((double)M * N) / (tiles * bm * bn);
  const double slots = (double)device_info().cus * per_cu;
  const double rounds = (tiles + slots - 1) / slots;
  const double fill = tiles / (double)((int64_t)rounds * slots);
  return useful * fill * shape_eff;
}

}  // namespace

namespace {
int launch_gemm_impl(const half_t* A, bool a_t, int lda, const half_t* B, bool b_t, int ldb, half_t* C, int ldc, int M,
                     int N, int K, const GemmEpilogue& ep, hipStream_t stream, float* partial, int64_t partial_floats, int splits) {
  NMT_REQUIRE(M > 0 && N > 0 && K > 0, "gemm: empty problem M=%d N=%d K=%d", M, N, K);
  NMT_REQUIRE(A && B && C, "gemm: null operand");
  NMT_REQUIRE(aligned16(A) && aligned16(B) && aligned16(C), "gemm: operands must be 16-byte aligned");
  NMT_REQUIRE(lda % 8 == 0 && ldb % 8 == 0 && ldc % 8 == 0 && N % 8 == 0, "gemm: lda/ldb/ldc/N must be multiples of 8");
  NMT_REQUIRE((a_t ? M : K) % 8 == 0 && (b_t ? N : K) % 8 == 0, "gemm: contiguous operand dimension must be a multiple of 8");
  NMT_REQUIRE(lda >= (a_t ? M : K) && ldb >= (b_t ? N : K) && ldc >= N, "gemm: leading dimension too small");
  NMT_REQUIRE(lda <= (1 << 20) && ldb <= (1 << 20) && ldc <= (1 << 20), "gemm: leading dimensions above 2^20 are not supported");
  NMT_REQUIRE(!ep.bias || aligned16(ep.bias), "gemm: bias must be 16-byte aligned");
  NMT_REQUIRE((!ep.add || aligned16(ep.add)) && (!ep.relu_src || aligned16(ep.relu_src)), "gemm: epilogue operand misaligned");
  NMT_REQUIRE(splits >= 0 && splits <= 64, "gemm: number of k splits %d outside [0, 64]", splits);
  const bool plain = !ep.bias && !ep.relu && !ep.drop.thr && !ep.add && !ep.relu_src;  // (out_scale is applied by the reduction)
  NMT_REQUIRE(splits <= 1 || (partial && plain), "gemm: splitting k needs a partial-sum buffer and no epilogue");
  NMT_REQUIRE(!partial || (reinterpret_cast<uintptr_t>(partial) & 15u) == 0, "gemm: partial-sum buffer must be 16-byte aligned");
  GemmArgs g{A, B, C, lda, ldb, ldc, M, N, K, 0, 0, 0, device_info().xcds, ep, partial, 0};
  const int cus = device_info().cus;
  const int64_t plane = (int64_t)M * N;
  // Work-groups of 256 x 256 tiles run one per compute unit; they pay off once there are enough of them.
  const int64_t t256 = (int64_t)ceil_div(M, 256) * ceil_div(N, 256);
  const int64_t full = 3 * (int64_t)cus / 4;  // large tiles from three quarters of a round on
  if (splits == 0) {  // choose: a short, wide problem (a weight gradient over many positions) is cut along k
    splits = 1;
    if (partial && plain && t256 < full) {
      int64_t want = (cus + t256 / 2) / t256;                   // large tiles: one work-group per compute unit
      want = want < K / 2048 ? want : K / 2048;                 // at least 2048 k per split
      want = want < partial_floats / plane ? want : partial_floats / plane;
      want = want < 64 ? want : 64;
      if (want >= 2) {
        splits = (int)want;
      } else {
        // a contraction too short for that (the weight gradient of a single sub-batch): 128 x 128 tiles, two
        // work-groups per compute unit, at least 512 k per split
        const int64_t t128 = (int64_t)ceil_div(M, 128) * ceil_div(N, 128);
        want = 2 * cus / t128;
        want = want < K / 512 ? want : K / 512;
        want = want < partial_floats / plane ? want : partial_floats / plane;
        want = want < 64 ? want : 64;
        if (want >= 2) splits = (int)want;
      }
    }
  }
  NMT_REQUIRE(splits == 1 || plane * splits <= partial_floats, "gemm: partial-sum buffer of %lld floats too small for %d splits",
              (long long)partial_floats, splits);
  if (const int forced = tuning().gemm_tile; forced && splits <= 1) {
    switch (forced) {
      case 1: return (!a_t && !b_t) ? launch_tile<256, 256, 64, 2, 8>(g, a_t, b_t, 1, stream) : launch_tile<256, 256, 32, 4, 8>(g, a_t, b_t, 1, stream);
      case 2: return launch_tile<128, 128, 64, 2>(g, a_t, b_t, 1, stream);
      case 3: return launch_tile<128, 64, 64, 2>(g, a_t, b_t, 1, stream);
      case 4: return launch_tile<64, 128, 64, 2>(g, a_t, b_t, 1, stream);
      default: return launch_tile<64, 64, 64, 2>(g, a_t, b_t, 1, stream);
    }
  }
  // (a caller that keeps several passes in flight says so: each product then counts on its share of the chip)
  const int64_t full_shared = full / tuning().gemm_share > 1 ? full / tuning().gemm_share : 1;
  if (t256 * splits >= full_shared) {
    // A last, partly filled round of 256 x 256 tiles leaves compute units idle for a whole tile's
    // time.  If that round is small, the rows it would cover are given to a second launch with small
    // tiles (two work-groups per compute unit), which costs about a third of a round.
    const int tiles_n = ceil_div(N, 256), rounds = (int)(t256 / cus);
    if (splits == 1 && rounds >= 1 && t256 % cus != 0) {
      const int main_tm = cus * rounds / tiles_n, m_main = main_tm * 256, m_tail = M - m_main;
      const int64_t tail128 = (int64_t)ceil_div(m_tail, 128) * ceil_div(N, 128);
      const double cost_split = ceil_div((int64_t)main_tm * tiles_n, cus) + 0.3 * ceil_div(tail128, 2 * cus);
      if (main_tm >= 1 && cost_split + 0.25 <= rounds + 1) {
        int rc = launch_gemm_impl(A, a_t, lda, B, b_t, ldb, C, ldc, m_main, N, K, ep, stream, nullptr, 0, 1);
        if (rc != NMT_OK) return rc;
        GemmEpilogue tail = ep;
        tail.row0 = ep.row0 + m_main;
        if (tail.add) tail.add += (size_t)m_main * ldc;
        if (tail.relu_src) tail.relu_src += (size_t)m_main * ldc;
        return launch_gemm_impl(a_t ? A + m_main : A + (size_t)m_main * lda, a_t, lda, B, b_t, ldb, C + (size_t)m_main * ldc, ldc, m_tail, N,
                                K, tail, stream, nullptr, 0, 1);
      }
    }
    // At least two tiles per compute unit, no split along k, row-major A, an epilogue that loads nothing per
    // element (bias, ReLU, scale): the persistent form.  (With an addend or a mask to load it gained 1-11 % on a
    // product running alone but nothing on the update, where the weight-gradient kernels of the second stream
    // share the chip and work-groups that never leave their compute unit cost more than they gain; the form no
    // longer has those epilogues.  Not for a k-major A either: the one such product without a split, the
    // vocabulary weight gradient, has so long a contraction that the tile change hardly counts, and measured
    // 6 % slower in this form.)
    const bool loads_in_epilogue = ep.add || ep.relu_src || ep.drop.thr;
    if (splits == 1 && t256 >= 2 * cus && !a_t && tuning().gemm_persist && !loads_in_epilogue) {
      GemmArgs pg = g;
      pg.tiles_m = ceil_div(M, 256);
      pg.tiles_n = ceil_div(N, 256);
      pg.group_m = tuning().gemm_group;
      pg.partial = nullptr;
      if (!b_t) hipLaunchKernelGGL((gemm_persistent_kernel<false, false, 64, 2>), dim3(cus), dim3(512), 0, stream, pg);
      else hipLaunchKernelGGL((gemm_persistent_kernel<false, true, 32, 4>), dim3(cus), dim3(512), 0, stream, pg);
      NMT_LAUNCH_CHECK();
      return NMT_OK;
    }
    // k-contiguous operands are fetched in whole 128-byte lines by 64-deep stages; transposed ones
    // gain more from the longer look-ahead of four 32-deep stages
    if (!a_t && !b_t) return launch_tile<256, 256, 64, 2, 8>(g, a_t, b_t, splits, stream);
    return launch_tile<256, 256, 32, 4, 8>(g, a_t, b_t, splits, stream);
  }
  if (splits > 1) return launch_tile<128, 128, 64, 2>(g, a_t, b_t, splits, stream);
  const double s128 = tile_score(M, N, 128, 128, 2, 1.0);
  const double s12864 = tile_score(M, N, 128, 64, 2, 0.85);
  const double s64128 = tile_score(M, N, 64, 128, 2, 0.85);
  const double s64 = tile_score(M, N, 64, 64, 4, 0.65);
  if (s128 >= s12864 && s128 >= s64128 && s128 >= s64) return launch_tile<128, 128, 64, 2>(g, a_t, b_t, 1, stream);
  if (s12864 >= s64128 && s12864 >= s64) return launch_tile<128, 64, 64, 2>(g, a_t, b_t, 1, stream);
  if (s64128 >= s64) return launch_tile<64, 128, 64, 2>(g, a_t, b_t, 1, stream);
  return launch_tile<64, 64, 64, 2>(g, a_t, b_t, 1, stream);
}

// Optional timing of every product with HIP events on the stream it is launched on (the benchmark's roofline leg):
// pairs of events from a pool that grows as needed and is read and reset by gemm_timing_read.
struct TimedProduct {
  hipEvent_t start, stop;
  double flops;
};
std::vector<TimedProduct> g_timed;
size_t g_timed_used = 0;
std::mutex g_timed_mutex;
}  // namespace

int launch_gemm(const half_t* A, bool a_t, int lda, const half_t* B, bool b_t, int ldb, half_t* C, int ldc, int M,
                int N, int K, const GemmEpilogue& ep, hipStream_t stream, float* partial, int64_t partial_floats, int splits) {
  if (!tuning().gemm_timing) return launch_gemm_impl(A, a_t, lda, B, b_t, ldb, C, ldc, M, N, K, ep, stream, partial, partial_floats, splits);
  TimedProduct t;
  {
    std::lock_guard<std::mutex> lock(g_timed_mutex);
    if (g_timed_used == g_timed.size()) {
      TimedProduct fresh = {};
      NMT_HIP_CHECK(hipEventCreate(&fresh.start));
      NMT_HIP_CHECK(hipEventCreate(&fresh.stop));
      g_timed.push_back(fresh);
    }
    g_timed[g_timed_used].flops = 2.0 * M * N * K;
    t = g_timed[g_timed_used++];
  }
  NMT_HIP_CHECK(hipEventRecord(t.start, stream));
  const int rc = launch_gemm_impl(A, a_t, lda, B, b_t, ldb, C, ldc, M, N, K, ep, stream, partial, partial_floats, splits);
  NMT_HIP_CHECK(hipEventRecord(t.stop, stream));
  return rc;
}

int gemm_timing_read(double* ms, int64_t* products, double* flops) {
  std::lock_guard<std::mutex> lock(g_timed_mutex);
  double total = 0.0, fl = 0.0;
  for (size_t i = 0; i < g_timed_used; ++i) {
    float one = 0.f;
    NMT_HIP_CHECK(hipEventSynchronize(g_timed[i].stop));
    NMT_HIP_CHECK(hipEventElapsedTime(&one, g_timed[i].start, g_timed[i].stop));
    total += one;
    fl += g_timed[i].flops;
  }
  if (ms) *ms = total;
  if (products) *products = (int64_t)g_timed_used;
  if (flops) *flops = fl;
  g_timed_used = 0;
  return NMT_OK;
}
