// HBM-bound update kernels: fp32 gradient accumulation, single-pass unscale + inf/NaN detection,
// Adam on fp32 master weights with fp16 weight refresh.  All are grid-stride loops over 16-byte
// (or wider) vectors so that each wavefront issues fully coalesced accesses.
#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 256 * 8;  // 8 work-groups per CU keeps enough loads in flight

// acc (+)= mult * float(g16); mult undoes the power-of-two factor a pass applied before rounding to fp16
__global__ void __launch_bounds__(kThreads) accumulate_kernel(const half_t* __restrict__ g16, float* __restrict__ acc, int64_t n,
                                                              int first, float mult) {
  const int64_t nvec = n >> 3;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
    const half8_t g = ld_half8(g16 + i * 8);
    floatx4* a = reinterpret_cast<floatx4*>(acc + i * 8);
    floatx4 lo, hi;
    if (first) {
      lo = floatx4{0, 0, 0, 0};
      hi = lo;
    } else {
      lo = a[0];
      hi = a[1];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      lo[e] += mult * (float)g[e];
      hi[e] += mult * (float)g[4 + e];
    }
    a[0] = lo;
    a[1] = hi;
  }
  // tail (n not a multiple of 8)
  for (int64_t i = (nvec << 3) + (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
    acc[i] = (first ? 0.f : acc[i]) + mult * (float)g16[i];
}

__global__ void set_flag_kernel(int32_t* flag, int32_t v) { *flag = v; }
__global__ void add_scalars_kernel(const float* loss, const int32_t* ntok, float* loss_total, int32_t* ntok_total, int first) {
  *loss_total = (first ? 0.f : *loss_total) + *loss;
  *ntok_total = (first ? 0 : *ntok_total) + *ntok;
}

__device__ __forceinline__ bool non_finite(float x) { return (__float_as_uint(x) & 0x7F800000u) == 0x7F800000u; }

// IN_PLACE: acc *= inv_scale in the same pass; otherwise the buffer is only read (the caller applies the factor later)
template <bool IN_PLACE>
__global__ void __launch_bounds__(kThreads) check_overflow_kernel(float* __restrict__ acc, int64_t n, float inv_scale,
                                                                  int32_t* __restrict__ flag) {
  const int64_t nvec = n >> 2;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  bool bad = false;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
    floatx4 v = ld_float4_nt(acc + i * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      bad |= non_finite(v[e]);
      v[e] *= inv_scale;
    }
    if (IN_PLACE) st_float4_nt(acc + i * 4, v);
  }
  for (int64_t i = (nvec << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    bad |= non_finite(acc[i]);
    if (IN_PLACE) acc[i] *= inv_scale;
  }
  if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(flag, 1);
}

__global__ void __launch_bounds__(kThreads) adam_kernel(float* __restrict__ master, float* __restrict__ m, float* __restrict__ v,
                                                        const float* __restrict__ g, half_t* __restrict__ w16, int64_t n, float lr,
                                                        float b1, float b2, float eps, float inv_bc1, float inv_bc2, float gscale,
                                                        const int32_t* __restrict__ flag) {
  if (flag && *flag != 0) return;  // overflow: skip the update, every buffer stays bit-identical
  const int64_t nvec = n >> 2;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
    floatx4 w = reinterpret_cast<floatx4*>(master)[i];
    floatx4 mm = reinterpret_cast<floatx4*>(m)[i];
    floatx4 vv = reinterpret_cast<floatx4*>(v)[i];
    const floatx4 gg = reinterpret_cast<const floatx4*>(g)[i] * gscale;   // the gradient in its original scale
    half4_t h;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      mm[e] = b1 * mm[e] + (1.f - b1) * gg[e];
      vv[e] = b2 * vv[e] + (1.f - b2) * gg[e] * gg[e];
      w[e] -= lr * (mm[e] * inv_bc1) / (sqrtf(vv[e] * inv_bc2) + eps);
      h[e] = (half_t)w[e];
    }
    reinterpret_cast<floatx4*>(master)[i] = w;
    reinterpret_cast<floatx4*>(m)[i] = mm;
    reinterpret_cast<floatx4*>(v)[i] = vv;
    *reinterpret_cast<half4_t*>(w16 + i * 4) = h;
  }
  for (int64_t i = (nvec << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    const float gg = g[i] * gscale;
    const float mm = b1 * m[i] + (1.f - b1) * gg;
    const float vv = b2 * v[i] + (1.f - b2) * gg * gg;
    const float w = master[i] - lr * (mm * inv_bc1) / (sqrtf(vv * inv_bc2) + eps);
    m[i] = mm;
    v[i] = vv;
    master[i] = w;
    w16[i] = (half_t)w;
  }
}

int grid_for(int64_t nvec) {
  int64_t b = (nvec + kThreads - 1) / kThreads;
  return (int)(b < 1 ? 1 : (b > kMaxBlocks ? kMaxBlocks : b));
}

}  // namespace

int launch_accumulate(const half_t* g16, float* acc, int64_t n, int first, hipStream_t stream, float mult) {
  NMT_REQUIRE(g16 && acc && n > 0, "accumulate: bad arguments");
  NMT_REQUIRE(aligned16(g16) && aligned16(acc), "accumulate: buffers must be 16-byte aligned");
  hipLaunchKernelGGL(accumulate_kernel, dim3(grid_for(n >> 3)), dim3(kThreads), 0, stream, g16, acc, n, first, mult);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_add_scalars(const float* loss, const int32_t* ntok, float* loss_total, int32_t* ntok_total, int first, hipStream_t stream) {
  hipLaunchKernelGGL(add_scalars_kernel, dim3(1), dim3(1), 0, stream, loss, ntok, loss_total, ntok_total, first);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_check_overflow(float* acc, int64_t n, float inv_scale, int32_t* flag, hipStream_t stream, bool in_place) {
  NMT_REQUIRE(acc && flag && n > 0, "check_overflow: bad arguments");
  NMT_REQUIRE(aligned16(acc), "check_overflow: buffer must be 16-byte aligned");
  hipLaunchKernelGGL(set_flag_kernel, dim3(1), dim3(1), 0, stream, flag, 0);
  NMT_LAUNCH_CHECK();
  if (in_place) hipLaunchKernelGGL(check_overflow_kernel<true>, dim3(grid_for(n >> 2)), dim3(kThreads), 0, stream, acc, n, inv_scale, flag);
  else hipLaunchKernelGGL(check_overflow_kernel<false>, dim3(grid_for(n >> 2)), dim3(kThreads), 0, stream, acc, n, 1.f, flag);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}

int launch_adam(float* master, float* m, float* v, const float* g, half_t* w16, int64_t n, float lr, float b1, float b2,
                float eps, int t, const int32_t* flag, hipStream_t stream, float grad_scale) {
  NMT_REQUIRE(master && m && v && g && w16 && n > 0 && t >= 1, "adam: bad arguments");
  NMT_REQUIRE(aligned16(master) && aligned16(m) && aligned16(v) && aligned16(g) && aligned16(w16), "adam: buffers must be 16-byte aligned");
  const double bc1 = 1.0 - pow((double)b1, (double)t), bc2 = 1.0 - pow((double)b2, (double)t);
  hipLaunchKernelGGL(adam_kernel, dim3(grid_for(n >> 2)), dim3(kThreads), 0, stream, master, m, v, g, w16, n, lr, b1, b2, eps,
                     (float)(1.0 / bc1), (float)(1.0 / bc2), grad_scale, flag);
  NMT_LAUNCH_CHECK();
  return NMT_OK;
}
