// Measurement aids: the two denominators a roofline is quoted against, measured on the machine at hand
// (Section 6.1 reports against vendor libraries; here the bounds are the chip's own copy rate and MFMA issue
// rate).  A plain copy kernel of known size also calibrates the profiler's byte counters.
#include <hip/hip_fp16.h>

#include "spc_internal.h"

namespace spc {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// Every wave keeps four independent 32x32x16 fp16 MFMA chains going from registers: nothing but matrix
// instructions in the loop, so the time per iteration is the issue rate of the matrix pipe.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* __restrict__ out) {
  probe_half8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = static_cast<_Float16>(0.001f * (threadIdx.x + i));
    b[i] = static_cast<_Float16>(0.002f * (threadIdx.x - i));
  }
  probe_floatx16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 123456.789f) out[0] = s;  // keeps the chains alive
}

}  // namespace spc

extern "C" int spc_probe_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  using namespace spc;
  if (!src || !dst || bytes < 16 || bytes % 16) return set_error(SPC_ERR_ARG, "NULL pointer or size not a multiple of 16");
  hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), bytes / 16);
  SPC_HIP_CHECK(hipGetLastError());
  return SPC_OK;
}

extern "C" int spc_probe_mfma(int32_t iters, float* sink, double* flops, void* stream) {
  using namespace spc;
  if (iters < 1 || !sink) return set_error(SPC_ERR_ARG, "iters < 1 or sink NULL");
  const int n_wg = 256 * 2;  // two workgroups of four waves per compute unit
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(n_wg), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
  SPC_HIP_CHECK(hipGetLastError());
  if (flops) *flops = double(n_wg) * 4 /*waves*/ * iters * 4 /*chains*/ * (2.0 * 32 * 32 * 16);
  return SPC_OK;
}
