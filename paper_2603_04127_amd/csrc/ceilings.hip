// Measured ceilings of the device the library runs on: three plain kernels whose achieved rates a benchmark
// reports next to the attention kernels' own (the published peaks assume clocks that a loaded chip does not
// hold).  No part of the attention path.
//   copy: 16 bytes per lane in, 16 bytes out, grid-stride  -> HBM read + write rate
//   read: 16 bytes per lane in, summed                      -> HBM read rate
//   mfma: independent chains of v_mfma_f32_32x32x16_f16     -> dense fp16 MFMA rate
#include "common.h"

namespace dark {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void k_ceiling_copy(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(256) void k_ceiling_read(const u32x4* __restrict__ src, size_t n, unsigned* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned acc = 0u;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;  // keeps the loads alive; practically never taken
}

// Four independent accumulators per wave: an MFMA of one chain issues while the previous ones of the other
// chains are still in the pipeline.  Two waves per SIMD.
__global__ __launch_bounds__(512) void k_ceiling_mfma(int iters, float* __restrict__ sink) {
  half8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (_Float16)(0.001f * (float)(threadIdx.x % 7));
    b[i] = (_Float16)(0.002f * (float)(threadIdx.x % 5));
  }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 12345.678f) sink[0] = s;
}

constexpr int kCeilingBlocks = 256 * 8;  // eight workgroups per compute unit

}  // namespace
}  // namespace dark

using namespace dark;

extern "C" dark_status dark_ceiling_copy(void* dst, const void* src, size_t nbytes, void* hip_stream) {
  if (dst == nullptr || src == nullptr || nbytes % 16 != 0) return DARK_EINVAL;
  if (nbytes == 0) return DARK_OK;
  hipLaunchKernelGGL(k_ceiling_copy, dim3(kCeilingBlocks), dim3(256), 0, (hipStream_t)hip_stream, (u32x4*)dst,
                     (const u32x4*)src, nbytes / 16);
  return hipGetLastError() == hipSuccess ? DARK_OK : DARK_EHIP;
}

extern "C" dark_status dark_ceiling_read(const void* src, size_t nbytes, void* sink, void* hip_stream) {
  if (src == nullptr || sink == nullptr || nbytes % 16 != 0) return DARK_EINVAL;
  if (nbytes == 0) return DARK_OK;
  hipLaunchKernelGGL(k_ceiling_read, dim3(kCeilingBlocks), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4*)src,
                     nbytes / 16, (unsigned*)sink);
  return hipGetLastError() == hipSuccess ? DARK_OK : DARK_EHIP;
}

extern "C" dark_status dark_ceiling_mfma(int iters, void* sink, double* flops, void* hip_stream) {
  if (iters < 0 || sink == nullptr || flops == nullptr) return DARK_EINVAL;
  const int blocks = 256;  // one workgroup of eight waves per compute unit
  *flops = (double)blocks * 8.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
  hipLaunchKernelGGL(k_ceiling_mfma, dim3(blocks), dim3(512), 0, (hipStream_t)hip_stream, iters, (float*)sink);
  return hipGetLastError() == hipSuccess ? DARK_OK : DARK_EHIP;
}
