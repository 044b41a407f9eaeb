// Calibration kernels: the bf16 matrix-core rate and the read-only HBM stream rate this chip
// sustains, for putting the roofline fractions in context.  Not part of the method.
//
// A loop of independent v_mfma_f32_32x32x16_bf16 on register operands, 2 workgroups of 4 waves
// per compute unit.  With `random_operands` the eight A and eight B fragments hold pseudo-random
// values and rotate from one instruction to the next (operand bits toggle as they do in real
// work); without, every fragment holds the same constant.  The difference between the two rates
// is the chip's power management, not the instruction stream.
#include <hip/hip_runtime.h>

#include "common.hpp"

namespace basa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kCalibGrid = 512, kCalibThreads = 256, kMfmaPerIter = 32;

__device__ inline uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

template <bool kRandom>
__global__ __launch_bounds__(kCalibThreads) void calib_mfma_kernel(float* out, int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int f = 0; f < 8; ++f)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (kRandom) {
        const uint32_t h1 = mix(threadIdx.x * 131u + f * 17u + i), h2 = mix(h1 + 977u);
        a[f][i] = (__bf16)(((int)(h1 & 0xffff) - 32768) / 16384.0f);
        b[f][i] = (__bf16)(((int)(h2 & 0xffff) - 32768) / 16384.0f);
      } else {
        a[f][i] = (__bf16)1.0f;
        b[f][i] = (__bf16)0.5f;
      }
    }
  floatx16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[(u + 1) & 7], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 3) & 7], b[u], c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 5) & 7], b[(u + 2) & 7], c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 6) & 7], b[(u + 7) & 7], c3, 0, 0, 0);
    }
    if ((it & 63) == 63) {   // keep the accumulators bounded
#pragma unroll
      for (int i = 0; i < 16; ++i) { c0[i] *= 0.001f; c1[i] *= 0.001f; c2[i] *= 0.001f; c3[i] *= 0.001f; }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  out[blockIdx.x * kCalibThreads + threadIdx.x] = s;
}

// Read-only stream over a buffer: 256 workgroups per launch wave, 8 x 16 bytes in flight per thread,
// streaming loads as in the selection passes (6.8 TB/s on this part; cached loads reach 6.3).
__global__ __launch_bounds__(256) void calib_read_kernel(const uint4* __restrict__ in, size_t n, uint32_t* out) {
  constexpr int kUnroll = 8;
  size_t i = ((size_t)blockIdx.x * kUnroll) * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256 * kUnroll;
  uint32_t acc = 0;
  for (; i + (kUnroll - 1) * 256 < n; i += stride) {
    uint4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
      v[u] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in + i + u * 256)));
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) out[0] = acc;     // keeps the loads alive; practically never taken
}

}  // namespace

hipError_t launch_calib_read(const void* buf, size_t bytes, uint32_t* out, hipStream_t stream) {
  hipLaunchKernelGGL(calib_read_kernel, dim3(4096), dim3(256), 0, stream, reinterpret_cast<const uint4*>(buf),
                     bytes / 16, out);
  return hipGetLastError();
}

size_t calib_mfma_out_elems() { return (size_t)kCalibGrid * kCalibThreads; }

double calib_mfma_flops(int iters) {
  return (double)kCalibGrid * (kCalibThreads / 64) * (double)iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
}

hipError_t launch_calib_mfma(bool random_operands, int iters, float* out, hipStream_t stream) {
  if (random_operands)
    hipLaunchKernelGGL(calib_mfma_kernel<true>, dim3(kCalibGrid), dim3(kCalibThreads), 0, stream, out, iters);
  else
    hipLaunchKernelGGL(calib_mfma_kernel<false>, dim3(kCalibGrid), dim3(kCalibThreads), 0, stream, out, iters);
  return hipGetLastError();
}

}  // namespace basa
