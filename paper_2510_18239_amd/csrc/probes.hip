// Achievable-peak probes for the benchmark: what this machine sustains for a plain streaming copy and for a
// register-resident loop of the matrix instruction every contraction here uses.  Roofline fractions are quoted
// against the published peaks; these two say how much of those a kernel can reach at all.
#include "../../include/lime.h"
#include "mfma.hpp"

namespace lime {
namespace {

// 16 bytes per lane and access, grid-stride, four accesses in flight per lane.
__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a, dst[i + stride] = b, dst[i + 2 * stride] = c, dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

constexpr int kMfmaChains = 4;  // independent accumulators per wave: the instruction's latency is covered
// Every wave issues iters * kMfmaChains v_mfma_f32_32x32x16_bf16 on operands that never leave registers.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int t = 0; t < 8; ++t) a[t] = static_cast<__bf16>(0.001f * (threadIdx.x % 7 + t)), b[t] = static_cast<__bf16>(0.002f * t);
  f32x16 acc[kMfmaChains];
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c) acc[c] = mfma32(a, b, acc[c]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  out[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

constexpr int kMfmaBlocksPerUnit = 2;  // 256 threads = one wave per SIMD; two blocks per unit keep every SIMD fed

}  // namespace
}  // namespace lime

extern "C" {
#pragma GCC visibility push(default)

int32_t lime_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) % 16 != 0)
    return LIME_INVALID_ARG;
  const size_t n16 = bytes / 16;
  const size_t want = (n16 + 255) / 256;
  const size_t cap = static_cast<size_t>(lime::compute_units()) * 8;
  lime::launch_timed(lime::kKernelProbeCopy, lime::probe_copy_kernel, dim3(static_cast<unsigned>(want < cap ? want : cap)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
  return hipGetLastError() == hipSuccess ? LIME_OK : LIME_LAUNCH_FAILED;
}

size_t lime_probe_mfma_out_bytes(void) {
  return static_cast<size_t>(lime::compute_units()) * lime::kMfmaBlocksPerUnit * 256 * sizeof(float);
}

double lime_probe_mfma(void* out, int32_t iters, void* stream) {
  if (!out || iters <= 0) return 0.0;
  const int blocks = lime::compute_units() * lime::kMfmaBlocksPerUnit;
  lime::launch_timed(lime::kKernelProbeMfma, lime::probe_mfma_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<float*>(out), iters);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return 2.0 * 32 * 32 * 16 * lime::kMfmaChains * static_cast<double>(iters) * 4 * blocks;
}

#pragma GCC visibility pop
}
