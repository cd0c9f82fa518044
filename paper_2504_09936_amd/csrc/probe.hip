// Measurement probes: what this GPU actually sustains, next to the published peaks that the
// roofline fractions are quoted against.  keepkv_probe_read streams a buffer with the same
// coalesced 16-byte-per-lane loads the kernels use; keepkv_probe_mfma issues back-to-back
// 32x32x16 bf16 MFMAs on independent accumulators.  Neither is part of the method.
#include "kk_common.hpp"

namespace kk {
namespace {

// every workgroup reads a contiguous share, a wavefront 1 KB per instruction, kDepth instructions in flight
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, size_t n_vec, float* sink) {
  constexpr int kDepth = 8;
  const size_t per_wg = (n_vec + gridDim.x - 1) / gridDim.x;
  const size_t begin = blockIdx.x * per_wg;
  const size_t end = begin + per_wg < n_vec ? begin + per_wg : n_vec;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t i = begin + threadIdx.x; i < end; i += 256 * kDepth) {
    uint4 r[kDepth];
#pragma unroll
    for (int u = 0; u < kDepth; ++u) {
      const size_t j = i + (size_t)u * 256;
      r[u] = src[j < end ? j : end - 1];
    }
#pragma unroll
    for (int u = 0; u < kDepth; ++u) {
      acc.x ^= r[u].x; acc.y ^= r[u].y; acc.z ^= r[u].z; acc.w ^= r[u].w;
    }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) *sink = 1.f;   // keeps the loads alive; practically never true
}

__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* sink) {
  const uint32_t t = threadIdx.x;
  const bf16x8_t a = __builtin_bit_cast(bf16x8_t, make_uint4(0x3f803f80u + (t & 1), 0x3f803f80u, 0x3f803f80u, 0x3f803f80u));
  const bf16x8_t b = __builtin_bit_cast(bf16x8_t, make_uint4(0x3f803f80u, 0x3f803f80u + (t & 2), 0x3f803f80u, 0x3f803f80u));
  f32x16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == -1.f) *sink = s;                                          // sums of positive products: never true
}

}  // namespace
}  // namespace kk

extern "C" keepkv_status keepkv_probe_read(const void* src, size_t bytes, int32_t n_workgroups, float* sink,
                                           void* stream) {
  using namespace kk;
  if (!src || !sink || bytes < 16 || (bytes & 15) || !aligned16(src) || n_workgroups < 1 || n_workgroups > (1 << 20))
    return KEEPKV_ERR_INVALID_ARG;
  probe_read_kernel<<<n_workgroups, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(
      reinterpret_cast<const uint4*>(src), bytes / 16, sink);
  return launch_status();
}

extern "C" keepkv_status keepkv_probe_mfma(int32_t n_workgroups, int32_t iters, float* sink, double* flops,
                                           void* stream) {
  using namespace kk;
  if (!sink || n_workgroups < 1 || n_workgroups > (1 << 20) || iters < 1) return KEEPKV_ERR_INVALID_ARG;
  if (flops) *flops = (double)n_workgroups * 4.0 * iters * 4.0 * (2.0 * 32 * 32 * 16);
  probe_mfma_kernel<<<n_workgroups, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(iters, sink);
  return launch_status();
}
