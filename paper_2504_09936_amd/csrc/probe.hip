// Measurement probes: what this GPU actually sustains, next to the published peaks that the
// roofline fractions are quoted against.  keepkv_probe_read streams a buffer with the same
// coalesced 16-byte-per-lane loads the kernels use; keepkv_probe_mfma issues back-to-back
// 32x32x16 bf16 MFMAs on independent accumulators, with uniform or with random operand values.
// Neither is part of the method.
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

// RANDOM: four operand pairs of pseudo-random bf16 values (random sign and mantissa, magnitudes 0.25 .. 4)
// that alternate, so that the multiplier inputs toggle as they do on real data; otherwise both operands
// are (nearly) all ones.  The sustained clock, and with it the rate, depends on this.
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* sink) {
  const uint32_t t = threadIdx.x;
  bf16x8_t a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t wa[4], wb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (RANDOM) {
        uint32_t h = (t * 16u + j * 4u + i + 1u) * 0x9E3779B9u;
        h ^= h >> 15; h *= 0x85EBCA6Bu; h ^= h >> 13;
        uint32_t g = h * 0xC2B2AE35u; g ^= g >> 16;
        // per 16-bit half: sign and 7 mantissa bits from the hash, exponent 125 .. 128
        wa[i] = (h & 0x807F807Fu) | ((125u + ((h >> 7) & 3u)) << 7) | ((125u + ((h >> 23) & 3u)) << 23);
        wb[i] = (g & 0x807F807Fu) | ((125u + ((g >> 7) & 3u)) << 7) | ((125u + ((g >> 23) & 3u)) << 23);
      } else {
        wa[i] = 0x3f803f80u + ((i == 0) ? (t & 1) : 0);
        wb[i] = 0x3f803f80u + ((i == 1) ? (t & 2) : 0);
      }
    }
    a[j] = __builtin_bit_cast(bf16x8_t, make_uint4(wa[0], wa[1], wa[2], wa[3]));
    b[j] = __builtin_bit_cast(bf16x8_t, make_uint4(wb[0], wb[1], wb[2], wb[3]));
  }
  f32x16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[2], c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3], b[3], c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == -1.2345e-30f) *sink = s;                                  // keeps the products alive; practically never true
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

extern "C" keepkv_status keepkv_probe_mfma(int32_t n_workgroups, int32_t iters, int32_t random_operands, float* sink,
                                           double* flops, void* stream) {
  using namespace kk;
  if (!sink || n_workgroups < 1 || n_workgroups > (1 << 20) || iters < 1) return KEEPKV_ERR_INVALID_ARG;
  if (flops) *flops = (double)n_workgroups * 4.0 * iters * 4.0 * (2.0 * 32 * 32 * 16);
  if (random_operands) probe_mfma_kernel<true><<<n_workgroups, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(iters, sink);
  else probe_mfma_kernel<false><<<n_workgroups, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(iters, sink);
  return launch_status();
}
