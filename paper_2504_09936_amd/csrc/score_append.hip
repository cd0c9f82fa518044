// keepkv_score (Eq. 8 EMA update in the log domain) and keepkv_append (cache update of Sec. 3.1,
// votes initialised to 1 as in Sec. 3.3.1).  Both are element-wise and bandwidth-trivial.
#include "kk_common.hpp"

namespace kk {
namespace {

// log_s <- ln(alpha * S + (1 - alpha) * exp(logit)) on slots < len[unit]; the head's step counter t_obs += 1, which
// is one more observation for every slot (a slot's count is t_obs - born)
__global__ __launch_bounds__(256) void score_kernel(float* __restrict__ log_s, int32_t* __restrict__ t_obs,
                                                    const float* __restrict__ logits, const int32_t* __restrict__ len,
                                                    int capacity, float ln_alpha, float ln_1m_alpha) {
  const int unit = blockIdx.y;
  const int n = len[unit];
  const size_t base = (size_t)unit * capacity;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const float a = ln_alpha + log_s[base + i];      // -inf when alpha == 0 or nothing observed
    const float b = ln_1m_alpha + logits[base + i];
    const float hi = fmaxf(a, b), lo = fminf(a, b);
    // ln(e^hi + e^lo) = hi + log1p(e^(lo - hi)); lo = -inf gives hi
    const float r = (lo == -INFINITY) ? hi : hi + log1pf(expf(lo - hi));
    log_s[base + i] = r;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) t_obs[unit] += 1;
}

template <typename T>
__global__ __launch_bounds__(128) void append_kernel(T* __restrict__ k, T* __restrict__ v, int32_t* __restrict__ votes,
                                                     float* __restrict__ log_s, int32_t* __restrict__ born,
                                                     const int32_t* __restrict__ t_obs, int32_t* __restrict__ len, const T* __restrict__ k_t,
                                                     const T* __restrict__ v_t, int32_t* overflow, int capacity, int D) {
  const int unit = blockIdx.x;
  const int i = len[unit];
  if (i >= capacity) {
    if (threadIdx.x == 0 && overflow != nullptr) *overflow = 1;
    return;
  }
  const size_t row = ((size_t)unit * capacity + i) * D;
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    k[row + d] = k_t[(size_t)unit * D + d];
    v[row + d] = v_t[(size_t)unit * D + d];
  }
  __syncthreads();   // every thread has read len[unit] before it is bumped
  if (threadIdx.x == 0) {
    votes[(size_t)unit * capacity + i] = 1;
    log_s[(size_t)unit * capacity + i] = -INFINITY;
    born[(size_t)unit * capacity + i] = t_obs[unit];       // no observation yet
    len[unit] = i + 1;
  }
}

}  // namespace
}  // namespace kk

extern "C" keepkv_status keepkv_score(const keepkv_layout* layout, keepkv_cache* cache, const float* logits,
                                      float alpha, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !logits) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (!(alpha >= 0.f && alpha < 1.f)) return KEEPKV_ERR_INVALID_ARG;
  const int units = layout->batch * layout->n_kv_heads;
  int bx = (cache->capacity + 255) / 256;
  if (bx > 64) bx = 64;
  const float la = alpha > 0.f ? logf(alpha) : -INFINITY;
  score_kernel<<<dim3(bx, units), 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(
      cache->log_s, cache->t_obs, logits, cache->len, cache->capacity, la, log1pf(-alpha));
  return launch_status();
}

extern "C" keepkv_status keepkv_append(const keepkv_layout* layout, keepkv_cache* cache, const void* k_t,
                                       const void* v_t, int32_t* overflow, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !k_t || !v_t) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (layout->head_dim < 1) return KEEPKV_ERR_INVALID_ARG;
  const int units = layout->batch * layout->n_kv_heads;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (layout->dtype == KEEPKV_BF16)
    append_kernel<uint16_t><<<units, 128, 0, st>>>((uint16_t*)cache->k, (uint16_t*)cache->v, cache->votes, cache->log_s,
                                                   cache->born, cache->t_obs, cache->len, (const uint16_t*)k_t, (const uint16_t*)v_t,
                                                   overflow, cache->capacity, layout->head_dim);
  else
    append_kernel<float><<<units, 128, 0, st>>>((float*)cache->k, (float*)cache->v, cache->votes, cache->log_s,
                                                cache->born, cache->t_obs, cache->len, (const float*)k_t, (const float*)v_t, overflow,
                                                cache->capacity, layout->head_dim);
  return launch_status();
}
