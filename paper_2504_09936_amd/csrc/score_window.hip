// keepkv_score_window: the EMA scores of Eq. 8 from a window of W queries in one pass over the keys
// (the t = L branch written as its sum; on an already observed cache it equals W consecutive
// keepkv_score updates).
//
// bf16 caches: the W*G query rows of one kv head against its keys is a dense contraction, done with
// 32x32x16 bf16 MFMA.  A workgroup of four wavefronts streams 128-key stages through LDS
// (global -> LDS without passing through registers, double buffered, rows XOR-swizzled so that the
// operand reads are free of bank conflicts); each wavefront owns 32 keys of a stage and keeps all
// query rows resident in registers as the A operand.  Rows are assigned to MFMA rows such that the
// 16 accumulators of a lane are 16 consecutive query rows (whole query groups), so the group mean,
// the weights (1 - alpha) alpha^(W-1-j) and the running log-sum stay inside the lane; the two lane
// halves of a key are joined once at the end.  The keys are read once: the pass is HBM-bound.
// f32 caches take a plain one-thread-per-key kernel.
#include "kk_common.hpp"

namespace kk {
namespace {

constexpr int kWinWaves = 4;
constexpr int kWinStageSlots = 128;
constexpr int kWinMaxRows = 128;           // W * G query rows held in registers

struct WinParams {
  const void* k;
  const void* q;             // [B, Hq, W, D]
  float* log_s;
  int32_t* n_obs;
  const int32_t* len;
  int capacity, W, G, n_q_heads, n_kv_heads, first_pos, slots_per_wg;
  float ln_alpha, ln_1m_alpha, scale_over_g;
};

// ln of the weight of query j's score in the window sum: ln((1 - alpha) alpha^(W-1-j))
__device__ __forceinline__ float win_coef(int j, int W, float ln_alpha, float ln_1m_alpha) {
  const float d = (float)(W - 1 - j);
  return ln_1m_alpha + (d > 0.f ? d * ln_alpha : 0.f);
}

// queries that see `slot`: j >= slot - first_pos (all of them when first_pos < 0)
__device__ __forceinline__ int win_first_query(int slot, int first_pos) {
  return first_pos < 0 ? 0 : max(0, slot - first_pos);
}

// fold (m2, s2) into the running (m, s) of sum = s * e^m
__device__ __forceinline__ void lse_join(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  const float ms = (mn == -INFINITY) ? 0.f : mn;
  s = s * expf(m - ms) + s2 * expf(m2 - ms);
  m = mn;
}

// log_s <- ln(alpha^n_vis S + e^m s), n_obs += n_vis
__device__ __forceinline__ void win_store(float* log_s, int32_t* n_obs, size_t at, int n_vis, float m, float s,
                                          float ln_alpha) {
  if (n_vis <= 0) return;
  const float fresh = m + logf(s);                       // s > 0: at least the last query contributes
  const float old = log_s[at] + (float)n_vis * ln_alpha; // -inf when alpha == 0 or nothing observed
  const float hi = fmaxf(old, fresh), lo = fminf(old, fresh);
  log_s[at] = (lo == -INFINITY) ? hi : hi + log1pf(expf(lo - hi));
  n_obs[at] += n_vis;
}

template <int D, int G>
__global__ __launch_bounds__(kWinWaves* kWave, 2) void score_window_mfma_kernel(WinParams p) {
  constexpr int ROWB = D * 2, CHUNKS = ROWB / 16, KS = D / 16;
  constexpr int STAGE_BYTES = kWinStageSlots * ROWB;
  constexpr int LOADS = kWinStageSlots * CHUNKS / (kWinWaves * kWave);
  constexpr int NT = kWinMaxRows / 32;
  constexpr int QPL = 16 / G;                // window queries per lane and tile
  extern __shared__ __align__(16) unsigned char s_stage[];   // 2 stages

  const int unit = blockIdx.y;
  const int n = p.len[unit];
  const int slot_begin = blockIdx.x * p.slots_per_wg;
  if (slot_begin >= n) return;               // uniform over the workgroup
  const int slot_end = min(n, slot_begin + p.slots_per_wg);
  const int n_stage = (slot_end - slot_begin + kWinStageSlots - 1) / kWinStageSlots;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const unsigned char* kbytes = reinterpret_cast<const unsigned char*>(p.k) + (size_t)unit * p.capacity * ROWB;

  auto issue_stage = [&](int s) {
    unsigned char* dst = s_stage + (s & 1) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int c = tid + i * (kWinWaves * kWave);
      const int col_l = c / CHUNKS, phys = c % CHUNKS;
      const int slot = min(slot_begin + s * kWinStageSlots + col_l, n - 1);
      const unsigned char* src = kbytes + (size_t)slot * ROWB + ((phys ^ (col_l & (CHUNKS - 1))) * 16);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(dst + (wave * 64 + i * (kWinWaves * kWave)) * 16),
                                       16, 0, 0);
    }
  };
  issue_stage(0);

  // ---- A operands: query row rho = j * G + g sits on MFMA row m such that accumulator i of lane
  // half h is row rho = 32 t + 16 h + i
  const int R = p.W * G;
  const int b = unit / p.n_kv_heads, kvh = unit % p.n_kv_heads;
  bf16x8_t a[NT][KS];
  {
    const int hm = (l32 >> 2) & 1, im = ((l32 >> 3) << 2) | (l32 & 3);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int rho = t * 32 + hm * 16 + im;
      const bool live = rho < R;
      const int j = live ? rho / G : 0, g = live ? rho % G : 0;
      const unsigned char* row = reinterpret_cast<const unsigned char*>(p.q) +
                                 (((size_t)b * p.n_q_heads + kvh * G + g) * p.W + j) * ROWB;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 x = *reinterpret_cast<const uint4*>(row + ks * 32 + half * 16);
        if (!live) x = make_uint4(0, 0, 0, 0);
        a[t][ks] = __builtin_bit_cast(bf16x8_t, x);
      }
    }
  }
  const int n_tile = (R + 31) / 32;

  for (int s = 0; s < n_stage; ++s) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                         // stage s has landed; everyone is done with stage s - 1
    if (s + 1 < n_stage) issue_stage(s + 1);
    const unsigned char* src = s_stage + (s & 1) * STAGE_BYTES;
    bf16x8_t bk[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      bk[ks] = *reinterpret_cast<const bf16x8_t*>(src + (wave * 32 + l32) * ROWB +
                                                  (((ks * 2 + half) ^ (l32 & (CHUNKS - 1))) * 16));
    const int slot = slot_begin + s * kWinStageSlots + wave * 32 + l32;
    const int j_first = win_first_query(slot, p.first_pos);
    float m = -INFINITY, sum = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < n_tile) {                      // uniform
        f32x16_t acc = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t][ks], bk[ks], acc, 0, 0, 0);
        float y[QPL];
        float ymax = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < QPL; ++jj) {
          float x = 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g) x += acc[jj * G + g];
          const int j = (t * 32 + half * 16) / G + jj;
          const bool vis = j < p.W && j >= j_first;
          y[jj] = vis ? x * p.scale_over_g + win_coef(j, p.W, p.ln_alpha, p.ln_1m_alpha) : -INFINITY;
          ymax = fmaxf(ymax, y[jj]);
        }
        const float mn = fmaxf(m, ymax);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        float add = 0.f;
#pragma unroll
        for (int jj = 0; jj < QPL; ++jj) add += expf(y[jj] - ms);
        sum = sum * expf(m - ms) + add;
        m = mn;
      }
    }
    lse_join(m, sum, __shfl_xor(m, 32), __shfl_xor(sum, 32));
    if (half == 0 && slot < slot_end)
      win_store(p.log_s, p.n_obs, (size_t)unit * p.capacity + slot, p.W - min(p.W, j_first), m, sum, p.ln_alpha);
  }
}

// f32 storage: one thread per key, the key row in registers, the query rows broadcast from LDS.
template <int D>
__global__ __launch_bounds__(128) void score_window_f32_kernel(WinParams p) {
  extern __shared__ __align__(16) unsigned char s_raw[];
  float* s_q = reinterpret_cast<float*>(s_raw);          // [R][D], row rho = j * G + g
  const int unit = blockIdx.y;
  const int n = p.len[unit];
  const int G = p.G, R = p.W * G;
  const int b = unit / p.n_kv_heads, kvh = unit % p.n_kv_heads;
  if ((int)(blockIdx.x * blockDim.x) >= n) return;
  const float* q = reinterpret_cast<const float*>(p.q);
  for (int e = threadIdx.x; e < R * D; e += blockDim.x) {
    const int rho = e / D, c = e % D, j = rho / G, g = rho % G;
    s_q[e] = q[(((size_t)b * p.n_q_heads + kvh * G + g) * p.W + j) * D + c];
  }
  __syncthreads();
  const int slot = blockIdx.x * blockDim.x + threadIdx.x;
  if (slot >= n) return;
  const float* krow = reinterpret_cast<const float*>(p.k) + ((size_t)unit * p.capacity + slot) * D;
  float kr[D];
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    const float4 x = *reinterpret_cast<const float4*>(krow + c);
    kr[c] = x.x, kr[c + 1] = x.y, kr[c + 2] = x.z, kr[c + 3] = x.w;
  }
  const int j_first = win_first_query(slot, p.first_pos);
  float m = -INFINITY, sum = 0.f;
  for (int j = j_first; j < p.W; ++j) {
    float x = 0.f;
    for (int g = 0; g < G; ++g) {
      const float* qr = s_q + (j * G + g) * D;
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) dot = fmaf(qr[c], kr[c], dot);
      x += dot;
    }
    lse_join(m, sum, x * p.scale_over_g + win_coef(j, p.W, p.ln_alpha, p.ln_1m_alpha), 1.f);
  }
  win_store(p.log_s, p.n_obs, (size_t)unit * p.capacity + slot, p.W - min(p.W, j_first), m, sum, p.ln_alpha);
}

template <int D>
void launch_mfma(const WinParams& p, dim3 grid, hipStream_t st) {
  const size_t smem = 2 * (size_t)kWinStageSlots * D * 2;
  switch (p.G) {
    case 1: score_window_mfma_kernel<D, 1><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
    case 2: score_window_mfma_kernel<D, 2><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
    case 4: score_window_mfma_kernel<D, 4><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
    default: score_window_mfma_kernel<D, 8><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
  }
}

}  // namespace
}  // namespace kk

extern "C" keepkv_status keepkv_score_window(const keepkv_layout* layout, keepkv_cache* cache, const void* q_win,
                                             int32_t window, float alpha, int32_t first_pos, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !q_win || !aligned16(q_win)) return KEEPKV_ERR_INVALID_ARG;
  if (!(alpha >= 0.f && alpha < 1.f) || window < 1) return KEEPKV_ERR_INVALID_ARG;
  if (!layout_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  const int G = layout->n_q_heads / layout->n_kv_heads;
  if ((int64_t)window * G > kWinMaxRows) return KEEPKV_ERR_UNSUPPORTED;
  const int units = layout->batch * layout->n_kv_heads;
  if (units > kMaxUnits) return KEEPKV_ERR_UNSUPPORTED;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);

  WinParams p;
  p.k = cache->k, p.q = q_win, p.log_s = cache->log_s, p.n_obs = cache->n_obs, p.len = cache->len;
  p.capacity = cache->capacity, p.W = window, p.G = G;
  p.n_q_heads = layout->n_q_heads, p.n_kv_heads = layout->n_kv_heads;
  p.first_pos = first_pos < 0 ? -1 : first_pos;
  p.ln_alpha = alpha > 0.f ? logf(alpha) : -INFINITY;
  p.ln_1m_alpha = log1pf(-alpha);
  p.scale_over_g = layout->scale / (float)G;
  const int bound = (cache->len_hint > 0 && cache->len_hint < cache->capacity) ? cache->len_hint : cache->capacity;

  if (layout->dtype == KEEPKV_BF16) {
    int spw = 1024;                                    // keys per workgroup: enough workgroups to fill the chip
    while (spw > kWinStageSlots && (int64_t)units * ((bound + spw - 1) / spw) < 1024) spw >>= 1;
    p.slots_per_wg = spw;
    const dim3 grid((bound + spw - 1) / spw, units);
    if (layout->head_dim == 128) launch_mfma<128>(p, grid, st);
    else launch_mfma<64>(p, grid, st);
  } else {
    p.slots_per_wg = 128;
    const dim3 grid((bound + 127) / 128, units);
    const size_t smem = (size_t)window * G * layout->head_dim * sizeof(float);
    if (layout->head_dim == 128) score_window_f32_kernel<128><<<grid, 128, smem, st>>>(p);
    else score_window_f32_kernel<64><<<grid, 128, smem, st>>>(p);
  }
  return launch_status();
}
