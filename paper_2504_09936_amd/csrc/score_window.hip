// keepkv_score_window: the EMA scores of Eq. 8 from a window of W queries in one pass over the keys
// (the t = L branch written as its sum; on an already observed cache it equals W consecutive
// keepkv_score updates).
//
// bf16 caches: the W*G query rows of one kv head against its keys is a dense contraction, done with
// 32x32x16 bf16 MFMA.  Every wavefront runs its own pipeline without workgroup barriers: it streams
// 32-key tiles (8 KB) through a private double buffer in LDS (global -> LDS without passing through
// registers, rows XOR-swizzled so that the operand reads are free of bank conflicts) and keeps all
// query rows resident in registers as the A operand.  Rows are assigned to MFMA rows such that the
// 16 accumulators of a lane are 16 consecutive query rows (whole query groups), so the group mean,
// the weights (1 - alpha) alpha^(W-1-j) and the running log-sum (held in base 2) stay inside the
// lane; the two lane halves of a key are joined once at the end.  The keys are read once: the pass
// is HBM-bound.  f32 caches take a plain one-thread-per-key kernel.
#include "kk_common.hpp"

namespace kk {
namespace {

constexpr int kWinWaves = 8;
constexpr int kWinTile = 32;               // keys per wavefront tile
constexpr int kWinMaxRows = 128;           // W * G query rows held in registers

struct WinParams {
  const void* k;
  const void* q;             // [B, Hq, W, D]
  float* log_s;
  int32_t* born;             // a slot's observation count is t_obs - born
  int32_t* t_obs;            // [B, Hkv] steps observed by the head: += W here
  const int32_t* len;
  int capacity, W, G, n_q_heads, n_kv_heads, first_pos, slots_per_wg;
  int alpha_zero;            // alpha == 0: only the last query of the window counts
  float ln_alpha;            // ln alpha, 0 when alpha == 0 (the weights are then handled by visibility)
  float ln_1m_alpha, scale_over_g;
};

// ln of the weight of query j's score in the window sum: ln((1 - alpha) alpha^(W-1-j))
__device__ __forceinline__ float win_coef(int j, int W, float ln_alpha, float ln_1m_alpha) {
  return ln_1m_alpha + (float)(W - 1 - j) * ln_alpha;
}

// first query that sees `slot`: j >= slot - first_pos (every query when first_pos < 0)
__device__ __forceinline__ int win_first_query(int slot, int first_pos) {
  return first_pos < 0 ? 0 : max(0, slot - first_pos);
}

// log_s <- ln(alpha^n_vis S + fresh), observation count += n_vis;  fresh = ln of the window's weighted sum.
// The head's step counter advances by W, so a slot seen by fewer than W queries moves its origin by the rest.
__device__ __forceinline__ void win_store(const WinParams& p, size_t at, int n_vis, float fresh) {
  if (n_vis < p.W) p.born[at] += p.W - n_vis;
  if (n_vis <= 0) return;
  const float old = p.alpha_zero ? -INFINITY : p.log_s[at] + (float)n_vis * p.ln_alpha;   // -inf: nothing observed
  const float hi = fmaxf(old, fresh), lo = fminf(old, fresh);
  p.log_s[at] = (lo == -INFINITY) ? hi : hi + log1pf(expf(lo - hi));
}

template <int D, int G>
__global__ __launch_bounds__(kWinWaves* kWave, 2) void score_window_mfma_kernel(WinParams p) {
  constexpr int ROWB = D * 2, CHUNKS = ROWB / 16, KS = D / 16;
  constexpr int TILE_BYTES = kWinTile * ROWB;
  constexpr int LOADS = TILE_BYTES / (kWave * 16);
  constexpr int NT = kWinMaxRows / 32;
  constexpr int QPL = 16 / G;                // window queries per lane and row tile
  extern __shared__ __align__(16) unsigned char s_buf[];   // [2][wave][TILE_BYTES]

  const int unit = blockIdx.y;
  const int n = p.len[unit];
  if (blockIdx.x == 0 && threadIdx.x == 0) p.t_obs[unit] += p.W;   // (no workgroup of this launch reads it)
  const int slot_begin = blockIdx.x * p.slots_per_wg;
  if (slot_begin >= n) return;               // uniform over the workgroup
  const int slot_end = min(n, slot_begin + p.slots_per_wg);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int n_tiles_wg = (slot_end - slot_begin + kWinTile - 1) / kWinTile;
  const unsigned char* kbytes = reinterpret_cast<const unsigned char*>(p.k) + (size_t)unit * p.capacity * ROWB;

  // key tile `tile` of this workgroup -> this wavefront's buffer it mod 2; chunk c of row r lands at
  // position c ^ (r mod CHUNKS)
  auto issue_tile = [&](int tile, int it) {
    unsigned char* dst = s_buf + ((it & 1) * kWinWaves + wave) * TILE_BYTES;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int c = lane + i * kWave;
      const int row = c / CHUNKS, phys = c % CHUNKS;
      const int slot = min(slot_begin + tile * kWinTile + row, n - 1);
      const unsigned char* src = kbytes + (size_t)slot * ROWB + ((phys ^ (row & (CHUNKS - 1))) * 16);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(dst + i * (kWave * 16)), 16, 0, 0);
    }
  };
  if (wave < n_tiles_wg) issue_tile(wave, 0);

  // ---- A operands.  The query rows (rho = j * G + g) are staged once per workgroup, with the same row
  // swizzle, in the second buffers (free until the loop below starts) and then held in registers;
  // row rho sits on MFMA row m such that accumulator i of lane half h is row rho = 32 t + 16 h + i.
  const int R = p.W * G;
  const int n_row_tiles = (R + 31) / 32;
  const int b = unit / p.n_kv_heads, kvh = unit % p.n_kv_heads;
  bf16x8_t a[NT][KS];
  {
    unsigned char* s_a = s_buf + kWinWaves * TILE_BYTES;
    const unsigned char* qbase = reinterpret_cast<const unsigned char*>(p.q) +
                                 ((size_t)b * p.n_q_heads + kvh * G) * p.W * ROWB;
    const int n_chunks = n_row_tiles * 32 * CHUNKS;                       // multiple of 64 * kWinWaves
    for (int c0 = 0; c0 < n_chunks; c0 += kWinWaves * kWave) {
      const int c = c0 + tid;
      const int row = min(c / CHUNKS, R - 1), phys = c % CHUNKS;            // rows past R repeat the last one
      const int j = row / G, g = row % G;
      const unsigned char* src = qbase + ((size_t)g * p.W + j) * ROWB + ((phys ^ ((c / CHUNKS) & (CHUNKS - 1))) * 16);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(s_a + (c0 + wave * kWave) * 16), 16, 0, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const int hm = (l32 >> 2) & 1, im = ((l32 >> 3) << 2) | (l32 & 3);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int rho = min(t, n_row_tiles - 1) * 32 + hm * 16 + im;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        a[t][ks] = *reinterpret_cast<const bf16x8_t*>(s_a + rho * ROWB + (((ks * 2 + half) ^ (rho & (CHUNKS - 1))) * 16));
    }
    __syncthreads();                         // the second buffers may now receive key tiles
  }
  if (wave >= n_tiles_wg) return;            // no barrier below: a wavefront without work may leave
  // base-2 exponent of query j's term: x * xs + c0 + j * cj
  const float xs = p.scale_over_g * kLog2e;
  const float cj = -p.ln_alpha * kLog2e;
  const float c0 = (p.ln_1m_alpha + (float)(p.W - 1) * p.ln_alpha) * kLog2e;
  const bool every_query = p.first_pos < 0 && !p.alpha_zero;      // uniform: no visibility mask needed

  // The read-modify-write of log_s (and, under a causal window, of born) trails the tiles by one iteration: the old values are
  // requested when a tile's arithmetic starts and consumed after the next tile's arrival has been
  // awaited, so neither their latency nor the stores' sit on the critical path.
  size_t pend_at = 0;
  int pend_nvis = 0, pend_born = 0;
  bool pend_writer = false;
  float pend_fresh = 0.f, pend_ls = 0.f;
  const bool causal = p.first_pos >= 0;       // uniform: only then can a live slot be seen by fewer than W queries
  auto finish = [&]() {
    if (causal && pend_writer && pend_nvis < p.W) p.born[pend_at] = pend_born + (p.W - pend_nvis);
    if (pend_nvis > 0) {
      const float old2 = p.alpha_zero ? -INFINITY : (pend_ls + (float)pend_nvis * p.ln_alpha) * kLog2e;
      const float hi = fmaxf(old2, pend_fresh), lo = fminf(old2, pend_fresh);      // base-2 logarithms
      const float r = (lo == -INFINITY) ? hi : hi + fast_log2(1.f + fast_exp2(lo - hi));
      p.log_s[pend_at] = r * kLn2;
    }
  };

  int it = 0;
  for (int tile = wave; tile < n_tiles_wg; tile += kWinWaves, ++it) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");               // this tile has landed
    finish();                                                      // previous tile's results
    if (tile + kWinWaves < n_tiles_wg) issue_tile(tile + kWinWaves, it + 1);
    const int slot = slot_begin + tile * kWinTile + l32;
    const int j_first = win_first_query(slot, p.first_pos);
    const int j_lo = p.alpha_zero ? max(j_first, p.W - 1) : j_first;
    const bool writer = half == 0 && slot < slot_end;
    const size_t at = (size_t)unit * p.capacity + min(slot, slot_end - 1);
    const float old_ls = p.log_s[at];
    const int old_born = causal ? p.born[at] : 0;
    const unsigned char* src = s_buf + ((it & 1) * kWinWaves + wave) * TILE_BYTES;
    bf16x8_t bk[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      bk[ks] = *reinterpret_cast<const bf16x8_t*>(src + l32 * ROWB + (((ks * 2 + half) ^ (l32 & (CHUNKS - 1))) * 16));
    float m = -INFINITY, sum = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < n_row_tiles) {                 // uniform
        f32x16_t acc = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t][ks], bk[ks], acc, 0, 0, 0);
        const int jbase = (t * 32 + half * 16) / G;
        const float cb = c0 + (float)jbase * cj;
        float y[QPL];
#pragma unroll
        for (int jj = 0; jj < QPL; ++jj) {
          float x = acc[jj * G];
#pragma unroll
          for (int g = 1; g < G; ++g) x += acc[jj * G + g];
          y[jj] = x * xs + (cb + (float)jj * cj);
        }
        if (!(every_query && t * 32 + 32 <= R)) {                  // window tail or causal / alpha = 0 masks
#pragma unroll
          for (int jj = 0; jj < QPL; ++jj) {
            const int j = jbase + jj;
            y[jj] = (j >= j_lo && j < p.W) ? y[jj] : -INFINITY;
          }
        }
        float ymax = y[0];
#pragma unroll
        for (int jj = 1; jj < QPL; ++jj) ymax = fmaxf(ymax, y[jj]);
        const float mn = fmaxf(m, ymax);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        float add = 0.f;
#pragma unroll
        for (int jj = 0; jj < QPL; ++jj) add += fast_exp2(y[jj] - ms);
        sum = sum * fast_exp2(m - ms) + add;
        m = mn;
      }
    }
    {                                        // join the two lane halves of the key
      const float m2 = __shfl_xor(m, 32), s2 = __shfl_xor(sum, 32);
      const float mn = fmaxf(m, m2);
      const float ms = (mn == -INFINITY) ? 0.f : mn;
      sum = sum * fast_exp2(m - ms) + s2 * fast_exp2(m2 - ms);
      m = mn;
    }
    pend_at = at;
    pend_nvis = writer ? p.W - min(p.W, j_first) : 0;
    pend_fresh = m + fast_log2(sum);         // base-2 logarithm of the window's weighted sum
    pend_ls = old_ls;
    pend_born = old_born;
    pend_writer = writer;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  finish();
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
  if (blockIdx.x == 0 && threadIdx.x == 0) p.t_obs[unit] += p.W;   // (no workgroup of this launch reads it)
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
  for (int j = p.alpha_zero ? max(j_first, p.W - 1) : j_first; j < p.W; ++j) {
    float x = 0.f;
    for (int g = 0; g < G; ++g) {
      const float* qr = s_q + (j * G + g) * D;
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) dot = fmaf(qr[c], kr[c], dot);
      x += dot;
    }
    const float y = x * p.scale_over_g + win_coef(j, p.W, p.ln_alpha, p.ln_1m_alpha);
    const float mn = fmaxf(m, y);
    sum = sum * expf(m - mn) + expf(y - mn);               // y is finite: mn is too
    m = mn;
  }
  win_store(p, (size_t)unit * p.capacity + slot, p.W - min(p.W, j_first), m + logf(sum));
}

template <int D, int G>
hipError_t allow_lds() {
  return hipFuncSetAttribute((const void*)score_window_mfma_kernel<D, G>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             2 * kWinWaves * kWinTile * D * 2);
}

template <int D>
bool launch_mfma(const WinParams& p, dim3 grid, hipStream_t st) {
  const size_t smem = (size_t)2 * kWinWaves * kWinTile * D * 2;
  static const hipError_t attr[4] = {allow_lds<D, 1>(), allow_lds<D, 2>(), allow_lds<D, 4>(), allow_lds<D, 8>()};
  for (hipError_t e : attr)
    if (e != hipSuccess) return false;
  switch (p.G) {
    case 1: score_window_mfma_kernel<D, 1><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
    case 2: score_window_mfma_kernel<D, 2><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
    case 4: score_window_mfma_kernel<D, 4><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
    default: score_window_mfma_kernel<D, 8><<<grid, kWinWaves * kWave, smem, st>>>(p); break;
  }
  return true;
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
  p.k = cache->k, p.q = q_win, p.log_s = cache->log_s, p.born = cache->born, p.t_obs = cache->t_obs, p.len = cache->len;
  p.capacity = cache->capacity, p.W = window, p.G = G;
  p.n_q_heads = layout->n_q_heads, p.n_kv_heads = layout->n_kv_heads;
  p.first_pos = first_pos < 0 ? -1 : first_pos;
  p.alpha_zero = alpha > 0.f ? 0 : 1;
  p.ln_alpha = alpha > 0.f ? logf(alpha) : 0.f;
  p.ln_1m_alpha = log1pf(-alpha);
  p.scale_over_g = layout->scale / (float)G;
  const int bound = (cache->len_hint > 0 && cache->len_hint < cache->capacity) ? cache->len_hint : cache->capacity;

  if (layout->dtype == KEEPKV_BF16) {
    int spw = 4096;                                    // keys per workgroup (one workgroup per CU fits): fill the chip
    while (spw > kWinWaves * kWinTile && (int64_t)units * ((bound + spw - 1) / spw) < 256) spw >>= 1;
    p.slots_per_wg = spw;
    const dim3 grid((bound + spw - 1) / spw, units);
    if (!(layout->head_dim == 128 ? launch_mfma<128>(p, grid, st) : launch_mfma<64>(p, grid, st)))
      return KEEPKV_ERR_DEVICE;
  } else {
    p.slots_per_wg = 128;
    const dim3 grid((bound + 127) / 128, units);
    const size_t smem = (size_t)window * G * layout->head_dim * sizeof(float);
    if (layout->head_dim == 128) score_window_f32_kernel<128><<<grid, 128, smem, st>>>(p);
    else score_window_f32_kernel<64><<<grid, 128, smem, st>>>(p);
  }
  return launch_status();
}
