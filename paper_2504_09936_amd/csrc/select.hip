// keepkv_select: per (batch, kv head) choose the retained set K_c and the to-be-evicted set K_e
// (Alg. 1 lines 2-3) under the fixed-budget sink / recent / heavy-hitter policy (App. B.3).
//
// One 1024-thread workgroup per head.  The ranking value ln p + ln s_hat is formed in f64 and
// mapped to an order-preserving u64, the (budget - n_sink - n_recent)-th largest is found by an
// 8-bit most-significant-digit radix select (LDS histograms, wavefront scan), and the slots are
// then compacted in index order so that equal values keep the lower index first.
#include "kk_common.hpp"

namespace kk {
namespace {

constexpr int kSelThreads = 1024;

__device__ __forceinline__ uint64_t sortable_u64(double x) {
  x = x + 0.0;  // -0.0 -> +0.0
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

// exclusive prefix sum over the block (thread order); returns the block total through `total`
__device__ __forceinline__ int block_excl_scan(int v, int* s_wave, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  __syncthreads();  // s_wave may still be read from a previous call
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  int before = 0, tot = 0;
  constexpr int nw = kSelThreads / 64;
#pragma unroll
  for (int w = 0; w < nw; ++w) {
    const int t = s_wave[w];
    before += (w < wave) ? t : 0;
    tot += t;
  }
  total = tot;
  return before + incl - v;
}

// EXT: the ranking value is read from a caller-supplied array (passed as log_s; n_obs and votes
// unused) instead of being formed from the cache's votes and EMA scores.
// LDSKEYS: the sortable keys of the head live in LDS (capacity * 8 bytes fit) instead of the workspace, so
// the radix passes and the compaction never leave the CU.
template <bool EXT, bool LDSKEYS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const float* __restrict__ log_s, const int32_t* __restrict__ n_obs, const int32_t* __restrict__ votes,
    const int32_t* __restrict__ len, uint64_t* __restrict__ keys, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ evict_idx, int32_t* __restrict__ n_evict, int capacity, int budget, int n_sink,
    int n_recent, double ln_alpha) {
  __shared__ int s_hist[256];
  __shared__ int s_wave[kSelThreads / 64];
  __shared__ int s_digit, s_need, s_bucket;
  extern __shared__ __align__(16) uint64_t s_keys[];

  const int unit = blockIdx.x;
  const int tid = threadIdx.x;
  const int n = len[unit];
  int32_t* keep_out = keep_idx + (size_t)unit * budget;
  int32_t* evict_out = evict_idx + (size_t)unit * (capacity - budget);

  if (n <= budget) {
    for (int i = tid; i < budget; i += kSelThreads) keep_out[i] = (i < n) ? i : -1;
    if (tid == 0) n_evict[unit] = 0;
    return;
  }

  const size_t base = (size_t)unit * capacity;
  uint64_t* key_g = keys + base;
  auto key = [&](int i) -> uint64_t& {
    if constexpr (LDSKEYS) return s_keys[i];
    else return key_g[i];
  };
  const int lo = n_sink, hi = n - n_recent;   // candidates are [lo, hi)
  const int n_heavy = budget - n_sink - n_recent;

  for (int i0 = lo + tid; i0 < hi; i0 += 4 * kSelThreads) {     // four slots per round trip
    int nn[4], pv[4];
    float ls[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = min(i0 + u * kSelThreads, hi - 1);
      nn[u] = EXT ? 1 : n_obs[base + i];
      pv[u] = EXT ? 1 : votes[base + i];
      ls[u] = log_s[base + i];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kSelThreads;
      if (i < hi) {
        double x;
        if (EXT) {
          x = (ls[u] == ls[u]) ? (double)ls[u] : -INFINITY;     // NaN ranks lowest
        } else if (nn[u] <= 0) {
          x = -INFINITY;
        } else {
          x = log((double)pv[u]) + (double)ls[u];
          if (ln_alpha > -INFINITY) x -= log(-expm1((double)nn[u] * ln_alpha));
        }
        key(i) = sortable_u64(x);
      }
    }
  }
  __syncthreads();

  // ---- radix select: tau = n_heavy-th largest key, need = how many keys equal to tau are kept
  uint64_t prefix = 0;
  int need = n_heavy;
  if (n_heavy > 0) {
    for (int pass = 7; pass >= 0; --pass) {
      if (tid < 256) s_hist[tid] = 0;
      __syncthreads();
      const int shift = 8 * pass;
      for (int i0 = lo + tid; i0 < hi; i0 += 4 * kSelThreads) {   // four keys per round trip
        uint64_t k4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) k4[u] = key(min(i0 + u * kSelThreads, hi - 1));
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint64_t k = k4[u];
          const bool in = (i0 + u * kSelThreads < hi) && ((pass == 7) || ((k >> (shift + 8)) == prefix));
          if (in) atomicAdd(&s_hist[(int)((k >> shift) & 255u)], 1);
        }
      }
      __syncthreads();
      if (tid < 64) {
        // lane covers digits 255-4*lane .. 252-4*lane, i.e. descending order over lanes
        int c[4], t = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          c[j] = s_hist[255 - 4 * tid - j];
          t += c[j];
        }
        int incl = t;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const int u = __shfl_up(incl, off);
          if (tid >= off) incl += u;
        }
        const uint64_t mask = __ballot(incl >= need);
        const int first = __ffsll((long long)mask) - 1;   // mask != 0: the candidates outnumber `need`
        if (tid == first) {
          int run = incl - t;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (run + c[j] >= need) {
              s_digit = 255 - 4 * tid - j;
              s_need = need - run;
              s_bucket = c[j];
              break;
            }
            run += c[j];
          }
        }
      }
      __syncthreads();
      prefix = (prefix << 8) | (uint64_t)s_digit;
      need = s_need;
      const bool whole_bucket = (s_bucket == need);   // every key with this prefix is kept: stop refining
      __syncthreads();
      if (whole_bucket && pass > 0 && prefix != 0) {
        // keep exactly the keys >= prefix << shift, i.e. key > tau with no equal keys to count
        prefix = (prefix << shift) - 1;                // prefix != 0 here: the candidates outnumber `need`
        need = 0;
        break;
      }
    }
  }
  const uint64_t tau = prefix;
  const int need_eq = need;

  // ---- ordered compaction ------------------------------------------------------------------------
  const int ipt = (n + kSelThreads - 1) / kSelThreads;
  const int i0 = min(n, tid * ipt), i1 = min(n, i0 + ipt);
  int eq = 0;
  if (n_heavy > 0)
    for (int i = max(i0, lo); i < min(i1, hi); ++i) eq += (key(i) == tau);
  int total;
  const int eq_start = block_excl_scan(eq, s_wave, total);   // equal keys at lower indices
  auto kept = [&](int i, int& er) -> bool {
    if (i < lo || i >= hi) return true;
    if (n_heavy <= 0) return false;
    const uint64_t k = key(i);
    if (k > tau) return true;
    if (k == tau) return er++ < need_eq;
    return false;
  };
  int nk = 0, er = eq_start;
  for (int i = i0; i < i1; ++i) nk += kept(i, er);
  int kpos = block_excl_scan(nk, s_wave, total);             // kept slots at lower indices
  er = eq_start;
  for (int i = i0; i < i1; ++i) {
    if (kept(i, er)) keep_out[kpos++] = i;
    else evict_out[i - kpos] = i;
  }
  if (tid == 0) n_evict[unit] = n - budget;
}

}  // namespace

constexpr int kSelLdsKeys = 16384;     // up to this capacity the keys of a head are kept in LDS (128 KB)

template <bool EXT>
void launch_select(int units, hipStream_t st, const float* log_s, const int32_t* n_obs, const int32_t* votes,
                   const int32_t* len, uint64_t* keys, int32_t* keep_idx, int32_t* evict_idx, int32_t* n_evict,
                   int capacity, int budget, int n_sink, int n_recent, double ln_alpha) {
  if (capacity <= kSelLdsKeys) {
    static const hipError_t attr = hipFuncSetAttribute((const void*)select_kernel<EXT, true>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kSelLdsKeys * 8);
    (void)attr;                              // a refusal shows up as a launch error
    select_kernel<EXT, true><<<units, kSelThreads, (size_t)capacity * 8, st>>>(
        log_s, n_obs, votes, len, keys, keep_idx, evict_idx, n_evict, capacity, budget, n_sink, n_recent, ln_alpha);
  } else {
    select_kernel<EXT, false><<<units, kSelThreads, 0, st>>>(
        log_s, n_obs, votes, len, keys, keep_idx, evict_idx, n_evict, capacity, budget, n_sink, n_recent, ln_alpha);
  }
}

SelectPlan plan_select(const keepkv_layout* L, int capacity) {
  SelectPlan pl;
  pl.keys_off = kWorkspaceHead;
  pl.bytes = kWorkspaceHead + align_up((size_t)L->batch * L->n_kv_heads * capacity * sizeof(uint64_t), 256);
  return pl;
}

}  // namespace kk

extern "C" keepkv_status keepkv_select(const keepkv_layout* layout, const keepkv_cache* cache, int32_t budget,
                                       int32_t n_sink, int32_t n_recent, float alpha, int32_t* keep_idx,
                                       int32_t* evict_idx, int32_t* n_evict, void* workspace, size_t workspace_bytes,
                                       void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !keep_idx || !n_evict) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (budget < 1 || budget > cache->capacity || n_sink < 0 || n_recent < 0 || n_sink + n_recent > budget)
    return KEEPKV_ERR_INVALID_ARG;
  if (budget < cache->capacity && !evict_idx) return KEEPKV_ERR_INVALID_ARG;
  if (!(alpha >= 0.f && alpha < 1.f)) return KEEPKV_ERR_INVALID_ARG;
  const SelectPlan pl = plan_select(layout, cache->capacity);
  if (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace)) return KEEPKV_ERR_WORKSPACE;
  const int units = layout->batch * layout->n_kv_heads;
  const double la = alpha > 0.f ? log((double)alpha) : -INFINITY;
  launch_select<false>(units, reinterpret_cast<hipStream_t>(stream),
      cache->log_s, cache->n_obs, cache->votes, cache->len,
      reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(workspace) + pl.keys_off), keep_idx, evict_idx, n_evict,
      cache->capacity, budget, n_sink, n_recent, la);
  return launch_status();
}

extern "C" keepkv_status keepkv_select_by_key(const keepkv_layout* layout, const keepkv_cache* cache,
                                              const float* rank, int32_t budget, int32_t n_sink, int32_t n_recent,
                                              int32_t* keep_idx, int32_t* evict_idx, int32_t* n_evict,
                                              void* workspace, size_t workspace_bytes, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache || !cache->len || !rank || !keep_idx || !n_evict) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (cache->capacity < 1 || cache->capacity > (1 << 20) || !aligned16(rank)) return KEEPKV_ERR_INVALID_ARG;
  if (budget < 1 || budget > cache->capacity || n_sink < 0 || n_recent < 0 || n_sink + n_recent > budget)
    return KEEPKV_ERR_INVALID_ARG;
  if (budget < cache->capacity && !evict_idx) return KEEPKV_ERR_INVALID_ARG;
  const SelectPlan pl = plan_select(layout, cache->capacity);
  if (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace)) return KEEPKV_ERR_WORKSPACE;
  const int units = layout->batch * layout->n_kv_heads;
  launch_select<true>(units, reinterpret_cast<hipStream_t>(stream),
      rank, nullptr, nullptr, cache->len,
      reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(workspace) + pl.keys_off), keep_idx, evict_idx, n_evict,
      cache->capacity, budget, n_sink, n_recent, 0.0);
  return launch_status();
}
