// keepkv_select: per (batch, kv head) choose the retained set K_c and the to-be-evicted set K_e
// (Alg. 1, selection step) under the fixed-budget sink / recent / heavy-hitter policy (App. B.3).
//
// One 1024-thread workgroup per head.  The ranking value ln p + ln s_hat is formed in f64 and
// mapped to an order-preserving u64, the (budget - n_sink - n_recent)-th largest is found by an
// 8-bit most-significant-digit radix select (LDS histograms, wavefront scan; digits in which no two
// keys differ are skipped), and the slots are then compacted in index order so that equal values
// keep the lower index first.
#include "kk_common.hpp"

namespace kk {
// Phase timestamps for kernel tuning; compiled in only with -DKEEPKV_TRACE (never in the product build).
#ifdef KEEPKV_TRACE
__device__ long long kk_trace_select[16 * 1024];
#define KS_TS(i) do { if (threadIdx.x == 0 && blockIdx.x < 1024) kk_trace_select[blockIdx.x * 16 + (i)] = wall_clock64(); } while (0)
#else
#define KS_TS(i) do { } while (0)
#endif
namespace {

constexpr int kSelThreads = 1024;
constexpr int kVotesTable = 256;       // ln p is tabulated for vote counts below this
constexpr int kTermTable = 2048;       // ln(1 - alpha^n) is tabulated for n below this (alpha up to 0.98 in full)

__device__ __forceinline__ uint64_t sortable_u64(double x) {
  x = x + 0.0;  // -0.0 -> +0.0
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
// OR over the wavefront, delivered to every lane (quad swaps, mirrors within 8 and 16 lanes, then two exchanges)
__device__ __forceinline__ uint32_t wave_or(uint32_t x) {
  x |= dpp_u32<0xB1>(x);
  x |= dpp_u32<0x4E>(x);
  x |= dpp_u32<0x141>(x);
  x |= dpp_u32<0x140>(x);
  x |= (uint32_t)__shfl_xor((int)x, 16);
  x |= (uint32_t)__shfl_xor((int)x, 32);
  return x;
}

// inclusive prefix sum over the wavefront in lane order: shifts within each row of 16 lanes (lanes without a
// source add zero), then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3
template <int CTRL, int ROWS>
__device__ __forceinline__ int dpp_add(int x) {
  return x + __builtin_amdgcn_update_dpp(0, x, CTRL, ROWS, 0xF, true);
}
__device__ __forceinline__ int wave_incl_scan(int x) {
  x = dpp_add<0x111, 0xF>(x);   // row_shr:1
  x = dpp_add<0x112, 0xF>(x);   // row_shr:2
  x = dpp_add<0x114, 0xF>(x);   // row_shr:4
  x = dpp_add<0x118, 0xF>(x);   // row_shr:8
  x = dpp_add<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
  x = dpp_add<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
  return x;
}

// number of set bits of `mask` below the calling lane
__device__ __forceinline__ int rank_in_wave(uint64_t mask) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// EXT: the ranking value is read from a caller-supplied array (passed as log_s; born, t_obs and votes
// unused) instead of being formed from the cache's votes and EMA scores.
// LDSKEYS: the sortable keys of the head live in LDS (capacity * 8 bytes fit) instead of the workspace, so
// the radix passes and the compaction never leave the CU.
// AGED: the live slots are not in age order.  `order` lists the slots below `budget` from oldest to newest and
// the slots from `budget` on follow in slot order (tokens appended since the last in-place event); the whole
// selection runs on the age rank i and reads and reports slot(i), so the lists come out in age order.
template <bool EXT, bool LDSKEYS, bool AGED>
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const float* __restrict__ log_s, const int32_t* __restrict__ born, const int32_t* __restrict__ t_obs,
    const int32_t* __restrict__ votes, const int32_t* __restrict__ len, uint64_t* __restrict__ keys, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ evict_idx, int32_t* __restrict__ n_evict, int capacity, int budget, int n_sink,
    int n_recent, double ln_alpha, int n_table, const int32_t* __restrict__ order) {
  constexpr int kWaves = kSelThreads / 64;
  __shared__ double s_lnterm[EXT ? 1 : kTermTable];
  __shared__ double s_lnvotes[EXT ? 1 : kVotesTable];
  __shared__ int s_hist[256];
  __shared__ int s_eq[kWaves], s_kept[kWaves];
  __shared__ uint64_t s_or[kWaves], s_nand[kWaves];
  __shared__ int s_digit, s_need, s_bucket;
  extern __shared__ __align__(16) uint64_t s_keys[];

  const int unit = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  KS_TS(0);
  const size_t base = (size_t)unit * capacity;
  const int32_t* ord = AGED ? order + (size_t)unit * budget : nullptr;
  auto slot_of = [&](int i) -> int {              // age rank -> slot
    if constexpr (AGED) return i < budget ? min(max(ord[i], 0), capacity - 1) : i;   // (clamped: never out of bounds)
    else return i;
  };
  const int lo = n_sink;
  // the first four candidate slots of every thread are requested together with the head's length
  int nn[4], pv[4];
  float ls[4];
  uint64_t k_or = 0, k_nand = 0;              // OR of this thread's keys and of their complements
  auto request = [&](int i0) {
    int sl[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) sl[u] = slot_of(min(i0 + u * kSelThreads, capacity - 1));
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = sl[u];
      nn[u] = EXT ? 0 : born[base + i];          // turned into the observation count t_obs - born at its use
      pv[u] = EXT ? 1 : votes[base + i];
      ls[u] = log_s[base + i];
    }
  };
  request(lo + tid);
  const int t_head = EXT ? 1 : t_obs[unit];
  const int n = len[unit];
  int32_t* keep_out = keep_idx + (size_t)unit * budget;
  int32_t* evict_out = evict_idx + (size_t)unit * (capacity - budget);

  if (n <= budget) {
    for (int i = tid; i < budget; i += kSelThreads) keep_out[i] = (i < n) ? slot_of(i) : -1;
    if (tid == 0) n_evict[unit] = 0;
    return;
  }

  KS_TS(13);
  // ln(1 - alpha^n) depends on the observation count alone, and the f64 library routines behind it are some
  // hundreds of instructions: one evaluation per count (n_table of them: beyond, the term rounds to zero)
  // instead of one per slot
  if constexpr (!EXT) {
    for (int m = tid; m < n_table; m += kSelThreads) s_lnterm[m] = m > 0 ? log(-expm1((double)m * ln_alpha)) : 0.0;
    // (the last wavefronts take the votes table: the first ones have the other one's entries)
    if (tid >= kSelThreads - kVotesTable) s_lnvotes[kSelThreads - 1 - tid] = log((double)(kSelThreads - 1 - tid));
    __syncthreads();
  }
  uint64_t* key_g = keys + base;
  auto key = [&](int i) -> uint64_t& {
    if constexpr (LDSKEYS) return s_keys[i];
    else return key_g[i];
  };
  const int hi = n - n_recent;   // candidates are [lo, hi)
  const int n_heavy = budget - n_sink - n_recent;

  for (int i0 = lo + tid; i0 < hi; i0 += 4 * kSelThreads) {     // four slots per round trip
    double x[4];
    if (EXT) {
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = (ls[u] == ls[u]) ? (double)ls[u] : -INFINITY;     // NaN ranks lowest
    } else {
      // ln p + ln S - ln(1 - alpha^n), the two logarithms from the tables; a wavefront evaluates them itself
      // only where one of its lanes has a count beyond a table.
#pragma unroll
      for (int u = 0; u < 4; ++u) nn[u] = t_head - nn[u];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool valid = i0 + u * kSelThreads < hi;
        const double t = (double)nn[u] * ln_alpha;
        x[u] = (double)ls[u];
        const bool small_p = pv[u] >= 1 && pv[u] < kVotesTable;
        if (__any(valid && !small_p)) x[u] = (small_p ? s_lnvotes[pv[u]] : log((double)pv[u])) + x[u];
        else x[u] = s_lnvotes[small_p ? pv[u] : 1] + x[u];
        const bool need = t > -40.0, listed = nn[u] > 0 && nn[u] < n_table;
        double term = (need && listed) ? s_lnterm[nn[u]] : 0.0;
        if (__any(valid && need && !listed)) term = (need && !listed) ? log(-expm1(t)) : term;   // alpha close to 1
        x[u] -= term;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (nn[u] <= 0) x[u] = -INFINITY;
    }
    if (i0 + 4 * kSelThreads < hi) request(i0 + 4 * kSelThreads);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kSelThreads;
      if (i < hi) {
        const uint64_t k = sortable_u64(x[u]);
        key(i) = k;
        k_or |= k;
        k_nand |= ~k;
      }
    }
  }
  // which bits differ between any two candidate keys of the head
  {
    const uint32_t o_lo = wave_or((uint32_t)k_or), o_hi = wave_or((uint32_t)(k_or >> 32));
    const uint32_t a_lo = wave_or((uint32_t)k_nand), a_hi = wave_or((uint32_t)(k_nand >> 32));
    if (lane == 0) {
      s_or[wave] = ((uint64_t)o_hi << 32) | o_lo;
      s_nand[wave] = ((uint64_t)a_hi << 32) | a_lo;
    }
  }
  if (tid < 256) s_hist[tid] = 0;
  __syncthreads();
  KS_TS(1);
  uint64_t all_or = 0, all_nand = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    all_or |= s_or[w];
    all_nand |= s_nand[w];
  }
  const uint64_t varying = all_or & all_nand;      // a bit that is 1 in some key and 0 in another

  // ---- radix select: tau = n_heavy-th largest key, need = how many keys equal to tau are kept.
  // A digit in which no two keys differ (the sign and exponent bits, as a rule) needs no histogram: it would
  // put every candidate into one bin, and same-address LDS atomics are served one lane at a time.
  uint64_t prefix = 0;
  int need = n_heavy;
  if (n_heavy > 0) {
    int n_cand = hi - lo;                             // keys that agree with the prefix so far
    bool first_hist = true;
    for (int pass = 7; pass >= 0; --pass) {
      const int shift = 8 * pass;
      int digit, bucket;
      if (((varying >> shift) & 255u) == 0) {
        digit = (int)((all_or >> shift) & 255u);
        bucket = n_cand;
      } else {
        // s_hist is zero here: cleared before the keys' barrier, and by the scan below after each use
        for (int i0 = lo + tid; i0 < hi; i0 += 4 * kSelThreads) {   // four keys per round trip
          uint64_t k4[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) k4[u] = key(min(i0 + u * kSelThreads, hi - 1));
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const uint64_t k = k4[u];
            const bool in = (i0 + u * kSelThreads < hi) && (first_hist || ((k >> (shift + 8)) == prefix));
            const int d = (int)((k >> shift) & 255u);
            // leading digits are shared by most keys: the lanes that agree with the first lane's digit add
            // their count once instead of queueing on one LDS word
            const uint64_t act = __ballot(in);
            if (act != 0) {
              const int first = __ffsll((long long)act) - 1;
              const int d0 = __builtin_amdgcn_readlane(d, first);
              const uint64_t same = __ballot(in && d == d0);
              if (in && d != d0) atomicAdd(&s_hist[d], 1);
              if (lane == first) atomicAdd(&s_hist[d0], __popcll(same));
            }
          }
        }
        first_hist = false;
        __syncthreads();
        if (tid < 64) {
          // lane covers digits 255-4*lane .. 252-4*lane, i.e. descending order over lanes
          int c[4], t = 0;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            c[j] = s_hist[255 - 4 * tid - j];
            s_hist[255 - 4 * tid - j] = 0;
            t += c[j];
          }
          const int incl = wave_incl_scan(t);
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
        __syncthreads();          // s_digit is next written behind the next histogram's barrier
        digit = s_digit;
        need = s_need;
        bucket = s_bucket;
      }
      KS_TS(2 + (7 - pass));
      prefix = (prefix << 8) | (uint64_t)digit;
      n_cand = bucket;
      if (bucket == need && pass > 0 && prefix != 0) {
        // every key with this prefix is kept: stop refining and keep exactly the keys >= prefix << shift,
        // i.e. key > tau with no equal keys to count (prefix != 0: the candidates outnumber `need`)
        prefix = (prefix << shift) - 1;
        need = 0;
        break;
      }
    }
  }
  KS_TS(10);
  const uint64_t tau = prefix;
  const int need_eq = need;

  // ---- ordered compaction ------------------------------------------------------------------------
  // A wavefront owns a run of 64-slot chunks, lane = slot within the chunk; positions inside a chunk come
  // from a ballot, the wavefronts exchange their totals through LDS.  Equal keys are kept lowest index first.
  const int n_chunks = (n + 63) >> 6;
  const int cpw = (n_chunks + kWaves - 1) / kWaves;
  const int c0 = min(n_chunks, wave * cpw), c1 = min(n_chunks, c0 + cpw);
  const bool count_equal = n_heavy > 0 && need_eq > 0;          // uniform over the workgroup
  int eq_run = 0;
  if (count_equal) {
    int cnt = 0;
    for (int c = c0; c < c1; ++c) {
      const int i = c * 64 + lane;
      cnt += __popcll(__ballot(i >= lo && i < hi && key(i) == tau));
    }
    if (lane == 0) s_eq[wave] = cnt;
    __syncthreads();
    for (int w = 0; w < wave; ++w) eq_run += s_eq[w];          // equal keys at lower indices
  }
  // which slots of chunk c are kept; eq advances over the chunk's equal keys
  auto kept_mask = [&](int c, int& eq) -> uint64_t {
    const int i = c * 64 + lane;
    const bool cand = i >= lo && i < hi;
    const uint64_t k = (cand && n_heavy > 0) ? key(i) : 0;
    bool kept = i < n && (!cand || (n_heavy > 0 && k > tau));
    if (count_equal) {                                          // every lane takes part in the ballot
      const bool is_eq = cand && k == tau;
      const uint64_t m_eq = __ballot(is_eq);
      if (is_eq) kept = eq + rank_in_wave(m_eq) < need_eq;
      eq += __popcll(m_eq);
    }
    return __ballot(kept);
  };
  int nk = 0, eq = eq_run;
  for (int c = c0; c < c1; ++c) nk += __popcll(kept_mask(c, eq));
  if (lane == 0) s_kept[wave] = nk;
  __syncthreads();
  KS_TS(11);
  int kpos = 0;
  for (int w = 0; w < wave; ++w) kpos += s_kept[w];            // kept slots at lower indices
  eq = eq_run;
  for (int c = c0; c < c1; ++c) {
    const int i = c * 64 + lane;
    const uint64_t m = kept_mask(c, eq);
    const int at = kpos + rank_in_wave(m);
    if (i < n) {
      const int s = slot_of(i);
      if ((m >> lane) & 1) keep_out[at] = s;
      else evict_out[i - at] = s;
    }
    kpos += __popcll(m);
  }
  if (tid == 0) n_evict[unit] = n - budget;
  KS_TS(12);
}

}  // namespace

constexpr int kSelLdsKeys = 16384;     // up to this capacity the keys of a head are kept in LDS (128 KB)

template <bool EXT, bool AGED = false>
void launch_select(int units, hipStream_t st, const float* log_s, const int32_t* born, const int32_t* t_obs,
                   const int32_t* votes, const int32_t* len, uint64_t* keys, int32_t* keep_idx, int32_t* evict_idx, int32_t* n_evict,
                   int capacity, int budget, int n_sink, int n_recent, double ln_alpha, const int32_t* order = nullptr) {
  // counts from which alpha^n is below half an ulp of 1 (n ln alpha <= -40) need no table entry
  int n_table = 0;
  if (!EXT && ln_alpha > -INFINITY && ln_alpha < 0.0) {
    const double n_zero = ceil(40.0 / -ln_alpha) + 1.0;
    n_table = n_zero < (double)kTermTable ? (int)n_zero : kTermTable;
  }
  if (capacity <= kSelLdsKeys) {
    static const hipError_t attr = hipFuncSetAttribute((const void*)select_kernel<EXT, true, AGED>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kSelLdsKeys * 8);
    (void)attr;                              // a refusal shows up as a launch error
    select_kernel<EXT, true, AGED><<<units, kSelThreads, (size_t)capacity * 8, st>>>(
        log_s, born, t_obs, votes, len, keys, keep_idx, evict_idx, n_evict, capacity, budget, n_sink, n_recent, ln_alpha,
        n_table, order);
  } else {
    select_kernel<EXT, false, AGED><<<units, kSelThreads, 0, st>>>(
        log_s, born, t_obs, votes, len, keys, keep_idx, evict_idx, n_evict, capacity, budget, n_sink, n_recent, ln_alpha,
        n_table, order);
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
      cache->log_s, cache->born, cache->t_obs, cache->votes, cache->len,
      reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(workspace) + pl.keys_off), keep_idx, evict_idx, n_evict,
      cache->capacity, budget, n_sink, n_recent, la);
  return launch_status();
}

extern "C" keepkv_status keepkv_select_aged(const keepkv_layout* layout, const keepkv_cache* cache,
                                            const int32_t* order, int32_t budget, int32_t n_sink, int32_t n_recent,
                                            float alpha, int32_t* keep_idx, int32_t* evict_idx, int32_t* n_evict,
                                            void* workspace, size_t workspace_bytes, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !order || !keep_idx || !n_evict) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (budget < 1 || budget > cache->capacity || n_sink < 0 || n_recent < 0 || n_sink + n_recent > budget)
    return KEEPKV_ERR_INVALID_ARG;
  if (budget < cache->capacity && !evict_idx) return KEEPKV_ERR_INVALID_ARG;
  if (!(alpha >= 0.f && alpha < 1.f)) return KEEPKV_ERR_INVALID_ARG;
  const SelectPlan pl = plan_select(layout, cache->capacity);
  if (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace)) return KEEPKV_ERR_WORKSPACE;
  const int units = layout->batch * layout->n_kv_heads;
  const double la = alpha > 0.f ? log((double)alpha) : -INFINITY;
  launch_select<false, true>(units, reinterpret_cast<hipStream_t>(stream),
      cache->log_s, cache->born, cache->t_obs, cache->votes, cache->len,
      reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(workspace) + pl.keys_off), keep_idx, evict_idx, n_evict,
      cache->capacity, budget, n_sink, n_recent, la, order);
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
      rank, nullptr, nullptr, nullptr, cache->len,
      reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(workspace) + pl.keys_off), keep_idx, evict_idx, n_evict,
      cache->capacity, budget, n_sink, n_recent, 0.0);
  return launch_status();
}

#ifdef KEEPKV_TRACE
extern "C" int keepkv_trace_read_select(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(kk::kk_trace_select), sizeof(long long) * n);
}
#endif
