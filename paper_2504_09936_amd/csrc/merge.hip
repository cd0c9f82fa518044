// keepkv_merge: multi-way Zero Inference-Perturbation Merging (Eq. 7 in the many-to-one form of
// App. A.3, with the EMA scores of App. A.4; Alg. 1, merging step) and compaction into the
// destination cache.
//
// Two kernels.  (1) Per head, the evicted slots are grouped by merge target into a CSR list: an LDS
// histogram of match[], a block scan for the row starts, and the (target, position) keys put in
// order in LDS (by counting inside each group when all groups are short, else by a bitonic network),
// so every group lists its members in ascending slot order (deterministic summation order, no float
// atomics).  With few evictable slots per head this kernel is not launched: the second one finds each
// group's members in the match list itself.  (2) One lane group (LPS lanes, 16 bytes of a row each) per retained
// position gathers its group: the merge weights w_i = p_i s_hat_i are formed in f64 relative to
// the group's largest ln s_hat, one member per lane, and broadcast; K and V rows are accumulated in
// f32 and scaled once at the end.  Positions without members are copied bit for bit.
#include "kk_common.hpp"

namespace kk {
#ifdef KEEPKV_TRACE
__device__ long long kk_trace_merge[8 * 1024];
#define KM_TS(i) do { if (threadIdx.x == 0 && blockIdx.x < 1024) kk_trace_merge[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define KM_TS(i) do { } while (0)
#endif
namespace {

constexpr int kGroupThreads = 1024;
constexpr int kMaxBudget = 4096;
constexpr int kRankSortMax = 256;      // longest group that is ordered by counting instead of the sorting network
constexpr int kMaxEvict = 32768;          // sort keys are (target << 15) | position
constexpr double kEllGuard = 1.0e-3;

// Groups the evicted slots of one head by merge target.  Keys (target << 15 | position in the evict
// list) are put in ascending order in LDS, so each group's members come out in ascending slot order;
// CSR starts come from a histogram and a block scan.
__global__ __launch_bounds__(kGroupThreads) void merge_group_kernel(
    const int32_t* __restrict__ match, const int32_t* __restrict__ evict_idx, const int32_t* __restrict__ n_evict,
    const int32_t* __restrict__ votes, int32_t* __restrict__ start, int32_t* __restrict__ members,
    int64_t* __restrict__ dropped_votes, int capacity, int budget, int max_evict, int key_words) {
  extern __shared__ unsigned int s_key[];          // key_words words: pow2ceil(max_evict) sort keys, twice if that fits
  __shared__ int s_cnt[kMaxBudget + 1];
  __shared__ int s_wave[kGroupThreads / 64];
  __shared__ long long s_drop;
  __shared__ int s_nm, s_longest;
  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_ev = n_evict[unit];
  const int32_t* mt = match + (size_t)unit * max_evict;
  const int32_t* ev = evict_idx + (size_t)unit * max_evict;
  int32_t* st = start + (size_t)unit * (budget + 1);
  int32_t* mem = members + (size_t)unit * capacity;

  KM_TS(0);
  for (int r = tid; r <= budget; r += kGroupThreads) s_cnt[r] = 0;
  if (tid == 0) {
    s_drop = 0;
    s_nm = 0;
    s_longest = 0;
  }
  __syncthreads();
  // histogram of targets; matched slots append their key to the (unordered) sort buffer, unmatched
  // slots give up their votes.  Loads of eight slots are issued together (two dependent round trips per batch).
  long long drop = 0;
  constexpr int kBatch = 8;
  for (int j0 = tid; j0 < n_ev; j0 += kBatch * kGroupThreads) {
    int t[kBatch], e[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int j = min(j0 + u * kGroupThreads, n_ev - 1);
      t[u] = mt[j];
      e[u] = ev[j];
    }
    int pv[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) pv[u] = votes[(size_t)unit * capacity + e[u]];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int j = j0 + u * kGroupThreads;
      if (j < n_ev) {
        if (t[u] >= 0) {
          atomicAdd(&s_cnt[t[u]], 1);
          s_key[atomicAdd(&s_nm, 1)] = ((unsigned int)t[u] << 15) | (unsigned int)j;
        } else {
          drop += pv[u];
        }
      }
    }
  }
  // one LDS add per wavefront: adds to one word are served a lane at a time
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) drop += __shfl_xor(drop, off);
  if (lane == 0 && drop != 0) atomicAdd((unsigned long long*)&s_drop, (unsigned long long)drop);
  __syncthreads();
  KM_TS(1);
  const int n_matched = s_nm;
  int n2 = 1;
  while (n2 < n_matched) n2 <<= 1;
  for (int i = n_matched + tid; i < n2; i += kGroupThreads) s_key[i] = 0xFFFFFFFFu;   // padding sorts to the end

  // exclusive scan of s_cnt[0..budget): thread t owns a contiguous run of positions
  const int per = (budget + kGroupThreads - 1) / kGroupThreads;
  const int r0 = min(budget, tid * per), r1 = min(budget, r0 + per);
  int mine = 0, longest = 0;
  for (int r = r0; r < r1; ++r) {
    mine += s_cnt[r];
    longest = max(longest, s_cnt[r]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) longest = max(longest, __shfl_xor(longest, off));
  if (lane == 0 && longest > 0) atomicMax(&s_longest, longest);
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int u = __shfl_up(incl, off);
    if (lane >= off) incl += u;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += s_wave[w];
  int run = before + incl - mine;
  for (int r = r0; r < r1; ++r) {
    const int cnt = s_cnt[r];
    st[r] = run;
    s_cnt[r] = run;                                  // from here on: where the group's next member goes
    run += cnt;
  }
  if (tid == kGroupThreads - 1) st[budget] = run;
  if (tid == 0 && dropped_votes != nullptr && s_drop != 0) dropped_votes[unit] += s_drop;
  KM_TS(2);
  if (n_matched == 0) return;                       // uniform over the block

  if (s_longest <= kRankSortMax && 2 * n2 <= key_words) {   // uniform over the block
    // Short groups (the rule): every key is dropped into its group's range in arrival order, then takes the
    // place given by the number of smaller keys in its group.  Three barriers; the sorting network below needs
    // 91 stages for 8192 keys and takes five times as long.
    __syncthreads();                                // cursors complete
    unsigned int* s_place = s_key + n2;             // the keys again, grouped; the launch reserves both halves
    for (int u0 = 0; u0 * kGroupThreads < n_matched; u0 += 8) {   // eight keys per thread at a time
      unsigned int mykey[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = tid + (u0 + u) * kGroupThreads;
        mykey[u] = i < n_matched ? s_key[i] : 0u;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (tid + (u0 + u) * kGroupThreads < n_matched) s_place[atomicAdd(&s_cnt[mykey[u] >> 15], 1)] = mykey[u];
    }
    __syncthreads();                                // s_cnt[r] is now the end of group r
    for (int u0 = 0; u0 * kGroupThreads < n_matched; u0 += 8) {
      unsigned int key[8];
      int slot[8], g0[8], g1[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = min(tid + (u0 + u) * kGroupThreads, n_matched - 1);
        key[u] = s_key[i];
        slot[u] = ev[key[u] & 0x7FFFu];
        const int r = (int)(key[u] >> 15);
        g0[u] = r > 0 ? s_cnt[r - 1] : 0;
        g1[u] = s_cnt[r];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int rank = 0;
        for (int m = g0[u]; m < g1[u]; m += 4) {    // four members per round trip
          unsigned int o[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = s_place[min(m + q, g1[u] - 1)];
#pragma unroll
          for (int q = 0; q < 4; ++q) rank += (m + q < g1[u]) && o[q] < key[u];
        }
        if (tid + (u0 + u) * kGroupThreads < n_matched) mem[g0[u] + rank] = slot[u];
      }
    }
    KM_TS(3);
    KM_TS(4);
    return;
  }

  // bitonic sort, ascending.  Thread i + 1024 m handles pair i of every stage; for strides j <= 64 both
  // elements of all pairs of a wavefront lie in that wavefront's own 128-element blocks, so those stages
  // need only a wavefront-level fence instead of a workgroup barrier.
  auto stage = [&](int j, int k) {
    // up to kMaxEvict / 2 / 1024 = 16 pairs per thread, four at a time so that the LDS reads overlap
    for (int i0 = tid; i0 < (n2 >> 1); i0 += 4 * kGroupThreads) {
      int lo[4], hi[4];
      unsigned int x[4], y[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = min(i0 + u * kGroupThreads, (n2 >> 1) - 1);
        lo[u] = ((i & ~(j - 1)) << 1) | (i & (j - 1));
        hi[u] = lo[u] | j;
        x[u] = s_key[lo[u]];
        y[u] = s_key[hi[u]];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool act = i0 + u * kGroupThreads < (n2 >> 1);
        const bool up = (lo[u] & k) == 0;
        if (act && (x[u] > y[u]) == up) {
          s_key[lo[u]] = y[u];
          s_key[hi[u]] = x[u];
        }
      }
    }
  };
  for (int k = 2; k <= n2; k <<= 1) {
    int j = k >> 1;
    for (; j > 64; j >>= 1) {
      stage(j, k);
      __syncthreads();
    }
    for (; j > 0; j >>= 1) {
      stage(j, k);
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
  }
  KM_TS(3);
  for (int i = tid; i < n_matched; i += kGroupThreads) mem[i] = ev[s_key[i] & 0x7FFFu];
  KM_TS(4);
}

struct MergeParams {
  const void *sk, *sv;
  const int32_t* svotes;
  const float* slog_s;
  const int32_t* sborn;        // a slot's observation count is t_obs - born
  const int32_t* st_obs;       // [units]
  const int32_t* slen;
  void *dk, *dv;
  int32_t* dvotes;
  float* dlog_s;
  int32_t* dborn;
  int32_t* dt_obs;             // receives st_obs
  int32_t* dlen;
  const int32_t* keep_idx;
  const int32_t* n_evict;
  const int32_t* start;
  const int32_t* members;
  const int32_t* match;        // the direct variant reads the match and evict lists itself
  const int32_t* evict_idx;
  int64_t* dropped_votes;
  int scap, dcap, budget, max_evict;
  int write_len;               // 0: the caller's grouping kernel has set dst.len (prefill pass)
  double ln_alpha;
};

constexpr int kDirectMaxEvict = 256;   // up to this many evictable slots per head no CSR list is built

// ln s_hat_i = ln S_i - ln(1 - alpha^n_i); -inf when never observed
__device__ __forceinline__ double log_s_hat(float log_s, int n, double ln_alpha) {
  if (n <= 0) return -INFINITY;
  double e = (double)log_s;
  if (ln_alpha > -INFINITY) e -= log(-expm1((double)n * ln_alpha));
  return e;
}

template <int LPS>
__device__ __forceinline__ double group_max_f64(double x) {
#pragma unroll
  for (int off = 1; off < LPS; off <<= 1) x = fmax(x, __shfl_xor(x, off));
  return x;
}
template <int LPS>
__device__ __forceinline__ double group_sum_f64(double x) {
#pragma unroll
  for (int off = 1; off < LPS; off <<= 1) x += __shfl_xor(x, off);
  return x;
}

// One retained slot c (row kc / vc, votes p_c, ln S ls_c, observation count n_c) absorbs the nm evicted slots
// listed in mem, in list order: the multi-way merge of App. A.3 / A.4 with weights p * s_hat formed in f64
// relative to the group's largest ln s_hat, rows accumulated in f32 and scaled once.  Called by all LPS lanes
// of the position's lane group (lane `sub` holds 16 bytes of each row; gbase = the group's first lane in the
// wavefront).  Shared by the compacting and the in-place kernels, so both produce the same bits.
struct MergedRow {
  uint4 k, v;
  int32_t votes;
  float log_s;
  int32_t n_r;       // observation count of the merged slot
};
template <typename T, int D>
__device__ __forceinline__ MergedRow merge_position(const MergeParams& p, size_t sbase, int t_head, int c, const uint4& kc,
                                                    const uint4& vc, int p_c, float ls_c, int n_c, const int32_t* mem,
                                                    int nm, int sub, int gbase) {
  constexpr int EPL = 16 / (int)sizeof(T), LPS = D / EPL;
  const uint4* sk = reinterpret_cast<const uint4*>(p.sk);
  const uint4* sv = reinterpret_cast<const uint4*>(p.sv);
  const double E_c = log_s_hat(ls_c, n_c, p.ln_alpha);

  // pass 1 over the scalars: largest ln s_hat and total votes of the group
  double mx = E_c;
  long long P = p_c;
  for (int i0 = 0; i0 < nm; i0 += LPS) {
    const int i = i0 + sub;
    double E = -INFINITY;
    int pv = 0;
    if (i < nm) {
      const int s = mem[i];
      pv = p.svotes[sbase + s];
      E = log_s_hat(p.slog_s[sbase + s], t_head - p.sborn[sbase + s], p.ln_alpha);
    }
    mx = fmax(mx, group_max_f64<LPS>(E));
    P += (long long)group_sum_f64<LPS>((double)pv);
  }
  const bool none_seen = !(mx > -INFINITY);

  // pass 2: weights, weighted sums of rows
  float ak[EPL], av[EPL];
  auto fma_row = [&](const uint4& x, float w, float* a) {
    if constexpr (sizeof(T) == 2) {
      const uint32_t u[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        a[2 * q] = fmaf(w, bf16_lo(u[q]), a[2 * q]);
        a[2 * q + 1] = fmaf(w, bf16_hi(u[q]), a[2 * q + 1]);
      }
    } else {
      const uint32_t u[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) a[q] = fmaf(w, __builtin_bit_cast(float, u[q]), a[q]);
    }
  };
#pragma unroll
  for (int e = 0; e < EPL; ++e) ak[e] = av[e] = 0.f;
  const double w_c = none_seen ? (double)p_c : (E_c > -INFINITY ? (double)p_c * exp(E_c - mx) : 0.0);
  double W = w_c, WE = (w_c > 0.0 && !none_seen) ? w_c * E_c : 0.0;
  fma_row(kc, (float)w_c, ak);
  fma_row(vc, (float)w_c, av);
  for (int i0 = 0; i0 < nm; i0 += LPS) {
    const int i = i0 + sub;
    double w = 0.0, E = 0.0;
    int s = c;
    if (i < nm) {
      s = mem[i];
      const int pv = p.svotes[sbase + s];
      E = log_s_hat(p.slog_s[sbase + s], t_head - p.sborn[sbase + s], p.ln_alpha);
      w = none_seen ? (double)pv : (E > -INFINITY ? (double)pv * exp(E - mx) : 0.0);
    }
    W += group_sum_f64<LPS>(w);
    WE += group_sum_f64<LPS>((w > 0.0 && !none_seen) ? w * E : 0.0);
    const float wf = (float)w;
    const int cnt = min(LPS, nm - i0);
    for (int q = 0; q < cnt; ++q) {
      const int sq = __shfl(s, gbase + q);
      const float wq = __shfl(wf, gbase + q);
      fma_row(sk[(sbase + sq) * LPS + sub], wq, ak);
      fma_row(sv[(sbase + sq) * LPS + sub], wq, av);
    }
  }

  double kscale, L = -INFINITY;
  int n_r = 0;
  float out_log_s = -INFINITY;
  if (none_seen) {
    kscale = 1.0 / W;                            // W = P: vote-weighted mean, stays unobserved
  } else {
    L = mx + log(W / (double)P);                 // ln(sum p s_hat / sum p)
    const double ell_bar = WE / W;               // sum w ln s_hat / W
    kscale = (fabs(ell_bar) < kEllGuard) ? 1.0 / W : (L / ell_bar) / W;
    n_r = n_c > 1 ? n_c : 1;
    double ls = L;
    if (p.ln_alpha > -INFINITY) ls += log(-expm1((double)n_r * p.ln_alpha));
    out_log_s = (float)ls;
  }
  const float fk = (float)kscale, fv = (float)(1.0 / W);
  uint4 ok, ov;
  if constexpr (sizeof(T) == 2) {
    ok.x = pack_bf16x2(ak[0] * fk, ak[1] * fk); ok.y = pack_bf16x2(ak[2] * fk, ak[3] * fk);
    ok.z = pack_bf16x2(ak[4] * fk, ak[5] * fk); ok.w = pack_bf16x2(ak[6] * fk, ak[7] * fk);
    ov.x = pack_bf16x2(av[0] * fv, av[1] * fv); ov.y = pack_bf16x2(av[2] * fv, av[3] * fv);
    ov.z = pack_bf16x2(av[4] * fv, av[5] * fv); ov.w = pack_bf16x2(av[6] * fv, av[7] * fv);
  } else {
    ok.x = __builtin_bit_cast(uint32_t, ak[0] * fk); ok.y = __builtin_bit_cast(uint32_t, ak[1] * fk);
    ok.z = __builtin_bit_cast(uint32_t, ak[2] * fk); ok.w = __builtin_bit_cast(uint32_t, ak[3] * fk);
    ov.x = __builtin_bit_cast(uint32_t, av[0] * fv); ov.y = __builtin_bit_cast(uint32_t, av[1] * fv);
    ov.z = __builtin_bit_cast(uint32_t, av[2] * fv); ov.w = __builtin_bit_cast(uint32_t, av[3] * fv);
  }
  MergedRow out;
  out.k = ok; out.v = ov; out.votes = (int32_t)P; out.log_s = out_log_s; out.n_r = n_r;
  return out;
}

// DIRECT (few evictable slots per head, the steady state): no CSR list has been built; the workgroup reads
// the head's match and evict lists into LDS and every lane group picks its own members out of them, in list
// (= ascending slot) order, so the summation order is the CSR variant's.  The first workgroup of a head
// also adds the votes of the unmatched evicted slots to the head's dropped count.
template <typename T, int D, bool DIRECT>
__global__ __launch_bounds__(256) void merge_apply_kernel(MergeParams p) {
  constexpr int EPL = 16 / (int)sizeof(T), LPS = D / EPL, GPB = 256 / LPS;
  __shared__ int s_match[DIRECT ? kDirectMaxEvict : 1], s_evict[DIRECT ? kDirectMaxEvict : 1];
  __shared__ int s_mem[DIRECT ? GPB : 1][DIRECT ? kDirectMaxEvict : 1];
  __shared__ long long s_drop;
  const int unit = blockIdx.y;
  const int r = blockIdx.x * GPB + threadIdx.x / LPS;
  const int sub = threadIdx.x % LPS;
  const int lane = threadIdx.x & 63;
  const int gbase = lane - sub;                 // first lane of this group within the wavefront
  const int t_head = p.st_obs[unit];            // the head's step counter: unchanged by a merge
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    p.dt_obs[unit] = t_head;
    if (p.write_len) {
      const int n = p.slen[unit];
      p.dlen[unit] = n < p.budget ? n : p.budget;
    }
  }
  const size_t sbase = (size_t)unit * p.scap, dbase = (size_t)unit * p.dcap;
  const uint4* sk = reinterpret_cast<const uint4*>(p.sk);
  const uint4* sv = reinterpret_cast<const uint4*>(p.sv);
  // The slot number of this position is requested first, and with DIRECT the retained row and its scalars are
  // requested before the head's lists are waited for: requests complete in the order of issue, so the
  // lists' round trip and the row's overlap instead of following each other.
  const int c = r < p.budget ? p.keep_idx[(size_t)unit * p.budget + r] : -1;
  int n_ev = 0;
  uint4 kc = make_uint4(0, 0, 0, 0), vc = make_uint4(0, 0, 0, 0);
  int p_c = 0, n_c = 0;
  float ls_c = 0.f;
  auto request_row = [&]() {
    const size_t at = sbase + max(c, 0);           // (a negative slot number: slot 0 stands in, unused)
    kc = sk[at * LPS + sub];
    vc = sv[at * LPS + sub];
    p_c = p.svotes[at];
    ls_c = p.slog_s[at];
    n_c = t_head - p.sborn[at];
  };
  if constexpr (DIRECT) {
    n_ev = min(p.n_evict[unit], kDirectMaxEvict);
    if (threadIdx.x == 0) s_drop = 0;
    int mt[kDirectMaxEvict / 256], ev[kDirectMaxEvict / 256];
    static_assert(kDirectMaxEvict == 256, "one list entry per thread");
    mt[0] = ev[0] = 0;
    if (n_ev > 0) {                                // uniform over the workgroup (the lists may be absent otherwise)
      const int li = min((int)threadIdx.x, n_ev - 1);
      mt[0] = p.match[(size_t)unit * p.max_evict + li];
      ev[0] = p.evict_idx[(size_t)unit * p.max_evict + li];
    }
    request_row();
    if ((int)threadIdx.x < n_ev) {
      s_match[threadIdx.x] = mt[0];
      s_evict[threadIdx.x] = ev[0];
    }
    __syncthreads();
    if (blockIdx.x == 0 && p.dropped_votes != nullptr) {       // uniform over the workgroup
      long long drop = 0;
      for (int i = threadIdx.x; i < n_ev; i += 256)
        if (s_match[i] < 0) drop += p.svotes[sbase + s_evict[i]];
      if (drop != 0) atomicAdd((unsigned long long*)&s_drop, (unsigned long long)drop);
      __syncthreads();
      if (threadIdx.x == 0 && s_drop != 0) p.dropped_votes[unit] += s_drop;   // no other workgroup touches it
    }
  }
  if (r >= p.budget) return;
  // (without DIRECT: two dependent round trips per row, (slot number, member range), then (rows, scalars))
  int m0 = 0, m1 = 0;
  if constexpr (!DIRECT) {
    m0 = p.start[(size_t)unit * (p.budget + 1) + r];
    m1 = p.start[(size_t)unit * (p.budget + 1) + r + 1];
  } else {
    // this group's members: positions of the evict list whose target is r, LPS candidates at a time
    int* mine = s_mem[threadIdx.x / LPS];
    for (int i0 = 0; i0 < n_ev; i0 += LPS) {
      const bool hit = i0 + sub < n_ev && s_match[i0 + sub] == r;
      const unsigned long long wave_hits = __ballot(hit);
      const unsigned int hits = (unsigned int)(wave_hits >> gbase) & (unsigned int)((1ull << LPS) - 1ull);   // LPS <= 32
      if (hit) mine[m1 + __popc(hits & ((1u << sub) - 1u))] = s_evict[i0 + sub];
      m1 += __popc(hits);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the list is read back by this group's own lanes
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if (c < 0) return;
  uint4* dk = reinterpret_cast<uint4*>(p.dk);
  uint4* dv = reinterpret_cast<uint4*>(p.dv);
  const int nm = m1 - m0;                        // evicted members of this group
  if constexpr (!DIRECT) request_row();

  if (nm == 0) {                                  // nothing merged here: copy
    dk[(dbase + r) * LPS + sub] = kc;
    dv[(dbase + r) * LPS + sub] = vc;
    if (sub == 0) {
      p.dvotes[dbase + r] = p_c;
      p.dlog_s[dbase + r] = ls_c;
      p.dborn[dbase + r] = t_head - n_c;
    }
    return;
  }

  const int32_t* mem = DIRECT ? s_mem[threadIdx.x / LPS] : p.members + sbase + m0;
  const MergedRow mr = merge_position<T, D>(p, sbase, t_head, c, kc, vc, p_c, ls_c, n_c, mem, nm, sub, gbase);
  dk[(dbase + r) * LPS + sub] = mr.k;
  dv[(dbase + r) * LPS + sub] = mr.v;
  if (sub == 0) {
    p.dvotes[dbase + r] = mr.votes;
    p.dlog_s[dbase + r] = mr.log_s;
    p.dborn[dbase + r] = t_head - mr.n_r;
  }
}

// ---------------------------------------------------------------------------------------------------
// Merge-first prefill pass (App. B.4), grouping.  near[i] is slot i's most similar earlier key above the
// threshold, or -1: the links form a forest.  A slot is absorbed by the slot it links to unless that slot is
// itself absorbed, i.e. slots at odd depth of their tree are absorbed by their parent and slots at even depth
// stay and receive their children.  Depth parity comes from pointer jumping in LDS (links point to lower
// slot numbers; ceil(log2 len) rounds); the receiving slots are numbered in ascending order by a block scan,
// the absorbed slots grouped by receiver (histogram, scan, scatter) and put in ascending slot order inside
// each group by counting, so the merge sums in a fixed order.  Output in the form merge_apply_kernel reads:
// keep_idx (receivers, -1 behind them), CSR starts and members, all with pitch `capacity`; dst.len = receivers.
// The two per-slot work arrays live in LDS up to kPrefillLdsSlots slots per head; beyond that (GLOBAL) they are
// in the workspace and are read and written with device-scope accesses: the same steps, an L2 round trip each.
constexpr int kPrefillLdsSlots = 16384;          // two int arrays of that many words fit in LDS
constexpr int kPrefillMaxSlots = 32768;

template <int kPfItems, bool GLOBAL>
__global__ __launch_bounds__(kGroupThreads) void prefill_group_kernel(
    const int32_t* __restrict__ near, const int32_t* __restrict__ slen, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ start, int32_t* __restrict__ members, int32_t* __restrict__ dlen, int capacity,
    int32_t* __restrict__ gwork) {
  extern __shared__ int s_pf[];                   // [2][n_pad] (unused when GLOBAL)
  __shared__ int s_wave[kGroupThreads / 64];
  // (device-scope stores of this workgroup are awaited before a barrier that publishes them to its other threads)
  auto sync = [] {
    if constexpr (GLOBAL) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };
  auto ld = [](const int* q, int i) -> int {
    if constexpr (GLOBAL) return __hip_atomic_load(q + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return q[i];
  };
  auto st_ = [](int* q, int i, int v) {
    if constexpr (GLOBAL) __hip_atomic_store(q + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else q[i] = v;
  };
  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = min(slen[unit], capacity);
  const int per = (capacity + kGroupThreads - 1) / kGroupThreads;     // slots per thread, a contiguous run (<= kPfItems)
  const int i0 = tid * per;
  const int32_t* nr = near + (size_t)unit * capacity;
  int* A = GLOBAL ? gwork + (size_t)unit * 2 * per * kGroupThreads : s_pf;
  int* B = A + per * kGroupThreads;

  // (ancestor << 1) | parity of the distance to it; a slot without a link is its own ancestor
  int link[kPfItems];
#pragma unroll
  for (int u = 0; u < kPfItems; ++u) {
    const int i = i0 + u;
    link[u] = -1;
    if (u < per && i < n) {
      const int l = nr[i];
      link[u] = (l >= 0 && l < i) ? l : -1;       // (a link that does not point to an earlier slot is ignored)
      st_(A, i, link[u] >= 0 ? ((link[u] << 1) | 1) : (i << 1));
    }
  }
  sync();
  int rounds = 0;
  while ((1 << rounds) < n) ++rounds;
  int* cur = A;
  int* nxt = B;
  for (int r = 0; r < rounds; ++r) {              // uniform trip count
#pragma unroll
    for (int u = 0; u < kPfItems; ++u) {
      const int i = i0 + u;
      if (u < per && i < n) {
        const int x = ld(cur, i);
        const int y = ld(cur, x >> 1);
        st_(nxt, i, (y & ~1) | ((x ^ y) & 1));
      }
    }
    sync();
    int* t = cur; cur = nxt; nxt = t;
  }
  // absorbed = odd depth; receivers numbered in slot order
  bool absorbed[kPfItems];
  int n_recv_mine = 0;
#pragma unroll
  for (int u = 0; u < kPfItems; ++u) {
    const int i = i0 + u;
    absorbed[u] = (u < per && i < n) ? (ld(cur, i) & 1) != 0 : false;
    if (u < per && i < n && !absorbed[u]) ++n_recv_mine;
  }
  auto block_exclusive = [&](int mine, int& total) {   // exclusive prefix of `mine` over the threads, and the sum
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off);
      if (lane >= off) incl += v;
    }
    __syncthreads();                              // previous use of s_wave is over
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
    for (int w = 0; w < kGroupThreads / 64; ++w) {
      const int v = s_wave[w];
      if (w < wave) before += v;
      all += v;
    }
    total = all;
    return before + incl - mine;
  };
  int n_recv = 0;
  int rpos = block_exclusive(n_recv_mine, n_recv);
  // nxt: receiver number of every receiving slot; then cur is free
#pragma unroll
  for (int u = 0; u < kPfItems; ++u) {
    const int i = i0 + u;
    if (u < per && i < n && !absorbed[u]) {
      st_(nxt, i, rpos);
      keep_idx[(size_t)unit * capacity + rpos] = i;
      ++rpos;
    }
  }
  for (int r = n_recv + tid; r < capacity; r += kGroupThreads) keep_idx[(size_t)unit * capacity + r] = -1;
  sync();
  int* cnt = cur;                                 // histogram over receiver numbers, then cursors
  for (int r = tid; r < n_recv; r += kGroupThreads) st_(cnt, r, 0);
  int pos[kPfItems];                              // receiver number of this thread's absorbed slots
#pragma unroll
  for (int u = 0; u < kPfItems; ++u) pos[u] = absorbed[u] ? ld(nxt, link[u]) : -1;
  sync();
#pragma unroll
  for (int u = 0; u < kPfItems; ++u)
    if (absorbed[u]) atomicAdd(&cnt[pos[u]], 1);
  sync();
  // exclusive scan of cnt[0 .. n_recv): thread t owns a contiguous run of receiver numbers
  const int rper = (n_recv + kGroupThreads - 1) / kGroupThreads;
  const int q0 = min(n_recv, tid * rper), q1 = min(n_recv, q0 + rper);
  int mine = 0;
  for (int r = q0; r < q1; ++r) mine += ld(cnt, r);
  int n_abs = 0;
  int run = block_exclusive(mine, n_abs);
  int32_t* st = start + (size_t)unit * (capacity + 1);
  for (int r = q0; r < q1; ++r) {
    const int c = ld(cnt, r);
    st[r] = run;
    st_(cnt, r, run);                             // where the group's next member goes
    run += c;
  }
  for (int r = n_recv + tid; r <= capacity; r += kGroupThreads) st[r] = n_abs;
  if (tid == 0) dlen[unit] = n_recv;
  sync();
  int* tmp = nxt;                                 // the receiver numbers are in registers now: members in arrival order
#pragma unroll
  for (int u = 0; u < kPfItems; ++u)
    if (absorbed[u]) st_(tmp, atomicAdd(&cnt[pos[u]], 1), i0 + u);
  sync();                                // cnt[r] is now the end of group r
  int32_t* mem = members + (size_t)unit * capacity;
#pragma unroll
  for (int u = 0; u < kPfItems; ++u) {
    if (!absorbed[u]) continue;
    const int g0 = pos[u] > 0 ? ld(cnt, pos[u] - 1) : 0, g1 = ld(cnt, pos[u]);
    int rank = 0;
    for (int m = g0; m < g1; ++m) rank += ld(tmp, m) < i0 + u;
    mem[g0 + rank] = i0 + u;
  }
}


// ---------------------------------------------------------------------------------------------------
// In-place event (the steady state without rewriting the cache).  The live slots are not kept in age order:
// the caller's `order` lists the slots below `budget` from oldest to newest and the slots from `budget` on
// (appended since the last event) follow in slot order.  The merged slots are rewritten where they are, the
// retained slots that absorb nothing are not touched at all, and the retained tokens of the append region move
// into the slots that evicted tokens leave below `budget` (there are exactly as many), so that afterwards the
// slots below `budget` are all live, len = budget, and decode steps append behind them as before.
//
// merge_inplace_kernel, one workgroup per head.  The head's match list (at most kDirectMaxEvict entries) is
// grouped by target in LDS: every entry counts the earlier entries with its target (its place in the group,
// so members keep list order, the compacting kernel's summation order) and all of them (the group's size); the
// first entry of each target is its leader, the leaders are numbered by a ballot compaction and a scan over
// their sizes gives each group its range of the member array.  The targets are then dealt to the lane groups,
// which write the merged row over the retained slot.  Nothing that any group reads (its own retained row,
// evicted rows) is written by another group.  The same workgroup then moves the append region's retained tokens.
constexpr int kInplaceThreads = 512;
template <typename T, int D>
__global__ __launch_bounds__(kInplaceThreads) void merge_inplace_kernel(MergeParams p, int32_t* __restrict__ order) {
  constexpr int EPL = 16 / (int)sizeof(T), LPS = D / EPL, GPB = kInplaceThreads / LPS, kWaves = kInplaceThreads / 64;
  static_assert(kInplaceThreads >= kDirectMaxEvict, "one list entry per thread");
  __shared__ int s_match[kDirectMaxEvict], s_evict[kDirectMaxEvict];
  __shared__ int s_tgt[kDirectMaxEvict], s_cnt[kDirectMaxEvict], s_start[kDirectMaxEvict], s_tidx[kDirectMaxEvict];
  __shared__ int s_members[kDirectMaxEvict];
  __shared__ int s_hole[kDirectMaxEvict], s_mover[kDirectMaxEvict];
  __shared__ int s_wcnt[kWaves];
  __shared__ long long s_drop;
  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = tid % LPS, grp = tid / LPS, gbase = lane - sub;
  const int t_head = p.st_obs[unit];
  const int n_ev = min(p.n_evict[unit], kDirectMaxEvict);
  if (n_ev <= 0) return;                              // uniform over the workgroup
  const size_t sbase = (size_t)unit * p.scap;
  int mt = -1, ev = 0;
  if (tid < n_ev) {
    mt = p.match[(size_t)unit * p.max_evict + tid];
    ev = p.evict_idx[(size_t)unit * p.max_evict + tid];
    s_match[tid] = mt;
    s_evict[tid] = ev;
  }
  if (tid == 0) s_drop = 0;
  __syncthreads();
  if (p.dropped_votes != nullptr && tid < n_ev && mt < 0) {
    const long long drop = p.svotes[sbase + ev];
    if (drop != 0) atomicAdd((unsigned long long*)&s_drop, (unsigned long long)drop);
  }
  const bool matched = tid < n_ev && mt >= 0 && mt < p.budget;
  int place = 0, size = 0, first = tid;               // among the entries with this entry's target
  if (matched)
    for (int j = 0; j < n_ev; ++j) {
      const bool same = s_match[j] == mt;
      size += same;
      place += same && j < tid;
      if (same && j < first) first = j;
    }
  const bool leader = matched && place == 0;
  // uniform helper: flagged threads below the caller, and in total (two barriers)
  auto compact = [&](bool flag, int& total) -> int {
    const unsigned long long m = __ballot(flag);
    __syncthreads();                                  // the previous use of s_wcnt is over
    if (lane == 0) s_wcnt[wave] = __popcll(m);
    __syncthreads();
    int below = 0;
    total = 0;
    for (int w = 0; w < kWaves; ++w) {
      if (w < wave) below += s_wcnt[w];
      total += s_wcnt[w];
    }
    return below + __popcll(m & ((1ull << lane) - 1ull));
  };
  int nt = 0;
  const int my_t = compact(leader, nt);               // the leader's group number (list order of first entries)
  if (leader) {
    s_tgt[my_t] = mt;
    s_cnt[my_t] = size;
    s_tidx[tid] = my_t;
  }
  __syncthreads();
  if (tid < nt) {                                     // start of each group's range: a scan over at most 256 sizes
    int run = 0;
    for (int t = 0; t < tid; ++t) run += s_cnt[t];
    s_start[tid] = run;
  }
  __syncthreads();
  if (matched) s_members[s_start[s_tidx[first]] + place] = ev;
  __syncthreads();
  if (tid == 0 && p.dropped_votes != nullptr && s_drop != 0) p.dropped_votes[unit] += s_drop;

  const uint4* sk = reinterpret_cast<const uint4*>(p.sk);
  const uint4* sv = reinterpret_cast<const uint4*>(p.sv);
  uint4* dk = reinterpret_cast<uint4*>(p.dk);
  uint4* dv = reinterpret_cast<uint4*>(p.dv);
  for (int t0 = 0; t0 < nt; t0 += GPB) {              // uniform trip count: a group without a target repeats the first one and writes nothing
    const bool active = t0 + grp < nt;
    const int ti = active ? t0 + grp : 0;
    const int r = s_tgt[ti];
    const int c = p.keep_idx[(size_t)unit * p.budget + r];
    const size_t at = sbase + max(c, 0);
    const uint4 kc = sk[at * LPS + sub], vc = sv[at * LPS + sub];
    const int p_c = p.svotes[at];
    const float ls_c = p.slog_s[at];
    const int n_c = t_head - p.sborn[at];
    const MergedRow mr = merge_position<T, D>(p, sbase, t_head, c, kc, vc, p_c, ls_c, n_c, s_members + s_start[ti], s_cnt[ti],
                                              sub, gbase);
    if (active && c >= 0) {
      dk[at * LPS + sub] = mr.k;
      dv[at * LPS + sub] = mr.v;
      if (sub == 0) {
        p.dvotes[at] = mr.votes;
        p.dlog_s[at] = mr.log_s;
        p.dborn[at] = t_head - mr.n_r;
      }
    }
  }

  // ---- move the retained tokens of the append region into the evicted slots below `budget`.  Every read of an
  // evicted row of this head happened above, in this workgroup: the barriers inside compact() order them before
  // the writes below.  The k-th retained token at or beyond `budget` (in keep-list order) goes to the k-th
  // evicted slot below `budget` (in evict-list order); `order` becomes the keep list with the moved tokens at
  // their new slots; len becomes the number of retained tokens.  Sources and destinations are disjoint.
  int32_t* ord = order + (size_t)unit * p.budget;
  const int32_t* keep = p.keep_idx + (size_t)unit * p.budget;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // this wavefront's merged rows are written (a mover may be one of them)
  int n_hole = 0;
  {
    const bool hole = tid < n_ev && ev >= 0 && ev < p.budget;
    const int at = compact(hole, n_hole);
    if (hole) s_hole[at] = ev;
  }
  int n_mover = 0;
  for (int r0 = 0; r0 < p.budget; r0 += kInplaceThreads) {   // uniform trip count
    const int r = r0 + tid;
    const int c = r < p.budget ? keep[r] : -1;
    const bool mover = c >= p.budget;
    int cnt = 0;
    const int at = n_mover + compact(mover, cnt);
    if (mover && at < kDirectMaxEvict) s_mover[at] = r;
    if (r < p.budget && !mover && c >= 0) ord[r] = c;
    n_mover += cnt;
  }
  __syncthreads();
  const int n_move = min(min(n_mover, n_hole), kDirectMaxEvict);
  for (int k = grp; k < n_move; k += GPB) {
    const int r = s_mover[k];
    const size_t src = sbase + keep[r], dst = sbase + s_hole[k];
    dk[dst * LPS + sub] = sk[src * LPS + sub];
    dv[dst * LPS + sub] = sv[src * LPS + sub];
    if (sub == 0) {
      p.dvotes[dst] = p.svotes[src];
      p.dlog_s[dst] = p.slog_s[src];
      p.dborn[dst] = p.sborn[src];
      ord[r] = s_hole[k];
    }
  }
  if (tid == 0) p.dlen[unit] = p.slen[unit] - n_ev;
}

}  // namespace

PrefillMergePlan plan_prefill_merge(const keepkv_layout* L, int capacity) {
  PrefillMergePlan pl;
  const size_t units = (size_t)L->batch * L->n_kv_heads;
  pl.keep_off = kWorkspaceHead;
  pl.start_off = pl.keep_off + align_up(units * capacity * sizeof(int32_t), 256);
  pl.member_off = pl.start_off + align_up(units * ((size_t)capacity + 1) * sizeof(int32_t), 256);
  pl.work_off = pl.member_off + align_up(units * capacity * sizeof(int32_t), 256);
  const size_t pad = (size_t)((capacity + kGroupThreads - 1) / kGroupThreads) * kGroupThreads;
  pl.bytes = pl.work_off + (capacity > kPrefillLdsSlots ? align_up(units * 2 * pad * sizeof(int32_t), 256) : 0);
  return pl;
}

MergePlan plan_merge(const keepkv_layout* L, int capacity, int budget) {
  MergePlan pl;
  const size_t units = (size_t)L->batch * L->n_kv_heads;
  pl.start_off = kWorkspaceHead;
  pl.member_off = kWorkspaceHead + align_up(units * (budget + 1) * sizeof(int32_t), 256);
  pl.bytes = pl.member_off + align_up(units * capacity * sizeof(int32_t), 256);
  return pl;
}

}  // namespace kk

extern "C" keepkv_status keepkv_merge(const keepkv_layout* layout, const keepkv_cache* src, keepkv_cache* dst,
                                      int32_t budget, const int32_t* keep_idx, const int32_t* evict_idx,
                                      const int32_t* n_evict, const int32_t* match, float alpha,
                                      int64_t* dropped_votes, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(src) || !cache_ok(dst) || !keep_idx || !n_evict) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (budget < 1 || budget > src->capacity || dst->capacity < budget) return KEEPKV_ERR_INVALID_ARG;
  const int max_evict = src->capacity - budget;
  if (max_evict > 0 && (!evict_idx || !match)) return KEEPKV_ERR_INVALID_ARG;
  if (!(alpha >= 0.f && alpha < 1.f)) return KEEPKV_ERR_INVALID_ARG;
  if (src->k == dst->k || src->v == dst->v || src->votes == dst->votes || src->log_s == dst->log_s ||
      src->born == dst->born || src->t_obs == dst->t_obs)
    return KEEPKV_ERR_INVALID_ARG;
  if (!aligned16(src->k) || !aligned16(src->v) || !aligned16(dst->k) || !aligned16(dst->v)) return KEEPKV_ERR_INVALID_ARG;
  if (layout->head_dim != 64 && layout->head_dim != 128) return KEEPKV_ERR_UNSUPPORTED;
  if (budget > kMaxBudget || max_evict > kMaxEvict) return KEEPKV_ERR_UNSUPPORTED;
  const MergePlan pl = plan_merge(layout, src->capacity, budget);
  if (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace)) return KEEPKV_ERR_WORKSPACE;
  const unsigned units = (unsigned)(layout->batch * layout->n_kv_heads);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  int32_t* start = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.start_off);
  int32_t* members = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.member_off);

  size_t key_bytes = 4;
  while (key_bytes < (size_t)max_evict * 4) key_bytes <<= 1;
  if (key_bytes <= kMaxEvict * 4 / 2) key_bytes *= 2;   // room for the grouped copy of the keys (counting path)
  if (key_bytes > 32 * 1024) {
    static const hipError_t attr = hipFuncSetAttribute((const void*)merge_group_kernel,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxEvict * 4);
    if (attr != hipSuccess) return KEEPKV_ERR_DEVICE;
  }
  const bool direct = max_evict <= kDirectMaxEvict;   // the steady state: the apply kernel finds its members itself
  if (!direct)
    merge_group_kernel<<<units, kGroupThreads, key_bytes, st>>>(match, evict_idx, n_evict, src->votes, start, members,
                                                                dropped_votes, src->capacity, budget, max_evict,
                                                                (int)(key_bytes / 4));
  MergeParams p;
  p.sk = src->k; p.sv = src->v; p.svotes = src->votes; p.slog_s = src->log_s; p.sborn = src->born; p.st_obs = src->t_obs; p.slen = src->len;
  p.dk = dst->k; p.dv = dst->v; p.dvotes = dst->votes; p.dlog_s = dst->log_s; p.dborn = dst->born; p.dt_obs = dst->t_obs; p.dlen = dst->len;
  p.keep_idx = keep_idx; p.n_evict = n_evict; p.start = start; p.members = members;
  p.match = match; p.evict_idx = evict_idx; p.dropped_votes = dropped_votes;
  p.scap = src->capacity; p.dcap = dst->capacity; p.budget = budget; p.max_evict = max_evict;
  p.write_len = 1;
  p.ln_alpha = alpha > 0.f ? log((double)alpha) : -INFINITY;
  const int esz = layout->dtype == KEEPKV_BF16 ? 2 : 4;
  const int lps = layout->head_dim * esz / 16, gpb = 256 / lps;
  const dim3 grid((budget + gpb - 1) / gpb, units);
  if (layout->dtype == KEEPKV_BF16) {
    if (layout->head_dim == 128) {
      if (direct) merge_apply_kernel<uint16_t, 128, true><<<grid, 256, 0, st>>>(p);
      else merge_apply_kernel<uint16_t, 128, false><<<grid, 256, 0, st>>>(p);
    } else {
      if (direct) merge_apply_kernel<uint16_t, 64, true><<<grid, 256, 0, st>>>(p);
      else merge_apply_kernel<uint16_t, 64, false><<<grid, 256, 0, st>>>(p);
    }
  } else {
    if (layout->head_dim == 128) {
      if (direct) merge_apply_kernel<float, 128, true><<<grid, 256, 0, st>>>(p);
      else merge_apply_kernel<float, 128, false><<<grid, 256, 0, st>>>(p);
    } else {
      if (direct) merge_apply_kernel<float, 64, true><<<grid, 256, 0, st>>>(p);
      else merge_apply_kernel<float, 64, false><<<grid, 256, 0, st>>>(p);
    }
  }
  return launch_status();
}

extern "C" keepkv_status keepkv_merge_inplace(const keepkv_layout* layout, keepkv_cache* cache, int32_t* order,
                                              int32_t budget, const int32_t* keep_idx, const int32_t* evict_idx,
                                              const int32_t* n_evict, const int32_t* match, float alpha,
                                              int64_t* dropped_votes, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !order || !keep_idx || !n_evict) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (budget < 1 || budget > cache->capacity) return KEEPKV_ERR_INVALID_ARG;
  const int max_evict = cache->capacity - budget;
  if (max_evict > 0 && (!evict_idx || !match)) return KEEPKV_ERR_INVALID_ARG;
  if (!(alpha >= 0.f && alpha < 1.f)) return KEEPKV_ERR_INVALID_ARG;
  if (!aligned16(cache->k) || !aligned16(cache->v)) return KEEPKV_ERR_INVALID_ARG;
  if (layout->head_dim != 64 && layout->head_dim != 128) return KEEPKV_ERR_UNSUPPORTED;
  if (budget > kMaxBudget || max_evict > kDirectMaxEvict) return KEEPKV_ERR_UNSUPPORTED;
  if (max_evict == 0) return KEEPKV_OK;                // nothing can have been evicted
  const unsigned units = (unsigned)(layout->batch * layout->n_kv_heads);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  MergeParams p;
  p.sk = cache->k; p.sv = cache->v; p.svotes = cache->votes; p.slog_s = cache->log_s; p.sborn = cache->born; p.st_obs = cache->t_obs; p.slen = cache->len;
  p.dk = cache->k; p.dv = cache->v; p.dvotes = cache->votes; p.dlog_s = cache->log_s; p.dborn = cache->born; p.dt_obs = cache->t_obs; p.dlen = cache->len;
  p.keep_idx = keep_idx; p.n_evict = n_evict; p.start = nullptr; p.members = nullptr;
  p.match = match; p.evict_idx = evict_idx; p.dropped_votes = dropped_votes;
  p.scap = cache->capacity; p.dcap = cache->capacity; p.budget = budget; p.max_evict = max_evict;
  p.write_len = 0;
  p.ln_alpha = alpha > 0.f ? log((double)alpha) : -INFINITY;
  if (layout->dtype == KEEPKV_BF16) {
    if (layout->head_dim == 128) {
      merge_inplace_kernel<uint16_t, 128><<<units, kInplaceThreads, 0, st>>>(p, order);
    } else {
      merge_inplace_kernel<uint16_t, 64><<<units, kInplaceThreads, 0, st>>>(p, order);
    }
  } else {
    if (layout->head_dim == 128) {
      merge_inplace_kernel<float, 128><<<units, kInplaceThreads, 0, st>>>(p, order);
    } else {
      merge_inplace_kernel<float, 64><<<units, kInplaceThreads, 0, st>>>(p, order);
    }
  }
  return launch_status();
}

extern "C" keepkv_status keepkv_prefill_merge(const keepkv_layout* layout, const keepkv_cache* src, keepkv_cache* dst,
                                              const int32_t* near, float alpha, void* workspace,
                                              size_t workspace_bytes, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(src) || !cache_ok(dst) || !near) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (dst->capacity < src->capacity || !(alpha >= 0.f && alpha < 1.f)) return KEEPKV_ERR_INVALID_ARG;
  if (src->k == dst->k || src->v == dst->v || src->votes == dst->votes || src->log_s == dst->log_s ||
      src->born == dst->born || src->t_obs == dst->t_obs || src->len == dst->len)
    return KEEPKV_ERR_INVALID_ARG;
  if (!aligned16(src->k) || !aligned16(src->v) || !aligned16(dst->k) || !aligned16(dst->v)) return KEEPKV_ERR_INVALID_ARG;
  if (layout->head_dim != 64 && layout->head_dim != 128) return KEEPKV_ERR_UNSUPPORTED;
  const int cap = src->capacity;
  if (cap > kPrefillMaxSlots) return KEEPKV_ERR_UNSUPPORTED;
  const PrefillMergePlan pl = plan_prefill_merge(layout, cap);
  if (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace)) return KEEPKV_ERR_WORKSPACE;
  const unsigned units = (unsigned)(layout->batch * layout->n_kv_heads);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  int32_t* keep = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.keep_off);
  int32_t* start = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.start_off);
  int32_t* members = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.member_off);

  const int per = (cap + kGroupThreads - 1) / kGroupThreads;
  if (cap <= kPrefillLdsSlots) {
    const size_t lds = (size_t)2 * per * kGroupThreads * sizeof(int);
    static const hipError_t attr = hipFuncSetAttribute((const void*)prefill_group_kernel<kPrefillLdsSlots / kGroupThreads, false>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       2 * kPrefillLdsSlots * (int)sizeof(int));
    if (attr != hipSuccess) return KEEPKV_ERR_DEVICE;
    prefill_group_kernel<kPrefillLdsSlots / kGroupThreads, false><<<units, kGroupThreads, lds, st>>>(
        near, src->len, keep, start, members, dst->len, cap, nullptr);
  } else {
    int32_t* work = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.work_off);
    prefill_group_kernel<kPrefillMaxSlots / kGroupThreads, true><<<units, kGroupThreads, 0, st>>>(
        near, src->len, keep, start, members, dst->len, cap, work);
  }

  MergeParams p;
  p.sk = src->k; p.sv = src->v; p.svotes = src->votes; p.slog_s = src->log_s; p.sborn = src->born; p.st_obs = src->t_obs; p.slen = src->len;
  p.dk = dst->k; p.dv = dst->v; p.dvotes = dst->votes; p.dlog_s = dst->log_s; p.dborn = dst->born; p.dt_obs = dst->t_obs; p.dlen = dst->len;
  p.keep_idx = keep; p.n_evict = nullptr; p.start = start; p.members = members;
  p.match = nullptr; p.evict_idx = nullptr; p.dropped_votes = nullptr;
  p.scap = cap; p.dcap = dst->capacity; p.budget = cap; p.max_evict = 0;
  p.write_len = 0;
  p.ln_alpha = alpha > 0.f ? log((double)alpha) : -INFINITY;
  const int esz = layout->dtype == KEEPKV_BF16 ? 2 : 4;
  const int lps = layout->head_dim * esz / 16, gpb = 256 / lps;
  const dim3 grid((cap + gpb - 1) / gpb, units);
  if (layout->dtype == KEEPKV_BF16) {
    if (layout->head_dim == 128) merge_apply_kernel<uint16_t, 128, false><<<grid, 256, 0, st>>>(p);
    else merge_apply_kernel<uint16_t, 64, false><<<grid, 256, 0, st>>>(p);
  } else {
    if (layout->head_dim == 128) merge_apply_kernel<float, 128, false><<<grid, 256, 0, st>>>(p);
    else merge_apply_kernel<float, 64, false><<<grid, 256, 0, st>>>(p);
  }
  return launch_status();
}

#ifdef KEEPKV_TRACE
extern "C" int keepkv_trace_read_merge(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(kk::kk_trace_merge), sizeof(long long) * n);
}
#endif
