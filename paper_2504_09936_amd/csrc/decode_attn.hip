// keepkv_decode_attn / keepkv_decode_step: vote-weighted flash-decode attention (Eq. 6) with
// split-K over slots, optionally fused with the cache append (Sec. 3.1) and the EMA score update
// (Eq. 8) so that one decode step of one layer is a single kernel.
//
// One workgroup handles one (batch, kv head, split).  bf16 caches run both contractions on the matrix
// cores (decode_mfma_kernel below, 4 or 8 wavefronts per workgroup).  In the vector-ALU kernel (f32
// caches, 4 wavefronts) a slot's row (D elements) is spread over LPS consecutive lanes, 16 bytes per lane, so one wavefront load instruction
// streams 64/LPS whole rows, fully coalesced.  Each lane group computes the G logits of its
// slot with bf16 dot2 (or f32 fma) plus a DPP all-reduce inside the group, keeps its own
// online-softmax state in the log2 domain with log2(votes) folded into the logit, and
// accumulates p * v for its 16-byte slice of V.  Lane groups and wavefronts are combined through
// shuffles and LDS; splits are combined by the last workgroup of each head to finish (a ticket
// counter in the workspace head), so no second kernel is launched.
#include <math.h>

#include <mutex>

#include <type_traits>

#include "kk_common.hpp"

namespace kk {

// Phase timestamps for kernel tuning; compiled in only with -DKEEPKV_TRACE (never in the product build).
#ifdef KEEPKV_TRACE
__device__ long long kk_trace[8 * 8192];
#define KK_TS(i) do { if (threadIdx.x == 0 && blockIdx.x < 8192) kk_trace[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define KK_TS(i) do { } while (0)
#endif

namespace {

struct DecodeParams {
  const void* q;
  void* k;            // written only in step mode (the appended row)
  void* v;
  int32_t* votes;
  float* log_s;       // step mode / score fusion
  int32_t* born;      // step mode: the new slot's origin (a slot's observation count is t_obs - born)
  int32_t* t_obs;     // step mode: [B * Hkv] steps observed by the head, += 1 per step
  int32_t* len;
  const void* k_t;    // step mode: [B, Hkv, D] new token, else null
  const void* v_t;
  int32_t* overflow;
  void* out;
  float* logits_out;
  float* lse_out;
  float* partial;     // [B*Hq, nsplit, D + 2]
  int32_t* ticket;    // [B*Hkv] zero between launches
  int n_kv_heads;
  int capacity;
  int nsplit;
  int per;          // slots per split
  int len_hint;     // caller's upper bound on len (0: none)
  int waves;        // wavefronts per workgroup of the matrix-core kernel (4 or 8)
  float scale;
  float ln_alpha, ln_1m_alpha;
};

constexpr int kWavesPerBlock = 4;   // the vector-ALU kernel
// The matrix-core kernel comes with 4 and with 8 wavefronts per workgroup (64 / 128 KB of tile buffers at
// D = 128: two workgroups or one per compute unit); plan_decode picks.


__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Everything after the workgroup's kParts partial softmax states (m, l, acc[D] per head) have been
// deposited in LDS and a barrier has passed: reduce them; a single split finishes the head, otherwise the
// partial result goes to the workspace and the last workgroup of the head to arrive combines the splits,
// resets the ticket and (step mode) publishes the new len.
template <typename T, int D, int G, int kParts, bool STEP, int WAVES>
__device__ __forceinline__ void combine_and_finish(const DecodeParams& p, const float* s_m, const float* s_l,
                                                   const float* s_acc, int* s_last_p, int unit, int split, bool grow,
                                                   int len, int t_old) {
  constexpr bool kBf16 = sizeof(T) == 2;
  int& s_last = *s_last_p;
  auto finish = [&](size_t row, int d, float M, float L, float A) {
    const float o = (L > 0.f) ? A / L : 0.f;
    if constexpr (kBf16)
      reinterpret_cast<uint16_t*>(p.out)[row * D + d] = (uint16_t)f32_to_bf16_bits(o);
    else
      reinterpret_cast<float*>(p.out)[row * D + d] = o;
    if (d == 0 && p.lse_out != nullptr) p.lse_out[row] = (L > 0.f) ? (M + fast_log2(L)) * kLn2 : -INFINITY;
  };

  for (int idx = threadIdx.x; idx < G * D; idx += WAVES * kWave) {
    const int g = idx / D, d = idx % D;
    float M = s_m[g];
#pragma unroll
    for (int w = 1; w < kParts; ++w) M = fmaxf(M, s_m[w * G + g]);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < kParts; ++w) {
      const float mw = s_m[w * G + g];
      const float c = (mw == -INFINITY) ? 0.f : fast_exp2(mw - M);
      L = fmaf(s_l[w * G + g], c, L);
      A = fmaf(s_acc[(w * G + g) * D + d], c, A);
    }
    const size_t row = (size_t)unit * G + g;   // == b * Hq + h * G + g
    if (p.nsplit == 1) {
      finish(row, d, M, L, A);
    } else {
      // device-coherent (write-through) stores: the combining workgroup may run on another XCD
      float* dst = p.partial + (row * p.nsplit + split) * (D + 2);
      st_agent(dst + 2 + d, A);
      if (d == 0) {
        st_agent(dst, M);
        st_agent(dst + 1, L);
      }
    }
  }

  if (p.nsplit == 1) {
    if (STEP && threadIdx.x == 0) p.t_obs[unit] = t_old + 1;   // one more observation of every slot of the head
    if (STEP && threadIdx.x == 0 && grow) p.len[unit] = len;   // every wavefront read len before the barrier above
    if (STEP && threadIdx.x == 0 && !grow && p.overflow != nullptr) *p.overflow = 1;
    return;
  }

  KK_TS(3);
  // ---- the last workgroup of this head to arrive combines the splits ------------------------------
  // The partial results were stored write-through at device scope, so it is enough that every
  // wavefront's stores have completed before the ticket is taken: each wavefront waits on its own
  // memory counter (stores count there on this part), then the barrier orders all of them before
  // thread 0's ticket.  A workgroup-scope release fence emits no such wait here (the workgroup shares
  // one L2, so the compiler needs none for that scope), and a device-scope release fence would write
  // back the whole L2 per workgroup.  The combining workgroup reads the partials with device-scope loads.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0)
    s_last = (__hip_atomic_fetch_add(&p.ticket[unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.nsplit - 1);
  __syncthreads();
  KK_TS(4);
  if (!s_last) return;
  // CH splits of EB output elements are fetched per round trip of device-scope loads: 8 splits of two
  // elements when that covers all splits (the common case; surplus loads would only cost), else 16 of one
  constexpr int kThreads = WAVES * kWave;
  constexpr int kPerThread = (G * D + kThreads - 1) / kThreads;   // output elements per thread
  auto combine = [&](auto ch_tag, auto eb_tag) {
    constexpr int CH = decltype(ch_tag)::value, EB = decltype(eb_tag)::value;
    for (int e0 = 0; e0 < kPerThread; e0 += EB) {
      int idx[EB];
      const float* src[EB];
      float M[EB], L[EB], A[EB];
#pragma unroll
      for (int j = 0; j < EB; ++j) {
        idx[j] = min((int)threadIdx.x + (e0 + j) * kThreads, G * D - 1);   // surplus threads repeat the last element
        src[j] = p.partial + ((size_t)unit * G + idx[j] / D) * p.nsplit * (D + 2);
        M[j] = -INFINITY;
        L[j] = 0.f;
        A[j] = 0.f;
      }
      for (int s0 = 0; s0 < p.nsplit; s0 += CH) {
        float ms[EB][CH], ls[EB][CH], as[EB][CH];
#pragma unroll
        for (int j = 0; j < EB; ++j)
#pragma unroll
          for (int i = 0; i < CH; ++i) {
            const int s = min(s0 + i, p.nsplit - 1);
            ms[j][i] = ld_agent(src[j] + s * (D + 2));
            ls[j][i] = ld_agent(src[j] + s * (D + 2) + 1);
            as[j][i] = ld_agent(src[j] + s * (D + 2) + 2 + idx[j] % D);
          }
#pragma unroll
        for (int j = 0; j < EB; ++j) {
          float mc = M[j];
#pragma unroll
          for (int i = 0; i < CH; ++i) mc = fmaxf(mc, ms[j][i]);
          const float c0 = (M[j] == -INFINITY) ? 0.f : fast_exp2(M[j] - mc);
          L[j] *= c0;
          A[j] *= c0;
#pragma unroll
          for (int i = 0; i < CH; ++i) {
            const float c = (s0 + i < p.nsplit && ms[j][i] != -INFINITY) ? fast_exp2(ms[j][i] - mc) : 0.f;
            L[j] = fmaf(ls[j][i], c, L[j]);
            A[j] = fmaf(as[j][i], c, A[j]);
          }
          M[j] = mc;
        }
      }
#pragma unroll
      for (int j = 0; j < EB; ++j)
        if ((int)threadIdx.x + (e0 + j) * kThreads < G * D)
          finish((size_t)unit * G + idx[j] / D, idx[j] % D, M[j], L[j], A[j]);
    }
  };
  if (p.nsplit <= 8) combine(std::integral_constant<int, 8>{}, std::integral_constant<int, (kPerThread >= 2 ? 2 : 1)>{});
  else combine(std::integral_constant<int, 16>{}, std::integral_constant<int, 1>{});
  KK_TS(5);
  if (threadIdx.x == 0) {
    __hip_atomic_store(&p.ticket[unit], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
    if (STEP) p.t_obs[unit] = t_old + 1;             // (every workgroup of the head read it before taking its ticket)
    if (STEP && grow) p.len[unit] = len;
    if (STEP && !grow && p.overflow != nullptr) *p.overflow = 1;
  }
}

// LPS lanes share one slot's row, each holding VPL 16-byte vectors of it (vector v of lane `sub` is
// row vector v * LPS + sub, so the LPS lanes of a group read LPS * 16 contiguous bytes per load).
// kUnroll slots per lane group are in flight per iteration.
// STEP: append (k_t, v_t) as a new slot, attend over old + new, update the EMA scores, bump len.
template <typename T, int D, int G, int LPS, int kUnroll, bool STEP>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void decode_attn_kernel(DecodeParams p) {
  constexpr int EPV = 16 / (int)sizeof(T);              // elements per 16-byte vector
  constexpr int RV = D / EPV;                           // vectors per row
  constexpr int VPL = RV / LPS;                         // vectors per lane
  constexpr int EPL = EPV * VPL;                        // elements per lane
  constexpr int GPW = kWave / LPS;                      // slots per load instruction
  constexpr int TILE = GPW * kUnroll;                   // slots per wavefront per iteration
  constexpr bool kBf16 = sizeof(T) == 2;
  static_assert(VPL >= 1 && RV % LPS == 0 && kUnroll <= LPS, "bad lane mapping");

  extern __shared__ __align__(16) float smem[];
  __shared__ int s_last;
  __shared__ uint4 s_new[2 * RV];             // step mode: the appended token's K row, then its V row

  const int unit = blockIdx.x / p.nsplit;    // b * Hkv + h
  const int split = blockIdx.x % p.nsplit;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPS, sub = lane % LPS;
  KK_TS(0);
  const int len_old = p.len[unit];          // needed only once the row loads are in flight (see `bound`)
  const int t_old = STEP ? p.t_obs[unit] : 0;   // used at the very end only
  // step mode: the new token becomes slot len_old (unless the head is full); it is attended as one
  // extra slot after the cache slots, so the streaming loop below never depends on it
  const int start = split * p.per;
  // The wavefront that will attend the appended token copies it to LDS asynchronously (no registers,
  // no wait), so that its extra slot costs no memory round trip after the streaming loop.
  // (the last wavefront of the last split: its own share of the cache is the shortest)
  const bool takes_new = STEP && split == p.nsplit - 1 && wave == kWavesPerBlock - 1;
  if (takes_new && lane < 2 * RV) {
    const uint4* src = (lane < RV ? reinterpret_cast<const uint4*>(p.k_t) : reinterpret_cast<const uint4*>(p.v_t)) +
                       (size_t)unit * RV + (lane % RV);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)s_new, 16, 0, 0);
  }
  // Rows are fetched up to `bound`: the caller's upper bound on len if given, so that the loads do
  // not wait for the len load; otherwise len itself.  Slots at or beyond len are masked out.
  const int bound = p.len_hint > 0 ? min(p.len_hint, p.capacity) : len_old;
  const int lim = min(bound, start + p.per);

  // query slice of this lane for each head of the group
  uint4 qv[G][VPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int v = 0; v < VPL; ++v)
      qv[g][v] = reinterpret_cast<const uint4*>(p.q)[((size_t)unit * G + g) * RV + v * LPS + sub];

  float m[G], l[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  const size_t ubase = (size_t)unit * p.capacity;
  uint4* kbase = reinterpret_cast<uint4*>(p.k) + ubase * RV + sub;
  uint4* vbase = reinterpret_cast<uint4*>(p.v) + ubase * RV + sub;
  const float sl2 = p.scale * kLog2e;

  // One tile: kUnroll slots per lane group.  `extra` is the appended token (step mode): lane group 0
  // takes it from (k_t, v_t) as its slot 0, every other slot of the tile is masked.
  auto tile = [&](int base, bool extra) {
    const int s0 = extra ? len_old : base + grp * kUnroll;
    uint4 kk_[kUnroll][VPL], vv_[kUnroll][VPL];
    int pv[kUnroll];
    bool live[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      if (extra) {                               // only slot 0 is real; it comes from LDS
        pv[j] = 1;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          kk_[j][v] = (j == 0) ? s_new[v * LPS + sub] : make_uint4(0, 0, 0, 0);
          vv_[j][v] = (j == 0) ? s_new[RV + v * LPS + sub] : make_uint4(0, 0, 0, 0);
        }
      } else {
        const int s = min(s0 + j, bound - 1);   // clamp: slots at or beyond `bound` are never read
        const uint4* ka = kbase + (size_t)s * RV;
        const uint4* va = vbase + (size_t)s * RV;
        pv[j] = p.votes[ubase + s];              // unconditional and in bounds: a branch behind a
#pragma unroll                                   // load would serialise the row loads
        for (int v = 0; v < VPL; ++v) {
          kk_[j][v] = load_once(ka + v * LPS);
          vv_[j][v] = load_once(va + v * LPS);
        }
      }
    }
    // EMA state of the slot this lane will update (lane `sub` < kUnroll owns slot s0 + sub)
    const int s_mine = s0 + (extra ? 0 : sub);
    float ls_old = -INFINITY;
    if (STEP && !extra) ls_old = p.log_s[ubase + min(s_mine, bound - 1)];
    // ---- first use of len: everything above was issued without waiting for it
    const int live_end = min(len_old, start + p.per);
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) live[j] = extra ? (grp == 0 && j == 0) : (s0 + j < live_end);
    if (extra || base + TILE > live_end) {       // uniform over the wavefront: the tile holds masked slots;
#pragma unroll                                   // zero their V so that 0 * garbage cannot make a NaN
      for (int j = 0; j < kUnroll; ++j) {
        const uint32_t keepmask = live[j] ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          vv_[j][v].x &= keepmask; vv_[j][v].y &= keepmask; vv_[j][v].z &= keepmask; vv_[j][v].w &= keepmask;
        }
      }
    }

    float z[G][kUnroll];
    float mean_logit[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const float lp = fast_log2((float)pv[j]);
      float sum = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          const uint4 a = kk_[j][v], b = qv[g][v];
          if constexpr (kBf16) {
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), d, false);
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), d, false);
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), d, false);
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), d, false);
          } else {
            d = fmaf(__builtin_bit_cast(float, a.x), __builtin_bit_cast(float, b.x), d);
            d = fmaf(__builtin_bit_cast(float, a.y), __builtin_bit_cast(float, b.y), d);
            d = fmaf(__builtin_bit_cast(float, a.z), __builtin_bit_cast(float, b.z), d);
            d = fmaf(__builtin_bit_cast(float, a.w), __builtin_bit_cast(float, b.w), d);
          }
        }
        d = group_sum<LPS>(d);
        sum += d;
        z[g][j] = live[j] ? fmaf(d, sl2, lp) : -INFINITY;
      }
      mean_logit[j] = sum * (p.scale * (1.0f / G));
    }

    {
      // every lane evaluates the update of slot s0 + (sub mod kUnroll); only the owning lanes store
      float x = mean_logit[0];
      if (!extra) {
#pragma unroll
        for (int j = 1; j < kUnroll; ++j) x = ((sub & (kUnroll - 1)) == j) ? mean_logit[j] : x;
      }
      const bool mine = extra ? (grp == 0 && sub == 0) : (sub < kUnroll && s_mine < live_end);
      if (p.logits_out != nullptr && mine) p.logits_out[ubase + s_mine] = x;
      if constexpr (STEP) {
        // log_s <- ln(alpha S + (1 - alpha) e^x)  (Eq. 8); the count advances with the head's t_obs
        const float a = p.ln_alpha + ls_old, b = p.ln_1m_alpha + x;
        const float hi = fmaxf(a, b), lo = fminf(a, b);
        const float r = (lo == -INFINITY) ? hi : hi + log1pf(expf(lo - hi));
        if (mine) p.log_s[ubase + s_mine] = r;
      }
    }
    if (STEP && extra && grp == 0) {
      // store the new token into the cache
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        kbase[(size_t)len_old * RV + v * LPS] = kk_[0][v];
        vbase[(size_t)len_old * RV + v * LPS] = vv_[0][v];
      }
      if (sub == 0) {
        p.votes[ubase + len_old] = 1;
        p.born[ubase + len_old] = t_old;          // first observed in this step
      }
    }

    // online softmax update for this group's kUnroll slots
    float pw[G][kUnroll];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float tm = z[g][0];
#pragma unroll
      for (int j = 1; j < kUnroll; ++j) tm = fmaxf(tm, z[g][j]);
      const float mn = fmaxf(m[g], tm);
      const float c = (mn == -INFINITY) ? 0.f : fast_exp2(m[g] - mn);
      m[g] = mn;
      float ps = 0.f;
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) {
        pw[g][j] = (mn == -INFINITY) ? 0.f : fast_exp2(z[g][j] - mn);
        ps += pw[g][j];
      }
      l[g] = fmaf(l[g], c, ps);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= c;
    }
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      float vf[EPL];
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        const uint4 x = vv_[j][v];
        if constexpr (kBf16) {
          vf[v * 8 + 0] = bf16_lo(x.x); vf[v * 8 + 1] = bf16_hi(x.x);
          vf[v * 8 + 2] = bf16_lo(x.y); vf[v * 8 + 3] = bf16_hi(x.y);
          vf[v * 8 + 4] = bf16_lo(x.z); vf[v * 8 + 5] = bf16_hi(x.z);
          vf[v * 8 + 6] = bf16_lo(x.w); vf[v * 8 + 7] = bf16_hi(x.w);
        } else {
          vf[v * 4 + 0] = __builtin_bit_cast(float, x.x); vf[v * 4 + 1] = __builtin_bit_cast(float, x.y);
          vf[v * 4 + 2] = __builtin_bit_cast(float, x.z); vf[v * 4 + 3] = __builtin_bit_cast(float, x.w);
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pw[g][j], vf[e], acc[g][e]);
    }
  };

  for (int base = start + wave * TILE; base < lim; base += kWavesPerBlock * TILE) tile(base, false);
  KK_TS(1);
  const bool grow = STEP && len_old < p.capacity;
  const int len = grow ? len_old + 1 : len_old;
  if (takes_new) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the asynchronous copy of the new token has landed
    if (grow) tile(0, true);
  }

  // ---- combine lane groups and wavefronts through LDS ----------------------------------------------
  // With 8 lanes per slot the two groups of a 16-lane row are merged first with one DPP rotation;
  // each row then deposits its (m, l, acc) and the workgroup reduces kParts partial states.
  if constexpr (LPS == 8) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = dpp_f32<0x128>(m[g]);        // row_ror:8 = the other group of this row
      const float mw = fmaxf(m[g], mo);
      const float c = (m[g] == -INFINITY) ? 0.f : fast_exp2(m[g] - mw);
      const float lc = l[g] * c;
      l[g] = lc + dpp_f32<0x128>(lc);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float a = acc[g][e] * c;
        acc[g][e] = a + dpp_f32<0x128>(a);
      }
      m[g] = mw;
    }
  }
  constexpr int LPR = LPS < 16 ? 16 : LPS;            // lanes per deposited part
  constexpr int kParts = kWavesPerBlock * (kWave / LPR);
  float* s_m = smem;                                  // [kParts][G]
  float* s_l = s_m + kParts * G;                      // [kParts][G]
  float* s_acc = s_l + kParts * G;                    // [kParts][G][D]
  {
    const int part = wave * (kWave / LPR) + lane / LPR;
    if ((lane % LPR) < LPS) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (sub == 0) {
          s_m[part * G + g] = m[g];
          s_l[part * G + g] = l[g];
        }
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          float4 t;
          if constexpr (EPV == 8) {
            t = make_float4(acc[g][v * 8 + 0], acc[g][v * 8 + 1], acc[g][v * 8 + 2], acc[g][v * 8 + 3]);
            *reinterpret_cast<float4*>(&s_acc[(part * G + g) * D + (v * LPS + sub) * 8]) = t;
            t = make_float4(acc[g][v * 8 + 4], acc[g][v * 8 + 5], acc[g][v * 8 + 6], acc[g][v * 8 + 7]);
            *reinterpret_cast<float4*>(&s_acc[(part * G + g) * D + (v * LPS + sub) * 8 + 4]) = t;
          } else {
            t = make_float4(acc[g][v * 4 + 0], acc[g][v * 4 + 1], acc[g][v * 4 + 2], acc[g][v * 4 + 3]);
            *reinterpret_cast<float4*>(&s_acc[(part * G + g) * D + (v * LPS + sub) * 4]) = t;
          }
        }
      }
    }
  }
  __syncthreads();
  KK_TS(2);

  combine_and_finish<T, D, G, kParts, STEP, kWavesPerBlock>(p, s_m, s_l, s_acc, &s_last, unit, split, grow, len, t_old);
}

// ---------------------------------------------------------------------------------------------------
// bf16 caches: the same decode step with both contractions on the matrix cores (16x16x32 bf16 MFMA).
//
// A wavefront owns 32-slot tiles.  Their K and V rows go global -> LDS without passing through
// registers (rows XOR-swizzled in 16-byte chunks).  Scores are formed transposed, S^T = K Q^T: the A
// operand is the K tile (row = slot), the B operand the query heads (column = head, heads repeated
// to fill 16 columns), so lane (column c, quarter q) receives the logits of head c mod G for the
// slots 16 st + 4 q + i (st = 0, 1; i = 0..3).  That is already the layout of an A operand whose row
// is the head and whose contraction index runs over those 8 slots, so the probabilities feed the
// second product O = P V without leaving their lanes; its B operand, 8 slots of one channel per
// lane, is what the LDS transpose read (ds_read_b64_tr_b16) returns from the row-major V tile.
// P is split into two bf16 terms (hi + lo, 16 significant bits), V is bf16 already, accumulation f32.
// Output rows are heads again (row r = head r mod G), 16 channels per MFMA.
constexpr int kMTile = 32;
// Cache policy of the K / V row loads: every row is read once per launch, so the loads carry the non-temporal
// hint (the `nt` bit) and do not displace what the caches hold for reuse (a plain stream of 453 MB read this way
// measured 6.9 TB/s against 6.0 TB/s without the hint, and the small read-modify-write traffic of the EMA state
// beside it cost 1 us instead of 12).
constexpr int kStreamOnce = 2;
// Per wavefront, behind the tile buffers: the head group's query rows (whole 1 KB pieces, one asynchronous
// 16-byte copy per lane each) and the tile's votes and ln S (4 bytes per lane each); the tile loop stages its
// updated ln S here instead.
constexpr int mfma_stage_bytes(int D, int G) { return (G * D * 2 + 1023) / 1024 * 1024 + 3 * 256; }

// LDS reads that the compiler does not see as such.  It orders an LDS read that it cannot tell apart from an
// outstanding global -> LDS copy behind ALL outstanding copies; these are for data whose copy the caller has
// already awaited, while later copies (to other addresses) are still under way.  The wait for the read itself
// is part of the statement.
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
__device__ __forceinline__ i32x4_t lds_read_b128_awaited(const void* lds_ptr) {
  i32x4_t r;
  const uint32_t a = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)lds_ptr;
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(a) : "memory");
  return r;
}
__device__ __forceinline__ int lds_read_b32_awaited(const void* lds_ptr) {
  int r;
  const uint32_t a = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)lds_ptr;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(a) : "memory");
  return r;
}

typedef __attribute__((ext_vector_type(4))) short v4i16_t;

template <int G>
__device__ __forceinline__ float head_sum(float x) {   // sum over the G heads held by G consecutive lanes
  if constexpr (G >= 2) x += dpp_f32<0xB1>(x);          // quad_perm [1,0,3,2]
  if constexpr (G >= 4) x += dpp_f32<0x4E>(x);          // quad_perm [2,3,0,1]
  if constexpr (G >= 8) x += dpp_f32<0x141>(x);         // row_half_mirror
  return x;
}

__device__ __forceinline__ uint32_t pack_hi16(float lo_elem, float hi_elem) {   // {bf16 trunc(lo_elem), bf16 trunc(hi_elem)}
  return (__builtin_bit_cast(uint32_t, lo_elem) >> 16) | (__builtin_bit_cast(uint32_t, hi_elem) & 0xFFFF0000u);
}

// ONE: a split is at most one tile per wavefront (128 or 256 slots), so there is no tile loop, no prefetch and no
// rescaling of the accumulators (the common steady-state shape).
template <int D, int G, bool STEP, bool ONE, int kMfmaWaves>
__global__ __launch_bounds__(kMfmaWaves* kWave, 2) void decode_mfma_kernel(DecodeParams p) {
  using T = uint16_t;
  constexpr int ROWB = D * 2, CHUNKS = ROWB / 16, KS = D / 32, NTILE = D / 16;
  constexpr int TILE_BYTES = kMTile * ROWB;
  constexpr int LOADS = TILE_BYTES / (kWave * 16);
  constexpr int kParts = kMfmaWaves;
  extern __shared__ __align__(16) unsigned char smem_raw[];     // [wave][K tile | V tile]; later the deposit
  __shared__ int s_last;
  __shared__ __align__(16) unsigned char s_new[2 * ROWB];       // step mode: the appended token's K row, V row

  const int unit = blockIdx.x / p.nsplit, split = blockIdx.x % p.nsplit;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, q = lane >> 4;
  KK_TS(0);
  const int len_old = p.len[unit];
  const int t_old = STEP ? p.t_obs[unit] : 0;   // used at the very end only
  const int start = split * p.per;
  const bool takes_new = STEP && split == p.nsplit - 1 && wave == kMfmaWaves - 1;
  if (takes_new && lane < 2 * CHUNKS) {        // asynchronous copy of (k_t, v_t) into LDS, awaited after the loop
    const unsigned char* src = reinterpret_cast<const unsigned char*>(lane < CHUNKS ? p.k_t : p.v_t) +
                               (size_t)unit * ROWB + (lane % CHUNKS) * 16;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)s_new, 16, 0, 0);
  }
  const int bound = p.len_hint > 0 ? min(p.len_hint, p.capacity) : len_old;
  const int lim = min(bound, start + p.per);
  const size_t ubase = (size_t)unit * p.capacity;
  const unsigned char* kbytes = reinterpret_cast<const unsigned char*>(p.k) + ubase * ROWB;
  const unsigned char* vbytes = reinterpret_cast<const unsigned char*>(p.v) + ubase * ROWB;
  // ONE: [K tile | V tile] of the wavefront's single tile.  Otherwise the K rows travel straight into registers
  // (below) and the two buffers hold the V rows of the current and of the next tile.
  unsigned char* const Tb = smem_raw + wave * (2 * TILE_BYTES);
  unsigned char* const Kb = Tb;
  unsigned char* Vb = ONE ? Tb + TILE_BYTES : Tb;
  // ONE: everything this wavefront waits for travels as asynchronous global -> LDS copies, requested in the
  // order query rows, K rows, votes and EMA state, V rows.  Such copies complete in the order of issue, so a
  // wait that leaves the V rows' LOADS copies outstanding guarantees all the others: the score product and
  // the softmax run while the V rows still travel.  (Loads into registers in the same queue would make the
  // compiler wait for everything at their first use.)
  constexpr int Q_PIECES = (G * ROWB + 1023) / 1024;
  unsigned char* s_q = smem_raw + kMfmaWaves * 2 * TILE_BYTES + wave * mfma_stage_bytes(D, G);
  unsigned char* s_sc = s_q + Q_PIECES * 1024;                  // [votes | ln S][64] 4-byte words
  if constexpr (ONE) {
    const unsigned char* qbase = reinterpret_cast<const unsigned char*>(p.q) + (size_t)unit * G * ROWB;
#pragma unroll
    for (int j = 0; j < Q_PIECES; ++j) {
      const int c = min(j * kWave + lane, G * CHUNKS - 1);       // surplus lanes repeat the last chunk
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(qbase + c * 16),
                                       (__attribute__((address_space(3))) void*)(s_q + j * 1024), 16, 0, 0);
    }
  }

  // chunk c of row r of a tile sits at position c ^ (r mod CHUNKS); rows at or beyond `bound` are never read
  auto issue_rows = [&](const unsigned char* rows, unsigned char* buf, int tbase) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int c = lane + i * kWave;
      const int row = c / CHUNKS, phys = c % CHUNKS;
      const size_t off = (size_t)min(tbase + row, bound - 1) * ROWB + ((phys ^ (row & (CHUNKS - 1))) * 16);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(rows + off),
                                       (__attribute__((address_space(3))) void*)(buf + i * (kWave * 16)), 16, 0, kStreamOnce);
    }
  };
  // !ONE: the K rows of a tile are loaded in the layout of the score product's A operand (lane (l16, q): rows
  // l16 and 16 + l16 of the tile, chunk 4 ks + q of the row for k-step ks), one tile ahead, so a tile's K rows
  // pass through no LDS at all and a wavefront has a whole tile (K in registers, V on its way to the other LDS
  // buffer) in flight during all of the arithmetic on the current one.
  bf16x8_t kn[2][KS], kreg[2][KS];
  auto issue_k = [&](int tbase) {
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      const unsigned char* row = kbytes + (size_t)min(tbase + 16 * st + l16, bound - 1) * ROWB + q * 16;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kn[st][ks] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(row + ks * 64));
    }
  };
  int base = start + wave * kMTile;
  const int wave_lim = lim;
  constexpr int kTileStep = kMfmaWaves * kMTile;
  if (base < wave_lim) {
    if constexpr (ONE) issue_rows(kbytes, Kb, base);
    else issue_k(base);
    if constexpr (ONE) {                         // slot base + lane of the tile (lanes beyond the tile repeat a slot)
      const size_t at = ubase + min(base + lane, bound - 1);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(p.votes + at),
                                       (__attribute__((address_space(3))) void*)s_sc, 4, 0, 0);
      if constexpr (STEP)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(p.log_s + at),
                                         (__attribute__((address_space(3))) void*)(s_sc + 256), 4, 0, 0);
    }
    issue_rows(vbytes, Vb, base);
  }
  // !ONE: the votes and EMA state of a tile are requested one tile ahead, like its rows (into registers: they
  // are first used behind the loop's full wait)
  int pv_next = 1;      // votes of slot tbase + lane mod 32; log2 is taken once per slot and handed round by lane shuffles
  float ls_next = -INFINITY;
  auto request_scalars = [&](int tbase) {
    pv_next = p.votes[ubase + min(tbase + (lane & 31), bound - 1)];
    if constexpr (STEP) ls_next = p.log_s[ubase + min(tbase + 16 * (l16 >> 2) + 4 * q + (l16 & 3), bound - 1)];
  };
  if constexpr (!ONE) {
    if (base < wave_lim) request_scalars(base);
  }

  // B operand of the score product: column l16 is head l16 mod G, this lane's 8 channels of every k-step
  bf16x8_t qb[KS];
  auto read_q = [&]() {                          // ONE: from this wavefront's LDS copy, once it has landed
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qb[ks] = *reinterpret_cast<const bf16x8_t*>(s_q + (l16 % G) * ROWB + ks * 64 + q * 16);
  };
  if constexpr (!ONE) {
    const unsigned char* qrow = reinterpret_cast<const unsigned char*>(p.q) + ((size_t)unit * G + (l16 % G)) * ROWB;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qb[ks] = *reinterpret_cast<const bf16x8_t*>(qrow + ks * 64 + q * 16);
  }

  // Tile loop, step mode: the updated EMA state (ln S, n) of a split is collected in LDS (the staging area the
  // single-tile variant uses for queries and scalars) and written out by the whole workgroup once all tiles
  // are done, when it fits: many small stores spread over the streaming phase slow the row stream down more
  // than their bytes account for, one burst per workgroup less so.
  unsigned char* const s_stage = smem_raw + kMfmaWaves * 2 * TILE_BYTES;
  const bool staged = !ONE && STEP && (size_t)p.per * 4 <= (size_t)kMfmaWaves * mfma_stage_bytes(D, G);
  const float sl2 = p.scale * kLog2e;
  float m_run = -INFINITY, l_run = 0.f;
  f32x4_t O[NTILE];
#pragma unroll
  for (int nt = 0; nt < NTILE; ++nt) O[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  bool first = true;
  const int live_end = min(len_old, start + p.per);

  // One tile.  `extra`: the appended token alone (row 0 of the tile, copied from s_new).
  // `next`: the wavefront's next tile (or -1); its K rows are requested as soon as the score product has
  // consumed the K buffer, its V rows after the second product, so both travel during the arithmetic.
  // `v_in_flight`: the V rows are still outstanding when the call starts (ONE, the wavefront's own tile).
  auto compute = [&](int tbase, bool extra, int next, const float (&lp)[2][4], float ls_old,
                     bool v_in_flight) {
    const int n_live = extra ? 1 : max(0, min(kMTile, live_end - tbase));
    auto clear_masked_v = [&]() {
      if (n_live < kMTile) {                     // uniform: clear the V rows of masked slots (0 * garbage could be NaN)
        for (int c = n_live * CHUNKS + lane; c < kMTile * CHUNKS; c += kWave)
          *reinterpret_cast<uint4*>(Vb + c * 16) = make_uint4(0, 0, 0, 0);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    };
    if (!v_in_flight) clear_masked_v();
    if (!ONE && next >= 0) {
      // the next tile: K rows and scalars into registers, V rows into the other buffer (after the clearing
      // stores above: the compiler orders LDS stores behind outstanding copies into LDS)
      issue_k(next);
      request_scalars(next);
      issue_rows(vbytes, Tb + (Vb == Tb ? TILE_BYTES : 0), next);
    }
    // ---- S^T = K Q^T
    f32x4_t s[2] = {f32x4_t{0.f, 0.f, 0.f, 0.f}, f32x4_t{0.f, 0.f, 0.f, 0.f}};
    if constexpr (!ONE) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[0][ks], qb[ks], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[1][ks], qb[ks], s[1], 0, 0, 0);
      }
    } else if (v_in_flight) {
      // the K tile through reads that the compiler does not order behind the V rows' copies (see above)
      i32x4_t a0[KS], a1[KS];
      uint32_t ad[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        ad[ks] = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)(
            Kb + l16 * ROWB + (((4 * ks + q) ^ (l16 & (CHUNKS - 1))) * 16));
      if constexpr (KS == 4) {                   // D = 128: rows 16 .. 31 of the tile are 4096 bytes further
        static_assert(KS != 4 || 16 * ROWB == 4096, "offset in the statement below");
        asm volatile(
            "ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:4096\n\t"
            "ds_read_b128 %2, %9\n\tds_read_b128 %3, %9 offset:4096\n\t"
            "ds_read_b128 %4, %10\n\tds_read_b128 %5, %10 offset:4096\n\t"
            "ds_read_b128 %6, %11\n\tds_read_b128 %7, %11 offset:4096\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(a0[0]), "=&v"(a1[0]), "=&v"(a0[1]), "=&v"(a1[1]), "=&v"(a0[2]), "=&v"(a1[2]), "=&v"(a0[3]), "=&v"(a1[3])
            : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3])
            : "memory");
      } else {                                   // D = 64: 2048 bytes further
        static_assert(KS == 4 || (KS == 2 && 16 * ROWB == 2048), "offset in the statement below");
        asm volatile(
            "ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:2048\n\t"
            "ds_read_b128 %2, %5\n\tds_read_b128 %3, %5 offset:2048\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(a0[0]), "=&v"(a1[0]), "=&v"(a0[1]), "=&v"(a1[1])
            : "v"(ad[0]), "v"(ad[1])
            : "memory");
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a0[ks]), qb[ks], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a1[ks]), qb[ks], s[1], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = l16 * ROWB + (((4 * ks + q) ^ (l16 & (CHUNKS - 1))) * 16);
        const bf16x8_t a0 = *reinterpret_cast<const bf16x8_t*>(Kb + off);
        const bf16x8_t a1 = *reinterpret_cast<const bf16x8_t*>(Kb + off + 16 * ROWB);
        s[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qb[ks], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qb[ks], s[1], 0, 0, 0);
      }
    }
    // ---- logits (log2 domain, log2(votes) folded in), group-mean logit for the EMA
    float z[2][4], xm[2][4];
    float tm = -INFINITY;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool live = (16 * st + 4 * q + i) < n_live;
        z[st][i] = live ? fmaf(s[st][i], sl2, lp[st][i]) : -INFINITY;
        tm = fmaxf(tm, z[st][i]);
        xm[st][i] = head_sum<G>(s[st][i]) * (p.scale * (1.0f / G));
      }
    tm = fmaxf(tm, __shfl_xor(tm, 16));
    tm = fmaxf(tm, __shfl_xor(tm, 32));
    const float mn = fmaxf(m_run, tm);
    const float c = (m_run == -INFINITY) ? 0.f : fast_exp2(m_run - mn);
    float pr[2][4], ps = 0.f;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pr[st][i] = (mn == -INFINITY) ? 0.f : fast_exp2(z[st][i] - mn);
        ps += pr[st][i];
      }
    l_run = fmaf(l_run, c, ps);
    m_run = mn;
    if (!first) {                                // uniform: rescale the accumulators, row r = head r mod G
                                                 // (with ONE only the extra tile of the appended token gets here)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float ci = __shfl(c, (lane & 48) | ((4 * q + i) % G));
#pragma unroll
        for (int nt = 0; nt < NTILE; ++nt) O[nt][i] *= ci;
      }
    }
    first = false;
    if (v_in_flight) {                           // before any store is issued: only the V rows are outstanding
      // (tied to the softmax sum, so that the wait is not scheduled ahead of the arithmetic it is meant to hide)
      asm volatile("s_waitcnt vmcnt(0)" : "+v"(l_run) : : "memory");
      clear_masked_v();
    }
    // ---- O += P V with P = hi + lo in bf16
    uint4 ah, al;
    {
      float lo_[2][4];
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          lo_[st][i] = pr[st][i] - __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, pr[st][i]) & 0xFFFF0000u);
      ah = make_uint4(pack_hi16(pr[0][0], pr[0][1]), pack_hi16(pr[0][2], pr[0][3]), pack_hi16(pr[1][0], pr[1][1]),
                      pack_hi16(pr[1][2], pr[1][3]));
      al = make_uint4(pack_hi16(lo_[0][0], lo_[0][1]), pack_hi16(lo_[0][2], lo_[0][3]), pack_hi16(lo_[1][0], lo_[1][1]),
                      pack_hi16(lo_[1][2], lo_[1][3]));
    }
    const bf16x8_t a_hi = __builtin_bit_cast(bf16x8_t, ah), a_lo = __builtin_bit_cast(bf16x8_t, al);
    // transpose read: lane s of a 16-lane block supplies the address of row s / 4, columns 4 (s mod 4) .. + 3, and
    // receives column s of the block's four rows
    // The V tile has landed (awaited above or at the top of the loop) while the next tile's K rows may be on
    // their way: the reads go through a statement the compiler does not order behind those copies.
    const int vrow = 4 * q + (l16 >> 2);
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
    u32x2_t b0[NTILE], b1[NTILE];
    uint32_t va[NTILE];
#pragma unroll
    for (int nt = 0; nt < NTILE; ++nt) {
      const int chunk = 2 * nt + ((l16 & 3) >> 1);
      va[nt] = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)(
          Vb + vrow * ROWB + ((chunk ^ (vrow & (CHUNKS - 1))) * 16) + (l16 & 1) * 8);
    }
    if constexpr (NTILE == 8) {                  // D = 128: rows 16 .. 31 of the tile are 4096 bytes further
      static_assert(NTILE != 8 || 16 * ROWB == 4096, "offset in the statement below");
      asm volatile(
          "ds_read_b64_tr_b16 %0, %16\n\tds_read_b64_tr_b16 %1, %16 offset:4096\n\t"
          "ds_read_b64_tr_b16 %2, %17\n\tds_read_b64_tr_b16 %3, %17 offset:4096\n\t"
          "ds_read_b64_tr_b16 %4, %18\n\tds_read_b64_tr_b16 %5, %18 offset:4096\n\t"
          "ds_read_b64_tr_b16 %6, %19\n\tds_read_b64_tr_b16 %7, %19 offset:4096\n\t"
          "ds_read_b64_tr_b16 %8, %20\n\tds_read_b64_tr_b16 %9, %20 offset:4096\n\t"
          "ds_read_b64_tr_b16 %10, %21\n\tds_read_b64_tr_b16 %11, %21 offset:4096\n\t"
          "ds_read_b64_tr_b16 %12, %22\n\tds_read_b64_tr_b16 %13, %22 offset:4096\n\t"
          "ds_read_b64_tr_b16 %14, %23\n\tds_read_b64_tr_b16 %15, %23 offset:4096\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(b0[0]), "=&v"(b1[0]), "=&v"(b0[1]), "=&v"(b1[1]), "=&v"(b0[2]), "=&v"(b1[2]), "=&v"(b0[3]), "=&v"(b1[3]),
            "=&v"(b0[4]), "=&v"(b1[4]), "=&v"(b0[5]), "=&v"(b1[5]), "=&v"(b0[6]), "=&v"(b1[6]), "=&v"(b0[7]), "=&v"(b1[7])
          : "v"(va[0]), "v"(va[1]), "v"(va[2]), "v"(va[3]), "v"(va[4]), "v"(va[5]), "v"(va[6]), "v"(va[7])
          : "memory");
    } else {                                     // D = 64: 2048 bytes further
      static_assert(NTILE == 8 || (NTILE == 4 && 16 * ROWB == 2048), "offset in the statement below");
      asm volatile(
          "ds_read_b64_tr_b16 %0, %8\n\tds_read_b64_tr_b16 %1, %8 offset:2048\n\t"
          "ds_read_b64_tr_b16 %2, %9\n\tds_read_b64_tr_b16 %3, %9 offset:2048\n\t"
          "ds_read_b64_tr_b16 %4, %10\n\tds_read_b64_tr_b16 %5, %10 offset:2048\n\t"
          "ds_read_b64_tr_b16 %6, %11\n\tds_read_b64_tr_b16 %7, %11 offset:2048\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(b0[0]), "=&v"(b1[0]), "=&v"(b0[1]), "=&v"(b1[1]), "=&v"(b0[2]), "=&v"(b1[2]), "=&v"(b0[3]), "=&v"(b1[3])
          : "v"(va[0]), "v"(va[1]), "v"(va[2]), "v"(va[3])
          : "memory");
    }
#pragma unroll
    for (int nt = 0; nt < NTILE; ++nt) {
      const uint4 bw = make_uint4(b0[nt][0], b0[nt][1], b1[nt][0], b1[nt][1]);
      const bf16x8_t b = __builtin_bit_cast(bf16x8_t, bw);
      O[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, b, O[nt], 0, 0, 0);
      O[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, b, O[nt], 0, 0, 0);
    }
    // ---- EMA update (Eq. 8) and optional logit output: lane (l16 < 8, q) owns slot 16 (l16 / 4) + 4 q + l16 % 4.
    // After the second product: the compiler orders the V reads behind every outstanding memory operation,
    // and stores issued before them would be waited for.
    {
      float x = xm[0][0];
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int i = 0; i < 4; ++i) x = (l16 == 4 * st + i) ? xm[st][i] : x;
      const int row_mine = 16 * (l16 >> 2) + 4 * q + (l16 & 3);
      const bool mine = l16 < 8 && row_mine < n_live;
      const size_t at = ubase + (extra ? len_old : tbase + row_mine);
      if (p.logits_out != nullptr && mine) p.logits_out[at] = x;
      if constexpr (STEP) {
        const float a = p.ln_alpha + ls_old, b = p.ln_1m_alpha + x;
        const float hi = fmaxf(a, b), lo = fminf(a, b);
        // ln(e^hi + e^lo) = hi + ln(1 + e^(lo - hi)) with the hardware exp2 / log2 (absolute error ~1e-7)
        const float r = (lo == -INFINITY) ? hi : hi + kLn2 * fast_log2(1.f + fast_exp2((lo - hi) * kLog2e));
        if (mine) {
          if (staged && !extra) {
            // (a statement the compiler does not see as an LDS store: it would order one behind the next
            // tile's outstanding copies into LDS)
            const uint32_t sa = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)(
                s_stage + (size_t)(tbase - start + row_mine) * 4);
            asm volatile("ds_write_b32 %0, %1" : : "v"(sa), "v"(r) : "memory");
          } else {
            p.log_s[at] = r;
          }
        }
      }
    }
  };

  while (base < wave_lim) {                      // a single pass with ONE
    float lp[2][4];                                // log2(votes) of the slots whose logits this lane holds
    float ls_old = -INFINITY;
    if constexpr (ONE) {
      // all copies but the youngest LOADS (the V rows) have landed: query rows, K rows, votes and EMA state
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
      read_q();
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        const i32x4_t x = lds_read_b128_awaited(s_sc + (16 * st + 4 * q) * 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) lp[st][i] = fast_log2((float)x[i]);
      }
      if constexpr (STEP) {
        const int mine = 16 * (l16 >> 2) + 4 * q + (l16 & 3);
        ls_old = __builtin_bit_cast(float, lds_read_b32_awaited(s_sc + 256 + mine * 4));
      }
      compute(base, false, -1, lp, ls_old, true);
      base = lim;
    } else {
      // the tile's K rows (registers), V rows (LDS) and scalars have landed; the K registers pass through the
      // statement so that no use of them is scheduled ahead of the wait
      if constexpr (KS == 4)
        asm volatile("s_waitcnt vmcnt(0)"
                     : "+v"(kn[0][0]), "+v"(kn[0][1]), "+v"(kn[0][2]), "+v"(kn[0][3]), "+v"(kn[1][0]), "+v"(kn[1][1]),
                       "+v"(kn[1][2]), "+v"(kn[1][3])
                     :
                     : "memory");
      else
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(kn[0][0]), "+v"(kn[0][1]), "+v"(kn[1][0]), "+v"(kn[1][1]) : : "memory");
#pragma unroll
      for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[st][ks] = kn[st][ks];
      }
      {
        const float lp_lane = fast_log2((float)pv_next);
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int i = 0; i < 4; ++i) lp[st][i] = __shfl(lp_lane, 16 * st + 4 * q + i);
      }
      ls_old = ls_next;
      const int next = base + kTileStep;
      compute(base, false, next < wave_lim ? next : -1, lp, ls_old, false);
      Vb = Tb + (Vb == Tb ? TILE_BYTES : 0);
      base = next;
    }
  }
  KK_TS(1);
  const bool grow = STEP && len_old < p.capacity;
  const int len = grow ? len_old + 1 : len_old;
  if (takes_new) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // the copy of the new token has landed
    if constexpr (ONE) read_q();                 // (a wavefront without a tile of its own has not read them yet)
    if (grow) {
      if constexpr (!ONE) {                      // the K operand of a tile whose row 0 is the new key, zero elsewhere
        Vb = Tb;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const uint4 x = *reinterpret_cast<const uint4*>(s_new + (4 * ks + q) * 16);
          const uint4 z4 = make_uint4(0, 0, 0, 0);
          kreg[0][ks] = __builtin_bit_cast(bf16x8_t, l16 == 0 ? x : z4);
          kreg[1][ks] = __builtin_bit_cast(bf16x8_t, z4);
        }
      }
      if (lane < 2 * CHUNKS) {
        const uint4 x = *reinterpret_cast<const uint4*>(s_new + lane * 16);
        // row 0 of the tile (its swizzle is the identity) and the cache row of the new slot
        if (ONE || lane >= CHUNKS) *reinterpret_cast<uint4*>((lane < CHUNKS ? Kb : Vb) + (lane % CHUNKS) * 16) = x;
        unsigned char* dst = reinterpret_cast<unsigned char*>(lane < CHUNKS ? p.k : p.v) + (ubase + len_old) * ROWB;
        *reinterpret_cast<uint4*>(dst + (lane % CHUNKS) * 16) = x;
      }
      if (lane == 0) {
        p.votes[ubase + len_old] = 1;
        p.born[ubase + len_old] = t_old;          // first observed in this step
      }
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
      __builtin_amdgcn_wave_barrier();
      const float one[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};   // one vote: log2 = 0
      compute(0, true, -1, one, -INFINITY, false);
    }
  }

  // ---- deposit this wavefront's state; the workgroup reduces kParts of them -------------------------
  float l_tot = l_run + __shfl_xor(l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  if constexpr (!ONE && STEP) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the staged EMA state is in LDS
  __syncthreads();                               // every wavefront is done with its tile buffers
  if constexpr (!ONE && STEP) {
    if (staged) {                                // the split's updated EMA state, slot by slot
      for (int j = threadIdx.x; j < live_end - start; j += kMfmaWaves * kWave) {
        // (write-through: measured faster at batch 128 than leaving megabytes of dirty lines to the caches)
        __hip_atomic_store(&p.log_s[ubase + start + j], *reinterpret_cast<const float*>(s_stage + (size_t)j * 4),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  float* s_m = reinterpret_cast<float*>(smem_raw);     // [kParts][G]
  float* s_l = s_m + kParts * G;                       // [kParts][G]
  float* s_acc = s_l + kParts * G;                     // [kParts][G][D]
  if (q == 0 && l16 < G) {
    s_m[wave * G + l16] = m_run;
    s_l[wave * G + l16] = l_tot;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int head = 4 * q + i;                  // output row; rows >= G repeat heads
    if (head < G) {
#pragma unroll
      for (int nt = 0; nt < NTILE; ++nt) s_acc[(wave * G + head) * D + 16 * nt + l16] = O[nt][i];
    }
  }
  __syncthreads();
  KK_TS(2);
  combine_and_finish<T, D, G, kParts, STEP, kMfmaWaves>(p, s_m, s_l, s_acc, &s_last, unit, split, grow, len, t_old);
}

template <typename T, int D, int G>
keepkv_status launch_decode(const DecodeParams& p, int units, bool step, bool valu, hipStream_t st) {
  // 8 lanes per slot (16 channels each at D = 128 bf16) halves the cross-lane reduction work; the
  // widest group keeps 16 lanes per slot so that its accumulators still fit two waves per SIMD.
  constexpr int RV = D * (int)sizeof(T) / 16;                       // 16-byte vectors per row
  constexpr int LPS = (G >= 8 && RV >= 16) ? RV / (RV >= 32 ? 2 : 1) : (RV >= 32 ? 16 : 8);
  constexpr int U = 4;
  const dim3 grid(units * p.nsplit), block(kWavesPerBlock * kWave);
  if constexpr (sizeof(T) == 2) {
    if (!valu) {
      auto go = [&](auto waves_tag) -> keepkv_status {
        constexpr int WV = decltype(waves_tag)::value;
        constexpr size_t tiles = (size_t)WV * 2 * kMTile * D * 2 + (size_t)WV * mfma_stage_bytes(D, G);
        // 64 or 128 KB of tile buffers at D = 128, the per-wavefront staging of queries and scalars, plus the
        // kernel's static LDS: allow it explicitly (once per process and instance)
        static const bool allowed =
            hipFuncSetAttribute((const void*)decode_mfma_kernel<D, G, true, true, WV>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)tiles) == hipSuccess &&
            hipFuncSetAttribute((const void*)decode_mfma_kernel<D, G, true, false, WV>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)tiles) == hipSuccess &&
            hipFuncSetAttribute((const void*)decode_mfma_kernel<D, G, false, true, WV>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)tiles) == hipSuccess &&
            hipFuncSetAttribute((const void*)decode_mfma_kernel<D, G, false, false, WV>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)tiles) == hipSuccess;
        if (!allowed) return KEEPKV_ERR_DEVICE;
        const dim3 mblock(WV * kWave);
        const bool one = p.per <= WV * kMTile;
        if (step && one) decode_mfma_kernel<D, G, true, true, WV><<<grid, mblock, tiles, st>>>(p);
        else if (step) decode_mfma_kernel<D, G, true, false, WV><<<grid, mblock, tiles, st>>>(p);
        else if (one) decode_mfma_kernel<D, G, false, true, WV><<<grid, mblock, tiles, st>>>(p);
        else decode_mfma_kernel<D, G, false, false, WV><<<grid, mblock, tiles, st>>>(p);
        return KEEPKV_OK;
      };
      if (p.waves == 8) return go(std::integral_constant<int, 8>{});
      return go(std::integral_constant<int, 4>{});
    }
  }
  constexpr int parts = kWavesPerBlock * (kWave / (LPS < 16 ? 16 : LPS));
  constexpr size_t smem = (size_t)parts * G * (D + 2) * sizeof(float);
  if constexpr (smem > 64 * 1024) {
    static const bool allowed =
        hipFuncSetAttribute((const void*)decode_attn_kernel<T, D, G, LPS, U, true>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess &&
        hipFuncSetAttribute((const void*)decode_attn_kernel<T, D, G, LPS, U, false>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    if (!allowed) return KEEPKV_ERR_DEVICE;
  }
  if (step) decode_attn_kernel<T, D, G, LPS, U, true><<<grid, block, smem, st>>>(p);
  else decode_attn_kernel<T, D, G, LPS, U, false><<<grid, block, smem, st>>>(p);
  return KEEPKV_OK;
}

template <typename T, int D>
keepkv_status dispatch_g(const DecodeParams& p, int units, int G, bool step, bool valu, hipStream_t st) {
  switch (G) {
    case 1: return launch_decode<T, D, 1>(p, units, step, valu, st);
    case 2: return launch_decode<T, D, 2>(p, units, step, valu, st);
    case 4: return launch_decode<T, D, 4>(p, units, step, valu, st);
    default: return launch_decode<T, D, 8>(p, units, step, valu, st);
  }
}

keepkv_status run_decode(const keepkv_layout* layout, const keepkv_cache* cache, const void* q, const void* k_t,
                         const void* v_t, void* out, float* logits_out, float* lse_out, float alpha, int32_t* overflow,
                         bool step, void* workspace, size_t workspace_bytes, void* stream) {
  if (!layout_ok(layout) || !cache_ok(cache) || !q || !out) return KEEPKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(out) || !aligned16(cache->k) || !aligned16(cache->v)) return KEEPKV_ERR_INVALID_ARG;
  if (step && (!k_t || !v_t || !aligned16(k_t) || !aligned16(v_t) || !(alpha >= 0.f && alpha < 1.f)))
    return KEEPKV_ERR_INVALID_ARG;
  if (!layout_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  const int units = layout->batch * layout->n_kv_heads;
  if (units > kMaxUnits) return KEEPKV_ERR_UNSUPPORTED;
  const int fw = cache->plan_wavefronts, fp = cache->plan_slots_per_split;
  if (!(fw == 0 || fw == 4 || fw == 8 || fw == -1) || fp < 0 || (fp > 0 && fp < 64)) return KEEPKV_ERR_INVALID_ARG;
  const DecodePlan pl = plan_decode(layout, cache->capacity, fp, fw);
  if (pl.nsplit > 1 && (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace))) return KEEPKV_ERR_WORKSPACE;

  DecodeParams p;
  p.q = q; p.k = cache->k; p.v = cache->v; p.votes = cache->votes; p.log_s = cache->log_s; p.born = cache->born; p.t_obs = cache->t_obs;
  p.len = cache->len; p.k_t = k_t; p.v_t = v_t; p.overflow = overflow;
  p.out = out; p.logits_out = logits_out; p.lse_out = lse_out;
  p.partial = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + pl.partial_off);
  p.ticket = reinterpret_cast<int32_t*>(workspace);
  p.n_kv_heads = layout->n_kv_heads; p.capacity = cache->capacity; p.nsplit = pl.nsplit; p.per = pl.per; p.waves = pl.waves; p.scale = layout->scale;
  p.len_hint = cache->len_hint > 0 ? cache->len_hint : 0;
  p.ln_alpha = (step && alpha > 0.f) ? logf(alpha) : -INFINITY;
  p.ln_1m_alpha = step ? log1pf(-alpha) : 0.f;

  const int G = layout->n_q_heads / layout->n_kv_heads;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  keepkv_status rc;
  if (layout->dtype == KEEPKV_BF16) {
    if (layout->head_dim == 128) rc = dispatch_g<uint16_t, 128>(p, units, G, step, pl.valu, st);
    else rc = dispatch_g<uint16_t, 64>(p, units, G, step, pl.valu, st);
  } else {
    if (layout->head_dim == 128) rc = dispatch_g<float, 128>(p, units, G, step, false, st);
    else rc = dispatch_g<float, 64>(p, units, G, step, false, st);
  }
  if (rc != KEEPKV_OK) return rc;
  return launch_status();
}

// ---- scratch for the entry point that takes no workspace --------------------------------------------------
// One array per GPU, held by the code object until the process ends.  In host code `scratch` is only a handle:
// the device address comes from hipGetSymbolAddress, once per device with that device current, and that address
// is what kernels receive.
constexpr size_t kStaticPartialBytes = (size_t)4 << 20;
constexpr size_t kStaticScratchBytes = kWorkspaceHead + kStaticPartialBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];     // per device, filled on the first call there
std::mutex g_scratch_mutex;

__global__ void clear_words_kernel(int32_t* w, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) w[i] = 0;
}

keepkv_status static_scratch(void** out, hipStream_t st) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KEEPKV_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return KEEPKV_ERR_DEVICE;
    // The control words (split tickets) must be zero when a call starts.  Every launch leaves them zero, so
    // they are cleared once, ahead of the first launch on this device (a kernel: it may be captured).
    const int n = (int)(kWorkspaceHead / sizeof(int32_t));
    clear_words_kernel<<<(n + 255) / 256, 256, 0, st>>>(reinterpret_cast<int32_t*>(ptr), n);
    if (hipGetLastError() != hipSuccess) return KEEPKV_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return KEEPKV_OK;
}

}  // namespace

DecodePlan plan_decode(const keepkv_layout* L, int capacity, int force_per, int force_waves) {
  // Slots per split, and for the matrix-core kernel its workgroup size, from a small cost model fitted to
  // measurements on MI355X (batch 1..128, 850..32768 slots per head).  Workgroups of 4 wavefronts fit two to
  // a compute unit (512 resident), those of 8 wavefronts one (128 KB of tile buffers at D = 128: 256
  // resident; 512 at D = 64).  Every round of workgroups costs ~3 us of start-up.  A wavefront streams at no
  // more than ~6.5 GB/s when all its tiles are requested at once and ~4.4 GB/s when it loops (its rows in
  // flight over the memory latency); all resident workgroups together reach ~5.1 TB/s when the chip is
  // full, and a compute unit with two workgroups beside one with a single one sets the pace.  The last
  // workgroup of a head combines the splits eight or sixteen at a time, ~2.3 / ~3.4 us per round trip of
  // device-scope loads.  Few long splits starve the chip, many short ones pay for rounds and for the
  // combine.  On the Llama-3-8B shape (64 heads, ~850 slots) 4 splits of 8 wavefronts are exactly one
  // workgroup per compute unit: 11.2 us against 11.9 us for 7 splits of 4 wavefronts (448 workgroups on 256
  // compute units); at 128 heads and more the smaller workgroups win (two rounds instead of four at batch 128).
  DecodePlan pl;
  const double units = (double)L->batch * L->n_kv_heads;
  const double slot_bytes = 2.0 * L->head_dim * (L->dtype == KEEPKV_BF16 ? 2 : 4) + 24.0;
  const bool valu = L->dtype == KEEPKV_BF16 && force_waves == -1;
  const bool mfma = L->dtype == KEEPKV_BF16 && !valu;
  const int rv = L->head_dim * (L->dtype == KEEPKV_BF16 ? 2 : 4) / 16;
  long per = 128;
  int waves = kWavesPerBlock;
  double best = 1e300;
  for (int wv = 4; wv <= (mfma ? 8 : 4); wv += 4) {
    // a split is a whole number of `unit_slots`; a workgroup consumes `granule` slots per loop iteration
    const long unit_slots = mfma ? kMTile : 64;
    const long granule = mfma ? (long)wv * kMTile : (L->dtype == KEEPKV_BF16 ? 128 : (rv >= 32 ? 64 : 128));
    const double res_max = (mfma && (size_t)wv * 2 * kMTile * L->head_dim * 2 > 72 * 1024) ? 256.0 : 512.0;
    const long max_ns = (capacity + unit_slots - 1) / unit_slots < 1024 ? (capacity + unit_slots - 1) / unit_slots : 1024;
    for (long ns = 1; ns <= max_ns; ++ns) {
      const long cand = ((capacity + ns - 1) / ns + unit_slots - 1) / unit_slots * unit_slots;
      const double n_split = (double)((capacity + cand - 1) / cand);
      const double wgs = units * n_split;
      const double resident = wgs < res_max ? wgs : res_max;
      const double rounds = (double)(long)((wgs + res_max - 1.0) / res_max);
      const double wg_rate = (cand <= granule ? 6.5 : 4.4) * wv;                        // GB/s
      double together = 5100.0 * pow(resident / res_max, 0.15);                         // GB/s, all resident workgroups
      if (resident > 256.0) together *= (resident / 256.0) / (double)(long)((resident + 255.0) / 256.0);
      if (together > wg_rate * resident) together = wg_rate * resident;
      const double streamed = (double)((cand + granule - 1) / granule * granule);       // whole iterations
      const double t_one = streamed * slot_bytes / (wg_rate * 1e3);                     // us, a workgroup alone
      const double t_all = units * capacity * slot_bytes / rounds / (together * 1e3);   // us, one round of them
      const double t_stream = rounds * (3.0 + (t_one > t_all ? t_one : t_all));
      const double t_trips = n_split <= 8.0 ? 2.3 : 3.4 * (double)(long)((n_split + 15.0) / 16.0);
      const double t_combine = n_split > 1.0 ? 1.0 + t_trips + 0.02 * n_split : 0.0;
      if (t_stream + t_combine < best) {
        best = t_stream + t_combine;
        per = cand;
        waves = wv;
      }
    }
  }
  if (mfma && (force_waves == 4 || force_waves == 8)) waves = force_waves;
  pl.waves = waves;
  pl.valu = valu;
  if (force_per >= 64) per = mfma ? force_per / 32 * 32 : force_per / 64 * 64;
  long ns = (capacity + per - 1) / per;
  if (ns > 1024) { ns = 1024; per = ((capacity + ns - 1) / ns + 63) / 64 * 64; ns = (capacity + per - 1) / per; }   // (max_ns caps it already)
  pl.nsplit = (int)ns;
  pl.per = (int)per;
  pl.partial_off = kWorkspaceHead;
  pl.bytes = kWorkspaceHead + align_up((size_t)L->batch * L->n_q_heads * ns * (L->head_dim + 2) * sizeof(float), 256);
  return pl;
}

}  // namespace kk

extern "C" keepkv_status keepkv_decode_attn(const keepkv_layout* layout, const keepkv_cache* cache,
                                            const void* q, void* out, float* logits_out, float* lse_out,
                                            void* workspace, size_t workspace_bytes, void* stream) {
  return kk::run_decode(layout, cache, q, nullptr, nullptr, out, logits_out, lse_out, 0.f, nullptr, false, workspace,
                        workspace_bytes, stream);
}

extern "C" keepkv_status keepkv_decode_step(const keepkv_layout* layout, keepkv_cache* cache, const void* q,
                                            const void* k_t, const void* v_t, void* out, float* logits_out,
                                            float alpha, int32_t* overflow, void* workspace, size_t workspace_bytes,
                                            void* stream) {
  return kk::run_decode(layout, cache, q, k_t, v_t, out, logits_out, nullptr, alpha, overflow, true, workspace,
                        workspace_bytes, stream);
}

extern "C" keepkv_status keepkv_decode_step_static(const keepkv_layout* layout, keepkv_cache* cache, const void* q,
                                                   const void* k_t, const void* v_t, void* out, float* logits_out,
                                                   float alpha, int32_t* overflow, void* stream) {
  using namespace kk;
  // validate first (nothing is launched, not even the one-time clear, on bad arguments), then size
  if (!layout_ok(layout) || !cache_ok(cache) || !q || !out || !k_t || !v_t) return KEEPKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(out) || !aligned16(cache->k) || !aligned16(cache->v) || !aligned16(k_t) ||
      !aligned16(v_t) || !(alpha >= 0.f && alpha < 1.f))
    return KEEPKV_ERR_INVALID_ARG;
  if (!layout_supported(layout) || !units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  const int fw = cache->plan_wavefronts, fp = cache->plan_slots_per_split;
  if (!(fw == 0 || fw == 4 || fw == 8 || fw == -1) || fp < 0 || (fp > 0 && fp < 64)) return KEEPKV_ERR_INVALID_ARG;
  const DecodePlan pl = plan_decode(layout, cache->capacity, fp, fw);
  if (pl.nsplit > 1 && pl.bytes > kStaticScratchBytes) return KEEPKV_ERR_UNSUPPORTED;   // partials beyond the static array
  void* ptr = nullptr;
  const keepkv_status rc = static_scratch(&ptr, reinterpret_cast<hipStream_t>(stream));
  if (rc != KEEPKV_OK) return rc;
  return run_decode(layout, cache, q, k_t, v_t, out, logits_out, nullptr, alpha, overflow, true, ptr,
                    kStaticScratchBytes, stream);
}

#ifdef KEEPKV_TRACE
extern "C" int keepkv_trace_read(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(kk::kk_trace), sizeof(long long) * n);
}
#endif
