// keepkv_decode_attn: vote-weighted flash-decode attention (Eq. 6) with split-K over slots.
//
// One workgroup (4 wavefronts) handles one (batch, kv head, split).  A slot's row (D elements)
// is spread over LPS consecutive lanes, 16 bytes per lane, so one wavefront load instruction
// streams 64/LPS whole rows, fully coalesced.  Each lane group computes the G logits of its
// slot with bf16 dot2 (or f32 fma) plus a DPP all-reduce inside the group, keeps its own
// online-softmax state in the log2 domain with log2(votes) folded into the logit, and
// accumulates p * v for its 16-byte slice of V.  Groups, wavefronts and splits are combined
// at the end (LDS, then a small second kernel when nsplit > 1).
#include "kk_common.hpp"

namespace kk {

namespace {

struct DecodeParams {
  const void* q;
  const void* k;
  const void* v;
  const int32_t* votes;
  const int32_t* len;
  void* out;
  float* logits_out;
  float* lse_out;
  float* partial;   // [B*Hq, nsplit, D + 2]
  int n_kv_heads;
  int capacity;
  int nsplit;
  float scale;
};

constexpr int kWavesPerBlock = 4;
constexpr int kUnroll = 4;  // slots per lane group per tile

template <typename T>
struct Vec16 {  // 16 bytes of a row as held by one lane
  uint4 raw;
};

template <typename T, int D, int G>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void decode_attn_kernel(DecodeParams p) {
  constexpr int EPL = 16 / (int)sizeof(T);   // elements per lane
  constexpr int LPS = D / EPL;               // lanes per slot
  constexpr int GPW = kWave / LPS;           // slots per load instruction
  constexpr int TILE = GPW * kUnroll;        // slots per wavefront per iteration
  constexpr bool kBf16 = sizeof(T) == 2;

  const int unit = blockIdx.x / p.nsplit;    // b * Hkv + h
  const int split = blockIdx.x % p.nsplit;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPS, sub = lane % LPS;
  const int b = unit / p.n_kv_heads, h = unit % p.n_kv_heads;
  const int len = p.len[unit];
  const int per = (((len + p.nsplit - 1) / p.nsplit) + 63) & ~63;
  const int start = split * per;
  const int end = min(len, start + per);

  // query slice of this lane for each head of the group
  uint4 qv[G];
  {
    const size_t qrow = ((size_t)b * p.n_kv_heads + h) * G;
#pragma unroll
    for (int g = 0; g < G; ++g)
      qv[g] = reinterpret_cast<const uint4*>(p.q)[(qrow + g) * LPS + sub];
  }

  float m[G], l[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  const uint4* kbase = reinterpret_cast<const uint4*>(p.k) + (size_t)unit * p.capacity * LPS;
  const uint4* vbase = reinterpret_cast<const uint4*>(p.v) + (size_t)unit * p.capacity * LPS;
  const int32_t* votes = p.votes + (size_t)unit * p.capacity;
  const float sl2 = p.scale * kLog2e;

  for (int base = start + wave * TILE; base < end; base += kWavesPerBlock * TILE) {
    const int s0 = base + grp * kUnroll;
    uint4 kk_[kUnroll], vv_[kUnroll];
    int pv[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const int s = min(s0 + j, len - 1);      // clamp: dead slots are never read
      kk_[j] = kbase[(size_t)s * LPS + sub];
      vv_[j] = vbase[(size_t)s * LPS + sub];
      pv[j] = votes[s];
    }

    float z[G][kUnroll];
    float mean_logit[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const bool live = (s0 + j) < end;
      const float lp = fast_log2((float)pv[j]);
      float sum = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d;
        if constexpr (kBf16) {
          d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kk_[j].x), __builtin_bit_cast(bf16x2_t, qv[g].x), 0.f, false);
          d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kk_[j].y), __builtin_bit_cast(bf16x2_t, qv[g].y), d, false);
          d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kk_[j].z), __builtin_bit_cast(bf16x2_t, qv[g].z), d, false);
          d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kk_[j].w), __builtin_bit_cast(bf16x2_t, qv[g].w), d, false);
        } else {
          d = __builtin_bit_cast(float, kk_[j].x) * __builtin_bit_cast(float, qv[g].x);
          d = fmaf(__builtin_bit_cast(float, kk_[j].y), __builtin_bit_cast(float, qv[g].y), d);
          d = fmaf(__builtin_bit_cast(float, kk_[j].z), __builtin_bit_cast(float, qv[g].z), d);
          d = fmaf(__builtin_bit_cast(float, kk_[j].w), __builtin_bit_cast(float, qv[g].w), d);
        }
        d = group_sum<LPS>(d);
        sum += d;
        z[g][j] = live ? fmaf(d, sl2, lp) : -INFINITY;
      }
      mean_logit[j] = sum * (p.scale * (1.0f / G));
    }

    if (p.logits_out != nullptr && sub < kUnroll) {
      float x = mean_logit[0];
#pragma unroll
      for (int j = 1; j < kUnroll; ++j) x = (sub == j) ? mean_logit[j] : x;
      if (s0 + sub < end) p.logits_out[(size_t)unit * p.capacity + s0 + sub] = x;
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
      if constexpr (kBf16) {
        vf[0] = bf16_lo(vv_[j].x); vf[1] = bf16_hi(vv_[j].x);
        vf[2] = bf16_lo(vv_[j].y); vf[3] = bf16_hi(vv_[j].y);
        vf[4] = bf16_lo(vv_[j].z); vf[5] = bf16_hi(vv_[j].z);
        vf[6] = bf16_lo(vv_[j].w); vf[7] = bf16_hi(vv_[j].w);
      } else {
        vf[0] = __builtin_bit_cast(float, vv_[j].x); vf[1] = __builtin_bit_cast(float, vv_[j].y);
        vf[2] = __builtin_bit_cast(float, vv_[j].z); vf[3] = __builtin_bit_cast(float, vv_[j].w);
      }
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pw[g][j], vf[e], acc[g][e]);
    }
  }

  // ---- combine the lane groups of this wavefront (lanes with equal `sub`) -----------------------
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mw = m[g];
#pragma unroll
    for (int off = LPS; off < kWave; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
    const float c = (m[g] == -INFINITY) ? 0.f : fast_exp2(m[g] - mw);
    float lw = l[g] * c;
#pragma unroll
    for (int off = LPS; off < kWave; off <<= 1) lw += __shfl_xor(lw, off);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float a = acc[g][e] * c;
#pragma unroll
      for (int off = LPS; off < kWave; off <<= 1) a += __shfl_xor(a, off);
      acc[g][e] = a;
    }
    m[g] = mw;
    l[g] = lw;
  }

  // ---- combine the wavefronts through LDS ------------------------------------------------------
  __shared__ float s_m[kWavesPerBlock][G];
  __shared__ float s_l[kWavesPerBlock][G];
  __shared__ float s_acc[kWavesPerBlock][G][D];
  if (grp == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (sub == 0) {
        s_m[wave][g] = m[g];
        s_l[wave][g] = l[g];
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_acc[wave][g][sub * EPL + e] = acc[g][e];
    }
  }
  __syncthreads();

  for (int idx = threadIdx.x; idx < G * D; idx += kWavesPerBlock * kWave) {
    const int g = idx / D, d = idx % D;
    float M = s_m[0][g];
#pragma unroll
    for (int w = 1; w < kWavesPerBlock; ++w) M = fmaxf(M, s_m[w][g]);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
      const float c = (s_m[w][g] == -INFINITY) ? 0.f : fast_exp2(s_m[w][g] - M);
      L = fmaf(s_l[w][g], c, L);
      A = fmaf(s_acc[w][g][d], c, A);
    }
    const size_t row = (size_t)unit * G + g;   // == b * Hq + h * G + g
    if (p.nsplit == 1) {
      const float o = (L > 0.f) ? A / L : 0.f;
      if constexpr (kBf16)
        reinterpret_cast<uint16_t*>(p.out)[row * D + d] = (uint16_t)f32_to_bf16_bits(o);
      else
        reinterpret_cast<float*>(p.out)[row * D + d] = o;
      if (d == 0 && p.lse_out != nullptr) p.lse_out[row] = (L > 0.f) ? (M + fast_log2(L)) * kLn2 : -INFINITY;
    } else {
      float* dst = p.partial + (row * p.nsplit + split) * (D + 2);
      dst[2 + d] = A;
      if (d == 0) {
        dst[0] = M;
        dst[1] = L;
      }
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(const float* __restrict__ partial, void* out,
                                                           float* lse_out, int nsplit) {
  const size_t row = blockIdx.x;
  const int d = threadIdx.x;
  const float* src = partial + row * nsplit * (D + 2);
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, src[s * (D + 2)]);
  float L = 0.f, A = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ms = src[s * (D + 2)];
    const float c = (ms == -INFINITY) ? 0.f : fast_exp2(ms - M);
    L = fmaf(src[s * (D + 2) + 1], c, L);
    A = fmaf(src[s * (D + 2) + 2 + d], c, A);
  }
  const float o = (L > 0.f) ? A / L : 0.f;
  if constexpr (sizeof(T) == 2)
    reinterpret_cast<uint16_t*>(out)[row * D + d] = (uint16_t)f32_to_bf16_bits(o);
  else
    reinterpret_cast<float*>(out)[row * D + d] = o;
  if (d == 0 && lse_out != nullptr) lse_out[row] = (L > 0.f) ? (M + fast_log2(L)) * kLn2 : -INFINITY;
}

template <typename T, int D, int G>
void launch_decode(const DecodeParams& p, int units, hipStream_t st) {
  decode_attn_kernel<T, D, G><<<units * p.nsplit, kWavesPerBlock * kWave, 0, st>>>(p);
  if (p.nsplit > 1)
    decode_combine_kernel<T, D><<<units * G, D, 0, st>>>(p.partial, p.out, p.lse_out, p.nsplit);
}

template <typename T, int D>
void dispatch_g(const DecodeParams& p, int units, int G, hipStream_t st) {
  switch (G) {
    case 1: launch_decode<T, D, 1>(p, units, st); break;
    case 2: launch_decode<T, D, 2>(p, units, st); break;
    case 4: launch_decode<T, D, 4>(p, units, st); break;
    default: launch_decode<T, D, 8>(p, units, st); break;
  }
}

}  // namespace

DecodePlan plan_decode(const keepkv_layout* L, int capacity) {
  DecodePlan pl;
  const int units = L->batch * L->n_kv_heads;
  const int max_split = (capacity + 63) / 64;
  int ns = (1024 + units - 1) / units;         // aim at ~4 workgroups per compute unit
  ns = ns < 1 ? 1 : ns;
  ns = ns > max_split ? max_split : ns;
  ns = ns > 256 ? 256 : ns;
  pl.nsplit = ns;
  pl.partial_off = 0;
  pl.bytes = align_up((size_t)L->batch * L->n_q_heads * ns * (L->head_dim + 2) * sizeof(float), 256);
  return pl;
}

}  // namespace kk

extern "C" keepkv_status keepkv_decode_attn(const keepkv_layout* layout, const keepkv_cache* cache,
                                            const void* q, void* out, float* logits_out, float* lse_out,
                                            void* workspace, size_t workspace_bytes, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !q || !out) return KEEPKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(out) || !aligned16(cache->k) || !aligned16(cache->v)) return KEEPKV_ERR_INVALID_ARG;
  if (!layout_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  const DecodePlan pl = plan_decode(layout, cache->capacity);
  if (pl.nsplit > 1 && (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace))) return KEEPKV_ERR_WORKSPACE;

  DecodeParams p;
  p.q = q; p.k = cache->k; p.v = cache->v; p.votes = cache->votes; p.len = cache->len;
  p.out = out; p.logits_out = logits_out; p.lse_out = lse_out;
  p.partial = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + pl.partial_off);
  p.n_kv_heads = layout->n_kv_heads; p.capacity = cache->capacity; p.nsplit = pl.nsplit; p.scale = layout->scale;
  const int units = layout->batch * layout->n_kv_heads;
  const int G = layout->n_q_heads / layout->n_kv_heads;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (layout->dtype == KEEPKV_BF16) {
    if (layout->head_dim == 128) dispatch_g<uint16_t, 128>(p, units, G, st);
    else dispatch_g<uint16_t, 64>(p, units, G, st);
  } else {
    if (layout->head_dim == 128) dispatch_g<float, 128>(p, units, G, st);
    else dispatch_g<float, 64>(p, units, G, st);
  }
  return launch_status();
}
