// Shared device/host helpers of the KeepKV HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "keepkv.h"

namespace kk {

constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// ---- bf16 <-> f32 (payload kept in integer registers) ---------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }

// round-to-nearest-even f32 -> bf16 payload, NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// ---- cross-lane ------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

// Sum over aligned groups of LANES consecutive lanes (LANES in {4, 8, 16, 32, 64}); every lane of a
// group receives the group's total.
template <int LANES>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_f32<0xB1>(x);                            // quad_perm [1,0,3,2]
  x += dpp_f32<0x4E>(x);                            // quad_perm [2,3,0,1]
  if constexpr (LANES >= 8) x += dpp_f32<0x141>(x);  // row_half_mirror
  if constexpr (LANES >= 16) x += dpp_f32<0x140>(x); // row_mirror
  if constexpr (LANES >= 32) x += __shfl_xor(x, 16);
  if constexpr (LANES >= 64) x += __shfl_xor(x, 32);
  return x;
}

// ---- loads of data that is read once per launch (non-temporal hint: do not keep it in the caches) ----------
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
__device__ __forceinline__ uint4 load_once(const uint4* p) {
  const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(r[0], r[1], r[2], r[3]);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- host side -------------------------------------------------------------------------------
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline bool layout_ok(const keepkv_layout* L) {
  if (!L) return false;
  if (L->batch < 1 || L->n_kv_heads < 1 || L->n_q_heads < 1) return false;
  if (L->n_q_heads % L->n_kv_heads) return false;
  if (L->dtype != KEEPKV_F32 && L->dtype != KEEPKV_BF16) return false;
  if (!(L->scale > 0.f)) return false;
  return true;
}
inline bool layout_supported(const keepkv_layout* L) {
  int g = L->n_q_heads / L->n_kv_heads;
  if (L->head_dim != 64 && L->head_dim != 128) return false;
  return g == 1 || g == 2 || g == 4 || g == 8;
}
inline bool cache_ok(const keepkv_cache* c) {
  return c && c->k && c->v && c->votes && c->log_s && c->born && c->t_obs && c->len && c->capacity >= 1 &&
         c->capacity <= (1 << 20);
}
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline keepkv_status launch_status() {
  return hipGetLastError() == hipSuccess ? KEEPKV_OK : KEEPKV_ERR_DEVICE;
}

// ---- workspace carving (one definition, used by keepkv_workspace_bytes and by every call) ------
// The first kWorkspaceHead bytes hold control words (split tickets) that must be zero between
// calls; keepkv_workspace_init clears them and every kernel leaves them cleared.  Scratch areas of
// all calls start behind the head.
constexpr int kMaxUnits = 16384;                         // batch * n_kv_heads
constexpr size_t kMatchCountersOff = kMaxUnits * sizeof(int32_t);   // match: [0] queued rows, [1] finished workgroups
constexpr size_t kWorkspaceHead = kMatchCountersOff + 256;
// grids put (batch, kv head) on one axis and the workspace head holds one control word per pair
inline bool units_supported(const keepkv_layout* L) { return (int64_t)L->batch * L->n_kv_heads <= kMaxUnits; }

struct DecodePlan {
  int nsplit;         // workgroups per (batch, kv head)
  int per;            // slots per split (a multiple of 32; of 64 for the vector-ALU kernel)
  int waves;          // wavefronts per workgroup of the matrix-core kernel (4 or 8)
  bool valu;          // a bf16 cache on the vector-ALU kernel (only by the caller's override)
  size_t partial_off; // float [B*Hq, nsplit, D + 2]
  size_t bytes;
};
// force_per / force_waves: the caller's overrides (keepkv_cache.plan_slots_per_split / plan_wavefronts), 0 = none
DecodePlan plan_decode(const keepkv_layout* L, int capacity, int force_per = 0, int force_waves = 0);

struct SelectPlan {
  size_t keys_off;    // uint64 [B*Hkv, capacity]
  size_t bytes;
};
SelectPlan plan_select(const keepkv_layout* L, int capacity);

struct MatchPlan {
  size_t rnorm_off;   // float [B*Hkv, budget]      1/|k_c| of the retained keys
  size_t flag_off;    // int32 [1 + B*Hkv*(capacity-budget)]  counter + flagged row list
  size_t panel_off;   // bf16 [B*Hkv, padded budget, D]  retained keys gathered for the first event's kernel
  size_t partial_off; // per-share results of the f64 kernel when it splits queued rows
  size_t small_partial_off; // per-share results of the steady-state kernel when workgroups share a row block
  size_t bytes;
};
MatchPlan plan_match(const keepkv_layout* L, int capacity, int budget);

struct PrefillMatchPlan {
  size_t rnorm_off;   // float [B*Hkv, capacity]      1/|k_i| of every live slot
  size_t flag_off;    // int32 [1 + B*Hkv*capacity]   queue of rows for the f64 kernel
  size_t partial_off; // per-share results of the f64 kernel
  size_t bytes;
};
PrefillMatchPlan plan_prefill_match(const keepkv_layout* L, int capacity);

struct PrefillMergePlan {
  size_t keep_off;    // int32 [B*Hkv, capacity]      receiving slots, ascending, -1 behind them
  size_t start_off;   // int32 [B*Hkv, capacity + 1]  CSR row starts
  size_t member_off;  // int32 [B*Hkv, capacity]      absorbed slots grouped by receiver
  size_t work_off;    // int32 [B*Hkv, 2, capacity padded to 1024]  per-slot work arrays, only above 16384 slots per head
  size_t bytes;
};
PrefillMergePlan plan_prefill_merge(const keepkv_layout* L, int capacity);

struct MergePlan {
  size_t start_off;   // int32 [B*Hkv, budget + 1]   CSR row starts
  size_t member_off;  // int32 [B*Hkv, capacity]     evicted slots grouped by target
  size_t bytes;
};
MergePlan plan_merge(const keepkv_layout* L, int capacity, int budget);

}  // namespace kk
