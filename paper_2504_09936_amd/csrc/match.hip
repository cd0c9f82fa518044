// keepkv_match: nearest retained key by cosine similarity for every to-be-evicted key
// (Alg. 1, matching step), the one dense contraction of the method.
//
// bf16 caches, first event (thousands of evicted rows per head): the retained keys of a head are first
// gathered into a panel in list order; one workgroup of 8 wavefronts per compute unit then walks blocks of
// 512 evicted rows in passes.  Each wavefront keeps its 64 rows (two 32-row MFMA operands over the whole
// head dimension) in registers for a pass and the panel streams through LDS in 128-column stages.
// Every 32x32 f32 accumulator tile is reduced on the spot (scale by 1/|k_c|, running maxima); the
// similarity matrix is never written.  Steady state (one period's worth of evicted rows): a workgroup
// of 8 wavefronts per 64 rows, the columns split over the wavefronts (and, with few heads, over up to
// four such workgroups that join their results through a ticket).
//
// Exactness: the f32 result decides a row only when the best value leads the second by more than
// the rounding envelope and is away from the threshold by as much; all other rows (a fraction of a
// percent) are queued and re-evaluated in f64, where products of bf16 or f32 values are exact and
// the sum is taken in channel order.  f32 caches go through the f64 kernel entirely.
#include "kk_common.hpp"

namespace kk {
// Phase timestamps for kernel tuning; compiled in only with -DKEEPKV_TRACE (never in the product build).
#ifdef KEEPKV_TRACE
// per workgroup: [0] start, [1] first loop start, [2] first loop end, [3] first loop's shader cycles,
// [4..7] end of pass 0..3 (100 MHz wall clock except [3])
__device__ long long kk_trace_match[8 * 2048];
#define KX_TS(i) do { const int b_ = blockIdx.x; if (threadIdx.x == 0 && b_ < 2048) \
  kk_trace_match[b_ * 8 + (i)] = wall_clock64(); } while (0)
#define KX_CYC(i, v) do { const int b_ = blockIdx.x; if (threadIdx.x == 0 && b_ < 2048) \
  kk_trace_match[b_ * 8 + (i)] = (v); } while (0)
// the steady-state kernel: indexed by head
#define KS_TS(i) do { if (threadIdx.x == 0 && blockIdx.y < 256) kk_trace_match[blockIdx.y * 8 + (i)] = wall_clock64(); } while (0)
#else
#define KX_TS(i) do { } while (0)
#define KX_CYC(i, v) do { } while (0)
#define KS_TS(i) do { } while (0)
#endif
namespace {

constexpr int kRowsPerWave = 64;
constexpr int kMWaves = 8;
constexpr int kRowsPerBlock = kRowsPerWave * kMWaves;   // 512 evicted rows per workgroup and pass
constexpr int kStageCols = 128;                         // retained keys per LDS stage
constexpr unsigned kResidentWorkgroups = 256;           // of the first event's kernel: one on each of 256 compute units
constexpr int kXcds = 8;                                // accelerator dies, each with its own L2

// ---------------------------------------------------------------------------------------------------
// 1/|k_c| (f32) of every retained key; 0 for padding and for zero keys.  With `panel`, the retained keys are
// also copied there in list order, rn_pitch rows per head (padding rows zero), each row with its 16-byte
// chunk c stored at position c ^ (row mod chunks): the LDS image that the first event's kernel wants, so
// that its stage loads are straight copies that need no slot index.
constexpr int kRnormRows = 4;
template <typename T, int D>
__global__ __launch_bounds__(256) void rnorm_kernel(const T* __restrict__ k, const int32_t* __restrict__ keep_idx,
                                                    const int32_t* __restrict__ n_evict, float* __restrict__ rnorm,
                                                    int capacity, int budget, int rn_pitch, uint4* __restrict__ panel) {
  constexpr int EPL = 16 / (int)sizeof(T), LPS = D / EPL, RPB = 256 / LPS;
  const int unit = blockIdx.y;
  const int sub = threadIdx.x % LPS;
  // kRnormRows rows per lane group, all requested before the first wait (slot numbers beside the head's
  // eviction count, then the rows)
  int r[kRnormRows], slot[kRnormRows];
#pragma unroll
  for (int i = 0; i < kRnormRows; ++i) {
    r[i] = (blockIdx.x * kRnormRows + i) * RPB + threadIdx.x / LPS;
    slot[i] = r[i] < budget ? keep_idx[(size_t)unit * budget + r[i]] : -1;
  }
  if (n_evict[unit] <= 0) return;
  uint4 x[kRnormRows];
#pragma unroll
  for (int i = 0; i < kRnormRows; ++i) {
    x[i] = make_uint4(0, 0, 0, 0);
    if (slot[i] >= 0) x[i] = reinterpret_cast<const uint4*>(k)[((size_t)unit * capacity + slot[i]) * LPS + sub];
  }
#pragma unroll
  for (int i = 0; i < kRnormRows; ++i) {
    if (r[i] >= rn_pitch) continue;              // whole lane groups
    float ss = 0.f;
    if constexpr (sizeof(T) == 2) {
      const uint32_t w[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a = bf16_lo(w[e]), b = bf16_hi(w[e]);
        ss = fmaf(a, a, ss);
        ss = fmaf(b, b, ss);
      }
    } else {
      const float w[4] = {__builtin_bit_cast(float, x[i].x), __builtin_bit_cast(float, x[i].y),
                          __builtin_bit_cast(float, x[i].z), __builtin_bit_cast(float, x[i].w)};
#pragma unroll
      for (int e = 0; e < 4; ++e) ss = fmaf(w[e], w[e], ss);
    }
    if (panel != nullptr) panel[((size_t)unit * rn_pitch + r[i]) * LPS + (sub ^ (r[i] & (LPS - 1)))] = x[i];
    ss = group_sum<LPS>(ss);
    // positions budget .. rn_pitch - 1 are padding: zero, so padded columns score 0; so do zero keys and
    // negative slot numbers
    if (sub == 0) rnorm[(size_t)unit * rn_pitch + r[i]] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
  }
}

// ---------------------------------------------------------------------------------------------------
struct ExactPartial;
struct MatchParams {
  const void* k;
  const int32_t* keep_idx;
  const int32_t* evict_idx;
  const int32_t* n_evict;
  const float* rnorm;
  const unsigned char* panel;   // retained keys in list order, rows pre-swizzled (first event's kernel only)
  int32_t* match;
  float* sim_out;
  struct ExactPartial* exact_partial;   // [kExactResident] per-share results of the f64 kernel
  int32_t* exact_ticket;                // control words at the head of the workspace
  int32_t* flag_count;   // [1] rows queued for the f64 kernel; zero between calls (the f64 kernel clears it)
  int32_t* exact_done;   // [1] queued rows that the f64 kernel has finished; zero between calls
  int32_t* flag_rows;    // [units * max_evict]: unit * max_evict + j
  int capacity, budget, max_evict, rn_pitch;
  float threshold, delta;
  int per_unit, n_units;   // first event's kernel: workgroups per head, heads
  int causal;              // prefill pass: row j is slot j and its columns are the slots before it (no lists)
  const int32_t* len;      // prefill pass: live slots per head
  int small_parts;         // steady-state kernel: workgroups that share the retained list of one 64-row block
  int32_t* small_partial;  // [row blocks * small_parts][64][3] their per-row results
};

__device__ __forceinline__ int imax(int a, int b) { return a > b ? a : b; }
__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
// median of three; the backend folds this into v_med3_i32
__device__ __forceinline__ int imed3(int a, int b, int c) { return imax(imin(a, b), imin(imax(a, b), c)); }

// A row whose best cosine lies below the threshold by more than the f32 arithmetic's error has no target
// whichever column holds that best value, so neither a small margin to the runner-up nor a best value that
// is not positive (`upper` is then 0: every value of the row is at most 0) makes it undecided, as long as
// the caller does not ask for the similarity itself.  A NaN in `upper` compares false and keeps the row queued.
__device__ __forceinline__ bool surely_below(const MatchParams& p, float upper, float ss, float rn_e) {
  return p.sim_out == nullptr && ss > 0.f && rn_e < INFINITY && upper + p.delta < p.threshold;
}

// Decision of one row from the integer images of its best value v1 (column c1) and of an upper bound v2 of
// every other column's value, both still lacking the factor 1/|k_e| (ss = |k_e|^2); a row that the f32
// arithmetic cannot decide is queued for the f64 kernel.
__device__ __forceinline__ void decide_row(const MatchParams& p, int unit, int j, int v1, int c1, int v2, float ss) {
  const float rn_e = 1.0f / sqrtf(ss);
  const float y1 = __builtin_bit_cast(float, v1), y2 = (v2 > 0) ? __builtin_bit_cast(float, v2) : 0.f;
  const float cos1 = y1 * rn_e;
  bool fragile = !(v1 > 0) || !(ss > 0.f) || !(rn_e < INFINITY) || (y1 - y2) * rn_e <= p.delta ||
                 fabsf(cos1 - p.threshold) <= p.delta || c1 >= p.budget;
  if (surely_below(p, (v1 > 0) ? cos1 : 0.f, ss, rn_e)) fragile = false;
  const size_t o = (size_t)unit * p.max_evict + j;
  p.match[o] = (cos1 > p.threshold) ? c1 : -1;
  if (p.sim_out != nullptr) p.sim_out[o] = cos1;
  if (fragile) {
    const int at = atomicAdd(p.flag_count, 1);
    p.flag_rows[at] = (int)o;
  }
}

// f32 decision of one row from its best value y1 (column c1) and an upper bound y2 of every other column's
// value, both still lacking the factor 1/|k_e|; rows that the f32 arithmetic cannot decide are queued.
__device__ __forceinline__ void decide_row_f32(const MatchParams& p, int unit, int j, float y1, int c1, float y2,
                                               float ss) {
  const float rn_e = 1.0f / sqrtf(ss);
  const float cos1 = y1 * rn_e;
  bool fragile = !(y1 > 0.f) || !(ss > 0.f) || !(rn_e < INFINITY) || !((y1 - y2) * rn_e > p.delta) ||
                 !(fabsf(cos1 - p.threshold) > p.delta) || c1 >= p.budget;
  if (surely_below(p, (y1 <= 0.f) ? 0.f : cos1, ss, rn_e)) fragile = false;
  const size_t o = (size_t)unit * p.max_evict + j;
  p.match[o] = (cos1 > p.threshold) ? c1 : -1;
  if (p.sim_out != nullptr) p.sim_out[o] = cos1;
  if (fragile) {
    const int at = atomicAdd(p.flag_count, 1);
    p.flag_rows[at] = (int)o;
  }
}

// The first event's kernel.  The product is taken transposed, retained keys as the A operand and the
// wavefront's evicted rows as B, so that lane (l32, half) holds, for ITS evicted row, the 16 retained columns
// 8 (i / 4) + 4 half + i % 4 of each 32-column block: all values in a lane belong to one row.  Per value the
// fold then costs a multiply by 1/|k_c| and a maximum into the running best of its column class i, plus a
// share of a max3 tree that gives the block's best, which goes into a running (best, second best, block)
// triple.  No column number travels with the values: at the end the winning class is the one whose running
// best equals the overall best, and the winning block is the triple's.  Every other column's value is
// bounded by the second best block value or by the best of the other classes, which is all that the
// exactness test needs.
template <int D>
__global__ __launch_bounds__(kMWaves* kWave, 2) void match_mfma_kernel(MatchParams p) {
  constexpr int KS = D / 16;                 // MFMA k-steps over the head dimension
  constexpr int ROWB = D * 2;                // bytes per key
  constexpr int CHUNKS = ROWB / 16;          // 16-byte chunks per key
  constexpr int STAGE_BYTES = kStageCols * ROWB;
  constexpr int LOADS = kStageCols * CHUNKS / (kMWaves * kWave);   // async 16-byte loads per lane per stage

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* s_stage = smem;                                        // 2 stages, swizzled rows
  float* s_rn = reinterpret_cast<float*>(smem + 2 * STAGE_BYTES);       // [2][kStageCols]

  // Workgroups are dealt to the 8 XCDs in turn, each with an L2 of its own.  All workgroups of a head are
  // placed on one XCD (when the heads divide evenly), so that the head's retained keys, which every pass of
  // every one of them streams again, stay in that L2.
  int unit, first_rb;
  if (p.n_units % kXcds == 0) {
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    unit = xcd * (p.n_units / kXcds) + slot / p.per_unit;
    first_rb = slot % p.per_unit;
  } else {
    unit = blockIdx.x / p.per_unit;
    first_rb = blockIdx.x % p.per_unit;
  }
  const int n_ev = p.n_evict[unit];
  const int n_rb = (n_ev + kRowsPerBlock - 1) / kRowsPerBlock;
  int rb = first_rb;                         // this pass's block of rows; later passes: rb + per_unit, ...
  if (rb >= n_rb) return;
  KX_TS(0);
  const int n_keep = p.budget;               // n_evict > 0 implies the retained list is full
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;

  const unsigned char* kbytes = reinterpret_cast<const unsigned char*>(p.k) + (size_t)unit * p.capacity * ROWB;
  const int32_t* evict = p.evict_idx + (size_t)unit * p.max_evict;
  const float* rn_c = p.rnorm + (size_t)unit * p.rn_pitch;

  // ---- stage loader: global -> LDS without passing through registers.  The panel holds the head's retained
  // keys in list order with chunk c of key `col` at position c ^ (col mod CHUNKS) of its row, which keeps the
  // MFMA operand reads below free of bank conflicts; a stage is one contiguous piece of it, copied as is.
  const unsigned char* panel = p.panel + (size_t)unit * p.rn_pitch * ROWB;
  auto issue_stage = [&](int s, int buf) {
    const unsigned char* src = panel + (size_t)s * STAGE_BYTES + tid * 16;
    unsigned char* dst = s_stage + buf * STAGE_BYTES + wave * 64 * 16;
#pragma unroll
    for (int i = 0; i < LOADS; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + i * (kMWaves * kWave) * 16),
                                       (__attribute__((address_space(3))) void*)(dst + i * (kMWaves * kWave) * 16), 16, 0, 0);
    if (wave < kStageCols / 64) {            // 1/|k_c| of the stage's keys (padded with zeros by rnorm_kernel)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(rn_c + s * kStageCols + tid),
                                       (__attribute__((address_space(3))) void*)(s_rn + buf * kStageCols + wave * 64),
                                       4, 0, 0);
    }
  };
  int par = 0;                               // LDS buffer of the stage being consumed
  issue_stage(0, 0);

  // ---- B operands: this wavefront's 64 evicted rows of the pass, resident in registers.  The byte offsets
  // of a pass's rows are fetched one pass ahead, the rows themselves as soon as the previous pass has
  // issued its last MFMA, so that their latency overlaps that pass's epilogue.
  // (the slot numbers as loaded: any arithmetic on them would be a first use, and the compiler waits for a
  // load at its first use -- here that is request_rows(), a whole pass later)
  auto row_offset = [&](int rb_, int t) {
    return evict[min(rb_ * kRowsPerBlock + wave * kRowsPerWave + t * 32 + l32, n_ev - 1)];
  };
  int row_off[2] = {row_offset(rb, 0), row_offset(rb, 1)};
  bf16x8_t e[2][KS];
  auto request_rows = [&]() {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        e[t][ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(
            kbytes + (uint32_t)row_off[t] * (uint32_t)ROWB + ks * 32 + half * 16));
  };
  request_rows();

  const int n_stage = (n_keep + kStageCols - 1) / kStageCols;
  const uint32_t frag0 = l32 * ROWB + (((l32 & (CHUNKS - 1)) ^ half) * 16);
  for (;;) {                                 // one pass per iteration
  float ss_row[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint4 x = __builtin_bit_cast(uint4, e[t][ks]);
      const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float lo = bf16_lo(w[i]), hi = bf16_hi(w[i]);
        ss = fmaf(lo, lo, ss);
        ss = fmaf(hi, hi, ss);
      }
    }
    ss_row[t] = ss + __shfl_xor(ss, 32);
  }
  const int rb_next = rb + p.per_unit;
  const bool more = rb_next < n_rb;          // uniform over the workgroup

  // running state per tile: best of each column class, and (best, second best, block) over block maxima.
  // Values are compared through their integer images (for positive floats the order is the same, and a
  // negative one loses to the initial 0): a row without a positive similarity is queued for the f64 kernel
  // anyway, and so is one whose best image is a NaN's.
  int cls[2][16];
  int b1[2] = {0, 0}, b2[2] = {0, 0};
  int g1[2] = {0, 0};
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) cls[t][i] = 0;
  // software pipeline: the MFMAs of column block cb are issued together with the fold of block
  // cb - 1.  Two accumulator sets alternate (even blocks write A and fold B, odd blocks the reverse), so
  // no accumulator is ever copied.  The first fold sees zeros and is harmless.
  // rn[g]: 1/|k_c| of the columns of accumulator registers 4g .. 4g+3, for the block being folded; each
  // group is replaced by the next block's as soon as its last value is folded.
  f32x16_t accA0 = {0}, accA1 = {0}, accB0 = {0}, accB1 = {0};
  f32x4_t rn[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) rn[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  int cb_prev = 0;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (rb == first_rb) KX_TS(1);
#ifdef KEEPKV_TRACE
  const long long cyc0 = clock64();
#endif
  if (more) {                                // next pass's row offsets: in flight during this pass's first stage
    row_off[0] = row_offset(rb_next, 0);
    row_off[1] = row_offset(rb_next, 1);
  }

  constexpr int VPK = 16 / KS;               // accumulator values folded per k-step and tile
  constexpr int BPS = kStageCols / 32;       // column blocks per stage (even)
  static_assert(BPS % 2 == 0, "the accumulator sets alternate by column block");
  static_assert(VPK == 2 || VPK == 4, "fold_vals handles two or four values per k-step");
  const int n_blk = (n_keep + 31) / 32;

  // values [ks * VPK, (ks + 1) * VPK) of one finished accumulator tile: scale, class maxima, block maximum
  auto fold_vals = [&](int ks, const f32x16_t& od, int (&c)[16], int& gm) {
#pragma unroll
    for (int i = ks * VPK; i < (ks + 1) * VPK; i += 2) {
      const int k0 = __builtin_bit_cast(int, od[i] * rn[i / 4][i % 4]);
      const int k1 = __builtin_bit_cast(int, od[i + 1] * rn[(i + 1) / 4][(i + 1) % 4]);
      c[i] = imax(c[i], k0);
      c[i + 1] = imax(c[i + 1], k1);
      if (i == 0) gm = imax(k0, k1);
      else asm("v_max3_i32 %0, %1, %2, %3" : "=v"(gm) : "v"(gm), "v"(k0), "v"(k1));   // kept in this order
    }
  };
  auto fold_group = [&](int gm, int ocb, int& v1, int& v2, int& blk) {
    blk = (gm > v1) ? ocb : blk;
    v2 = imed3(v1, v2, gm);
    v1 = imax(v1, gm);
  };

  for (int s = 0; s < n_stage; ++s) {
    if (s + 1 < n_stage) issue_stage(s + 1, par ^ 1);
    else if (more) issue_stage(0, par ^ 1);                   // the next pass starts over at the first columns
    // operand fragment of key 32 cbl + l32: chunk (2 ks + half) ^ (l32 mod CHUNKS) of its row, which is the
    // lane's chunk of k-step 0 with 32 ks XORed into the byte offset
    const uint32_t frag_cur = frag0 + par * STAGE_BYTES;
    auto frag = [&](int cbl, int ks) {
      return *reinterpret_cast<const bf16x8_t*>(s_stage + ((frag_cur ^ (uint32_t)(ks * 32)) + cbl * 32 * ROWB));
    };
    bf16x8_t bq = frag(0, 0);
    // Explicit interleave: each MFMA is followed by the fold of VPK values of the previous column
    // block, and nothing may be scheduled across the fences, so the matrix pipe and the vector ALU of
    // this wavefront run side by side.
    auto block = [&](int cbl, f32x16_t& nw0, f32x16_t& nw1, const f32x16_t& od0, const f32x16_t& od1) {
      const f32x16_t zero = {0};
      // 1/|k_c| of the 16 columns that this lane's accumulator registers hold in block cbl
      const f32x4_t* rn_src = reinterpret_cast<const f32x4_t*>(s_rn + par * kStageCols + cbl * 32 + 4 * half);
      int gm0 = 0, gm1 = 0;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t bnext = (ks + 1 < KS) ? frag(cbl, ks + 1) : frag((cbl + 1) % BPS, 0);
        nw0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq, e[0][ks], ks == 0 ? zero : nw0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        fold_vals(ks, od0, cls[0], gm0);
        __builtin_amdgcn_sched_barrier(0);
        nw1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq, e[1][ks], ks == 0 ? zero : nw1, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        fold_vals(ks, od1, cls[1], gm1);
        if (((ks + 1) * VPK) % 4 == 0) rn[((ks + 1) * VPK) / 4 - 1] = rn_src[2 * (((ks + 1) * VPK) / 4 - 1)];
        __builtin_amdgcn_sched_barrier(0);
        bq = bnext;
      }
      fold_group(gm0, cb_prev, b1[0], b2[0], g1[0]);
      fold_group(gm1, cb_prev, b1[1], b2[1], g1[1]);
    };
#pragma unroll
    for (int cbl = 0; cbl < BPS; ++cbl) {
      const int cb = s * BPS + cbl;                           // global column block
      if (cb < n_blk) {                                       // uniform over the workgroup
        if (cbl % 2 == 0) block(cbl, accA0, accA1, accB0, accB1);
        else block(cbl, accB0, accB1, accA0, accA1);
        cb_prev = cb;
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    par ^= 1;
  }
  if (rb == first_rb) { KX_TS(2); KX_CYC(3, clock64() - cyc0); }
  if (more) request_rows();                                   // the operand registers are free: next pass's rows
  {                                                           // the last block is still unfolded
    const bool even_last = (n_blk & 1) != 0;
    int gm0 = 0, gm1 = 0;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (even_last) {
        fold_vals(ks, accA0, cls[0], gm0);
        fold_vals(ks, accA1, cls[1], gm1);
      } else {
        fold_vals(ks, accB0, cls[0], gm0);
        fold_vals(ks, accB1, cls[1], gm1);
      }
    }
    fold_group(gm0, cb_prev, b1[0], b2[0], g1[0]);
    fold_group(gm1, cb_prev, b1[1], b2[1], g1[1]);
  }

  // ---- finish: winning class per tile, then the two lanes of a row (the halves) meet ----------------
  float y1[2], y2[2];
  int c1[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    int s1 = cls[t][0], s2 = 0, ci = 0;
#pragma unroll
    for (int i = 1; i < 16; ++i) {
      const int x = cls[t][i];
      const bool up = x > s1;
      s2 = up ? s1 : imax(s2, x);
      ci = up ? i : ci;
      s1 = up ? x : s1;
    }
    // s1 equals b1[t]: both are the largest value of this lane's half of the row
    const int col = 32 * g1[t] + 8 * (ci / 4) + 4 * half + (ci % 4);
    const int rest = imax(b2[t], s2);                         // bounds every other column of this half
    const int o1 = __shfl_xor(s1, 32), orest = __shfl_xor(rest, 32), ocol = __shfl_xor(col, 32);
    y1[t] = __builtin_bit_cast(float, imax(s1, o1));
    c1[t] = (s1 > o1) ? col : ((o1 > s1) ? ocol : min(col, ocol));
    y2[t] = __builtin_bit_cast(float, imax(imax(rest, orest), imin(s1, o1)));
  }
  const int j = rb * kRowsPerBlock + wave * kRowsPerWave + lane;   // lane = 32 half + l32 finishes row l32 of tile `half`
  if (j < n_ev)
    decide_row_f32(p, unit, j, half ? y1[1] : y1[0], half ? c1[1] : c1[0], half ? y2[1] : y2[0],
                   half ? ss_row[1] : ss_row[0]);
  { const int pass = (rb - first_rb) / p.per_unit; if (pass < 4) KX_TS(4 + pass); }
  if (!more) break;
  rb = rb_next;
  }
}

// Few evicted rows per head (the steady state: one period's worth).  One workgroup of 8 wavefronts per
// 64-row block, so the work of one head spreads over a whole compute unit instead of a single
// wavefront.  The 64 evicted rows are copied once into LDS (swizzled like the stages above) and serve as
// the B operand of every wavefront; a wavefront takes every 8th block of 32 retained columns and requests
// the keys of four of its blocks at once, straight into registers as A operands, because the kernel is
// all memory latency: nothing is reused and little is computed.  1/|k_c| is formed here from the operand
// registers (the two lanes of a column hold one half of its channels each).  The fold is the transposed one
// of the first event's kernel (a lane holds one evicted row; class maxima and a (best, second, block) triple).
constexpr int kSmallWaves = 8;
constexpr int kSmallBatch = 4;        // column blocks in flight per wavefront
constexpr int kSmallMaxParts = 4;     // workgroups that may share one 64-row block
template <int D>
__global__ __launch_bounds__(kSmallWaves* kWave, 2) void match_small_kernel(MatchParams p) {
  constexpr int KS = D / 16, ROWB = D * 2, CHUNKS = ROWB / 16;
  constexpr int ROW_LOADS = 64 * CHUNKS / (kSmallWaves * kWave);       // 16-byte copies per thread for the 64 rows
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* s_rows = smem;                                         // [64][ROWB], chunk c at c ^ (row mod CHUNKS)
  int* s_top = reinterpret_cast<int*>(smem + 64 * ROWB);                // [kSmallWaves][64][3]
  float* s_rn = reinterpret_cast<float*>(s_top + kSmallWaves * 64 * 3); // [kSmallWaves][32]: a wavefront's current block

  const int unit = blockIdx.y;
  const int part = blockIdx.z, parts = p.small_parts;
  KS_TS(0);
  const int n_ev = p.n_evict[unit];
  const int row_blk = blockIdx.x * 64;
  if (row_blk >= n_ev) return;                 // all parts of the block alike
  KS_TS(1);
  const int n_keep = p.budget;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const unsigned char* kbytes = reinterpret_cast<const unsigned char*>(p.k) + (size_t)unit * p.capacity * ROWB;
  const int32_t* keep = p.keep_idx + (size_t)unit * p.budget;
  const int32_t* evict = p.evict_idx + (size_t)unit * p.max_evict;
  const int ncb = (n_keep + 31) / 32;

  // ---- requests, all issued before the first wait ---------------------------------------------------
  // (1) slot numbers of the evicted rows this thread copies, and of the first batch's retained keys
  int ev_slot[ROW_LOADS];
#pragma unroll
  for (int i = 0; i < ROW_LOADS; ++i) {
    const int q = tid + i * (kSmallWaves * kWave);
    ev_slot[i] = evict[min(row_blk + q / CHUNKS, n_ev - 1)];
  }
  auto col_slot = [&](int cb) { return keep[min(cb * 32 + l32, n_keep - 1)]; };
  // column blocks of this wavefront: first_cb, first_cb + stride, ...; kSmallBatch of them in flight
  const int first_cb = part * kSmallWaves + wave, stride = parts * kSmallWaves;
  int slot[kSmallBatch];
  bool slot_ok[kSmallBatch];
#pragma unroll
  for (int i = 0; i < kSmallBatch; ++i) slot[i] = col_slot(min(first_cb + i * stride, ncb - 1));
  // (2) the first batch of retained keys, as A operands: lane (l32, half) holds chunks 2 ks + half of column l32.
  // They are requested BEFORE the evicted rows' asynchronous copies: the compiler waits for a load into
  // registers (here the slot numbers) behind every outstanding asynchronous copy, so the other order put the
  // rows' whole round trip in front of these requests, and each block's requests behind the previous block's.
  uint4 akey[kSmallBatch][KS];
  auto request_keys = [&](int cb_first) {
    // one wait for all slot numbers, then all requests: a wait placed behind a conditional batch of requests
    // would cover that batch as well
    static_assert(kSmallBatch == 4, "the statement below names four slot numbers");
    asm volatile("" : "+v"(slot[0]), "+v"(slot[1]), "+v"(slot[2]), "+v"(slot[3]));   // first use of all four: here
#pragma unroll
    for (int i = 0; i < kSmallBatch; ++i) {
      slot_ok[i] = slot[i] >= 0;             // (a negative slot number: slot 0 stands in, its column scores 0)
      if (cb_first + i * stride < ncb) {     // uniform over the wavefront; blocks beyond the list are not fetched
        const unsigned char* row = kbytes + ((uint32_t)max(slot[i], 0) * ROWB + half * 16);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) akey[i][ks] = *reinterpret_cast<const uint4*>(row + ks * 32);
      }
    }
  };
  // (the evicted rows' slot numbers too have their first use here, ahead of the key requests: their wait
  // would otherwise come behind those requests and cover them)
#pragma unroll
  for (int i = 0; i < ROW_LOADS; ++i) asm volatile("" : "+v"(ev_slot[i]));
  request_keys(first_cb);
  // (3) the evicted rows -> LDS; a wavefront instruction deposits 64 consecutive 16-byte chunks
#pragma unroll
  for (int i = 0; i < ROW_LOADS; ++i) {
    const int q = tid + i * (kSmallWaves * kWave);
    const int r = q / CHUNKS, phys = q % CHUNKS;
    const unsigned char* src = kbytes + ((uint32_t)ev_slot[i] * ROWB + ((phys ^ (r & (CHUNKS - 1))) * 16));
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(s_rows + (q - lane) * 16), 16, 0, 0);
  }

  int cls[2][16];
  int b1[2] = {0, 0}, b2[2] = {0, 0}, g1[2] = {0, 0};
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) cls[t][i] = 0;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();                           // the rows are in LDS
  KS_TS(2);

  const uint32_t frag0 = l32 * ROWB + (((l32 & (CHUNKS - 1)) ^ half) * 16);
  auto efrag = [&](int t, int ks) {          // B operand: evicted row 32 t + l32, chunk (2 ks + half) ^ (row mod CHUNKS)
    return *reinterpret_cast<const bf16x8_t*>(s_rows + ((frag0 ^ (uint32_t)(ks * 32)) + t * 32 * ROWB));
  };
  for (int cb0 = first_cb; cb0 < ncb; cb0 += kSmallBatch * stride) {
#pragma unroll
    for (int i = 0; i < kSmallBatch; ++i) {
      const int cb = cb0 + i * stride;
      if (cb < ncb) {                        // uniform over the wavefront
        asm volatile("" ::: "memory");       // the evicted rows are read from LDS again for every block: kept
                                             // in registers beside four blocks of keys they would spill
        // 1/|k_c| of this block's columns: each lane squares its half of column l32's channels, the halves
        // meet, and the 32 values pass through this wavefront's corner of LDS to reach the lanes that hold
        // the columns' products (registers 4 g + e of a lane: columns 8 g + 4 half + e).  Zero for a column
        // beyond the list, a negative slot number or a zero key: such a column scores 0.
        {
          float ssq = 0.f;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const uint32_t w4[4] = {akey[i][ks].x, akey[i][ks].y, akey[i][ks].z, akey[i][ks].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float lo = bf16_lo(w4[e]), hi = bf16_hi(w4[e]);
              ssq = fmaf(lo, lo, ssq);
              ssq = fmaf(hi, hi, ssq);
            }
          }
          ssq += __shfl_xor(ssq, 32);
          const bool real = cb * 32 + l32 < n_keep && slot_ok[i] && ssq > 0.f;
          if (half == 0) s_rn[wave * 32 + l32] = real ? 1.0f / sqrtf(ssq) : 0.f;
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        const f32x4_t* rn_src = reinterpret_cast<const f32x4_t*>(s_rn + wave * 32 + 4 * half);
#pragma unroll
        for (int t = 0; t < 2; ++t) {        // one 32-row tile after the other: 16 accumulator registers
          f32x16_t acc = {0};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, akey[i][ks]), efrag(t, ks), acc, 0, 0, 0);
          int gm = 0;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4_t rn = rn_src[2 * g];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int k = __builtin_bit_cast(int, acc[4 * g + e] * rn[e]);
              cls[t][4 * g + e] = imax(cls[t][4 * g + e], k);
              gm = imax(gm, k);
            }
          }
          g1[t] = (gm > b1[t]) ? cb : g1[t];
          b2[t] = imed3(b1[t], b2[t], gm);
          b1[t] = imax(b1[t], gm);
        }
      }
    }
    if (cb0 + kSmallBatch * stride < ncb) {   // a long retained list: the next batch (its latency is exposed)
#pragma unroll
      for (int i = 0; i < kSmallBatch; ++i)
        slot[i] = col_slot(min(cb0 + (kSmallBatch + i) * stride, ncb - 1));
      request_keys(cb0 + kSmallBatch * stride);
    }
  }

  KS_TS(3);
  // ---- this wavefront's result per row: winning class per tile, then the two halves of a row meet ----
  int y1[2], y2[2], c1[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    int s1 = cls[t][0], s2 = 0, ci = 0;
#pragma unroll
    for (int i = 1; i < 16; ++i) {
      const int x = cls[t][i];
      const bool up = x > s1;
      s2 = up ? s1 : imax(s2, x);
      ci = up ? i : ci;
      s1 = up ? x : s1;
    }
    const int col = 32 * g1[t] + 8 * (ci / 4) + 4 * half + (ci % 4);
    const int rest = imax(b2[t], s2);                         // bounds every other column of this half
    const int o1 = __shfl_xor(s1, 32), orest = __shfl_xor(rest, 32), ocol = __shfl_xor(col, 32);
    y1[t] = imax(s1, o1);
    c1[t] = (s1 > o1) ? col : ((o1 > s1) ? ocol : min(col, ocol));
    y2[t] = imax(imax(rest, orest), imin(s1, o1));
  }
  {                                                           // lane = 32 half + l32 speaks for row l32 of tile `half`
    int* t3 = s_top + (wave * 64 + lane) * 3;
    t3[0] = half ? y1[1] : y1[0];
    t3[1] = half ? c1[1] : c1[0];
    t3[2] = half ? y2[1] : y2[0];
  }
  __syncthreads();
  KS_TS(4);
  if (wave != 0) return;
  const int j = row_blk + lane;
  int v1 = (int)0x80000000, v2 = (int)0x80000000, cc = 0;
  auto join = [&](int val, int col, int val2) {      // another share's (best, column, runner-up) for this row
    if (val > v1 || (val == v1 && col < cc)) {
      v2 = imax(v1, val2);
      v1 = val;
      cc = col;
    } else {
      v2 = imax(v2, val);
    }
  };
  for (int w = 0; w < kSmallWaves; ++w) {
    const int* t3 = s_top + (w * 64 + lane) * 3;
    join(t3[0], t3[1], t3[2]);
  }
  if (parts > 1) {
    // The workgroups that share this row block meet the way the decode splits do: device-scope stores of the
    // per-row results, a ticket (a control word at the head of the workspace, zero between calls), and the
    // last one to arrive joins all shares, in list order, and clears the ticket.
    const int blk = unit * (int)gridDim.x + (int)blockIdx.x;
    int32_t* mine = p.small_partial + ((size_t)(blk * parts + part) * 64 + lane) * 3;
    __hip_atomic_store(mine + 0, v1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(mine + 1, cc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(mine + 2, v2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // the wavefront's write-through stores have completed
    int ticket = 0;
    if (lane == 0) ticket = __hip_atomic_fetch_add(&p.exact_ticket[blk], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket != parts - 1) return;
    v1 = (int)0x80000000; v2 = (int)0x80000000; cc = 0;
    int val[kSmallMaxParts], col[kSmallMaxParts], val2[kSmallMaxParts];
#pragma unroll
    for (int q = 0; q < kSmallMaxParts; ++q) {       // one round trip for all shares
      const int32_t* r = p.small_partial + ((size_t)(blk * parts + min(q, parts - 1)) * 64 + lane) * 3;
      val[q] = __hip_atomic_load(r + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      col[q] = __hip_atomic_load(r + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      val2[q] = __hip_atomic_load(r + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#pragma unroll
    for (int q = 0; q < kSmallMaxParts; ++q)
      if (q < parts) join(val[q], col[q], val2[q]);
    if (lane == 0) __hip_atomic_store(&p.exact_ticket[blk], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (j >= n_ev) return;
  // |k_e|^2 of this lane's row, from the LDS copy
  float ss = 0.f;
  {
    const unsigned char* row = s_rows + lane * ROWB;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const uint4 x = *reinterpret_cast<const uint4*>(row + c * 16);   // the order of the chunks does not matter here
      const uint32_t w4[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float lo = bf16_lo(w4[i]), hi = bf16_hi(w4[i]);
        ss = fmaf(lo, lo, ss);
        ss = fmaf(hi, hi, ss);
      }
    }
  }
  decide_row(p, unit, j, v1, cc, v2, ss);
  KS_TS(5);
}

// queue every live evicted row (f32 caches)
__global__ void flag_all_kernel(const int32_t* __restrict__ n_evict, int32_t* flag_count, int32_t* flag_rows,
                                int max_evict) {
  const int unit = blockIdx.y;
  const int n = n_evict[unit];
  for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x) {
    const int at = atomicAdd(flag_count, 1);
    flag_rows[at] = unit * max_evict + j;
  }
}


// ---------------------------------------------------------------------------------------------------
// f64 evaluation of queued rows: threads stride over the retained keys (each thread evaluates whole keys,
// channels in index order, so the sums match an index-order f64 sum).  One workgroup per row; when the
// queue is so short that the compute units would mostly idle (the steady state: a handful of rows), up to
// kExactMaxParts workgroups per row, each over a contiguous share of the retained list.  Their results
// meet the way the decode splits do: device-scope stores, a ticket, the last one to arrive combines and
// clears the ticket (the tickets are control words at the head of the workspace, zero between calls).
constexpr int kExactMaxParts = 8;
constexpr int kExactResident = 512;     // workgroups of the bf16 f64 kernel that run at once (two per compute unit); size of the partial array
constexpr int kExactResidentGeneric = 256;   // the generic kernel's registers allow one per compute unit
struct ExactPartial {
  unsigned long long best_bits;
  int best_c, pad;
};

// The queue counter is a control word that must be zero when the next call starts.  A workgroup adds the
// number of queued rows it has finished to the exit counter (nothing if it finished none: with an empty queue
// no workgroup touches either word), and the workgroup whose addition completes the queue clears both.
// Every workgroup that had work read the queue counter before it started, and the others do nothing whatever
// value they read, so clearing it then is safe.
__device__ __forceinline__ void exact_exit(const MatchParams& p, int n_flag, int rows_finished) {
  if (threadIdx.x == 0 && rows_finished > 0 &&
      __hip_atomic_fetch_add(p.exact_done, rows_finished, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + rows_finished == n_flag) {
    __hip_atomic_store(p.flag_count, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p.exact_done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void match_exact_kernel(MatchParams p) {
  __shared__ double s_e[D];
  __shared__ double s_best[4];
  __shared__ int s_bestc[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_flag = *p.flag_count;
  int rows_finished = 0;                 // (thread 0) queued rows whose result this workgroup has written
  const T* kall = reinterpret_cast<const T*>(p.k);
  constexpr int EPV = 16 / (int)sizeof(T), NV = D / EPV;
  int parts = 1;
  {
    const int room = imin((int)gridDim.x, kExactResidentGeneric);
    while (parts < kExactMaxParts && (long)n_flag * (parts * 2) <= (long)room) parts *= 2;
  }
  for (int w = blockIdx.x; w < n_flag * parts; w += gridDim.x) {
    const int f = w / parts, part = w % parts;
    const int o = p.flag_rows[f];
    const int unit = o / p.max_evict, j = o % p.max_evict;
    const T* kunit = kall + (size_t)unit * p.capacity * D;
    // causal (the prefill pass): the row is slot j itself and its columns are the slots 0 .. j - 1
    const int32_t* keep = p.causal ? nullptr : p.keep_idx + (size_t)unit * p.budget;
    const int e = p.causal ? j : p.evict_idx[(size_t)unit * p.max_evict + j];
    const int n_cols = p.causal ? j : p.budget;
    const int share = (n_cols + parts - 1) / parts;
    const int c_lo = part * share, c_hi = imin(n_cols, c_lo + share);
    __syncthreads();                      // previous row's shared values are no longer read
    for (int d = tid; d < D; d += 256) {
      if constexpr (sizeof(T) == 2) s_e[d] = (double)bf16_to_f32(reinterpret_cast<const uint16_t*>(kunit)[(size_t)e * D + d]);
      else s_e[d] = (double)kunit[(size_t)e * D + d];
    }
    __syncthreads();
    double ss_e = 0.0;
    for (int d = 0; d < D; ++d) ss_e = fma(s_e[d], s_e[d], ss_e);
    const double rn_e = 1.0 / sqrt(ss_e);
    double best = -INFINITY;
    int best_c = 0x7FFFFFFF;
    for (int c = c_lo + tid; c < c_hi; c += 256) {
      const int slot = p.causal ? c : keep[c];
      if (slot < 0) continue;
      const T* kc = kunit + (size_t)slot * D;
      uint4 rowv[NV];
#pragma unroll
      for (int v = 0; v < NV; ++v) rowv[v] = reinterpret_cast<const uint4*>(kc)[v];   // one round trip per key
      double dot = 0.0, ss_c = 0.0;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int d0 = v * EPV;
        const uint4 x = rowv[v];
        if constexpr (sizeof(T) == 2) {
          const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const double lo = (double)bf16_lo(w[i]), hi = (double)bf16_hi(w[i]);
            dot = fma(s_e[d0 + 2 * i], lo, dot);
            ss_c = fma(lo, lo, ss_c);
            dot = fma(s_e[d0 + 2 * i + 1], hi, dot);
            ss_c = fma(hi, hi, ss_c);
          }
        } else {
          const float w[4] = {__builtin_bit_cast(float, x.x), __builtin_bit_cast(float, x.y),
                              __builtin_bit_cast(float, x.z), __builtin_bit_cast(float, x.w)};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            dot = fma(s_e[d0 + i], (double)w[i], dot);
            ss_c = fma((double)w[i], (double)w[i], ss_c);
          }
        }
      }
      const double rn_c = 1.0 / sqrt(ss_c);
      double u = (dot * rn_e) * rn_c;
      if (!(fabs(u) <= 1.79e308)) u = -INFINITY;   // zero-norm keys (nan / inf) match nothing
      if (u > best) {
        best = u;
        best_c = c;
      }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const double ob = __shfl_xor(best, off);
      const int oc = __shfl_xor(best_c, off);
      if (ob > best || (ob == best && oc < best_c)) {
        best = ob;
        best_c = oc;
      }
    }
    if (lane == 0) {
      s_best[wave] = best;
      s_bestc[wave] = best_c;
    }
    __syncthreads();
    if (tid == 0) {
      for (int w = 1; w < 4; ++w)
        if (s_best[w] > best || (s_best[w] == best && s_bestc[w] < best_c)) {
          best = s_best[w];
          best_c = s_bestc[w];
        }
      bool finish = parts == 1;
      if (!finish) {
        // with parts > 1 every workgroup has at most one work item, w < gridDim.x
        ExactPartial* mine = p.exact_partial + w;
        __hip_atomic_store(&mine->best_bits, __builtin_bit_cast(unsigned long long, best), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&mine->best_c, best_c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // the two write-through stores have completed
        finish = __hip_atomic_fetch_add(&p.exact_ticket[f], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == parts - 1;
        if (finish) {                     // the last share of this row: join them, in list order
          best = -INFINITY;
          best_c = 0x7FFFFFFF;
          for (int q = 0; q < parts; ++q) {
            const ExactPartial* r = p.exact_partial + f * parts + q;
            const double rb = __builtin_bit_cast(double, __hip_atomic_load(&r->best_bits, __ATOMIC_RELAXED,
                                                                           __HIP_MEMORY_SCOPE_AGENT));
            const int rc = __hip_atomic_load(&r->best_c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (rb > best) {
              best = rb;
              best_c = rc;
            }
          }
          __hip_atomic_store(&p.exact_ticket[f], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
        }
      }
      if (finish) {
        p.match[o] = (best > (double)p.threshold) ? best_c : -1;
        if (p.sim_out != nullptr) p.sim_out[o] = (float)best;
        ++rows_finished;
      }
    }
  }
  exact_exit(p, n_flag, rows_finished);
}

// ---------------------------------------------------------------------------------------------------
// Merge-first prefill pass (App. B.4): for every live slot its most similar EARLIER key.  The same dense
// contraction as above with rows = columns = the head's own keys and a causal mask, so the keys need no
// gathering: a workgroup of 4 wavefronts takes 128 consecutive slots as rows (32 per wavefront, resident in
// registers as B operands) and streams the slots before them through LDS in 64-key stages, copied straight
// from the cache with the row swizzle applied on the address side.  A lane holds one row; the products are
// folded as in the first event's kernel (class maxima and a triple over block maxima; ties go to the f64 kernel).
// Column blocks wholly behind a wavefront's rows are skipped, the one block on the diagonal is masked.
// Rows that the f32 arithmetic cannot decide are queued for the f64 kernel (causal mode).
constexpr int kPfWaves = 4;
constexpr int kPfRowsPerWave = 32;
constexpr int kPfRows = kPfWaves * kPfRowsPerWave;      // 128 rows per workgroup
constexpr int kPfStage = 64;                            // keys per LDS stage

// 1/|k_i| (f32) of every live slot; 0 for zero keys and beyond len
template <typename T, int D>
__global__ __launch_bounds__(256) void slot_rnorm_kernel(const T* __restrict__ k, const int32_t* __restrict__ len,
                                                         float* __restrict__ rn, int capacity) {
  constexpr int EPL = 16 / (int)sizeof(T), LPS = D / EPL, RPB = 256 / LPS;
  const int unit = blockIdx.y, sub = threadIdx.x % LPS;
  const int r = blockIdx.x * RPB + threadIdx.x / LPS;
  const int n = len[unit];
  if (r >= capacity) return;
  float ss = 0.f;
  if (r < n) {
    const uint4 x = reinterpret_cast<const uint4*>(k)[((size_t)unit * capacity + r) * LPS + sub];
    if constexpr (sizeof(T) == 2) {
      const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a = bf16_lo(w[e]), b = bf16_hi(w[e]);
        ss = fmaf(a, a, ss);
        ss = fmaf(b, b, ss);
      }
    } else {
      const float w[4] = {__builtin_bit_cast(float, x.x), __builtin_bit_cast(float, x.y),
                          __builtin_bit_cast(float, x.z), __builtin_bit_cast(float, x.w)};
#pragma unroll
      for (int e = 0; e < 4; ++e) ss = fmaf(w[e], w[e], ss);
    }
  }
  ss = group_sum<LPS>(ss);
  if (sub == 0) rn[(size_t)unit * capacity + r] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
}

template <int D>
__global__ __launch_bounds__(kPfWaves* kWave) void prefill_near_kernel(MatchParams p) {
  constexpr int KS = D / 16, ROWB = D * 2, CHUNKS = ROWB / 16;
  constexpr int STAGE_BYTES = kPfStage * ROWB;
  constexpr int LOADS = kPfStage * CHUNKS / (kPfWaves * kWave);
  __shared__ __align__(16) unsigned char s_stage[2 * STAGE_BYTES];
  __shared__ __align__(16) float s_rn[2][kPfStage];

  const int unit = blockIdx.y;
  const int n = p.len[unit];
  const int r0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * kPfRows;   // the long rows first
  if (r0 >= n) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const unsigned char* kbytes = reinterpret_cast<const unsigned char*>(p.k) + (size_t)unit * p.capacity * ROWB;
  const float* rn_all = p.rnorm + (size_t)unit * p.capacity;
  const int row_lo = r0 + wave * kPfRowsPerWave;         // this wavefront's rows: row_lo .. row_lo + 31
  const int row = row_lo + l32;                          // this lane's row (both halves)
  const int n_cols = min(n, r0 + kPfRows) - 1;           // columns 0 .. n_cols - 1 are needed by some row here
  const int n_stage = (n_cols + kPfStage - 1) / kPfStage;

  auto issue_stage = [&](int s, int buf) {
    const int col0 = s * kPfStage;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int c = tid + i * (kPfWaves * kWave);
      const int r = c / CHUNKS, phys = c % CHUNKS;
      const size_t off = (size_t)min(col0 + r, n - 1) * ROWB + ((phys ^ (r & (CHUNKS - 1))) * 16);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kbytes + off),
                                       (__attribute__((address_space(3))) void*)(s_stage + buf * STAGE_BYTES +
                                                                               (i * (kPfWaves * kWave) + wave * 64) * 16),
                                       16, 0, 0);
    }
    if (wave == 0)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(rn_all + min(col0 + lane, n - 1)),
                                       (__attribute__((address_space(3))) void*)(&s_rn[buf][0]), 4, 0, 0);
  };
  if (n_stage > 0) issue_stage(0, 0);

  // B operands: this lane's row, its 8 channels of every k-step
  bf16x8_t e[KS];
  {
    const unsigned char* rp = kbytes + (size_t)min(row, n - 1) * ROWB + half * 16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) e[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(rp + ks * 32));
  }
  const float rn_row = rn_all[min(row, n - 1)];

  // Running state per lane (its row, its 16 columns of every 32-column block), as in the first event's kernel:
  // the best value of each column class i, and (best, second best, block) over the blocks' maxima, all as integer
  // images (the order of positive floats; a masked or negative value loses to the initial 0, and a row without
  // a positive similarity is queued for the f64 kernel or has no target anyway).  No column number travels
  // with the values: at the end the winning class is the one whose best equals the overall best and the
  // winning block is the triple's; every other column is bounded by the second-best block or another class.
  int cls[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) cls[i] = 0;
  int b1 = 0, b2 = 0, g1 = 0;
  int par = 0;
  for (int s = 0; s < n_stage; ++s) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                     // stage s has landed; everyone is done with stage s - 1
    if (s + 1 < n_stage) issue_stage(s + 1, par ^ 1);
    const int col0 = s * kPfStage;
#pragma unroll
    for (int cbl = 0; cbl < kPfStage / 32; ++cbl) {
      const int cb0 = col0 + 32 * cbl;                   // first column of the block
      if (cb0 >= row_lo + kPfRowsPerWave || cb0 >= n_cols) continue;   // uniform over the wavefront: nothing before a row
      f32x16_t acc = {0};
      const unsigned char* frag = s_stage + par * STAGE_BYTES + (32 * cbl + l32) * ROWB;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(frag + (((2 * ks + half) ^ (l32 & (CHUNKS - 1))) * 16));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, e[ks], acc, 0, 0, 0);
      }
      const bool diagonal = cb0 + 32 > row_lo;           // uniform: the block holds columns at or behind some row
      int gm = 0;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4_t rn4 = *reinterpret_cast<const f32x4_t*>(&s_rn[par][32 * cbl + 8 * g + 4 * half]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int k = __builtin_bit_cast(int, acc[4 * g + i] * rn4[i]);
          if (diagonal) {                                // only earlier columns count (and none beyond the last one needed)
            const int col = cb0 + 8 * g + 4 * half + i;
            k = (col < row && col < n_cols) ? k : 0;
          }
          cls[4 * g + i] = imax(cls[4 * g + i], k);
          gm = imax(gm, k);
        }
      }
      const int cb = cb0 >> 5;
      g1 = (gm > b1) ? cb : g1;                          // strict: the first of equal blocks stays
      b2 = imed3(b1, b2, gm);
      b1 = imax(b1, gm);
    }
    par ^= 1;
  }
  // winning class of this lane's half of the row, then the two lanes of a row (the halves) meet; equal values:
  // the lower column, and the margin is zero
  float best, second;
  int bcol;
  {
    int s1 = cls[0], s2 = 0, ci = 0;
#pragma unroll
    for (int i = 1; i < 16; ++i) {
      const int x = cls[i];
      const bool up = x > s1;
      s2 = up ? s1 : imax(s2, x);
      ci = up ? i : ci;
      s1 = up ? x : s1;
    }
    const int col = 32 * g1 + 8 * (ci / 4) + 4 * half + (ci % 4);
    const int rest = imax(b2, s2);                       // bounds every other column of this half
    const int o1 = __shfl_xor(s1, 32), orest = __shfl_xor(rest, 32), ocol = __shfl_xor(col, 32);
    best = __builtin_bit_cast(float, imax(s1, o1));
    bcol = (s1 > o1) ? col : ((o1 > s1) ? ocol : min(col, ocol));
    second = __builtin_bit_cast(float, imax(imax(rest, orest), imin(s1, o1)));
  }
  if (half != 0 || row >= n) return;
  const size_t o = (size_t)unit * p.max_evict + row;
  if (row == 0) {                                        // no earlier key
    p.match[o] = -1;
    if (p.sim_out != nullptr) p.sim_out[o] = -INFINITY;
    return;
  }
  const float cos1 = best * rn_row;
  bool fragile = !(best > 0.f) || !(rn_row > 0.f) || !(rn_row < INFINITY) || !((best - second) * rn_row > p.delta) ||
                 !(fabsf(cos1 - p.threshold) > p.delta);
  if (surely_below(p, (best <= 0.f) ? 0.f : cos1, rn_row, rn_row)) fragile = false;
  p.match[o] = (cos1 > p.threshold) ? bcol : -1;
  if (p.sim_out != nullptr) p.sim_out[o] = cos1;
  if (fragile) {
    const int at = atomicAdd(p.flag_count, 1);
    p.flag_rows[at] = (int)o;
  }
}

// queue every live row but the first (f32 caches: the f64 kernel decides all rows)
__global__ void flag_all_causal_kernel(const int32_t* __restrict__ len, int32_t* flag_count, int32_t* flag_rows,
                                       int32_t* near, float* sim_out, int capacity) {
  const int unit = blockIdx.y;
  const int n = len[unit];
  for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x) {
    if (j == 0) {
      near[(size_t)unit * capacity] = -1;
      if (sim_out != nullptr) sim_out[(size_t)unit * capacity] = -INFINITY;
      continue;
    }
    const int at = atomicAdd(flag_count, 1);
    flag_rows[at] = unit * capacity + j;
  }
}

// The f64 kernel for bf16 caches.  Products of bf16 values are exact in f64 and so are their sums over the head
// dimension (for any ordinary exponent spread), whatever the order, so a key's channels may be split over lanes:
// four lanes share a key, each holding a quarter of the channels of the evicted row in registers (as f64) and
// loading the same quarter of the key, 64 keys per workgroup at a time and kExactBatch such rounds in flight.
// One workgroup per queued row, or per share of a row's columns when the queue is short (joined by a ticket, as
// in the generic kernel below).  The first event reads the retained keys from the gathered panel (no slot
// list to wait for); otherwise the slot numbers of a whole batch are requested first, then their rows.
constexpr int kExactBatch = 4;
template <int D>
__global__ __launch_bounds__(256) void match_exact_bf16_kernel(MatchParams p) {
  constexpr int ROWB = D * 2, CHUNKS = ROWB / 16, CPL = CHUNKS / 4, EPL = CPL * 8;   // chunks / channels per lane
  __shared__ double s_best[4];
  __shared__ int s_bestc[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int quad = tid >> 2, sub = tid & 3;
  const int n_flag = *p.flag_count;
  int rows_finished = 0;                 // (thread 0) queued rows whose result this workgroup has written
  const unsigned char* kall = reinterpret_cast<const unsigned char*>(p.k);
  int parts = 1;
  {
    const int room = imin((int)gridDim.x, kExactResident);
    while (parts < kExactMaxParts && (long)n_flag * (parts * 2) <= (long)room) parts *= 2;
  }
  for (int w = blockIdx.x; w < n_flag * parts; w += gridDim.x) {
    const int f = w / parts, part = w % parts;
    const int o = p.flag_rows[f];
    const int unit = o / p.max_evict, j = o % p.max_evict;
    const unsigned char* kunit = kall + (size_t)unit * p.capacity * ROWB;
    const int32_t* keep = p.causal ? nullptr : p.keep_idx + (size_t)unit * p.budget;
    const unsigned char* panel = (p.panel != nullptr && !p.causal) ? p.panel + (size_t)unit * p.rn_pitch * ROWB : nullptr;
    const int n_cols = p.causal ? j : p.budget;
    const int share = (n_cols + parts - 1) / parts;
    const int c_lo = part * share, c_hi = imin(n_cols, c_lo + share);
    // this lane's quarter of the evicted row (its slot number is one more round trip; the keys below do not wait for it)
    const int e = p.causal ? j : p.evict_idx[(size_t)unit * p.max_evict + j];
    uint4 ev[CPL];
#pragma unroll
    for (int q = 0; q < CPL; ++q) ev[q] = *reinterpret_cast<const uint4*>(kunit + (size_t)e * ROWB + (sub * CPL + q) * 16);
    double ed[EPL];
    double ss_e = 0.0;
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
      const uint32_t wv[4] = {ev[q].x, ev[q].y, ev[q].z, ev[q].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ed[q * 8 + 2 * i] = (double)bf16_lo(wv[i]);
        ed[q * 8 + 2 * i + 1] = (double)bf16_hi(wv[i]);
        ss_e = fma(ed[q * 8 + 2 * i], ed[q * 8 + 2 * i], ss_e);
        ss_e = fma(ed[q * 8 + 2 * i + 1], ed[q * 8 + 2 * i + 1], ss_e);
      }
    }
    ss_e += __shfl_xor(ss_e, 1);
    ss_e += __shfl_xor(ss_e, 2);
    const double rn_e = 1.0 / sqrt(ss_e);
    double best = -INFINITY;
    int best_c = 0x7FFFFFFF;
    for (int c0 = c_lo; c0 < c_hi; c0 += 64 * kExactBatch) {
      int slot[kExactBatch];
      uint4 row[kExactBatch][CPL];
      if (panel == nullptr) {
#pragma unroll
        for (int b = 0; b < kExactBatch; ++b) {
          const int c = c0 + b * 64 + quad;
          slot[b] = (c < c_hi) ? (p.causal ? c : keep[c]) : -1;
        }
      }
#pragma unroll
      for (int b = 0; b < kExactBatch; ++b) {
        const int c = c0 + b * 64 + quad;
        if (panel != nullptr) {                  // key c of the list, its chunk ch stored at position ch ^ (c mod CHUNKS)
          slot[b] = c < c_hi ? c : -1;
          const unsigned char* rp = panel + (size_t)imin(c, n_cols - 1) * ROWB;
#pragma unroll
          for (int q = 0; q < CPL; ++q)
            row[b][q] = *reinterpret_cast<const uint4*>(rp + (((sub * CPL + q) ^ (imin(c, n_cols - 1) & (CHUNKS - 1))) * 16));
        } else {
          const unsigned char* rp = kunit + (size_t)imax(slot[b], 0) * ROWB + sub * CPL * 16;
#pragma unroll
          for (int q = 0; q < CPL; ++q) row[b][q] = *reinterpret_cast<const uint4*>(rp + q * 16);
        }
      }
#pragma unroll
      for (int b = 0; b < kExactBatch; ++b) {
        double dot = 0.0, ss_c = 0.0;
#pragma unroll
        for (int q = 0; q < CPL; ++q) {
          const uint32_t wv[4] = {row[b][q].x, row[b][q].y, row[b][q].z, row[b][q].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const double lo = (double)bf16_lo(wv[i]), hi = (double)bf16_hi(wv[i]);
            dot = fma(ed[q * 8 + 2 * i], lo, dot);
            ss_c = fma(lo, lo, ss_c);
            dot = fma(ed[q * 8 + 2 * i + 1], hi, dot);
            ss_c = fma(hi, hi, ss_c);
          }
        }
        dot += __shfl_xor(dot, 1);
        ss_c += __shfl_xor(ss_c, 1);
        dot += __shfl_xor(dot, 2);
        ss_c += __shfl_xor(ss_c, 2);
        const double rn_c = 1.0 / sqrt(ss_c);
        double u = (dot * rn_e) * rn_c;
        if (!(fabs(u) <= 1.79e308)) u = -INFINITY;   // zero-norm keys (nan / inf) match nothing
        const int c = c0 + b * 64 + quad;
        if (slot[b] >= 0 && u > best) {              // ascending c per lane and strict: the first maximiser stays
          best = u;
          best_c = c;
        }
      }
    }
#pragma unroll
    for (int off = 4; off < 64; off <<= 1) {         // (the four lanes of a quad hold the same pair)
      const double ob = __shfl_xor(best, off);
      const int oc = __shfl_xor(best_c, off);
      if (ob > best || (ob == best && oc < best_c)) {
        best = ob;
        best_c = oc;
      }
    }
    __syncthreads();                                 // the previous row's shared values are no longer read
    if (lane == 0) {
      s_best[wave] = best;
      s_bestc[wave] = best_c;
    }
    __syncthreads();
    if (tid == 0) {
      for (int ww = 1; ww < 4; ++ww)
        if (s_best[ww] > best || (s_best[ww] == best && s_bestc[ww] < best_c)) {
          best = s_best[ww];
          best_c = s_bestc[ww];
        }
      bool finish = parts == 1;
      if (!finish) {
        ExactPartial* mine = p.exact_partial + w;    // with parts > 1 every workgroup has at most one work item
        __hip_atomic_store(&mine->best_bits, __builtin_bit_cast(unsigned long long, best), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&mine->best_c, best_c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // the two write-through stores have completed
        finish = __hip_atomic_fetch_add(&p.exact_ticket[f], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == parts - 1;
        if (finish) {                                // the last share of this row: join them, in list order
          best = -INFINITY;
          best_c = 0x7FFFFFFF;
          for (int q = 0; q < parts; ++q) {
            const ExactPartial* r = p.exact_partial + f * parts + q;
            const double rb = __builtin_bit_cast(double, __hip_atomic_load(&r->best_bits, __ATOMIC_RELAXED,
                                                                           __HIP_MEMORY_SCOPE_AGENT));
            const int rc = __hip_atomic_load(&r->best_c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (rb > best) {
              best = rb;
              best_c = rc;
            }
          }
          __hip_atomic_store(&p.exact_ticket[f], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
        }
      }
      if (finish) {
        p.match[o] = (best > (double)p.threshold) ? best_c : -1;
        if (p.sim_out != nullptr) p.sim_out[o] = (float)best;
        ++rows_finished;
      }
    }
  }
  exact_exit(p, n_flag, rows_finished);
}

template <int D>
constexpr size_t mfma_smem_bytes() {
  return 2 * (size_t)kStageCols * (D * 2) + 2 * kStageCols * sizeof(float);
}
inline size_t small_smem_bytes(int head_dim) {   // evicted rows, per-wavefront results, 1/|k_c| of a block per wavefront
  return (size_t)64 * head_dim * 2 + (size_t)kSmallWaves * 64 * 3 * 4 + (size_t)kSmallWaves * 32 * 4;
}
constexpr int kSmallMaxEvict = 256;   // up to this many evictable slots per head the column-split kernel is used
constexpr int kSmallMaxShares = 256;  // workgroups of that kernel when row blocks are shared (one per compute unit)

inline int rn_pitch_of(int budget) { return (budget + kStageCols - 1) / kStageCols * kStageCols; }

template <int D>
keepkv_status launch_bf16(const MatchParams& p, const void* k, unsigned units, hipStream_t st) {
  constexpr int rows_per_block = 256 / (D * 2 / 16);
  const bool small = p.max_evict <= kSmallMaxEvict;
  if (!small)   // the steady-state kernel forms its own norms
    rnorm_kernel<uint16_t, D><<<dim3((p.rn_pitch + rows_per_block * kRnormRows - 1) / (rows_per_block * kRnormRows), units), 256, 0, st>>>(
        (const uint16_t*)k, p.keep_idx, p.n_evict, const_cast<float*>(p.rnorm), p.capacity, p.budget, p.rn_pitch,
        reinterpret_cast<uint4*>(const_cast<unsigned char*>(p.panel)));
  static const hipError_t a1 = hipFuncSetAttribute((const void*)match_mfma_kernel<D>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)mfma_smem_bytes<D>());
  static const hipError_t a2 = hipFuncSetAttribute((const void*)match_small_kernel<D>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   (int)small_smem_bytes(D));
  if (a1 != hipSuccess || a2 != hipSuccess) return KEEPKV_ERR_DEVICE;
  if (small) {
    // With few heads the row blocks alone leave most compute units idle, and one compute unit takes long to
    // pull a head's whole retained list: up to four workgroups share a row block, each over every fourth
    // batch of column blocks, as long as all of them are resident at once.
    const int row_blocks = (p.max_evict + 63) / 64, ncb = (p.budget + 31) / 32;
    int parts = 1;
    while (parts < kSmallMaxParts && (long)units * row_blocks * (parts * 2) <= kSmallMaxShares && parts * 2 * kSmallWaves < ncb + kSmallWaves)
      parts *= 2;
    MatchParams q = p;
    q.small_parts = parts;
    match_small_kernel<D><<<dim3(row_blocks, units, parts), kSmallWaves * kWave, small_smem_bytes(D), st>>>(q);
  } else {
    // One workgroup fills a compute unit (8 wavefronts of 256 registers).  With fewer heads than compute
    // units each head gets an equal share of them, and a workgroup walks its head's row blocks in passes;
    // with more heads than that, one workgroup per head does all passes.
    const unsigned row_blocks = (p.max_evict + kRowsPerBlock - 1) / kRowsPerBlock;
    unsigned per_unit = kResidentWorkgroups / units;
    per_unit = per_unit < 1 ? 1 : (per_unit > row_blocks ? row_blocks : per_unit);
    MatchParams q = p;
    q.per_unit = (int)per_unit;
    q.n_units = (int)units;
    match_mfma_kernel<D><<<per_unit * units, kMWaves * kWave, mfma_smem_bytes<D>(), st>>>(q);
  }
  return KEEPKV_OK;
}

}  // namespace

MatchPlan plan_match(const keepkv_layout* L, int capacity, int budget) {
  MatchPlan pl;
  const size_t units = (size_t)L->batch * L->n_kv_heads;
  pl.rnorm_off = kWorkspaceHead;
  pl.flag_off = kWorkspaceHead + align_up(units * rn_pitch_of(budget) * sizeof(float), 256);
  pl.panel_off = pl.flag_off + align_up((1 + units * (size_t)(capacity - budget)) * sizeof(int32_t) + 256, 256);
  // the panel is used by bf16 caches with more evictable slots than the column-split kernel takes
  const bool panel = L->dtype == KEEPKV_BF16 && capacity - budget > kSmallMaxEvict;
  pl.partial_off = pl.panel_off + (panel ? align_up(units * rn_pitch_of(budget) * (size_t)L->head_dim * 2, 256) : 0);
  pl.small_partial_off = pl.partial_off + (size_t)kExactResident * 16;
  pl.bytes = pl.small_partial_off + (size_t)kSmallMaxShares * 64 * 3 * sizeof(int32_t);
  return pl;
}

PrefillMatchPlan plan_prefill_match(const keepkv_layout* L, int capacity) {
  PrefillMatchPlan pl;
  const size_t units = (size_t)L->batch * L->n_kv_heads;
  pl.rnorm_off = kWorkspaceHead;
  pl.flag_off = pl.rnorm_off + align_up(units * capacity * sizeof(float), 256);
  pl.partial_off = pl.flag_off + align_up((1 + units * (size_t)capacity) * sizeof(int32_t) + 256, 256);
  pl.bytes = pl.partial_off + (size_t)kExactResident * 16;
  return pl;
}

}  // namespace kk

extern "C" keepkv_status keepkv_prefill_match(const keepkv_layout* layout, const keepkv_cache* cache, float threshold,
                                              int32_t* near, float* sim_out, void* workspace, size_t workspace_bytes,
                                              void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !near) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (!(threshold == threshold) || !aligned16(cache->k)) return KEEPKV_ERR_INVALID_ARG;
  if (layout->head_dim != 64 && layout->head_dim != 128) return KEEPKV_ERR_UNSUPPORTED;
  const size_t units = (size_t)layout->batch * layout->n_kv_heads;
  const int cap = cache->capacity;
  if (units * (size_t)cap >= (size_t)1 << 31) return KEEPKV_ERR_UNSUPPORTED;
  const PrefillMatchPlan pl = plan_prefill_match(layout, cap);
  if (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace)) return KEEPKV_ERR_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);

  MatchParams p;
  p.k = cache->k; p.keep_idx = nullptr; p.evict_idx = nullptr; p.n_evict = nullptr;
  p.rnorm = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + pl.rnorm_off);
  p.panel = nullptr;
  p.flag_count = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + kMatchCountersOff);
  p.exact_done = p.flag_count + 1;
  p.flag_rows = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.flag_off);
  p.exact_partial = reinterpret_cast<ExactPartial*>(reinterpret_cast<char*>(workspace) + pl.partial_off);
  p.exact_ticket = reinterpret_cast<int32_t*>(workspace);
  p.match = near; p.sim_out = sim_out;
  p.capacity = cap; p.budget = 0; p.max_evict = cap; p.rn_pitch = cap;
  p.threshold = threshold; p.delta = 1.6e-5f;
  p.per_unit = 0; p.n_units = 0; p.small_parts = 1; p.small_partial = nullptr;
  p.causal = 1; p.len = cache->len;

  long eb = (long)units * cap / 16;
  const int exact_blocks = (int)(eb < 64 ? 64 : (eb > 512 ? 512 : eb));
  if (layout->dtype == KEEPKV_BF16) {
    const int lps = layout->head_dim * 2 / 16, rpb = 256 / lps;
    const dim3 ngrid((cap + rpb - 1) / rpb, (unsigned)units);
    const dim3 pgrid((cap + kPfRows - 1) / kPfRows, (unsigned)units);
    if (layout->head_dim == 128) {
      slot_rnorm_kernel<uint16_t, 128><<<ngrid, 256, 0, st>>>((const uint16_t*)cache->k, cache->len,
                                                            const_cast<float*>(p.rnorm), cap);
      prefill_near_kernel<128><<<pgrid, kPfWaves * kWave, 0, st>>>(p);
      match_exact_bf16_kernel<128><<<exact_blocks, 256, 0, st>>>(p);
    } else {
      slot_rnorm_kernel<uint16_t, 64><<<ngrid, 256, 0, st>>>((const uint16_t*)cache->k, cache->len,
                                                           const_cast<float*>(p.rnorm), cap);
      prefill_near_kernel<64><<<pgrid, kPfWaves * kWave, 0, st>>>(p);
      match_exact_bf16_kernel<64><<<exact_blocks, 256, 0, st>>>(p);
    }
  } else {
    int bx = (cap + 255) / 256;
    if (bx > 64) bx = 64;
    flag_all_causal_kernel<<<dim3(bx, (unsigned)units), 256, 0, st>>>(cache->len, p.flag_count, p.flag_rows, near, sim_out, cap);
    if (layout->head_dim == 128) match_exact_kernel<float, 128><<<exact_blocks, 256, 0, st>>>(p);
    else match_exact_kernel<float, 64><<<exact_blocks, 256, 0, st>>>(p);
  }
  return launch_status();
}

extern "C" keepkv_status keepkv_match(const keepkv_layout* layout, const keepkv_cache* cache, int32_t budget,
                                      const int32_t* keep_idx, const int32_t* evict_idx, const int32_t* n_evict,
                                      float threshold, int32_t* match, float* sim_out, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  using namespace kk;
  if (!layout_ok(layout) || !cache_ok(cache) || !keep_idx || !n_evict) return KEEPKV_ERR_INVALID_ARG;
  if (!units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  if (budget < 1 || budget > cache->capacity) return KEEPKV_ERR_INVALID_ARG;
  const int max_evict = cache->capacity - budget;
  if (max_evict == 0) return KEEPKV_OK;   // nothing can be evicted
  if (!evict_idx || !match) return KEEPKV_ERR_INVALID_ARG;
  if (!(threshold == threshold)) return KEEPKV_ERR_INVALID_ARG;
  if (!aligned16(cache->k)) return KEEPKV_ERR_INVALID_ARG;
  if (layout->head_dim != 64 && layout->head_dim != 128) return KEEPKV_ERR_UNSUPPORTED;
  if (budget > 4096) return KEEPKV_ERR_UNSUPPORTED;
  const size_t units = (size_t)layout->batch * layout->n_kv_heads;
  if (units * (size_t)max_evict >= (size_t)1 << 31) return KEEPKV_ERR_UNSUPPORTED;
  const MatchPlan pl = plan_match(layout, cache->capacity, budget);
  if (!workspace || workspace_bytes < pl.bytes || !aligned16(workspace)) return KEEPKV_ERR_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);

  MatchParams p;
  p.k = cache->k; p.keep_idx = keep_idx; p.evict_idx = evict_idx; p.n_evict = n_evict;
  p.rnorm = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + pl.rnorm_off);
  // queue counter and the f64 kernel's exit counter: control words, zero between calls
  p.flag_count = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + kMatchCountersOff);
  p.exact_done = p.flag_count + 1;
  p.flag_rows = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.flag_off);
  p.panel = reinterpret_cast<const unsigned char*>(workspace) + pl.panel_off;
  p.exact_partial = reinterpret_cast<ExactPartial*>(reinterpret_cast<char*>(workspace) + pl.partial_off);
  p.exact_ticket = reinterpret_cast<int32_t*>(workspace);
  p.causal = 0; p.len = cache->len;
  p.small_parts = 1;
  p.small_partial = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + pl.small_partial_off);
  p.match = match; p.sim_out = sim_out;
  p.capacity = cache->capacity; p.budget = budget; p.max_evict = max_evict;
  p.threshold = threshold;
  p.per_unit = 0; p.n_units = 0;   // set by the first event's launch
  // Margin below which the f32 result does not decide a row.  An f32 similarity carries the accumulation of
  // D exact products (at most D * 2^-24 relative to |k_e||k_c|, far less in practice) and the roundings of
  // the two norms; what is compared are two such values, or one and the threshold.
  p.delta = 1.6e-5f;

  p.rn_pitch = rn_pitch_of(budget);
  long eb = (long)units * max_evict / 16;      // queued rows are a small fraction of all rows
  const int exact_blocks = (int)(eb < 64 ? 64 : (eb > 512 ? 512 : eb));
  if (max_evict <= kSmallMaxEvict || layout->dtype != KEEPKV_BF16) p.panel = nullptr;   // only the first event's path gathers it
  if (layout->dtype == KEEPKV_BF16) {
    keepkv_status rc;
    if (layout->head_dim == 128) {
      rc = launch_bf16<128>(p, cache->k, (unsigned)units, st);
      if (rc != KEEPKV_OK) return rc;
      match_exact_bf16_kernel<128><<<exact_blocks, 256, 0, st>>>(p);
    } else {
      rc = launch_bf16<64>(p, cache->k, (unsigned)units, st);
      if (rc != KEEPKV_OK) return rc;
      match_exact_bf16_kernel<64><<<exact_blocks, 256, 0, st>>>(p);
    }
  } else {
    int bx = (max_evict + 255) / 256;
    if (bx > 64) bx = 64;
    flag_all_kernel<<<dim3(bx, (unsigned)units), 256, 0, st>>>(n_evict, p.flag_count, p.flag_rows, max_evict);
    if (layout->head_dim == 128) match_exact_kernel<float, 128><<<exact_blocks, 256, 0, st>>>(p);
    else match_exact_kernel<float, 64><<<exact_blocks, 256, 0, st>>>(p);
  }
  return launch_status();
}

#ifdef KEEPKV_TRACE
extern "C" int keepkv_trace_read_match(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(kk::kk_trace_match), sizeof(long long) * n);
}
#endif
