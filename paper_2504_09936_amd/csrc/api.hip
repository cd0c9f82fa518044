// Host-only entry points of the KeepKV C ABI: status names, version, workspace sizing.
#include "kk_common.hpp"

extern "C" const char* keepkv_strerror(keepkv_status st) {
  switch (st) {
    case KEEPKV_OK: return "ok";
    case KEEPKV_ERR_INVALID_ARG: return "invalid argument";
    case KEEPKV_ERR_UNSUPPORTED: return "unsupported shape";
    case KEEPKV_ERR_WORKSPACE: return "workspace missing or too small";
    case KEEPKV_ERR_DEVICE: return "device launch error";
  }
  return "unknown status";
}

extern "C" int32_t keepkv_version(void) { return 101; }

namespace {
__global__ void clear_head_kernel(int32_t* w, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) w[i] = 0;
}
}  // namespace

extern "C" keepkv_status keepkv_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  using namespace kk;
  if (!workspace || !aligned16(workspace) || workspace_bytes < kWorkspaceHead) return KEEPKV_ERR_WORKSPACE;
  const int n = (int)(kWorkspaceHead / sizeof(int32_t));
  clear_head_kernel<<<(n + 255) / 256, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(
      reinterpret_cast<int32_t*>(workspace), n);
  return launch_status();
}

extern "C" keepkv_status keepkv_decode_plan(const keepkv_layout* layout, int32_t capacity, int32_t* n_split,
                                            int32_t* slots_per_split, int32_t* wavefronts) {
  using namespace kk;
  if (!layout_ok(layout) || capacity < 1 || capacity > (1 << 20)) return KEEPKV_ERR_INVALID_ARG;
  if (!layout_supported(layout) || !units_supported(layout)) return KEEPKV_ERR_UNSUPPORTED;
  const DecodePlan pl = plan_decode(layout, capacity);
  if (n_split) *n_split = pl.nsplit;
  if (slots_per_split) *slots_per_split = pl.per;
  if (wavefronts) *wavefronts = layout->dtype == KEEPKV_BF16 ? pl.waves : 4;
  return KEEPKV_OK;
}

extern "C" size_t keepkv_workspace_bytes(const keepkv_layout* layout, int32_t capacity, int32_t budget) {
  using namespace kk;
  if (!layout_ok(layout) || capacity < 1 || capacity > (1 << 20) || budget < 1 || budget > capacity) return 0;
  size_t need = plan_decode(layout, capacity).bytes;
  const size_t s = plan_select(layout, capacity).bytes;
  const size_t m = plan_match(layout, capacity, budget).bytes;
  const size_t g = plan_merge(layout, capacity, budget).bytes;
  need = need > s ? need : s;
  need = need > m ? need : m;
  need = need > g ? need : g;
  const size_t pm = plan_prefill_match(layout, capacity).bytes;
  const size_t pg = plan_prefill_merge(layout, capacity).bytes;
  need = need > pm ? need : pm;
  need = need > pg ? need : pg;
  return need;
}
