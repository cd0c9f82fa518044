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

extern "C" int32_t keepkv_version(void) { return 100; }

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
  return need;
}
