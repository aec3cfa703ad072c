// Host-side internals shared by the library's host sources (not part of the C ABI, never included by device code
// headers): the plan object, error reporting and small helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "st_internal.h"

namespace st {

// Sets the thread-local message returned by st_last_error_message() and returns `s`.
st_status fail(st_status s, const char* fmt, ...);
st_status hip_fail(hipError_t e, const char* what);

inline int elem_size(int dt) { return dt == ST_DT_F32 ? 4 : 2; }
inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

}  // namespace st

#define ST_HIP(call)                                       \
  do {                                                     \
    hipError_t e_ = (call);                                \
    if (e_ != hipSuccess) return st::hip_fail(e_, #call);  \
  } while (0)

struct st_plan {
  std::vector<st_conv_desc> descs;
  std::vector<st_tenant_info> info;
  std::vector<st::TenantDev> tenants;       // host mirror of the device table
  std::vector<st_work_item> items_fused;    // order of the fused launch
  std::vector<st_work_item> items_tenant;   // tenant-major, sliced by the baselines
  bool host_only = false;
  int64_t flops = 0, bytes = 0, workspace_bytes = 0;
  int64_t ws_floats = 0, n_counters = 0;    // split-K: fp32 elements of all partial tiles, arrival counters
  // device
  st::TenantDev* d_tenants = nullptr;
  st_work_item* d_items_fused = nullptr;
  st_work_item* d_items_tenant = nullptr;
  char* d_arena = nullptr;                  // the one device allocation the four pointers below point into
  char* d_workspace = nullptr;              // split-K counters, then all tenants' partial tiles
  hipEvent_t ev_fork = nullptr;
  std::vector<hipEvent_t> ev_join;          // one per stream slot used by space-only
  // pinned staging slots for stream-ordered uploads of the tenant table (st_conv_plan_rebind_all)
  static constexpr int kStageSlots = 4;
  st::TenantDev* h_stage[kStageSlots] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t ev_stage[kStageSlots] = {nullptr, nullptr, nullptr, nullptr};
  bool stage_used[kStageSlots] = {false, false, false, false};
  int stage_next = 0;
};
