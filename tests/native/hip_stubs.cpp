// Host-only stand-ins for the functions that touch the GPU, so that the planner and the C ABI can be
// built with AddressSanitizer / UBSan and exercised on a machine without a GPU.  Test code only.
#include "tpx_internal.hpp"

namespace tpx {
tpx_status hip_upload_tables(void*, const tpx_plan_s&, void*) { return fail(TPX_ERR_HIP, "stub: no GPU in this build"); }
tpx_status hip_launch_tiles(const void*, const tpx_plan_s&, const void* const*, uint32_t, void* const*, uint32_t, uint64_t, void*) {
  return fail(TPX_ERR_HIP, "stub: no GPU in this build");
}
tpx_status hip_probe_copy(void*, const void*, uint64_t, void*) { return fail(TPX_ERR_HIP, "stub: no GPU in this build"); }
tpx_status hip_probe_read(const void*, uint64_t, void*, void*) { return fail(TPX_ERR_HIP, "stub: no GPU in this build"); }
tpx_status hip_probe_fill(void*, uint64_t, uint32_t, void*) { return fail(TPX_ERR_HIP, "stub: no GPU in this build"); }
tpx_status hip_execute_static(const tpx_plan_s&, const void* const*, uint32_t, void* const*, uint32_t, uint64_t, void*) {
  return fail(TPX_ERR_HIP, "stub: no GPU in this build");
}
tpx_status hip_read_header(const void*, void*, WorkspaceHeader*) { return fail(TPX_ERR_HIP, "stub: no GPU in this build"); }
}  // namespace tpx
