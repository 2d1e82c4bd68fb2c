// Host-only parts of the C ABI: status strings and workspace sizing.
#include "aero_device.h"

namespace aero {
size_t loss_workspace_bytes(int64_t T);
size_t fused_workspace_bytes(int64_t T, int32_t V, int32_t H);
}  // namespace aero

extern "C" const char* aero_status_string(aero_status s) {
  switch (s) {
    case AERO_OK: return "ok";
    case AERO_ERR_NULL: return "a required pointer is NULL";
    case AERO_ERR_SHAPE: return "invalid size or leading dimension";
    case AERO_ERR_DTYPE: return "unsupported dtype";
    case AERO_ERR_ALIGN: return "pointer or leading dimension is misaligned";
    case AERO_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case AERO_ERR_HIP: return "HIP launch failed";
    case AERO_ERR_LIMIT: return "size exceeds the fixed capacity of this entry point";
    default: return "unknown status";
  }
}

extern "C" size_t aero_workspace_bytes(int32_t op, int64_t T, int32_t V, int32_t H, int32_t R, int32_t Q) {
  (void)R;
  (void)Q;
  if (T < 0) return 0;
  switch (op) {
    case AERO_OP_GRPO_LOSS_BWD: return aero::loss_workspace_bytes(T);
    case AERO_OP_LMHEAD_FUSED: return aero::fused_workspace_bytes(T, V, H);
    default: return 0;
  }
}
