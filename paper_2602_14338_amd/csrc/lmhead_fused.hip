// LM head fused into the softmax statistics and the loss gradients (work in progress).
#include "aero_device.h"
namespace aero {
size_t fused_workspace_bytes(int64_t T, int32_t V, int32_t H) { return 0; }
}
