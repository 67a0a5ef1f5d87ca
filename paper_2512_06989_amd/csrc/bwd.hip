// placeholder until the fused backward kernels land
#include "mhffn_device.h"
#include "mhffn_internal.h"
namespace mhffn {
size_t bwd_workspace_bytes(const Problem&, int) { return 0; }
int launch_bwd(const Problem&, int, const void*, const void*, const void*, const void*, const void*,
               const void*, void*, void*, void*, void*, void*, void*, void*) { return -1; }
}  // namespace mhffn
