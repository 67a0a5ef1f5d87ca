// C ABI of the fused Multi-Head FFN library: argument validation on the host,
// then dispatch to the gfx950 kernels.  Nothing here allocates, synchronises or
// keeps data between calls; see include/mhffn.h for the contract.
#include "../../include/mhffn.h"

#include "mhffn_device.h"
#include "mhffn_internal.h"

#include <mutex>

// Scratch of mhffn_forward_static: one copy per GPU that the library runs on, held until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress, never
// a device address; kernels get the per-device address resolved below.
static __device__ __align__(256) unsigned char scratch[MHFFN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the calling thread's current device, resolved once per device.
int static_scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MHFFN_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MHFFN_ERR_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MHFFN_OK;
}
}  // namespace

namespace mhffn {
LdsKernelEntry*& lds_kernel_list() {
  static LdsKernelEntry* head = nullptr;   // constant-initialised: safe during static initialisation
  return head;
}
}  // namespace mhffn

namespace {

using mhffn::Problem;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elt_size(int dtype) { return dtype == MHFFN_BF16 ? 2 : 4; }

// Descriptor checks common to all entry points.
int check_desc(const mhffn_desc* d, Problem* p) {
  if (!d) return MHFFN_ERR_NULL;
  if (d->n_tokens < 0 || d->n_heads < 1 || d->d_head < 1 || d->n_sub < 1 || d->d_sub < 1)
    return MHFFN_ERR_SHAPE;
  if (d->dtype != MHFFN_F32 && d->dtype != MHFFN_BF16) return MHFFN_ERR_UNSUPPORTED;
  if (d->route_mode != MHFFN_ROUTE_PARAMS && d->route_mode != MHFFN_ROUTE_WEIGHTS)
    return MHFFN_ERR_UNSUPPORTED;
  if (!(d->eps >= 0.0f)) return MHFFN_ERR_SHAPE;  // also rejects NaN
  const int64_t dm = (int64_t)d->n_heads * d->d_head;
  if ((d->ld_x != 0 && d->ld_x < dm) || (d->ld_y != 0 && d->ld_y < dm)) return MHFFN_ERR_SHAPE;
  // sizes whose products would not fit the index arithmetic of the kernels
  if (d->n_tokens > ((int64_t)1 << 40) || dm > (1 << 24) ||
      (int64_t)d->n_sub * d->d_sub > (1 << 24))
    return MHFFN_ERR_SHAPE;
  p->N = d->n_tokens;
  p->H = d->n_heads; p->dh = d->d_head; p->E = d->n_sub; p->de = d->d_sub;
  p->ldx = d->ld_x ? d->ld_x : dm;
  p->ldy = d->ld_y ? d->ld_y : dm;
  p->route_mode = d->route_mode;
  p->eps = d->eps;
  const size_t es = elt_size(d->dtype);
  if ((p->ldx * es) % 16 != 0 || (p->ldy * es) % 16 != 0) return MHFFN_ERR_ALIGN;
  return MHFFN_OK;
}

// Can the fused kernels run this shape?
int check_fused_shape(const mhffn_desc* d, const Problem& p, bool backward = false) {
  if (d->dtype == MHFFN_BF16) {
    if ((p.dh != 64 && p.dh != 128 && p.dh != 256) || p.de % 32 != 0 || p.E > mhffn::kFwdBf16MaxSub)
      return MHFFN_ERR_UNSUPPORTED;
    if (backward && p.E > mhffn::bwd_bf16_max_sub(p)) return MHFFN_ERR_UNSUPPORTED;
    const size_t lds = backward ? mhffn::bwd_bf16_lds_bytes(p) : mhffn::fwd_bf16_lds_bytes(p);
    if (lds > mhffn::kLdsBytesPerWorkgroup) return MHFFN_ERR_UNSUPPORTED;
  } else {
    if (p.dh % 4 != 0 || p.dh > 256) return MHFFN_ERR_UNSUPPORTED;
    const size_t lds = backward ? mhffn::bwd_f32_lds_bytes(p) : mhffn::fwd_f32_lds_bytes(p);
    if (lds > mhffn::kLdsBytesPerWorkgroup) return MHFFN_ERR_UNSUPPORTED;
  }
  return MHFFN_OK;
}

int check_workspace(size_t need, const void* ws, size_t have) {
  if (need == 0) return MHFFN_OK;
  if (!ws || have < need) return MHFFN_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MHFFN_ERR_ALIGN;
  return MHFFN_OK;
}

}  // namespace

extern "C" {

const char* mhffn_status_string(int status) {
  switch (status) {
    case MHFFN_OK: return "ok";
    case MHFFN_ERR_NULL: return "a required pointer is NULL";
    case MHFFN_ERR_SHAPE: return "invalid size or stride";
    case MHFFN_ERR_UNSUPPORTED: return "shape, dtype or mode not supported by this kernel set";
    case MHFFN_ERR_ALIGN: return "pointer or stride not 16-byte aligned (workspace: 256)";
    case MHFFN_ERR_WORKSPACE: return "workspace missing or too small";
    case MHFFN_ERR_LAUNCH: return "HIP kernel launch failed";
    case MHFFN_ERR_STATIC_SCRATCH: return "problem needs more scratch than the library's static buffer holds";
    default: return "unknown status";
  }
}

const char* mhffn_version(void) { return "mhffn-gfx950 0.2"; }

int mhffn_init(void) {
  for (mhffn::LdsKernelEntry* e = mhffn::lds_kernel_list(); e; e = e->next)
    if (e->ensure() != hipSuccess) return MHFFN_ERR_LAUNCH;
  void* p = nullptr;
  return static_scratch_address(&p);
}

size_t mhffn_workspace_bytes(const mhffn_desc* desc, int op) {
  Problem p;
  if (check_desc(desc, &p) != MHFFN_OK) return 0;
  switch (op) {
    case MHFFN_OP_FORWARD:
      if (desc->dtype != MHFFN_BF16 || check_fused_shape(desc, p) != MHFFN_OK) return 0;
      return mhffn::fwd_bf16_workspace_bytes(p);
    case MHFFN_OP_BACKWARD:
      if (check_fused_shape(desc, p, true) != MHFFN_OK) return 0;
      return mhffn::bwd_workspace_bytes(p, desc->dtype);
    case MHFFN_OP_MODULE_FORWARD:
      if (p.route_mode != MHFFN_ROUTE_PARAMS || check_fused_shape(desc, p) != MHFFN_OK) return 0;
      return mhffn::module_workspace_bytes(p, desc->dtype, false);
    case MHFFN_OP_MODULE_BACKWARD:
      if (p.route_mode != MHFFN_ROUTE_PARAMS || check_fused_shape(desc, p, true) != MHFFN_OK) return 0;
      return mhffn::module_workspace_bytes(p, desc->dtype, true);
    case MHFFN_OP_UNFUSED_FORWARD: return mhffn::unfused_workspace_bytes(p, desc->dtype, false);
    case MHFFN_OP_UNFUSED_BACKWARD: return mhffn::unfused_workspace_bytes(p, desc->dtype, true);
    default: return 0;
  }
}

namespace {
// Common part of mhffn_forward and mhffn_forward_static.  `static_scratch`: take the scratch
// from the library's static device buffer instead of the caller's workspace.
int forward_impl(const mhffn_desc* desc, const void* X, const void* W_gate, const void* W_up,
                 const void* W_down, const void* route, void* Y, void* workspace,
                 size_t workspace_bytes, void* hip_stream, bool static_scratch) {
  Problem p;
  int rc = check_desc(desc, &p);
  if (rc) return rc;
  // an empty batch has no rows: X and Y (and R, in weights mode) may then be NULL
  const bool empty = (p.N == 0);
  if (!W_gate || !W_up || !W_down) return MHFFN_ERR_NULL;
  if (!empty && (!X || !Y || !route)) return MHFFN_ERR_NULL;
  if (!route && p.route_mode == MHFFN_ROUTE_PARAMS) return MHFFN_ERR_NULL;
  if (!aligned16(X) || !aligned16(W_gate) || !aligned16(W_up) || !aligned16(W_down) ||
      !aligned16(route) || !aligned16(Y))
    return MHFFN_ERR_ALIGN;
  rc = check_fused_shape(desc, p);
  if (rc) return rc;
  if (p.N == 0) return MHFFN_OK;
  if (desc->dtype == MHFFN_BF16) {
    // non-zero only for small N, where the intermediate dimension is split over workgroups
    const size_t need = mhffn::fwd_bf16_workspace_bytes(p);
    if (static_scratch) {
      if (need > (size_t)MHFFN_STATIC_SCRATCH_BYTES) return MHFFN_ERR_STATIC_SCRATCH;
      workspace = nullptr;
      if (need) {
        rc = static_scratch_address(&workspace);
        if (rc) return rc;
      }
    } else {
      rc = check_workspace(need, workspace, workspace_bytes);
      if (rc) return rc;
    }
  }
  const int e = (desc->dtype == MHFFN_BF16)
                    ? mhffn::launch_fwd_bf16(p, X, W_gate, W_up, W_down, route, Y, workspace,
                                             hip_stream)
                    : mhffn::launch_fwd_f32(p, X, W_gate, W_up, W_down, route, Y, hip_stream);
  return e == 0 ? MHFFN_OK : MHFFN_ERR_LAUNCH;
}
}  // namespace

int mhffn_forward(const mhffn_desc* desc, const void* X, const void* W_gate, const void* W_up,
                  const void* W_down, const void* route, void* Y, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  return forward_impl(desc, X, W_gate, W_up, W_down, route, Y, workspace, workspace_bytes,
                      hip_stream, false);
}

int mhffn_forward_static(const mhffn_desc* desc, const void* X, const void* W_gate,
                         const void* W_up, const void* W_down, const void* route, void* Y,
                         void* hip_stream) {
  return forward_impl(desc, X, W_gate, W_up, W_down, route, Y, nullptr, 0, hip_stream, true);
}

int mhffn_backward(const mhffn_desc* desc, const void* X, const void* W_gate, const void* W_up,
                   const void* W_down, const void* route, const void* dY, void* dX,
                   void* dW_gate, void* dW_up, void* dW_down, void* d_route, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  return mhffn_backward_phases(desc, X, W_gate, W_up, W_down, route, dY, dX, dW_gate, dW_up,
                               dW_down, d_route, workspace, workspace_bytes, hip_stream, nullptr, 0);
}

int mhffn_backward_phases(const mhffn_desc* desc, const void* X, const void* W_gate,
                          const void* W_up, const void* W_down, const void* route,
                          const void* dY, void* dX, void* dW_gate, void* dW_up, void* dW_down,
                          void* d_route, void* workspace, size_t workspace_bytes,
                          void* hip_stream, void* const* phase_events, int n_phase_events) {
  if (n_phase_events < 0 || (n_phase_events > 0 && !phase_events)) return MHFFN_ERR_NULL;
  Problem p;
  int rc = check_desc(desc, &p);
  if (rc) return rc;
  const bool empty = (p.N == 0);  // no rows: X, dY, dX (and R) may be NULL
  if (!W_gate || !W_up || !W_down) return MHFFN_ERR_NULL;
  if (!empty && (!X || !dY || !route)) return MHFFN_ERR_NULL;
  if (!route && p.route_mode == MHFFN_ROUTE_PARAMS) return MHFFN_ERR_NULL;
  const void* ptrs[] = {X, W_gate, W_up, W_down, route, dY, dX, dW_gate, dW_up, dW_down, d_route};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MHFFN_ERR_ALIGN;
  rc = check_fused_shape(desc, p, true);
  if (rc) return rc;
  rc = check_workspace(mhffn::bwd_workspace_bytes(p, desc->dtype), workspace, workspace_bytes);
  if (rc) return rc;
  const int e = mhffn::launch_bwd(p, desc->dtype, X, W_gate, W_up, W_down, route, dY, dX, dW_gate,
                                  dW_up, dW_down, d_route, workspace, hip_stream, phase_events,
                                  n_phase_events);
  if (e == -1) return MHFFN_ERR_UNSUPPORTED;
  return e == 0 ? MHFFN_OK : MHFFN_ERR_LAUNCH;
}

int mhffn_reference_unfused(const mhffn_desc* desc, const void* X, const void* W_gate,
                            const void* W_up, const void* W_down, const void* route, void* Y,
                            const void* dY, void* dX, void* dW_gate, void* dW_up, void* dW_down,
                            void* d_route, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  Problem p;
  int rc = check_desc(desc, &p);
  if (rc) return rc;
  const bool empty = (p.N == 0);
  if (!W_gate || !W_up || !W_down) return MHFFN_ERR_NULL;
  if (!empty && (!X || !Y || !route)) return MHFFN_ERR_NULL;
  if (!route && p.route_mode == MHFFN_ROUTE_PARAMS) return MHFFN_ERR_NULL;
  const void* ptrs[] = {X, W_gate, W_up, W_down, route, Y, dY, dX, dW_gate, dW_up, dW_down, d_route};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MHFFN_ERR_ALIGN;
  if (p.dh % 8 != 0) return MHFFN_ERR_UNSUPPORTED;
  rc = check_workspace(mhffn::unfused_workspace_bytes(p, desc->dtype, dY != nullptr), workspace,
                       workspace_bytes);
  if (rc) return rc;
  const int e = mhffn::launch_unfused(p, desc->dtype, X, W_gate, W_up, W_down, route, Y, dY, dX,
                                      dW_gate, dW_up, dW_down, d_route, workspace, hip_stream);
  if (e == -1) return MHFFN_ERR_UNSUPPORTED;
  return e == 0 ? MHFFN_OK : MHFFN_ERR_LAUNCH;
}

int mhffn_module_forward(const mhffn_desc* desc, const void* X, const void* W_in,
                         const void* W_gate, const void* W_up, const void* W_down,
                         const void* W_r, const void* W_out, void* O, void* Q, void* S,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  Problem p;
  int rc = check_desc(desc, &p);
  if (rc) return rc;
  if (p.route_mode != MHFFN_ROUTE_PARAMS) return MHFFN_ERR_UNSUPPORTED;
  const bool empty = (p.N == 0);
  if (!W_in || !W_gate || !W_up || !W_down || !W_r || !W_out) return MHFFN_ERR_NULL;
  if (!empty && (!X || !O || !Q || !S)) return MHFFN_ERR_NULL;
  const void* ptrs[] = {X, W_in, W_gate, W_up, W_down, W_r, W_out, O, Q, S};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MHFFN_ERR_ALIGN;
  rc = check_fused_shape(desc, p);
  if (rc) return rc;
  if (empty) return MHFFN_OK;
  rc = check_workspace(mhffn::module_workspace_bytes(p, desc->dtype, false), workspace, workspace_bytes);
  if (rc) return rc;
  const int e = mhffn::launch_module_forward(p, desc->dtype, X, W_in, W_gate, W_up, W_down, W_r,
                                             W_out, O, Q, S, workspace, hip_stream);
  return e == 0 ? MHFFN_OK : MHFFN_ERR_LAUNCH;
}

int mhffn_module_backward(const mhffn_desc* desc, const void* X, const void* W_in,
                          const void* W_gate, const void* W_up, const void* W_down,
                          const void* W_r, const void* W_out, const void* Q, const void* S,
                          const void* dO, void* dX, void* dW_in, void* dW_gate, void* dW_up,
                          void* dW_down, void* dW_r, void* dW_out, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  Problem p;
  int rc = check_desc(desc, &p);
  if (rc) return rc;
  if (p.route_mode != MHFFN_ROUTE_PARAMS) return MHFFN_ERR_UNSUPPORTED;
  const bool empty = (p.N == 0);
  if (!W_in || !W_gate || !W_up || !W_down || !W_r || !W_out) return MHFFN_ERR_NULL;
  if (!empty && (!X || !Q || !S || !dO)) return MHFFN_ERR_NULL;
  const void* ptrs[] = {X, W_in, W_gate, W_up, W_down, W_r, W_out, Q, S, dO,
                        dX, dW_in, dW_gate, dW_up, dW_down, dW_r, dW_out};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MHFFN_ERR_ALIGN;
  rc = check_fused_shape(desc, p, true);
  if (rc) return rc;
  rc = check_workspace(mhffn::module_workspace_bytes(p, desc->dtype, true), workspace, workspace_bytes);
  if (rc) return rc;
  const int e = mhffn::launch_module_backward(p, desc->dtype, X, W_in, W_gate, W_up, W_down, W_r,
                                              W_out, Q, S, dO, dX, dW_in, dW_gate, dW_up, dW_down,
                                              dW_r, dW_out, workspace, hip_stream);
  if (e == -1) return MHFFN_ERR_UNSUPPORTED;
  return e == 0 ? MHFFN_OK : MHFFN_ERR_LAUNCH;
}

}  // extern "C"
