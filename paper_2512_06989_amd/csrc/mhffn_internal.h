// Host-side declarations shared by the C-ABI layer (api.cpp) and the kernel
// translation units.  Every launcher enqueues on `stream`, never synchronises,
// and returns the hipError_t of the launch as an int (0 = success).
#pragma once

#include <stddef.h>
#include <stdint.h>

namespace mhffn {

// Problem description after validation; strides are always filled in.
struct Problem {
  int64_t N;        // tokens
  int H, dh, E, de; // heads, head width, sub-networks per head, sub-network width
  int64_t ldx, ldy; // row strides (elements) of X/dX and Y/dY
  int route_mode;   // 0: route = W_r (gating parameters), 1: route = R (weights)
  float eps;
};

// ---- fused forward ---------------------------------------------------------
// bf16, d_h in {64, 128, 256}, d_e % 32 == 0, E <= kFwdBf16MaxSub, LDS within the limit.
constexpr int kFwdBf16MaxSub = 96;
size_t fwd_bf16_lds_bytes(const Problem& p);
// Scratch of the bf16 forward: 0 unless the token tiles cannot fill the chip and the
// intermediate dimension is split over workgroups (fp32 partial outputs).
size_t fwd_bf16_workspace_bytes(const Problem& p);
int launch_fwd_bf16(const Problem& p, const void* X, const void* Wg, const void* Wu,
                    const void* Wd, const void* route, void* Y, void* ws, void* stream);
// fp32, d_h % 4 == 0, d_h <= 256.
int launch_fwd_f32(const Problem& p, const void* X, const void* Wg, const void* Wu,
                   const void* Wd, const void* route, void* Y, void* stream);
size_t fwd_f32_lds_bytes(const Problem& p);
constexpr size_t kLdsBytesPerWorkgroup = 160 * 1024;

// ---- fused backward --------------------------------------------------------
// bf16 limits of the backward kernels for a shape (d_h in {64, 128, 256})
int bwd_bf16_max_sub(const Problem& p);
size_t bwd_bf16_lds_bytes(const Problem& p);
size_t bwd_workspace_bytes(const Problem& p, int dtype);
int launch_bwd(const Problem& p, int dtype, const void* X, const void* Wg, const void* Wu,
               const void* Wd, const void* route, const void* dY, void* dX, void* dWg,
               void* dWu, void* dWd, void* d_route, void* ws, void* stream,
               void* const* phase_events = nullptr, int n_phase_events = 0);
// Phases of the fused backward, in launch order (see mhffn_backward_phases).
constexpr int kBwdPhases = 3;
// fp32 companion (d_h % 4 == 0, d_h <= 256, tiles must fit in LDS)
size_t bwd_f32_lds_bytes(const Problem& p);
size_t bwd_f32_workspace_bytes(const Problem& p);
int launch_bwd_f32(const Problem& p, const void* X, const void* Wg, const void* Wu,
                   const void* Wd, const void* route, const void* dY, void* dX, void* dWg,
                   void* dWu, void* dWd, void* d_route, void* ws, void* stream);

// ---- unfused baseline ------------------------------------------------------
size_t unfused_workspace_bytes(const Problem& p, int dtype, bool backward);
int launch_unfused(const Problem& p, int dtype, const void* X, const void* Wg,
                   const void* Wu, const void* Wd, const void* route, void* Y,
                   const void* dY, void* dX, void* dWg, void* dWu, void* dWd,
                   void* d_route, void* ws, void* stream);

}  // namespace mhffn
