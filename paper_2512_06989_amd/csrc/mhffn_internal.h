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

// Zero `bytes` (a multiple of 4) of device memory with a fill kernel (safe under graph capture).
int launch_fill_zero(void* p, size_t bytes, void* stream);

// Plain strided product C[m][n] = sum_k A(m,k) B(n,k) on the generic MFMA GEMM of the
// unfused baseline (element strides; n is contiguous in C).  M, N or K of 0 launches nothing
// (K = 0 leaves C untouched: callers zero-fill themselves).
int launch_gemm(int dtype, const void* A, int64_t a_ms, int64_t a_ks, const void* B, int64_t b_ns,
                int64_t b_ks, void* C, int64_t c_ms, int64_t M, int64_t N, int64_t K, void* stream);

// Tuned bf16 product C[m][n] = sum_k A(m,k) B(n,k) (C row-major, ldc).  a_tr / b_tr: the
// operand is stored with its row index contiguous ([K][rows], leading dimension = row
// stride of k) instead of k contiguous ([rows][K]).  Forms: (false,true), (false,false),
// (true,true).  gemm_bf16_supported() says whether sizes and alignment fit the kernel.
bool gemm_bf16_supported(bool a_tr, bool b_tr, const void* A, int64_t lda, const void* B,
                         int64_t ldb, const void* C, int64_t ldc, int64_t M, int64_t N, int64_t K);
// Scratch (fp32 partial outputs, 256-byte aligned) when the contraction is split over
// workgroups because the output tiles alone cannot fill the chip; 0 otherwise.
size_t gemm_bf16_workspace_bytes(int64_t M, int64_t N, int64_t K);
int launch_gemm_bf16(bool a_tr, bool b_tr, const void* A, int64_t lda, const void* B, int64_t ldb,
                     void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, void* ws, void* stream,
                     bool accumulate = false);

// ---- whole module: projections around the fused path -------------------------
// Problem::ldx / ldy are the row strides of the module's input X (dX) and output O (dO);
// Q and S are dense [N][H*d_h].
size_t module_workspace_bytes(const Problem& p, int dtype, bool backward);
int launch_module_forward(const Problem& p, int dtype, const void* X, const void* W_in,
                          const void* Wg, const void* Wu, const void* Wd, const void* Wr,
                          const void* W_out, void* O, void* Q, void* S, void* ws, void* stream);
int launch_module_backward(const Problem& p, int dtype, const void* X, const void* W_in,
                           const void* Wg, const void* Wu, const void* Wd, const void* Wr,
                           const void* W_out, const void* Q, const void* S, const void* dO,
                           void* dX, void* dW_in, void* dWg, void* dWu, void* dWd, void* dWr,
                           void* dW_out, void* ws, void* stream);

}  // namespace mhffn
