// The whole FlashMHF module around the fused path (Methodology: Q = split_H(X W_in),
// O = concat_H(S) W_out): two d_model x d_model projections forward, four products
// backward, composed on the host from the library's own kernels.  Nothing is allocated:
// Q and S (the activations a training step keeps, [N][d_model] each) belong to the caller,
// dS and dQ live in the workspace next to the fused backward's scratch.
#include "mhffn_internal.h"

namespace mhffn {
namespace {

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
size_t elt(int dtype) { return dtype == 1 ? 2 : 4; }

// the fused path on the dense [N][d_model] buffers between the projections
Problem inner(const Problem& p) {
  Problem q = p;
  q.ldx = q.ldy = (int64_t)p.H * p.dh;
  q.route_mode = 0;
  return q;
}

size_t fused_fwd_ws(const Problem& p, int dtype) { return dtype == 1 ? fwd_bf16_workspace_bytes(inner(p)) : 0; }

// scratch of the projection products of one pass (they run one after the other and share it)
size_t gemm_ws(const Problem& p, int dtype, bool backward) {
  if (dtype != 1) return 0;
  const int64_t dm = (int64_t)p.H * p.dh;
  size_t need = gemm_bf16_workspace_bytes(p.N, dm, dm);                  // activations x weights
  if (backward) {
    const size_t w = gemm_bf16_workspace_bytes(dm, dm, p.N);             // weight gradients
    need = need > w ? need : w;
  }
  return align256(need);
}

// The three products of a linear layer.  bf16 goes to the tuned kernel whenever sizes and
// alignment fit it, everything else to the generic strided GEMM.
// C[M][N] = A[M][K] B[K][N]
int product_nn(int dtype, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
               int64_t ldc, int64_t M, int64_t N, int64_t K, void* gws, void* stream) {
  if (dtype == 1 && gemm_bf16_supported(false, true, A, lda, B, ldb, C, ldc, M, N, K))
    return launch_gemm_bf16(false, true, A, lda, B, ldb, C, ldc, M, N, K, gws, stream);
  return launch_gemm(dtype, A, lda, 1, B, 1, ldb, C, ldc, M, N, K, stream);
}
// C[M][N] = A[M][K] B[N][K]^T
int product_nt(int dtype, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
               int64_t ldc, int64_t M, int64_t N, int64_t K, void* gws, void* stream) {
  if (dtype == 1 && gemm_bf16_supported(false, false, A, lda, B, ldb, C, ldc, M, N, K))
    return launch_gemm_bf16(false, false, A, lda, B, ldb, C, ldc, M, N, K, gws, stream);
  return launch_gemm(dtype, A, lda, 1, B, ldb, 1, C, ldc, M, N, K, stream);
}
// C[M][N] = A[K][M]^T B[K][N]
int product_tn(int dtype, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
               int64_t ldc, int64_t M, int64_t N, int64_t K, void* gws, void* stream) {
  if (dtype == 1 && gemm_bf16_supported(true, true, A, lda, B, ldb, C, ldc, M, N, K))
    return launch_gemm_bf16(true, true, A, lda, B, ldb, C, ldc, M, N, K, gws, stream);
  return launch_gemm(dtype, A, 1, lda, B, 1, ldb, C, ldc, M, N, K, stream);
}

}  // namespace

size_t module_workspace_bytes(const Problem& p, int dtype, bool backward) {
  if (p.N == 0) return 0;
  if (!backward) return align256(fused_fwd_ws(p, dtype)) + gemm_ws(p, dtype, false);
  const size_t act = align256((size_t)p.N * p.H * p.dh * elt(dtype));
  return 2 * act + align256(bwd_workspace_bytes(inner(p), dtype)) + gemm_ws(p, dtype, true);
}

int launch_module_forward(const Problem& p, int dtype, const void* X, const void* W_in,
                          const void* Wg, const void* Wu, const void* Wd, const void* Wr,
                          const void* W_out, void* O, void* Q, void* S, void* ws, void* stream) {
  if (p.N == 0) return 0;
  const int64_t dm = (int64_t)p.H * p.dh;
  const Problem q = inner(p);
  void* gws = static_cast<unsigned char*>(ws) + align256(fused_fwd_ws(p, dtype));
  // Q[l][j] = sum_i X[l][i] W_in[i][j]
  int e = product_nn(dtype, X, p.ldx, W_in, dm, Q, dm, p.N, dm, dm, gws, stream);
  if (e) return e;
  e = dtype == 1 ? launch_fwd_bf16(q, Q, Wg, Wu, Wd, Wr, S, ws, stream)
                 : launch_fwd_f32(q, Q, Wg, Wu, Wd, Wr, S, stream);
  if (e) return e;
  // O[l][j] = sum_i S[l][i] W_out[i][j]
  return product_nn(dtype, S, dm, W_out, dm, O, p.ldy, p.N, dm, dm, gws, stream);
}

int launch_module_backward(const Problem& p, int dtype, const void* X, const void* W_in,
                           const void* Wg, const void* Wu, const void* Wd, const void* Wr,
                           const void* W_out, const void* Q, const void* S, const void* dO,
                           void* dX, void* dW_in, void* dWg, void* dWu, void* dWd, void* dWr,
                           void* dW_out, void* ws, void* stream) {
  const int64_t dm = (int64_t)p.H * p.dh;
  const Problem q = inner(p);
  if (p.N == 0) {
    // no tokens: every parameter gradient is zero (the fused backward zero-fills its own)
    const size_t bytes = (size_t)dm * dm * elt(dtype);
    int e = launch_fill_zero(dW_in, bytes, stream);
    if (!e) e = launch_fill_zero(dW_out, bytes, stream);
    if (e) return e;
    return launch_bwd(q, dtype, Q, Wg, Wu, Wd, Wr, nullptr, nullptr, dWg, dWu, dWd, dWr, ws, stream);
  }
  const size_t act = align256((size_t)p.N * dm * elt(dtype));
  unsigned char* w = static_cast<unsigned char*>(ws);
  void* dS = w;
  void* dQ = w + act;
  void* fused_ws = w + 2 * act;
  void* gws = w + 2 * act + align256(bwd_workspace_bytes(q, dtype));
  // dS[l][i] = sum_j dO[l][j] W_out[i][j]
  int e = product_nt(dtype, dO, p.ldy, W_out, dm, dS, dm, p.N, dm, dm, gws, stream);
  if (e) return e;
  // dW_out[i][j] = sum_l S[l][i] dO[l][j]
  if (dW_out) {
    e = product_tn(dtype, S, dm, dO, p.ldy, dW_out, dm, dm, dm, p.N, gws, stream);
    if (e) return e;
  }
  const bool need_dq = dX || dW_in;
  e = launch_bwd(q, dtype, Q, Wg, Wu, Wd, Wr, dS, need_dq ? dQ : nullptr, dWg, dWu, dWd, dWr,
                 fused_ws, stream);
  if (e) return e;
  // dW_in[i][j] = sum_l X[l][i] dQ[l][j]
  if (dW_in) {
    e = product_tn(dtype, X, p.ldx, dQ, dm, dW_in, dm, dm, dm, p.N, gws, stream);
    if (e) return e;
  }
  // dX[l][i] = sum_j dQ[l][j] W_in[i][j]
  if (dX) e = product_nt(dtype, dQ, dm, W_in, dm, dX, p.ldx, p.N, dm, dm, gws, stream);
  return e;
}

}  // namespace mhffn
