/*
 * mhffn_oracle.h -- fp64 CPU oracle for the gated Multi-Head FFN (FlashMHF).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, host-only transcription of
 * the paper's definitions; it exists so that the GPU library can be checked
 * against something that can be verified by eye.  It shares no source, header,
 * table or helper with the GPU library and must never be called from it.
 * Only tests, the smoke check and the bench's cpu_baseline leg use it.
 *
 * What is computed (paper: Preliminary "FFN~ definition", eq:intuitive-ffn;
 * "Headwise Operation Functions"; Methodology "Parallel FFN Sub-Networks":
 * gating logits P^h = Q_h W^h, eq:routing, and the sub-network aggregation
 * equation):
 *
 *   q      = X[l, h*d_h : (h+1)*d_h]                               (split_H)
 *   p[e]   = sum_j q[j] * W_r[h][j][e]                             (logits)
 *   s[e]   = sigmoid(p[e]);  Z = sum_e s[e];  r[e] = s[e]/(Z+eps)  (eq:routing)
 *   g[e,c] = sum_j q[j] * K[h][e][c][j]      (gate pre-activation, "M")
 *   u[e,c] = sum_j q[j] * U[h][e][c][j]      (up projection, "N")
 *   a[e,c] = g*sigmoid(g)*u                  (SiLU(M) .* N)
 *   y_e[j] = sum_c a[e,c] * V[h][e][c][j]    (FFN~ of sub-network e)
 *   Y[l, h*d_h + j] = sum_e r[e] * y_e[j]    (aggregation, concat_H)
 *
 * The backward is the exact derivative of the above (tile formulas in the
 * appendix algorithms "Backward (dQ,dR)" and "Backward (dK,dU,dV)"; the
 * derivative through eq:routing is derived here because the paper leaves it
 * to automatic differentiation).
 *
 * Layouts (all host pointers, all double, all row-major, contiguous unless a
 * leading dimension is given):
 *   X, Y, dX, dY : [n_tokens][ld] with ld >= n_heads*d_head
 *   W_gate (K), W_up (U), W_down (V) : [n_heads][n_sub][d_sub][d_head]
 *   route, route_mode 0 : W_r [n_heads][d_head][n_sub]   (gating parameters)
 *   route, route_mode 1 : R   [n_tokens][n_heads][n_sub] (weights used as given)
 *   d_route has the shape of route for the mode in use (dW_r or dR).
 *
 * Pins (tests/test_oracle_*.py): SwiGLU special case, one-hot weights, token
 * permutation equivariance, brute-force element loops, uniform-gate MH-FFN,
 * identical sub-networks, block-size independence, head independence,
 * linearity, row sums of R, central finite differences, <dy, y_e> identity.
 */
#ifndef MHFFN_ORACLE_H
#define MHFFN_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int64_t n_tokens;   /* N >= 0                                            */
  int32_t n_heads;    /* H                                                 */
  int32_t d_head;     /* d_h                                               */
  int32_t n_sub;      /* E, sub-networks per head                          */
  int32_t d_sub;      /* d_e, width of one sub-network                     */
  int64_t ld_x;       /* row stride of X and dX in elements; 0 => H*d_h    */
  int64_t ld_y;       /* row stride of Y and dY in elements; 0 => H*d_h    */
  int32_t route_mode; /* 0: route = W_r, weights from eq:routing; 1: route = R */
  double  eps;        /* epsilon of eq:routing                             */
} mhffn_oracle_desc;

/* Returns 0 on success, 1 on a null pointer, 2 on a bad shape. */

/* Forward.  R_out (optional, may be NULL) receives the gating weights
 * [n_tokens][n_heads][n_sub] that were used. */
int mhffn_oracle_forward_f64(const mhffn_oracle_desc* d, const double* X,
                             const double* W_gate, const double* W_up,
                             const double* W_down, const double* route,
                             double* Y, double* R_out);

/* Un-weighted sub-network outputs y_e for every token:
 * Ysub [n_tokens][n_heads][n_sub][d_head].  Used by the <dy, y_e> pin. */
int mhffn_oracle_subnet_outputs_f64(const mhffn_oracle_desc* d, const double* X,
                                    const double* W_gate, const double* W_up,
                                    const double* W_down, double* Ysub);

/* Backward.  Any of dX, dW_gate, dW_up, dW_down, d_route may be NULL (skipped).
 * Outputs are overwritten, never accumulated into. */
int mhffn_oracle_backward_f64(const mhffn_oracle_desc* d, const double* X,
                              const double* W_gate, const double* W_up,
                              const double* W_down, const double* route,
                              const double* dY, double* dX, double* dW_gate,
                              double* dW_up, double* dW_down, double* d_route);

/* Number of OpenMP threads the calls above will use. */
int mhffn_oracle_threads(void);

#ifdef __cplusplus
}
#endif
#endif
