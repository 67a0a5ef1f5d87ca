/*
 * mhffn_oracle.c -- fp64 CPU oracle for the gated Multi-Head FFN (FlashMHF).
 *
 * TEST INFRASTRUCTURE ONLY (see mhffn_oracle.h).  Plain loops in the order of
 * the paper's definitions; the only concession to speed is OpenMP over
 * independent tokens (forward, input gradient) or independent (head,
 * sub-network) pairs (weight gradients), and `omp simd` on the innermost
 * contiguous loops, which changes nothing but the rounding order of a sum.
 *
 * Readings of the paper taken here:
 *  - epsilon of eq:routing is an argument (the paper gives no value);
 *  - the normaliser is sigmoid / sum of sigmoids over all E sub-networks,
 *    dense, no top-k;
 *  - the gate and the sub-networks read the same per-head slice q;
 *  - in the appendix algorithm "Backward (dQ,dR)" the row accumulator for dR
 *    is per sub-network (dr[e] = <dy, y_e>), i.e. it restarts for every e;
 *  - the gating weights are differentiated through (no stop-gradient).
 */
#include "mhffn_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* sigmoid evaluated without overflow for either sign of x */
static double sigmoid_f64(double x) {
  if (x >= 0.0) {
    return 1.0 / (1.0 + exp(-x));
  } else {
    double t = exp(x);
    return t / (1.0 + t);
  }
}

/* sum_j a[j]*b[j] over a contiguous run */
static double dot_f64(const double* a, const double* b, int n) {
  double acc = 0.0;
#pragma omp simd reduction(+ : acc)
  for (int j = 0; j < n; ++j) acc += a[j] * b[j];
  return acc;
}

static int check_desc(const mhffn_oracle_desc* d) {
  if (!d) return 1;
  if (d->n_tokens < 0 || d->n_heads < 1 || d->d_head < 1 || d->n_sub < 1 ||
      d->d_sub < 1)
    return 2;
  int64_t dm = (int64_t)d->n_heads * d->d_head;
  if (d->ld_x != 0 && d->ld_x < dm) return 2;
  if (d->ld_y != 0 && d->ld_y < dm) return 2;
  if (d->route_mode != 0 && d->route_mode != 1) return 2;
  return 0;
}

int mhffn_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Gating weights of one (token, head): eq:routing.  q [d_h]; Wr_h = W_r[h],
 * laid out [d_h][E].  Writes p, s, r (each [E]) and returns Z. */
static double gating_f64(const double* q, const double* Wr_h, int d_h, int E,
                         double eps, double* p, double* s, double* r) {
  for (int e = 0; e < E; ++e) p[e] = 0.0;
  for (int j = 0; j < d_h; ++j) {
    const double qj = q[j];
    const double* w = Wr_h + (size_t)j * E;
    for (int e = 0; e < E; ++e) p[e] += qj * w[e];
  }
  double Z = 0.0;
  for (int e = 0; e < E; ++e) {
    s[e] = sigmoid_f64(p[e]);
    Z += s[e];
  }
  for (int e = 0; e < E; ++e) r[e] = s[e] / (Z + eps);
  return Z;
}

int mhffn_oracle_forward_f64(const mhffn_oracle_desc* d, const double* X,
                             const double* W_gate, const double* W_up,
                             const double* W_down, const double* route,
                             double* Y, double* R_out) {
  int rc = check_desc(d);
  if (rc) return rc;
  if (!X || !W_gate || !W_up || !W_down || !route || !Y) return 1;
  const int64_t N = d->n_tokens;
  const int H = d->n_heads, dh = d->d_head, E = d->n_sub, de = d->d_sub;
  const int64_t ldx = d->ld_x ? d->ld_x : (int64_t)H * dh;
  const int64_t ldy = d->ld_y ? d->ld_y : (int64_t)H * dh;
  const size_t wsub = (size_t)de * dh; /* one sub-network's matrix */

#pragma omp parallel
  {
    double* p = (double*)malloc(sizeof(double) * E);
    double* s = (double*)malloc(sizeof(double) * E);
    double* r = (double*)malloc(sizeof(double) * E);
    double* ye = (double*)malloc(sizeof(double) * dh);
    double* y = (double*)malloc(sizeof(double) * dh);
#pragma omp for collapse(2) schedule(static)
    for (int64_t l = 0; l < N; ++l) {
      for (int h = 0; h < H; ++h) {
        const double* q = X + l * ldx + (size_t)h * dh; /* split_H */
        if (d->route_mode == 0) {
          gating_f64(q, route + (size_t)h * dh * E, dh, E, d->eps, p, s, r);
        } else {
          for (int e = 0; e < E; ++e) r[e] = route[((size_t)l * H + h) * E + e];
        }
        if (R_out)
          for (int e = 0; e < E; ++e) R_out[((size_t)l * H + h) * E + e] = r[e];
        for (int j = 0; j < dh; ++j) y[j] = 0.0;
        for (int e = 0; e < E; ++e) {
          const double* K = W_gate + ((size_t)h * E + e) * wsub;
          const double* U = W_up + ((size_t)h * E + e) * wsub;
          const double* V = W_down + ((size_t)h * E + e) * wsub;
          /* y_e = (SiLU(q K^T) .* (q U^T)) V : eq:intuitive-ffn */
          for (int j = 0; j < dh; ++j) ye[j] = 0.0;
          for (int c = 0; c < de; ++c) {
            const double g = dot_f64(q, K + (size_t)c * dh, dh);
            const double u = dot_f64(q, U + (size_t)c * dh, dh);
            const double a = g * sigmoid_f64(g) * u;
            const double* v = V + (size_t)c * dh;
#pragma omp simd
            for (int j = 0; j < dh; ++j) ye[j] += a * v[j];
          }
          /* aggregation: S = sum_e R_e * FFN~_e */
          for (int j = 0; j < dh; ++j) y[j] += r[e] * ye[j];
        }
        double* out = Y + l * ldy + (size_t)h * dh; /* concat_H */
        for (int j = 0; j < dh; ++j) out[j] = y[j];
      }
    }
    free(p); free(s); free(r); free(ye); free(y);
  }
  return 0;
}

int mhffn_oracle_subnet_outputs_f64(const mhffn_oracle_desc* d, const double* X,
                                    const double* W_gate, const double* W_up,
                                    const double* W_down, double* Ysub) {
  int rc = check_desc(d);
  if (rc) return rc;
  if (!X || !W_gate || !W_up || !W_down || !Ysub) return 1;
  const int64_t N = d->n_tokens;
  const int H = d->n_heads, dh = d->d_head, E = d->n_sub, de = d->d_sub;
  const int64_t ldx = d->ld_x ? d->ld_x : (int64_t)H * dh;
  const size_t wsub = (size_t)de * dh;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t l = 0; l < N; ++l) {
    for (int h = 0; h < H; ++h) {
      const double* q = X + l * ldx + (size_t)h * dh;
      for (int e = 0; e < E; ++e) {
        const double* K = W_gate + ((size_t)h * E + e) * wsub;
        const double* U = W_up + ((size_t)h * E + e) * wsub;
        const double* V = W_down + ((size_t)h * E + e) * wsub;
        double* ye = Ysub + (((size_t)l * H + h) * E + e) * dh;
        for (int j = 0; j < dh; ++j) ye[j] = 0.0;
        for (int c = 0; c < de; ++c) {
          const double g = dot_f64(q, K + (size_t)c * dh, dh);
          const double u = dot_f64(q, U + (size_t)c * dh, dh);
          const double a = g * sigmoid_f64(g) * u;
          for (int j = 0; j < dh; ++j) ye[j] += a * V[(size_t)c * dh + j];
        }
      }
    }
  }
  return 0;
}

int mhffn_oracle_backward_f64(const mhffn_oracle_desc* d, const double* X,
                              const double* W_gate, const double* W_up,
                              const double* W_down, const double* route,
                              const double* dY, double* dX, double* dW_gate,
                              double* dW_up, double* dW_down, double* d_route) {
  int rc = check_desc(d);
  if (rc) return rc;
  if (!X || !W_gate || !W_up || !W_down || !route || !dY) return 1;
  const int64_t N = d->n_tokens;
  const int H = d->n_heads, dh = d->d_head, E = d->n_sub, de = d->d_sub;
  const int64_t ldx = d->ld_x ? d->ld_x : (int64_t)H * dh;
  const int64_t ldy = d->ld_y ? d->ld_y : (int64_t)H * dh;
  const size_t wsub = (size_t)de * dh;
  const int params_mode = (d->route_mode == 0);
  const size_t nhe = (size_t)N * H * E;

  /* r and dp per (token, head, sub-network), handed from the token-major
   * pass to the weight-major pass (small: E values, not d_ff values). */
  double* Rbuf = (double*)malloc(sizeof(double) * (nhe ? nhe : 1));
  double* DPbuf = (double*)malloc(sizeof(double) * (nhe ? nhe : 1));
  if (!Rbuf || !DPbuf) { free(Rbuf); free(DPbuf); return 2; }

  /* ---- pass 1, per (token, head): r, dr, dp, dX ------------------------ */
#pragma omp parallel
  {
    double* p = (double*)malloc(sizeof(double) * E);
    double* s = (double*)malloc(sizeof(double) * E);
    double* r = (double*)malloc(sizeof(double) * E);
    double* dr = (double*)malloc(sizeof(double) * E);
    double* dp = (double*)malloc(sizeof(double) * E);
    double* dq = (double*)malloc(sizeof(double) * dh);
#pragma omp for collapse(2) schedule(static)
    for (int64_t l = 0; l < N; ++l) {
      for (int h = 0; h < H; ++h) {
        const double* q = X + l * ldx + (size_t)h * dh;
        const double* dy = dY + l * ldy + (size_t)h * dh;
        const double* Wr_h = route + (size_t)h * dh * E;
        double Z = 0.0;
        if (params_mode) {
          Z = gating_f64(q, Wr_h, dh, E, d->eps, p, s, r);
        } else {
          for (int e = 0; e < E; ++e) r[e] = route[((size_t)l * H + h) * E + e];
        }
        for (int j = 0; j < dh; ++j) dq[j] = 0.0;
        for (int e = 0; e < E; ++e) {
          const double* K = W_gate + ((size_t)h * E + e) * wsub;
          const double* U = W_up + ((size_t)h * E + e) * wsub;
          const double* V = W_down + ((size_t)h * E + e) * wsub;
          double dre = 0.0;
          for (int c = 0; c < de; ++c) {
            const double* k = K + (size_t)c * dh;
            const double* u_ = U + (size_t)c * dh;
            const double g = dot_f64(q, k, dh);             /* M */
            const double u = dot_f64(q, u_, dh);            /* N */
            const double sg = sigmoid_f64(g);
            const double silu = g * sg;
            const double a = silu * u;                      /* SiLU(M).*N */
            const double da = dot_f64(dy, V + (size_t)c * dh, dh); /* dS V^T */
            dre += da * a;                                  /* dR row sum */
            const double dn = r[e] * da * silu;
            const double dm = r[e] * da * u * (sg + g * sg * (1.0 - sg));
#pragma omp simd
            for (int j = 0; j < dh; ++j) dq[j] += dm * k[j] + dn * u_[j];
          }
          dr[e] = dre;
        }
        if (params_mode) {
          /* derivative through r[e] = s[e]/(Z+eps), s = sigmoid(p), p = q W_r */
          double dot_dr_r = 0.0;
          for (int e = 0; e < E; ++e) dot_dr_r += dr[e] * r[e];
          for (int e = 0; e < E; ++e) {
            const double ds = (dr[e] - dot_dr_r) / (Z + d->eps);
            dp[e] = ds * s[e] * (1.0 - s[e]);
          }
          for (int j = 0; j < dh; ++j) {
            double acc = 0.0;
            for (int e = 0; e < E; ++e) acc += dp[e] * Wr_h[(size_t)j * E + e];
            dq[j] += acc;
          }
        }
        for (int e = 0; e < E; ++e) {
          const size_t idx = ((size_t)l * H + h) * E + e;
          Rbuf[idx] = r[e];
          DPbuf[idx] = params_mode ? dp[e] : dr[e];
        }
        if (dX) {
          double* out = dX + l * ldx + (size_t)h * dh;
          for (int j = 0; j < dh; ++j) out[j] = dq[j];
        }
      }
    }
    free(p); free(s); free(r); free(dr); free(dp); free(dq);
  }

  if (d_route && !params_mode) memcpy(d_route, DPbuf, sizeof(double) * nhe);

  /* ---- pass 2, per (head, sub-network): sums over all tokens ----------- */
  const int want_w = (dW_gate || dW_up || dW_down);
  const int want_wr = (d_route && params_mode);
  if (want_w || want_wr) {
#pragma omp parallel
    {
      double* dK = (double*)malloc(sizeof(double) * wsub);
      double* dU = (double*)malloc(sizeof(double) * wsub);
      double* dV = (double*)malloc(sizeof(double) * wsub);
      double* dwr = (double*)malloc(sizeof(double) * dh);
#pragma omp for collapse(2) schedule(dynamic, 1)
      for (int h = 0; h < H; ++h) {
        for (int e = 0; e < E; ++e) {
          const double* K = W_gate + ((size_t)h * E + e) * wsub;
          const double* U = W_up + ((size_t)h * E + e) * wsub;
          const double* V = W_down + ((size_t)h * E + e) * wsub;
          memset(dK, 0, sizeof(double) * wsub);
          memset(dU, 0, sizeof(double) * wsub);
          memset(dV, 0, sizeof(double) * wsub);
          memset(dwr, 0, sizeof(double) * dh);
          for (int64_t l = 0; l < N; ++l) {
            const double* q = X + l * ldx + (size_t)h * dh;
            const double* dy = dY + l * ldy + (size_t)h * dh;
            const double re = Rbuf[((size_t)l * H + h) * E + e];
            if (want_w) {
              for (int c = 0; c < de; ++c) {
                const double g = dot_f64(q, K + (size_t)c * dh, dh);
                const double u = dot_f64(q, U + (size_t)c * dh, dh);
                const double sg = sigmoid_f64(g);
                const double silu = g * sg;
                const double a = silu * u;
                const double da = dot_f64(dy, V + (size_t)c * dh, dh);
                const double dn = re * da * silu;
                const double dm = re * da * u * (sg + g * sg * (1.0 - sg));
                const double ra = re * a; /* gated activation */
                double* dk = dK + (size_t)c * dh;
                double* du = dU + (size_t)c * dh;
                double* dv = dV + (size_t)c * dh;
#pragma omp simd
                for (int j = 0; j < dh; ++j) {
                  dv[j] += ra * dy[j];  /* dV += A_gated^T dS */
                  dk[j] += dm * q[j];   /* dK += dM^T Q       */
                  du[j] += dn * q[j];   /* dU += dN^T Q       */
                }
              }
            }
            if (want_wr) {
              const double dpe = DPbuf[((size_t)l * H + h) * E + e];
              for (int j = 0; j < dh; ++j) dwr[j] += q[j] * dpe;
            }
          }
          const size_t off = ((size_t)h * E + e) * wsub;
          if (dW_gate) memcpy(dW_gate + off, dK, sizeof(double) * wsub);
          if (dW_up) memcpy(dW_up + off, dU, sizeof(double) * wsub);
          if (dW_down) memcpy(dW_down + off, dV, sizeof(double) * wsub);
          if (want_wr)
            for (int j = 0; j < dh; ++j)
              d_route[((size_t)h * dh + j) * E + e] = dwr[j];
        }
      }
      free(dK); free(dU); free(dV); free(dwr);
    }
  }
  free(Rbuf);
  free(DPbuf);
  return 0;
}
