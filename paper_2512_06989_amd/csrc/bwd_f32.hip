// Fused, recompute-based backward of the Multi-Head FFN in fp32 (storage and
// arithmetic), gfx950.  Shape-generic companion of the bf16 MFMA kernels: any E,
// any d_e, d_h a multiple of 4 up to 256 (as long as the LDS tiles fit; weight chunks
// of 32 neurons, of 16 where 32 would not fit, i.e. for d_h above 232).  Same two
// sweeps as the bf16 path (appendix algorithms "Backward (dQ,dR)" and "Backward
// (dK,dU,dV)", plus the derivative through eq:routing); nothing of the
// [N][H][d_ff] intermediate is saved or written.  Plain fp32 FMAs on tiles staged
// in LDS: this path exists for parity at fp32 accuracy, not for throughput.
//
//   bwd_f32_tok_kernel   32 tokens x one head: R, dX, dr_e -> dp_e (or dR)
//   bwd_f32_wgt_kernel   32 (16) neurons of one sub-network, all tokens: dK, dU, dV
//   bwd_f32_route_kernel dW_r[h][j][e] = sum_tok q[tok][j] dp[tok][e]
// Every sum runs in a fixed order: results are bit-identical run to run.
#include "mhffn_device.h"
#include "mhffn_internal.h"

namespace mhffn {
namespace {

constexpr int kTM = 32;       // tokens per tile
// neurons per weight chunk: template parameter BC of the kernels, 32 or 16
constexpr int kThreads = 256;

struct BwdF32Args {
  const float* X;
  const float* Wg;
  const float* Wu;
  const float* Wd;
  const void* route;
  const float* dY;
  float* dX;
  float* dWg;
  float* dWu;
  float* dWd;
  float* d_route;
  float* Rws;   // [H][E][N]
  float* DPws;  // [H][E][N]  dp (params mode)
  int64_t N, ldx, ldy, n_tiles, n_items;
  int H, dh, E, de, route_mode, chunks_per_sub;
  float eps;
};

__device__ __forceinline__ float sigmoid_f32(float x) {
  // exact division, branch on sign so exp never overflows
  if (x >= 0.f) return 1.0f / (1.0f + __expf(-x));
  const float t = __expf(x);
  return t / (1.0f + t);
}

// sum over the BC lanes with equal tid / BC, fixed order
template <int BC>
__device__ __forceinline__ float lane_group_sum(float v) {
  if (BC == 32) v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 8);
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 1);
  return v;
}

// ---------------------------------------------------------------------------
// token-major: R (to the workspace), dX, dp or dR
// ---------------------------------------------------------------------------
template <int BC>
__global__ __launch_bounds__(kThreads) void bwd_f32_tok_kernel(BwdF32Args a) {
  constexpr int kBC = BC;
  constexpr int TPT = kTM * BC / kThreads;   // tokens per thread in the products: 4 or 2
  extern __shared__ __attribute__((aligned(16))) float smem_f[];
  const int dh = a.dh, E = a.E, de = a.de;
  const int kst = dh + 1;                  // padded row stride of the weight chunks
  float* Qs = smem_f;                      // [32][dh]
  float* Ys = Qs + kTM * dh;               // [32][dh]   dY
  float* Ks = Ys + kTM * dh;               // [BC][dh+1]
  float* Us = Ks + kBC * kst;              // [BC][dh+1]
  float* Vs = Us + kBC * kst;              // [BC][dh+1]
  float* DMs = Vs + kBC * kst;             // [32 tokens][BC+1]
  float* DNs = DMs + kTM * (kBC + 1);      // [32 tokens][BC+1]
  float* Rs = DNs + kTM * (kBC + 1);       // [32 tokens][E]
  float* DRs = Rs + kTM * E;               // [32 tokens][E]  dr_e, later dp_e
  float* Zinv = DRs + kTM * E;             // [32]  1 / (Z + eps)

  const int tid = threadIdx.x;
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;
  const int h = (int)(item / a.n_tiles);
  const int64_t tok0 = (item % a.n_tiles) * kTM;
  const int64_t N = a.N;

  for (int idx = tid; idx < kTM * dh; idx += kThreads) {
    const int t = idx / dh, j = idx - t * dh;
    const int64_t tok = tok0 + t;
    Qs[idx] = (tok < N) ? a.X[tok * a.ldx + (size_t)h * dh + j] : 0.f;
    Ys[idx] = (tok < N) ? a.dY[tok * a.ldy + (size_t)h * dh + j] : 0.f;
  }
  for (int idx = tid; idx < kTM * E; idx += kThreads) DRs[idx] = 0.f;
  __syncthreads();

  // gating weights: eq:routing
  if (a.route_mode == 0) {
    const float* Wr = reinterpret_cast<const float*>(a.route) + (size_t)h * dh * E;
    for (int idx = tid; idx < kTM * E; idx += kThreads) {
      const int t = idx / E, e = idx - t * E;
      float p = 0.f;
      for (int j = 0; j < dh; ++j) p = fmaf(Qs[t * dh + j], Wr[(size_t)j * E + e], p);
      Rs[idx] = sigmoid_f32(p);
    }
    __syncthreads();
    if (tid < kTM) {
      float z = 0.f;
      for (int e = 0; e < E; ++e) z += Rs[tid * E + e];
      const float zi = 1.0f / (z + a.eps);
      Zinv[tid] = zi;
      for (int e = 0; e < E; ++e) Rs[tid * E + e] *= zi;
    }
  } else {
    const float* R = reinterpret_cast<const float*>(a.route);
    for (int idx = tid; idx < kTM * E; idx += kThreads) {
      const int t = idx / E, e = idx - t * E;
      const int64_t tok = tok0 + t;
      Rs[idx] = (tok < N) ? R[((size_t)tok * a.H + h) * E + e] : 0.f;
    }
  }
  __syncthreads();
  // R for the weight-major kernel
  for (int idx = tid; idx < kTM * E; idx += kThreads) {
    const int e = idx / kTM, t = idx - e * kTM;
    const int64_t tok = tok0 + t;
    if (tok < N) a.Rws[((size_t)h * E + e) * N + tok] = Rs[t * E + e];
  }

  // thread roles
  const int c1 = tid % BC, tg1 = tid / BC;   // products: neuron c1, tokens TPT*tg1 .. +TPT-1
  const int jq = tid & 63, tq = tid >> 6;    // dX: columns jq + 64*i, tokens 8*tq .. +7
  float acc[8][4];
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[t][i] = 0.f;

  const size_t head_off = (size_t)h * E * de * dh;
  for (int e = 0; e < E; ++e) {
    for (int cb = 0; cb < de; cb += kBC) {
      const int rows = min(kBC, de - cb);
      const size_t base = head_off + ((size_t)e * de + cb) * dh;
      for (int idx = tid; idx < kBC * dh; idx += kThreads) {
        const int c = idx / dh, j = idx - c * dh;
        const bool ok = c < rows;
        Ks[c * kst + j] = ok ? a.Wg[base + idx] : 0.f;
        Us[c * kst + j] = ok ? a.Wu[base + idx] : 0.f;
        Vs[c * kst + j] = ok ? a.Wd[base + idx] : 0.f;
      }
      __syncthreads();
      float m[TPT], n[TPT], da[TPT];
#pragma unroll
      for (int t = 0; t < TPT; ++t) { m[t] = 0.f; n[t] = 0.f; da[t] = 0.f; }
      for (int j = 0; j < dh; ++j) {
        const float kv = Ks[c1 * kst + j], uv = Us[c1 * kst + j], vv = Vs[c1 * kst + j];
#pragma unroll
        for (int t = 0; t < TPT; ++t) {
          const float qv = Qs[(TPT * tg1 + t) * dh + j];
          m[t] = fmaf(qv, kv, m[t]);
          n[t] = fmaf(qv, uv, n[t]);
          da[t] = fmaf(Ys[(TPT * tg1 + t) * dh + j], vv, da[t]);
        }
      }
#pragma unroll
      for (int t = 0; t < TPT; ++t) {
        const int tok = TPT * tg1 + t;
        const float sg = sigmoid_f32(m[t]);
        const float silu = m[t] * sg;
        const float rw = Rs[tok * E + e];
        // dr_e += sum_c dA SiLU(M) N : the BC neurons of the chunk sit in adjacent lanes
        const float part = lane_group_sum<BC>(da[t] * silu * n[t]);
        if (c1 == 0) DRs[tok * E + e] += part;
        const float rda = rw * da[t];
        DNs[tok * (kBC + 1) + c1] = rda * silu;
        DMs[tok * (kBC + 1) + c1] = rda * n[t] * fmaf(silu, 1.0f - sg, sg);  // SiLU'(m)
      }
      __syncthreads();
      // dX += dM K + dN U
      for (int c = 0; c < kBC; ++c) {
        float kk[4], uu[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = jq + 64 * i;
          kk[i] = (j < dh) ? Ks[c * kst + j] : 0.f;
          uu[i] = (j < dh) ? Us[c * kst + j] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const float dm = DMs[(8 * tq + t) * (kBC + 1) + c], dn = DNs[(8 * tq + t) * (kBC + 1) + c];
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[t][i] = fmaf(dm, kk[i], fmaf(dn, uu[i], acc[t][i]));
        }
      }
      __syncthreads();
    }
  }

  if (a.route_mode == 0) {
    // through r = s / (Z + eps), s = sigmoid(p):
    //   ds_e = (dr_e - sum_e' dr_e' r_e') / (Z + eps),  dp_e = ds_e s_e (1 - s_e)
    if (tid < kTM) {
      const int64_t tok = tok0 + tid;
      float dot = 0.f;
      for (int e = 0; e < E; ++e) dot = fmaf(DRs[tid * E + e], Rs[tid * E + e], dot);
      const float zi = Zinv[tid], zpe = 1.0f / zi;
      for (int e = 0; e < E; ++e) {
        const float s = Rs[tid * E + e] * zpe;
        const float dp = (DRs[tid * E + e] - dot) * zi * s * (1.0f - s);
        DRs[tid * E + e] = dp;
        if (tok < N) a.DPws[((size_t)h * E + e) * N + tok] = dp;
      }
    }
    __syncthreads();
    // dX += dp W_r^T
    const float* Wr = reinterpret_cast<const float*>(a.route) + (size_t)h * dh * E;
    for (int e = 0; e < E; ++e) {
      float ww[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = jq + 64 * i;
        ww[i] = (j < dh) ? Wr[(size_t)j * E + e] : 0.f;
      }
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float dp = DRs[(8 * tq + t) * E + e];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[t][i] = fmaf(dp, ww[i], acc[t][i]);
      }
    }
  } else if (a.d_route) {
    for (int idx = tid; idx < kTM * E; idx += kThreads) {
      const int t = idx / E, e = idx - t * E;
      const int64_t tok = tok0 + t;
      if (tok < N) a.d_route[((size_t)tok * a.H + h) * E + e] = DRs[idx];
    }
  }

  if (a.dX) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int64_t tok = tok0 + 8 * tq + t;
      if (tok < N) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = jq + 64 * i;
          if (j < dh) a.dX[tok * a.ldx + (size_t)h * dh + j] = acc[t][i];
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// weight-major: dK, dU, dV of one chunk of 32 neurons, summed over all tokens
// ---------------------------------------------------------------------------
template <int BC>
__global__ __launch_bounds__(kThreads) void bwd_f32_wgt_kernel(BwdF32Args a) {
  constexpr int kBC = BC;
  constexpr int TPT = kTM * BC / kThreads;   // tokens per thread in the products
  constexpr int TPN = kThreads / BC;         // threads per neuron in the gradients: 8 or 16
  constexpr int NI = 256 / TPN;              // columns per thread at d_h = 256
  extern __shared__ __attribute__((aligned(16))) float smem_f[];
  const int dh = a.dh, E = a.E, de = a.de;
  const int kst = dh + 1;
  float* Qs = smem_f;                      // [32][dh]
  float* Ys = Qs + kTM * dh;               // [32][dh]
  float* Ks = Ys + kTM * dh;               // [BC][dh+1]
  float* Us = Ks + kBC * kst;
  float* Vs = Us + kBC * kst;
  float* DMs = Vs + kBC * kst;             // [32 tokens][BC+1]
  float* DNs = DMs + kTM * (kBC + 1);
  float* AGs = DNs + kTM * (kBC + 1);      // r SiLU(m) n
  float* Rt = AGs + kTM * (kBC + 1);       // [32] r of this sub-network

  const int tid = threadIdx.x;
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;
  const int per_head = E * a.chunks_per_sub;
  const int h = (int)(item / per_head);
  const int ec = (int)(item % per_head);
  const int e = ec / a.chunks_per_sub, cb = (ec % a.chunks_per_sub) * kBC;
  const int rows = min(kBC, de - cb);
  const int64_t N = a.N;
  const size_t base = (((size_t)h * E + e) * de + cb) * dh;

  for (int idx = tid; idx < kBC * dh; idx += kThreads) {
    const int c = idx / dh, j = idx - c * dh;
    const bool ok = c < rows;
    Ks[c * kst + j] = ok ? a.Wg[base + idx] : 0.f;
    Us[c * kst + j] = ok ? a.Wu[base + idx] : 0.f;
    Vs[c * kst + j] = ok ? a.Wd[base + idx] : 0.f;
  }

  const int c1 = tid % BC, tg1 = tid / BC;   // products: neuron c1, tokens TPT*tg1 .. +TPT-1
  const int c2 = tid / TPN, j0 = tid % TPN;  // gradients: neuron c2, columns j0 + TPN*i
  float gk[NI], gu[NI], gv[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) { gk[i] = 0.f; gu[i] = 0.f; gv[i] = 0.f; }
  const int ni = (dh + TPN - 1) / TPN;
  const float* Rrow = a.Rws + ((size_t)h * E + e) * N;

  for (int64_t tok0 = 0; tok0 < N; tok0 += kTM) {
    __syncthreads();   // previous block consumed (and the weight chunk staged)
    for (int idx = tid; idx < kTM * dh; idx += kThreads) {
      const int t = idx / dh, j = idx - t * dh;
      const int64_t tok = tok0 + t;
      Qs[idx] = (tok < N) ? a.X[tok * a.ldx + (size_t)h * dh + j] : 0.f;
      Ys[idx] = (tok < N) ? a.dY[tok * a.ldy + (size_t)h * dh + j] : 0.f;
    }
    if (tid < kTM) Rt[tid] = (tok0 + tid < N) ? Rrow[tok0 + tid] : 0.f;
    __syncthreads();
    float m[TPT], n[TPT], da[TPT];
#pragma unroll
    for (int t = 0; t < TPT; ++t) { m[t] = 0.f; n[t] = 0.f; da[t] = 0.f; }
    for (int j = 0; j < dh; ++j) {
      const float kv = Ks[c1 * kst + j], uv = Us[c1 * kst + j], vv = Vs[c1 * kst + j];
#pragma unroll
      for (int t = 0; t < TPT; ++t) {
        const float qv = Qs[(TPT * tg1 + t) * dh + j];
        m[t] = fmaf(qv, kv, m[t]);
        n[t] = fmaf(qv, uv, n[t]);
        da[t] = fmaf(Ys[(TPT * tg1 + t) * dh + j], vv, da[t]);
      }
    }
#pragma unroll
    for (int t = 0; t < TPT; ++t) {
      const int tok = TPT * tg1 + t;
      const float sg = sigmoid_f32(m[t]);
      const float silu = m[t] * sg;
      const float rw = Rt[tok];
      const float rda = rw * da[t];
      AGs[tok * (kBC + 1) + c1] = rw * silu * n[t];
      DNs[tok * (kBC + 1) + c1] = rda * silu;
      DMs[tok * (kBC + 1) + c1] = rda * n[t] * fmaf(silu, 1.0f - sg, sg);
    }
    __syncthreads();
    // dV[c][j] += A_gated[tok][c] dY[tok][j]; dK[c][j] += dM[tok][c] q[tok][j]; dU likewise
    for (int t = 0; t < kTM; ++t) {
      const float dm = DMs[t * (kBC + 1) + c2], dn = DNs[t * (kBC + 1) + c2], ag = AGs[t * (kBC + 1) + c2];
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        if (i < ni) {
          const int j = j0 + TPN * i;
          const float qv = (j < dh) ? Qs[t * dh + j] : 0.f;
          const float yv = (j < dh) ? Ys[t * dh + j] : 0.f;
          gk[i] = fmaf(dm, qv, gk[i]);
          gu[i] = fmaf(dn, qv, gu[i]);
          gv[i] = fmaf(ag, yv, gv[i]);
        }
      }
    }
  }
  if (c2 < rows) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int j = j0 + TPN * i;
      if (i < ni && j < dh) {
        const size_t o = base + (size_t)c2 * dh + j;
        if (a.dWg) a.dWg[o] = gk[i];
        if (a.dWu) a.dWu[o] = gu[i];
        if (a.dWd) a.dWd[o] = gv[i];
      }
    }
  }
}

// dW_r[h][j][e] = sum_tok q[tok][j] dp[tok][e], tokens in order
__global__ void bwd_f32_route_kernel(BwdF32Args a) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)a.H * a.dh * a.E;
  if (idx >= total) return;
  const int e = (int)(idx % a.E);
  const int j = (int)((idx / a.E) % a.dh);
  const int h = (int)(idx / ((int64_t)a.E * a.dh));
  const float* dp = a.DPws + ((size_t)h * a.E + e) * a.N;
  const float* x = a.X + (size_t)h * a.dh + j;
  float s = 0.f;
  for (int64_t t = 0; t < a.N; ++t) s = fmaf(x[t * a.ldx], dp[t], s);
  a.d_route[idx] = s;
}

__global__ void fill_zero_f32_kernel(float* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t tok_lds_bytes(const Problem& p, int bc) {
  const size_t dh = p.dh;
  return sizeof(float) * (2 * kTM * dh + 3 * bc * (dh + 1) + 2 * kTM * (bc + 1) +
                          2 * (size_t)kTM * p.E + kTM);
}
size_t wgt_lds_bytes(const Problem& p, int bc) {
  const size_t dh = p.dh;
  return sizeof(float) * (2 * kTM * dh + 3 * bc * (dh + 1) + 3 * kTM * (bc + 1) + kTM);
}
size_t lds_bytes_for(const Problem& p, int bc) {
  const size_t t = tok_lds_bytes(p, bc), w = wgt_lds_bytes(p, bc);
  return t > w ? t : w;
}
// neurons per weight chunk: 32 where the tiles fit in LDS, else 16
int chunk_neurons(const Problem& p) { return lds_bytes_for(p, 32) <= kLdsBytesPerWorkgroup ? 32 : 16; }

template <int BC>
int launch_kernels(const Problem& p, BwdF32Args a, bool weights, hipStream_t stream) {
  if (hipError_t e0 = LdsLimit<&bwd_f32_tok_kernel<BC>, (int)kLdsBytesPerWorkgroup>::ensure(); e0 != hipSuccess)
    return (int)e0;
  if (hipError_t e0 = LdsLimit<&bwd_f32_wgt_kernel<BC>, (int)kLdsBytesPerWorkgroup>::ensure(); e0 != hipSuccess)
    return (int)e0;
  a.chunks_per_sub = (p.de + BC - 1) / BC;
  // token-major kernel (always: it also produces R for the weight-major kernel)
  a.n_tiles = (p.N + kTM - 1) / kTM;
  a.n_items = a.n_tiles * p.H;
  hipLaunchKernelGGL(bwd_f32_tok_kernel<BC>, dim3((unsigned)xcd_grid_size(a.n_items)), dim3(kThreads),
                     tok_lds_bytes(p, BC), stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !weights) return (int)e;
  a.n_items = (int64_t)p.H * p.E * a.chunks_per_sub;
  hipLaunchKernelGGL(bwd_f32_wgt_kernel<BC>, dim3((unsigned)xcd_grid_size(a.n_items)), dim3(kThreads),
                     wgt_lds_bytes(p, BC), stream, a);
  return (int)hipGetLastError();
}

}  // namespace

size_t bwd_f32_lds_bytes(const Problem& p) { return lds_bytes_for(p, chunk_neurons(p)); }

size_t bwd_f32_workspace_bytes(const Problem& p) {
  if (p.N == 0) return 0;
  return 2 * align256((size_t)p.N * p.H * p.E * sizeof(float));
}

int launch_bwd_f32(const Problem& p, const void* X, const void* Wg, const void* Wu,
                   const void* Wd, const void* route, const void* dY, void* dX, void* dWg,
                   void* dWu, void* dWd, void* d_route, void* ws, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const size_t wcount = (size_t)p.H * p.E * p.de * p.dh;
  if (p.N == 0) {   // no tokens: the weight gradients are zero, there is nothing else
    float* outs[4] = {static_cast<float*>(dWg), static_cast<float*>(dWu), static_cast<float*>(dWd),
                      p.route_mode == 0 ? static_cast<float*>(d_route) : nullptr};
    const size_t counts[4] = {wcount, wcount, wcount, (size_t)p.H * p.dh * p.E};
    for (int i = 0; i < 4; ++i) {
      if (!outs[i] || !counts[i]) continue;
      hipLaunchKernelGGL(fill_zero_f32_kernel, dim3((unsigned)((counts[i] + 255) / 256)), dim3(256),
                         0, stream, outs[i], counts[i]);
    }
    return (int)hipGetLastError();
  }
  BwdF32Args a;
  a.X = static_cast<const float*>(X);
  a.Wg = static_cast<const float*>(Wg);
  a.Wu = static_cast<const float*>(Wu);
  a.Wd = static_cast<const float*>(Wd);
  a.route = route;
  a.dY = static_cast<const float*>(dY);
  a.dX = static_cast<float*>(dX);
  a.dWg = static_cast<float*>(dWg);
  a.dWu = static_cast<float*>(dWu);
  a.dWd = static_cast<float*>(dWd);
  a.d_route = static_cast<float*>(d_route);
  const size_t nhe = align256((size_t)p.N * p.H * p.E * sizeof(float));
  a.Rws = reinterpret_cast<float*>(static_cast<unsigned char*>(ws));
  a.DPws = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + nhe);
  a.N = p.N; a.ldx = p.ldx; a.ldy = p.ldy;
  a.H = p.H; a.dh = p.dh; a.E = p.E; a.de = p.de; a.route_mode = p.route_mode; a.eps = p.eps;
  a.chunks_per_sub = 0; a.n_tiles = 0; a.n_items = 0;

  const bool weights = dWg || dWu || dWd;
  const int rc = chunk_neurons(p) == 32 ? launch_kernels<32>(p, a, weights, stream)
                                        : launch_kernels<16>(p, a, weights, stream);
  if (rc != 0) return rc;
  hipError_t e = hipSuccess;
  if (d_route && p.route_mode == 0) {
    const int64_t total = (int64_t)p.H * p.dh * p.E;
    hipLaunchKernelGGL(bwd_f32_route_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       stream, a);
    e = hipGetLastError();
  }
  return (int)e;
}

}  // namespace mhffn
