// Fused Multi-Head FFN forward in fp32 (storage and arithmetic), gfx950.
//
// Shape-generic companion of the bf16 MFMA kernel: any E, any d_e, d_h a
// multiple of 4 up to 256.  Same structure as eq:flash-ffn-loop / appendix
// algorithm "SRAMFFN-Forward": a workgroup owns 32 tokens of one head, keeps
// q and the gating weights R in LDS, and walks the intermediate dimension in
// chunks of 32 neurons whose K, U, V rows are staged in LDS; M, N, A and the
// output accumulator never leave the chip.  Plain fp32 FMAs: this path exists
// for the 1e-5 parity configuration, not for throughput.
#include "mhffn_device.h"
#include "mhffn_internal.h"

namespace mhffn {
namespace {

constexpr int kTM = 32;       // tokens per workgroup
constexpr int kBC = 32;       // neurons per chunk
constexpr int kThreads = 256;
constexpr int kMaxDh = 256;

struct F32Args {
  const float* X;
  const float* Wg;
  const float* Wu;
  const float* Wd;
  const void* route;
  float* Y;
  int64_t N, ldx, ldy, n_tiles, n_items;
  int H, dh, E, de, route_mode;
  float eps;
};

__device__ __forceinline__ float sigmoid_f32(float x) {
  // exact division, branch on sign so exp never overflows
  if (x >= 0.f) return 1.0f / (1.0f + __expf(-x));
  const float t = __expf(x);
  return t / (1.0f + t);
}

__global__ __launch_bounds__(kThreads) void fwd_f32_kernel(F32Args a) {
  extern __shared__ __attribute__((aligned(16))) float smem_f[];
  const int dh = a.dh, E = a.E, de = a.de;
  const int kst = dh + 1;                 // padded row stride of K/U chunks
  float* Qs = smem_f;                     // [32][dh]
  float* Ks = Qs + kTM * dh;              // [32][dh+1]
  float* Us = Ks + kBC * kst;             // [32][dh+1]
  float* Vs = Us + kBC * kst;             // [32][dh]
  float* As = Vs + kBC * dh;              // [32 tokens][33]
  float* Rs = As + kTM * (kBC + 1);       // [32 tokens][E]

  const int tid = threadIdx.x;
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;
  const int h = (int)(item / a.n_tiles);
  const int64_t tok0 = (item % a.n_tiles) * kTM;

  for (int idx = tid; idx < kTM * dh; idx += kThreads) {
    const int t = idx / dh, j = idx - t * dh;
    const int64_t tok = tok0 + t;
    Qs[idx] = (tok < a.N) ? a.X[tok * a.ldx + (size_t)h * dh + j] : 0.f;
  }
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
    float zinv = 0.f;
    if (tid < kTM) {
      float z = 0.f;
      for (int e = 0; e < E; ++e) z += Rs[tid * E + e];
      zinv = 1.0f / (z + a.eps);
      for (int e = 0; e < E; ++e) Rs[tid * E + e] *= zinv;
    }
  } else {
    const float* R = reinterpret_cast<const float*>(a.route);
    for (int idx = tid; idx < kTM * E; idx += kThreads) {
      const int t = idx / E, e = idx - t * E;
      const int64_t tok = tok0 + t;
      Rs[idx] = (tok < a.N) ? R[((size_t)tok * a.H + h) * E + e] : 0.f;
    }
  }
  __syncthreads();

  // thread roles
  const int c1 = tid & 31, tg1 = tid >> 5;   // products: neuron c1, tokens 4*tg1 .. +3
  const int jq = tid & 63, tq = tid >> 6;    // output: columns jq + 64*i, tokens 8*tq .. +7
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
        Vs[idx] = ok ? a.Wd[base + idx] : 0.f;
      }
      __syncthreads();
      float m[4] = {0.f, 0.f, 0.f, 0.f}, n[4] = {0.f, 0.f, 0.f, 0.f};
      for (int j = 0; j < dh; ++j) {
        const float kv = Ks[c1 * kst + j], uv = Us[c1 * kst + j];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float qv = Qs[(4 * tg1 + t) * dh + j];
          m[t] = fmaf(qv, kv, m[t]);
          n[t] = fmaf(qv, uv, n[t]);
        }
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int tok = 4 * tg1 + t;
        As[tok * (kBC + 1) + c1] = m[t] * sigmoid_f32(m[t]) * n[t] * Rs[tok * E + e];
      }
      __syncthreads();
      for (int c = 0; c < kBC; ++c) {
        float vv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = jq + 64 * i;
          vv[i] = (j < dh) ? Vs[c * dh + j] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const float av = As[(8 * tq + t) * (kBC + 1) + c];
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[t][i] = fmaf(av, vv[i], acc[t][i]);
        }
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int64_t tok = tok0 + 8 * tq + t;
    if (tok < a.N) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = jq + 64 * i;
        if (j < dh) a.Y[tok * a.ldy + (size_t)h * dh + j] = acc[t][i];
      }
    }
  }
}

}  // namespace

size_t fwd_f32_lds_bytes(const Problem& p) {
  const size_t dh = p.dh;
  return sizeof(float) * (kTM * dh + 2 * kBC * (dh + 1) + kBC * dh + kTM * (kBC + 1) +
                          (size_t)kTM * p.E);
}

int launch_fwd_f32(const Problem& p, const void* X, const void* Wg, const void* Wu,
                   const void* Wd, const void* route, void* Y, void* stream) {
  if (p.dh > kMaxDh) return (int)hipErrorInvalidValue;
  F32Args a;
  a.X = static_cast<const float*>(X);
  a.Wg = static_cast<const float*>(Wg);
  a.Wu = static_cast<const float*>(Wu);
  a.Wd = static_cast<const float*>(Wd);
  a.route = route;
  a.Y = static_cast<float*>(Y);
  a.N = p.N; a.ldx = p.ldx; a.ldy = p.ldy;
  a.H = p.H; a.dh = p.dh; a.E = p.E; a.de = p.de; a.route_mode = p.route_mode; a.eps = p.eps;
  a.n_tiles = (p.N + kTM - 1) / kTM;
  a.n_items = a.n_tiles * p.H;
  const size_t lds = fwd_f32_lds_bytes(p);
  if (hipError_t e0 = LdsLimit<&fwd_f32_kernel, (int)kLdsBytesPerWorkgroup>::ensure(); e0 != hipSuccess)
    return (int)e0;
  hipLaunchKernelGGL(fwd_f32_kernel, dim3((unsigned)xcd_grid_size(a.n_items)), dim3(kThreads),
                     lds, static_cast<hipStream_t>(stream), a);
  return (int)hipGetLastError();
}

}  // namespace mhffn
