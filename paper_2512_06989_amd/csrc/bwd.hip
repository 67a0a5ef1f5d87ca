// Fused, recompute-based backward of the Multi-Head FFN, bf16 / fp32 accumulate.
//
// Nothing of the [N][H][d_ff] intermediate is saved by the forward or written
// here: both kernels recompute M = q K^T and N = q U^T tile by tile.
//
//   bwd_tok_kernel   (appendix algorithm "Backward (dQ,dR)", plus eq:routing)
//       one workgroup = BM tokens of one head, loop over neuron tiles:
//         M^T, N^T, dA^T = V dY^T                         (3 MFMA products)
//         dr_e += sum_c dA .* SiLU(M) .* N                 (per token, per sub-network)
//         dN = r dA SiLU(M);  dM = r dA N SiLU'(M)
//         dX^T += K^T dM^T + U^T dN^T                      (2 MFMA products)
//       then, per token, the derivative through r = s/(Z+eps), s = sigmoid(p):
//         dp_e = (dr_e - sum_e' dr_e' r_e') / (Z+eps) * s_e (1 - s_e)
//         dX^T += W_r dp^T                                 (MFMA)
//       R and dp are left in the workspace as [H][E][N] fp32 for the other
//       kernels (E values per token and head, not d_ff values).
//   bwd_wgt_kernel   (appendix algorithm "Backward (dK,dU,dV)")
//       one wave = 32 neurons of one head, K/U/V rows resident in registers as
//       MFMA operands, loop over all tokens:
//         M, N, dA recomputed; dV^T += dY^T A_gated, dK^T += q^T dM, dU^T += q^T dN
//       (the q / dY tiles are read from LDS both row-wise and transposed).
//   bwd_route_kernel dW_r = sum_tokens q^T dp, two deterministic stages.
//
// LDS tiles are [32 rows][128 bf16] with the 16-byte chunks of a row permuted
// by swz(row): both the row-wise operand reads (one row per lane) and the
// transposing reads (4 consecutive rows, 64-byte windows) are then free of
// bank conflicts without padding.
#include "mhffn_device.h"
#include "mhffn_internal.h"

namespace mhffn {
namespace {

#define MHFFN_SB() __builtin_amdgcn_sched_barrier(0)

constexpr int kDh = 128;
constexpr int kTileBytes = 32 * kDh * 2;  // 8 KB

struct BwdArgs {
  const uint16_t* X;
  const uint16_t* Wg;
  const uint16_t* Wu;
  const uint16_t* Wd;
  const void* route;
  const uint16_t* dY;
  uint16_t* dX;
  uint16_t* dWg;
  uint16_t* dWu;
  uint16_t* dWd;
  void* d_route;
  float* Rws;   // [H][E][N]
  float* DPws;  // [H][E][N]  dp (params mode) or dr (weights mode)
  float* WRws;  // [H][S][128][E] partial dW_r
  int64_t N, ldx, ldy, n_tiles, n_items;
  int H, E, de, route_mode, n_split;
  float eps;
};

// ---------------------------------------------------------------------------
// token-major kernel: dX, R, dp
// ---------------------------------------------------------------------------
constexpr int kTokStageBytes = 3 * kTileBytes;  // K, U, V
constexpr int kTokStages = 2;

template <int TB, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_tok_kernel(BwdArgs a) {
  constexpr int BM = 32 * TB * NW;
  constexpr int THREADS = 64 * NW;
  constexpr int CH = 512 / THREADS;
  static_assert(CH >= 1, "");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* stage_base = smem;
  float* DRs = reinterpret_cast<float*>(smem + kTokStages * kTokStageBytes);  // [E][BM]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;
  const int h = (int)(item / a.n_tiles);
  const int64_t tile_tok0 = (item % a.n_tiles) * BM;
  const int wtok = wave * 32 * TB;
  const int E = a.E;
  const int64_t N = a.N;
  float* Rh = a.Rws + (size_t)h * E * N;
  float* DPh = a.DPws + (size_t)h * E * N;

  bf16x8 q[TB][8], dy[TB][8];
  int64_t tok[TB];
  bool valid[TB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    tok[tb] = tile_tok0 + wtok + 32 * tb + r;
    valid[tb] = tok[tb] < N;
    const int64_t t = valid[tb] ? tok[tb] : 0;
    const uint16_t* sx = a.X + t * a.ldx + h * kDh + 8 * g;
    const uint16_t* sy = a.dY + t * a.ldy + h * kDh + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      bf16x8 vx = *reinterpret_cast<const bf16x8*>(sx + 16 * ks);
      bf16x8 vy = *reinterpret_cast<const bf16x8*>(sy + 16 * ks);
      if (!valid[tb]) { vx = bf16x8{0, 0, 0, 0, 0, 0, 0, 0}; vy = vx; }
      q[tb][ks] = vx;
      dy[tb][ks] = vy;
    }
  }

  // ---- gating weights -> workspace R[h][e][tok] ----------------------------
  float inv[TB];  // 1 / (Z + eps)
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) inv[tb] = 0.f;
  if (a.route_mode == 0) {
    const int EB = (E + 31) >> 5;
    uint16_t* WrT = reinterpret_cast<uint16_t*>(stage_base);  // [32*EB][128] bf16, swizzled rows
    const uint16_t* Wr = reinterpret_cast<const uint16_t*>(a.route) + (size_t)h * kDh * E;
    for (int idx = tid; idx < kDh * E; idx += THREADS) {
      const int j = idx / E, e = idx - j * E;
      *reinterpret_cast<uint16_t*>(stage_base + tile_off(e, j >> 3) + (j & 7) * 2) = Wr[idx];
    }
    for (int idx = tid; idx < (32 * EB - E) * kDh; idx += THREADS) {
      const int e = E + idx / kDh, j = idx % kDh;
      *reinterpret_cast<uint16_t*>(stage_base + tile_off(e, j >> 3) + (j & 7) * 2) = 0;
    }
    (void)WrT;
    __syncthreads();
    float zsum[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) zsum[tb] = 0.f;
    for (int pass = 0; pass < 2; ++pass) {
      for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          f32x16 acc = {0};
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 af = *reinterpret_cast<const bf16x8*>(stage_base + tile_off(32 * eb + r, 2 * ks + g));
            acc = mfma32(af, q[tb][ks], acc);
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int e = 32 * eb + 8 * (v / 4) + 4 * g + (v % 4);
            const float s = (e < E) ? sigmoid_fast(acc[v]) : 0.f;
            if (pass == 0) {
              zsum[tb] += s;
            } else if (e < E && valid[tb]) {
              Rh[(size_t)e * N + tok[tb]] = s * inv[tb];
            }
          }
        }
      }
      if (pass == 0) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          const float z = zsum[tb] + __shfl_xor(zsum[tb], 32);
          inv[tb] = 1.0f / (z + a.eps);
        }
      }
    }
  } else {
    const float* R = reinterpret_cast<const float*>(a.route);
    for (int idx = tid; idx < BM * E; idx += THREADS) {
      const int tl = idx / E, e = idx - tl * E;
      const int64_t t = tile_tok0 + tl;
      if (t < N) Rh[(size_t)e * N + t] = R[((size_t)t * a.H + h) * E + e];
    }
  }
  __threadfence();   // R written above is read back (by this workgroup) below
  __syncthreads();

  // ---- main loop -------------------------------------------------------------
  const int tiles_per_sub = a.de / 32;
  const int T = E * tiles_per_sub;
  const size_t head_off = (size_t)h * E * a.de * kDh;
  const uint16_t* Kh = a.Wg + head_off;
  const uint16_t* Uh = a.Wu + head_off;
  const uint16_t* Vh = a.Wd + head_off;

  u32x4 kreg[CH], ureg[CH], vreg[CH];
  auto gload = [&](int t) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int chunk = tid + THREADS * i;
      const size_t off = ((size_t)t * 32 + (chunk >> 4)) * kDh + (chunk & 15) * 8;
      kreg[i] = *reinterpret_cast<const u32x4*>(Kh + off);
      ureg[i] = *reinterpret_cast<const u32x4*>(Uh + off);
      vreg[i] = *reinterpret_cast<const u32x4*>(Vh + off);
    }
  };
  auto lstore = [&](int s) {
    unsigned char* st = stage_base + s * kTokStageBytes;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int chunk = tid + THREADS * i;
      const int off = tile_off(chunk >> 4, chunk & 15);
      *reinterpret_cast<u32x4*>(st + off) = kreg[i];
      *reinterpret_cast<u32x4*>(st + kTileBytes + off) = ureg[i];
      *reinterpret_cast<u32x4*>(st + 2 * kTileBytes + off) = vreg[i];
    }
  };

  f32x16 dXa[TB][4];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) dXa[tb][jb] = f32x16{0};

  float rw[TB], rw_next[TB], drp[TB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    rw_next[tb] = valid[tb] ? Rh[tok[tb]] : 0.f;
    rw[tb] = 0.f;
    drp[tb] = 0.f;
  }
  gload(0);
  lstore(0);
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    const bool more = (t + 1 < T);
    if (more) gload(t + 1);
    const int e = t / tiles_per_sub;
    if (t % tiles_per_sub == 0) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        rw[tb] = rw_next[tb];
        rw_next[tb] = (e + 1 < E && valid[tb]) ? Rh[(size_t)(e + 1) * N + tok[tb]] : 0.f;
      }
    }
    const unsigned char* st = stage_base + (t & 1) * kTokStageBytes;

    f32x16 accM[TB], accN[TB], accA[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) { accM[tb] = f32x16{0}; accN[tb] = f32x16{0}; accA[tb] = f32x16{0}; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const int off = tile_off(r, 2 * ks + g);
      const bf16x8 ak = *reinterpret_cast<const bf16x8*>(st + off);
      const bf16x8 au = *reinterpret_cast<const bf16x8*>(st + kTileBytes + off);
      const bf16x8 av = *reinterpret_cast<const bf16x8*>(st + 2 * kTileBytes + off);
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        accM[tb] = mfma32(ak, q[tb][ks], accM[tb]);
        accN[tb] = mfma32(au, q[tb][ks], accN[tb]);
        accA[tb] = mfma32(av, dy[tb][ks], accA[tb]);
      }
    }
    bf16x8 dmf[TB][2], dnf[TB][2];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        u32x4 pm, pn;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float dmv[2], dnv[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int v = 8 * t2 + 2 * i + u;
            const float m = accM[tb][v], n = accN[tb][v], da = accA[tb][v];
            const float sg = sigmoid_fast(m);
            const float silu = m * sg;
            drp[tb] = fmaf(da * silu, n, drp[tb]);
            const float rda = rw[tb] * da;
            dnv[u] = rda * silu;
            dmv[u] = rda * n * fmaf(silu, 1.0f - sg, sg);  // SiLU'(m) = sg + silu (1 - sg)
          }
          pm[i] = pack_bf16(dmv[0], dmv[1]);
          pn[i] = pack_bf16(dnv[0], dnv[1]);
        }
        dmf[tb][t2] = __builtin_bit_cast(bf16x8, pm);
        dnf[tb][t2] = __builtin_bit_cast(bf16x8, pn);
      }
    }
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
      for (int jb = 0; jb < 4; ++jb) {
        const bf16x8 kt = tile_read_tr(st, 16 * t2 + 4 * g, 32 * jb, lane);
        const bf16x8 ut = tile_read_tr(st + kTileBytes, 16 * t2 + 4 * g, 32 * jb, lane);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          dXa[tb][jb] = mfma32(kt, dmf[tb][t2], dXa[tb][jb]);
          dXa[tb][jb] = mfma32(ut, dnf[tb][t2], dXa[tb][jb]);
        }
      }
    }
    if ((t + 1) % tiles_per_sub == 0) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        const float dr = drp[tb] + __shfl_xor(drp[tb], 32);
        if (g == 0) DRs[e * BM + wtok + 32 * tb + r] = dr;
        drp[tb] = 0.f;
      }
    }
    if (more) lstore((t + 1) & 1);
    __syncthreads();
  }

  // ---- derivative through the gating weights ------------------------------------
  if (a.route_mode == 0) {
    // stage W_r[h] as rows j, columns e (zero padded to 32*EB), for the A operand
    const int EB = (E + 31) >> 5;
    const int wr_stride = 64 * EB + 16;  // bytes per row; +16 keeps rows off the same banks
    const uint16_t* Wr = reinterpret_cast<const uint16_t*>(a.route) + (size_t)h * kDh * E;
    for (int idx = tid; idx < kDh * 32 * EB; idx += THREADS) {
      const int j = idx / (32 * EB), e = idx - j * (32 * EB);
      *reinterpret_cast<uint16_t*>(stage_base + j * wr_stride + e * 2) = (e < E) ? Wr[j * E + e] : 0;
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      float* drcol = DRs + wtok + 32 * tb + r;
      float dot = 0.f;
      if (valid[tb])
        for (int e = 0; e < E; ++e) dot = fmaf(drcol[e * BM], Rh[(size_t)e * N + tok[tb]], dot);
      const float zpe = 1.0f / inv[tb];
      // lanes g = 0 and g = 1 of a token split the sub-networks between them
      for (int e = g; e < E; e += 2) {
        float dp = 0.f;
        if (valid[tb]) {
          const float rr = Rh[(size_t)e * N + tok[tb]];
          const float s = rr * zpe;
          dp = (drcol[e * BM] - dot) * inv[tb] * s * (1.0f - s);
          DPh[(size_t)e * N + tok[tb]] = dp;
        }
        drcol[e * BM] = dp;
      }
    }
    __syncthreads();  // W_r staged; dp of both half-waves visible
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      for (int ks = 0; ks < 2 * EB; ++ks) {
        if (16 * ks >= E) break;
        u32x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int e0 = 16 * ks + 8 * g + 2 * i;
          const float d0 = (e0 < E) ? DRs[e0 * BM + wtok + 32 * tb + r] : 0.f;
          const float d1 = (e0 + 1 < E) ? DRs[(e0 + 1) * BM + wtok + 32 * tb + r] : 0.f;
          pk[i] = pack_bf16(d0, d1);
        }
        const bf16x8 bp = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
          const bf16x8 aw = *reinterpret_cast<const bf16x8*>(stage_base + (32 * jb + r) * wr_stride +
                                                             (16 * ks + 8 * g) * 2);
          dXa[tb][jb] = mfma32(aw, bp, dXa[tb][jb]);
        }
      }
    }
  } else {
    // weights mode: dR is an output, laid out like R
    float* dR = reinterpret_cast<float*>(a.d_route);
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      if (valid[tb]) {
        for (int e = g; e < E; e += 2) {
          const float dr = DRs[e * BM + wtok + 32 * tb + r];
          if (dR) dR[((size_t)tok[tb] * a.H + h) * E + e] = dr;
        }
      }
    }
  }

  if (a.dX) {
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      if (valid[tb]) {
        uint16_t* dst = a.dX + tok[tb] * a.ldx + h * kDh + 4 * g;
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            u32x2 pk;
            pk[0] = pack_bf16(dXa[tb][jb][4 * vq], dXa[tb][jb][4 * vq + 1]);
            pk[1] = pack_bf16(dXa[tb][jb][4 * vq + 2], dXa[tb][jb][4 * vq + 3]);
            *reinterpret_cast<u32x2*>(dst + 32 * jb + 8 * vq) = pk;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// weight-major kernel: dK, dU, dV
// ---------------------------------------------------------------------------
constexpr int kWgtWaves = 4;
constexpr int kWgtThreads = 64 * kWgtWaves;
constexpr int kWgtStageBytes = 2 * kTileBytes + kWgtWaves * 32 * 4;  // q tile, dY tile, r per wave

__global__ __launch_bounds__(kWgtThreads) void bwd_wgt_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int nblk = a.E * a.de / 32;              // 32-neuron blocks per head
  const int wg_per_head = (nblk + kWgtWaves - 1) / kWgtWaves;
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;
  const int h = (int)(item / wg_per_head);
  const int blk = (int)(item % wg_per_head) * kWgtWaves + wave;
  const bool active = blk < nblk;
  const int blk_c = active ? blk : nblk - 1;     // idle waves shadow a valid block, store nothing
  const int64_t N = a.N;
  const size_t row0 = (size_t)h * nblk * 32 + (size_t)blk_c * 32;  // first neuron row of this wave

  // resident weight operands: lane (neuron r, half g) holds columns 16ks + 8g ..
  // (re-reading them from a wave-private LDS copy every step instead was measured
  // 17 % slower: the LDS pipe is the scarcer resource)
  bf16x8 Kf[8], Uf[8], Vf[8];
  {
    const size_t off = (row0 + r) * kDh + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      Kf[ks] = *reinterpret_cast<const bf16x8*>(a.Wg + off + 16 * ks);
      Uf[ks] = *reinterpret_cast<const bf16x8*>(a.Wu + off + 16 * ks);
      Vf[ks] = *reinterpret_cast<const bf16x8*>(a.Wd + off + 16 * ks);
    }
  }
  f32x16 dK[4], dU[4], dV[4];
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) { dK[jb] = f32x16{0}; dU[jb] = f32x16{0}; dV[jb] = f32x16{0}; }

  // per-wave sub-network of the r values each thread stages (threads 0..127)
  const int stage_wave = tid >> 5, stage_tok = tid & 31;
  int e_stage = 0;
  {
    const int b2 = (int)(item % wg_per_head) * kWgtWaves + stage_wave;
    e_stage = (b2 < nblk ? b2 : nblk - 1) / (a.de / 32);
  }
  const float* Rh = a.Rws + (size_t)h * a.E * N;

  u32x4 qreg[2], yreg[2];
  float rreg = 0.f;
  auto gload = [&](int64_t tok0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int chunk = tid + kWgtThreads * i;
      const int64_t t = tok0 + (chunk >> 4);
      if (t < N) {
        qreg[i] = *reinterpret_cast<const u32x4*>(a.X + t * a.ldx + h * kDh + (chunk & 15) * 8);
        yreg[i] = *reinterpret_cast<const u32x4*>(a.dY + t * a.ldy + h * kDh + (chunk & 15) * 8);
      } else {
        qreg[i] = u32x4{0, 0, 0, 0};
        yreg[i] = u32x4{0, 0, 0, 0};
      }
    }
    if (tid < 128) {
      const int64_t t = tok0 + stage_tok;
      rreg = (t < N) ? Rh[(size_t)e_stage * N + t] : 0.f;
    }
  };
  auto lstore = [&](int s) {
    unsigned char* st = smem + s * kWgtStageBytes;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int chunk = tid + kWgtThreads * i;
      const int off = tile_off(chunk >> 4, chunk & 15);
      *reinterpret_cast<u32x4*>(st + off) = qreg[i];
      *reinterpret_cast<u32x4*>(st + kTileBytes + off) = yreg[i];
    }
    if (tid < 128) reinterpret_cast<float*>(st + 2 * kTileBytes)[tid] = rreg;
  };

  const int64_t nb = (N + 31) / 32;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int64_t b = 0; b < nb; ++b) {
    const bool more = (b + 1 < nb);
    if (more) gload((b + 1) * 32);
    const unsigned char* st = smem + (b & 1) * kWgtStageBytes;
    const unsigned char* qt = st;
    const unsigned char* yt = st + kTileBytes;
    const float* rt = reinterpret_cast<const float*>(st + 2 * kTileBytes) + wave * 32;

    // One wave per SIMD: nothing but this wave's own instruction stream can keep the
    // MFMA pipe and the VALU busy at the same time, so the step is written as an
    // explicit interleave (scheduling barriers pin it):
    //   1. M and N chains (16 MFMA)
    //   2. dA chain (8 MFMA)            || everything that needs only m, n, r   (12 VALU / element)
    //   3. gradient MFMAs of tokens 0-15 || dn, dm, rounding of tokens 16-31
    //   4. gradient MFMAs of tokens 16-31
    // M[tok][c], N[tok][c], dA[tok][c]: lane = neuron column, registers = token rows;
    // registers 8*t2 + 4*hi + x hold tokens 16*t2 + 8*hi + 4g + x.
    f32x4 rv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rv[i] = *reinterpret_cast<const f32x4*>(rt + 8 * i + 4 * g);
    bf16x8 oa[4], ob[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) oa[ks] = *reinterpret_cast<const bf16x8*>(qt + tile_off(r, 2 * ks + g));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) ob[ks] = *reinterpret_cast<const bf16x8*>(qt + tile_off(r, 2 * (ks + 4) + g));
    MHFFN_SB();
    f32x16 accM, accN, accA;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks == 0) { accM = mfma32(oa[0], Kf[0], f32x16{0}); accN = mfma32(oa[0], Uf[0], f32x16{0}); }
      else { accM = mfma32(oa[ks], Kf[ks], accM); accN = mfma32(oa[ks], Uf[ks], accN); }
    }
    MHFFN_SB();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) oa[ks] = *reinterpret_cast<const bf16x8*>(yt + tile_off(r, 2 * ks + g));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) { accM = mfma32(ob[ks], Kf[ks + 4], accM); accN = mfma32(ob[ks], Uf[ks + 4], accN); }
    MHFFN_SB();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) ob[ks] = *reinterpret_cast<const bf16x8*>(yt + tile_off(r, 2 * (ks + 4) + g));
    // transposed operands of tokens 0-15, fetched under the arithmetic below
    bf16x8 yT[4], qT[4];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      yT[jb] = tile_read_tr(yt, 4 * g, 32 * jb, lane);
      qT[jb] = tile_read_tr(qt, 4 * g, 32 * jb, lane);
    }
    MHFFN_SB();
    float Pw[16], Qw[16];   // r silu(m)  and  r n silu'(m)
    u32x4 pa[2];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (ks == 0) accA = mfma32(oa[0], Vf[0], f32x16{0});
      else accA = mfma32(ks < 4 ? oa[ks] : ob[ks - 4], Vf[ks], accA);
      float av[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int v = 2 * ks + u;
        const float rwv = rv[v >> 2][v & 3];
        const float m = accM[v], n = accN[v];
        const float t = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * m);
        const float sg = __builtin_amdgcn_rcpf(1.0f + t);
        const float sw = rwv * sg;
        const float x = (1.0f + m) - m * sg;   // silu'(m) = sg (1 + m - silu(m))
        Pw[v] = m * sw;
        Qw[v] = (n * sw) * x;
        av[u] = Pw[v] * n;
      }
      pa[ks >> 2][ks & 3] = pack_bf16(av[0], av[1]);
      MHFFN_SB();
    }
    // tokens 0-15: dn = P da, dm = Q da
    u32x4 pm, pn;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pm[i] = pack_bf16(Qw[2 * i] * accA[2 * i], Qw[2 * i + 1] * accA[2 * i + 1]);
      pn[i] = pack_bf16(Pw[2 * i] * accA[2 * i], Pw[2 * i + 1] * accA[2 * i + 1]);
    }
    bf16x8 agf = __builtin_bit_cast(bf16x8, pa[0]);
    bf16x8 dmf = __builtin_bit_cast(bf16x8, pm), dnf = __builtin_bit_cast(bf16x8, pn);
    MHFFN_SB();
    // dV^T[j][c] += dY^T A_g ; dK^T[j][c] += q^T dM ; dU^T[j][c] += q^T dN  (contraction over tokens)
    u32x4 pm1, pn1;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      dV[jb] = mfma32(yT[jb], agf, dV[jb]);
      dK[jb] = mfma32(qT[jb], dmf, dK[jb]);
      dU[jb] = mfma32(qT[jb], dnf, dU[jb]);
      yT[jb] = tile_read_tr(yt, 16 + 4 * g, 32 * jb, lane);   // operands of tokens 16-31
      qT[jb] = tile_read_tr(qt, 16 + 4 * g, 32 * jb, lane);
      pm1[jb] = pack_bf16(Qw[8 + 2 * jb] * accA[8 + 2 * jb], Qw[9 + 2 * jb] * accA[9 + 2 * jb]);
      pn1[jb] = pack_bf16(Pw[8 + 2 * jb] * accA[8 + 2 * jb], Pw[9 + 2 * jb] * accA[9 + 2 * jb]);
      MHFFN_SB();
    }
    agf = __builtin_bit_cast(bf16x8, pa[1]);
    dmf = __builtin_bit_cast(bf16x8, pm1);
    dnf = __builtin_bit_cast(bf16x8, pn1);
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      dV[jb] = mfma32(yT[jb], agf, dV[jb]);
      dK[jb] = mfma32(qT[jb], dmf, dK[jb]);
      dU[jb] = mfma32(qT[jb], dnf, dU[jb]);
    }
    if (more) lstore((b + 1) & 1);
    __syncthreads();
  }

  if (active) {
    // accumulators are [j][c]: lane = neuron column r, register v = row 32jb + 8(v/4) + 4g + v%4
    const size_t off = (row0 + r) * kDh + 4 * g;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const size_t o = off + 32 * jb + 8 * vq;
        if (a.dWg) {
          u32x2 pk;
          pk[0] = pack_bf16(dK[jb][4 * vq], dK[jb][4 * vq + 1]);
          pk[1] = pack_bf16(dK[jb][4 * vq + 2], dK[jb][4 * vq + 3]);
          *reinterpret_cast<u32x2*>(a.dWg + o) = pk;
        }
        if (a.dWu) {
          u32x2 pk;
          pk[0] = pack_bf16(dU[jb][4 * vq], dU[jb][4 * vq + 1]);
          pk[1] = pack_bf16(dU[jb][4 * vq + 2], dU[jb][4 * vq + 3]);
          *reinterpret_cast<u32x2*>(a.dWu + o) = pk;
        }
        if (a.dWd) {
          u32x2 pk;
          pk[0] = pack_bf16(dV[jb][4 * vq], dV[jb][4 * vq + 1]);
          pk[1] = pack_bf16(dV[jb][4 * vq + 2], dV[jb][4 * vq + 3]);
          *reinterpret_cast<u32x2*>(a.dWd + o) = pk;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// dW_r[h][j][e] = sum_tok q[tok][j] dp[tok][e]: partial sums per token split,
// then a fixed-order reduction (deterministic).
// ---------------------------------------------------------------------------
constexpr int kRouteSplit = 16;                 // workgroups per head
constexpr int kRouteParts = kRouteSplit * 4;    // one partial per wave
constexpr int kRouteMaxSub = 96;

// D[j][e] += sum_tok q^T[j][tok] dp[tok][e] on the MFMA: the A operand is the
// transposing LDS read of a [32 tok][128] tile of X, the B operand (contraction
// slot s <-> token 16*t2 + 8*(s/4) + 4g + s%4, column e) comes straight from
// the [H][E][N] dp array.  Each wave walks its own token blocks and leaves its
// own partial [128][E] in the workspace.
template <int EB>
__global__ __launch_bounds__(256) void bwd_route_partial_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char tiles[4 * kTileBytes];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int h = blockIdx.x;
  const int part = blockIdx.y * 4 + wave;
  const int64_t N = a.N;
  const int E = a.E;
  const int64_t nb = (N + 31) / 32;
  const int64_t iters = (nb + kRouteParts - 1) / kRouteParts;  // same for every wave
  const float* DPh = a.DPws + (size_t)h * E * N;
  unsigned char* tile = tiles + wave * kTileBytes;
  f32x16 acc[EB][4];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) acc[eb][jb] = f32x16{0};

  for (int64_t it = 0; it < iters; ++it) {
    const int64_t b = it * kRouteParts + part;
    const int64_t tok0 = b * 32;   // may lie beyond N: then everything loaded is zero
    // X tile -> this wave's LDS tile (8 chunks per lane)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int chunk = lane + 64 * i;
      const int64_t t = tok0 + (chunk >> 4);
      u32x4 v = {0, 0, 0, 0};
      if (t < N) v = *reinterpret_cast<const u32x4*>(a.X + t * a.ldx + h * kDh + (chunk & 15) * 8);
      *reinterpret_cast<u32x4*>(tile + tile_off(chunk >> 4, chunk & 15)) = v;
    }
    // dp operands
    bf16x8 bp[EB][2];
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) {
      const int e = 32 * eb + r;
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        float v[8];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
          const int64_t t = tok0 + 16 * t2 + 8 * (s8 >> 2) + 4 * g + (s8 & 3);
          v[s8] = (e < E && t < N) ? DPh[(size_t)e * N + t] : 0.f;
        }
        u32x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) pk[i] = pack_bf16(v[2 * i], v[2 * i + 1]);
        bp[eb][t2] = __builtin_bit_cast(bf16x8, pk);
      }
    }
    __syncthreads();
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
      for (int jb = 0; jb < 4; ++jb) {
        const bf16x8 qT = tile_read_tr(tile, 16 * t2 + 4 * g, 32 * jb, lane);
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) acc[eb][jb] = mfma32(qT, bp[eb][t2], acc[eb][jb]);
      }
    }
    __syncthreads();
  }
  float* out = a.WRws + ((size_t)h * kRouteParts + part) * kDh * E;
#pragma unroll
  for (int eb = 0; eb < EB; ++eb) {
    const int e = 32 * eb + r;
    if (e < E) {
#pragma unroll
      for (int jb = 0; jb < 4; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int j = 32 * jb + 8 * (v / 4) + 4 * g + (v % 4);
          out[j * E + e] = acc[eb][jb][v];
        }
    }
  }
}

__global__ void bwd_route_reduce_kernel(BwdArgs a) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_head = (int64_t)kDh * a.E;
  if (idx >= per_head * a.H) return;
  const int h = (int)(idx / per_head);
  const int64_t o = idx % per_head;
  float sum = 0.f;
  for (int s = 0; s < a.n_split; ++s) sum += a.WRws[((size_t)h * a.n_split + s) * per_head + o];
  reinterpret_cast<uint16_t*>(a.d_route)[idx] = (uint16_t)(pack_bf16(sum, 0.f) & 0xFFFFu);
}

// zero-fill for the N == 0 case (gradients of an empty batch are zero)
__global__ void fill_zero_kernel(uint32_t* p, size_t n_words) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) p[i] = 0;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t bwd_workspace_bytes(const Problem& p, int dtype) {
  if (dtype != 1 || p.N == 0) return 0;   // an empty batch only zero-fills the weight gradients
  const size_t nhe = align256((size_t)p.N * p.H * p.E * sizeof(float));
  const size_t wr = align256((size_t)p.H * kRouteParts * kDh * p.E * sizeof(float));
  return 2 * nhe + wr;
}

int launch_bwd(const Problem& p, int dtype, const void* X, const void* Wg, const void* Wu,
               const void* Wd, const void* route, const void* dY, void* dX, void* dWg,
               void* dWu, void* dWd, void* d_route, void* ws, void* stream_,
               void* const* phase_events, int n_phase_events) {
  if (dtype != 1) return -1;        // fp32 fused backward: not built
  if (p.E > kRouteMaxSub) return -1;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // event i is recorded after phase i-1 (event 0: before anything is launched)
  auto mark = [&](int i) -> hipError_t {
    if (i < n_phase_events && phase_events && phase_events[i])
      return hipEventRecord(static_cast<hipEvent_t>(phase_events[i]), stream);
    return hipSuccess;
  };
  if (mark(0) != hipSuccess) return (int)hipErrorInvalidHandle;
  const size_t wcount = (size_t)p.H * p.E * p.de * kDh;
  if (p.N == 0) {
    void* outs[4] = {dWg, dWu, dWd, p.route_mode == 0 ? d_route : nullptr};
    const size_t words[4] = {wcount / 2, wcount / 2, wcount / 2, (size_t)p.H * kDh * p.E / 2};
    for (int i = 0; i < 4; ++i) {
      if (!outs[i] || !words[i]) continue;
      hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words[i] + 255) / 256)), dim3(256), 0,
                         stream, static_cast<uint32_t*>(outs[i]), words[i]);
    }
    return (int)hipGetLastError();
  }
  BwdArgs a;
  a.X = static_cast<const uint16_t*>(X);
  a.Wg = static_cast<const uint16_t*>(Wg);
  a.Wu = static_cast<const uint16_t*>(Wu);
  a.Wd = static_cast<const uint16_t*>(Wd);
  a.route = route;
  a.dY = static_cast<const uint16_t*>(dY);
  a.dX = static_cast<uint16_t*>(dX);
  a.dWg = static_cast<uint16_t*>(dWg);
  a.dWu = static_cast<uint16_t*>(dWu);
  a.dWd = static_cast<uint16_t*>(dWd);
  a.d_route = d_route;
  const size_t nhe = align256((size_t)p.N * p.H * p.E * sizeof(float));
  a.Rws = reinterpret_cast<float*>(static_cast<unsigned char*>(ws));
  a.DPws = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + nhe);
  a.WRws = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + 2 * nhe);
  a.N = p.N; a.ldx = p.ldx; a.ldy = p.ldy;
  a.H = p.H; a.E = p.E; a.de = p.de; a.route_mode = p.route_mode; a.eps = p.eps;
  a.n_split = kRouteParts;

  // token-major kernel (always: it also produces R for the weight-major kernel)
  {
    constexpr int TB = 1, NW = 8, BM = 32 * TB * NW;
    a.n_tiles = (p.N + BM - 1) / BM;
    a.n_items = a.n_tiles * p.H;
    const size_t lds = (size_t)kTokStages * kTokStageBytes + (size_t)p.E * BM * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_tok_kernel<TB, NW>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)kLdsBytesPerWorkgroup);
      if (e != hipSuccess) return (int)e;
      attr_set = true;
    }
    hipLaunchKernelGGL((bwd_tok_kernel<TB, NW>), dim3((unsigned)xcd_grid_size(a.n_items)),
                       dim3(64 * NW), lds, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  if (mark(1) != hipSuccess) return (int)hipErrorInvalidHandle;
  if (dWg || dWu || dWd) {
    const int nblk = p.E * p.de / 32;
    const int wg_per_head = (nblk + kWgtWaves - 1) / kWgtWaves;
    a.n_items = (int64_t)wg_per_head * p.H;
    hipLaunchKernelGGL(bwd_wgt_kernel, dim3((unsigned)xcd_grid_size(a.n_items)), dim3(kWgtThreads),
                       2 * kWgtStageBytes, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  if (mark(2) != hipSuccess) return (int)hipErrorInvalidHandle;
  if (d_route && p.route_mode == 0) {
    const dim3 rgrid(p.H, kRouteSplit);
    if (p.E <= 32) hipLaunchKernelGGL(bwd_route_partial_kernel<1>, rgrid, dim3(256), 0, stream, a);
    else if (p.E <= 64) hipLaunchKernelGGL(bwd_route_partial_kernel<2>, rgrid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(bwd_route_partial_kernel<3>, rgrid, dim3(256), 0, stream, a);
    const int64_t n = (int64_t)p.H * kDh * p.E;
    hipLaunchKernelGGL(bwd_route_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  if (mark(3) != hipSuccess) return (int)hipErrorInvalidHandle;
  return 0;
}

}  // namespace mhffn
