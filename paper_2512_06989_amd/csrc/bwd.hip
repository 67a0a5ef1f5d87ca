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
//   bwd_wgt16_kernel (appendix algorithm "Backward (dK,dU,dV)")
//       one wave = 16 neurons of one head, K/U/V rows resident in registers as
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

#include <type_traits>

namespace mhffn {
namespace {

// Tile layout of the kernels in this file with 32x32x16 products (token-major kernel, gating
// scratch, routing-gradient kernel).  d_h = 128 and 256: the general swizzled tile.  d_h = 64
// (rows of 128 bytes, two rows per 256-byte line): the eight chunks of a row are permuted by
//     s(row) = b1 | b2 << 1 | (b1 ^ b3) << 2        (b_i = bit i of the row number),
// with which the row reads (one row per lane, lane groups of a 16-byte read) and the
// transposing reads (rows 4g + i/4 and + 8 in the two 32-byte windows of a lane half) are
// both free of bank conflicts; with the general d_h = 64 layout the transposing reads of this
// geometry took twice their cycles.
template <int DH>
__device__ __forceinline__ int btile_off(int row, int chunk) {
  if constexpr (DH == 64) {
    const int s = ((row >> 1) & 1) | (((row >> 2) & 1) << 1) | ((((row >> 1) ^ (row >> 3)) & 1) << 2);
    return row * 128 + ((chunk ^ s) << 4);
  } else {
    return tile_off_dh<DH>(row, chunk);
  }
}
template <int DH>
__device__ __forceinline__ int btile_off8(int row, int col) {
  return btile_off<DH>(row, col >> 3) + ((col & 4) << 1);
}
template <int DH>
__device__ __forceinline__ bf16x8 btile_read_tr(const unsigned char* tile, int r0, int c0, int lane) {
  const int li = lane & 15;
  const int row = r0 + (li >> 2);
  const int col = c0 + 16 * ((lane >> 4) & 1) + 4 * (li & 3);
  return join_tr(lds_read_tr16(tile + btile_off8<DH>(row, col)), lds_read_tr16(tile + btile_off8<DH>(row + 8, col)));
}

#define MHFFN_SB() __builtin_amdgcn_sched_barrier(0)

constexpr int kDh = 128;
constexpr int kTileBytes = 32 * kDh * 2;  // 8 KB

template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

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
  // weight-major kernel with the tokens shared out over `wsplit` workgroups per neuron group
  // (only when the neuron groups alone fill less than a round of the chip well): fp32
  // partial gradients [wsplit][3][H*E*d_e][128], summed in fixed order afterwards
  float* WPws;
  int wsplit;
  int64_t blocks_per_seg;
  // d_h = 128 weight-major kernel: the neuron groups of an XCD's share are `gpx` (of `n_groups`
  // in all); the first `full_px` of them take all tokens and store their gradients, the
  // others share the tokens out over `wsplit` workgroups each and leave fp32 partials
  // [wsplit][3][8 * (gpx - full_px) groups][128 rows][128]
  int gpx, full_px, n_groups;
  int64_t N, ldx, ldy, n_tiles, n_items;
  int H, E, de, dh, route_mode, n_split;
  float eps;
};

// ---------------------------------------------------------------------------
// token-major kernel: dX, R, dp
// ---------------------------------------------------------------------------
constexpr int tok_stage_bytes(int dh) { return 3 * 32 * dh * 2; }  // K, U, V tiles of 32 rows
// Weight tiles reach LDS either through registers (two stages: loaded at the top of a step,
// stored at its end) or, DMA = true (d_h = 128, 512 threads: one 16-byte chunk of each tile
// per thread), by direct global -> LDS loads into three stages, requested two steps ahead:
// no staging registers, no LDS stores, and the step ends on a counted wait and a bare barrier.
constexpr int tok_stages(bool dma) { return dma ? 3 : 2; }

// PHASED (with DMA): the two waves of a SIMD run half a step apart.  A step is two halves,
// the gate/up/dA products (MFMA only) and the activation arithmetic plus the dX products
// (VALU, then MFMA), each closed by a barrier; waves NW/2 .. NW-1 pass one barrier more before
// the loop and the others one more after it, so that a SIMD always has one wave in each half
// and the arithmetic of one hides behind the products of the other.  Same code for both, no
// extra registers.  A tile is then read during three consecutive half-steps; its stage is
// requested again at the start of the fourth (the late waves are then at the top of a step,
// the early ones in its middle), and every wave waits for its own requests at the end of the
// half-step in which it made them, two half-steps before the first use.
template <int DH, int TB, int NW, bool DMA = false, bool PHASED = false, bool PIPE = false>
__global__ __launch_bounds__(64 * NW, DH == 64 ? 2 : 1) void bwd_tok_kernel(BwdArgs a) {
  static_assert(!DMA || (TB == 1 && ((DH == 128 && NW == 8) || (DH == 256 && NW == 4))),
                "direct staging: a wave-wide load moves 1 KB, a tile is 32 rows");
  static_assert(DMA || !PHASED, "the half-step schedule relies on direct staging");
  static_assert(!PIPE || (DMA && !PHASED && DH == 256), "the one-wave pipeline is written for d_h = 256");
  constexpr int kTokStages = tok_stages(DMA);
  constexpr int BM = 32 * TB * NW;
  constexpr int THREADS = 64 * NW;
  constexpr int KS = DH / 16;              // contraction steps over the head width
  constexpr int JB = DH / 32;              // 32-row output tiles over the head width
  constexpr int CPR = DH / 8;              // 16-byte chunks per row
  constexpr int kTileBytes = 32 * DH * 2;
  constexpr int kTokStageBytes = tok_stage_bytes(DH);
  constexpr int CHUNKS = 32 * CPR;
  constexpr int CH = (CHUNKS + THREADS - 1) / THREADS;
  constexpr bool kAllLoad = (CHUNKS % THREADS == 0);   // else the upper threads carry none
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];   // (the one-wave pipeline XORs address bits)
  unsigned char* stage_base = smem;
  float* DRs = reinterpret_cast<float*>(smem + kTokStages * kTokStageBytes);  // [E][BM]: r_e, then dr_e

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

  const int tiles_per_sub = a.de / 32;
  const int T = E * tiles_per_sub;
  const size_t head_off = (size_t)h * E * a.de * DH;
  const uint16_t* Kh = a.Wg + head_off;
  const uint16_t* Uh = a.Wu + head_off;
  const uint16_t* Vh = a.Wd + head_off;
  // direct staging: a wave-wide load fills 1 KB of a tile, kDmaRows rows; the NW waves fill
  // kDmaRows NW rows per round, a tile in kDmaRounds rounds (d_h = 128: one round of 8 waves x 4
  // rows; d_h = 256: four rounds of 4 waves x 2 rows).  Lane l lands at chunk position l % CPR
  // of its row and fetches the global chunk that the swizzle maps there (the swizzle is an
  // involution on the chunk index of a row).
  constexpr int kDmaRows = DMA ? 1024 / (2 * DH) : 1;
  constexpr int kDmaRounds = DMA ? 32 / (kDmaRows * NW) : 1;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  int dma_goff[kDmaRounds];   // elements
#pragma unroll
  for (int i = 0; i < kDmaRounds; ++i) {
    const int drow = kDmaRows * (NW * i + wave) + lane / CPR;
    const int dchunk = (btile_off<DH>(drow, lane % CPR) - drow * 2 * DH) >> 4;
    dma_goff[i] = drow * DH + dchunk * 8;
  }
  auto dma_round = [&](int t, int stage, int i) {
    const size_t off = (size_t)t * (32 * DH) + dma_goff[i];
    unsigned char* dst = stage_base + stage * kTokStageBytes + (NW * i + wave_u) * 1024;
    global_to_lds_16B(Kh + off, dst);
    global_to_lds_16B(Uh + off, dst + kTileBytes);
    global_to_lds_16B(Vh + off, dst + 2 * kTileBytes);
  };
  auto dma = [&](int t, int stage) {
#pragma unroll
    for (int i = 0; i < kDmaRounds; ++i) dma_round(t, stage, i);
  };
  // the gating prologue stages W_r^T (up to 24 KB) in one stage: the last one, so that the
  // first two tiles can be on their way meanwhile (the epilogue, with all stages retired,
  // starts from the first)
  unsigned char* scratch = stage_base + (DMA ? 2 * kTokStageBytes : 0);

  bf16x8 q[TB][KS], dy[TB][KS];
  int64_t tok[TB];
  bool valid[TB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    tok[tb] = tile_tok0 + wtok + 32 * tb + r;
    valid[tb] = tok[tb] < N;
    const int64_t t = valid[tb] ? tok[tb] : 0;
    const uint16_t* sx = a.X + t * a.ldx + h * DH + 8 * g;
    const uint16_t* sy = a.dY + t * a.ldy + h * DH + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 vx = *reinterpret_cast<const bf16x8*>(sx + 16 * ks);
      bf16x8 vy = *reinterpret_cast<const bf16x8*>(sy + 16 * ks);
      if (!valid[tb]) { vx = bf16x8{0, 0, 0, 0, 0, 0, 0, 0}; vy = vx; }
      q[tb][ks] = vx;
      dy[tb][ks] = vy;
    }
  }
  if constexpr (DMA) {
    dma(0, 0);
    if (T > 1) dma(1, 1);
  }

  // ---- gating weights -> workspace R[h][e][tok] ----------------------------
  float inv[TB];  // 1 / (Z + eps)
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) inv[tb] = 0.f;
  if (a.route_mode == 0) {
    const int EB = (E + 31) >> 5;
    // W_r^T as [32*EB][DH] bf16, swizzled rows
    const uint16_t* Wr = reinterpret_cast<const uint16_t*>(a.route) + (size_t)h * DH * E;
    for (int idx = tid; idx < DH * E; idx += THREADS) {
      const int j = idx / E, e = idx - j * E;
      *reinterpret_cast<uint16_t*>(scratch + btile_off<DH>(e, j >> 3) + (j & 7) * 2) = Wr[idx];
    }
    for (int idx = tid; idx < (32 * EB - E) * DH; idx += THREADS) {
      const int e = E + idx / DH, j = idx % DH;
      *reinterpret_cast<uint16_t*>(scratch + btile_off<DH>(e, j >> 3) + (j & 7) * 2) = 0;
    }
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
          for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 af = *reinterpret_cast<const bf16x8*>(scratch + btile_off<DH>(32 * eb + r, 2 * ks + g));
            acc = mfma32(af, q[tb][ks], acc);
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int e = 32 * eb + 8 * (v / 4) + 4 * g + (v % 4);
            const float s = (e < E) ? sigmoid_fast(acc[v]) : 0.f;
            if (pass == 0) {
              zsum[tb] += s;
            } else if (e < E) {
              const float rv = s * inv[tb];
              if (valid[tb]) Rh[(size_t)e * N + tok[tb]] = rv;
              DRs[e * BM + wtok + 32 * tb + r] = rv;   // until sub-network e has been swept
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
      const float rv = (t < N) ? R[((size_t)t * a.H + h) * E + e] : 0.f;
      if (t < N) Rh[(size_t)e * N + t] = rv;
      DRs[e * BM + tl] = rv;
    }
  }
  __threadfence();   // R written above is read back (by this workgroup) in the epilogue
  __syncthreads();   // (waits for every load in flight: direct staging has tiles 0 and 1 in place)

  // ---- main loop -------------------------------------------------------------
  u32x4 kreg[DMA ? 1 : CH], ureg[DMA ? 1 : CH], vreg[DMA ? 1 : CH];
  auto gload = [&](int t) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int chunk = tid + THREADS * i;
      if (!kAllLoad && chunk >= CHUNKS) continue;
      const size_t off = ((size_t)t * 32 + chunk / CPR) * DH + (chunk % CPR) * 8;
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
      if (!kAllLoad && chunk >= CHUNKS) continue;
      const int off = btile_off<DH>(chunk / CPR, chunk % CPR);
      *reinterpret_cast<u32x4*>(st + off) = kreg[i];
      *reinterpret_cast<u32x4*>(st + kTileBytes + off) = ureg[i];
      *reinterpret_cast<u32x4*>(st + 2 * kTileBytes + off) = vreg[i];
    }
  };

  f32x16 dXa[TB][JB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) dXa[tb][jb] = f32x16{0};

  float rw[TB], drp[TB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    rw[tb] = 0.f;
    drp[tb] = 0.f;
  }
  if constexpr (!DMA) {
    gload(0);
    lstore(0);
    __syncthreads();
  }
  int stage = 0;   // t % kTokStages
  const bool late = PHASED && wave_u >= NW / 2;   // the second wave of each SIMD
  auto bare_barrier = [&]() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  // wait for the tiles requested before the newest request (all, if none was made), and for
  // this wave's LDS traffic
  auto wait_tiles = [&](bool requested) {
    asm volatile("" ::: "memory");
    if (requested) __builtin_amdgcn_s_waitcnt(0x0073);  // vmcnt(3) lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0) lgkmcnt(0)
  };
  if constexpr (PIPE) {
    // One wave per SIMD (d_h = 256: the accumulators and token operands of a wave take 256
    // registers), so nothing hides one wave's arithmetic but its own products: the loop is a
    // software pipeline inside the wave.  Step t = the 48 products M, N, dA of tile t+1, each
    // followed by up to five VALU instructions of the activation arithmetic of tile t (a wave
    // issues one VALU instruction per six cycles or so, a product runs for 32), then the 32 dX
    // products of tile t, between which the 12 direct loads of tile t+2 are issued.  The
    // arithmetic of an element pair is laid over six product slots such that no slot holds
    // more than five instructions and a transcendental result is first used a slot later;
    // 8 pairs x 6 slots = the 48 products.  Accumulators M, N, dA in two sets by parity of the
    // tile.  Three stages: tile t (windows), t+1 (rows), t+2 (in flight); one barrier per step.
    constexpr int NOP = 3 * KS, NT = 2 * JB * 2, kWinP = 4, kWinD = 4;
    static_assert(NOP == 48, "eight element pairs x six slots");
    f32x16 accM[2], accN[2], accA[2];
    u32x4 pmv[2], pnv[2];   // packed dM, dN of the two 16-neuron halves of the tile
    bf16x8 op[NOP];
    s16x4 lo[NT], hi[NT];
    float tt[16], sg[16], silu[16], rda[16], rn[16], om[16], sp[16], ds[16], dnv[16], dmv[16];
    const int li = lane & 15;
    const int trow = 4 * g + (li >> 2), tcol = 16 * ((lane >> 4) & 1) + 4 * (li & 3);
    const unsigned sto0 = lds_addr_of(stage_base);
    // direct loads with a wave-uniform base and a 32-bit lane offset (bytes).  Round i moves
    // rows 8 i + 2 w, + 1: 4096 i bytes further, and the swizzle of a row 8 further differs in
    // one bit of the chunk index.
    const unsigned dma_b0 = 2u * (unsigned)dma_goff[0], dma_b1 = dma_b0 ^ 32u;
    // load n of a request (0..11): round n / 3 of matrix n % 3 (K, U, V)
    auto dma_one = [&](int t, int stage, auto N_) __attribute__((always_inline)) {
      constexpr int i = decltype(N_)::value / 3, which = decltype(N_)::value % 3;
      const size_t base = ((size_t)t * (32 * DH) + i * 8 * DH) * 2;
      const unsigned lane_off = (i & 1) ? dma_b1 : dma_b0;
      unsigned char* dst = stage_base + stage * kTokStageBytes + (NW * i + wave_u) * 1024 + which * kTileBytes;
      const uint16_t* src = which == 0 ? Kh : which == 1 ? Uh : Vh;
      global_to_lds_16B(reinterpret_cast<const unsigned char*>(src) + base + lane_off, dst);
    };

    // slot SL (0..5) of the arithmetic of pair PR (0..7; elements 2 PR and 2 PR + 1 of set R)
    auto pair_slot = [&](auto PR_, auto SL_, auto R_) __attribute__((always_inline)) {
      constexpr int pr = decltype(PR_)::value, sl = decltype(SL_)::value, R = decltype(R_)::value;
      constexpr int v0 = 2 * pr, v1 = 2 * pr + 1, t2 = pr / 4, i = pr % 4;
      if constexpr (sl == 0) {
        tt[v0] = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * accM[R][v0]);
        tt[v1] = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * accM[R][v1]);
        rda[v0] = rw[0] * accA[R][v0];
      } else if constexpr (sl == 1) {
        sg[v0] = __builtin_amdgcn_rcpf(1.0f + tt[v0]);
        sg[v1] = __builtin_amdgcn_rcpf(1.0f + tt[v1]);
        rda[v1] = rw[0] * accA[R][v1];
      } else if constexpr (sl == 2) {
        silu[v0] = accM[R][v0] * sg[v0];
        om[v0] = 1.0f - sg[v0];
        silu[v1] = accM[R][v1] * sg[v1];
        om[v1] = 1.0f - sg[v1];
        rn[v0] = rda[v0] * accN[R][v0];
      } else if constexpr (sl == 3) {
        rn[v1] = rda[v1] * accN[R][v1];
        sp[v0] = fmaf(silu[v0], om[v0], sg[v0]);   // SiLU'(m) = sg + silu (1 - sg)
        sp[v1] = fmaf(silu[v1], om[v1], sg[v1]);
        ds[v0] = accA[R][v0] * silu[v0];
        ds[v1] = accA[R][v1] * silu[v1];
      } else if constexpr (sl == 4) {
        drp[0] = fmaf(ds[v0], accN[R][v0], drp[0]);
        drp[0] = fmaf(ds[v1], accN[R][v1], drp[0]);
        dnv[v0] = rda[v0] * silu[v0];
        dnv[v1] = rda[v1] * silu[v1];
        dmv[v0] = rn[v0] * sp[v0];
      } else {
        dmv[v1] = rn[v1] * sp[v1];
        pmv[t2][i] = pack_bf16(dmv[v0], dmv[v1]);
        pnv[t2][i] = pack_bf16(dnv[v0], dnv[v1]);
      }
    };
    // products of the tile in stage `sto` into set W, arithmetic on set 1 - W in their shadow
    // (REQ_ is a compile-time flag: a branch around a load would split the stream into basic
    // blocks, and the compiler then gathers the arithmetic of all slots in one of them)
    auto row_products = [&](unsigned sto, auto W_, auto ARITH_, auto REQ_, int t_req, int stage_req) __attribute__((always_inline)) {
      constexpr int W = decltype(W_)::value;
      constexpr bool kArith = decltype(ARITH_)::value, kReq = decltype(REQ_)::value;
      // chunk 2 ks + g of a row, swizzled: the address of ks = 0 with bits 5..7 XORed by ks % 8
      // (the stage base is a multiple of 256), 256 bytes further for ks >= 8: one address
      // register instead of sixteen
      const unsigned pb = sto + btile_off<DH>(r, g);
      auto issue = [&](auto C_) __attribute__((always_inline)) {
        constexpr int c = decltype(C_)::value, ks = c / 3, which = c % 3;
        op[c] = lds_read_b128_untracked<which * kTileBytes + (ks >> 3) * 256>(pb ^ ((ks & 7) << 5));
      };
      static_for<0, kWinP>(issue);
      static_for<0, NOP>([&](auto C_) __attribute__((always_inline)) {
        constexpr int c = decltype(C_)::value, ks = c / 3, which = c % 3;
        if constexpr (c + kWinP < NOP) issue(std::integral_constant<int, c + kWinP>{});
        lds_wait<(NOP - 1 - c) < kWinP ? (NOP - 1 - c) : kWinP>(op[c]);
        if constexpr (which == 0) accM[W] = mfma32(op[c], q[0][ks], ks == 0 ? f32x16{0} : accM[W]);
        if constexpr (which == 1) accN[W] = mfma32(op[c], q[0][ks], ks == 0 ? f32x16{0} : accN[W]);
        if constexpr (which == 2) accA[W] = mfma32(op[c], dy[0][ks], ks == 0 ? f32x16{0} : accA[W]);
        // three slots of arithmetic (pieces 0..35: pairs 0..5), then one with a load of the tile
        // after next (a direct load is tracked by vmcnt, the reads above by lgkmcnt)
        if constexpr (c % 4 == 3) {
          if constexpr (kReq) dma_one(t_req, stage_req, std::integral_constant<int, c / 4>{});
        } else if constexpr (kArith) {
          constexpr int piece = c - c / 4;
          pair_slot(std::integral_constant<int, piece / 6>{}, std::integral_constant<int, piece % 6>{},
                    std::integral_constant<int, 1 - W>{});
        }
        MHFFN_SB();
      });
    };
    auto arith_alone = [&](auto R_) __attribute__((always_inline)) {
      static_for<0, 36>([&](auto C_) {
        constexpr int c = decltype(C_)::value;
        pair_slot(std::integral_constant<int, c / 6>{}, std::integral_constant<int, c % 6>{}, R_);
      });
    };
    // dX products of the tile in stage `sto`; the loads of tile t_req go out between them
    auto window_products = [&](unsigned sto, auto R_) __attribute__((always_inline)) {
      // columns 32 jb + tcol of a row: chunk 4 jb + tcol / 8, i.e. the address of jb = 0 with
      // bits 6..7 XORed by jb % 4, 256 bytes further for jb >= 4
      const unsigned wlo = sto + btile_off8<DH>(trow, tcol), whi = sto + btile_off8<DH>(trow + 8, tcol);
      unsigned wl[4], wh[4];   // (the row operands are dead here: eight registers are to be had)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        wl[k] = wlo ^ (k << 6);
        wh[k] = whi ^ (k << 6);
      }
      auto issue2 = [&](auto C_) __attribute__((always_inline)) {
        constexpr int c = decltype(C_)::value, which = c & 1, jb = (c >> 1) % JB, t2 = c / (2 * JB);
        constexpr int OFF = which * kTileBytes + t2 * 16 * 2 * DH + (jb >> 2) * 256;   // 16 rows further: same swizzle
        lo[c] = lds_read_tr16_untracked<OFF>(wl[jb & 3]);
        hi[c] = lds_read_tr16_untracked<OFF>(wh[jb & 3]);
      };
      static_for<0, kWinD>(issue2);
      static_for<0, NT>([&](auto C_) __attribute__((always_inline)) {
        constexpr int c = decltype(C_)::value, which = c & 1, jb = (c >> 1) % JB, t2 = c / (2 * JB);
        if constexpr (c + kWinD < NT) issue2(std::integral_constant<int, c + kWinD>{});
        lds_wait<2 * ((NT - 1 - c) < kWinD ? (NT - 1 - c) : kWinD)>(lo[c], hi[c]);
        const bf16x8 xt = join_tr(lo[c], hi[c]);
        dXa[0][jb] = mfma32(xt, __builtin_bit_cast(bf16x8, which ? pnv[t2] : pmv[t2]), dXa[0][jb]);
        // pieces 36..47 of the arithmetic (pairs 6 and 7, operands of the windows from item 16 on)
        if constexpr (c < 12)
          pair_slot(std::integral_constant<int, (36 + c) / 6>{}, std::integral_constant<int, (36 + c) % 6>{}, R_);
        MHFFN_SB();
      });
    };
    auto step = [&](int t, auto S_) __attribute__((always_inline)) {
      constexpr int S = decltype(S_)::value;
      const int e = t / tiles_per_sub;
      if (t % tiles_per_sub == 0) rw[0] = DRs[e * BM + wtok + r];
      const int st_t = t % 3, st_n = (t + 1) % 3, st_r = (t + 2) % 3;
      if (t + 2 < T) row_products(sto0 + st_n * kTokStageBytes, std::integral_constant<int, 1 - S>{}, std::true_type{}, std::true_type{}, t + 2, st_r);
      else if (t + 1 < T) row_products(sto0 + st_n * kTokStageBytes, std::integral_constant<int, 1 - S>{}, std::true_type{}, std::false_type{}, 0, 0);
      else arith_alone(S_);
      window_products(sto0 + st_t * kTokStageBytes, S_);
      if ((t + 1) % tiles_per_sub == 0) {
        const float dr = drp[0] + __shfl_xor(drp[0], 32);
        if (g == 0) DRs[e * BM + wtok + r] = dr;
        drp[0] = 0.f;
      }
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0): this wave's part of tile t+2 is in
      bare_barrier();
    };
    row_products(sto0, std::integral_constant<int, 0>{}, std::false_type{}, std::false_type{}, 0, 0);
    for (int t = 0; t < T; t += 2) {
      step(t, std::integral_constant<int, 0>{});
      if (t + 1 < T) step(t + 1, std::integral_constant<int, 1>{});
    }
  } else
  if constexpr (PHASED) {
    // Half A of step t: the dX products of tile t-1 (operands packed in half B of step t-1),
    // then the gate/up/dA products of tile t: 40 MFMAs and their LDS reads, no VALU work.
    // Half B: the activation arithmetic, no MFMA.  A SIMD's two waves are always in opposite
    // halves.  Tile t is read in four consecutive half-steps (A of step t and of step t+1, for
    // the early and the late waves); its stage is requested again at the start of the fifth,
    // for tile t+3, by the early waves at the top of their half A and by the late ones at the
    // top of their half B, and each wave waits for its request at the end of its next half,
    // one barrier before the first read.
    f32x16 accM, accN, accA;
    bf16x8 dmf[2], dnf[2];
    // Half A as one stream of LDS reads and MFMAs: items 0 .. NT-1 are the K^T / U^T windows of
    // the previous tile (two transposing reads each, one dX product), items NT .. NT+NOP-1 the
    // K / U / V row operands of this tile (one read, one product each).  Reads run kWin items
    // ahead of their use with counted waits; the first kWin items (all windows of the previous
    // tile, which has been in place for a step) are issued before the barrier that opens the
    // half, so their latency is hidden behind it.
    constexpr int NT = 2 * JB * 2, NOP = 3 * KS, kWin = 4;
    static_assert(kWin <= NT, "the reads issued before the barrier touch the previous tile only");
    s16x4 lo[NT], hi[NT];
    bf16x8 op[NOP];
    const int li = lane & 15;
    const int trow = 4 * g + (li >> 2), tcol = 16 * ((lane >> 4) & 1) + 4 * (li & 3);
    auto issue_item = [&](auto C_, unsigned sto_prev, unsigned sto_cur) {
      constexpr int c = decltype(C_)::value;
      if constexpr (c < NT) {
        constexpr int which = c & 1, jb = (c >> 1) % JB, t2 = c / (2 * JB);
        constexpr int OFF = which * kTileBytes + t2 * 16 * 2 * DH;   // 16 rows further: same swizzle
        lo[c] = lds_read_tr16_untracked<OFF>(sto_prev + btile_off8<DH>(trow, 32 * jb + tcol));
        hi[c] = lds_read_tr16_untracked<OFF>(sto_prev + btile_off8<DH>(trow + 8, 32 * jb + tcol));
      } else {
        constexpr int k = c - NT, ks = k / 3, which = k % 3;
        op[k] = lds_read_b128_untracked<which * kTileBytes>(sto_cur + btile_off<DH>(r, 2 * ks + g));
      }
    };
    // LDS operations issued after those of item c when item c is consumed
    auto pending_after = [](int c, int n_all) {
      int n = 0;
      for (int i = c + 1; i <= c + kWin && i < n_all; ++i) n += (i < NT) ? 2 : 1;
      return n;
    };
    auto prefetch_windows = [&](unsigned sto_prev) {
      static_for<0, kWin>([&](auto C_) { issue_item(C_, sto_prev, 0u); });
    };
    // the stream from item FIRST on (the kWin items from FIRST on have been issued)
    auto run_stream = [&](auto FIRST_, auto NALL_, unsigned sto_prev, unsigned sto_cur) {
      constexpr int FIRST = decltype(FIRST_)::value, NALL = decltype(NALL_)::value;
      static_for<FIRST, NALL>([&](auto C_) {
        constexpr int c = decltype(C_)::value;
        if constexpr (c + kWin < NALL) issue_item(std::integral_constant<int, c + kWin>{}, sto_prev, sto_cur);
        constexpr int pend = pending_after(c, NALL);
        if constexpr (c < NT) {
          constexpr int which = c & 1, jb = (c >> 1) % JB, t2 = c / (2 * JB);
          lds_wait<pend>(lo[c], hi[c]);
          const bf16x8 xt = join_tr(lo[c], hi[c]);
          dXa[0][jb] = mfma32(xt, which ? dnf[t2] : dmf[t2], dXa[0][jb]);
        } else {
          constexpr int k = c - NT, ks = k / 3, which = k % 3;
          lds_wait<pend>(op[k]);
          if constexpr (which == 0) accM = mfma32(op[k], q[0][ks], ks == 0 ? f32x16{0} : accM);
          if constexpr (which == 1) accN = mfma32(op[k], q[0][ks], ks == 0 ? f32x16{0} : accN);
          if constexpr (which == 2) accA = mfma32(op[k], dy[0][ks], ks == 0 ? f32x16{0} : accA);
        }
      });
    };
    using IC0 = std::integral_constant<int, 0>;
    using ICT = std::integral_constant<int, NT>;
    using ICA = std::integral_constant<int, NT + NOP>;
    auto arith = [&]() {
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        u32x4 pm, pn;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float dmv[2], dnv[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int v = 8 * t2 + 2 * i + u;
            const float m = accM[v], n = accN[v], da = accA[v];
            const float sg = sigmoid_fast(m);
            const float silu = m * sg;
            drp[0] = fmaf(da * silu, n, drp[0]);
            const float rda = rw[0] * da;
            dnv[u] = rda * silu;
            dmv[u] = rda * n * fmaf(silu, 1.0f - sg, sg);  // SiLU'(m) = sg + silu (1 - sg)
          }
          pm[i] = pack_bf16(dmv[0], dmv[1]);
          pn[i] = pack_bf16(dnv[0], dnv[1]);
        }
        dmf[t2] = __builtin_bit_cast(bf16x8, pm);
        dnf[t2] = __builtin_bit_cast(bf16x8, pn);
      }
    };
    // end of a half: this wave's LDS traffic (and its tile request, if one is due) has landed;
    // with `windows_of`, the first reads of the next half A go out ahead of the barrier
    auto close_half = [&](bool own_request_due, bool prefetch, unsigned windows_of) {
      asm volatile("" ::: "memory");
      if (own_request_due) __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
      else __builtin_amdgcn_s_waitcnt(0xC07F);                   // lgkmcnt(0)
      if (prefetch) prefetch_windows(windows_of);
      bare_barrier();
    };
    // A request is made by the early waves alone, at the top of their half A (the shorter of
    // the two halves): wave w moves its own rows and those of wave w + NW/2.
    auto dma_pair = [&](int t, int stage) {
      const size_t off = (size_t)t * (32 * DH) + dma_goff[0];
      unsigned char* dst = stage_base + stage * kTokStageBytes + wave_u * 1024;
      constexpr int kHalfTile = (NW / 2) * 4 * DH;   // elements: rows 4 (w + NW/2) .. +3
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        global_to_lds_16B(Kh + off + hf * kHalfTile, dst + hf * (kTileBytes / 2));
        global_to_lds_16B(Uh + off + hf * kHalfTile, dst + hf * (kTileBytes / 2) + kTileBytes);
        global_to_lds_16B(Vh + off + hf * kHalfTile, dst + hf * (kTileBytes / 2) + 2 * kTileBytes);
      }
    };
    const unsigned sto0 = lds_addr_of(stage_base);
    int prev = 2;   // (t - 1) % 3
    if (late) bare_barrier();
    // (the first step, which has no previous tile, is a copy of its own: as a branch inside the
    // loop it can cost the loop sixty spilled registers)
    auto step = [&](int t, auto FIRST_) {
      constexpr bool kFirst = decltype(FIRST_)::value;
      const int e = t / tiles_per_sub;
      if (t % tiles_per_sub == 0) rw[0] = DRs[e * BM + wtok + r];
      const unsigned sto_cur = sto0 + stage * kTokStageBytes, sto_prev = sto0 + prev * kTokStageBytes;
      // ---- half A
      const bool request = !late && t >= 1 && t + 1 < T;
      if (request) dma_pair(t + 1, stage == 2 ? 0 : stage + 1);
      if constexpr (kFirst) {
        static_for<NT, NT + kWin>([&](auto C_) { issue_item(C_, 0u, sto_cur); });
        run_stream(ICT{}, ICA{}, 0u, sto_cur);
      } else {
        run_stream(IC0{}, ICA{}, sto_prev, sto_cur);
      }
      close_half(false, false, 0u);
      // ---- half B
      __builtin_amdgcn_s_setprio(1);
      arith();
      // (left alone, the compiler sinks half of the arithmetic below the wait that closes the half)
      asm volatile("" : "+v"(dmf[0]), "+v"(dmf[1]), "+v"(dnf[0]), "+v"(dnf[1]), "+v"(drp[0]));
      __builtin_amdgcn_s_setprio(0);
      if ((t + 1) % tiles_per_sub == 0) {
        const float dr = drp[0] + __shfl_xor(drp[0], 32);
        if (g == 0) DRs[e * BM + wtok + r] = dr;
        drp[0] = 0.f;
      }
      close_half(!late, true, sto_cur);
      prev = stage;
      stage = (stage == 2) ? 0 : stage + 1;
    };
    step(0, std::true_type{});
    for (int t = 1; t < T; ++t) step(t, std::false_type{});
    run_stream(IC0{}, ICT{}, sto0 + prev * kTokStageBytes, 0u);
    close_half(false, false, 0u);
    if (!late) bare_barrier();
  } else {
  if (late) bare_barrier();
  for (int t = 0; t < T; ++t) {
    const bool more = (t + 1 < T);
    const bool ahead = DMA && (t + 2 < T);
    const int e = t / tiles_per_sub;
    // The gating weight of sub-network e waits in LDS, in the slot that takes dr_e once the
    // sub-network has been swept (a load from the workspace here would have to stay in flight
    // across the loop's back edge, where the compiler waits for every load, tile requests
    // included).
    if (t % tiles_per_sub == 0) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) rw[tb] = DRs[e * BM + wtok + 32 * tb + r];
    }
    if constexpr (DMA) {
      // the stage that step t-1 retired (for the late waves; the early ones wait half a step)
      if (ahead && (!PHASED || late)) dma(t + 2, stage == 0 ? 2 : stage - 1);
    } else {
      if (more) gload(t + 1);
    }
    const unsigned char* st = stage_base + stage * kTokStageBytes;

    __builtin_amdgcn_s_setprio(1);
    f32x16 accM[TB], accN[TB], accA[TB];   // started by their first product (C operand 0)
    // K/U/V row operands, item c = 3 ks + {0: K, 1: U, 2: V}: each is read six items (two
    // contraction steps) ahead of its use, with counted waits.  Left to the compiler, each
    // step's three reads are issued and waited for back to back, and every step pays the
    // full LDS latency.
    {
      const unsigned sto = lds_addr_of(st);
      constexpr int NOP = 3 * KS;
      bf16x8 op[NOP];
      auto issue = [&](auto C_) {
        constexpr int c = decltype(C_)::value, ks = c / 3, which = c % 3;
        op[c] = lds_read_b128_untracked<which * kTileBytes>(sto + btile_off<DH>(r, 2 * ks + g));
      };
      static_for<0, 6>(issue);
      static_for<0, NOP>([&](auto C_) {
        constexpr int c = decltype(C_)::value, ks = c / 3, which = c % 3;
        if constexpr (c + 6 < NOP) issue(std::integral_constant<int, c + 6>{});
        lds_wait<(NOP - 1 - c) < 6 ? (NOP - 1 - c) : 6>(op[c]);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          if constexpr (which == 0) accM[tb] = mfma32(op[c], q[tb][ks], ks == 0 ? f32x16{0} : accM[tb]);
          if constexpr (which == 1) accN[tb] = mfma32(op[c], q[tb][ks], ks == 0 ? f32x16{0} : accN[tb]);
          if constexpr (which == 2) accA[tb] = mfma32(op[c], dy[tb][ks], ks == 0 ? f32x16{0} : accA[tb]);
        }
      });
    }
    if constexpr (PHASED) {
      if (late) wait_tiles(ahead);
      else __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this half's operand reads
      bare_barrier();
      if (ahead && !late) dma(t + 2, stage == 0 ? 2 : stage - 1);
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
    __builtin_amdgcn_s_setprio(0);
    // K^T / U^T operands, item c = (t2, jb, which): transposing reads issued four items ahead
    // of their use with counted waits, like the row operands above
    {
      const unsigned sto = lds_addr_of(st);
      constexpr int NI = 2 * JB * 2, W2 = 4;
      s16x4 lo[NI], hi[NI];
      const int li = lane & 15;
      const int trow = 4 * g + (li >> 2), tcol = 16 * ((lane >> 4) & 1) + 4 * (li & 3);
      auto issue2 = [&](auto C_) {
        constexpr int c = decltype(C_)::value, which = c & 1, jb = (c >> 1) % JB, t2 = c / (2 * JB);
        constexpr int OFF = which * kTileBytes + t2 * 16 * 2 * DH;   // 16 rows further: same swizzle
        lo[c] = lds_read_tr16_untracked<OFF>(sto + btile_off8<DH>(trow, 32 * jb + tcol));
        hi[c] = lds_read_tr16_untracked<OFF>(sto + btile_off8<DH>(trow + 8, 32 * jb + tcol));
      };
      static_for<0, W2>(issue2);
      static_for<0, NI>([&](auto C_) {
        constexpr int c = decltype(C_)::value, which = c & 1, jb = (c >> 1) % JB, t2 = c / (2 * JB);
        if constexpr (c + W2 < NI) issue2(std::integral_constant<int, c + W2>{});
        lds_wait<2 * ((NI - 1 - c) < W2 ? (NI - 1 - c) : W2)>(lo[c], hi[c]);
        const bf16x8 xt = join_tr(lo[c], hi[c]);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
          dXa[tb][jb] = mfma32(xt, which ? dnf[tb][t2] : dmf[tb][t2], dXa[tb][jb]);
      });
    }
    if ((t + 1) % tiles_per_sub == 0) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        const float dr = drp[tb] + __shfl_xor(drp[tb], 32);
        if (g == 0) DRs[e * BM + wtok + 32 * tb + r] = dr;
        drp[tb] = 0.f;
      }
    }
    stage = (stage + 1 == kTokStages) ? 0 : stage + 1;
    if constexpr (DMA) {
      // Publish tile t+1 (requested one step ago; the three loads issued in this step may stay
      // in flight) and retire this step's stage.  A bare barrier: __syncthreads() would wait
      // for every load in flight.
      if (PHASED && late) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
      } else {
        wait_tiles(ahead);
      }
      bare_barrier();
    } else {
      if (more) lstore(stage);
      __syncthreads();
    }
  }
  if (PHASED && !late) bare_barrier();
  }

  // ---- derivative through the gating weights ------------------------------------
  if (a.route_mode == 0) {
    // stage W_r[h] as rows j, columns e (zero padded to 32*EB), for the A operand
    const int EB = (E + 31) >> 5;
    const int wr_stride = 64 * EB + 16;  // bytes per row; +16 keeps rows off the same banks
    const uint16_t* Wr = reinterpret_cast<const uint16_t*>(a.route) + (size_t)h * DH * E;
    for (int idx = tid; idx < DH * 32 * EB; idx += THREADS) {
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
        for (int jb = 0; jb < JB; ++jb) {
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
        uint16_t* dst = a.dX + tok[tb] * a.ldx + h * DH + 4 * g;
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
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
// weight-major kernel, 16 neurons per wave (two waves per SIMD)
//
// One wave owns 16 neurons of one head: their K/U/V rows are resident as B
// operands of v_mfma_f32_16x16x32_bf16 (48 VGPR) and the accumulators dK^T, dU^T,
// dV^T take 96 VGPR, so a wave fits in 256 registers and two waves share a SIMD
// (the fp32 VALU issues at twice the rate when it can alternate between two
// waves, and one wave's arithmetic hides behind the other's MFMAs).
// Eight waves share the q / dY token tiles, which go global -> LDS directly in
// four stages, requested two steps ahead.  Per 32 tokens and wave:
//   M, N [32 tok][16]  = q K^T, q U^T          16 MFMA   (A: q rows from LDS)
//   dA   [32 tok][16]  = dY V^T                  8 MFMA
//   a, dn, dm                                     fp32 VALU, 8 elements per lane
//   dV^T[j][c] += dY^T a; dK^T += q^T dm; dU^T += q^T dn   24 MFMA (A: transposing reads)
// LDS layout of the q / dY tiles here: rows of 256 bytes whose 16-byte chunks are permuted
// by w16_swz(row) = 2 (row % 8).  Two kinds of reads hit a tile, and the hardware serves
// them in different lane groups: a 16-byte row read in the four groups {0-3, 12-15, 20-23,
// 24-27}, {4-7, 8-11, 16-19, 28-31} (and the same + 32), a transposing 8-byte read in
// lanes 0-31 and 32-63.  With this permutation the 16 lanes of a row-read group (eight token
// rows of one column group, eight of the other) land on 16 different chunks, and the eight
// token rows that one half of a transposing read touches (32 bytes each) on eight different
// chunk pairs: both are free of bank conflicts (measured 4.2 and 2.1 cycles per read; with
// the general tile swizzle of the other kernels the transposing reads of this lane geometry
// took 4.0).  All LDS reads are issued untracked with explicit waits.
// Rows past N are read from row N-1 (finite data) and get r = 0 in the last block,
// so they add nothing to any gradient.
// ---------------------------------------------------------------------------
constexpr int kW16Waves = 8;
constexpr int kW16Threads = 64 * kW16Waves;
// LDS: one ring per tensor, so that every operand address is a 16-bit immediate offset
// from a per-lane register: q tiles | dY tiles | r (64 floats per wave, 32 used)
constexpr int kW16RSlot = kW16Waves * 64 * 4;
constexpr int kW16Stages = 4;
constexpr int kW16YRing = kW16Stages * kTileBytes;        // start of the dY ring
constexpr int kW16RRing = 2 * kW16Stages * kTileBytes;    // start of the r ring
constexpr int kW16LdsBytes = kW16RRing + kW16Stages * kW16RSlot;
static_assert(kW16YRing + (kW16Stages - 1) * kTileBytes + 4096 < 65536, "LDS read offsets are 16-bit");
constexpr int kW16Window = 6;   // operands kept in flight ahead of the one being consumed
// LDS read instructions behind issue position p of a step's operand stream (see the kernel)
constexpr int w16_instrs(int p) { return (p >= 12 && p < 28) ? 2 : 1; }
// last position that has been issued when item c is consumed (item c sits at position c - 4)
constexpr int w16_issued_before(int c) { return c - 4 + kW16Window > 33 ? 33 : c - 4 + kW16Window; }
// read instructions issued after item c when it is consumed
constexpr int w16_pending(int c) {
  int n = 0;
  for (int p = c - 4 + 1; p <= w16_issued_before(c); ++p) n += w16_instrs(p);
  return n;
}


__global__ __launch_bounds__(kW16Threads) void bwd_wgt16_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cn = lane & 15, gq = lane >> 4;
  // this kernel's tile layout (see above): byte offset of 16-byte chunk `chunk` of `row`,
  // and of the 8-byte piece that starts at bf16 column `col`
  auto w16_swz = [](int row) { return (row & 7) << 1; };
  auto w16_off = [&](int row, int chunk) { return row * 256 + ((chunk ^ w16_swz(row)) << 4); };
  auto w16_off8 = [&](int row, int col) { return w16_off(row, col >> 3) + ((col & 4) << 1); };
  const int nblk = a.E * a.de / 16;              // 16-neuron blocks per head
  const int wg_per_head = (nblk + kW16Waves - 1) / kW16Waves;
  // Workgroups go to the XCDs round robin by blockIdx and are started in that order: XCD x
  // takes neuron groups x gpx .. (x+1) gpx - 1 (so that its workgroups stream the same
  // heads' token tiles through its L2), first the groups that take all tokens, one workgroup
  // each, then, `wsplit` workgroups each, the groups of the last round, which would leave
  // CUs idle if every group were one workgroup (704 groups on 256 CUs: 2.75 rounds).
  const int xcd = blockIdx.x & 7, widx = blockIdx.x >> 3;
  const int g_first = xcd * a.gpx;
  const int n_here = min(a.n_groups - g_first, a.gpx);       // groups of this XCD
  const int n_full = min(a.full_px, n_here);
  int group, seg = 0, cgroup = 0;
  bool split = false;
  if (widx < n_full) {
    group = g_first + widx;
  } else {
    const int j = widx - n_full, lt = j / a.wsplit;
    if (n_full + lt >= n_here) return;   // whole workgroup leaves together
    group = g_first + n_full + lt;
    seg = j - lt * a.wsplit;
    split = a.wsplit > 1;
    cgroup = xcd * (a.gpx - a.full_px) + lt;
  }
  const int h = group / wg_per_head;
  const int blk = (group % wg_per_head) * kW16Waves + wave;
  const bool active = blk < nblk;
  const int blk_c = active ? blk : nblk - 1;     // idle waves shadow a valid block, store nothing
  const int64_t N = a.N;
  const size_t row0 = ((size_t)h * nblk + blk_c) * 16;   // first neuron row of this wave
  const int e_wave = blk_c / (a.de / 16);

  // resident weight operands: lane (neuron cn, group gq) holds columns 32ks + 8gq ..
  bf16x8 Kf[4], Uf[4], Vf[4];
  {
    const size_t off = (row0 + cn) * kDh + 8 * gq;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      Kf[ks] = *reinterpret_cast<const bf16x8*>(a.Wg + off + 32 * ks);
      Uf[ks] = *reinterpret_cast<const bf16x8*>(a.Wu + off + 32 * ks);
      Vf[ks] = *reinterpret_cast<const bf16x8*>(a.Wd + off + 32 * ks);
    }
  }
  f32x4 dK[8], dU[8], dV[8];
#pragma unroll
  for (int jb = 0; jb < 8; ++jb) { dK[jb] = f32x4{0, 0, 0, 0}; dU[jb] = dK[jb]; dV[jb] = dK[jb]; }

  // ---- staging -----------------------------------------------------------------
  // wave w moves rows 4w..4w+3 of the q and dY tiles (one 1 KB swizzled image each)
  // and the 32 r values of its own sub-network.
  const int drow = 4 * wave + (lane >> 4);
  const int dcol = h * kDh + (((lane & 15) ^ w16_swz(drow)) << 3);   // element column in X / dY
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const float* Rw = a.Rws + ((size_t)h * a.E + e_wave) * N;
  // (three loads per wave and block; the r load is a full wave wide, its upper half
  // repeats the lower one into the unused half of the wave's slot)
  // Blocks are requested in order, each once: the per-lane source pointers just advance.
  const int64_t nb = (N + 31) / 32;                       // all blocks of 32 tokens
  const int64_t b0 = split ? seg * a.blocks_per_seg : 0;  // this workgroup's blocks: b0 .. b1-1
  const int64_t b1 = (split && b0 + a.blocks_per_seg < nb) ? b0 + a.blocks_per_seg : nb;
  const int rrow = lane & 31;   // r of the block's tokens in order (the upper half-wave repeats it)
  const uint16_t* xsrc = a.X + (b0 * 32 + drow) * a.ldx + dcol;
  const uint16_t* ysrc = a.dY + (b0 * 32 + drow) * a.ldy + dcol;
  const float* rsrc = Rw + b0 * 32 + rrow;
  auto dma = [&](int64_t blkidx, int stage) {
    const uint16_t* xs = xsrc;
    const uint16_t* ys = ysrc;
    const float* rs = rsrc;
    if (blkidx == nb - 1) {   // the last block may be ragged: rows past N read row N-1
      int64_t t = blkidx * 32 + drow, tr = blkidx * 32 + rrow;
      t = t < N ? t : N - 1;
      tr = tr < N ? tr : N - 1;
      xs = a.X + t * a.ldx + dcol;
      ys = a.dY + t * a.ldy + dcol;
      rs = Rw + tr;
    }
    unsigned char* dst = smem + stage * kTileBytes + wave_u * 1024;
    global_to_lds_16B(xs, dst);
    global_to_lds_16B(ys, dst + kW16YRing);
    __builtin_amdgcn_global_load_lds(
        (__attribute__((address_space(1))) const void*)rs,
        (__attribute__((address_space(3))) void*)(smem + kW16RRing + stage * kW16RSlot + wave_u * 256),
        4, 0, 0);
    xsrc += 32 * a.ldx;
    ysrc += 32 * a.ldy;
    rsrc += 32;
  };
  dma(b0, 0);
  if (b0 + 1 < b1) dma(b0 + 1, 1);
  if (b0 + 2 < b1) dma(b0 + 2, 2);
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
  __syncthreads();

  // ---- loop-invariant LDS addresses -----------------------------------------------
  const unsigned lbase = lds_addr_of(smem);
  unsigned qaddr[4];   // A operand of M/N/dA: token row cn, 16-byte chunk 4ks + gq
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qaddr[ks] = lbase + w16_off(cn, 4 * ks + gq);
  unsigned taddr[8];   // transposed operand: token rows 4gq + cn/4 (+16), columns 16jb + 4(cn%4)
#pragma unroll
  for (int jb = 0; jb < 8; ++jb)
    taddr[jb] = lbase + w16_off8(4 * gq + (cn >> 2), 16 * jb + 4 * (cn & 3));
  const unsigned raddr = lbase + kW16RRing + wave * 256 + 16 * gq;  // r of MFMA rows 4gq.. (+64: next 16 tokens)

  // Operand stream of one step, in issue order (position p):
  //   0..3   Q4..Q7   q rows, tokens 16..31, contraction steps 0..3        (1 LDS read each)
  //   4..11  Y0..Y7   dY rows                                              (1)
  //   12..27 X0..X15  transposed windows: dY^T 0, q^T 0, dY^T 1, q^T 1 ..  (2)
  //   28,29  R', 30..33 Q0'..Q3': r and the first q rows of the NEXT block (1)
  // and in consumption order (item c): Q0..Q7, Y0..Y7, X0..X15; Q0..Q3 and r were
  // read by the previous step.  Before item c is consumed everything up to kW16Window
  // positions ahead of it has been issued, and the wait names exactly the number of
  // reads issued after it.
  bf16x8 opc[4];   // Q0..Q3 of the current block
  f32x4 rvc[2];    // r of this lane's tokens, current block
  asm volatile("ds_read_b128 %0, %1" : "=v"(rvc[0]) : "v"(raddr));
  asm volatile("ds_read_b128 %0, %1 offset:64" : "=v"(rvc[1]) : "v"(raddr));
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) opc[ks] = lds_read_b128_untracked<0>(qaddr[ks]);

  auto step = [&](int64_t b, auto S_) {
    constexpr int S = decltype(S_)::value;
    constexpr int SN1 = (S + 1) % kW16Stages;               // next block's stage
    constexpr int SO = S * kTileBytes, SN = SN1 * kTileBytes;   // tile offsets inside a ring
    const bool more2 = (b + 2 < b1), more3 = (b + 3 < b1);
    if (b == nb - 1) {   // rows past N were read from row N-1: give them r = 0
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (b * 32 + 16 * tb + 4 * gq + v >= N) rvc[tb][v] = 0.f;
    }

    bf16x8 op[16], opn[4];
    f32x4 rvn[2];
    s16x4 xlo[16], xhi[16];
    auto issue = [&](auto P_) {
      constexpr int P = decltype(P_)::value;
      if constexpr (P < 4) {
        op[4 + P] = lds_read_b128_untracked<SO + 4096>(qaddr[P]);
      } else if constexpr (P < 12) {
        op[4 + P] = lds_read_b128_untracked<kW16YRing + SO + ((P - 4) >> 2) * 4096>(qaddr[(P - 4) & 3]);
      } else if constexpr (P < 28) {
        constexpr int J = P - 12, TO = SO + ((J & 1) ? 0 : kW16YRing);
        xlo[J] = lds_read_tr16_untracked<TO>(taddr[J >> 1]);
        xhi[J] = lds_read_tr16_untracked<TO + 4096>(taddr[J >> 1]);
      } else if constexpr (P == 28) {
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(rvn[0]) : "v"(raddr), "n"(SN1 * kW16RSlot));
      } else if constexpr (P == 29) {
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(rvn[1]) : "v"(raddr), "n"(SN1 * kW16RSlot + 64));
      } else {
        opn[P - 30] = lds_read_b128_untracked<SN>(qaddr[P - 30]);
      }
    };
    // issue what item C needs to have in flight, beyond what item C-1 already required
    auto advance = [&](auto C_) {
      constexpr int C = decltype(C_)::value;
      constexpr int lo = (C == 0) ? 0 : w16_issued_before(C - 1) + 1;
      static_for<lo, w16_issued_before(C) + 1>(issue);
    };

    __builtin_amdgcn_s_setprio(1);
    f32x4 M[2], Nn[2], Ad[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) { M[tb] = f32x4{0, 0, 0, 0}; Nn[tb] = M[tb]; Ad[tb] = M[tb]; }
    // gate / up products
    static_for<0, 8>([&](auto C_) {
      constexpr int C = decltype(C_)::value;
      advance(C_);
      bf16x8& o = (C < 4) ? opc[C & 3] : op[C];
      lds_wait<w16_pending(C)>(o);
      M[C >> 2] = mfma16(o, Kf[C & 3], M[C >> 2]);
      Nn[C >> 2] = mfma16(o, Uf[C & 3], Nn[C >> 2]);
    });
    // dA products, with everything that needs only m, n, r computed under them
    float Pw[8], Qw[8];   // r silu(m)  and  r n silu'(m)
    float Aw[8];          // r silu(m) n
    static_for<8, 16>([&](auto C_) {
      constexpr int C = decltype(C_)::value, I = C - 8, TB = I >> 2, V = I & 3;
      advance(C_);
      lds_wait<w16_pending(C)>(op[C]);
      Ad[TB] = mfma16(op[C], Vf[I & 3], Ad[TB]);
      const float rwv = rvc[TB][V];
      const float m = M[TB][V], n = Nn[TB][V];
      const float t = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * m);
      const float sg = __builtin_amdgcn_rcpf(1.0f + t);
      const float sw = rwv * sg;
      const float x = (1.0f + m) - m * sg;   // silu'(m) = sg (1 + m - silu(m))
      Pw[I] = m * sw;
      Qw[I] = (n * sw) * x;
      Aw[I] = Pw[I] * n;
    });
    // k-slot s = 4tb + v of every gradient product is token 16tb + 4gq + v
    u32x4 pa, pm, pn;
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) {
      const int s0 = 2 * s2, s1 = 2 * s2 + 1;
      const float d0 = Ad[s0 >> 2][s0 & 3], d1 = Ad[s1 >> 2][s1 & 3];
      pa[s2] = pack_bf16(Aw[s0], Aw[s1]);
      pn[s2] = pack_bf16(Pw[s0] * d0, Pw[s1] * d1);
      pm[s2] = pack_bf16(Qw[s0] * d0, Qw[s1] * d1);
    }
    const bf16x8 agf = __builtin_bit_cast(bf16x8, pa);
    const bf16x8 dmf = __builtin_bit_cast(bf16x8, pm), dnf = __builtin_bit_cast(bf16x8, pn);

    // Barrier: the next block's tiles (requested two steps ago) and r have landed for every
    // wave, and every wave is done with the previous block's stage, which the request below
    // overwrites.  Bare barrier, no LDS wait: transposed operands are already in flight.
    asm volatile("" ::: "memory");
    if (more2) __builtin_amdgcn_s_waitcnt(0x0F73);  // vmcnt(3): only the newest request may be pending
    else __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (more3) dma(b + 3, (S + 3) % kW16Stages);
    __builtin_amdgcn_s_setprio(0);

    // dV^T[j][c] += dY^T a ; dK^T[j][c] += q^T dM ; dU^T[j][c] += q^T dN  (contraction over tokens)
    static_for<16, 32>([&](auto C_) {
      constexpr int C = decltype(C_)::value, J = C - 16, JB = J >> 1;
      advance(C_);
      lds_wait<w16_pending(C)>(xlo[J], xhi[J]);
      const bf16x8 xt = join_tr(xlo[J], xhi[J]);
      if constexpr ((J & 1) == 0) {
        dV[JB] = mfma16(xt, agf, dV[JB]);
      } else {
        dK[JB] = mfma16(xt, dmf, dK[JB]);
        dU[JB] = mfma16(xt, dnf, dU[JB]);
      }
    });
    // the reads of the next block's first operands are in flight; hand them over
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) opc[ks] = opn[ks];
    rvc[0] = rvn[0];
    rvc[1] = rvn[1];
    // second barrier of the step: keeps the two halves of the workgroup half a step apart
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  using C2 = std::integral_constant<int, 2>;
  using C3 = std::integral_constant<int, 3>;
  // Waves w and w + 4 share a SIMD.  Waves 4-7 pass one barrier more before the loop and waves
  // 0-3 one more after it, so that a SIMD always has one wave in the first half of a step
  // (recompute products and the arithmetic) and one in the second (gradient products): the
  // arithmetic of one runs beside the products of the other.  The stage a request overwrites
  // was last read two barriers before the request by either half.
  if (wave >= 4) __builtin_amdgcn_s_barrier();
  for (int64_t b = b0; b < b1; b += 4) {
    step(b, C0{});
    if (b + 1 < b1) step(b + 1, C1{});
    if (b + 2 < b1) step(b + 2, C2{});
    if (b + 3 < b1) step(b + 3, C3{});
  }
  if (wave < 4) __builtin_amdgcn_s_barrier();
  // drain the reads issued for a block that does not exist
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(opc[0]), "+v"(opc[1]), "+v"(opc[2]), "+v"(opc[3]),
                                        "+v"(rvc[0]), "+v"(rvc[1]));

  if (active && split) {
    // fp32 partial gradients of this token segment: [seg][K | U | V][split group][wave][16][128]
    const size_t rows = (size_t)8 * (a.gpx - a.full_px) * (kW16Waves * 16);
    float* dst = a.WPws + (((size_t)seg * 3) * rows + ((size_t)cgroup * kW16Waves + wave) * 16 + cn) * kDh + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) {
      *reinterpret_cast<f32x4*>(dst + 16 * jb) = dK[jb];
      *reinterpret_cast<f32x4*>(dst + rows * kDh + 16 * jb) = dU[jb];
      *reinterpret_cast<f32x4*>(dst + 2 * rows * kDh + 16 * jb) = dV[jb];
    }
  } else if (active) {
    // accumulators are [j][c]: lane = neuron column cn, register v = row 16jb + 4gq + v
    const size_t off = (row0 + cn) * kDh + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) {
      const size_t o = off + 16 * jb;
      if (a.dWg) {
        u32x2 pk = {pack_bf16(dK[jb][0], dK[jb][1]), pack_bf16(dK[jb][2], dK[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWg + o) = pk;
      }
      if (a.dWu) {
        u32x2 pk = {pack_bf16(dU[jb][0], dU[jb][1]), pack_bf16(dU[jb][2], dU[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWu + o) = pk;
      }
      if (a.dWd) {
        u32x2 pk = {pack_bf16(dV[jb][0], dV[jb][1]), pack_bf16(dV[jb][2], dV[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWd + o) = pk;
      }
    }
  }
}

// bwd_wgt256_kernel (d_h = 256, further down): a workgroup takes four blocks of 16 neurons
constexpr int kW2Dh = 256;
constexpr int kW2Blocks = 4;

// dW[i] = bf16(sum_seg partial[seg][which][i]) for which = K, U, V; fixed order
__global__ void bwd_wgt_reduce_kernel(BwdArgs a, size_t count) {
  const size_t idx = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (idx >= count) return;
  uint16_t* outs[3] = {a.dWg, a.dWu, a.dWd};
#pragma unroll
  for (int which = 0; which < 3; ++which) {
    if (!outs[which]) continue;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int sgm = 0; sgm < a.wsplit; ++sgm)
      sum += *reinterpret_cast<const f32x4*>(a.WPws + ((size_t)sgm * 3 + which) * count + idx);
    u32x2 pk = {pack_bf16(sum[0], sum[1]), pack_bf16(sum[2], sum[3])};
    *reinterpret_cast<u32x2*>(outs[which] + idx) = pk;
  }
}

// The same for bwd_wgt16_kernel and bwd_wgt256_kernel, whose partials cover only the neuron
// groups that share their tokens out: thread = 4 columns of one row of those groups.
__global__ void bwd_wgt16_reduce_kernel(BwdArgs a, size_t crows) {
  const int dh = a.dh, per_group = (dh == kW2Dh) ? kW2Blocks : kW16Waves;   // 16-neuron blocks per group
  const size_t idx = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (idx >= crows * dh) return;
  const size_t crow = idx / dh;
  const int col = (int)(idx % dh);
  const int cgroup = (int)(crow / (per_group * 16)), wv = (int)(crow / 16) % per_group, cn = (int)(crow % 16);
  const int per = a.gpx - a.full_px;
  const int xcd = cgroup / per, lt = cgroup % per;
  const int g_first = xcd * a.gpx;
  const int n_here = min(a.n_groups - g_first, a.gpx);
  const int n_full = min(a.full_px, n_here);
  if (n_full + lt >= n_here) return;
  const int group = g_first + n_full + lt;
  const int nblk = a.E * a.de / 16;
  const int wg_per_head = (nblk + per_group - 1) / per_group;
  const int h = group / wg_per_head, blk = (group % wg_per_head) * per_group + wv;
  if (blk >= nblk) return;
  const size_t o = (((size_t)h * nblk + blk) * 16 + cn) * dh + col;
  uint16_t* outs[3] = {a.dWg, a.dWu, a.dWd};
#pragma unroll
  for (int which = 0; which < 3; ++which) {
    if (!outs[which]) continue;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int sgm = 0; sgm < a.wsplit; ++sgm)
      sum += *reinterpret_cast<const f32x4*>(a.WPws + ((size_t)sgm * 3 + which) * crows * dh + idx);
    u32x2 pk = {pack_bf16(sum[0], sum[1]), pack_bf16(sum[2], sum[3])};
    *reinterpret_cast<u32x2*>(outs[which] + o) = pk;
  }
}

// Tokens are shared out only when that shortens the kernel by a fifth or more: its time goes in
// rounds of 256 workgroups (one per CU), so S segments cost ceil(groups * S / 256) / S rounds.
struct WgtSplit { int segs; int64_t blocks_per_seg; };
// waves per workgroup and workgroups the chip holds at once, per head width
constexpr int wgt_waves(int dh) { return dh == kDh ? kW16Waves : 4; }
constexpr int wgt_slots(int dh) { return dh == 64 ? 768 : 256; }
WgtSplit plan_wgt_split(const Problem& p) {
  const int64_t nb = (p.N + 31) / 32;
  const int waves = wgt_waves(p.dh), slots = wgt_slots(p.dh);
  const int64_t groups = (int64_t)p.H * (((int64_t)p.E * p.de / 16 + waves - 1) / waves);
  auto rounds = [&](int64_t S) { return (double)((groups * S + slots - 1) / slots) / (double)S; };
  int best = 1;
  for (int S = 2; S <= 8; ++S)
    if (nb / S >= 16 && rounds(S) < 0.9 * rounds(best)) best = S;   // more segments only for a clear gain
  if (rounds(best) > 0.8 * rounds(1)) best = 1;
  WgtSplit w;
  w.blocks_per_seg = (nb + best - 1) / best;
  w.segs = (int)((nb + w.blocks_per_seg - 1) / w.blocks_per_seg);
  if (w.segs < 1) { w.segs = 1; w.blocks_per_seg = nb > 0 ? nb : 1; }
  return w;
}
// d_h = 128: the groups of an XCD's share that fill whole rounds of its 32 CUs take all tokens;
// the groups of the last, partly filled round share the tokens out over S workgroups each
// when that pays: the round then takes ceil(tail S / 32) / S of a round instead of one, and
// only those groups leave partials (1.3B shape: 88 groups per XCD = 64 + 24, S = 4: 2.75 rounds
// instead of 3; 370M shape: 22 groups, S = 4: 0.75 instead of 1).
struct Wgt16Plan { int n_groups, gpx, full_px, segs; int64_t blocks_per_seg; size_t crows; };
Wgt16Plan plan_wgt16(const Problem& p) {
  Wgt16Plan w;
  const int64_t nb = (p.N + 31) / 32;
  const int nblk = p.E * p.de / 16;
  const int per_group = (p.dh == kW2Dh) ? kW2Blocks : kW16Waves;   // 16-neuron blocks per workgroup
  w.n_groups = p.H * ((nblk + per_group - 1) / per_group);
  w.gpx = (w.n_groups + 7) / 8;
  w.full_px = w.gpx;
  w.segs = 1;
  w.blocks_per_seg = nb > 0 ? nb : 1;
  w.crows = 0;
  constexpr int slots = 32;                       // CUs of an XCD, one workgroup each
  const int full = (w.gpx / slots) * slots, tail = w.gpx - full;
  if (tail == 0) return w;
  // a round walks nb blocks of 32 tokens at about 1.4 us each; partials (196608 bytes per
  // workgroup) are written and read once more, at about 4 TB/s, plus one more launch
  const double round_us = 1.4 * (double)nb;
  double best_net = 0.02 * round_us * (double)((w.gpx + slots - 1) / slots);   // at least 2 % of the kernel
  for (int S = 2; S <= 8; ++S) {
    if (nb / S < 16) break;
    const double r = (double)((tail * S + slots - 1) / slots) / (double)S;
    const double net = (1.0 - r) * round_us - (8.0 * tail * S * 196608.0 * 2.0 / 4e6 + 10.0);
    if (net > best_net) { best_net = net; w.segs = S; }
  }
  if (w.segs > 1) {
    w.full_px = full;
    w.blocks_per_seg = (nb + w.segs - 1) / w.segs;
    w.segs = (int)((nb + w.blocks_per_seg - 1) / w.blocks_per_seg);
    w.crows = (size_t)8 * tail * (per_group * 16);
  }
  return w;
}

// bwd_wgt256_kernel addresses a block's rows with 32-bit byte offsets
bool wgt256_takes(const Problem& p) {
  return p.dh == kW2Dh && p.ldx < ((int64_t)1 << 24) && p.ldy < ((int64_t)1 << 24);
}

size_t wgt_split_bytes(const Problem& p) {
  if (p.N == 0) return 0;
  if (p.dh == kDh || wgt256_takes(p)) {
    const Wgt16Plan w16 = plan_wgt16(p);
    return w16.segs > 1 ? (size_t)w16.segs * 3 * w16.crows * p.dh * sizeof(float) : 0;
  }
  const WgtSplit w = plan_wgt_split(p);
  return w.segs > 1 ? (size_t)w.segs * 3 * p.H * p.E * p.de * p.dh * sizeof(float) : 0;
}

// ---------------------------------------------------------------------------
// weight-major kernel for the other head widths (d_h = 64, 256)
//
// Same decomposition as bwd_wgt16_kernel (one wave = 16 neurons, K/U/V rows resident as
// operands of the 16x16x32 product, loop over all tokens in blocks of 32, transposed
// tiles for the gradient products), written plainly: the q / dY tiles go through
// registers into two alternating LDS buffers, one barrier per block.  At d_h = 256 the resident operands (96) and the accumulators
// (192 registers) leave room for one wave per SIMD only; the launcher then uses
// workgroups of 4 waves.  Tile layout as in bwd_wgt16_kernel, for the same two kinds of reads:
// the 16-byte chunks of a 256-byte line are permuted by 2 (row % 8) at d_h = 256 (a row is two
// lines), the eight chunks of a 128-byte row by row & 6 at d_h = 64 (two rows share a line);
// tokens stay in MFMA row order.  Row reads and transposing reads are then both free of bank
// conflicts (with the general tile layout of the other kernels the row reads at d_h = 64 and
// the transposing reads at d_h = 256 took twice their cycles in this lane geometry).
// ---------------------------------------------------------------------------
template <int DH>
__device__ __forceinline__ int wdh_off(int row, int chunk) {
  static_assert(DH == 64 || DH == 256, "head widths of this kernel");
  if constexpr (DH == 64) return row * 128 + ((chunk ^ (row & 6)) << 4);
  else return row * 512 + ((chunk & ~15) << 4) + (((chunk & 15) ^ ((row & 7) << 1)) << 4);
}
template <int DH>
__device__ __forceinline__ int wdh_off8(int row, int col) {
  return wdh_off<DH>(row, col >> 3) + ((col & 4) << 1);
}

constexpr int kDhWindow = 6;   // operands in flight ahead of the one being consumed
// last stream position issued when item c is consumed; LDS read instructions behind the
// positions after c up to there (a row operand is one read, a transposed window two)
constexpr int dh_issued_before(int c, int ntot) { return c + kDhWindow > ntot - 1 ? ntot - 1 : c + kDhWindow; }
constexpr int dh_pending(int c, int na, int ntot) {
  int n = 0;
  for (int p = c + 1; p <= dh_issued_before(c, ntot); ++p) n += (p < na) ? 1 : 2;
  return n;
}

template <int DH, int NW>
__global__ __launch_bounds__(64 * NW, DH == 64 ? 2 : 1) void bwd_wgt_dh_kernel(BwdArgs a) {
  constexpr int THREADS = 64 * NW;
  constexpr int KS = DH / 32;              // contraction steps of the 16x16x32 products over d_h
  constexpr int JB = DH / 16;              // 16-row output tiles over d_h
  constexpr int CPR = DH / 8;              // 16-byte chunks per row
  constexpr int kTileBytes = 32 * DH * 2;
  constexpr int CHUNKS = 32 * CPR;
  constexpr int CH = (CHUNKS + THREADS - 1) / THREADS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // 2 x (q tile | dY tile)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cn = lane & 15, gq = lane >> 4;
  const int nblk = a.E * a.de / 16;              // 16-neuron blocks per head
  const int wg_per_head = (nblk + NW - 1) / NW;
  const int64_t item_s = xcd_work_item(blockIdx.x, a.n_items);
  if (item_s >= a.n_items) return;
  const int seg = (int)(item_s % a.wsplit);          // this workgroup's share of the tokens
  const int64_t item = item_s / a.wsplit;
  const int h = (int)(item / wg_per_head);
  const int blk = (int)(item % wg_per_head) * NW + wave;
  const bool active = blk < nblk;
  const int blk_c = active ? blk : nblk - 1;     // idle waves shadow a valid block, store nothing
  const int64_t N = a.N;
  const size_t row0 = ((size_t)h * nblk + blk_c) * 16;
  const int e_wave = blk_c / (a.de / 16);
  const float* Rw = a.Rws + ((size_t)h * a.E + e_wave) * N;

  bf16x8 Kf[KS], Uf[KS], Vf[KS];
  {
    const size_t off = (row0 + cn) * DH + 8 * gq;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Kf[ks] = *reinterpret_cast<const bf16x8*>(a.Wg + off + 32 * ks);
      Uf[ks] = *reinterpret_cast<const bf16x8*>(a.Wu + off + 32 * ks);
      Vf[ks] = *reinterpret_cast<const bf16x8*>(a.Wd + off + 32 * ks);
    }
  }
  f32x4 dK[JB], dU[JB], dV[JB];
#pragma unroll
  for (int jb = 0; jb < JB; ++jb) { dK[jb] = f32x4{0, 0, 0, 0}; dU[jb] = dK[jb]; dV[jb] = dK[jb]; }

  // ---- staging: rows past N are read from row N-1 (finite data) and get r = 0, so they add
  // nothing.  The loop is bound by instruction issue (at d_h = 64 the arithmetic alone keeps
  // the VALU busier than the products keep the MFMA pipe), so everything around it is kept
  // short: source pointers that advance block by block, r as two 16-byte loads, LDS read
  // addresses in registers with the buffer as an immediate offset, no per-row branches.
  static_assert(CHUNKS % THREADS == 0, "every thread moves CH chunks of each tile");
  const int64_t nb = (N + 31) / 32;
  const int64_t b0 = seg * a.blocks_per_seg;              // this workgroup's blocks: b0 .. b1-1
  const int64_t b1 = b0 + a.blocks_per_seg < nb ? b0 + a.blocks_per_seg : nb;
  // Two register sets: while block b is consumed from LDS, block b+1 sits in one set (stored
  // at the end of the step) and the loads of block b+2 are in flight into the other.  At
  // d_h = 256 there are no registers for a second set: one set, requested one block ahead.
  constexpr int SETS = (DH == 256) ? 1 : 2;
  constexpr int RSTEP = THREADS / CPR;          // rows between a thread's chunks
  u32x4 xreg[SETS][CH], yreg[SETS][CH];
  f32x4 rnext[SETS][2];
  typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
  const int srow = tid / CPR, scol = h * DH + (tid % CPR) * 8;
  // blocks are loaded in order, each once: the pointers just advance
  const uint16_t* xp = a.X + (b0 * 32 + srow) * a.ldx + scol;
  const uint16_t* yp = a.dY + (b0 * 32 + srow) * a.ldy + scol;
  const float* rp = Rw + b0 * 32 + 4 * gq;
  auto gload = [&](int64_t b, auto S_) {
    constexpr int S = decltype(S_)::value;
    if (b != nb - 1) {
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        xreg[S][i] = *reinterpret_cast<const u32x4*>(xp + (int64_t)(RSTEP * i) * a.ldx);
        yreg[S][i] = *reinterpret_cast<const u32x4*>(yp + (int64_t)(RSTEP * i) * a.ldy);
      }
      rnext[S][0] = *reinterpret_cast<const f32x4_a4*>(rp);
      rnext[S][1] = *reinterpret_cast<const f32x4_a4*>(rp + 16);
    } else {   // the last block may be ragged
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        int64_t t = b * 32 + srow + RSTEP * i;
        t = t < N ? t : N - 1;
        xreg[S][i] = *reinterpret_cast<const u32x4*>(a.X + t * a.ldx + scol);
        yreg[S][i] = *reinterpret_cast<const u32x4*>(a.dY + t * a.ldy + scol);
      }
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int64_t t = b * 32 + 16 * tb + 4 * gq + v;
          rnext[S][tb][v] = (t < N) ? Rw[t] : 0.f;
        }
    }
    xp += 32 * a.ldx;
    yp += 32 * a.ldy;
    rp += 32;
  };
  int soff[CH];   // where this thread's chunks go in a tile
#pragma unroll
  for (int i = 0; i < CH; ++i) soff[i] = wdh_off<DH>(srow + RSTEP * i, tid % CPR);
  auto lstore = [&](auto BUF_, auto S_) {
    constexpr int S = decltype(S_)::value;
    unsigned char* dst = smem + decltype(BUF_)::value * 2 * kTileBytes;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      *reinterpret_cast<u32x4*>(dst + soff[i]) = xreg[S][i];
      *reinterpret_cast<u32x4*>(dst + kTileBytes + soff[i]) = yreg[S][i];
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using SB = std::integral_constant<int, SETS - 1>;   // the second set, if there is one
  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;
  gload(b0, S0{});
  if (SETS == 2 && b0 + 1 < b1) gload(b0 + 1, SB{});
  lstore(B0{}, S0{});
  // LDS read addresses (buffer, tensor and token half are immediate offsets): rows of the
  // q / dY tiles: token row cn (+16), columns 32ks + 8gq ..; transposed windows: lane (cn, gq)
  // points at token row 4gq + cn/4 (+16), columns 16jb + 4(cn%4) ..
  const unsigned lbase = lds_addr_of(smem);
  unsigned arow[KS], atr[JB];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) arow[ks] = lbase + wdh_off<DH>(cn, 4 * ks + gq);
#pragma unroll
  for (int jb = 0; jb < JB; ++jb) atr[jb] = lbase + wdh_off8<DH>(4 * gq + (cn >> 2), 16 * jb + 4 * (cn & 3));
  __syncthreads();

  // block b: its tiles are in LDS buffer BUF and its r in register set SL, which is then
  // free and receives block b+2; SS holds block b+1
  auto step = [&](int64_t b, auto BUF_, auto SL, auto SS) {
    constexpr int BO = decltype(BUF_)::value * 2 * kTileBytes;   // dY tile: + kTileBytes
    const bool more = (b + 1 < b1);
    const f32x4 rv0 = rnext[decltype(SL)::value][0], rv1 = rnext[decltype(SL)::value][1];
    if (b + SETS < b1) gload(b + SETS, SL);

    // All LDS operands of the step form one stream, issued untracked kDhWindow items ahead
    // of their use with counted waits (the compiler, left alone, waits for each read right
    // after issuing it): items 0 .. NA-1 rows of the q / dY tiles, items NA .. transposed
    // windows, dY^T and q^T alternating.
    constexpr int NA = 4 * KS, NTOT = NA + 2 * JB;
    bf16x8 opa[NA];
    s16x4 xlo[2 * JB], xhi[2 * JB];
    auto issue = [&](auto P_) {
      constexpr int P = decltype(P_)::value;
      if constexpr (P < NA) {
        constexpr int tb = P / (2 * KS), ks = (P / 2) % KS, which = P & 1;   // 0: q, 1: dY
        opa[P] = lds_read_b128_untracked<BO + which * kTileBytes + tb * 16 * 2 * DH>(arow[ks]);   // 16 rows further: same swizzle
      } else {
        constexpr int J = P - NA, jb = J >> 1, TO = BO + ((J & 1) ? 0 : kTileBytes);  // even: dY^T, odd: q^T
        xlo[J] = lds_read_tr16_untracked<TO>(atr[jb]);
        xhi[J] = lds_read_tr16_untracked<TO + 16 * 2 * DH>(atr[jb]);
      }
    };
    auto advance = [&](auto C_) {
      constexpr int C = decltype(C_)::value;
      constexpr int lo = (C == 0) ? 0 : dh_issued_before(C - 1, NTOT) + 1;
      static_for<lo, dh_issued_before(C, NTOT) + 1>(issue);
    };
    f32x4 M[2], Nn[2], Ad[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) { M[tb] = f32x4{0, 0, 0, 0}; Nn[tb] = M[tb]; Ad[tb] = M[tb]; }
    static_for<0, NA>([&](auto C_) {
      constexpr int C = decltype(C_)::value, tb = C / (2 * KS), ks = (C / 2) % KS;
      advance(C_);
      lds_wait<dh_pending(C, NA, NTOT)>(opa[C]);
      if constexpr ((C & 1) == 0) {
        M[tb] = mfma16(opa[C], Kf[ks], M[tb]);
        Nn[tb] = mfma16(opa[C], Uf[ks], Nn[tb]);
      } else {
        Ad[tb] = mfma16(opa[C], Vf[ks], Ad[tb]);
      }
    });
    // element (tb, v): token 16tb + 4gq + v, neuron cn; it becomes contraction slot
    // 4tb + v of the gradient products
    float ag[8], dm[8], dn[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tb = i >> 2, v = i & 3;
      const float m = M[tb][v], n = Nn[tb][v], da = Ad[tb][v], rw = tb ? rv1[v] : rv0[v];
      const float t = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * m);
      const float sg = __builtin_amdgcn_rcpf(1.0f + t);
      const float sw = rw * sg;
      const float x = (1.0f + m) - m * sg;   // silu'(m) = sg (1 + m - silu(m))
      const float pw = m * sw;
      ag[i] = pw * n;
      dn[i] = pw * da;
      dm[i] = ((n * sw) * x) * da;
    }
    u32x4 pa, pm, pn;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pa[i] = pack_bf16(ag[2 * i], ag[2 * i + 1]);
      pm[i] = pack_bf16(dm[2 * i], dm[2 * i + 1]);
      pn[i] = pack_bf16(dn[2 * i], dn[2 * i + 1]);
    }
    const bf16x8 agf = __builtin_bit_cast(bf16x8, pa);
    const bf16x8 dmf = __builtin_bit_cast(bf16x8, pm), dnf = __builtin_bit_cast(bf16x8, pn);

    // dV^T[j][c] += dY^T a ; dK^T[j][c] += q^T dM ; dU^T[j][c] += q^T dN
    static_for<NA, NTOT>([&](auto C_) {
      constexpr int C = decltype(C_)::value, J = C - NA, jb = J >> 1;
      advance(C_);
      lds_wait<dh_pending(C, NA, NTOT)>(xlo[J], xhi[J]);
      const bf16x8 xt = join_tr(xlo[J], xhi[J]);
      if constexpr ((J & 1) == 0) {
        dV[jb] = mfma16(xt, agf, dV[jb]);
      } else {
        dK[jb] = mfma16(xt, dmf, dK[jb]);
        dU[jb] = mfma16(xt, dnf, dU[jb]);
      }
    });
    if (more) lstore(std::integral_constant<int, 1 - decltype(BUF_)::value>{}, SS);
    __syncthreads();
  };
  for (int64_t b = b0; b < b1; b += 2) {
    step(b, B0{}, S0{}, SB{});
    if (b + 1 < b1) step(b + 1, B1{}, SB{}, S0{});
  }

  if (active && a.wsplit > 1) {
    // fp32 partial gradients of this token segment: [seg][K | U | V][row][d_h]
    const size_t rows = (size_t)a.H * nblk * 16;
    float* dst = a.WPws + (((size_t)seg * 3) * rows + row0 + cn) * DH + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
      *reinterpret_cast<f32x4*>(dst + 16 * jb) = dK[jb];
      *reinterpret_cast<f32x4*>(dst + rows * DH + 16 * jb) = dU[jb];
      *reinterpret_cast<f32x4*>(dst + 2 * rows * DH + 16 * jb) = dV[jb];
    }
  } else if (active) {
    // accumulators are [j][c]: lane = neuron column cn, register v = row 16jb + 4gq + v
    const size_t off = (row0 + cn) * DH + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
      const size_t o = off + 16 * jb;
      if (a.dWg) {
        u32x2 pk = {pack_bf16(dK[jb][0], dK[jb][1]), pack_bf16(dK[jb][2], dK[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWg + o) = pk;
      }
      if (a.dWu) {
        u32x2 pk = {pack_bf16(dU[jb][0], dU[jb][1]), pack_bf16(dU[jb][2], dU[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWu + o) = pk;
      }
      if (a.dWd) {
        u32x2 pk = {pack_bf16(dV[jb][0], dV[jb][1]), pack_bf16(dV[jb][2], dV[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWd + o) = pk;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// weight-major kernel for d_h = 64
//
// Same decomposition as bwd_wgt16_kernel (one wave = 16 neurons, K/U/V rows resident, loop
// over all tokens in blocks of 32), for a head width at which the arithmetic, not the
// products, is the longer pipe: per block a wave runs 24 MFMAs (384 cycles) against about
// 650 cycles of VALU work on its 8 elements per lane.  What helps is more waves to fill the
// VALU and as few other instructions as possible: workgroups of 4 waves with about 160
// registers each, three per CU; token tiles ([32][64] bf16 of q and of dY, chunks permuted as
// in bwd_wgt_dh_kernel) and r go global -> LDS directly into four stages, requested three
// blocks ahead (no staging registers, no LDS stores); one barrier per block.
// ---------------------------------------------------------------------------
constexpr int kW6Dh = 64;
constexpr int kW6Waves = 4;
constexpr int kW6Threads = 64 * kW6Waves;
constexpr int kW6Tile = 32 * kW6Dh * 2;             // 4 KB
constexpr int kW6Stages = 4;
constexpr int kW6YRing = kW6Stages * kW6Tile;       // start of the dY ring
constexpr int kW6RRing = 2 * kW6YRing;              // start of the r ring
constexpr int kW6RSlot = kW6Waves * 64 * 4;
constexpr int kW6LdsBytes = kW6RRing + kW6Stages * kW6RSlot;   // 36 KB
constexpr int kW6DmaInstrs = 3;                     // direct loads per wave and block
constexpr int kW6Window = 4;                        // operands kept in flight ahead of the one being consumed
// operand stream of a block: items 0..7 rows of the q / dY tiles (1 LDS read each), items
// 8..15 transposed windows, dY^T and q^T alternating (2 reads each)
constexpr int w6_issued_before(int c) { return c + kW6Window > 15 ? 15 : c + kW6Window; }
constexpr int w6_pending(int c) {
  int n = 0;
  for (int p = c + 1; p <= w6_issued_before(c); ++p) n += (p < 8) ? 1 : 2;
  return n;
}

__global__ __launch_bounds__(kW6Threads, 3) void bwd_wgt64_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cn = lane & 15, gq = lane >> 4;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int nblk = a.E * a.de / 16;              // 16-neuron blocks per head
  const int wg_per_head = (nblk + kW6Waves - 1) / kW6Waves;
  const int64_t item_s = xcd_work_item(blockIdx.x, a.n_items);
  if (item_s >= a.n_items) return;
  const int seg = (int)(item_s % a.wsplit);          // this workgroup's share of the tokens
  const int64_t item = item_s / a.wsplit;
  const int h = (int)(item / wg_per_head);
  const int blk = (int)(item % wg_per_head) * kW6Waves + wave_u;
  const bool active = blk < nblk;
  const int blk_c = active ? blk : nblk - 1;     // idle waves shadow a valid block, store nothing
  const int64_t N = a.N;
  const size_t row0 = ((size_t)h * nblk + blk_c) * 16;
  const int e_wave = blk_c / (a.de / 16);

  // resident weight operands: lane (neuron cn, group gq) holds columns 32ks + 8gq ..
  bf16x8 Kf[2], Uf[2], Vf[2];
  {
    const size_t off = (row0 + cn) * kW6Dh + 8 * gq;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      Kf[ks] = *reinterpret_cast<const bf16x8*>(a.Wg + off + 32 * ks);
      Uf[ks] = *reinterpret_cast<const bf16x8*>(a.Wu + off + 32 * ks);
      Vf[ks] = *reinterpret_cast<const bf16x8*>(a.Wd + off + 32 * ks);
    }
  }
  f32x4 dK[4], dU[4], dV[4];
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) { dK[jb] = f32x4{0, 0, 0, 0}; dU[jb] = dK[jb]; dV[jb] = dK[jb]; }

  // ---- staging -----------------------------------------------------------------
  // Wave w moves rows 8w .. 8w+7 of the q and of the dY tile (one 1 KB image each: LDS position
  // p of a row holds chunk p ^ (row & 6)) and the 32 r values of its own sub-network.  Addresses
  // are a wave-uniform base that advances block by block plus a 32-bit per-lane byte offset.
  // Rows past N are read from row N-1 (finite data) and get r = 0, so they add nothing.
  const int64_t nb = (N + 31) / 32;
  const int64_t b0 = seg * a.blocks_per_seg;              // this workgroup's blocks: b0 .. b1-1
  const int64_t b1 = b0 + a.blocks_per_seg < nb ? b0 + a.blocks_per_seg : nb;
  auto lane_col = [&](int l) {   // element column inside the head of the chunk lane l moves
    const int row = 8 * wave_u + (l >> 3);
    return ((l & 7) ^ (row & 6)) << 3;
  };
  const unsigned vx = (unsigned)(((8 * wave_u + (lane >> 3)) * a.ldx + lane_col(lane)) * 2);
  const unsigned vy = (unsigned)(((8 * wave_u + (lane >> 3)) * a.ldy + lane_col(lane)) * 2);
  const unsigned vr = 4 * (lane & 31);
  const unsigned char* xbase = reinterpret_cast<const unsigned char*>(a.X + b0 * 32 * a.ldx + h * kW6Dh);
  const unsigned char* ybase = reinterpret_cast<const unsigned char*>(a.dY + b0 * 32 * a.ldy + h * kW6Dh);
  const float* Rw = a.Rws + ((size_t)h * a.E + e_wave) * N;
  const unsigned char* rbase = reinterpret_cast<const unsigned char*>(Rw + b0 * 32);
  // blocks are requested in order, each once: the bases just advance
  auto dma = [&](int64_t blkidx, int stage) {
    unsigned x0 = vx, y0 = vy, r0 = vr;
    if (blkidx == nb - 1) {   // the last block may be ragged
      int l = lane;
      asm volatile("" : "+v"(l));   // recomputed here, not kept in registers through the loop
      const int64_t last = N - 1 - blkidx * 32;   // >= 0
      const int64_t ra = 8 * wave_u + (l >> 3), rr = l & 31;
      const int64_t ca = ra < last ? ra : last;
      x0 = (unsigned)((ca * a.ldx + lane_col(l)) * 2);
      y0 = (unsigned)((ca * a.ldy + lane_col(l)) * 2);
      r0 = 4 * (unsigned)(rr < last ? rr : last);
    }
    unsigned char* dst = smem + stage * kW6Tile + wave_u * 1024;
    global_to_lds_16B(xbase + x0, dst);
    global_to_lds_16B(ybase + y0, dst + kW6YRing);
    __builtin_amdgcn_global_load_lds(
        (__attribute__((address_space(1))) const void*)(rbase + r0),
        (__attribute__((address_space(3))) void*)(smem + kW6RRing + stage * kW6RSlot + wave_u * 256),
        4, 0, 0);
    xbase += 64 * a.ldx;
    ybase += 64 * a.ldy;
    rbase += 128;
  };
  dma(b0, 0);
  if (b0 + 1 < b1) dma(b0 + 1, 1);
  if (b0 + 2 < b1) dma(b0 + 2, 2);

  // LDS read addresses (stage, tensor and token half are immediate offsets): rows of the
  // q / dY tiles: token row cn (+16), columns 32ks + 8gq ..; transposed windows: lane (cn, gq)
  // points at token row 4gq + cn/4 (+16), columns 16jb + 4(cn%4) ..
  const unsigned lbase = lds_addr_of(smem);
  unsigned arow[2], atr[4];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) arow[ks] = lbase + wdh_off<kW6Dh>(cn, 4 * ks + gq);
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) atr[jb] = lbase + wdh_off8<kW6Dh>(4 * gq + (cn >> 2), 16 * jb + 4 * (cn & 3));
  const unsigned raddr = lbase + kW6RRing + wave * 256 + 16 * gq;   // r of MFMA rows 4gq.. (+64: next 16 tokens)

  // block b, in stage S
  auto step = [&](int64_t b, auto S_) {
    constexpr int S = decltype(S_)::value, SO = S * kW6Tile;
    // Own requests in flight: blocks b, b+1, b+2 as far as they exist; block b must have landed.
    // After the barrier every wave's part of it is visible and every wave is done with block
    // b-1, whose stage the next request overwrites.
    if (b + 2 < b1) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * kW6DmaInstrs));
    else if (b + 1 < b1) __builtin_amdgcn_s_waitcnt(0x0F70 | kW6DmaInstrs);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (b + 3 < b1) dma(b + 3, (S + 3) % kW6Stages);

    f32x4 rv[2];
    bf16x8 opa[8];
    s16x4 xlo[8], xhi[8];
    auto issue = [&](auto P_) {
      constexpr int P = decltype(P_)::value;
      if constexpr (P < 8) {
        constexpr int tb = P >> 2, ks = (P >> 1) & 1, which = P & 1;   // 0: q, 1: dY
        opa[P] = lds_read_b128_untracked<SO + which * kW6YRing + tb * 2048>(arow[ks]);   // 16 rows further: same permutation
      } else {
        constexpr int J = P - 8, jb = J >> 1, TO = SO + ((J & 1) ? 0 : kW6YRing);  // even: dY^T, odd: q^T
        xlo[J] = lds_read_tr16_untracked<TO>(atr[jb]);
        xhi[J] = lds_read_tr16_untracked<TO + 2048>(atr[jb]);
      }
    };
    auto advance = [&](auto C_) {
      constexpr int C = decltype(C_)::value;
      constexpr int lo = (C == 0) ? 0 : w6_issued_before(C - 1) + 1;
      static_for<lo, w6_issued_before(C) + 1>(issue);
    };
    rv[0] = __builtin_bit_cast(f32x4, lds_read_b128_untracked<S * kW6RSlot>(raddr));
    rv[1] = __builtin_bit_cast(f32x4, lds_read_b128_untracked<S * kW6RSlot + 64>(raddr));
    f32x4 M[2], Nn[2], Ad[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) { M[tb] = f32x4{0, 0, 0, 0}; Nn[tb] = M[tb]; Ad[tb] = M[tb]; }
    static_for<0, 8>([&](auto C_) {
      constexpr int C = decltype(C_)::value, tb = C >> 2, ks = (C >> 1) & 1;
      advance(C_);
      lds_wait<w6_pending(C)>(opa[C]);
      if constexpr ((C & 1) == 0) {
        M[tb] = mfma16(opa[C], Kf[ks], M[tb]);
        Nn[tb] = mfma16(opa[C], Uf[ks], Nn[tb]);
      } else {
        Ad[tb] = mfma16(opa[C], Vf[ks], Ad[tb]);
      }
    });
    // (the r reads are older than every read of the stream)
    asm volatile("" : "+v"(rv[0]), "+v"(rv[1]));
    if (b == nb - 1) {   // rows past N were read from row N-1: give them r = 0
      asm volatile("" ::: "memory");   // (a real branch: the last block only)
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (b * 32 + 16 * tb + 4 * gq + v >= N) rv[tb][v] = 0.f;
    }
    // element (tb, v): token 16tb + 4gq + v, neuron cn; it becomes contraction slot
    // 4tb + v of the gradient products
    float ag[8], dm[8], dn[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tb = i >> 2, v = i & 3;
      const float m = M[tb][v], n = Nn[tb][v], da = Ad[tb][v];
      const float t = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * m);
      const float sg = __builtin_amdgcn_rcpf(1.0f + t);
      const float sw = rv[tb][v] * sg;
      const float x = (1.0f + m) - m * sg;   // silu'(m) = sg (1 + m - silu(m))
      const float pw = m * sw;
      ag[i] = pw * n;
      dn[i] = pw * da;
      dm[i] = ((n * sw) * x) * da;
    }
    u32x4 pa, pm, pn;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pa[i] = pack_bf16(ag[2 * i], ag[2 * i + 1]);
      pm[i] = pack_bf16(dm[2 * i], dm[2 * i + 1]);
      pn[i] = pack_bf16(dn[2 * i], dn[2 * i + 1]);
    }
    const bf16x8 agf = __builtin_bit_cast(bf16x8, pa);
    const bf16x8 dmf = __builtin_bit_cast(bf16x8, pm), dnf = __builtin_bit_cast(bf16x8, pn);

    // dV^T[j][c] += dY^T a ; dK^T[j][c] += q^T dM ; dU^T[j][c] += q^T dN
    static_for<8, 16>([&](auto C_) {
      constexpr int C = decltype(C_)::value, J = C - 8, jb = J >> 1;
      advance(C_);
      lds_wait<w6_pending(C)>(xlo[J], xhi[J]);
      const bf16x8 xt = join_tr(xlo[J], xhi[J]);
      if constexpr ((J & 1) == 0) {
        dV[jb] = mfma16(xt, agf, dV[jb]);
      } else {
        dK[jb] = mfma16(xt, dmf, dK[jb]);
        dU[jb] = mfma16(xt, dnf, dU[jb]);
      }
    });
  };
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  using C2 = std::integral_constant<int, 2>;
  using C3 = std::integral_constant<int, 3>;
  for (int64_t b = b0; b < b1; b += 4) {
    step(b, C0{});
    if (b + 1 < b1) step(b + 1, C1{});
    if (b + 2 < b1) step(b + 2, C2{});
    if (b + 3 < b1) step(b + 3, C3{});
  }

  if (active && a.wsplit > 1) {
    // fp32 partial gradients of this token segment: [seg][K | U | V][row][d_h]
    const size_t rows = (size_t)a.H * nblk * 16;
    float* dst = a.WPws + (((size_t)seg * 3) * rows + row0 + cn) * kW6Dh + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      *reinterpret_cast<f32x4*>(dst + 16 * jb) = dK[jb];
      *reinterpret_cast<f32x4*>(dst + rows * kW6Dh + 16 * jb) = dU[jb];
      *reinterpret_cast<f32x4*>(dst + 2 * rows * kW6Dh + 16 * jb) = dV[jb];
    }
  } else if (active) {
    // accumulators are [j][c]: lane = neuron column cn, register v = row 16jb + 4gq + v
    const size_t off = (row0 + cn) * kW6Dh + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      const size_t o = off + 16 * jb;
      if (a.dWg) {
        u32x2 pk = {pack_bf16(dK[jb][0], dK[jb][1]), pack_bf16(dK[jb][2], dK[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWg + o) = pk;
      }
      if (a.dWu) {
        u32x2 pk = {pack_bf16(dU[jb][0], dU[jb][1]), pack_bf16(dU[jb][2], dU[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWu + o) = pk;
      }
      if (a.dWd) {
        u32x2 pk = {pack_bf16(dV[jb][0], dV[jb][1]), pack_bf16(dV[jb][2], dV[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWd + o) = pk;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// weight-major kernel for d_h = 256, two waves per SIMD
//
// The 16 neurons of a block have 3 x 16 x 256 resident operands and as many fp32 gradient
// accumulators: more than one wave's 256 registers.  Two waves share the block instead: wave
// `hf` of the pair owns columns 128 hf .. 128 hf + 127 of d_h and finishes tokens 16 hf ..
// 16 hf + 15 of every block of 32.  Per block:
//   M, N, dA [32 tok][16]: each wave contracts over its own 128 columns (24 MFMA) and hands the
//       partial sums of the partner's 16 tokens over through LDS (exchange 1)
//   a, dn, dm of its own 16 tokens: fp32 VALU on 4 elements per lane; the packed bf16 results
//       go to the partner through LDS as well (exchange 2)
//   dV^T[j][c] += dY^T a; dK^T += q^T dm; dU^T += q^T dn for the wave's own 128 rows j (24 MFMA)
// so a wave needs 48 resident + 96 accumulator registers, as in bwd_wgt16_kernel, and the
// workgroup's eight waves (four blocks of 16 neurons) run two per SIMD.  A step has two
// barriers: A, after the partial sums are written, and B, after the packed results are.  Waves
// 4-7 pass one barrier more before the loop and waves 0-3 one more after it, so that the two
// waves of a SIMD are half a step apart: one does the arithmetic (between A and B) while the
// other runs its 48 MFMAs (between B and the next A: the gradient products of block b, then
// the recompute products of block b + 1, as one operand stream, at raised priority).
// What bounds a step is instruction issue, not the MFMA pipe: a wave's stream of 44 LDS reads,
// 32 waits and 48 MFMAs takes about 1250 cycles alone on its SIMD against 768 cycles of MFMA,
// and the other wave's VALU and load instructions come on top.  Hence no address arithmetic in
// the stream (all operand addresses are loop-invariant registers plus immediate offsets), the
// arithmetic shared out over the pair, and the few staging loads per wave.
// Token tiles ([32][256] bf16 of q and of dY, chunks permuted as in bwd_wgt_dh_kernel) go
// global -> LDS directly into three stages; see the loop for when a stage may be requested again.
// ---------------------------------------------------------------------------
constexpr int kW2Waves = 8;
constexpr int kW2Threads = 64 * kW2Waves;
constexpr int kW2Tile = 32 * kW2Dh * 2;            // 16 KB
constexpr int kW2Stages = 3;
constexpr int kW2YRing = kW2Stages * kW2Tile;      // start of the dY ring
constexpr int kW2RRing = 2 * kW2YRing;             // start of the r ring
constexpr int kW2RSlot = kW2Waves * 64 * 4;
// exchange slots per wave, read by its partner: 3 KB of partial sums, 1.5 KB of packed results
constexpr int kW2Xchg1 = kW2RRing + kW2Stages * kW2RSlot;
constexpr int kW2Xchg1Slot = 3 * 1024;
constexpr int kW2Xchg2 = kW2Xchg1 + kW2Waves * kW2Xchg1Slot;
constexpr int kW2Xchg2Slot = 3 * 512;
constexpr int kW2LdsBytes = kW2Xchg2 + kW2Waves * kW2Xchg2Slot;
static_assert(kW2LdsBytes <= 160 * 1024, "LDS of a CU");
static_assert((kW2Stages - 1) * kW2Tile + 4096 < 65536, "LDS read offsets are 16-bit");
constexpr int kW2Window = 4;   // operands kept in flight ahead of the one being consumed
// Operand stream of a step (position = consumption order):
//   0..15   transposed windows of block b: dY^T 0, q^T 0, dY^T 1, q^T 1 ..       (2 LDS reads each)
//   16..23  q rows of block b + 1: own 16 tokens steps 0..3, the partner's 16    (1)
//   24..31  dY rows of block b + 1                                                (1)
// A pass that starts at position 16 does only the recompute products (the first block).
constexpr int w2_instrs(int p) { return p < 16 ? 2 : 1; }
constexpr int w2_issued_before(int c) { return c + kW2Window > 31 ? 31 : c + kW2Window; }
constexpr int w2_pending(int c) {
  int n = 0;
  for (int p = c + 1; p <= w2_issued_before(c); ++p) n += w2_instrs(p);
  return n;
}

__global__ __launch_bounds__(kW2Threads) void bwd_wgt256_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];   // (address bits are XORed: see below)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cn = lane & 15, gq = lane >> 4;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int pair = wave_u >> 1, hf = wave_u & 1;
  const bool lag = wave_u >= 4;
  const int nblk = a.E * a.de / 16;              // 16-neuron blocks per head
  const int wg_per_head = (nblk + kW2Blocks - 1) / kW2Blocks;
  // work list as in bwd_wgt16_kernel: XCD x takes neuron groups x gpx .. (x+1) gpx - 1, first
  // those that take all tokens, then, `wsplit` workgroups each, the groups of its last round
  const int xcd = blockIdx.x & 7, widx = blockIdx.x >> 3;
  const int g_first = xcd * a.gpx;
  const int n_here = min(a.n_groups - g_first, a.gpx);
  const int n_full = min(a.full_px, n_here);
  int group, seg = 0, cgroup = 0;
  bool split = false;
  if (widx < n_full) {
    group = g_first + widx;
  } else {
    const int j = widx - n_full, lt = j / a.wsplit;
    if (n_full + lt >= n_here) return;   // whole workgroup leaves together
    group = g_first + n_full + lt;
    seg = j - lt * a.wsplit;
    split = a.wsplit > 1;
    cgroup = xcd * (a.gpx - a.full_px) + lt;
  }
  const int h = group / wg_per_head;
  const int blk = (group % wg_per_head) * kW2Blocks + pair;
  const bool active = blk < nblk;
  const int blk_c = active ? blk : nblk - 1;     // idle pairs shadow a valid block, store nothing
  const int64_t N = a.N;
  const size_t row0 = ((size_t)h * nblk + blk_c) * 16;   // first neuron row of this pair
  const int e_wave = blk_c / (a.de / 16);

  // resident weight operands: lane (neuron cn, group gq) holds columns 128hf + 32ks + 8gq ..
  bf16x8 Kf[4], Uf[4], Vf[4];
  {
    const size_t off = (row0 + cn) * kW2Dh + 128 * hf + 8 * gq;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      Kf[ks] = *reinterpret_cast<const bf16x8*>(a.Wg + off + 32 * ks);
      Uf[ks] = *reinterpret_cast<const bf16x8*>(a.Wu + off + 32 * ks);
      Vf[ks] = *reinterpret_cast<const bf16x8*>(a.Wd + off + 32 * ks);
    }
  }
  f32x4 dK[8], dU[8], dV[8];
#pragma unroll
  for (int jb = 0; jb < 8; ++jb) { dK[jb] = f32x4{0, 0, 0, 0}; dU[jb] = dK[jb]; dV[jb] = dK[jb]; }

  // ---- staging -----------------------------------------------------------------
  // Wave w moves rows 2w, 2w+1 and 2w+16, 2w+17 of the q and dY tiles (a 1 KB image of two
  // rows per load; LDS position p of a row holds chunk (p & 16) | ((p & 15) ^ 2 (row % 8)),
  // the same for rows 16 apart) and the 32 r values of its own sub-network.  Addresses are a
  // wave-uniform base that advances block by block plus a 32-bit per-lane byte offset.
  const float* Rw = a.Rws + ((size_t)h * a.E + e_wave) * N;
  const int64_t nb = (N + 31) / 32;                       // all blocks of 32 tokens
  const int64_t b0 = split ? seg * a.blocks_per_seg : 0;  // this workgroup's blocks: b0 .. b1-1
  const int64_t b1 = (split && b0 + a.blocks_per_seg < nb) ? b0 + a.blocks_per_seg : nb;
  auto lane_col = [&](int l) {   // element column inside the head of the chunk lane l moves
    const int row = 2 * wave_u + (l >> 5), pos = l & 31;
    return ((pos & 16) | ((pos & 15) ^ ((row & 7) << 1))) << 3;
  };
  const unsigned vx = (unsigned)(((2 * wave_u + (lane >> 5)) * a.ldx + lane_col(lane)) * 2);
  const unsigned vy = (unsigned)(((2 * wave_u + (lane >> 5)) * a.ldy + lane_col(lane)) * 2);
  const unsigned vr = 4 * (lane & 31);
  const unsigned char* xbase = reinterpret_cast<const unsigned char*>(a.X + b0 * 32 * a.ldx + h * kW2Dh);
  const unsigned char* ybase = reinterpret_cast<const unsigned char*>(a.dY + b0 * 32 * a.ldy + h * kW2Dh);
  const unsigned char* rbase = reinterpret_cast<const unsigned char*>(Rw + b0 * 32);
  // blocks are requested in order, each once: the bases just advance
  auto dma = [&](int64_t blkidx, int stage) {
    unsigned x0 = vx, x1 = vx + (unsigned)(32 * a.ldx), y0 = vy, y1 = vy + (unsigned)(32 * a.ldy), r0 = vr;
    if (blkidx == nb - 1) {   // the last block may be ragged: rows past N read row N-1
      int l = lane;
      asm volatile("" : "+v"(l));   // recomputed here, not kept in registers through the loop
      const int64_t last = N - 1 - blkidx * 32;   // >= 0
      const int64_t ra = 2 * wave_u + (l >> 5), rb = ra + 16, rr = l & 31;
      const int64_t ca = ra < last ? ra : last, cb = rb < last ? rb : last;
      x0 = (unsigned)((ca * a.ldx + lane_col(l)) * 2);
      x1 = (unsigned)((cb * a.ldx + lane_col(l)) * 2);
      y0 = (unsigned)((ca * a.ldy + lane_col(l)) * 2);
      y1 = (unsigned)((cb * a.ldy + lane_col(l)) * 2);
      r0 = 4 * (unsigned)(rr < last ? rr : last);
    }
    unsigned char* dst = smem + stage * kW2Tile + wave_u * 1024;
    global_to_lds_16B(xbase + x0, dst);
    global_to_lds_16B(xbase + x1, dst + 8192);
    global_to_lds_16B(ybase + y0, dst + kW2YRing);
    global_to_lds_16B(ybase + y1, dst + kW2YRing + 8192);
    __builtin_amdgcn_global_load_lds(
        (__attribute__((address_space(1))) const void*)(rbase + r0),
        (__attribute__((address_space(3))) void*)(smem + kW2RRing + stage * kW2RSlot + wave_u * 256),
        4, 0, 0);
    xbase += 64 * a.ldx;
    ybase += 64 * a.ldy;
    rbase += 128;
  };
  dma(b0, 0);
  if (b0 + 1 < b1) dma(b0 + 1, 1);
  if (b0 + 2 < b1) dma(b0 + 2, 2);

  // ---- loop-invariant LDS addresses -----------------------------------------------
  const unsigned lbase = lds_addr_of(smem);
  // Row operands: token row cn (+16), 16-byte chunk 16hf + 4ks + gq; transposed operands: token
  // rows 4gq + cn/4 (+16), columns 128hf + 16jb + 4(cn%4).  The chunk permutation is an XOR on
  // address bits 5-7, so the address for step ks is that for step 0 ^ (ks << 6) and the one for
  // row tile jb that for tile 0 ^ (jb << 5).
  const unsigned qa0 = lbase + wdh_off<kW2Dh>(cn, 16 * hf + gq), ya0 = qa0 + kW2YRing;
  const unsigned ta0 = lbase + wdh_off8<kW2Dh>(4 * gq + (cn >> 2), 128 * hf + 4 * (cn & 3)), tya0 = ta0 + kW2YRing;
  const unsigned raddr = lbase + kW2RRing + wave * 256 + 16 * gq;   // r of MFMA rows 4gq.. (+64: next 16 tokens)
  // exchange slots: own (written) and the partner's (read)
  float* x1own = reinterpret_cast<float*>(smem + kW2Xchg1 + wave_u * kW2Xchg1Slot) + 4 * lane;
  const unsigned x1par = lbase + kW2Xchg1 + (wave ^ 1) * kW2Xchg1Slot + 16 * lane;
  unsigned* x2own = reinterpret_cast<unsigned*>(smem + kW2Xchg2 + wave_u * kW2Xchg2Slot) + 2 * lane;
  const unsigned x2par = lbase + kW2Xchg2 + (wave ^ 1) * kW2Xchg2Slot + 8 * lane;
  // all 24 operand addresses stay in registers (immediate offsets select stage and token
  // half): an XOR in front of every read costs the stream more than the registers do
  unsigned qx[4], yx[4], tx[8], tyx[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) { qx[i] = qa0 ^ (i << 6); yx[i] = ya0 ^ (i << 6); }
#pragma unroll
  for (int i = 0; i < 8; ++i) { tx[i] = ta0 ^ (i << 5); tyx[i] = tya0 ^ (i << 5); }

  f32x4 M[2], Nn[2], Ad[2];   // this wave's partial M, N, dA of the next block to be finished
  bf16x8 agf, dmf, dnf;       // B operands of the gradient products of the current block

  // One pass over the operand stream from position FIRST: the gradient products of the block
  // in stage S (FIRST = 0), then the partial recompute products of the block in stage S + 1.
  // Before item c is consumed everything up to kW2Window positions ahead of it has been
  // issued, and the wait names exactly the number of reads issued after it.
  auto stream = [&](auto S_, auto FIRST_, auto PREFETCH_ONLY_, bf16x8 (&op)[16], s16x4 (&xlo)[16], s16x4 (&xhi)[16]) {
    constexpr int S = decltype(S_)::value, FIRST = decltype(FIRST_)::value;
    constexpr bool PREFETCH_ONLY = decltype(PREFETCH_ONLY_)::value;
    constexpr int SO = S * kW2Tile, SN = ((S + 1) % kW2Stages) * kW2Tile;

    auto issue = [&](auto P_) {
      constexpr int P = decltype(P_)::value;
      if constexpr (P < 16) {
        constexpr int J = P, JB = J >> 1;
        if constexpr ((J & 1) == 0) {
          xlo[J] = lds_read_tr16_untracked<SO>(tyx[JB]);
          xhi[J] = lds_read_tr16_untracked<SO + 8192>(tyx[JB]);   // 16 rows further: same permutation
        } else {
          xlo[J] = lds_read_tr16_untracked<SO>(tx[JB]);
          xhi[J] = lds_read_tr16_untracked<SO + 8192>(tx[JB]);
        }
      } else if constexpr (P < 24) {
        constexpr int I = P - 16;
        op[I] = lds_read_b128_untracked<SN + (I >> 2) * 8192>(qx[I & 3]);
      } else {
        constexpr int I = P - 16;
        op[I] = lds_read_b128_untracked<SN + ((I - 8) >> 2) * 8192>(yx[I & 3]);
      }
    };
    if constexpr (PREFETCH_ONLY) {
      static_for<FIRST, w2_issued_before(FIRST) + 1>(issue);
    } else {
      auto advance = [&](auto C_) {   // what item C needs in flight beyond what item C-1 required
        constexpr int C = decltype(C_)::value;
        if constexpr (C > FIRST) static_for<w2_issued_before(C - 1) + 1, w2_issued_before(C) + 1>(issue);
      };
      static_for<FIRST, 16>([&](auto C_) {
        constexpr int C = decltype(C_)::value, J = C, JB = J >> 1;
        advance(C_);
        lds_wait<w2_pending(C)>(xlo[J], xhi[J]);
        const bf16x8 xt = join_tr(xlo[J], xhi[J]);
        if constexpr ((J & 1) == 0) {
          dV[JB] = mfma16(xt, agf, dV[JB]);
        } else {
          dK[JB] = mfma16(xt, dmf, dK[JB]);
          dU[JB] = mfma16(xt, dnf, dU[JB]);
        }
      });
#pragma unroll
      for (int t = 0; t < 2; ++t) { M[t] = f32x4{0, 0, 0, 0}; Nn[t] = M[t]; Ad[t] = M[t]; }
      static_for<16, 24>([&](auto C_) {
        constexpr int C = decltype(C_)::value, I = C - 16;
        advance(C_);
        lds_wait<w2_pending(C)>(op[I]);
        M[I >> 2] = mfma16(op[I], Kf[I & 3], M[I >> 2]);
        Nn[I >> 2] = mfma16(op[I], Uf[I & 3], Nn[I >> 2]);
      });
      static_for<24, 32>([&](auto C_) {
        constexpr int C = decltype(C_)::value, I = C - 16;
        advance(C_);
        lds_wait<w2_pending(C)>(op[I]);
        Ad[(I - 8) >> 2] = mfma16(op[I], Vf[I & 3], Ad[(I - 8) >> 2]);
      });
      // exchange 1: the partial sums of the partner's tokens (wave hf finishes tokens 16hf ..)
      if (hf == 0) {
        *reinterpret_cast<f32x4*>(x1own) = M[1];
        *reinterpret_cast<f32x4*>(x1own + 256) = Nn[1];
        *reinterpret_cast<f32x4*>(x1own + 512) = Ad[1];
      } else {
        *reinterpret_cast<f32x4*>(x1own) = M[0];
        *reinterpret_cast<f32x4*>(x1own + 256) = Nn[0];
        *reinterpret_cast<f32x4*>(x1own + 512) = Ad[0];
      }
    }
  };
  using T = std::true_type;
  using F = std::false_type;
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  using C2 = std::integral_constant<int, 2>;
  using C16 = std::integral_constant<int, 16>;

  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the first blocks have landed
  __syncthreads();
  {
    // recompute products of block b0 (stage 0 = the stage after stage 2)
    bf16x8 op[16];
    s16x4 xlo[16], xhi[16];
    stream(C2{}, C16{}, T{}, op, xlo, xhi);
    stream(C2{}, C16{}, F{}, op, xlo, xhi);
  }

  // Between the barriers A and B of block b (in stage S), for wave HF of a pair: finish M, N,
  // dA of the tokens 16 HF .. of the block, arithmetic on them, packed results to the partner;
  // after B the partner's packed results complete the B operands of the gradient products.
  auto finish = [&](int64_t b, bool req, auto S_, auto HF_, bf16x8 (&op)[16], s16x4 (&xlo)[16], s16x4 (&xhi)[16]) {
    constexpr int S = decltype(S_)::value, HF = decltype(HF_)::value, S2 = (S + 2) % kW2Stages;
    f32x4 pp[3], rv;   // the partner's partial sums of these tokens; their r
#pragma unroll
    for (int i = 0; i < 3; ++i)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(pp[i]) : "v"(x1par), "n"(i * 1024));
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(rv) : "v"(raddr), "n"(S * kW2RSlot + 64 * HF));
    stream(S_, C0{}, T{}, op, xlo, xhi);   // first transposed windows of block b: in flight under the arithmetic
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(pp[0]), "+v"(pp[1]), "+v"(pp[2]), "+v"(rv) : "n"(2 * (kW2Window + 1)));
    if (b == nb - 1) {   // rows past N were read from row N-1: give them r = 0
      asm volatile("" ::: "memory");   // (a real branch: the last block only)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (b * 32 + 16 * HF + 4 * gq + v >= N) rv[v] = 0.f;
    }
    float Aw[4], Dn[4], Dm[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float m = M[HF][v] + pp[0][v], n = Nn[HF][v] + pp[1][v], d = Ad[HF][v] + pp[2][v];
      const float e = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * m);
      const float sg = __builtin_amdgcn_rcpf(1.0f + e);
      const float sw = rv[v] * sg;
      const float x = (1.0f + m) - m * sg;   // silu'(m) = sg (1 + m - silu(m))
      const float pw = m * sw;
      Aw[v] = pw * n;
      Dn[v] = pw * d;
      Dm[v] = ((n * sw) * x) * d;
    }
    const u32x2 pa_o = {pack_bf16(Aw[0], Aw[1]), pack_bf16(Aw[2], Aw[3])};
    const u32x2 pm_o = {pack_bf16(Dm[0], Dm[1]), pack_bf16(Dm[2], Dm[3])};
    const u32x2 pn_o = {pack_bf16(Dn[0], Dn[1]), pack_bf16(Dn[2], Dn[3])};
    // exchange 2 (the stores also keep the arithmetic on this side of the barrier)
    *reinterpret_cast<u32x2*>(x2own) = pa_o;
    *reinterpret_cast<u32x2*>(x2own + 128) = pm_o;
    *reinterpret_cast<u32x2*>(x2own + 256) = pn_o;
    // ---- barrier B: packed results written; early waves: their request of a step ago has landed
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (!lag) __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    s16x4 pa_p, pm_p, pn_p;
    asm volatile("ds_read_b64 %0, %1" : "=v"(pa_p) : "v"(x2par));
    asm volatile("ds_read_b64 %0, %1 offset:512" : "=v"(pm_p) : "v"(x2par));
    asm volatile("ds_read_b64 %0, %1 offset:1024" : "=v"(pn_p) : "v"(x2par));
    if (!lag && req) dma(b + 2, S2);
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(pa_p), "+v"(pm_p), "+v"(pn_p));
    // k-slot s = 4t + v of every gradient product is token 16t + 4gq + v
    const s16x4 ao = __builtin_bit_cast(s16x4, pa_o), mo = __builtin_bit_cast(s16x4, pm_o);
    const s16x4 no = __builtin_bit_cast(s16x4, pn_o);
    if constexpr (HF == 0) { agf = join_tr(ao, pa_p); dmf = join_tr(mo, pm_p); dnf = join_tr(no, pn_p); }
    else { agf = join_tr(pa_p, ao); dmf = join_tr(pm_p, mo); dnf = join_tr(pn_p, no); }
  };
  // block b: barrier A, the part above, then the stream of gradient products of b and recompute
  // products of b + 1
  auto step = [&](int64_t b, auto S_) {
    constexpr int S = decltype(S_)::value, S2 = (S + 2) % kW2Stages;
    const bool req = (b + 2 >= b0 + 3) && (b + 2 < b1);   // the first three blocks were requested up front
    // ---- barrier A: partial sums written; late waves: their request of a step ago has landed
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (lag) __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (lag && req) dma(b + 2, S2);
    bf16x8 op[16];
    s16x4 xlo[16], xhi[16];
    if (hf == 0) finish(b, req, S_, C0{}, op, xlo, xhi);
    else finish(b, req, S_, C1{}, op, xlo, xhi);
    // the wave that feeds the MFMA pipe goes first; the other wave's arithmetic fills the gaps
    __builtin_amdgcn_s_setprio(1);
    stream(S_, C0{}, F{}, op, xlo, xhi);
    __builtin_amdgcn_s_setprio(0);
  };
  // Waves w and w + 4 share a SIMD: waves 4-7 pass one barrier more before the loop, waves 0-3
  // one more after it.  Barrier events then alternate between (early waves at A, late at B) and
  // (early at B, late at A).  Block b is last read in the early waves' pass after their B(b)
  // and in the late waves' pass one event later, which ends at the event where the early waves
  // are at B(b+1) and the late ones at A(b+1): both request block b + 3 into its stage right
  // after that event, and wait for that request two events (one step) later, before the
  // event after which block b + 3 is first read.
  if (lag) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
  }
  for (int64_t b = b0; b < b1; b += 3) {
    step(b, C0{});
    if (b + 1 < b1) step(b + 1, C1{});
    if (b + 2 < b1) step(b + 2, C2{});
  }
  // (the last pass has run the recompute products on a block that does not exist)
  if (!lag) __builtin_amdgcn_s_barrier();

  if (active && split) {
    // fp32 partial gradients of this token segment: [seg][K | U | V][split group][block][16][256]
    const size_t rows = (size_t)8 * (a.gpx - a.full_px) * (kW2Blocks * 16);
    float* dst = a.WPws + (((size_t)seg * 3) * rows + ((size_t)cgroup * kW2Blocks + pair) * 16 + cn) * kW2Dh +
                 128 * hf + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) {
      *reinterpret_cast<f32x4*>(dst + 16 * jb) = dK[jb];
      *reinterpret_cast<f32x4*>(dst + rows * kW2Dh + 16 * jb) = dU[jb];
      *reinterpret_cast<f32x4*>(dst + 2 * rows * kW2Dh + 16 * jb) = dV[jb];
    }
  } else if (active) {
    // accumulators are [j][c]: lane = neuron column cn, register v = row 128hf + 16jb + 4gq + v
    const size_t off = (row0 + cn) * kW2Dh + 128 * hf + 4 * gq;
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) {
      const size_t o = off + 16 * jb;
      if (a.dWg) {
        u32x2 pk = {pack_bf16(dK[jb][0], dK[jb][1]), pack_bf16(dK[jb][2], dK[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWg + o) = pk;
      }
      if (a.dWu) {
        u32x2 pk = {pack_bf16(dU[jb][0], dU[jb][1]), pack_bf16(dU[jb][2], dU[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWu + o) = pk;
      }
      if (a.dWd) {
        u32x2 pk = {pack_bf16(dV[jb][0], dV[jb][1]), pack_bf16(dV[jb][2], dV[jb][3])};
        *reinterpret_cast<u32x2*>(a.dWd + o) = pk;
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
// transposing LDS read of a [32 tok][d_h] tile of X, the B operand (contraction
// slot s <-> token 16*t2 + 8*(s/4) + 4g + s%4, column e) comes straight from
// the [H][E][N] dp array.  Each wave walks its own token blocks and leaves its
// own partial [128][E] in the workspace.
template <int DH, int EB>
__global__ __launch_bounds__(256) void bwd_route_partial_kernel(BwdArgs a) {
  constexpr int JB = DH / 32, CPR = DH / 8, kTileBytes = 32 * DH * 2;
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
  f32x16 acc[EB][JB];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) acc[eb][jb] = f32x16{0};

  // Every wave owns its LDS tile and its token blocks: no workgroup barrier is needed, and the
  // loads of the next block are requested before the products of the current one.
  constexpr int XC = 32 * CPR / 64;               // 16-byte chunks of the X tile per lane
  u32x4 xv[XC];
  float dv[EB][2][8];
  auto request = [&](int64_t it) {
    const int64_t tok0 = (it * kRouteParts + part) * 32;   // may lie beyond N: then everything loaded is zero
#pragma unroll
    for (int i = 0; i < XC; ++i) {
      const int chunk = lane + 64 * i;
      const int64_t t = tok0 + chunk / CPR;
      xv[i] = u32x4{0, 0, 0, 0};
      if (t < N) xv[i] = *reinterpret_cast<const u32x4*>(a.X + t * a.ldx + h * DH + (chunk % CPR) * 8);
    }
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) {
      const int e = 32 * eb + r;
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
          const int64_t t = tok0 + 16 * t2 + 8 * (s8 >> 2) + 4 * g + (s8 & 3);
          dv[eb][t2][s8] = (e < E && t < N) ? DPh[(size_t)e * N + t] : 0.f;
        }
    }
  };
  request(0);
  for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < XC; ++i) {
      const int chunk = lane + 64 * i;
      *reinterpret_cast<u32x4*>(tile + btile_off<DH>(chunk / CPR, chunk % CPR)) = xv[i];
    }
    bf16x8 bp[EB][2];
#pragma unroll
    for (int eb = 0; eb < EB; ++eb)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        u32x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) pk[i] = pack_bf16(dv[eb][t2][2 * i], dv[eb][t2][2 * i + 1]);
        bp[eb][t2] = __builtin_bit_cast(bf16x8, pk);
      }
    if (it + 1 < iters) request(it + 1);
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
        const bf16x8 qT = btile_read_tr<DH>(tile, 16 * t2 + 4 * g, 32 * jb, lane);
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) acc[eb][jb] = mfma32(qT, bp[eb][t2], acc[eb][jb]);
      }
    }
  }
  float* out = a.WRws + ((size_t)h * kRouteParts + part) * DH * E;
#pragma unroll
  for (int eb = 0; eb < EB; ++eb) {
    const int e = 32 * eb + r;
    if (e < E) {
#pragma unroll
      for (int jb = 0; jb < JB; ++jb)
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
  const int64_t per_head = (int64_t)a.dh * a.E;
  if (idx >= per_head * a.H) return;
  const int h = (int)(idx / per_head);
  const int64_t o = idx % per_head;
  float sum = 0.f;
  int s = 0;
  for (; s + 8 <= a.n_split; s += 8) {   // eight loads in flight, summed in the order of s
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = a.WRws[((size_t)h * a.n_split + s + i) * per_head + o];
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += v[i];
  }
  for (; s < a.n_split; ++s) sum += a.WRws[((size_t)h * a.n_split + s) * per_head + o];
  reinterpret_cast<uint16_t*>(a.d_route)[idx] = (uint16_t)(pack_bf16(sum, 0.f) & 0xFFFFu);
}

// zero-fill for the N == 0 case (gradients of an empty batch are zero)
__global__ void fill_zero_kernel(uint32_t* p, size_t n_words) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) p[i] = 0;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr int kFullLds = (int)kLdsBytesPerWorkgroup;

constexpr int tok_block_tokens(int dh) { return dh == 128 ? 256 : 128; }

// LDS of the token-major kernel: the weight stages and dr_e of every token of the block
size_t tok_lds_bytes(const Problem& p, bool dma) {
  return (size_t)tok_stages(dma) * tok_stage_bytes(p.dh) +
         (size_t)p.E * tok_block_tokens(p.dh) * sizeof(float);
}
// direct staging (three stages) where it fits: d_h = 128 with up to 88 sub-networks, d_h = 256
// (stages of 48 KB) with up to 32
bool tok_direct_staging(const Problem& p) {
  return (p.dh == 128 || p.dh == 256) && tok_lds_bytes(p, true) <= kLdsBytesPerWorkgroup;
}

template <int DH, int TB, int NW, bool DMA = false, bool PHASED = false, bool PIPE = false>
int launch_tok(const Problem& p, BwdArgs a, hipStream_t stream) {
  constexpr int BM = 32 * TB * NW;
  static_assert(BM == tok_block_tokens(DH), "bwd_bf16_lds_bytes assumes this block size");
  a.n_tiles = (p.N + BM - 1) / BM;
  a.n_items = a.n_tiles * p.H;
  const size_t lds = tok_lds_bytes(p, DMA);
  if (hipError_t e = LdsLimit<&bwd_tok_kernel<DH, TB, NW, DMA, PHASED, PIPE>, kFullLds>::ensure(); e != hipSuccess)
    return (int)e;
  hipLaunchKernelGGL((bwd_tok_kernel<DH, TB, NW, DMA, PHASED, PIPE>), dim3((unsigned)xcd_grid_size(a.n_items)),
                     dim3(64 * NW), lds, stream, a);
  return (int)hipGetLastError();
}

int launch_wgt16(const Problem& p, BwdArgs a, hipStream_t stream) {
  const Wgt16Plan wsp = plan_wgt16(p);
  a.wsplit = wsp.segs;
  a.blocks_per_seg = wsp.blocks_per_seg;
  a.gpx = wsp.gpx;
  a.full_px = wsp.full_px;
  a.n_groups = wsp.n_groups;
  const unsigned grid = 8u * (unsigned)(wsp.full_px + (wsp.gpx - wsp.full_px) * wsp.segs);
  a.n_items = grid;
  if (p.dh == kW2Dh) {
    if (hipError_t e = LdsLimit<&bwd_wgt256_kernel, kFullLds>::ensure(); e != hipSuccess) return (int)e;
    hipLaunchKernelGGL(bwd_wgt256_kernel, dim3(grid), dim3(kW2Threads), kW2LdsBytes, stream, a);
  } else {
    if (hipError_t e = LdsLimit<&bwd_wgt16_kernel, kFullLds>::ensure(); e != hipSuccess) return (int)e;
    hipLaunchKernelGGL(bwd_wgt16_kernel, dim3(grid), dim3(kW16Threads), kW16LdsBytes, stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || wsp.segs == 1) return (int)e;
  const size_t count4 = wsp.crows * p.dh / 4;
  hipLaunchKernelGGL(bwd_wgt16_reduce_kernel, dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0,
                     stream, a, wsp.crows);
  return (int)hipGetLastError();
}

template <int DH, int NW>
int launch_wgt_dh(const Problem& p, BwdArgs a, hipStream_t stream) {
  static_assert(NW == wgt_waves(DH), "plan_wgt_split assumes this workgroup size");
  const int nblk = p.E * p.de / 16;
  const int wg_per_head = (nblk + NW - 1) / NW;
  const WgtSplit wsp = plan_wgt_split(p);
  a.wsplit = wsp.segs;
  a.blocks_per_seg = wsp.blocks_per_seg;
  a.n_items = (int64_t)wg_per_head * p.H * wsp.segs;
  constexpr size_t lds = 2 * 2 * 32 * DH * 2;   // two buffers of a q and a dY tile
  if (hipError_t e = LdsLimit<&bwd_wgt_dh_kernel<DH, NW>, kFullLds>::ensure(); e != hipSuccess) return (int)e;
  hipLaunchKernelGGL((bwd_wgt_dh_kernel<DH, NW>), dim3((unsigned)xcd_grid_size(a.n_items)),
                     dim3(64 * NW), lds, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || wsp.segs == 1) return (int)e;
  const size_t count = (size_t)p.H * p.E * p.de * DH;
  hipLaunchKernelGGL(bwd_wgt_reduce_kernel, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0,
                     stream, a, count);
  return (int)hipGetLastError();
}

int launch_wgt64(const Problem& p, BwdArgs a, hipStream_t stream) {
  static_assert(kW6Waves == wgt_waves(kW6Dh) && 3 * 256 == wgt_slots(kW6Dh), "plan_wgt_split assumes this launch shape");
  const int nblk = p.E * p.de / 16;
  const int wg_per_head = (nblk + kW6Waves - 1) / kW6Waves;
  const WgtSplit wsp = plan_wgt_split(p);
  a.wsplit = wsp.segs;
  a.blocks_per_seg = wsp.blocks_per_seg;
  a.n_items = (int64_t)wg_per_head * p.H * wsp.segs;
  if (hipError_t e = LdsLimit<&bwd_wgt64_kernel, kFullLds>::ensure(); e != hipSuccess) return (int)e;
  hipLaunchKernelGGL(bwd_wgt64_kernel, dim3((unsigned)xcd_grid_size(a.n_items)), dim3(kW6Threads),
                     kW6LdsBytes, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || wsp.segs == 1) return (int)e;
  const size_t count = (size_t)p.H * p.E * p.de * kW6Dh;
  hipLaunchKernelGGL(bwd_wgt_reduce_kernel, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0,
                     stream, a, count);
  return (int)hipGetLastError();
}

template <int DH>
int launch_route(const Problem& p, const BwdArgs& a, hipStream_t stream) {
  const dim3 rgrid(p.H, kRouteSplit);
  if (p.E <= 32) hipLaunchKernelGGL((bwd_route_partial_kernel<DH, 1>), rgrid, dim3(256), 0, stream, a);
  else if (p.E <= 64) hipLaunchKernelGGL((bwd_route_partial_kernel<DH, 2>), rgrid, dim3(256), 0, stream, a);
  else if constexpr (DH <= 128) hipLaunchKernelGGL((bwd_route_partial_kernel<DH, 3>), rgrid, dim3(256), 0, stream, a);
  else return -1;   // excluded by bwd_bf16_max_sub
  const int64_t n = (int64_t)p.H * DH * p.E;
  hipLaunchKernelGGL(bwd_route_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     stream, a);
  return (int)hipGetLastError();
}

}  // namespace

int launch_fill_zero(void* p, size_t bytes, void* stream) {
  const size_t words = bytes / 4;
  if (!p || !words) return 0;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint32_t*>(p), words);
  return (int)hipGetLastError();
}

// d_h = 256: the routing-gradient kernel keeps 8 accumulator tiles per 32 sub-networks
int bwd_bf16_max_sub(const Problem& p) { return p.dh == 256 ? 64 : kRouteMaxSub; }

size_t bwd_bf16_lds_bytes(const Problem& p) { return tok_lds_bytes(p, tok_direct_staging(p)); }

size_t bwd_workspace_bytes(const Problem& p, int dtype) {
  if (dtype != 1) return bwd_f32_workspace_bytes(p);
  if (p.N == 0) return 0;   // an empty batch only zero-fills the weight gradients
  const size_t nhe = align256((size_t)p.N * p.H * p.E * sizeof(float));
  const size_t wr = align256((size_t)p.H * kRouteParts * p.dh * p.E * sizeof(float));
  return 2 * nhe + wr + wgt_split_bytes(p);
}

int launch_bwd(const Problem& p, int dtype, const void* X, const void* Wg, const void* Wu,
               const void* Wd, const void* route, const void* dY, void* dX, void* dWg,
               void* dWu, void* dWd, void* d_route, void* ws, void* stream_,
               void* const* phase_events, int n_phase_events) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // event i is recorded after phase i-1 (event 0: before anything is launched)
  auto mark = [&](int i) -> hipError_t {
    if (i < n_phase_events && phase_events && phase_events[i])
      return hipEventRecord(static_cast<hipEvent_t>(phase_events[i]), stream);
    return hipSuccess;
  };
  if (mark(0) != hipSuccess) return (int)hipErrorInvalidHandle;
  if (dtype != 1) {   // fp32 companion kernels; its phases are not timed separately
    const int e = launch_bwd_f32(p, X, Wg, Wu, Wd, route, dY, dX, dWg, dWu, dWd, d_route, ws, stream_);
    if (e != 0) return e;
    for (int i = 1; i <= kBwdPhases; ++i)
      if (mark(i) != hipSuccess) return (int)hipErrorInvalidHandle;
    return 0;
  }
  if (p.E > bwd_bf16_max_sub(p)) return -1;
  const size_t wcount = (size_t)p.H * p.E * p.de * p.dh;
  if (p.N == 0) {
    void* outs[4] = {dWg, dWu, dWd, p.route_mode == 0 ? d_route : nullptr};
    const size_t words[4] = {wcount / 2, wcount / 2, wcount / 2, (size_t)p.H * p.dh * p.E / 2};
    for (int i = 0; i < 4; ++i) {
      if (!outs[i] || !words[i]) continue;
      hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words[i] + 255) / 256)), dim3(256), 0,
                         stream, static_cast<uint32_t*>(outs[i]), words[i]);
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return (int)e;
    // an empty batch still records every phase event, so that a caller's elapsed-time
    // queries between them succeed
    for (int i = 1; i <= kBwdPhases; ++i)
      if (mark(i) != hipSuccess) return (int)hipErrorInvalidHandle;
    return 0;
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
  a.WPws = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + 2 * nhe +
                                    align256((size_t)p.H * kRouteParts * p.dh * p.E * sizeof(float)));
  a.wsplit = 1;
  a.blocks_per_seg = (p.N + 31) / 32;
  a.gpx = 0; a.full_px = 0; a.n_groups = 0;
  a.N = p.N; a.ldx = p.ldx; a.ldy = p.ldy;
  a.H = p.H; a.E = p.E; a.de = p.de; a.dh = p.dh; a.route_mode = p.route_mode; a.eps = p.eps;
  a.n_split = kRouteParts;

  // token-major kernel (always: it also produces R for the weight-major kernel)
  int rc;
  // d_h = 64: workgroups of 4 waves, two or three of them per CU in different phases of
  // their steps (measured 4 % and 11 % faster than one workgroup of 8 waves)
  if (p.dh == 64) rc = launch_tok<64, 1, 4>(p, a, stream);
  else if (p.dh == 256 && tok_direct_staging(p)) rc = launch_tok<256, 1, 4, true, false, true>(p, a, stream);
  else if (p.dh == 256) rc = launch_tok<256, 1, 4>(p, a, stream);   // needs one wave per SIMD: see the kernel
  else if (tok_direct_staging(p)) rc = launch_tok<kDh, 1, 8, true, true>(p, a, stream);
  else rc = launch_tok<kDh, 1, 8>(p, a, stream);
  if (rc) return rc;
  if (mark(1) != hipSuccess) return (int)hipErrorInvalidHandle;
  if (dWg || dWu || dWd) {
    if (p.dh == 64 && p.ldx < ((int64_t)1 << 24) && p.ldy < ((int64_t)1 << 24)) rc = launch_wgt64(p, a, stream);
    else if (p.dh == 64) rc = launch_wgt_dh<64, 4>(p, a, stream);
    else if (p.dh == 256 && !wgt256_takes(p)) rc = launch_wgt_dh<256, 4>(p, a, stream);
    else rc = launch_wgt16(p, a, stream);   // d_h = 128 and 256
    if (rc) return rc;
  }
  if (mark(2) != hipSuccess) return (int)hipErrorInvalidHandle;
  if (d_route && p.route_mode == 0) {
    if (p.dh == 64) rc = launch_route<64>(p, a, stream);
    else if (p.dh == 256) rc = launch_route<256>(p, a, stream);
    else rc = launch_route<kDh>(p, a, stream);
    if (rc) return rc;
  }
  if (mark(3) != hipSuccess) return (int)hipErrorInvalidHandle;
  return 0;
}

}  // namespace mhffn
