// Fused Multi-Head FFN forward, bf16 storage / fp32 accumulation, gfx950.
//
// One workgroup owns BM tokens of one head and walks the head's whole
// intermediate dimension in tiles of 32 neurons (the block loop of
// eq:flash-ffn-loop; appendix algorithm "SRAMFFN-Forward"):
//
//   per tile:  M^T = K_tile q^T,  N^T = U_tile q^T          (bf16 MFMA, fp32 acc)
//              A^T = SiLU(M^T) .* N^T .* r_e                 (fp32 VALU, one bf16 rounding)
//              O^T += V_tile^T A^T                           (bf16 MFMA, fp32 acc)
//
// Products are kept transposed (neurons on the MFMA row axis, tokens on the
// column axis): the fp32 accumulator of M^T/N^T then has exactly the lane
// layout of a B operand of the third product, so A never leaves registers.
// V is read from LDS with the transposing LDS load, so all three weight tiles
// are staged in their natural [neuron][d_h] layout.
//
// The gating weights of eq:routing are computed in the same kernel (P^T = W_r^T
// q^T on the MFMA, sigmoid and the sum over sub-networks in fp32, the two
// half-waves of a token combined with one cross-lane exchange) and parked in
// LDS as 1/R[e][token]; nothing but X, the weights and Y touches device memory.
#include "mhffn_device.h"
#include "mhffn_internal.h"

#include <type_traits>

namespace mhffn {
namespace {

constexpr int kDh = 128;            // head width this kernel is built for
constexpr int kBI = 32;             // neurons per tile
// fwd_bf16_kernel<DH, ..>: LDS rows of a K/U tile carry 16 bytes of padding (row-wise
// operand reads), rows of a V tile 64 (transposing reads); 27648 bytes per stage at d_h = 128
constexpr int fwd_ku_stride(int dh) { return 2 * dh + 16; }
constexpr int fwd_v_stride(int dh) { return 2 * dh + 64; }
constexpr int fwd_stage_bytes(int dh) { return kBI * (2 * fwd_ku_stride(dh) + fwd_v_stride(dh)); }
constexpr int kStages = 2;

// LDS keeps 1/r (clamped, so r = 0 stays finite): the weight then rides along in the
// sigmoid's own reciprocal and costs no multiply of its own,
//   SiLU(m) n r = m n r / (1 + 2^(-m log2 e)) = m n * rcp((1 + t) / r),   (1 + t)/r = fma(t, 1/r, 1/r)
// four full-rate and two transcendental VALU instructions per element.
__device__ __forceinline__ float inv_weight(float r) {
  const float v = __builtin_amdgcn_rcpf(r);   // 1 ulp; a full-precision division is ten instructions
  return fminf(fmaxf(v, -1e30f), 1e30f);
}
#define MHFFN_SB() __builtin_amdgcn_sched_barrier(0)

struct FwdArgs {
  const uint16_t* X;
  const uint16_t* Wg;
  const uint16_t* Wu;
  const uint16_t* Wd;
  const void* route;
  uint16_t* Y;
  float* P;     // [n_split][N][H*128] fp32 partial outputs (only when n_split > 1)
  int64_t N, ldx, ldy, n_tiles, n_items;
  int H, E, de, dh, route_mode;
  int n_split, tiles_per_split;
  float eps;
};

template <int DH, int TB, int NW>
__global__ __launch_bounds__(64 * NW, NW == 2 ? 2 : 1) void fwd_bf16_kernel(FwdArgs a) {
  constexpr int BM = 32 * TB * NW;
  constexpr int THREADS = 64 * NW;
  constexpr int KS = DH / 16;                  // contraction steps over the head width
  constexpr int JB = DH / 32;                  // 32-row output tiles over the head width
  constexpr int CPR = DH / 8;                  // 16-byte chunks per weight row
  constexpr int kKUStride = fwd_ku_stride(DH), kVStride = fwd_v_stride(DH);
  constexpr int kKBytes = kBI * kKUStride, kStageBytes = fwd_stage_bytes(DH);
  constexpr int CHUNKS = kBI * CPR;            // 16-byte chunks per tile
  constexpr int CH = (CHUNKS + THREADS - 1) / THREADS;   // per thread
  constexpr bool kAllLoad = (CHUNKS % THREADS == 0);     // else the upper threads carry none
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* stage_base = smem;
  float* Rs = reinterpret_cast<float*>(smem + kStages * kStageBytes);  // [E][BM]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;  // whole workgroup leaves together
  // item = (head * n_tiles + token tile) * n_split + split: the splits of one
  // token tile sit next to each other and share the head's weights in L2
  const int split = (int)(item % a.n_split);
  const int64_t ht = item / a.n_split;
  const int h = (int)(ht / a.n_tiles);
  const int64_t tile_tok0 = (ht % a.n_tiles) * BM;
  const int wtok = wave * 32 * TB;  // first token of this wave inside the tile
  const int E = a.E;

  // ---- q fragments (B operands), resident for the whole kernel -------------
  bf16x8 q[TB][KS];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    const int64_t tok = tile_tok0 + wtok + 32 * tb + r;
    const bool valid = tok < a.N;
    const uint16_t* src = a.X + (valid ? tok : 0) * a.ldx + h * DH + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
      if (!valid) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      q[tb][ks] = v;
    }
  }

  // ---- weight-tile stream: global -> registers -> LDS, two tiles in flight ----
  const int tiles_per_sub = a.de / kBI;
  const int T_all = E * tiles_per_sub;
  const int t_begin = split * a.tiles_per_split;          // this workgroup's share of the
  const int T = min(T_all, t_begin + a.tiles_per_split);   // intermediate dimension
  const size_t head_off = (size_t)h * E * a.de * DH;
  const uint16_t* Kh = a.Wg + head_off;
  const uint16_t* Uh = a.Wu + head_off;
  const uint16_t* Vh = a.Wd + head_off;

  // Two register sets: while tile t is being consumed from LDS, tile t+1 sits in one
  // set (to be stored at the end of the step) and the loads of tile t+2 are already
  // in flight into the other.  The first two tiles are requested before the gating
  // phase, so their memory latency hides behind it.
  u32x4 kreg[2][CH], ureg[2][CH], vreg[2][CH];
  auto gload = [&](int t, auto S) {
    constexpr int s = decltype(S)::value;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int chunk = tid + THREADS * i;
      if (!kAllLoad && chunk >= CHUNKS) continue;
      const size_t off = ((size_t)t * kBI + chunk / CPR) * DH + (chunk % CPR) * 8;
      kreg[s][i] = *reinterpret_cast<const u32x4*>(Kh + off);
      ureg[s][i] = *reinterpret_cast<const u32x4*>(Uh + off);
      vreg[s][i] = *reinterpret_cast<const u32x4*>(Vh + off);
    }
  };
  auto lstore = [&](int stage, auto S) {
    constexpr int s = decltype(S)::value;
    unsigned char* st = stage_base + stage * kStageBytes;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int chunk = tid + THREADS * i;
      if (!kAllLoad && chunk >= CHUNKS) continue;
      const int row = chunk / CPR, c16 = chunk % CPR;
      *reinterpret_cast<u32x4*>(st + row * kKUStride + c16 * 16) = kreg[s][i];
      *reinterpret_cast<u32x4*>(st + kKBytes + row * kKUStride + c16 * 16) = ureg[s][i];
      *reinterpret_cast<u32x4*>(st + 2 * kKBytes + row * kVStride + c16 * 16) = vreg[s][i];
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  gload(t_begin, S0{});
  if (t_begin + 1 < T) gload(t_begin + 1, S1{});

  // ---- gating weights R[e][token] into LDS ---------------------------------
  if (a.route_mode == 0) {
    const int EB = (E + 31) >> 5;
    uint16_t* WrT = reinterpret_cast<uint16_t*>(stage_base);  // [32*EB][136] bf16
    const uint16_t* Wr = reinterpret_cast<const uint16_t*>(a.route) + (size_t)h * DH * E;
    for (int idx = tid; idx < DH * E; idx += THREADS) {
      const int j = idx / E, e = idx - j * E;
      WrT[e * (kKUStride / 2) + j] = Wr[idx];
    }
    for (int idx = tid; idx < (32 * EB - E) * DH; idx += THREADS) {
      const int e = E + idx / DH, j = idx % DH;
      WrT[e * (kKUStride / 2) + j] = 0;
    }
    __syncthreads();
    float zsum[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) zsum[tb] = 0.f;
    // pass 0 accumulates Z = sum_e sigmoid(p_e); pass 1 recomputes and writes r_e.
    float inv[TB];
    for (int pass = 0; pass < 2; ++pass) {
      for (int eb = 0; eb < EB; ++eb) {
        const unsigned char* arow =
            reinterpret_cast<const unsigned char*>(WrT) + (32 * eb + r) * kKUStride + 16 * g;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          f32x16 acc = {0};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            bf16x8 af = *reinterpret_cast<const bf16x8*>(arow + 32 * ks);
            acc = mfma32(af, q[tb][ks], acc);
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int e = 32 * eb + 8 * (v / 4) + 4 * g + (v % 4);
            const float s = (e < E) ? sigmoid_fast(acc[v]) : 0.f;
            if (pass == 0) {
              zsum[tb] += s;
            } else if (e < E) {
              Rs[e * BM + wtok + 32 * tb + r] = inv_weight(s * inv[tb]);
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
      const int64_t tok = tile_tok0 + tl;
      Rs[e * BM + tl] = inv_weight((tok < a.N) ? R[((size_t)tok * a.H + h) * E + e] : 0.f);
    }
  }
  __syncthreads();  // R complete; the staging area is free again

  f32x16 O[TB][JB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) O[tb][jb] = f32x16{0};

  // per-lane byte offsets of the operand reads inside a stage
  const int ku_off = r * kKUStride + 16 * g;
  // transposing V read: 16-lane block b = lane/16 serves rows 4*(b/2).. and columns 16*(b%2)..
  const int li = lane & 15;
  const int v_off = 2 * kKBytes + (4 * g + (li >> 2)) * kVStride + (16 * ((lane >> 4) & 1) + 4 * (li & 3)) * 2;

  // ---- main loop over tiles of 32 neurons ----------------------------------
  lstore(0, S0{});
  __syncthreads();
  float rw[TB];
  // one tile: its data is in LDS stage (t - t_begin) & 1; SL = register set that is free
  // (receives tile t+2), SS = register set holding tile t+1 (stored at the end)
  auto tile_step = [&](int t, auto SL, auto SS) {
    if (t + 2 < T) gload(t + 2, SL);
    if (t % tiles_per_sub == 0 || t == t_begin) {
      const int e = t / tiles_per_sub;
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) rw[tb] = Rs[e * BM + wtok + 32 * tb + r];
    }
    const unsigned char* st = stage_base + ((t - t_begin) & 1) * kStageBytes;

    // gate and up products
    f32x16 accM[TB], accN[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) { accM[tb] = f32x16{0}; accN[tb] = f32x16{0}; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 ak = *reinterpret_cast<const bf16x8*>(st + ku_off + 32 * ks);
      const bf16x8 au = *reinterpret_cast<const bf16x8*>(st + kKBytes + ku_off + 32 * ks);
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        accM[tb] = mfma32(ak, q[tb][ks], accM[tb]);
        accN[tb] = mfma32(au, q[tb][ks], accN[tb]);
      }
    }
    // activation, weighting, one rounding to bf16; registers 8*t2 .. 8*t2+7 of
    // the accumulator are the 8 contraction slots of down-projection step t2.
    bf16x8 bfrag[TB][2];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        // eight elements at a time, each step for all eight before the next step:
        // dependent VALU instructions (exp -> fma -> rcp -> mul) end up eight issue
        // slots apart instead of back to back
        float t[8], s[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * accM[tb][8 * t2 + i]);
        MHFFN_SB();
#pragma unroll
        for (int i = 0; i < 8; ++i) s[i] = __builtin_amdgcn_rcpf(__builtin_fmaf(t[i], rw[tb], rw[tb]));
        MHFFN_SB();
        u32x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float a0 = (accM[tb][8 * t2 + 2 * i] * accN[tb][8 * t2 + 2 * i]) * s[2 * i];
          const float a1 = (accM[tb][8 * t2 + 2 * i + 1] * accN[tb][8 * t2 + 2 * i + 1]) * s[2 * i + 1];
          pk[i] = pack_bf16(a0, a1);
        }
        bfrag[tb][t2] = __builtin_bit_cast(bf16x8, pk);
      }
    }
    // down projection: contraction slot s of step t2 is neuron
    // 16*t2 + 8*(s/4) + 4g + s%4, so the V operand is two transposed reads of
    // 4 consecutive tile rows each.
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
        const unsigned char* vp = st + v_off + (16 * t2) * kVStride + 64 * jb;
        const s16x4 lo = lds_read_tr16(vp);
        const s16x4 hi = lds_read_tr16(vp + 8 * kVStride);
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 av = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) O[tb][jb] = mfma32(av, bfrag[tb][t2], O[tb][jb]);
      }
    }
    if (t + 1 < T) lstore((t + 1 - t_begin) & 1, SS);
    __syncthreads();
  };
  for (int t = t_begin; t < T; t += 2) {
    tile_step(t, S0{}, S1{});
    if (t + 1 < T) tile_step(t + 1, S1{}, S0{});
  }

  // ---- split runs leave an fp32 partial; fwd_bf16_reduce_kernel sums them ---
  if (a.n_split > 1) {
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int64_t tok = tile_tok0 + wtok + 32 * tb + r;
      if (tok < a.N) {
        float* dst = a.P + (((size_t)split * a.N + tok) * a.H + h) * DH + 4 * g;
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            f32x4 o = {O[tb][jb][4 * vq], O[tb][jb][4 * vq + 1], O[tb][jb][4 * vq + 2],
                       O[tb][jb][4 * vq + 3]};
            *reinterpret_cast<f32x4*>(dst + 32 * jb + 8 * vq) = o;
          }
      }
    }
    return;
  }
  // ---- store Y (concat_H: head h owns columns h*d_h ..) --------------------
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    const int64_t tok = tile_tok0 + wtok + 32 * tb + r;
    if (tok < a.N) {
      uint16_t* dst = a.Y + tok * a.ldy + h * DH + 4 * g;
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          u32x2 pk;
          pk[0] = pack_bf16(O[tb][jb][4 * vq], O[tb][jb][4 * vq + 1]);
          pk[1] = pack_bf16(O[tb][jb][4 * vq + 2], O[tb][jb][4 * vq + 3]);
          *reinterpret_cast<u32x2*>(dst + 32 * jb + 8 * vq) = pk;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Pipelined kernel for up to 64 sub-networks at d_h = 128 (256 tokens per workgroup, 8 waves
// of 32 tokens, two waves per SIMD).  Same arithmetic and tiling as fwd_bf16_kernel; what
// differs is how a wave's instruction stream is laid out, because that, not the MFMA rate,
// bounds the kernel:
//   * weight tiles go global -> LDS directly (one 1 KB image of four swizzled rows per
//     wave-wide load) into three rings of four stages (K | U | V): staging costs no
//     registers, no LDS-store instructions and no wait inside the step;
//   * the issue port that MFMA and VALU instructions share is the scarce resource: a
//     32x32x16 product holds it for about 20 of its 32 cycles, a plain VALU instruction for
//     about 3, a transcendental one for about 8, and one wave issues at most one
//     instruction every 5 cycles.  Four to five VALU instructions behind every product are
//     therefore almost free, while a run of products with nothing between them, or a run of
//     arithmetic with few products, leaves one of the two pipes idle.  So a step works on
//     three tiles at once:
//         gate/up products of tile i+1 | activation of tile i | down projection of tile i-1
//     in 12 slots of two products and eight to nine VALU instructions each (slot pattern:
//     gate+up, gate+up, down+down).  The activation of an element pair runs in three stages
//     (A: 2^(-m log2 e) and m*n;  B: rcp((1+t)/r);  C: product and rounding) that sit one to
//     two slots apart, the last ones of a tile in the first slots of the next step;
//   * LDS operands are read two slots ahead into three rotating register sets, untracked,
//     with counted waits, and the stream of reads runs across the step boundary: a K/U tile
//     is published by the barrier two steps before its products (requested four steps
//     ahead), a V tile one step before its down projection (requested two steps ahead);
//   * the loop is unrolled over stage x accumulator set (4 bodies), which makes every LDS
//     operand address an immediate offset from a loop-invariant per-lane register.
// One barrier per step: it publishes the tiles requested one step ago and retires the K/U
// stage of tile i+1 and the V stage of tile i-1.
// ---------------------------------------------------------------------------
constexpr int kPipeStages = 4;
constexpr int kPipeTile = kBI * kDh * 2;            // 8 KB, rows of 256 B, chunks swizzled
constexpr int kPipeRing = kPipeStages * kPipeTile;  // one ring per tensor: K | U | V
constexpr int kPipeWaves = 8;
constexpr int kPipeBM = 32 * kPipeWaves;
constexpr int kPipeMaxSub = (kLdsBytesPerWorkgroup - 3 * kPipeRing) / (kPipeBM * 4);
constexpr int kPipeMaxSubStatic = 64;   // = kPipeMaxSub, as a literal for array bounds
static_assert(kPipeMaxSub == kPipeMaxSubStatic, "gating code is written for up to two blocks of 32");
template <int N, typename T0, typename T1, typename T2, typename T3>
__device__ __forceinline__ void lds_wait4(T0& a, T1& b, T2& c, T3& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}

__global__ __launch_bounds__(64 * kPipeWaves) void fwd_bf16_flow_kernel(FwdArgs a) {
  constexpr int BM = kPipeBM;
  constexpr int THREADS = 64 * kPipeWaves;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* Rs = reinterpret_cast<float*>(smem + 3 * kPipeRing);  // [E][BM], 1/r

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;  // whole workgroup leaves together
  const int split = (int)(item % a.n_split);
  const int64_t ht = item / a.n_split;
  const int h = (int)(ht / a.n_tiles);
  const int64_t tile_tok0 = (ht % a.n_tiles) * BM;
  const int wtok = wave * 32;
  const int E = a.E;
  const bool active = tile_tok0 + wtok < a.N;

  const int tiles_per_sub = a.de / kBI;
  const int t_begin = split * a.tiles_per_split;
  const int T = min(E * tiles_per_sub, t_begin + a.tiles_per_split) - t_begin;
  const size_t head_off = ((size_t)h * E * a.de + (size_t)t_begin * kBI) * kDh;
  const uint16_t* Kh = a.Wg + head_off;
  const uint16_t* Uh = a.Wu + head_off;
  const uint16_t* Vh = a.Wd + head_off;

  // direct global -> LDS staging: wave w moves rows 4w..4w+3 of each tile (lane l lands at LDS chunk position l%16 of row 4w + l/16, so it fetches the global chunk that the swizzle maps there)
  const int drow = 4 * wave + (lane >> 4);
  const unsigned dma_goff = (unsigned)(drow * kDh + (((lane & 15) ^ swz(drow)) << 3));  // elements
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma1 = [&](const uint16_t* base, int t, int ring, int stage) {
    global_to_lds_16B(base + (size_t)t * (kBI * kDh) + dma_goff,
                      smem + ring * kPipeRing + stage * kPipeTile + wave_u * 1024);
  };

  bf16x8 q[8];
  {
    const int64_t tok = tile_tok0 + wtok + r;
    const bool valid = tok < a.N;
    const uint16_t* src = a.X + (valid ? tok : 0) * a.ldx + h * kDh + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
      if (!valid) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      q[ks] = v;
    }
  }
  // first requests: K/U tiles 0..2 and V tiles 0, 1 (stage 3 of every ring is the scratch of
  // the gating phase; K/U tile 3 follows it)
  auto first_requests = [&]() {
#pragma unroll
    for (int t = 0; t < 3; ++t)
      if (t < T) { dma1(Kh, t, 0, t); dma1(Uh, t, 1, t); }
    dma1(Vh, 0, 2, 0);
    if (T > 1) dma1(Vh, 1, 2, 1);
  };

  // ---- gating weights 1/R[e][token] into LDS; scratch: stage 3 of all rings ----
  // (a [96][128] bf16 image needs 24 KB: rows 0-31 in the K ring, 32-63 U, 64-95 V)
  if (a.route_mode == 0) {
    const int EB = (E + 31) >> 5;
    auto wr_off = [&](int e, int chunk) { return (e >> 5) * kPipeRing + 3 * kPipeTile + tile_off(e & 31, chunk); };
    const uint16_t* Wr = reinterpret_cast<const uint16_t*>(a.route) + (size_t)h * kDh * E;
    constexpr int kWrIter = (kDh * kPipeMaxSubStatic / 8 + THREADS - 1) / THREADS;
    u32x4 wv[kWrIter];
#pragma unroll
    for (int it = 0; it < kWrIter; ++it) {
      const int c = tid + it * THREADS;
      wv[it] = u32x4{0, 0, 0, 0};
      if (c < kDh * E / 8) wv[it] = *reinterpret_cast<const u32x4*>(Wr + 8 * c);
    }
    first_requests();
    // (rows E.. of the operand keep whatever the memory held: a row of the product depends on
    // its own row of the operand only, and rows E.. are masked below)
#pragma unroll
    for (int it = 0; it < kWrIter; ++it) {
      const int c = tid + it * THREADS;
      if (c < kDh * E / 8) {
        int j = (8 * c) / E, e = 8 * c - j * E;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint16_t w = (uint16_t)(wv[it][i >> 1] >> (16 * (i & 1)));
          *reinterpret_cast<uint16_t*>(smem + wr_off(e, j >> 3) + (j & 7) * 2) = w;
          if (++e == E) { e = 0; ++j; }
        }
      }
    }
    __syncthreads();
    if (active) {
      f32x16 acc[2] = {f32x16{0}, f32x16{0}};
      bf16x8 af[2][8];
#pragma unroll
      for (int eb = 0; eb < 2; ++eb)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          af[eb][ks] = *reinterpret_cast<const bf16x8*>(smem + wr_off(32 * (eb < EB ? eb : 0) + r, 2 * ks + g));
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        acc[0] = mfma32(af[0][ks], q[ks], acc[0]);
        if (EB > 1) acc[1] = mfma32(af[1][ks], q[ks], acc[1]);
      }
      float sg[2][16];
      float zsum = 0.f;
#pragma unroll
      for (int eb = 0; eb < 2; ++eb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int e = 32 * eb + 8 * (v / 4) + 4 * g + (v % 4);
          sg[eb][v] = (e < E) ? sigmoid_fast(acc[eb][v]) : 0.f;
          zsum += sg[eb][v];
        }
      const float inv = 1.0f / (zsum + __shfl_xor(zsum, 32) + a.eps);
      float* rs_lane = Rs + wtok + r;   // 64 rows are allocated: rows E.. are written and never read
#pragma unroll
      for (int eb = 0; eb < 2; ++eb) {
        if (eb >= EB) break;
#pragma unroll
        for (int v = 0; v < 16; ++v)
          rs_lane[(32 * eb + 8 * (v / 4) + 4 * g + (v % 4)) * BM] = inv_weight(sg[eb][v] * inv);
      }
    }
  } else {
    first_requests();
    const float* R = reinterpret_cast<const float*>(a.route);
    for (int idx = tid; idx < BM * E; idx += THREADS) {
      const int tl = idx / E, e = idx - tl * E;
      const int64_t tok = tile_tok0 + tl;
      Rs[e * BM + tl] = inv_weight((tok < a.N) ? R[((size_t)tok * a.H + h) * E + e] : 0.f);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): the first tiles have landed
  __syncthreads();
  if (T > 3) { dma1(Kh, 3, 0, 3); dma1(Uh, 3, 1, 3); }   // the scratch stage is free now

  // ---- loop-invariant operand addresses (LDS byte addresses) -------------------
  const unsigned lds0 = lds_addr_of(smem);
  unsigned kaddr[8];      // K/U operand of contraction step ks: row r, chunk 2ks+g
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) kaddr[ks] = lds0 + tile_off(r, 2 * ks + g);
  unsigned vaddr[4][2];   // V operand, transposing read: rows 4g + li/4 (+8), 64-byte window jb
  {
    const int li = lane & 15;
    const int row = 4 * g + (li >> 2);
    const int colb = 16 * ((lane >> 4) & 1) + 4 * (li & 3);
    const unsigned vbase = lds0 + 2 * kPipeRing;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      vaddr[jb][0] = vbase + tile_off8(row, 32 * jb + colb);
      vaddr[jb][1] = vbase + tile_off8(row + 8, 32 * jb + colb);
    }
  }
  const unsigned rs_lane = lds_addr_of(Rs) + (unsigned)(wtok + r) * 4;

  f32x16 O[4];
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) O[jb] = f32x16{0};
  f32x16 accM[2], accN[2];
  u32x4 pk[2][2] = {{u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}}, {u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}}};
  float tt[8][2], ss[8][2], mn[8][2];
#pragma unroll
  for (int p = 0; p < 8; ++p) { tt[p][0] = tt[p][1] = 0.f; ss[p][0] = ss[p][1] = 0.f; mn[p][0] = mn[p][1] = 0.f; }
  float rwv[2] = {1.f, 1.f};
  bf16x8 gK[2], gU[2];    // operands of the gate/up slots in flight
  s16x4 dV[4];            // operands of the down slot in flight

  // gate/up products of tile 0 (K/U stage 0), then the operands of the first two slots of
  // step 0 (gate/up steps 0, 1 of tile 1) and 1/r of tile 0
  if (active) {
    bf16x8 ak[8], au[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      ak[ks] = *reinterpret_cast<const bf16x8*>(smem + tile_off(r, 2 * ks + g));
      au[ks] = *reinterpret_cast<const bf16x8*>(smem + kPipeRing + tile_off(r, 2 * ks + g));
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (ks == 0) { accM[0] = mfma32(ak[0], q[0], f32x16{0}); accN[0] = mfma32(au[0], q[0], f32x16{0}); }
      else { accM[0] = mfma32(ak[ks], q[ks], accM[0]); accN[0] = mfma32(au[ks], q[ks], accN[0]); }
    }
  }
  // all waves are through with stage 0 of K/U before step 0 requests tile 4 into it
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0), vmcnt untouched
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // scalar bookkeeping of the sub-network of the *next* tile (for its 1/r)
  int sub_cnt = __builtin_amdgcn_readfirstlane(t_begin % tiles_per_sub);
  unsigned rs_off = (unsigned)__builtin_amdgcn_readfirstlane(t_begin / tiles_per_sub) * (BM * 4);
  if (active) {
    gK[0] = lds_read_b128_untracked<1 * kPipeTile>(kaddr[0]);
    gU[0] = lds_read_b128_untracked<1 * kPipeTile + kPipeRing>(kaddr[0]);
    asm volatile("ds_read_b32 %0, %1" : "=v"(rwv[0]) : "v"(rs_lane + rs_off));
    gK[1] = lds_read_b128_untracked<1 * kPipeTile>(kaddr[1]);
    gU[1] = lds_read_b128_untracked<1 * kPipeTile + kPipeRing>(kaddr[1]);
  }
  const unsigned rs_off_max = (unsigned)(E - 1) * (BM * 4);
  if (++sub_cnt == tiles_per_sub) { sub_cnt = 0; rs_off = min(rs_off + BM * 4, rs_off_max); }

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;

  // step i: tile i has its gate/up accumulators in set P and K/U stage S = i % 4.
  // MODE 0: ordinary step, 1: first step (no tile i-1), 2: the step after the last tile
  // (only the last stages of tile T-1 and its down projection).
  auto step = [&](int i, auto S_, auto P_, auto MODE_) {
    constexpr int S = decltype(S_)::value, P = decltype(P_)::value, Qs = 1 - P;
    constexpr int MODE = decltype(MODE_)::value;
    const bool more_ku = (i + 4 < T), more_v = (i + 2 < T);
    if (more_ku) { dma1(Kh, i + 4, 0, S); dma1(Uh, i + 4, 1, S); }
    if (more_v) dma1(Vh, i + 2, 2, (S + 2) % 4);
    if (active) {
      // activation stages of pair p (registers 2p, 2p+1 of the accumulators), see above
      auto stA1 = [&](auto p_) {
        constexpr int p = decltype(p_)::value;
        tt[p][0] = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * accM[P][2 * p]);
        tt[p][1] = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * accM[P][2 * p + 1]);
      };
      auto stA2 = [&](auto p_) {
        constexpr int p = decltype(p_)::value;
        mn[p][0] = accM[P][2 * p] * accN[P][2 * p];
        mn[p][1] = accM[P][2 * p + 1] * accN[P][2 * p + 1];
      };
      auto stB = [&](auto p_, float rw) {
        constexpr int p = decltype(p_)::value;
        ss[p][0] = __builtin_amdgcn_rcpf(__builtin_fmaf(tt[p][0], rw, rw));
        ss[p][1] = __builtin_amdgcn_rcpf(__builtin_fmaf(tt[p][1], rw, rw));
      };
      auto stC = [&](auto p_, auto set_) {
        constexpr int p = decltype(p_)::value, set = decltype(set_)::value;
        pk[set][p >> 2][p & 3] = pack_bf16(mn[p][0] * ss[p][0], mn[p][1] * ss[p][1]);
      };
      auto slot = [&](auto s_) {
        constexpr int s = decltype(s_)::value;
        constexpr int k = s / 3, ph = s % 3;
        // ---- operands of slot s+2 ----
        // (the step after the last tile requests nothing for a step that never comes: a
        // register whose read is never waited for could be handed out again too early)
        constexpr int ts = (s + 2) % 12, so = (s + 2) / 12;
        if constexpr (MODE == 2 && so == 1) {
        } else if constexpr (ts % 3 != 2) {
          constexpr int ks = 2 * (ts / 3) + ts % 3;
          constexpr int off = ((S + 1 + so) % 4) * kPipeTile;
          gK[ts % 3] = lds_read_b128_untracked<off>(kaddr[ks]);
          gU[ts % 3] = lds_read_b128_untracked<off + kPipeRing>(kaddr[ks]);
        } else {
          constexpr int d0 = 2 * (ts / 3), t2 = d0 / 4, jb0 = d0 % 4;
          constexpr int off = ((S + 3 + so) % 4) * kPipeTile + t2 * 4096;
          dV[0] = lds_read_tr16_untracked<off>(vaddr[jb0][0]);
          dV[1] = lds_read_tr16_untracked<off>(vaddr[jb0][1]);
          dV[2] = lds_read_tr16_untracked<off>(vaddr[jb0 + 1][0]);
          dV[3] = lds_read_tr16_untracked<off>(vaddr[jb0 + 1][1]);
        }
        if constexpr (s == 10 && MODE != 2)   // 1/r of tile i+1 (set Qs)
          asm volatile("ds_read_b32 %0, %1" : "=v"(rwv[Qs]) : "v"(rs_lane + rs_off));
        // ---- wait for this slot's operands: all but the reads issued in slots s-1 and s ----
        constexpr int n_issued[12] = {4, 2, 2, 4, 2, 2, 4, 2, 2, 4, MODE == 2 ? 0 : 3, MODE == 2 ? 0 : 2};
        constexpr int n_before = (s == 0) ? 2 : n_issued[(s + 11) % 12];   // slot 11 of the step before
        constexpr int nwait = n_before + n_issued[s];
        if constexpr (ph != 2) {
          constexpr int ks = 2 * k + ph;
          lds_wait<nwait>(gK[ph], gU[ph]);
          if constexpr (s == 0) asm volatile("" : "+v"(rwv[P]));   // read in slot 10 of the last step
          if constexpr (MODE != 2) {
            if constexpr (ks == 0) accM[Qs] = mfma32(gK[ph], q[0], f32x16{0});
            else accM[Qs] = mfma32(gK[ph], q[ks], accM[Qs]);
          }
          MHFFN_SB();
          if constexpr (ph == 0) { if constexpr (MODE != 2) stA1(std::integral_constant<int, 2 * k>{}); }
          else {
            if constexpr (k == 0) stB(std::integral_constant<int, 7>{}, rwv[Qs]);
            else if constexpr (MODE != 2) stB(std::integral_constant<int, (2 * k + 7) % 8>{}, rwv[P]);
          }
          MHFFN_SB();
          if constexpr (MODE != 2) {
            if constexpr (ks == 0) accN[Qs] = mfma32(gU[ph], q[0], f32x16{0});
            else accN[Qs] = mfma32(gU[ph], q[ks], accN[Qs]);
          }
          MHFFN_SB();
          if constexpr (ph == 0) {
            if constexpr (k == 0) stC(std::integral_constant<int, 6>{}, std::integral_constant<int, Qs>{});
            else if constexpr (MODE != 2) stC(std::integral_constant<int, 2 * k - 2>{}, std::integral_constant<int, P>{});
            if constexpr (MODE != 2) stA2(std::integral_constant<int, 2 * k>{});
          } else {
            if constexpr (MODE != 2) stA1(std::integral_constant<int, 2 * k + 1>{});
          }
          MHFFN_SB();
        } else {
          constexpr int d0 = 2 * k, t2 = d0 / 4, jb0 = d0 % 4;
          lds_wait4<nwait>(dV[0], dV[1], dV[2], dV[3]);
          const bf16x8 b = __builtin_bit_cast(bf16x8, pk[Qs][t2]);
          if constexpr (MODE != 1) O[jb0] = mfma32(join_tr(dV[0], dV[1]), b, O[jb0]);
          MHFFN_SB();
          if constexpr (MODE != 2) stB(std::integral_constant<int, 2 * k>{}, rwv[P]);
          MHFFN_SB();
          if constexpr (MODE != 1) O[jb0 + 1] = mfma32(join_tr(dV[2], dV[3]), b, O[jb0 + 1]);
          MHFFN_SB();
          if constexpr (k == 0) stC(std::integral_constant<int, 7>{}, std::integral_constant<int, Qs>{});
          else if constexpr (MODE != 2) stC(std::integral_constant<int, 2 * k - 1>{}, std::integral_constant<int, P>{});
          if constexpr (MODE != 2) stA2(std::integral_constant<int, 2 * k + 1>{});
          MHFFN_SB();
        }
      };
      slot(std::integral_constant<int, 0>{});
      slot(std::integral_constant<int, 1>{});
      slot(std::integral_constant<int, 2>{});
      slot(std::integral_constant<int, 3>{});
      slot(std::integral_constant<int, 4>{});
      slot(std::integral_constant<int, 5>{});
      slot(std::integral_constant<int, 6>{});
      slot(std::integral_constant<int, 7>{});
      slot(std::integral_constant<int, 8>{});
      slot(std::integral_constant<int, 9>{});
      slot(std::integral_constant<int, 10>{});
      slot(std::integral_constant<int, 11>{});
    }
    if (++sub_cnt == tiles_per_sub) { sub_cnt = 0; rs_off = min(rs_off + BM * 4, rs_off_max); }
    // Publish what was requested one step ago (K/U tile i+3, V tile i+1; this step's own
    // requests may stay in flight) and retire K/U stage S+1 and V stage S+3.  The LDS reads
    // in flight belong to the next step's first slots and to stages that stay.
    asm volatile("" ::: "memory");
    if (more_ku) __builtin_amdgcn_s_waitcnt(0x0f73);       // vmcnt(3), lgkmcnt untouched
    else if (more_v) __builtin_amdgcn_s_waitcnt(0x0f71);   // vmcnt(1)
    else __builtin_amdgcn_s_waitcnt(0x0f70);               // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  step(0, I0{}, I0{}, I1{});
  for (int i = 1; i < T; i += 4) {
    step(i, I1{}, I1{}, I0{});
    if (i + 1 < T) step(i + 1, I2{}, I0{}, I0{});
    if (i + 2 < T) step(i + 2, I3{}, I1{}, I0{});
    if (i + 3 < T) step(i + 3, I0{}, I0{}, I0{});
  }
  // the step after the last tile: the remaining stages of tile T-1 and its down projection
  switch (T & 3) {
    case 0: step(T, I0{}, I0{}, I2{}); break;
    case 1: step(T, I1{}, I1{}, I2{}); break;
    case 2: step(T, I2{}, I0{}, I2{}); break;
    default: step(T, I3{}, I1{}, I2{}); break;
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the reads issued for a step that never comes

  const int64_t tok = tile_tok0 + wtok + r;
  if (a.n_split > 1) {
    if (tok < a.N) {
      float* dst = a.P + (((size_t)split * a.N + tok) * a.H + h) * kDh + 4 * g;
#pragma unroll
      for (int jb = 0; jb < 4; ++jb)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          f32x4 o = {O[jb][4 * vq], O[jb][4 * vq + 1], O[jb][4 * vq + 2], O[jb][4 * vq + 3]};
          *reinterpret_cast<f32x4*>(dst + 32 * jb + 8 * vq) = o;
        }
    }
    return;
  }
  if (tok < a.N) {
    uint16_t* dst = a.Y + tok * a.ldy + h * kDh + 4 * g;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        u32x2 pkw;
        pkw[0] = pack_bf16(O[jb][4 * vq], O[jb][4 * vq + 1]);
        pkw[1] = pack_bf16(O[jb][4 * vq + 2], O[jb][4 * vq + 3]);
        *reinterpret_cast<u32x2*>(dst + 32 * jb + 8 * vq) = pkw;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Decode-sized inputs at d_h = 128 (at most 32 * NB tokens, NB in {1, 2, 4}): the launch is a
// weight-streaming problem (every weight byte is used once by a handful of tokens) and its
// floor is the time the memory system needs to deliver the weights.  About one workgroup
// per CU takes one head and a contiguous share of its tiles.  A wave that asks for more
// bytes than its CU may have in flight is held at the load instruction until older requests
// return, so a wave that both requests and computes does neither for most of the time;
// here the two are different waves:
//   * waves 4-7 only move weights: plain coalesced 16-byte loads into two register sets of
//     two tiles each (96 KB per CU in flight, re-requested set by set: the registers, not
//     LDS stages, hold the bytes in flight; more sets in flight were measured and are no
//     faster), each set stored into its own LDS buffer when it has arrived;
//   * waves 0-3 (one per SIMD, beside one loading wave) compute: token block = wave % NB,
//     tile group = wave / NB; a wave takes the tiles of the buffer that belong to its group
//     while the loading waves fill the other buffer; one workgroup barrier per buffer;
//   * the per-group partial outputs are summed through LDS in the fixed order of the groups
//     by all 512 threads, which also store them.
// Arithmetic, lane layouts and the swizzled tile image are those of the kernels above.
// ---------------------------------------------------------------------------
constexpr int kDecodeTile = 3 * kPipeTile;           // K | U | V image of one tile, 24 KB
constexpr int kDecodeThreads = 512;
constexpr int kDecodeBuf = 2 * kDecodeTile;          // one LDS buffer: two tiles
constexpr int kDecodeSetTiles = 2;                   // tiles per register set (one buffer's worth)
constexpr int kDecodeRegSets = 2;                    // register sets of the loading waves: 96 KB per CU in flight
// LDS: two buffers | 1/r [64][32 NB] fp32 | token rows [NB][32][128] bf16
constexpr int decode_lds_bytes(int nb) { return 2 * kDecodeBuf + kPipeMaxSubStatic * 32 * nb * 4 + nb * kPipeTile; }
static_assert(decode_lds_bytes(4) <= (int)kLdsBytesPerWorkgroup, "decode kernel LDS");

template <int NB>
__global__ __launch_bounds__(kDecodeThreads) void fwd_bf16_decode_kernel(FwdArgs a) {
  constexpr int NG = 4 / NB;                         // tile groups among the four computing waves
  constexpr int BT = 32 * NB;                        // token slots of the workgroup
  constexpr int CT = 256;                            // threads of either role
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* buf0 = smem;
  unsigned char* buf1 = smem + kDecodeBuf;
  float* Rs = reinterpret_cast<float*>(smem + 2 * kDecodeBuf);         // [64][BT], 1/r
  unsigned char* Qs = smem + 2 * kDecodeBuf + kPipeMaxSubStatic * BT * 4;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int item = (int)xcd_work_item(blockIdx.x, a.n_items);
  if (item >= (int)a.n_items) return;  // whole workgroup leaves together
  const int split = item % a.n_split;
  const int h = item / a.n_split;
  const int E = a.E;
  const bool loader = wave >= 4;
  const int rt = tid & (CT - 1);                     // thread index inside its role
  const int tb = wave % NB, grp = (wave & 3) / NB;   // computing waves: token block, tile group
  const int tiles_per_sub = a.de / kBI;
  const int t_begin = split * a.tiles_per_split;
  const int T = min(E * tiles_per_sub, t_begin + a.tiles_per_split) - t_begin;
  const int n_sets = (T + kDecodeSetTiles - 1) / kDecodeSetTiles;
  // Two sets per round, every round alike (a round that skipped its second set would leave
  // the number of loads between two uses of a register set unknown to the compiler, and its
  // waits would drain the whole stream): an odd number of sets is preceded by an empty set
  // -1, copies of tile 0 that are stored and never used.
  const int s_first = -(n_sets & 1);
  const size_t head_off = ((size_t)h * E * a.de + (size_t)t_begin * kBI) * kDh;
  const uint16_t* Kh = a.Wg + head_off;
  const uint16_t* Uh = a.Wu + head_off;
  const uint16_t* Vh = a.Wd + head_off;

  // ---- loading waves: thread = chunks (row rt/16 and rt/16 + 16, chunk rt%16) of every
  // tile.  Requests are unconditional (a tile index outside the share is clamped and the
  // copy is never used), so the number of loads in flight behind a set is a constant.
  const int srow = rt >> 4, schunk = rt & 15;
  const unsigned s_goff = (unsigned)(srow * kDh + schunk * 8);          // elements inside a tile
  const int s_loff = tile_off(srow, schunk);                            // bytes; row + 16: + 4096
  u32x4 st[kDecodeRegSets][kDecodeSetTiles][6];
  auto request = [&](int s, auto S_) {
    constexpr int S = decltype(S_)::value;
#pragma unroll
    for (int j = 0; j < kDecodeSetTiles; ++j) {
      const unsigned off = (unsigned)min(max(s * kDecodeSetTiles + j, 0), T - 1) * (kBI * kDh) + s_goff;
      st[S][j][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Kh + off));
      st[S][j][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Kh + off + 16 * kDh));
      st[S][j][2] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Uh + off));
      st[S][j][3] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Uh + off + 16 * kDh));
      st[S][j][4] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Vh + off));
      st[S][j][5] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Vh + off + 16 * kDh));
    }
  };
  auto store_set = [&](auto S_, unsigned char* buf) {
    constexpr int S = decltype(S_)::value;
#pragma unroll
    for (int jj = 0; jj < kDecodeSetTiles; ++jj) {
      unsigned char* slot = buf + jj * kDecodeTile + s_loff;
#pragma unroll
      for (int i = 0; i < 6; ++i)
        *reinterpret_cast<u32x4*>(slot + (i >> 1) * kPipeTile + (i & 1) * 4096) = st[S][jj][i];
    }
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;

  const unsigned char* qrow = Qs + tb * kPipeTile;   // + tile_off(r, 2 ks + g): a lane's operand of step ks
  const int tok = tb * 32 + r;
  f32x16 O[4];
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) O[jb] = f32x16{0};

  // The two roles are two code paths with the same sequence of workgroup barriers: two before
  // the rounds (token rows and gating operand staged | 1/r complete), one per set, one after
  // the last set.  Set s lives in buffer and register set (s - s_first) % 2.  A loading wave
  // stores a set, passes the barrier that hands it over, and only then asks for the set that
  // takes the freed registers: that request is the instruction at which it is held, and the
  // computing waves work on the handed-over buffer meanwhile.  The stream does not wait for
  // the gating phase and the gating phase does not wait for the stream: one set is requested
  // before the first barrier; between the two barriers the loading waves request the second
  // and store the first into buffer 0 (the gating operand lies in buffer 1).
  if (loader) {
    request(s_first, I0{});
    __syncthreads();
    request(s_first + 1, I1{});
    MHFFN_SB();   // the request stays ahead of the wait for the first set
    store_set(I0{}, buf0);
    __syncthreads();
    request(s_first + 2, I0{});
    MHFFN_SB();
    store_set(I1{}, buf1);
    __syncthreads();
    request(s_first + 3, I1{});
    MHFFN_SB();
    for (int s = s_first + 2; s < n_sets; s += 2) {
      store_set(I0{}, buf0);
      __syncthreads();
      request(s + 2, I0{});
      MHFFN_SB();
      store_set(I1{}, buf1);
      __syncthreads();
      request(s + 3, I1{});
      MHFFN_SB();
    }
    __syncthreads();
  } else {
    // ---- token rows into LDS as NB tile images [32 tokens][128], and the gating operand
    // W_r^T as [64][128] in two tile images (in buffer 1; rows E.. keep whatever the memory
    // held: a row of the product depends on its own row of the operand only, and rows E..
    // are masked below)
    constexpr int kWrIter = kDh * kPipeMaxSubStatic / 8 / CT;   // 4
    constexpr int kRIter = BT * kPipeMaxSubStatic / CT;         // 8, 16, 32
    u32x4 xv[2 * NB];
#pragma unroll
    for (int i = 0; i < 2 * NB; ++i) {
      const int t_row = i * 16 + srow;
      xv[i] = *reinterpret_cast<const u32x4*>(a.X + (int64_t)(t_row < a.N ? t_row : 0) * a.ldx + h * kDh + schunk * 8);
    }
    if (a.route_mode == 0) {
      const uint16_t* Wr = reinterpret_cast<const uint16_t*>(a.route) + (size_t)h * kDh * E;
      u32x4 wv[kWrIter];
#pragma unroll
      for (int it = 0; it < kWrIter; ++it) {
        const int c = rt + it * CT;
        wv[it] = *reinterpret_cast<const u32x4*>(Wr + 8 * (c < kDh * E / 8 ? c : 0));
      }
      auto wr_off = [&](int e, int j) { return (e >> 5) * kPipeTile + tile_off(e & 31, j >> 3) + (j & 7) * 2; };
#pragma unroll
      for (int it = 0; it < kWrIter; ++it) {
        const int c = rt + it * CT;
        if (c < kDh * E / 8) {
          int j = (8 * c) / E, e = 8 * c - j * E;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            *reinterpret_cast<uint16_t*>(buf1 + wr_off(e, j)) = (uint16_t)(wv[it][i >> 1] >> (16 * (i & 1)));
            if (++e == E) { e = 0; ++j; }
          }
        }
      }
    } else {
      const float* R = reinterpret_cast<const float*>(a.route);
      float rv[kRIter];
#pragma unroll
      for (int it = 0; it < kRIter; ++it) {
        const int idx = rt + it * CT;
        const int tl = idx / E, e = idx - tl * E;
        const bool ok = idx < BT * E && tl < a.N;
        rv[it] = R[ok ? ((size_t)tl * a.H + h) * E + e : 0];
      }
#pragma unroll
      for (int it = 0; it < kRIter; ++it) {
        const int idx = rt + it * CT;
        const int tl = idx / E, e = idx - tl * E;
        if (idx < BT * E) Rs[e * BT + tl] = inv_weight(tl < a.N ? rv[it] : 0.f);
      }
    }
#pragma unroll
    for (int i = 0; i < 2 * NB; ++i) {
      const int t_row = i * 16 + srow;
      *reinterpret_cast<u32x4*>(Qs + (t_row >> 5) * kPipeTile + tile_off(t_row & 31, schunk)) =
          (t_row < a.N) ? xv[i] : u32x4{0, 0, 0, 0};
    }
    __syncthreads();
    if (grp == 0 && a.route_mode == 0) {
      const bool two = E > 32;
      f32x16 acc[2] = {f32x16{0}, f32x16{0}};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 qk = *reinterpret_cast<const bf16x8*>(qrow + tile_off(r, 2 * ks + g));
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(buf1 + tile_off(r, 2 * ks + g));
        acc[0] = mfma32(a0, qk, acc[0]);
        if (two) {
          const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(buf1 + kPipeTile + tile_off(r, 2 * ks + g));
          acc[1] = mfma32(a1, qk, acc[1]);
        }
      }
      float sg[2][16];
      float zsum = 0.f;
#pragma unroll
      for (int eb = 0; eb < 2; ++eb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int e = 32 * eb + 8 * (v / 4) + 4 * g + (v % 4);
          sg[eb][v] = (e < E) ? sigmoid_fast(acc[eb][v]) : 0.f;
          zsum += sg[eb][v];
        }
      const float inv = 1.0f / (zsum + __shfl_xor(zsum, 32) + a.eps);
      float* rs_lane = Rs + tok;
#pragma unroll
      for (int eb = 0; eb < 2; ++eb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int e = 32 * eb + 8 * (v / 4) + 4 * g + (v % 4);
          rs_lane[e * BT] = inv_weight(sg[eb][v] * inv);   // rows E..63 exist and are never read
        }
    }
    __syncthreads();  // 1/r complete; buffer 1 is free again

    // the tiles of one buffer that belong to this wave's group (tile_base: index of the
    // buffer's first tile inside the workgroup's share; outside the share: nothing to do)
    auto compute = [&](const unsigned char* buf, int tile_base) {
#pragma unroll
      for (int jj = 0; jj < kDecodeSetTiles; ++jj) {
        const int t = tile_base + jj;
        if (NG > 1 && jj != grp) continue;             // one group: both tiles; else tile `grp` (groups 2, 3 idle)
        if ((unsigned)t >= (unsigned)T) continue;
        const unsigned char* sl = buf + jj * kDecodeTile;
        const float rw = Rs[((t_begin + t) / tiles_per_sub) * BT + tok];
        f32x16 accM = f32x16{0}, accN = f32x16{0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 qk = *reinterpret_cast<const bf16x8*>(qrow + tile_off(r, 2 * ks + g));
          const bf16x8 ak = *reinterpret_cast<const bf16x8*>(sl + tile_off(r, 2 * ks + g));
          const bf16x8 au = *reinterpret_cast<const bf16x8*>(sl + kPipeTile + tile_off(r, 2 * ks + g));
          accM = mfma32(ak, qk, accM);
          accN = mfma32(au, qk, accN);
        }
        bf16x8 bfrag[2];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          float tt[8], ss[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) tt[i] = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * accM[8 * t2 + i]);
#pragma unroll
          for (int i = 0; i < 8; ++i) ss[i] = __builtin_amdgcn_rcpf(__builtin_fmaf(tt[i], rw, rw));
          u32x4 pk;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float a0 = (accM[8 * t2 + 2 * i] * accN[8 * t2 + 2 * i]) * ss[2 * i];
            const float a1 = (accM[8 * t2 + 2 * i + 1] * accN[8 * t2 + 2 * i + 1]) * ss[2 * i + 1];
            pk[i] = pack_bf16(a0, a1);
          }
          bfrag[t2] = __builtin_bit_cast(bf16x8, pk);
        }
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int jb = 0; jb < 4; ++jb)
            O[jb] = mfma32(tile_read_tr(sl + 2 * kPipeTile, 16 * t2 + 4 * g, 32 * jb, lane), bfrag[t2], O[jb]);
      }
    };
    compute(buf0, kDecodeSetTiles * s_first);
    __syncthreads();
    for (int s = s_first + 2; s < n_sets; s += 2) {
      compute(buf1, kDecodeSetTiles * (s - 1));
      __syncthreads();
      compute(buf0, kDecodeSetTiles * s);
      __syncthreads();
    }
    compute(buf1, kDecodeSetTiles * (n_sets - 1));   // the number of sets from s_first on is even: the last one is in buffer 1
    __syncthreads();
  }

  // ---- sum over the groups in the fixed order 0, 1, ..: every computing wave leaves its
  // accumulators in LDS as [wave][quad 4 jb + vq][lane] f32x4 (wave = group * NB + token
  // block), then all threads share out the quads, add and store (16 bytes per lane: 4
  // consecutive columns of Y) ------------------------------------------------------------
  f32x4* red = reinterpret_cast<f32x4*>(smem);
  if (!loader) {
    f32x4* dst = red + (size_t)(wave * 16) * 64 + lane;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq)
        dst[(4 * jb + vq) * 64] = f32x4{O[jb][4 * vq], O[jb][4 * vq + 1], O[jb][4 * vq + 2], O[jb][4 * vq + 3]};
  }
  __syncthreads();
  constexpr int QPT = 2 * NB;                        // quads per thread: 16 NB quads per lane, 8 waves
  if (tok >= a.N) return;
  const int qbase = (wave / NB) * QPT;               // wave / NB runs over 8 / NB values
#pragma unroll
  for (int qi = 0; qi < QPT; ++qi) {
    const int q4 = qbase + qi;
    f32x4 sum = red[(size_t)(tb * 16 + q4) * 64 + lane];
#pragma unroll
    for (int gg = 1; gg < NG; ++gg) sum += red[(size_t)((gg * NB + tb) * 16 + q4) * 64 + lane];
    const int col = 32 * (q4 >> 2) + 8 * (q4 & 3) + 4 * g;
    if (a.n_split > 1) {
      *reinterpret_cast<f32x4*>(a.P + (((size_t)split * a.N + tok) * a.H + h) * kDh + col) = sum;
    } else {
      u32x2 pkw;
      pkw[0] = pack_bf16(sum[0], sum[1]);
      pkw[1] = pack_bf16(sum[2], sum[3]);
      *reinterpret_cast<u32x2*>(a.Y + (int64_t)tok * a.ldy + h * kDh + col) = pkw;
    }
  }
}

// Y[tok][col] = bf16(sum_s P[s][tok][col]), fixed order
__global__ void fwd_bf16_reduce_kernel(FwdArgs a) {
  const int64_t dm = (int64_t)a.H * a.dh;
  const int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (idx >= a.N * dm) return;
  f32x4 sum = {0.f, 0.f, 0.f, 0.f};
  const size_t stride = (size_t)a.N * dm;
  int s = 0;
  for (; s + 8 <= a.n_split; s += 8) {   // eight loads in flight, summed in the order of s
    f32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const f32x4*>(a.P + (size_t)(s + i) * stride + idx);
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += v[i];
  }
  for (; s < a.n_split; ++s)
    sum += *reinterpret_cast<const f32x4*>(a.P + (size_t)s * stride + idx);
  const int64_t tok = idx / dm, col = idx % dm;
  u32x2 pk;
  pk[0] = pack_bf16(sum[0], sum[1]);
  pk[1] = pack_bf16(sum[2], sum[3]);
  *reinterpret_cast<u32x2*>(a.Y + tok * a.ldy + col) = pk;
}

// How the intermediate dimension is shared out when the token tiles alone
// cannot fill the chip (decode / short prefill).  The pipelined kernel (one workgroup of
// 256 tokens per CU) is split down to about one workgroup per CU: with few tokens it
// is a weight-streaming kernel, and its deep ring of direct loads is what keeps
// enough bytes in flight.  The older kernel (more than 64 sub-networks) aims for
// two smaller workgroups per CU.
struct SplitPlan { int bm, n_split, tiles_per_split; bool pipe; int decode_nb; };
constexpr int kDecodeMaxTokens = 128;
SplitPlan plan_split(const Problem& p) {
  SplitPlan s;
  s.pipe = p.dh == kDh && p.E <= kPipeMaxSub;
  s.decode_nb = 0;
  if (s.pipe && p.N <= kDecodeMaxTokens) {
    // decode kernel: about one workgroup per CU, each a head and a share of its tiles
    s.decode_nb = p.N <= 32 ? 1 : p.N <= 64 ? 2 : 4;
    s.bm = 32 * s.decode_nb;
    const int T = p.E * (p.de / kBI);
    int want = 256 / p.H;
    if (want < 1) want = 1;
    if (want > T) want = T;
    s.tiles_per_split = (T + want - 1) / want;
    s.n_split = (T + s.tiles_per_split - 1) / s.tiles_per_split;
    return s;
  }
  s.bm = (!s.pipe && p.N <= 128) ? 64 : 256;
  if (p.dh == 256) s.bm = 128;   // 4 waves of up to 512 registers (see launch_fwd_bf16)
  const int64_t base = ((p.N + s.bm - 1) / s.bm) * p.H;
  const int T = p.E * (p.de / kBI);
  int want = 1;
  if (s.pipe) {
    if (base <= 128) want = (int)(256 / base);
  } else if (base < 384) {
    want = (int)((512 + base - 1) / base);
  }
  if (want > T / 2) want = T / 2 > 0 ? T / 2 : 1;   // at least two tiles per split
  s.tiles_per_split = (T + want - 1) / want;
  s.n_split = (T + s.tiles_per_split - 1) / s.tiles_per_split;
  return s;
}

template <int DH, int TB, int NW>
int launch_variant(const Problem& p, FwdArgs a, const SplitPlan& sp, hipStream_t stream) {
  constexpr int BM = 32 * TB * NW;
  a.n_tiles = (p.N + BM - 1) / BM;
  a.n_split = sp.n_split;
  a.tiles_per_split = sp.tiles_per_split;
  a.n_items = a.n_tiles * p.H * sp.n_split;
  const size_t lds = (size_t)kStages * fwd_stage_bytes(DH) + (size_t)p.E * BM * sizeof(float);
  if (hipError_t e0 = LdsLimit<&fwd_bf16_kernel<DH, TB, NW>, (int)kLdsBytesPerWorkgroup>::ensure(); e0 != hipSuccess)
    return (int)e0;
  const dim3 grid((unsigned)xcd_grid_size(a.n_items));
  hipLaunchKernelGGL((fwd_bf16_kernel<DH, TB, NW>), grid, dim3(64 * NW), lds, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.n_split == 1) return (int)e;
  const int64_t n4 = p.N * p.H * DH / 4;
  hipLaunchKernelGGL(fwd_bf16_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                     stream, a);
  return (int)hipGetLastError();
}

int launch_pipe(const Problem& p, FwdArgs a, const SplitPlan& sp, hipStream_t stream) {
  a.n_tiles = (p.N + kPipeBM - 1) / kPipeBM;
  a.n_split = sp.n_split;
  a.tiles_per_split = sp.tiles_per_split;
  a.n_items = a.n_tiles * p.H * sp.n_split;
  const size_t lds = (size_t)3 * kPipeRing + (size_t)kPipeMaxSub * kPipeBM * sizeof(float);   // 1/r: 64 rows
  if (hipError_t e0 = LdsLimit<&fwd_bf16_flow_kernel, (int)kLdsBytesPerWorkgroup>::ensure(); e0 != hipSuccess)
    return (int)e0;
  hipLaunchKernelGGL(fwd_bf16_flow_kernel, dim3((unsigned)xcd_grid_size(a.n_items)),
                     dim3(64 * kPipeWaves), lds, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.n_split == 1) return (int)e;
  const int64_t n4 = p.N * p.H * kDh / 4;
  hipLaunchKernelGGL(fwd_bf16_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                     stream, a);
  return (int)hipGetLastError();
}

template <int NB>
int launch_decode(const Problem& p, FwdArgs a, const SplitPlan& sp, hipStream_t stream) {
  a.n_tiles = 1;
  a.n_split = sp.n_split;
  a.tiles_per_split = sp.tiles_per_split;
  a.n_items = (int64_t)p.H * sp.n_split;
  const size_t lds = (size_t)decode_lds_bytes(NB);
  if (hipError_t e0 = LdsLimit<&fwd_bf16_decode_kernel<NB>, (int)kLdsBytesPerWorkgroup>::ensure(); e0 != hipSuccess)
    return (int)e0;
  hipLaunchKernelGGL(fwd_bf16_decode_kernel<NB>, dim3((unsigned)xcd_grid_size(a.n_items)),
                     dim3(kDecodeThreads), lds, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.n_split == 1) return (int)e;
  const int64_t n4 = p.N * p.H * kDh / 4;
  hipLaunchKernelGGL(fwd_bf16_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                     stream, a);
  return (int)hipGetLastError();
}

}  // namespace

size_t fwd_bf16_workspace_bytes(const Problem& p) {
  if (p.N == 0) return 0;
  const SplitPlan sp = plan_split(p);
  return sp.n_split > 1 ? (size_t)sp.n_split * p.N * p.H * p.dh * sizeof(float) : 0;
}

int launch_fwd_bf16(const Problem& p, const void* X, const void* Wg, const void* Wu,
                    const void* Wd, const void* route, void* Y, void* ws, void* stream) {
  FwdArgs a;
  a.X = static_cast<const uint16_t*>(X);
  a.Wg = static_cast<const uint16_t*>(Wg);
  a.Wu = static_cast<const uint16_t*>(Wu);
  a.Wd = static_cast<const uint16_t*>(Wd);
  a.route = route;
  a.Y = static_cast<uint16_t*>(Y);
  a.P = static_cast<float*>(ws);
  a.N = p.N; a.ldx = p.ldx; a.ldy = p.ldy;
  a.H = p.H; a.E = p.E; a.de = p.de; a.dh = p.dh; a.route_mode = p.route_mode; a.eps = p.eps;
  a.n_tiles = 0; a.n_items = 0; a.n_split = 1; a.tiles_per_split = 0;
  const SplitPlan sp = plan_split(p);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // 8 waves x 32 tokens (two waves per SIMD) measured 25% faster than 4 waves x
  // 64 tokens at the 1.3B shape: the second wave hides LDS and barrier latency.
  if (sp.decode_nb == 1) return launch_decode<1>(p, a, sp, st);
  if (sp.decode_nb == 2) return launch_decode<2>(p, a, sp, st);
  if (sp.decode_nb == 4) return launch_decode<4>(p, a, sp, st);
  if (sp.pipe) return launch_pipe(p, a, sp, st);
  if (p.dh == 64) {
    if (sp.bm == 64) return launch_variant<64, 1, 2>(p, a, sp, st);
    return launch_variant<64, 1, 8>(p, a, sp, st);
  }
  if (p.dh == 256) {
    // the output accumulators alone are 128 registers per wave and the token operands 64:
    // one wave per SIMD with the whole register file rather than two that spill
    return launch_variant<256, 1, 4>(p, a, sp, st);
  }
  if (sp.bm == 64) return launch_variant<kDh, 1, 2>(p, a, sp, st);
  return launch_variant<kDh, 1, 8>(p, a, sp, st);
}

size_t fwd_bf16_lds_bytes(const Problem& p) {
  const SplitPlan sp = plan_split(p);
  if (sp.decode_nb) return (size_t)decode_lds_bytes(sp.decode_nb);
  if (sp.pipe) return (size_t)3 * kPipeRing + (size_t)kPipeMaxSub * kPipeBM * sizeof(float);
  return (size_t)kStages * fwd_stage_bytes(p.dh) + (size_t)p.E * sp.bm * sizeof(float);
}

}  // namespace mhffn
