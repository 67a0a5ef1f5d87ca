// bf16 matrix product for the module's d_model x d_model projections (Methodology:
// Q = split_H(X W_in), O = concat_H(S) W_out, and the four products of their backward).
//
//   C[m][n] = sum_k A(m,k) B(n,k),   C row-major bf16, fp32 accumulation on the MFMA,
//
// each operand given either with k contiguous ("row form": [rows][K]) or with its row
// index contiguous ("transposed form": [K][rows]), so all three products of a linear
// layer read their operands where they lie:
//   Y = X W      A = X row form,   B = W transposed form
//   dX = dY W^T  A = dY row form,  B = W row form
//   dW = X^T dY  A = X transposed, B = dY transposed
//
// Workgroup = 16 waves = 256 (m) x 256 (n) output tile, wave = 64 x 64 (2 x 2 products of
// 32 x 32), k in slices of 64.  What sets the shape is the global -> LDS rate: measured,
// a CU takes about 27 bytes per clock through direct loads (14 TB/s over the chip), so a
// 256 x 128 tile (1.6 GB of operand traffic for a 16384 x 2048 x 2048 product) spends
// 0.116 ms on loads alone; 256 x 256 needs 1.07 GB.  Four waves per SIMD at 128 registers
// then hide each other's LDS latency without a second register set.  The n side sits on
// the MFMA row axis and the m side on the column axis, so a lane ends up with four
// consecutive n of one row m and stores 8 bytes.  Operand slices go global -> LDS
// directly into two 64 KB stages (four wave-wide loads per wave and slice), requested
// one slice ahead; one bare barrier per slice.
// LDS images: row form [rows][64] with the eight 16-byte chunks of a row permuted,
// transposed form the swizzled [32][128] tile of the fused kernels; both are free of
// bank conflicts for their reads.  Operand reads are issued untracked, eight at a time,
// and waited for by count.
// With a transposed operand in play the contraction slots of one MFMA step follow the
// transposing read (slot s of lane group g <-> k = 8 (s / 4) + 4 g + s % 4); a row-form
// partner is then read as two 8-byte halves with the same mapping.
#include "mhffn_device.h"
#include "mhffn_internal.h"

#include <type_traits>

namespace mhffn {
namespace {

constexpr int kGWaves = 16, kGThreads = 64 * kGWaves;
constexpr int kGTileM = 256, kGTileN = 256, kGBK = 64;
constexpr int kGMBytes = kGTileM * kGBK * 2;   // 32 KB
constexpr int kGNBytes = kGTileN * kGBK * 2;   // 32 KB
constexpr int kGStageBytes = kGMBytes + kGNBytes;
constexpr int kGStages = 2;
constexpr int kGLdsBytes = kGStages * kGStageBytes;   // 128 KB
constexpr int kGLoads = (kGStageBytes / 1024) / kGWaves;   // wave-wide 1 KB loads per wave and slice
static_assert(kGLdsBytes <= (int)kLdsBytesPerWorkgroup, "both stages must fit in LDS");
static_assert(kGLoads == 4, "2 images of the m side and 2 of the n side per wave");

struct TunedGemmArgs {
  const uint16_t* A;   // m side
  const uint16_t* B;   // n side
  uint16_t* C;
  int64_t M, N, K, lda, ldb, ldc;
  int64_t n_items, tiles_n;
  // split-k: each output tile is shared out over `splits` workgroups, slices_per_split
  // slices of k each; they leave fp32 partial tiles in P [splits][M][N]
  int splits;
  int64_t slices_per_split;
  float* P;
  int accumulate;   // add to what C holds (one more rounding to bf16)
};

template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

// LDS image of one side of a slice (256 rows):
//   row form:        [rows][64 k], 128-byte rows, chunks permuted as in the 64-wide tile
//   transposed form: swizzled [32 k][128] tiles, tile index = (k / 32) * (rows / 128) + row / 128
// Both are contiguous in 1 KB images (8 rows, or 4 k rows of one tile), which is what one
// wave-wide direct load writes.

template <bool A_TR, bool B_TR>
__global__ __launch_bounds__(kGThreads) void gemm_bf16_kernel(TunedGemmArgs a) {
  constexpr bool kTrSlots = A_TR || B_TR;   // contraction slots follow the transposing read
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave_u >> 2, wn = wave_u & 3;      // 4 x 4 waves
  const int64_t item = xcd_work_item(blockIdx.x, a.n_items);
  if (item >= a.n_items) return;
  const int split = (int)(item % a.splits);
  const int64_t tile = item / a.splits;
  const int64_t m0 = (tile / a.tiles_n) * kGTileM, n0 = (tile % a.tiles_n) * kGTileN;
  const int64_t K = a.K;
  const int64_t KT_all = (K + kGBK - 1) / kGBK;
  const int64_t kbase = split * a.slices_per_split;           // first slice of this workgroup
  const int64_t kend = kbase + a.slices_per_split < KT_all ? kbase + a.slices_per_split : KT_all;
  const int64_t KT = kend - kbase;                            // its number of slices (>= 1)

  // ---- staging: four wave-wide 1 KB loads per wave and slice -----------------------------
  // images 2w, 2w+1 of the 32 of the m side and of the 32 of the n side.
  // Row form: image i = rows 8i .. 8i+7, lane l -> row 8i + l/8, physical chunk l%8.
  // Transposed form: image i = k rows 4(i%8) .. +3 of tile i/8, lane l -> k row + l/16,
  // physical chunk l%16.  Rows / columns past the edge are clamped (their products are never
  // stored); k rows past K are clamped too and their slots cleared before use.
  const uint16_t* src[kGLoads];
  int64_t kstride[kGLoads];   // transposed form: element stride of k
  int krow[kGLoads];          // transposed form: k row of this lane inside a slice (else -1)
  int lds_img[kGLoads];       // byte offset of the image inside a stage
  auto setup = [&](int slot, bool tr, const uint16_t* base, int64_t ld, int64_t row0, int64_t rows,
                   int tile_rows, int img, int side_off) {
    if (!tr) {
      const int row = 8 * img + (lane >> 3);
      const int u = row >> 1;
      const int sw = ((u & 1) << 1) | ((u & 2) << 1) | ((u >> 2) & 1);   // as in tile_off_dh<64>
      const int chunk = (lane & 7) ^ sw;
      int64_t gr = row0 + row;
      gr = gr < rows ? gr : rows - 1;
      src[slot] = base + gr * ld + chunk * 8;
      kstride[slot] = 0;
      krow[slot] = -1;
    } else {
      const int tile = img >> 3, halves = tile_rows >> 7;
      const int kr = 32 * (tile / halves) + 4 * (img & 7) + (lane >> 4);
      const int chunk = (lane & 15) ^ swz(kr & 31);
      int64_t gc = row0 + 128 * (tile % halves) + chunk * 8;
      gc = gc + 8 <= rows ? gc : rows - 8;
      src[slot] = base + gc;      // + k row * ld, added per slice (clamped)
      kstride[slot] = ld;
      krow[slot] = kr;
    }
    lds_img[slot] = side_off + img * 1024;
  };
#pragma unroll
  for (int i = 0; i < 2; ++i) setup(i, A_TR, a.A, a.lda, m0, a.M, kGTileM, 2 * wave_u + i, 0);
#pragma unroll
  for (int i = 0; i < 2; ++i) setup(2 + i, B_TR, a.B, a.ldb, n0, a.N, kGTileN, 2 * wave_u + i, kGMBytes);
  auto dma_one = [&](int64_t kt, int stage, int s) {
    const uint16_t* p;
    if (krow[s] < 0) {
      p = src[s] + kt * kGBK;
    } else {
      int64_t k = kt * kGBK + krow[s];
      k = k < K ? k : K - 1;
      p = src[s] + k * kstride[s];
    }
    global_to_lds_16B(p, smem + stage * kGStageBytes + lds_img[s]);
  };
  auto dma = [&](int64_t kt, int stage) {
#pragma unroll
    for (int s = 0; s < kGLoads; ++s) dma_one(kt, stage, s);
  };

  // ---- operand addresses inside a stage --------------------------------------------------
  // item = (t2, idx, side): t2 = 16-wide contraction step 0..3, idx = 32-row block of the
  // wave's 64, side 0 = n (MFMA rows), 1 = m (MFMA columns).  Split reads (8 bytes twice)
  // whenever the contraction slots follow the transposing read.  What does not depend on
  // the lane goes into the instruction's offset field:
  //   row form:        register per t2 (the chunk permutation is an XOR), idx = +32 rows = +4096
  //   transposed form: register per idx, t2 = +16 k rows (+4096) and, from t2 = 2 on, the
  //                    next group of 32-row tiles; the swizzle does not depend on t2
  const unsigned lbase = lds_addr_of(smem);
  unsigned arow[2][4], arow2[2][4];   // row form [side][t2]: first / second half of a split read
  unsigned atr[2][2], atr2[2][2];     // transposed form [side][idx]: k rows .. and .. + 8
#pragma unroll
  for (int side = 0; side < 2; ++side) {
    const bool tr = side ? A_TR : B_TR;
    const int wrow = side ? 64 * wm : 64 * wn;
    const unsigned sbase = lbase + (side ? 0 : kGMBytes);
    if (!tr) {
#pragma unroll
      for (int t2 = 0; t2 < 4; ++t2) {
        const int row = wrow + r;
        arow[side][t2] = sbase + (kTrSlots ? tile_off_dh<64>(row, 2 * t2) + 8 * g
                                           : tile_off_dh<64>(row, 2 * t2 + g));
        arow2[side][t2] = sbase + tile_off_dh<64>(row, 2 * t2 + 1) + 8 * g;
      }
    } else {
#pragma unroll
      for (int idx = 0; idx < 2; ++idx) {
        const int li = lane & 15;
        const int kr = 4 * g + (li >> 2);
        const int col = wrow + 32 * idx + 16 * ((lane >> 4) & 1) + 4 * (li & 3);
        atr[side][idx] = sbase + (col >> 7) * 8192 + tile_off8(kr, col & 127);
        atr2[side][idx] = sbase + (col >> 7) * 8192 + tile_off8(kr + 8, col & 127);
      }
    }
  }

  f32x16 acc[2][2];   // [n block][m block]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x16{0};

  // ---- main loop ----------------------------------------------------------------------------
  // Two stages.  Iteration kt: barrier (slice kt has landed everywhere, everyone is done with
  // slice kt-1), request slice kt+1 into the other stage, then the slice in two halves of
  // two contraction steps: eight operand reads issued, eight products consumed with counted
  // waits.  Four waves share a SIMD, so one wave's LDS latency is another's MFMA time.
  constexpr bool kSplit = kTrSlots;
  constexpr int kInstr = kSplit ? 2 : 1;   // LDS read instructions per operand
  struct Half {
    s16x4 lo[8], hi[8];   // split reads
    bf16x8 full[8];       // 16-byte reads
  };
  auto issue_half = [&](Half& f, unsigned so, auto HB_) {
    static_for<0, 8>([&](auto IT_) {
      constexpr int it = decltype(IT_)::value, t2 = 2 * decltype(HB_)::value + (it >> 2);
      constexpr int idx = (it >> 1) & 1, side = it & 1;
      constexpr bool tr = side ? A_TR : B_TR;
      if constexpr (tr) {
        constexpr int OFF = (t2 & 1) * 4096 + (t2 >> 1) * 16384;   // two 32-row tiles per group of 32 k rows
        f.lo[it] = lds_read_tr16_untracked<OFF>(atr[side][idx] + so);
        f.hi[it] = lds_read_tr16_untracked<OFF>(atr2[side][idx] + so);
      } else if constexpr (kSplit) {
        f.lo[it] = lds_read_b64_untracked<4096 * idx>(arow[side][t2] + so);
        f.hi[it] = lds_read_b64_untracked<4096 * idx>(arow2[side][t2] + so);
      } else {
        f.full[it] = lds_read_b128_untracked<4096 * idx>(arow[side][t2] + so);
      }
    });
  };
  auto compute_half = [&](Half& f, int64_t kt, auto HB_) {
    const bool ragged_last = kTrSlots && (kt == KT_all - 1) && (K % kGBK) != 0;
    static_for<0, 2>([&](auto TT_) {
      constexpr int tt = decltype(TT_)::value, t2 = 2 * decltype(HB_)::value + tt;
      bf16x8 nf[2], mf[2];
      static_for<0, 4>([&](auto Q_) {
        constexpr int it = 4 * tt + decltype(Q_)::value, idx = (it >> 1) & 1, side = it & 1;
        constexpr int pending = (7 - it) * kInstr;   // reads issued after this item
        bf16x8 v;
        if constexpr (kSplit) {
          lds_wait<pending>(f.lo[it], f.hi[it]);
          v = join_tr(f.lo[it], f.hi[it]);
        } else {
          lds_wait<pending>(f.full[it]);
          v = f.full[it];
        }
        if constexpr (side == 0) {
          if (ragged_last) {
            // k rows past K were clamped when the slice was requested: clear their slots on the
            // n side (slot s of lane group g <-> k = 16 t2 + 8 (s / 4) + 4 g + s % 4)
#pragma unroll
            for (int sl = 0; sl < 8; ++sl)
              if (kt * kGBK + 16 * t2 + 8 * (sl >> 2) + 4 * g + (sl & 3) >= K) v[sl] = (__bf16)0.0f;
          }
          nf[idx] = v;
        } else {
          mf[idx] = v;
        }
      });
      acc[0][0] = mfma32(nf[0], mf[0], acc[0][0]);
      acc[1][0] = mfma32(nf[1], mf[0], acc[1][0]);
      acc[0][1] = mfma32(nf[0], mf[1], acc[0][1]);
      acc[1][1] = mfma32(nf[1], mf[1], acc[1][1]);
    });
  };

  dma(kbase, 0);
  auto iteration = [&](int64_t kt, auto STAGE_) {
    constexpr int stage = decltype(STAGE_)::value;
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of slice kt
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kt + 1 < KT) dma(kbase + kt + 1, stage ^ 1);
    Half f;
    issue_half(f, stage * kGStageBytes, std::integral_constant<int, 0>{});
    compute_half(f, kbase + kt, std::integral_constant<int, 0>{});
    issue_half(f, stage * kGStageBytes, std::integral_constant<int, 1>{});
    compute_half(f, kbase + kt, std::integral_constant<int, 1>{});
  };
  for (int64_t kt = 0; kt < KT; kt += 2) {
    iteration(kt, std::integral_constant<int, 0>{});
    if (kt + 1 < KT) iteration(kt + 1, std::integral_constant<int, 1>{});
  }

  // ---- store: lane = row m, registers = four consecutive n per group ----------------------
#pragma unroll
  for (int im = 0; im < 2; ++im) {
    const int64_t m = m0 + 64 * wm + 32 * im + r;
    if (m >= a.M) continue;
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int64_t n = n0 + 64 * wn + 32 * jn + 8 * vq + 4 * g;
        if (n + 4 > a.N) continue;
        if (a.splits > 1) {
          const f32x4 v = {acc[jn][im][4 * vq], acc[jn][im][4 * vq + 1], acc[jn][im][4 * vq + 2],
                           acc[jn][im][4 * vq + 3]};
          *reinterpret_cast<f32x4*>(a.P + ((size_t)split * a.M + m) * a.N + n) = v;
        } else {
          float o[4] = {acc[jn][im][4 * vq], acc[jn][im][4 * vq + 1], acc[jn][im][4 * vq + 2],
                        acc[jn][im][4 * vq + 3]};
          u32x2* dst = reinterpret_cast<u32x2*>(a.C + m * a.ldc + n);
          if (a.accumulate) {
            const u32x2 old = *dst;
            o[0] += __builtin_bit_cast(float, old[0] << 16);
            o[1] += __builtin_bit_cast(float, old[0] & 0xFFFF0000u);
            o[2] += __builtin_bit_cast(float, old[1] << 16);
            o[3] += __builtin_bit_cast(float, old[1] & 0xFFFF0000u);
          }
          u32x2 pk;
          pk[0] = pack_bf16(o[0], o[1]);
          pk[1] = pack_bf16(o[2], o[3]);
          *dst = pk;
        }
      }
    }
  }
}

// C[m][n] = bf16(sum_s P[s][m][n]), fixed order
__global__ void gemm_bf16_reduce_kernel(TunedGemmArgs a) {
  const int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (idx >= a.M * a.N) return;
  f32x4 sum = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < a.splits; ++s)
    sum += *reinterpret_cast<const f32x4*>(a.P + (size_t)s * a.M * a.N + idx);
  const int64_t m = idx / a.N, n = idx % a.N;
  u32x2* dst = reinterpret_cast<u32x2*>(a.C + m * a.ldc + n);
  if (a.accumulate) {
    const u32x2 old = *dst;
    sum[0] += __builtin_bit_cast(float, old[0] << 16);
    sum[1] += __builtin_bit_cast(float, old[0] & 0xFFFF0000u);
    sum[2] += __builtin_bit_cast(float, old[1] << 16);
    sum[3] += __builtin_bit_cast(float, old[1] & 0xFFFF0000u);
  }
  u32x2 pk;
  pk[0] = pack_bf16(sum[0], sum[1]);
  pk[1] = pack_bf16(sum[2], sum[3]);
  *dst = pk;
}

// Split k only when the output tiles alone leave most of the chip idle (the weight-gradient
// products: d_model x d_model outputs, contraction over all tokens).
struct SplitK { int splits; int64_t slices_per_split; };
SplitK plan_split_k(int64_t M, int64_t N, int64_t K) {
  const int64_t tiles = ((M + kGTileM - 1) / kGTileM) * ((N + kGTileN - 1) / kGTileN);
  const int64_t KT = (K + kGBK - 1) / kGBK;
  int64_t want = tiles >= 192 ? 1 : (256 + tiles - 1) / tiles;
  if (want > 16) want = 16;
  if (want > KT / 8) want = KT / 8 > 0 ? KT / 8 : 1;   // at least eight slices per workgroup
  SplitK s;
  s.slices_per_split = (KT + want - 1) / want;
  s.splits = (int)((KT + s.slices_per_split - 1) / s.slices_per_split);
  return s;
}

template <bool A_TR, bool B_TR>
int launch_form(const TunedGemmArgs& a, hipStream_t stream) {
  if (hipError_t e0 = LdsLimit<&gemm_bf16_kernel<A_TR, B_TR>, kGLdsBytes>::ensure(); e0 != hipSuccess)
    return (int)e0;
  hipLaunchKernelGGL((gemm_bf16_kernel<A_TR, B_TR>), dim3((unsigned)xcd_grid_size(a.n_items)),
                     dim3(kGThreads), kGLdsBytes, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.splits == 1) return (int)e;
  const int64_t n4 = a.M * a.N / 4;
  hipLaunchKernelGGL(gemm_bf16_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                     stream, a);
  return (int)hipGetLastError();
}

}  // namespace

bool gemm_bf16_supported(bool a_tr, bool b_tr, const void* A, int64_t lda, const void* B,
                         int64_t ldb, const void* C, int64_t ldc, int64_t M, int64_t N, int64_t K) {
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (M < 1 || N < 8 || K < 1 || N % 8 != 0) return false;
  if (!al16(A) || !al16(B) || !al16(C) || lda % 8 != 0 || ldb % 8 != 0 || ldc % 4 != 0) return false;
  // a row-form operand is read in whole 32-wide slices of k; a transposed one in whole
  // 8-wide groups of its row index
  if ((!a_tr || !b_tr) && K % kGBK != 0) return false;
  if (a_tr && (M < 8 || M % 8 != 0)) return false;
  if (b_tr && N % 8 != 0) return false;
  return true;
}

size_t gemm_bf16_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  const SplitK sk = plan_split_k(M, N, K);
  return sk.splits > 1 ? (size_t)sk.splits * M * N * sizeof(float) : 0;
}

int launch_gemm_bf16(bool a_tr, bool b_tr, const void* A, int64_t lda, const void* B, int64_t ldb,
                     void* C, int64_t ldc, int64_t M, int64_t N, int64_t K, void* ws, void* stream,
                     bool accumulate) {
  TunedGemmArgs a;
  a.accumulate = accumulate ? 1 : 0;
  a.A = static_cast<const uint16_t*>(A);
  a.B = static_cast<const uint16_t*>(B);
  a.C = static_cast<uint16_t*>(C);
  a.M = M; a.N = N; a.K = K; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
  a.tiles_n = (N + kGTileN - 1) / kGTileN;
  const SplitK sk = plan_split_k(M, N, K);
  a.splits = sk.splits;
  a.slices_per_split = sk.slices_per_split;
  a.P = static_cast<float*>(ws);
  if (a.splits > 1 && !ws) return -1;
  a.n_items = ((M + kGTileM - 1) / kGTileM) * a.tiles_n * a.splits;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!a_tr && b_tr) return launch_form<false, true>(a, st);
  if (!a_tr && !b_tr) return launch_form<false, false>(a, st);
  if (a_tr && b_tr) return launch_form<true, true>(a, st);
  return -1;   // transposed A with row-form B: no caller
}

}  // namespace mhffn
