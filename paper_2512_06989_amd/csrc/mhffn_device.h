// Device-side helpers shared by the gfx950 kernels of the fused Multi-Head FFN.
//
// MFMA lane layouts used throughout (wave64, lane l, g = l / 32, r = l % 32):
//   v_mfma_f32_32x32x16_bf16  D[32x32] += A[32x16] * B[16x32]
//     A operand: lane holds row r,    k = 8g .. 8g+7   (8 bf16, k contiguous)
//     B operand: lane holds column r, k = 8g .. 8g+7
//     D / C    : lane holds column r, register v (0..15) is row 8*(v/4) + 4g + v%4
// Every kernel computes the *transposed* products (intermediate neurons on the
// MFMA row axis, tokens on the column axis), so that the accumulator of the
// gate/up products is, register for register, a B operand of the following
// down-projection: the chained contraction never leaves the register file.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace mhffn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define MHFFN_LOG2E 1.4426950408889634f

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
//   v_mfma_f32_16x16x32_bf16  D[16x16] += A[16x32] * B[32x16]   (lane l, i = l % 16, gq = l / 16)
//     A operand: row i,    k = 8gq .. 8gq+7;   B operand: column i, k = 8gq .. 8gq+7
//     D / C    : column i, register v (0..3) is row 4gq + v
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// 1 / (1 + 2^(-x*log2e)): one v_exp_f32 and one v_rcp_f32 (1 ulp each), safe
// for either sign: exp2 overflows to +inf for very negative x and rcp(inf) = 0.
__device__ __forceinline__ float sigmoid_fast(float x) {
  float t = __builtin_amdgcn_exp2f(-MHFFN_LOG2E * x);
  return __builtin_amdgcn_rcpf(1.0f + t);
}

// Two fp32 -> packed bf16 (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 p;
  p[0] = (__bf16)a;
  p[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, p);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}

// LDS transpose read (gfx950 ds_read_b64_tr_b16).  Within each block of 16
// lanes, lane i supplies the address of 4 consecutive 16-bit elements and
// receives element (i % 4) of the 4 lanes 4e + i/4, e = 0..3:
//     out[i][e] = in[4e + i/4][i % 4].
// Pointing lane i at row (i / 4), columns 4*(i % 4).. of a row-major [k][n]
// tile therefore returns, to lane i, column i of rows 0..3: an MFMA operand
// whose contraction index is the tile's slow dimension.
__device__ __forceinline__ s16x4 lds_read_tr16(const void* lds_ptr) {
  typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)lds_ptr);
}

// Swizzled LDS tile: [rows][128 bf16], 256 bytes per row, the 16-byte chunks of a
// row permuted by swz(row).  Row-wise operand reads (one row per lane) and
// transposing reads (4 consecutive rows, 64-byte windows) are both free of bank
// conflicts without padding, and a tile is a contiguous image of 4-row groups of
// 1 KB, which is what a wave-wide direct global->LDS load writes.
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
// byte offset of logical 16-byte chunk `chunk` of `row` inside a tile
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * 256 + ((chunk ^ swz(row)) << 4);
}
// byte offset of the 8-byte piece starting at bf16 column `col` (multiple of 4)
__device__ __forceinline__ int tile_off8(int row, int col) {
  return tile_off(row, col >> 3) + ((col & 4) << 1);
}

// Transposed operand for one MFMA step: rows {r0..r0+3} and {r0+8..r0+11} of a
// tile, columns c0 + (lane % 32); lane geometry as in lds_read_tr16.
__device__ __forceinline__ bf16x8 tile_read_tr(const unsigned char* tile, int r0, int c0, int lane) {
  const int li = lane & 15;
  const int row = r0 + (li >> 2);
  const int col = c0 + 16 * ((lane >> 4) & 1) + 4 * (li & 3);
  const s16x4 lo = lds_read_tr16(tile + tile_off8(row, col));
  const s16x4 hi = lds_read_tr16(tile + tile_off8(row + 8, col));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// The same tile for other head widths DH (rows of DH bf16, no padding).  The bank of a
// byte is its position inside a 256-byte line, so a 512-byte row (DH = 256) is two
// lines, each swizzled like a row of the 128-wide tile, and inherits its properties.
// A 128-byte row (DH = 64) shares its line with its neighbour; there the 8 chunks are
// permuted by a function of row/2 chosen such that the rows one 16-byte read cycle
// serves (see the lane groups in the weight-major kernel's notes) land on different
// chunks, and rows r, r+2 of a transposing read on different chunk pairs.
template <int DH>
__device__ __forceinline__ int tile_off_dh(int row, int chunk) {
  static_assert(DH == 64 || DH == 128 || DH == 256, "head width");
  if constexpr (DH == 128) {
    return tile_off(row, chunk);
  } else if constexpr (DH == 64) {
    const int u = row >> 1;
    const int s = ((u & 1) << 1) | ((u & 2) << 1) | ((u >> 2) & 1);
    return row * 128 + ((chunk ^ s) << 4);
  } else {
    return row * (2 * DH) + ((chunk & ~15) << 4) + (((chunk & 15) ^ swz(row)) << 4);
  }
}
template <int DH>
__device__ __forceinline__ int tile_off8_dh(int row, int col) {
  return tile_off_dh<DH>(row, col >> 3) + ((col & 4) << 1);
}
template <int DH>
__device__ __forceinline__ bf16x8 tile_read_tr_dh(const unsigned char* tile, int r0, int c0, int lane) {
  const int li = lane & 15;
  const int row = r0 + (li >> 2);
  const int col = c0 + 16 * ((lane >> 4) & 1) + 4 * (li & 3);
  const s16x4 lo = lds_read_tr16(tile + tile_off8_dh<DH>(row, col));
  const s16x4 hi = lds_read_tr16(tile + tile_off8_dh<DH>(row + 8, col));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// Direct global -> LDS load, 16 bytes per lane: lane l of the wave writes LDS bytes
// [lds_wave_base + 16 l, +16) with the 16 bytes at its own global address.
// lds_wave_base must be wave-uniform.  Completion is counted by vmcnt.
__device__ __forceinline__ void global_to_lds_16B(const void* gptr, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) const void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// ---- LDS reads issued behind the compiler's back -----------------------------
// Kernels that stage tiles with direct global->LDS loads read their operands
// through these: the compiler makes every transposing read wait for all such
// loads in flight (it cannot tell the stages apart), and once some reads are
// invisible to its counters, its own waits for the visible ones would be too
// early or too late to reason about.  The caller counts: LDS operations return in
// order, so "lgkmcnt(n)" before a use means all but the n newest have landed.
// lds_wait<N>(regs...) also ties the registers to the wait, so that no consumer
// can be scheduled ahead of it.
template <int OFFSET>
__device__ __forceinline__ bf16x8 lds_read_b128_untracked(unsigned lds_addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(OFFSET));
  return v;
}
template <int OFFSET>
__device__ __forceinline__ s16x4 lds_read_tr16_untracked(unsigned lds_addr) {
  s16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(OFFSET));
  return v;
}
template <int OFFSET>
__device__ __forceinline__ s16x4 lds_read_b64_untracked(unsigned lds_addr) {
  s16x4 v;
  asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(OFFSET));
  return v;
}
template <int N, typename T0>
__device__ __forceinline__ void lds_wait(T0& a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N));
}
template <int N, typename T0, typename T1>
__device__ __forceinline__ void lds_wait(T0& a, T1& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}
// LDS byte address of a pointer into the workgroup's shared memory
__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
  return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// XCD-aware work distribution.  Workgroups are handed to the 8 XCDs round
// robin by blockIdx, and every XCD has a private L2.  The head-major work list
// (item = head * n_tiles + tile) is cut into 8 contiguous chunks, one per XCD,
// so the workgroups resident on an XCD stream the same head's weights at the
// same time and all but the first reader of a weight tile hit that XCD's L2.
__device__ __forceinline__ int64_t xcd_work_item(int64_t bid, int64_t n_items) {
  const int64_t per_xcd = (n_items + 7) / 8;
  return (bid % 8) * per_xcd + bid / 8;
}
__host__ __device__ __forceinline__ int64_t xcd_grid_size(int64_t n_items) {
  return 8 * ((n_items + 7) / 8);
}

// Host side.  A kernel's dynamic-LDS limit is an attribute of the kernel on one device:
// raise it the first time the kernel is launched on each device.  `done` is the launcher's
// own bit mask of devices (one static per kernel instantiation); concurrent first launches
// from several threads at worst set the attribute twice.
inline hipError_t allow_lds_bytes(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = (uint64_t)1 << (dev & 63);
  if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev < 64) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Every kernel that needs more dynamic LDS than the default limit has one entry in a list
// that is built while the library loads (one static object per kernel instantiation, made by
// the LdsLimit template below wherever a launcher names the kernel).  A launcher calls
// LdsLimit<&kernel, bytes>::ensure() before its launch; mhffn_init() walks the whole list, so
// that after it no launch changes a kernel attribute any more (a caller that records
// launches into a graph wants that).
struct LdsKernelEntry {
  const void* kernel;
  int bytes;
  std::atomic<uint64_t> done{0};
  LdsKernelEntry* next;
  LdsKernelEntry(const void* k, int b);
  hipError_t ensure() { return allow_lds_bytes(kernel, bytes, done); }
};
LdsKernelEntry*& lds_kernel_list();   // head of the list (api.cpp)
inline LdsKernelEntry::LdsKernelEntry(const void* k, int b) : kernel(k), bytes(b), next(lds_kernel_list()) {
  lds_kernel_list() = this;
}
template <auto Kernel, int Bytes>
struct LdsLimit {
  static inline LdsKernelEntry entry{reinterpret_cast<const void*>(Kernel), Bytes};
  static hipError_t ensure() { return entry.ensure(); }
};

}  // namespace mhffn
