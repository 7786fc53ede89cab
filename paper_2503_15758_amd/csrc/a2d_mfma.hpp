// Building blocks shared by the bf16 MFMA tile kernels (H = 128, 96, 80, 64): the MFMA wrapper and its
// fragment layouts, LDS fragment reads, the "dual" LDS tile layout, scalar-base global loads and
// the XCD-aware work mapping.
//
// MFMA used everywhere: v_mfma_f32_32x32x16_bf16, D(32x32) += A(32x16) * B(16x32).
//   A fragment: lane holds row (lane & 31), contraction indices 8*(lane>>5) + 0..7
//   B fragment: lane holds column (lane & 31), contraction indices 8*(lane>>5) + 0..7
//   D: lane holds column (lane & 31); register r is row 8*(r>>2) + 4*(lane>>5) + (r&3)
// Two kinds of fragment reads from a row-major LDS tile (rows x padded head size, bf16):
//   - "natural" fragments (contraction along H): one 128-bit read per lane;
//   - "transposed" fragments (contraction along the row index): two ds_read_b64_tr_b16, where a
//     16-lane group reads 4 consecutive rows x 16 columns and every lane receives a column.
#pragma once
#include <type_traits>

#include "a2d_common.hpp"

namespace a2d {
namespace mfma {

// Head sizes of the MFMA kernels: the tiles are laid out for HD = 64, 96 or 128 columns (multiples
// of the 32-column accumulator tile); a head size of 80 runs as HD = 96 with its last 16 columns
// zero in LDS and in the register fragments and left out of every store.
__host__ __device__ constexpr int padded_head(int h) { return h > 96 ? 128 : (h > 64 ? 96 : 64); }

// compile-time loop: f(std::integral_constant<int, B>{}), ..., f(std::integral_constant<int, E - 1>{})
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

__device__ __forceinline__ f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// eight consecutive D registers -> one bf16 B/A fragment (round to nearest even)
__device__ __forceinline__ bf16x8 pack8(const f32x16& s, int base) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)s[base + e];
  return r;
}

// s_waitcnt vmcnt(0) only (gfx9 encoding: lgkmcnt and expcnt fields left at their maxima).
// Placed after a prologue's one-off global loads it tells the compiler's wait-count insertion that
// those registers are complete, so that uses inside the main loop do not have to be guarded by
// waits that would also cover the loop's own freshly issued prefetches.
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Global-memory pointer that is the same in every lane, held in scalar registers, so that loads
// through it use the scalar-base + 32-bit-lane-offset addressing form (no per-lane 64-bit address
// arithmetic).  It carries the global address space: a generic pointer rebuilt from integers would
// turn the loads into FLAT ones, which also count on the LDS wait counter.
typedef const __attribute__((address_space(1))) char* gptr_t;
__device__ __forceinline__ gptr_t uniform_gptr(const void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<gptr_t>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ u32x4 gload_b128(gptr_t base, unsigned byte_off) {
  return *reinterpret_cast<const __attribute__((address_space(1))) u32x4*>(base + byte_off);
}

// LDS reads by byte address (address space 3)
__device__ __forceinline__ bf16x8 lds_load_b128(unsigned addr) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>((uintptr_t)addr);
}
__device__ __forceinline__ bf16x8 lds_load_tr(unsigned addr_lo, unsigned addr_hi) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)addr_lo);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)addr_hi);
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// "Dual" LDS tile layout for tiles read BOTH ways (natural and transposed) with
// immediate-only addressing: rows of 320 B (256 B data + 64 B pad), and within a row the
// 16-byte chunk c sits at position c ^ ((row >> 2) & 3).
//   - the 64 B pad shifts consecutive rows by 16 banks, so the four rows of a transposing
//     32-lane pass use four disjoint 16-bank windows;
//   - the XOR on the two low chunk bits separates the rows r, r+4, r+8, r+12 that share a
//     window in a 16-row natural (128-bit) pass.
// Every fragment address is then one of four per-lane bases plus a compile-time constant:
//   natural fragment x of rows RB + (lane & 31), RB a multiple of 32:
//       (x & 1 ? nat_o : nat_e) + 64 * (x >> 1) + RB * 320
//   transposing reads of column tile ct, rows RB + {0..7 | 8..15}, RB a multiple of 16:
//       (tr_lo | tr_hi) + 64 * ct + RB * 320
constexpr int DUAL_LD = 320;
constexpr int DUAL64_BYTES = 64 * DUAL_LD;
struct DualAddr {
  unsigned nat_e, nat_o, tr_lo, tr_hi;
  __device__ __forceinline__ void init(int lane, unsigned tile_base) {
    const int l32 = lane & 31, half = lane >> 5;
    const int kap = (l32 >> 2) & 3;
    nat_e = tile_base + l32 * DUAL_LD + 32 * (kap >> 1) + 16 * (half ^ (kap & 1));
    nat_o = nat_e ^ 32;      // bit 5 of the address is exactly the (x & 1) ^ (kap >> 1) term
    const int g16 = lane >> 4, j16 = lane & 15;
    const int row = 4 * (g16 >> 1) + (j16 >> 2);           // 0..7, (row >> 2) & 3 = g16 >> 1
    const int cl = 2 * (g16 & 1) + ((j16 & 3) >> 1);       // logical chunk within a 64-byte column tile
    const int sub = 8 * (j16 & 1);
    tr_lo = tile_base + row * DUAL_LD + 16 * (cl ^ (g16 >> 1)) + sub;
    tr_hi = tile_base + (row + 8) * DUAL_LD + 16 * (cl ^ ((g16 >> 1) + 2)) + sub;
  }
  __device__ __forceinline__ void shift(int delta) { nat_e += delta; nat_o += delta; tr_lo += delta; tr_hi += delta; }
};
// byte offset inside a dual tile at which the 16-byte chunk `c` of row `r` is stored
__device__ __forceinline__ int dual_store_off(int r, int c) { return r * DUAL_LD + ((c ^ ((r >> 2) & 3)) << 4); }

// XCD-aware work mapping.  MI355X has 8 XCDs, each with its own L2, and hands consecutive
// workgroup ids to consecutive XCDs (id % 8).  All blocks of one head read the same K / V (or
// Q / dO) rows, so they are placed on ONE XCD.  Two orders inside an XCD (k-th workgroup of XCD x,
// id = 8 k + x):
//   by head  (by_size = false): head 8 * (k / nblocks) + x, block k % nblocks - a head's blocks run
//            back to back and share its rows in L2; used when all blocks cost the same;
//   by block (by_size = true):  the XCD's heads in chunks of kSizeChunk; inside a chunk block b of
//            every head before any block b + 1.  The callers number the blocks heaviest first, so
//            under a causal mask that crosses the tile the workgroups start longest first and the
//            compute units finish together (diagonal forward tile -7 %); chunks of 2 to 12 heads
//            all gave the same time, 4 keeps most of a head's rows shared in L2 (the unmasked
//            tile loses 2-3 % with this order, which is why it is not the default).
// Grid size: 8 * ceil(heads / 8) * nblocks; workgroups whose head is out of range exit.
constexpr int kXcds = 8;
constexpr int kSizeChunk = 4;
__host__ __device__ inline int xcd_grid(int heads, int nblocks) {
  return kXcds * ((heads + kXcds - 1) / kXcds) * nblocks;
}
__device__ __forceinline__ bool xcd_map(int heads, int nblocks, bool by_size, int& head, int& block) {
  const int id = blockIdx.x;
  const int x = id % kXcds, k = id / kXcds;
  if (by_size) {
    const int hpx = (heads + kXcds - 1) / kXcds;
    const int c = k / (kSizeChunk * nblocks), kk = k - c * (kSizeChunk * nblocks);
    const int width = min(kSizeChunk, hpx - c * kSizeChunk);   // the last chunk may hold fewer heads
    head = kXcds * (c * kSizeChunk + kk % width) + x;
    block = kk / width;
  } else {
    head = kXcds * (k / nblocks) + x;
    block = k % nblocks;
  }
  return head < heads;
}

}  // namespace mfma
}  // namespace a2d
