// Streaming 64-row x 64-dim bf16 tiles from global memory straight into LDS (gfx950
// global_load_lds_dwordx4), and reading them back as MFMA operands, plain or transposed
// (ds_read_b64_tr_b16).  No registers are spent on staging, so several tiles can be in flight.
//
// LDS tile layout: 64 rows of 128 bytes, no padding; the eight 16-byte chunks of row r are
// stored XOR-swizzled, chunk c at slot c ^ swz(r), with swz(r) built from bits 1..3 of r:
//   * 16 consecutive rows read at one chunk index (plain 16-byte operand reads) hit 16 distinct
//     (bank-half, slot) pairs;
//   * 4 consecutive rows read at two adjacent chunks (transposing 8-byte reads) do too.
// A wave-wide load instruction deposits lane l's 16 bytes at (LDS base) + 16 l, i.e. rows
// l / 8 of an 8-row group, slot l % 8; the swizzle is applied by choosing which global chunk
// each lane fetches.
//
// Hardware facts this relies on (checked on the device with known data):
//   * global_load_lds_dwordx4: lane l's data lands at M0-base + 16 l.
//   * ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives element (i & 3) of the
//     four 8-byte rows addressed by lanes (i >> 2), (i >> 2) + 4, + 8, + 12 of the group.
#pragma once
#include <hip/hip_runtime.h>

#include "mfma_common.h"

namespace mate {

constexpr int kTileBytes = 64 * 128;  // one streamed tile in LDS

__device__ inline int swz(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }

typedef short s16x4 __attribute__((ext_vector_type(4)));

// ---- issuing loads -------------------------------------------------------------------------
// A wavefront covers rows 16 w .. 16 w + 15 of a tile with two instructions (8 rows each).
struct LoadLane {
  int row0;    // this lane's row for instruction 0 (instruction 1: row0 + 8)
  int chunk0;  // global chunk this lane fetches for instruction 0 (instruction 1: chunk0 ^ 2)
};
__device__ inline LoadLane make_load_lane(int wave, int lane) {
  LoadLane l;
  l.row0 = 16 * wave + (lane >> 3);
  l.chunk0 = (lane & 7) ^ swz(l.row0 & 15);  // swz(row0 + 8) = swz(row0) ^ 2
  return l;
}

// The load instructions are written as inline assembly on purpose: the compiler then does not
// know that they write LDS, so it does not guard later LDS reads with "wait for every
// outstanding load" (which would drain the prefetches of later tiles on every iteration).
// Ordering against the LDS reads is by the explicit waits and barriers of the caller.  The
// compiler's own vmcnt bookkeeping for ordinary loads stays safe: loads it cannot see only make
// its waits stricter, since loads retire in issue order.
__device__ inline unsigned lds_addr(const void* p) {
  return __builtin_amdgcn_readfirstlane(
      (unsigned)(size_t)(const __attribute__((address_space(3))) char*)p);
}
// Address form: 64-bit base in scalar registers (wave-uniform) plus a 32-bit byte offset per
// lane, so the per-lane address arithmetic is one shift-add.
__device__ inline void load_to_lds_16(const void* base /* wave-uniform */, unsigned byte_off,
                                      const void* lds_dst /* wave-uniform */) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(byte_off), "s"(base), "s"(lds_addr(lds_dst)) : "memory", "m0");
}
__device__ inline void load_to_lds_4(const void* base /* wave-uniform */, unsigned byte_off,
                                     const void* lds_dst /* wave-uniform */) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(byte_off), "s"(base), "s"(lds_addr(lds_dst)) : "memory", "m0");
}

// Rows `tok0` / `tok1` (token positions of this lane's two rows) of tensor X (wave-uniform
// base; a (sequence, head) slice, so byte offsets fit 32 bits) into the tile at LDS address
// `tile` (wave-uniform).
__device__ inline void issue_tile(const unsigned short* X, int tok0, int tok1,
                                  const LoadLane& l, const char* tile, int wave) {
  const char* d0 = tile + (16 * wave) * 128;
  load_to_lds_16(X, (unsigned)tok0 * 128u + l.chunk0 * 16, d0);
  load_to_lds_16(X, (unsigned)tok1 * 128u + (l.chunk0 ^ 2) * 16, d0 + 8 * 128);
}

// One 32-bit word per lane, word `index` of the array at `base` (wave-uniform), to 64
// consecutive words at `dst` (wave-uniform LDS address): token indices, or per-row statistics,
// of a streamed tile.
__device__ inline void issue_row_words(const void* base, int index, const void* dst) {
  load_to_lds_4(base, (unsigned)index * 4u, dst);
}

// ---- waiting ------------------------------------------------------------------------------
// "At most n of my vector-memory loads still outstanding" (n wave-uniform, 0 <= n; values above
// kMax are treated as kMax).  Loads complete in issue order, so this retires everything issued
// before the last n.  n is rounded down to a value with an encoding below (waiting for more is
// always safe).
template <int kMax = 12>
__device__ inline void wait_vmcnt_le(int n) {
  if (kMax >= 12 && n >= 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
  else if (kMax >= 11 && n >= 11) asm volatile("s_waitcnt vmcnt(11)" ::: "memory");
  else if (kMax >= 10 && n >= 10) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
  else if (kMax >= 9 && n >= 9) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
  else if (kMax >= 8 && n >= 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if (kMax >= 6 && n >= 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
  else if (kMax >= 5 && n >= 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
  else if (kMax >= 4 && n >= 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Workgroup barrier without the release/acquire fence of __syncthreads (which would wait for
// every outstanding load, including the prefetches of later tiles).  The caller has already
// waited for exactly the loads that must be visible.
__device__ inline void barrier_no_fence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// ---- reading operands -----------------------------------------------------------------------
// Plain operand: tile row = 32 blk + m, dims 16 ks + 8 hl .. + 7 (A operand with k = dims).
// plain_off(ks) is per lane; add blk * 32 * 128 bytes.
__device__ inline int plain_off(int m, int hl, int ks) {
  return m * 128 + (((2 * ks + hl) ^ swz(m & 15)) << 4);
}
__device__ inline bf16x8 read_plain(const char* tile, int off) {
  return *reinterpret_cast<const bf16x8*>(tile + off);
}

// Transposed operand: A row = dim 32 db + m, k = tile rows.  For a C tile computed with rows =
// tile rows (no permutation), the eight registers 8 tt .. 8 tt + 7 of a lane in half hl are tile
// rows 16 tt + 4 hl + {0..3} and 16 tt + 8 + 4 hl + {0..3} of the 32-row block: two transposing
// reads.  tr_off(db, half) is per lane; add (32 blk + 16 tt) * 128 bytes.
__device__ inline int tr_off(int lane, int db, int half) {
  const int i = lane & 15, g = lane >> 4, hl = g >> 1;
  const int jl = 4 * hl + (i >> 2) + 8 * half;              // row inside the 16-row group
  const int chunk = db * 4 + 2 * (g & 1) + ((i & 3) >> 1);  // dims 32 db + 16 (g & 1) + 4 (i & 3)
  return jl * 128 + ((chunk ^ swz(jl)) << 4) + ((i & 1) << 3);
}
__device__ inline bf16x8 read_transposed(const char* tile, int off_lo, int off_hi) {
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(tile + off_lo));
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(tile + off_hi));
  union { s16x4 h[2]; bf16x8 v; } u;
  u.h[0] = a;
  u.h[1] = b;
  return u.v;
}

// Tile row (0..31 inside a 32-row block) held in C register c of a lane in half hl when the A
// operand rows are fed unpermuted.
__device__ inline int c_row(int c, int hl) { return 8 * (c >> 2) + 4 * hl + (c & 3); }

}  // namespace mate
