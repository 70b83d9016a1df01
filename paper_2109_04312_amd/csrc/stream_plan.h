// Work decomposition shared by the bf16 MFMA forward / dQ / dK-dV kernels.
//
// Every kernel has the same shape: a workgroup OWNS 128 rows (queries, or keys for dK/dV) and
// STREAMS 64-row tiles of the other side.  By the attention pattern of Section 3 the two sides
// are symmetric: an owned table token meets the question tokens plus the table tokens of its
// own row / column segment; an owned question token meets every non-pad token.
//
// Units per (sequence, head), in launch order (longest first, surplus last):
//   [0, n_lt)          table-token owners, 128 consecutive slots of the head kind's sorted order
//   then n_pt          pad owners (zero fill);  n_lt + n_pt <= UG + 1
//   [UG + 1, 2 UG + 1) question-token owners.  Their streamed side is the whole sequence, so it
//                      is cut into chunks of >= kMinChunkTiles tiles that run as separate
//                      workgroups and leave partial results, merged by a finalize kernel.
// with UG = ceil(N / 128).  G, L, P live on the device, so the host launches the worst case
// (2 * UG + 1 units) and surplus workgroups exit at once.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_common.h"

namespace mate {

constexpr int BM = 128;            // owned rows per workgroup (32 per wavefront)
constexpr int BN = 64;             // streamed rows per tile
constexpr int kThreads = 256;
constexpr int kTileElems = BN * kLdsRow;
constexpr int kFinalizeBlocks = 4; // workgroups per (b,h) in the finalize kernels (32 rows each, strided)
constexpr int kMinChunkTiles = 8;  // streamed tiles per chunk of a question-token owner

__host__ __device__ inline int owner_slots(int N) { return (N + BM - 1) / BM; }  // UG
inline int units_per_bh(int N) { return 2 * owner_slots(N) + 1; }

// How the streamed side of question-token owners is chunked (same answer in every kernel).
struct GlobalSplit {
  int n_gt;      // owner tiles of question tokens
  int n_st;      // streamed tiles in total: question tiles then table tiles
  int n_chunks;  // units per owner tile (>= 1); partial results are used iff n_chunks > 1
  int per;       // streamed tiles per chunk
};
__device__ inline GlobalSplit global_split(int G, int L, int N) {
  GlobalSplit s;
  s.n_gt = (G + BM - 1) / BM;
  s.n_st = (G + BN - 1) / BN + (L + BN - 1) / BN;
  const int want = (s.n_st + kMinChunkTiles - 1) / kMinChunkTiles;
  const int cap = s.n_gt ? owner_slots(N) / s.n_gt : 1;
  const int n = max(1, min(want, cap));
  s.per = (s.n_st + n - 1) / n;
  s.n_chunks = s.per ? (s.n_st + s.per - 1) / s.per : 1;  // drop empty trailing chunks
  return s;
}

enum { UNIT_NONE = 0, UNIT_GLOBAL = 1, UNIT_LOCAL = 2, UNIT_PAD = 3 };

struct UnitPlan {
  int kind;
  int t0;                // first owned slot in own_list
  const int* own_list;   // global_idx, perm[view] or pad_idx
  int own_count;
  const int* str_list;   // streamed table tokens: perm[view] (perm[0] for question owners)
  int s_lo, s_hi;        // streamed sorted-slot window
  int n_t0;              // streamed question-token tiles; table tiles follow
  int t_begin, t_end;    // streamed tiles of this unit
  int part;              // partial-result slot (unit index) or -1: results are final
  int G, L, P;
};

__device__ inline UnitPlan plan_unit(const AttnArgs& a, int b, int view, int unit) {
  const int N = a.N;
  const int* cnt = a.seg.counts + (size_t)b * kCountWords;
  UnitPlan u;
  u.kind = UNIT_NONE;
  u.G = cnt[C_G];
  u.L = cnt[C_L];
  u.P = cnt[C_P];
  u.part = -1;
  u.n_t0 = (u.G + BN - 1) / BN;
  const int UG = owner_slots(N);
  if (unit > UG) {
    unit -= UG + 1;
    const GlobalSplit s = global_split(u.G, u.L, N);
    if (s.n_gt == 0) return u;
    const int gt = unit / s.n_chunks, c = unit % s.n_chunks;
    if (gt >= s.n_gt) return u;
    u.kind = UNIT_GLOBAL;
    u.t0 = gt * BM;
    u.own_list = a.seg.global_idx + (size_t)b * N;
    u.own_count = u.G;
    u.str_list = a.seg.perm[0] + (size_t)b * N;  // row order: the contiguous one
    u.s_lo = 0;
    u.s_hi = u.L;
    u.t_begin = c * s.per;
    u.t_end = min(s.n_st, u.t_begin + s.per);
    if (s.n_chunks > 1) u.part = unit;
    return u;
  }
  const int n_lt = (u.L + BM - 1) / BM, n_pt = (u.P + BM - 1) / BM;
  const int t = unit;
  if (t < n_lt) {
    u.kind = UNIT_LOCAL;
    u.t0 = t * BM;
    u.own_list = a.seg.perm[view] + (size_t)b * N;
    u.own_count = u.L;
    u.str_list = u.own_list;
    const int2* rng = a.seg.slot_rng[view] + (size_t)b * N;
    u.s_lo = rng[u.t0].x;
    u.s_hi = rng[min(u.t0 + BM, u.L) - 1].y;
    u.t_begin = 0;
    u.t_end = u.n_t0 + (u.s_hi - u.s_lo + BN - 1) / BN;
  } else if (t < n_lt + n_pt) {
    u.kind = UNIT_PAD;
    u.t0 = (t - n_lt) * BM;
    u.own_list = a.seg.pad_idx + (size_t)b * N;
    u.own_count = u.P;
  }
  return u;
}

// Streamed tile t of a unit: which index list, first slot, last valid slot.
__device__ inline void tile_source(const UnitPlan& u, const int* global_idx, int t,
                                   const int*& list, int& base, int& last) {
  if (t < u.n_t0) { list = global_idx; base = t * BN; last = u.G - 1; }
  else { list = u.str_list; base = u.s_lo + (t - u.n_t0) * BN; last = u.s_hi - 1; }
}

// Per-lane view of the owned row: position, and the streamed-slot window it may meet.
struct OwnedRow {
  int pos;            // token position (rows past the end repeat the last valid one)
  bool valid;
  int lo, hi;         // this row's window of streamed table slots
  int w_lo, w_hi;     // union over the wavefront's 32 rows
  int a_lo, a_hi;     // intersection over the wavefront's rows
  bool wave_active;   // the wavefront owns at least one valid row
};
__device__ inline OwnedRow owned_row(const UnitPlan& u, const AttnArgs& a, int b, int view,
                                     int wave, int m) {
  OwnedRow r;
  const int slot_raw = u.t0 + wave * 32 + m;
  const int slot = min(slot_raw, u.own_count - 1);
  r.valid = slot_raw < u.own_count;
  r.wave_active = u.t0 + wave * 32 < u.own_count;
  r.pos = u.own_list[slot];
  r.lo = 0;
  r.hi = u.L;
  if (u.kind == UNIT_LOCAL) {
    const int2 g = a.seg.slot_rng[view][(size_t)b * a.N + slot];
    r.lo = g.x;
    r.hi = g.y;
  }
  r.w_lo = __builtin_amdgcn_readlane(r.lo, 0);   // wave-uniform, kept in scalar registers
  r.w_hi = __builtin_amdgcn_readlane(r.hi, 31);
  r.a_lo = __builtin_amdgcn_readlane(r.lo, 31);
  r.a_hi = __builtin_amdgcn_readlane(r.hi, 0);
  return r;
}

struct TileRegs {
  uint4 r[4];
};
struct TileIdx {
  int tok[4];
};

// Staging a streamed tile is split in two so that the index loads of tile t+2 are in flight
// while tile t+1's rows are fetched: x in [0,128) names a (4 rows x 8 dims) block.
__device__ inline void load_tile_idx(TileIdx& ix, const int* __restrict__ list, int base,
                                     int last, int x) {
  const int jg = x & 15;
#pragma unroll
  for (int u = 0; u < 4; ++u) ix.tok[u] = list[min(base + jg * 4 + u, last)];
}
__device__ inline void load_tile_rows(TileRegs& t, const unsigned short* __restrict__ X,
                                      const TileIdx& ix, int x) {
  const int dg = x >> 4;
#pragma unroll
  for (int u = 0; u < 4; ++u)
    t.r[u] = *reinterpret_cast<const uint4*>(X + (size_t)ix.tok[u] * kD + dg * 8);
}

// 128 threads fetch a 64-row x 64-dim tile as (4 rows x 8 dims) blocks; x in [0,128).
__device__ inline void load_block4x8(TileRegs& t, const unsigned short* __restrict__ X,
                                     const int* __restrict__ list, int base, int last, int x) {
  const int jg = x & 15, dg = x >> 4;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int tok = list[min(base + jg * 4 + u, last)];
    t.r[u] = *reinterpret_cast<const uint4*>(X + (size_t)tok * kD + dg * 8);
  }
}
// ... and write it to LDS as [row][dim] (nat) and / or transposed as [dim][row] (tr).
__device__ inline void store_block4x8(const TileRegs& t, unsigned short* nat, unsigned short* tr,
                                      int x) {
  const int jg = x & 15, dg = x >> 4;
  if (nat) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
      *reinterpret_cast<uint4*>(nat + (jg * 4 + u) * kLdsRow + dg * 8) = t.r[u];
  }
  if (tr) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      *reinterpret_cast<uint2*>(tr + (dg * 8 + e) * kLdsRow + jg * 4) = transpose_pick(t.r, e);
  }
}

// Final results: a C tile pair (columns = owned rows, registers = head dims) scaled, rounded to
// bf16, transposed through LDS and stored as whole 128-byte token rows.  Two barriers.
__device__ inline void store_owned_rows(const f32x16 acc[2], float mul, unsigned short* stage,
                                        unsigned short* __restrict__ out, const int* row_tok,
                                        int wave, int lane) {
  const int m = lane & 31, hl = lane >> 5;
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = f32_to_bf16_bits(acc[db][4 * g] * mul) |
            ((unsigned)f32_to_bf16_bits(acc[db][4 * g + 1] * mul) << 16);
      w.y = f32_to_bf16_bits(acc[db][4 * g + 2] * mul) |
            ((unsigned)f32_to_bf16_bits(acc[db][4 * g + 3] * mul) << 16);
      *reinterpret_cast<uint2*>(stage + (wave * 32 + m) * kLdsRow + db * 32 + 8 * g + 4 * hl) = w;
    }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = wave * 32 + it * 8 + (lane >> 3), piece = lane & 7;
    const int tok = row_tok[row];
    if (tok >= 0)
      *reinterpret_cast<uint4*>(out + (size_t)tok * kD + piece * 8) =
          *reinterpret_cast<const uint4*>(stage + row * kLdsRow + piece * 8);
  }
  __syncthreads();
}

// Partial results of a chunked question-token owner: fp32 [128][64], row = owned row.
__device__ inline void store_partial(const f32x16 acc[2], float mul, float* __restrict__ part,
                                     int wave, int lane) {
  const int m = lane & 31, hl = lane >> 5;
  float* row = part + (size_t)(wave * 32 + m) * kD;
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<float4*>(row + db * 32 + 8 * g + 4 * hl) =
          make_float4(acc[db][4 * g] * mul, acc[db][4 * g + 1] * mul, acc[db][4 * g + 2] * mul,
                      acc[db][4 * g + 3] * mul);
}

__device__ inline void zero_pad_rows(unsigned short* __restrict__ out, const UnitPlan& u, int tid) {
  for (int x = tid; x < BM * 8; x += kThreads) {
    const int row = x >> 3, piece = x & 7;
    if (u.t0 + row < u.own_count)
      *reinterpret_cast<uint4*>(out + (size_t)u.own_list[u.t0 + row] * kD + piece * 8) =
          make_uint4(0, 0, 0, 0);
  }
}

// Development aid (compiled out unless MATE_TRACE is defined): one record per workgroup with
// its start / end time (100 MHz wall clock), hardware placement and unit description.
#ifdef MATE_TRACE
#define MATE_TRACE_KERNEL(body_call, kernel_no)                                            \
  const long long t_start_ = wall_clock64();                                               \
  const int info_ = body_call;                                                             \
  if (a.trace && threadIdx.x == 0) {                                                       \
    long long* r_ = a.trace + ((size_t)(kernel_no) * (1 << 16) + blockIdx.x) * 4;          \
    r_[0] = t_start_;                                                                      \
    r_[1] = wall_clock64();                                                                \
    r_[2] = info_;                                                                         \
    r_[3] = ((long long)__builtin_amdgcn_s_getreg(63508) << 32) |                          \
            (unsigned)__builtin_amdgcn_s_getreg(63492);                                    \
  }
#else
#define MATE_TRACE_KERNEL(body_call, kernel_no) (void)body_call;
#endif
// what a unit body reports to the trace: kind | streamed tiles << 4
__device__ inline int unit_info(const UnitPlan& u) {
  return u.kind | ((u.kind == UNIT_GLOBAL || u.kind == UNIT_LOCAL ? u.t_end - u.t_begin : 0) << 4);
}

__device__ inline bool tables_match(const AttnArgs& a) {
  return a.seg.hdr[0] == kMagic && a.seg.hdr[1] == a.B && a.seg.hdr[2] == a.N;
}

// Workspace carving (float words).  Partial buffers are per (b,h): [UG][BM][64].
__host__ __device__ inline size_t part_words_per_bh(int N) { return (size_t)owner_slots(N) * BM * kD; }
__host__ __device__ inline size_t stat_words_per_bh(int N) { return (size_t)owner_slots(N) * BM * 2; }

}  // namespace mate
