// Work decomposition shared by the bf16 MFMA forward / dQ / dK-dV kernels.
//
// Every kernel has the same shape: a workgroup OWNS 128 rows (queries, or keys for dK/dV) and
// STREAMS 64-row tiles of the other side.  By the attention pattern of Section 3 the two sides
// are symmetric: an owned table token meets the question tokens plus the table tokens of its
// own row / column segment; an owned question token meets every non-pad token.
//
// Units of one (sequence, head) -- listed by the segment builder, see seg_layout.h:
//   local   table-token owners, up to 128 consecutive slots of the head kind's sorted order
//           that never straddle the boundary of a long segment; listed longest stream first
//   pad     ceil(P / 1024) pad owners (zero fill)
//   global  question-token owners.  Their streamed side is the whole sequence, so it is cut into
//           chunks that run as separate units and leave partial results, merged by a finalize
//           kernel.
// Workgroup -> unit is arithmetic on the workgroup index plus one record read: no counters, no
// atomics, no dependent loads.  Workgroup i serves queue i mod 8 (consecutive workgroups go to
// consecutive XCDs, so a queue stays on one XCD and the units of one (sequence, head) pair
// share an L2).  Column-head pairs are numbered c = b n_col + i and belong to queue c mod 8, row-
// head pairs r = b n_row + i to queue (r + B n_col) mod 8.  Order inside a queue, longest units first:
//   1. column heads: record 0 (the longest unit) of every pair, record 1 of every pair, ... up
//      to record T - 1
//   2. the first T / 8 + 2 question-token unit records of all pairs, the same way (all of the
//      real ones unless a sequence has more than 128 question tokens)
//   3. row heads, as in 1
//   4. what is left of the three lists (real records only in the cases named above)
// The two backward kernels run 2 before 1: there the question-token chunks are as long as the
// column-head units, and more of both exist than workgroup slots, so whichever kind comes second
// has members that start late and end last; the chunks first measured 1-6 us better on four of
// the five benchmark shapes and the same on the fifth.  In the forward the empty records at the
// end of 2 (a sequence with few chunks) would then sit in front of every column-head unit, which
// cost more than the order won.
// Records of kind "none" pad every pair to the same count; their workgroups exit at once.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_common.h"

namespace mate {

constexpr int kThreads = 256;
constexpr int kFinalizeBlocks = 4; // workgroups per (b,h) in the finalize kernels (32 rows each, strided)

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

// ---- workgroup -> unit ---------------------------------------------------------------------
struct Work {
  int bh, view;
  UnitPlan u;
};

inline int unit_grid(int B, int H, int N, int n_col) {
  const int T = owner_slots(N), U = view_units(N), nc = (B * n_col + 7) / 8, nr = (B * (H - n_col) + 7) / 8;
  return 8 * ((nc + nr) * U + (nc + nr) * T);
}

// Entry i of the head order.  A byte indexed by a run-time value would be fetched with a vector
// load (a memory round trip at the start of every workgroup); the containing 32-bit word comes
// through the scalar cache with the other kernel arguments.
__device__ inline int head_at(const AttnArgs& a, int i) {
  const unsigned word = reinterpret_cast<const unsigned*>(a.head_order)[i >> 2];
  return (word >> (8 * (i & 3))) & 0xffu;
}

// Returns false if this workgroup has nothing to do.  Everything here is wave-uniform and
// stays in scalar registers.
template <bool kChunksFirst>
__device__ inline bool take_unit(const AttnArgs& a, Work& w) {
  const int T = a.seg.tiles, U = a.seg.units, N = a.N, n_col = a.n_col, n_row = a.H - n_col;
  const int q = blockIdx.x & 7;
  // row-head pairs are dealt to the queues starting where the column-head pairs stopped, so that
  // a handful of pairs still spreads over as many XCDs as possible
  const int qr = (q - a.B * n_col) & 7;
  const int nc = (a.B * n_col - q + 7) >> 3, nr = (a.B * n_row - qr + 7) >> 3;  // pairs of this queue
  // Records are listed longest first and the empty ones last, and how many are real is only
  // known on the device: a workgroup that finds an empty record leaves at once, but it still
  // took a slot for a microsecond, and a thousand of them ahead of real units delay those by
  // several.  So the early part of each list (where the real records are unless a sequence is
  // filled to the last position, resp. has more than 128 question tokens) comes first for all
  // three kinds of unit, the remainders after them.
  const int E = min(U, T), T1 = min(T, (T >> 3) + 2);
  int t = blockIdx.x >> 3;
  // region -> (first pair, pairs, first record, records per pair)
  const int n_all = nc + nr;
  // the first two regions: column heads then question-token owners (early parts), or the reverse
  const int len_a = kChunksFirst ? n_all * T1 : nc * E, len_b = kChunksFirst ? nc * E : n_all * T1;
  bool glob = kChunksFirst;
  int first = 0, pairs = glob ? n_all : nc, k0 = 0, per = glob ? T1 : E;
  if (t >= len_a) {
    t -= len_a; glob = !kChunksFirst; pairs = glob ? n_all : nc; per = glob ? T1 : E;
    if (t >= len_b) {                      // row heads, early part
      t -= len_b; first = nc; pairs = nr; k0 = 0; per = E; glob = false;
      if (t >= nr * E) {                   // column heads, rest
        t -= nr * E; first = 0; pairs = nc; k0 = E; per = U - E;
        if (t >= nc * (U - E)) {           // row heads, rest
          t -= nc * (U - E); first = nc; pairs = nr;
          if (t >= nr * (U - E)) {         // question-token owners, rest
            t -= nr * (U - E); first = 0; pairs = n_all; k0 = T1; per = T - T1; glob = true;
          }
        }
      }
    }
  }
  if (pairs <= 0) return false;
  // The hardware hands consecutive workgroups of an XCD to its shader engines in rotation and
  // stalls when the engine whose turn it is has no room, so each engine must see the same mix
  // of units: the pair order rotates from sweep to sweep.
  const int kk = t / pairs, j = first + (t + kk) % pairs, k = k0 + kk;
  if (kk >= per) return false;
  int b, h;
  if (j < nc) {
    const int c = q + 8 * j;
    b = c / n_col;
    h = head_at(a, c % n_col);
    w.view = 1;
  } else {
    const int r = qr + 8 * (j - nc);
    b = r / n_row;
    h = head_at(a, n_col + r % n_row);
    w.view = 0;
  }
  w.bh = b * a.H + h;
  const int4* rec = glob ? a.seg.gunit + ((size_t)b * T + k) * 2
                         : a.seg.unit[w.view] + ((size_t)b * U + k) * 2;
  // The header is fetched together with the record (one scalar round trip for both): tables
  // built for another (B, N), or never built, make every workgroup leave before it uses a word
  // of them.  All of these reads stay inside the mate_segments_bytes(B, N) bytes the caller
  // must provide.
  const int h_magic = a.seg.hdr[0], h_B = a.seg.hdr[1], h_N = a.seg.hdr[2];
  const int4 r0 = rec[0], r1 = rec[1];
  const int* cnt = a.seg.counts + (size_t)b * kCountWords;
  UnitPlan& u = w.u;
  u.kind = r0.x;
  if (h_magic != kMagic || h_B != a.B || h_N != a.N) return false;
  if (u.kind == UNIT_NONE) return false;
  u.t0 = r0.y;
  u.s_lo = r0.z;
  u.s_hi = r0.w;
  u.t_begin = r1.x;
  u.t_end = r1.y;
  u.part = r1.z;
  u.G = cnt[C_G];
  u.L = cnt[C_L];
  u.P = cnt[C_P];
  u.n_t0 = (u.G + BN - 1) / BN;
  const int* perm_v = a.seg.perm[w.view] + (size_t)b * N;
  u.str_list = glob ? a.seg.perm[0] + (size_t)b * N : perm_v;  // row order: the contiguous one
  u.own_list = glob ? a.seg.global_idx + (size_t)b * N
                    : u.kind == UNIT_LOCAL ? perm_v : a.seg.pad_idx + (size_t)b * N;
  u.own_count = glob ? u.G : u.kind == UNIT_LOCAL ? r1.w : u.P;
  return true;
}

// Streamed tile t of a unit: which index list, first slot, last valid slot.
__device__ inline void tile_source(const UnitPlan& u, const int* global_idx, int t,
                                   const int*& list, int& base, int& last) {
  if (t < u.n_t0) { list = global_idx; base = t * BN; last = u.G - 1; }
  else { list = u.str_list; base = u.s_lo + (t - u.n_t0) * BN; last = u.s_hi - 1; }
}

// Per-lane view of the owned row: position, and the streamed-slot window it may meet.
struct OwnedRow {
  int stage_tok;      // token position of owned row threadIdx.x (-1 past the end or past row 127):
                      // what the epilogue's row table holds, fetched together with `pos`
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
  {
    const int row = u.t0 + (int)threadIdx.x;
    r.stage_tok = threadIdx.x < BM && row < u.own_count ? u.own_list[row] : -1;
  }
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

// Final results: C tile pairs (columns = owned rows, registers = head dims) scaled, rounded to
// bf16, transposed through LDS and stored as whole 128-byte token rows.  `stage` needs 16 KB per
// tensor: 128 rows of 128 bytes whose 16-byte chunks are XOR-swizzled with the row number so
// that both the column-wise writes and the row-wise reads spread over all banks.  One barrier;
// the staging area must not be reused by the caller afterwards without another one.
template <int kTensors>
__device__ inline void store_owned_rows(const f32x16 (*acc[kTensors])[2], const float (&mul)[kTensors],
                                        unsigned short* const (&out)[kTensors], char* stage,
                                        const int* row_tok, int wave, int lane) {
  const int m = lane & 31, hl = lane >> 5;
  const int wrow = wave * 32 + m;
#pragma unroll
  for (int x = 0; x < kTensors; ++x)
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x16& a = (*acc[x])[db];
        uint2 w;
        w.x = f32_to_bf16_bits(a[4 * g] * mul[x]) | ((unsigned)f32_to_bf16_bits(a[4 * g + 1] * mul[x]) << 16);
        w.y = f32_to_bf16_bits(a[4 * g + 2] * mul[x]) | ((unsigned)f32_to_bf16_bits(a[4 * g + 3] * mul[x]) << 16);
        *reinterpret_cast<uint2*>(stage + x * (BM * 128) + wrow * 128 + (((4 * db + g) ^ (wrow & 7)) << 4) + 8 * hl) = w;
      }
  __syncthreads();
#pragma unroll
  for (int x = 0; x < kTensors; ++x)
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = wave * 32 + it * 8 + (lane >> 3), piece = lane & 7;
      const int tok = row_tok[row];
      if (tok >= 0)
        *reinterpret_cast<uint4*>(out[x] + (size_t)tok * kD + piece * 8) =
            *reinterpret_cast<const uint4*>(stage + x * (BM * 128) + row * 128 + ((piece ^ (row & 7)) << 4));
    }
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

// Zero fill of the rows of a pad unit in kTensors tensors.  The positions of all the rows a
// thread will write are loaded first (independent loads, one round trip), then the stores go
// out back to back.
template <int kTensors>
__device__ inline void zero_pad_rows(unsigned short* const (&out)[kTensors], const UnitPlan& u, int tid) {
  constexpr int kRounds = kPadSlots * 8 / kThreads;  // rows of 8 pieces; 32 rows per round
  const int piece = tid & 7;
  int tok[kRounds];
#pragma unroll
  for (int i = 0; i < kRounds; ++i) {
    const int row = u.t0 + (tid >> 3) + i * (kThreads / 8);
    tok[i] = row < u.own_count ? u.own_list[row] : -1;
  }
#pragma unroll
  for (int x = 0; x < kTensors; ++x)
#pragma unroll
    for (int i = 0; i < kRounds; ++i)
      if (tok[i] >= 0)
        *reinterpret_cast<uint4*>(out[x] + (size_t)tok[i] * kD + piece * 8) = make_uint4(0, 0, 0, 0);
}

__device__ inline bool tables_match(const AttnArgs& a) {
  return a.seg.hdr[0] == kMagic && a.seg.hdr[1] == a.B && a.seg.hdr[2] == a.N;
}

// Workspace carving (float words).  Partial buffers are per (b,h): [UG][BM][64].
__host__ __device__ inline size_t part_words_per_bh(int N) { return (size_t)owner_slots(N) * BM * kD; }
__host__ __device__ inline size_t stat_words_per_bh(int N) { return (size_t)owner_slots(N) * BM * 2; }

}  // namespace mate
