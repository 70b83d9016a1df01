// Work decomposition shared by the bf16 MFMA forward / dQ / dK-dV kernels.
//
// Every kernel has the same shape: a workgroup OWNS 128 rows (queries, or keys for dK/dV) and
// STREAMS 64-row tiles of the other side.  By the attention pattern of Section 3 the two sides
// are symmetric: an owned table token meets the question tokens plus the table tokens of its
// own row / column segment; an owned question token meets every non-pad token.
//
// Units of one (sequence, head):
//   local   n_lt = ceil(L / 128) table-token owners, 128 consecutive slots of the head kind's
//           sorted order
//   global  question-token owners.  Their streamed side is the whole sequence, so it is cut into
//           chunks of >= kMinChunkTiles tiles that run as separate units and leave partial
//           results, merged by a finalize kernel.  n_gt * n_chunks <= UG = ceil(N / 128).
//   pad     n_pt = ceil(P / 128) pad owners (zero fill)
// G, L, P live on the device, so a small plan kernel counts the units and lays them out in
// eight work queues, one per XCD (queue q holds the (sequence, head) pairs b H + h = q mod 8, so
// that the units of one pair share an L2).  Every workgroup draws one ticket from the queue of
// its own XCD and steals from the others when that runs dry.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_common.h"

namespace mate {

constexpr int BM = 128;            // owned rows per workgroup (32 per wavefront)
constexpr int BN = 64;             // streamed rows per tile
constexpr int kThreads = 256;
constexpr int kFinalizeBlocks = 4; // workgroups per (b,h) in the finalize kernels (32 rows each, strided)
constexpr int kMinChunkTiles = 8;  // streamed tiles per chunk of a question-token owner

__host__ __device__ inline int owner_slots(int N) { return (N + BM - 1) / BM; }  // UG

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

// ---- plan buffer (ints, in the caller's workspace) -------------------------------------------
//   [0, 16)    ticket counters: [kernel slot 0..1][queue 0..7]
//   [32 + q]   tickets of queue q
//   [40 + q]   (sequence, head) pairs of queue q: bh = q + 8 j, j < pairs
//   [48 + q]   the largest number of table-token tiles of one of those pairs
//   [64 + (2 q + k)(nq + 1) + j]  k = 0: exclusive prefix over the queue's pairs of their pad
//              units, k = 1: of their question-token units; nq = ceil(B H / 8)
// Ticket order of a queue: table-token tile 0 of every pair, tile 1 of every pair, ... (tickets
// of pairs that have fewer tiles are empty), then the pad units, then the question-token units.
constexpr int kPlanCounters = 0, kPlanTotal = 32, kPlanPairs = 40, kPlanMost = 48, kPlanPref = 64;
__host__ __device__ inline int plan_nq(int BH) { return (BH + 7) >> 3; }
__host__ __device__ inline size_t plan_words(int BH) {
  return (size_t)kPlanPref + 16 * (size_t)(plan_nq(BH) + 1);
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

__device__ inline UnitPlan plan_base(const AttnArgs& a, int b) {
  const int* cnt = a.seg.counts + (size_t)b * kCountWords;
  UnitPlan u;
  u.kind = UNIT_NONE;
  u.G = cnt[C_G];
  u.L = cnt[C_L];
  u.P = cnt[C_P];
  u.part = -1;
  u.n_t0 = (u.G + BN - 1) / BN;
  u.t_begin = u.t_end = 0;
  return u;
}
// Table-token owner described by `desc` = (first slot, streamed window lo, hi) of (b, view).
__device__ inline UnitPlan plan_local(const AttnArgs& a, int b, int view, int4 desc) {
  UnitPlan u = plan_base(a, b);
  u.kind = UNIT_LOCAL;
  u.t0 = desc.x;
  u.own_list = a.seg.perm[view] + (size_t)b * a.N;
  u.own_count = u.L;
  u.str_list = u.own_list;
  u.s_lo = desc.y;
  u.s_hi = desc.z;
  u.t_end = u.n_t0 + (u.s_hi - u.s_lo + BN - 1) / BN;
  return u;
}
// Question-token unit number `gu` of sequence b: owner tile gu / n_chunks, chunk gu % n_chunks.
__device__ inline UnitPlan plan_global(const AttnArgs& a, int b, int gu) {
  UnitPlan u = plan_base(a, b);
  const int N = a.N;
  const GlobalSplit s = global_split(u.G, u.L, N);
  const int gt = gu / s.n_chunks, c = gu % s.n_chunks;
  u.kind = UNIT_GLOBAL;
  u.t0 = gt * BM;
  u.own_list = a.seg.global_idx + (size_t)b * N;
  u.own_count = u.G;
  u.str_list = a.seg.perm[0] + (size_t)b * N;  // row order: the contiguous one
  u.s_lo = 0;
  u.s_hi = u.L;
  u.t_begin = c * s.per;
  u.t_end = min(s.n_st, u.t_begin + s.per);
  if (s.n_chunks > 1) u.part = gu;
  return u;
}
__device__ inline UnitPlan plan_pad(const AttnArgs& a, int b, int tile) {
  UnitPlan u = plan_base(a, b);
  u.kind = UNIT_PAD;
  u.t0 = tile * BM;
  u.own_list = a.seg.pad_idx + (size_t)b * a.N;
  u.own_count = u.P;
  return u;
}

// Development aid (compiled out unless MATE_TRACE is defined): one record per unit with its
// start / end time (100 MHz wall clock), hardware placement and description.
#ifdef MATE_TRACE
#define MATE_TRACE_BEGIN const long long t_start_ = wall_clock64();
#define MATE_TRACE_END(kernel_no, q, t, info)                                              \
  if (a.trace && threadIdx.x == 0 && (t) < 8192) {                                         \
    long long* r_ = a.trace + ((size_t)(kernel_no) * (1 << 16) + (q) * 8192 + (t)) * 4;    \
    r_[0] = t_start_;                                                                      \
    r_[1] = wall_clock64();                                                                \
    r_[2] = (info);                                                                        \
    r_[3] = ((long long)__builtin_amdgcn_s_getreg(63508) << 32) |                          \
            (unsigned)__builtin_amdgcn_s_getreg(63492);                                    \
  }
#else
#define MATE_TRACE_BEGIN
#define MATE_TRACE_END(kernel_no, q, t, info) (void)(info);
#endif

// ---- work queues -------------------------------------------------------------------------------
struct Work {
  int bh, view;
  UnitPlan u;
};

__device__ inline int xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | 20) & 7; }  // XCC_ID[3:0]

// Ticket `t` of queue `q` -> which (b,h), which unit (kind UNIT_NONE: an empty ticket).  All
// inputs wave-uniform.
__device__ inline Work decode_ticket(const AttnArgs& a, int q, int t) {
  const int nq = plan_nq(a.B * a.H);
  const int pairs = a.plan[kPlanPairs + q], most = a.plan[kPlanMost + q];
  Work w;
  if (t < pairs * most) {
    const int j = t % pairs, k = t / pairs;
    w.bh = q + 8 * j;
    const int b = w.bh / a.H;
    w.view = a.head_kind[w.bh % a.H];
    const int4 desc = a.seg.tile_desc[w.view][(size_t)b * a.seg.tiles + k];
    if (desc.x < 0) w.u.kind = UNIT_NONE;
    else w.u = plan_local(a, b, w.view, desc);
    return w;
  }
  t -= pairs * most;
  const int* pref = a.plan + kPlanPref + 2 * q * (nq + 1);
  const int is_global = t >= pref[nq];
  if (is_global) {
    t -= pref[nq];
    pref += nq + 1;
  }
  int lo = 0, hi = nq;  // largest j with pref[j] <= t
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (pref[mid] <= t) lo = mid; else hi = mid;
  }
  w.bh = q + 8 * lo;
  const int b = w.bh / a.H;
  w.view = a.head_kind[w.bh % a.H];
  w.u = is_global ? plan_global(a, b, t - pref[lo]) : plan_pad(a, b, t - pref[lo]);
  return w;
}

// One unit per workgroup: draw a ticket from the queue of this workgroup's XCD, or, if that
// queue is exhausted, from the others in turn.  The host launches as many workgroups as there
// can be units (upper bound from B, H, N); the surplus finds every queue empty and exits.
// (A persistent loop over tickets was tried and lost: with the unit body inside a loop the
// compiler runs out of scalar registers and moves the wave-uniform bookkeeping into vector
// registers and vector ALU work; the hardware's workgroup dispatcher is the faster loop.)
// Returns false if there is nothing left to do.
__device__ inline bool take_unit(const AttnArgs& a, int kernel_slot, Work& w, int& queue, int& ticket) {
  __shared__ int s_ticket, s_queue;
  if (threadIdx.x == 0) {
    int* counters = a.plan + kPlanCounters + 8 * kernel_slot;
    int q = xcc_id(), t = -1;
    for (int tried = 0; tried < 8; ++tried, q = (q + 1) & 7) {
      if (counters[q] >= a.plan[kPlanTotal + q]) continue;  // looks exhausted: do not bump it
      t = atomicAdd(&counters[q], 1);
      if (t < a.plan[kPlanTotal + q]) break;
      t = -1;
    }
    s_ticket = t;
    s_queue = q;
  }
  __syncthreads();
  // wave-uniform values: keep the whole unit description in scalar registers
  ticket = __builtin_amdgcn_readfirstlane(s_ticket);
  queue = __builtin_amdgcn_readfirstlane(s_queue);
  if (ticket < 0) return false;
  w = decode_ticket(a, queue, ticket);
  return w.u.kind != UNIT_NONE;
}
inline int units_upper_bound(int B, int H, int N) { return B * H * (2 * owner_slots(N) + 1); }

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
