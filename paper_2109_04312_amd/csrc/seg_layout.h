// Layout of the caller-owned segment-table buffer (all int32 words), shared by the builder
// kernel and the attention kernels.  Every array starts on a 16-byte boundary.
//
//   hdr[16]            magic, B, N, 0, global-part limit and radius of the bucketed mode (N and 0
//                      without it), rest 0
//   counts[B][12]      G, L, P (pad count), S_row, S_col, bad ids seen (rows, cols), rest 0
//   global_idx[B][N]   ascending positions of GLOBAL tokens; entries past G are not written
//   pad_idx[B][N]      ascending positions of PAD tokens; entries past P are not written
//   gunit[B][T][8]     work units of question-token owners (T = ceil(N / 128)), see below
//   per view v (0 rows, 1 columns):
//     perm[B][N]         sorted slot -> token position; entries past L are not written
//     seg_off[B][N+1]    first slot of each segment, L at index S; nothing written past that
//     seg_of_tok[B][N]   token position -> segment index, -1 for GLOBAL / PAD
//     slot_rng[B][N][2]  per sorted slot: [first slot, one-past-last slot) of its window = its
//                        segment, in bucketed mode cut to its own and the two adjacent buckets
//     unit[B][U][8]      work units of table-token owners (up to 128 consecutive slots of the
//                        sorted order each), longest streamed side first, then of pad owners
//                        (1024 pad positions each), then empty records; U = view_units(N)
//
// A work unit is what one workgroup of the bf16 attention kernels does: it owns up to 128 rows
// and streams 64-row tiles of the other side.  Record (8 words):
//   kind (0 none, 1 question-token owner, 2 table-token owner, 3 pad owner), first owned slot,
//   streamed sorted-slot window [lo, hi), first and one-past-last streamed tile, partial-result
//   slot or -1, one past the last owned slot (table-token owners)
// For a table-token owner [lo, hi) is the union of the windows of its slots.  Its slots are a
// 128-slot piece of a "run": a segment of at least kBigSegment slots is a run of its own, the
// shorter segments between two such segments form one run.  So no unit straddles the boundary
// of a long segment (it would stream both segments' windows with half of its wavefronts idle
// on each, and be the longest unit of the launch).  If that needs more records than there
// are, the sorted order is cut every 128 slots regardless of segments.
// The streamed side of question-token owners is the whole sequence; it is cut into chunks of at
// least kMinChunkTiles tiles, one unit each, that leave partial results.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace mate {

constexpr int kMagic = 0x4D415445;  // "MATE"
constexpr int kHdrWords = 16;
constexpr int kCountWords = 12;
enum { C_G = 0, C_L = 1, C_P = 2, C_SROW = 3, C_SCOL = 4 };
constexpr int kTileSlots = 128;    // sorted slots per tile (= rows owned by one workgroup)
constexpr int kMaxTiles = 128;     // MATE_MAX_N / kTileSlots
constexpr int kPadSlots = 1024;    // pad positions zero-filled by one pad unit
constexpr int kUnitWords = 8;
constexpr int kBigSegment = 128;   // a segment this long starts a unit of its own
constexpr int BM = kTileSlots;     // owned rows per workgroup (32 per wavefront)
constexpr int BN = 64;             // streamed rows per tile
constexpr int kMinChunkTiles = 16; // streamed tiles per chunk of a question-token owner
enum { UNIT_NONE = 0, UNIT_GLOBAL = 1, UNIT_LOCAL = 2, UNIT_PAD = 3 };

__host__ __device__ inline int owner_slots(int N) { return (N + BM - 1) / BM; }  // T
// Unit records per (sequence, view): table-token owners, pad owners, spare.
__host__ __device__ inline int view_units(int N) { const int T = owner_slots(N); return T + T / 2 + 2; }

// How the streamed side of question-token owners is chunked.  n_gt * n_chunks <= T.
struct GlobalSplit {
  int n_gt;      // owner tiles of question tokens
  int n_st;      // streamed tiles in total: question tiles then table tiles
  int n_chunks;  // units per owner tile (>= 1); partial results are used iff n_chunks > 1
  int per;       // streamed tiles per chunk
};
__host__ __device__ inline GlobalSplit global_split(int G, int L, int N) {
  GlobalSplit s;
  s.n_gt = (G + BM - 1) / BM;
  s.n_st = (G + BN - 1) / BN + (L + BN - 1) / BN;
  const int want = (s.n_st + kMinChunkTiles - 1) / kMinChunkTiles;
  const int cap = s.n_gt ? owner_slots(N) / s.n_gt : 1;
  const int n = want < cap ? (want > 1 ? want : 1) : (cap > 1 ? cap : 1);
  s.per = (s.n_st + n - 1) / n;
  s.n_chunks = s.per ? (s.n_st + s.per - 1) / s.per : 1;  // drop empty trailing chunks
  return s;
}

__host__ __device__ inline size_t align4(size_t w) { return (w + 3) & ~size_t(3); }

struct SegLayout {
  int B, N;
  int tiles, units;
  size_t counts, global_idx, pad_idx, gunit, view0, view_stride, perm, seg_off, seg_of_tok,
      slot_rng, unit, total;

  __host__ __device__ SegLayout(int B_, int N_) : B(B_), N(N_) {
    size_t bn = align4((size_t)B * N);
    counts = kHdrWords;
    global_idx = counts + align4((size_t)B * kCountWords);
    pad_idx = global_idx + bn;
    tiles = (N + kTileSlots - 1) / kTileSlots;
    units = view_units(N);
    gunit = pad_idx + bn;
    view0 = gunit + (size_t)B * tiles * kUnitWords;
    perm = 0;
    seg_off = perm + bn;
    seg_of_tok = seg_off + align4((size_t)B * (N + 1));
    slot_rng = seg_of_tok + bn;
    unit = slot_rng + align4((size_t)B * N * 2);
    view_stride = unit + (size_t)B * units * kUnitWords;
    total = view0 + 2 * view_stride;
  }
};

// Read-only view handed to the attention kernels.
struct SegTables {
  const int* hdr;
  const int* counts;      // [B][12]
  const int* global_idx;  // [B][N]
  const int* pad_idx;     // [B][N]
  const int* perm[2];     // [B][N]
  const int* seg_off[2];  // [B][N+1]
  const int* seg_of_tok[2];
  const int2* slot_rng[2];  // [B][N]
  const int4* unit[2];    // [B][units][2]
  const int4* gunit;      // [B][tiles][2]
  int tiles, units;
};

inline SegTables make_tables(const void* segments, int B, int N) {
  SegLayout L(B, N);
  const int* w = static_cast<const int*>(segments);
  SegTables t;
  t.hdr = w;
  t.counts = w + L.counts;
  t.global_idx = w + L.global_idx;
  t.pad_idx = w + L.pad_idx;
  for (int v = 0; v < 2; ++v) {
    const int* base = w + L.view0 + v * L.view_stride;
    t.perm[v] = base + L.perm;
    t.seg_off[v] = base + L.seg_off;
    t.seg_of_tok[v] = base + L.seg_of_tok;
    t.slot_rng[v] = reinterpret_cast<const int2*>(base + L.slot_rng);
    t.unit[v] = reinterpret_cast<const int4*>(base + L.unit);
  }
  t.gunit = reinterpret_cast<const int4*>(w + L.gunit);
  t.tiles = L.tiles;
  t.units = L.units;
  return t;
}

}  // namespace mate
