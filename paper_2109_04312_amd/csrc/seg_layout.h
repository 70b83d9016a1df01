// Layout of the caller-owned segment-table buffer (all int32 words), shared by the builder
// kernel and the attention kernels.  Every array starts on a 16-byte boundary.
//
//   hdr[16]            magic, B, N, status (0 ok, 1 = bad id / flag seen), rest 0
//   counts[B][12]      G, L, P (pad count), S_row, S_col, bad ids seen (rows, cols), 0,
//                      streamed 64-slot tiles of all table-token units (rows, cols), 0, 0
//   global_idx[B][N]   ascending positions of GLOBAL tokens, -1 past G
//   pad_idx[B][N]      ascending positions of PAD tokens, -1 past P
//   per view v (0 rows, 1 columns):
//     perm[B][N]         sorted slot -> token position, -1 past L
//     seg_off[B][N+1]    first slot of each segment, L at index S, -1 past that
//     seg_of_tok[B][N]   token position -> segment index, -1 for GLOBAL / PAD
//     slot_rng[B][N][2]  per sorted slot: [first slot, one-past-last slot) of its segment
//     tile_desc[B][T][4] per 128-slot tile of the sorted order (T = ceil(N / 128)): first slot,
//                        then the slot window [lo, hi) spanned by the segments the tile
//                        touches, 0; first slot -1 past the last tile
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace mate {

constexpr int kMagic = 0x4D415445;  // "MATE"
constexpr int kHdrWords = 16;
constexpr int kCountWords = 12;
enum { C_G = 0, C_L = 1, C_P = 2, C_SROW = 3, C_SCOL = 4, C_COST_ROW = 8, C_COST_COL = 9 };
constexpr int kTileSlots = 128;    // sorted slots per tile (= rows owned by one workgroup)
constexpr int kMaxTiles = 128;     // MATE_MAX_N / kTileSlots

__host__ __device__ inline size_t align4(size_t w) { return (w + 3) & ~size_t(3); }

struct SegLayout {
  int B, N;
  int tiles;
  size_t counts, global_idx, pad_idx, view0, view_stride, perm, seg_off, seg_of_tok, slot_rng,
      tile_desc, total;

  __host__ __device__ SegLayout(int B_, int N_) : B(B_), N(N_) {
    size_t bn = align4((size_t)B * N);
    counts = kHdrWords;
    global_idx = counts + align4((size_t)B * kCountWords);
    pad_idx = global_idx + bn;
    view0 = pad_idx + bn;
    perm = 0;
    seg_off = perm + bn;
    seg_of_tok = seg_off + align4((size_t)B * (N + 1));
    slot_rng = seg_of_tok + bn;
    tiles = (N + kTileSlots - 1) / kTileSlots;
    tile_desc = slot_rng + align4((size_t)B * N * 2);
    view_stride = tile_desc + (size_t)B * tiles * 4;
    total = view0 + 2 * view_stride;
  }
};

// Read-only view handed to the attention kernels.
struct SegTables {
  const int* hdr;
  const int* counts;      // [B][8]
  const int* global_idx;  // [B][N]
  const int* pad_idx;     // [B][N]
  const int* perm[2];     // [B][N]
  const int* seg_off[2];  // [B][N+1]
  const int* seg_of_tok[2];
  const int2* slot_rng[2];  // [B][N]
  const int4* tile_desc[2];  // [B][tiles]
  int tiles;
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
    t.tile_desc[v] = reinterpret_cast<const int4*>(base + L.tile_desc);
  }
  t.tiles = L.tiles;
  return t;
}

}  // namespace mate
