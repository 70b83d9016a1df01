// Layout of the caller-owned segment-table buffer (all int32 words), shared by the builder
// kernel and the attention kernels.  Every array starts on a 16-byte boundary.
//
//   hdr[16]            magic, B, N, status (0 ok, 1 = bad id / flag seen), rest 0
//   counts[B][8]       G, L, P (pad count), S_row, S_col, 0, 0, 0
//   global_idx[B][N]   ascending positions of GLOBAL tokens, -1 past G
//   pad_idx[B][N]      ascending positions of PAD tokens, -1 past P
//   per view v (0 rows, 1 columns):
//     perm[B][N]         sorted slot -> token position, -1 past L
//     seg_off[B][N+1]    first slot of each segment, L at index S, -1 past that
//     seg_of_tok[B][N]   token position -> segment index, -1 for GLOBAL / PAD
//     slot_rng[B][N][2]  per sorted slot: [first slot, one-past-last slot) of its segment
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace mate {

constexpr int kMagic = 0x4D415445;  // "MATE"
constexpr int kHdrWords = 16;
constexpr int kCountWords = 8;
enum { C_G = 0, C_L = 1, C_P = 2, C_SROW = 3, C_SCOL = 4 };

__host__ __device__ inline size_t align4(size_t w) { return (w + 3) & ~size_t(3); }

struct SegLayout {
  int B, N;
  size_t counts, global_idx, pad_idx, view0, view_stride, perm, seg_off, seg_of_tok, slot_rng, total;

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
    view_stride = slot_rng + align4((size_t)B * N * 2);
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
  }
  return t;
}

}  // namespace mate
