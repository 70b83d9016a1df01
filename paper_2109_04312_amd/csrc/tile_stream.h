// The streaming loop shared by the forward, dQ and dK/dV kernels: a ring of NS LDS stages, each
// holding one 64-row tile of two tensors (plus, optionally, one float per row of a third
// array), filled NS - 1 tiles ahead of the compute by asynchronous global->LDS loads.
//
// The token indices of a tile's 64 rows travel the same way (one word per lane into a ring
// shared by the workgroup; wavefront t mod 4 fetches the indices of tile t), a further NS - 1
// tiles ahead, so no load of the loop has a register destination and the only waits are the
// explicit ones in acquire().  `since[k]` counts this wavefront's vector loads issued after
// the data loads of tile (current + k).  An index load is issued just before the data loads of
// the same iteration, so the wait for that tile's data NS - 1 iterations later also retires
// it, and the barrier that follows the wait publishes it to the other wavefronts -- in the very
// iteration that first reads it.
#pragma once
#include <hip/hip_runtime.h>

#include "d2l.h"
#include "stream_plan.h"

namespace mate {

constexpr int kIdxSlots = 8;  // >= 2 NS - 1 tiles of indices live at once (power of two)

// NS = ring stages: tiles in flight + the one being consumed (2 <= NS <= 4).
template <int kStageBytes, int NS>
struct TileStream {
  const UnitPlan& u;
  const int* global_idx;
  char* stages;               // NS * kStageBytes of LDS
  int (*ring)[BN];            // the workgroup's index ring [kIdxSlots][64]
  const unsigned short* X0;   // tensor staged at stage offset 0
  const unsigned short* X1;   // tensor staged at stage offset kTileBytes
  const float* row_src;       // optional: one float per streamed row -> stage offset row_off
  int row_off;
  int wave, lane;
  LoadLane ll;
  int since[NS];

  __device__ TileStream(const UnitPlan& u_, const int* gidx, char* st, int (*rg)[BN],
                        const unsigned short* x0, const unsigned short* x1, const float* rs,
                        int row_off_, int wave_, int lane_)
      : u(u_), global_idx(gidx), stages(st), ring(rg), X0(x0), X1(x1), row_src(rs), row_off(row_off_), wave(wave_),
        lane(lane_), ll(make_load_lane(wave_, lane_)) {
#pragma unroll
    for (int k = 0; k < NS; ++k) since[k] = 0;
  }

  __device__ void note(int n) {
#pragma unroll
    for (int k = 0; k < NS; ++k) since[k] += n;
  }
  __device__ void issue_idx(int t) {
    const int* list; int base, last;
    if (wave != (t & 3)) return;
    tile_source(u, global_idx, t, list, base, last);
    issue_row_words(list, min(base + lane, last), &ring[t & (kIdxSlots - 1)][0]);
    note(1);
  }
  __device__ void issue_data(int t, int k /* = t - current tile */) {
    const int* r = ring[t & (kIdxSlots - 1)];
    const int x0 = r[ll.row0], x1 = r[ll.row0 + 8];
    char* st = stages + ((t - u.t_begin) % NS) * kStageBytes;
    issue_tile(X0, x0, x1, ll, st, wave);
    issue_tile(X1, x0, x1, ll, st + kTileBytes, wave);
    note(4);
    if (row_src) {
      issue_row_words(row_src, r[lane], st + row_off);
      note(1);
    }
    since[k] = 0;
  }
  // Before the loop, in two steps so that the caller's own first loads (which rows it owns) can
  // travel together with the first index loads, and its row loads together with the first tiles:
  // begin() issues the indices of the first 2 NS - 2 tiles; prime() waits for them and issues the
  // data of the first NS - 1 tiles.
  __device__ void begin() {
#pragma unroll
    for (int s = 0; s < 2 * NS - 2; ++s)
      if (u.t_begin + s < u.t_end) issue_idx(u.t_begin + s);
  }
  __device__ void prime() {
    wait_vmcnt_le(0);
    barrier_no_fence();  // every wavefront's share of the first indices is in the ring
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (u.t_begin + s < u.t_end) issue_data(u.t_begin + s, s);
  }
  // Top of iteration t: tile t is complete in LDS for every wavefront, tile t - 1's stage is
  // free; keep the pipeline full.  Returns the stage holding tile t.
  __device__ const char* acquire(int t) {
    // my share of tile t has landed (with two stages nothing is ever issued between a tile's
    // data and the wait for it, so the count is known at compile time)
    // (otherwise at most NS - 2 tiles' worth: 5 loads per tile and one index load each)
    if (NS == 2) wait_vmcnt_le<0>(0); else wait_vmcnt_le<6 * (NS - 2)>(since[0]);
    barrier_no_fence();       // ... everyone's has, and everyone is done with tile t - 1
    if (t + 2 * NS - 2 < u.t_end) issue_idx(t + 2 * NS - 2);
    if (t + NS - 1 < u.t_end) issue_data(t + NS - 1, NS - 1);
    return stages + ((t - u.t_begin) % NS) * kStageBytes;
  }
  __device__ void release() {
#pragma unroll
    for (int k = 0; k + 1 < NS; ++k) since[k] = since[k + 1];
  }
};

}  // namespace mate
