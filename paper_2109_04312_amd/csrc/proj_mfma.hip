// The projections either side of the attention, bf16 MFMA (gfx950):
//   QKV:  q[b,i,k,:] = W_Q^i x[b,k,:], likewise K and V -- the W^i X_k of the head equation of
//         Section 3 for all heads at once, written straight into the [B, H, N, 64] layout the
//         attention kernels read (the head split costs nothing);
//   out:  y[b,k,:] = W_O concat_i o[b,i,k,:], reading the attention output head by head in the
//         layout it was written in (no concatenation pass).
// Pad tokens are not computed when a whole token tile is padding, and are stored as zeros.
//
// Both are one kernel template: C^T[f, tok] = sum_k W[f, k] T[tok, k] with W rows (features) as
// the MFMA A operand and token rows as the B operand, so a lane owns a token column and its
// registers run over features -- the layout of the attention kernels' accumulators, and the same
// transposing epilogue through LDS to whole 128-byte rows.  Both operands are K-contiguous and
// are streamed in 64-row x 64-k tiles of 128-byte rows straight from global memory into LDS
// (global_load_lds_dwordx4), XOR-swizzled for conflict-free 16-byte operand reads, through a
// ring of stages with explicit vmcnt waits.
//
// Workgroup tile: kTokTiles x 64 tokens by kFeatTiles x 64 features; a wavefront owns 32 kBT
// tokens by 64 features (one head of Q, K or V).  Workgroup i runs on XCD i mod 8; every XCD
// takes a contiguous range of token tiles and walks the feature tiles fastest, so the token
// rows it streams stay in its L2 while the (small) weight matrix cycles.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "d2l.h"
#include "launch.h"
#include "mfma_common.h"

namespace mate {
namespace {

template <int kTokTiles_, int kFeatTiles_, int kWavesTok_, int kStages_>
struct ProjShape {
  static constexpr int kTokTiles = kTokTiles_, kFeatTiles = kFeatTiles_;
  static constexpr int kWavesTok = kWavesTok_, kWavesFeat = kFeatTiles_;  // 64 features per wavefront
  static constexpr int kWaves = kWavesTok * kWavesFeat;
  static constexpr int kThreadsP = 64 * kWaves;
  static constexpr int kBT = kTokTiles * 2 / kWavesTok;       // 32-token blocks per wavefront
  static constexpr int kStages = kStages_;
  static constexpr int kStageBytesP = (kTokTiles + kFeatTiles) * kTileBytes;
  static constexpr int kQuarters = 4 * (kTokTiles + kFeatTiles) / kWaves;  // 16-row loads per wavefront and stage
  static_assert(4 * (kTokTiles + kFeatTiles) % kWaves == 0, "loads must divide evenly");
  static_assert(kTokTiles * 2 % kWavesTok == 0, "token blocks must divide evenly");
};

struct ProjArgs {
  const unsigned short* w;       // [F][K] row-major
  const unsigned short* tok;     // kOut false: [B*N][K] row-major (x, or dy in the backward)
  const unsigned short* tok3[3]; // kOut true: [B][H][N][64] tensors whose heads are the k steps, one
                                 // after the other (o; or dq, dk, dv in the backward)
  const float* bias;             // [F] or null
  const unsigned char* flags;    // [B][N]
  unsigned short* out[3];        // QKV: q, k, v [B][H][N][64];  out: y [B][N][E] in out[0]
  int B, N, H, E;
  int F, K;                      // features, contraction length
  int tok_tiles_per_seq;         // ceil(N / tile tokens)
  int feat_tiles;                // F / tile features
  int total;                     // workgroups with work
};

// One stage: kTokTiles token tiles then kFeatTiles weight tiles of 64 rows x 128 bytes.
template <class S, bool kOut>
__global__ __launch_bounds__(S::kThreadsP, S::kWaves == 4 ? 2 : 1) void proj_kernel(ProjArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  constexpr int kTokRows = S::kTokTiles * 64, kFeatRows = S::kFeatTiles * 64;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = lane & 31, hl = lane >> 5;

  // workgroup -> (token tile, feature tile): XCD q owns a contiguous range of the linear order
  const int q = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int per = (a.total + 7) >> 3;
  const int idx = q * per + j;
  if (j >= per || idx >= a.total) return;
  const int tt = idx / a.feat_tiles, ft = idx - tt * a.feat_tiles;
  const int b = tt / a.tok_tiles_per_seq, n0 = (tt - b * a.tok_tiles_per_seq) * kTokRows;
  const int f0 = ft * kFeatRows;
  const int rows_valid = min(kTokRows, a.N - n0);

  const int wt = wave / S::kWavesFeat, wf = wave - wt * S::kWavesFeat;
  // where this wavefront's 64 features go: QKV -> tensor and head; out -> a 128-byte piece of y
  unsigned short* dst;
  size_t dst_stride;  // elements between consecutive tokens
  if (kOut) {
    dst = a.out[0] + ((size_t)b * a.N + n0) * a.E + f0 + 64 * wf;
    dst_stride = a.E;
  } else {
    const int head_slot = f0 / 64 + wf, t = head_slot / a.H, h = head_slot - t * a.H;
    dst = a.out[t] + (((size_t)b * a.H + h) * a.N + n0) * kD;
    dst_stride = kD;
  }
  const unsigned char* fl = a.flags + (size_t)b * a.N + n0;

  // a tile of padding only: zeros, no arithmetic.  The flags stay in LDS for the epilogue (read
  // from global memory there, every store would wait for a flag load and for the store before it).
  __shared__ unsigned char tok_flag[kTokRows];
  int any = 0;
  for (int r = tid; r < rows_valid; r += S::kThreadsP) {
    const unsigned char f = fl[r];
    tok_flag[r] = f;
    any |= f != 2;
  }
  any = __syncthreads_or(any);

  // ---- operand streams ------------------------------------------------------------------
  // token operand: row r of the tile at tok_base + r * tok_stride bytes, advancing tok_step
  // bytes per 64-wide k step; weights likewise
  const char* tok_base;
  unsigned tok_stride, tok_step;
  if (kOut) {  // k step = one head of one of the head-layout tensors
    tok_base = reinterpret_cast<const char*>((((size_t)b * a.H) * a.N + n0) * kD * 2);  // offset only
    tok_stride = kD * 2;
    tok_step = (unsigned)a.N * kD * 2;
  } else {
    tok_base = reinterpret_cast<const char*>(a.tok + ((size_t)b * a.N + n0) * a.E);
    tok_stride = (unsigned)a.E * 2;
    tok_step = 128;
  }
  const char* w_base = reinterpret_cast<const char*>(a.w + (size_t)f0 * a.K);
  const unsigned w_stride = (unsigned)a.K * 2;

  // this wavefront's share of a stage: kQuarters loads of 16 rows (two instructions of 8 rows)
  const LoadLane ll = make_load_lane(0, lane);  // row inside a 16-row group, swizzled chunk
  unsigned goff[S::kQuarters][2];
  int loff[S::kQuarters];
  bool is_w[S::kQuarters];
#pragma unroll
  for (int i = 0; i < S::kQuarters; ++i) {
    const int qi = wave + S::kWaves * i;          // quarter index in the stage
    const int tile = qi >> 2, r0 = (qi & 3) * 16 + ll.row0;
    loff[i] = tile * kTileBytes + (qi & 3) * 16 * 128;
    is_w[i] = tile >= S::kTokTiles;
    if (is_w[i]) {
      const int row = (tile - S::kTokTiles) * 64 + r0;
      goff[i][0] = (unsigned)row * w_stride + ll.chunk0 * 16;
      goff[i][1] = (unsigned)(row + 8) * w_stride + (ll.chunk0 ^ 2) * 16;
    } else {
      const int row = tile * 64 + r0;  // rows past the end of the sequence repeat the last one
      goff[i][0] = (unsigned)min(row, rows_valid - 1) * tok_stride + ll.chunk0 * 16;
      goff[i][1] = (unsigned)min(row + 8, rows_valid - 1) * tok_stride + (ll.chunk0 ^ 2) * 16;
    }
  }
  auto issue_stage = [&](int ks) {
    char* st = lds + (ks % S::kStages) * S::kStageBytesP;
    const char* tb;
    if (kOut) {
      const int t = ks / a.H, h = ks - t * a.H;
      const unsigned short* tensor = t == 0 ? a.tok3[0] : t == 1 ? a.tok3[1] : a.tok3[2];
      tb = reinterpret_cast<const char*>(tensor) + (size_t)tok_base + (size_t)h * tok_step;
    } else {
      tb = tok_base + (size_t)ks * tok_step;
    }
    const char* wb = w_base + (size_t)ks * 128;
#pragma unroll
    for (int i = 0; i < S::kQuarters; ++i) {
      const char* base = is_w[i] ? wb : tb;
      load_to_lds_16(base, goff[i][0], st + loff[i]);
      load_to_lds_16(base, goff[i][1], st + loff[i] + 8 * 128);
    }
  };

  f32x16 acc[2][S::kBT];
#pragma unroll
  for (int bf = 0; bf < 2; ++bf)
#pragma unroll
    for (int bt = 0; bt < S::kBT; ++bt) acc[bf][bt] = zero16();

  if (any) {
    const int nk = a.K / 64;
    int poff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) poff[ks] = plain_off(m, hl, ks);
#pragma unroll
    for (int s = 0; s < S::kStages - 1; ++s)
      if (s < nk) issue_stage(s);
    constexpr int kLoadsPerStage = 2 * S::kQuarters;
    for (int ks = 0; ks < nk; ++ks) {
      // stage ks has landed: everything but the younger stages' loads (fewer near the end)
      const int younger = min(S::kStages - 2, nk - 1 - ks);
      wait_vmcnt_le<kLoadsPerStage * (S::kStages - 2)>(younger * kLoadsPerStage);
      barrier_no_fence();  // ... for every wavefront, and everyone is done with stage ks - 1
      if (ks + S::kStages - 1 < nk) issue_stage(ks + S::kStages - 1);
      const char* st = lds + (ks % S::kStages) * S::kStageBytesP;
      const char* tok_t = st + wt * S::kBT * 32 * 128;
      const char* w_t = st + S::kTokTiles * kTileBytes + wf * 64 * 128;
      // operand fragments are read one 16-wide k slice ahead of the contractions that use them
      bf16x8 wfrag[2][2], tfrag[2][S::kBT];
      auto read_slice = [&](int buf, int k16) {
#pragma unroll
        for (int bf = 0; bf < 2; ++bf) wfrag[buf][bf] = read_plain(w_t + bf * 32 * 128, poff[k16]);
#pragma unroll
        for (int bt = 0; bt < S::kBT; ++bt) tfrag[buf][bt] = read_plain(tok_t + bt * 32 * 128, poff[k16]);
      };
      read_slice(0, 0);
#pragma unroll
      for (int k16 = 0; k16 < 4; ++k16) {
        if (k16 + 1 < 4) read_slice((k16 + 1) & 1, k16 + 1);
#pragma unroll
        for (int bf = 0; bf < 2; ++bf)
#pragma unroll
          for (int bt = 0; bt < S::kBT; ++bt)
            acc[bf][bt] = mfma(wfrag[k16 & 1][bf], tfrag[k16 & 1][bt], acc[bf][bt]);
      }
    }
  }
  __syncthreads();  // the stages are free: reuse them for the epilogue

  // ---- epilogue: + bias, round to bf16, transpose through this wavefront's own 4 KB of LDS,
  // store whole 128-byte pieces per token ------------------------------------------------------
  float4 bias4[2][4];
#pragma unroll
  for (int bf = 0; bf < 2; ++bf)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      bias4[bf][g] = a.bias && any ? *reinterpret_cast<const float4*>(a.bias + f0 + 64 * wf + 32 * bf + 8 * g + 4 * hl)
                                   : make_float4(0.f, 0.f, 0.f, 0.f);
  char* stage = lds + wave * (32 * 128);
#pragma unroll
  for (int bt = 0; bt < S::kBT; ++bt) {
#pragma unroll
    for (int bf = 0; bf < 2; ++bf)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x16& c = acc[bf][bt];
        const float4 bb = bias4[bf][g];
        uint2 v;
        v.x = f32_to_bf16_bits(c[4 * g] + bb.x) | ((unsigned)f32_to_bf16_bits(c[4 * g + 1] + bb.y) << 16);
        v.y = f32_to_bf16_bits(c[4 * g + 2] + bb.z) | ((unsigned)f32_to_bf16_bits(c[4 * g + 3] + bb.w) << 16);
        *reinterpret_cast<uint2*>(stage + m * 128 + (((4 * bf + g) ^ (m & 7)) << 4) + 8 * hl) = v;
      }
    // same wavefront writes and reads: LDS executes a wavefront's accesses in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = it * 8 + (lane >> 3), piece = lane & 7;
      const int r = (wt * S::kBT + bt) * 32 + row;  // token row inside the workgroup tile
      if (r < rows_valid) {
        uint4 v = *reinterpret_cast<const uint4*>(stage + row * 128 + ((piece ^ (row & 7)) << 4));
        if (tok_flag[r] == 2) v = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(dst + (size_t)r * dst_stride + piece * 8) = v;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

template <class S, bool kOut>
hipError_t launch_proj(ProjArgs a, int kernel_id, hipStream_t stream) {
  constexpr int kTokRows = S::kTokTiles * 64, kFeatRows = S::kFeatTiles * 64;
  a.tok_tiles_per_seq = (a.N + kTokRows - 1) / kTokRows;
  a.feat_tiles = a.F / kFeatRows;
  a.total = a.B * a.tok_tiles_per_seq * a.feat_tiles;
  const int grid = 8 * ((a.total + 7) / 8);
  const size_t lds_bytes = (size_t)S::kStages * S::kStageBytesP;
  // more than 64 KB of dynamic LDS has to be allowed explicitly (a host-side setting, no state here)
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_kernel<S, kOut>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  ProfileScope prof(kernel_id, stream);
  hipLaunchKernelGGL((proj_kernel<S, kOut>), dim3(grid), dim3(S::kThreadsP), lds_bytes, stream, a);
  return hipGetLastError();
}

// Two shapes.  Large: 256 tokens x 256 features, eight wavefronts of 128 x 64, two stages of
// 64 KB (one workgroup per CU): half the operand traffic per flop of the small shape and the
// faster of the two once its tiles fill the chip (measured on the 16384 x 3072 x 1024 product:
// 106 us against 122 us).  Small: 128 x 128, four wavefronts of 64 x 64, two workgroups per CU:
// for feature counts that are not a multiple of 256 and for products with few tiles.
using LargeShape = ProjShape<4, 4, 2, 2>;
using SmallShape = ProjShape<2, 2, 2, 2>;

template <bool kOut>
hipError_t launch_proj_any(const ProjArgs& a, int kernel_id, hipStream_t stream) {
  const long large_tiles = (long)a.B * ((a.N + 255) / 256) * (a.F / 256);
  if (a.F % 256 == 0 && large_tiles >= 256) return launch_proj<LargeShape, kOut>(a, kernel_id, stream);
  return launch_proj<SmallShape, kOut>(a, kernel_id, stream);
}


// ======================================================================================
// Backward of the projections
// ======================================================================================
// Gradient with respect to the input of a projection (dx from dq, dk, dv; d_o from dy) is the
// same product as the forward with the weight matrix transposed, so it runs the kernel above
// on a transposed copy of the weights that a small preparation kernel leaves in the workspace
// (the weights are a few MB; the copy costs microseconds).  Gradient with respect to the
// weights contracts over TOKENS: dW[f, e] = sum_tok G[tok, f] X[tok, e].  Both operands are
// token-major, so their 64-token x 64-column tiles go into LDS as they are and both MFMA
// operands come from transposing reads (which permute the 16 tokens of a slice the same way
// on both sides).  A workgroup owns 256 x 128 or 256 x 256 of dW and a range of the token blocks; partial
// sums of the ranges are added in a fixed order by a finalize kernel (no atomics: the result is
// bit-reproducible).  The bias gradient (column sums of G) rides along in the workgroups of
// the first column tile.  Rows of pad tokens are cleared in LDS after a block has landed, and
// blocks of padding only are skipped; which rows are pad comes from one 64-bit mask per block,
// written by the preparation kernel and read through the scalar cache.

// Token-major matrix whose 64-column blocks are either columns of a flat [B*N][ld] matrix or
// heads of up to three [B][H][N][64] tensors (column block c <-> tensor c / H, head c % H).
struct TokMat {
  const unsigned short* p[3];
  int heads;          // 1: head layout, 0: flat
  int ld;             // flat: elements per row
};
// A pointer the compiler can keep in scalar registers (the value is the same in every lane).
__device__ inline const char* uniform_ptr(const char* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const char*>(((unsigned long long)hi << 32) | lo);
}

struct WgradArgs {
  TokMat g, x;                    // G [tok][F-side], X [tok][E-side]
  const unsigned long long* pad;  // [B * blocks_per_seq]: bit r set = row r of the block is pad / past N
  float* out;                     // [F][E] (final when splits == 1)
  float* out_bias;                // [F] or null
  float* part;                    // [splits][F][E] partial sums (splits > 1)
  float* part_bias;               // [splits][F]
  int B, N, H;
  int F, E;                       // rows and columns of dW
  int blocks_per_seq;             // ceil(N / 64)
  int splits, per_split;          // token-block ranges
  int want_bias;
};

// Workgroup: 8 wavefronts, 256 rows x (64 KX) columns of dW, KX = 2 or 4; a wavefront owns 64 rows x
// 32 KX columns; one block of 64 tokens per stage (four G tiles, KX X tiles).  The wide shape
// halves the operand reads per contraction and is used when its tiles still fill the chip without
// cutting the tokens into many ranges (each range leaves an fp32 partial matrix behind).
constexpr int kWgRows = 256, kWgThreads = 512;
template <int KX>
struct WgShape {
  static constexpr int kCols = 64 * KX, kTiles = 4 + KX, kStageBytesW = kTiles * kTileBytes;
  static constexpr int kStagesW = KX == 2 ? 3 : 2;
  static constexpr int kQuartersW = 4 * kTiles / 8;          // 16-row loads per wavefront and stage
  static constexpr int kLoadsW = 2 * kQuartersW;
  static constexpr int kXF = KX;                              // 32-column X fragments per wavefront
};
template <int KX>
__global__ __launch_bounds__(kWgThreads, 1) void proj_wgrad_kernel(WgradArgs a) {
  using S = WgShape<KX>;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = lane & 31, hl = lane >> 5;
  const int e_tiles = a.E / S::kCols, tiles = ((a.F + kWgRows - 1) / kWgRows) * e_tiles;
  // Workgroup -> (token range, tile): XCD q = blockIdx % 8 takes a contiguous piece of the list
  // ordered by token range first, so the workgroups that stream the same tokens share an L2
  // (dealt round-robin, every XCD would fetch all of G from memory: 8 x the traffic).
  const int total = tiles * a.splits, per_xcd = (total + 7) >> 3;
  const int q = blockIdx.x & 7, jx = blockIdx.x >> 3, idx = q * per_xcd + jx;
  if (jx >= per_xcd || idx >= total) return;
  const int split = idx / tiles, tile = idx - split * tiles;
  const int ft = tile / e_tiles, et = tile - ft * e_tiles;
  const int f0 = ft * kWgRows, e0 = et * S::kCols;
  const int wf = wave >> 1, we = wave & 1;           // this wavefront: rows 64 wf .., columns 32 KX we ..
  const int total_blocks = a.B * a.blocks_per_seq;
  const int s_begin = split * a.per_split, s_end = min(total_blocks, s_begin + a.per_split);

  // tile i of a stage: 0..3 = G column blocks f0 / 64 + i;  4.. = X column blocks e0 / 64 + i - 4.
  // Wavefront w loads quarter w + 8 j of the stage: 16 rows of tile (w + 8 j) / 4.
  const LoadLane ll = make_load_lane(0, lane);
  const char* base[S::kQuartersW];
  unsigned row_stride[S::kQuartersW];
  size_t seq_stride[S::kQuartersW];
  int row16[S::kQuartersW], lds_off[S::kQuartersW];
#pragma unroll
  for (int j = 0; j < S::kQuartersW; ++j) {
    const int qi = wave + 8 * j, i = qi >> 2;
    const bool is_g = i < 4;
    // (F is a multiple of 128, not of 256: the last row tile repeats its last column block of G
    // and does not store the rows past F)
    const int c = is_g ? min(f0 / 64 + i, a.F / 64 - 1) : e0 / 64 + i - 4;
    const bool heads = is_g ? a.g.heads != 0 : a.x.heads != 0;
    const int ld = is_g ? a.g.ld : a.x.ld;
    const int t = c / a.H, h = c - t * a.H;
    const unsigned short* p0 = is_g ? a.g.p[0] : a.x.p[0];
    const unsigned short* p1 = is_g ? a.g.p[1] : a.x.p[1];
    const unsigned short* p2 = is_g ? a.g.p[2] : a.x.p[2];
    const unsigned short* tensor = !heads || t == 0 ? p0 : t == 1 ? p1 : p2;
    base[j] = uniform_ptr(reinterpret_cast<const char*>(tensor + (heads ? (size_t)h * a.N * kD : (size_t)c * 64)));
    row_stride[j] = heads ? kD * 2 : (unsigned)ld * 2;
    seq_stride[j] = heads ? (size_t)a.H * a.N * kD * 2 : (size_t)a.N * ld * 2;
    row16[j] = 16 * (qi & 3);
    lds_off[j] = i * kTileBytes + row16[j] * 128;
  }
  auto issue_stage = [&](int s, int slot) {
    const int b = s / a.blocks_per_seq, n0 = (s - b * a.blocks_per_seq) * 64;
    char* st = lds + slot * S::kStageBytesW;
#pragma unroll
    for (int j = 0; j < S::kQuartersW; ++j) {
      const int r0 = min(n0 + row16[j] + ll.row0, a.N - 1), r1 = min(n0 + row16[j] + ll.row0 + 8, a.N - 1);
      const char* bp = uniform_ptr(base[j] + (size_t)b * seq_stride[j]);
      load_to_lds_16(bp, (unsigned)r0 * row_stride[j] + ll.chunk0 * 16, st + lds_off[j]);
      load_to_lds_16(bp, (unsigned)r1 * row_stride[j] + (ll.chunk0 ^ 2) * 16, st + lds_off[j] + 8 * 128);
    }
  };
  // next block at or after s that has a non-pad row (all of this is scalar)
  auto next_live = [&](int s) {
    while (s < s_end && a.pad[s] == ~0ull) ++s;
    return s;
  };

  f32x16 acc[2][S::kXF];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < S::kXF; ++j) acc[i][j] = zero16();
  float bias_acc[2] = {0.f, 0.f};
  const bool do_bias = a.want_bias && et == 0 && we == 0;

  int toff[2][2];
#pragma unroll
  for (int db = 0; db < 2; ++db) {
    toff[db][0] = tr_off(lane, db, 0);
    toff[db][1] = tr_off(lane, db, 1);
  }

  // blocks in flight: `cur` (being waited for, then consumed) and the kStagesW - 1 after it
  int nx[S::kStagesW];  // nx[0] = cur
  nx[0] = next_live(s_begin);
#pragma unroll
  for (int k = 1; k < S::kStagesW; ++k) nx[k] = next_live(nx[k - 1] + 1);
#pragma unroll
  for (int k = 0; k + 1 < S::kStagesW; ++k)
    if (nx[k] < s_end) issue_stage(nx[k], k);
  int it = 0;
  while (nx[0] < s_end) {
    const unsigned long long padmask = a.pad[nx[0]];
    // block nx[0] has landed: everything but the loads of the blocks after it that were issued
    int younger = 0;
#pragma unroll
    for (int k = 1; k + 1 < S::kStagesW; ++k) younger += nx[k] < s_end;
    wait_vmcnt_le<S::kLoadsW * (S::kStagesW - 2)>(younger * S::kLoadsW);
    barrier_no_fence();          // ... for everyone; and everyone is done with the block before it
    if (nx[S::kStagesW - 1] < s_end) issue_stage(nx[S::kStagesW - 1], (it + S::kStagesW - 1) % S::kStagesW);
    char* st = lds + (it % S::kStagesW) * S::kStageBytesW;
    if (padmask) {               // uniform: clear the pad rows of all tiles (0 x anything = 0 then)
      const int row = tid & 63, which = tid >> 6;
      if (which < S::kTiles && ((padmask >> row) & 1ull)) {
        uint4* p = reinterpret_cast<uint4*>(st + which * kTileBytes + row * 128);
#pragma unroll
        for (int c = 0; c < 8; ++c) p[c] = make_uint4(0, 0, 0, 0);
      }
      __syncthreads();
    }
    const char* g_t = st + wf * kTileBytes;
    const char* x_t = st + (4 + we * (KX / 2)) * kTileBytes;
    // operand fragments are read one 16-token slice ahead of the contractions that use them
    bf16x8 gf[2][2], xf[2][S::kXF];
    auto read_slice = [&](int buf, int k16) {
#pragma unroll
      for (int db = 0; db < 2; ++db) gf[buf][db] = read_transposed(g_t + 16 * k16 * 128, toff[db][0], toff[db][1]);
#pragma unroll
      for (int j = 0; j < S::kXF; ++j)
        xf[buf][j] = read_transposed(x_t + (j >> 1) * kTileBytes + 16 * k16 * 128, toff[j & 1][0], toff[j & 1][1]);
    };
    read_slice(0, 0);
#pragma unroll
    for (int k16 = 0; k16 < 4; ++k16) {
      if (k16 + 1 < 4) read_slice((k16 + 1) & 1, k16 + 1);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < S::kXF; ++j) acc[i][j] = mfma(gf[k16 & 1][i], xf[k16 & 1][j], acc[i][j]);
      if (do_bias) {
        bias_acc[0] = sum8(gf[k16 & 1][0], bias_acc[0]);
        bias_acc[1] = sum8(gf[k16 & 1][1], bias_acc[1]);
      }
    }
#pragma unroll
    for (int k = 0; k + 1 < S::kStagesW; ++k) nx[k] = nx[k + 1];
    nx[S::kStagesW - 1] = next_live(nx[S::kStagesW - 2] + 1);
    ++it;
  }

  // C tile: lane (m, hl) holds column m, register 4 g + r holds row 8 g + 4 hl + r
  float* dst = (a.splits > 1 ? a.part + (size_t)split * a.F * a.E : a.out);
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < S::kXF; ++j)
#pragma unroll
      for (int c = 0; c < 16; ++c) {
        const int row = f0 + 64 * wf + 32 * i + 8 * (c >> 2) + 4 * hl + (c & 3);
        if (row < a.F) dst[(size_t)row * a.E + e0 + 32 * KX * we + 32 * j + m] = acc[i][j][c];
      }
  if (do_bias) {
    float* bd = a.splits > 1 ? a.part_bias + (size_t)split * a.F : a.out_bias;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const float v = half_sum(bias_acc[i]);
      if (hl == 0 && f0 + 64 * wf + 32 * i + m < a.F) bd[f0 + 64 * wf + 32 * i + m] = v;
    }
  }
}

// Adds the partial sums of the token-block ranges in range order.
__global__ __launch_bounds__(256) void proj_wgrad_finalize_kernel(WgradArgs a) {
  const size_t n4 = (size_t)a.F * a.E / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    float4 s = reinterpret_cast<const float4*>(a.part)[i];
    for (int k = 1; k < a.splits; ++k) {
      const float4 v = reinterpret_cast<const float4*>(a.part + (size_t)k * a.F * a.E)[i];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    reinterpret_cast<float4*>(a.out)[i] = s;
  }
  if (a.want_bias)
    for (int f = blockIdx.x * 256 + threadIdx.x; f < a.F; f += gridDim.x * 256) {
      float s = a.part_bias[f];
      for (int k = 1; k < a.splits; ++k) s += a.part_bias[(size_t)k * a.F + f];
      a.out_bias[f] = s;
    }
}

// Preparation: blocks [0, R / 64 * C / 64) transpose the bf16 matrix w [R][C] into wt [C][R]
// (skipped when wt is null); the blocks after them write the pad masks of the token blocks.
__global__ __launch_bounds__(256) void proj_bwd_prep_kernel(const unsigned short* __restrict__ w,
                                                            unsigned short* __restrict__ wt, int R, int C,
                                                            const unsigned char* __restrict__ flags, int B,
                                                            int N, unsigned long long* __restrict__ pad) {
  __shared__ unsigned short t[64][66];
  const int n_tr = wt ? (R / 64) * (C / 64) : 0;
  if ((int)blockIdx.x < n_tr) {
    const int r0 = (blockIdx.x / (C / 64)) * 64, c0 = (blockIdx.x % (C / 64)) * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) t[i >> 6][i & 63] = w[(size_t)(r0 + (i >> 6)) * C + c0 + (i & 63)];
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) wt[(size_t)(c0 + (i >> 6)) * R + r0 + (i & 63)] = t[i & 63][i >> 6];
    return;
  }
  const int bps = (N + 63) / 64, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int s = ((int)blockIdx.x - n_tr) * 4 + wave; s < B * bps; s += ((int)gridDim.x - n_tr) * 4) {
    const int b = s / bps, n = (s - b * bps) * 64 + lane;
    const bool is_pad = n >= N || flags[(size_t)b * N + n] >= 2;
    const unsigned long long mask = __ballot(is_pad);
    if (lane == 0) pad[s] = mask;
  }
}

}  // namespace

hipError_t launch_qkv_project(const void* x, const void* w_qkv, const float* bias,
                              const unsigned char* flags, int B, int N, int H, int E, void* q,
                              void* k, void* v, hipStream_t stream) {
  ProjArgs a = {};
  a.w = static_cast<const unsigned short*>(w_qkv);
  a.tok = static_cast<const unsigned short*>(x);
  a.bias = bias;
  a.flags = flags;
  a.out[0] = static_cast<unsigned short*>(q);
  a.out[1] = static_cast<unsigned short*>(k);
  a.out[2] = static_cast<unsigned short*>(v);
  a.B = B; a.N = N; a.H = H; a.E = E;
  a.F = 3 * H * kD;
  a.K = E;
  return launch_proj_any<false>(a, 8, stream);
}

hipError_t launch_out_project(const void* o, const void* w_o, const float* bias,
                              const unsigned char* flags, int B, int N, int H, int E, void* y,
                              hipStream_t stream) {
  ProjArgs a = {};
  a.w = static_cast<const unsigned short*>(w_o);
  a.tok3[0] = static_cast<const unsigned short*>(o);
  a.bias = bias;
  a.flags = flags;
  a.out[0] = static_cast<unsigned short*>(y);
  a.B = B; a.N = N; a.H = H; a.E = E;
  a.F = E;
  a.K = H * kD;
  return launch_proj_any<true>(a, 9, stream);
}

}  // namespace mate

namespace mate {

namespace {
size_t align256(size_t n) { return (n + 255) & ~size_t(255); }
struct BwdPlan {
  int blocks_per_seq, splits, per_split, kx;
  size_t wt_off, pad_off, part_off, bias_off, total;
};
// F x E = shape of the weight gradient; `wt_elems` = elements of the transposed weight copy.
BwdPlan plan_bwd(int B, int N, int F, int E, size_t wt_elems) {
  BwdPlan p;
  p.blocks_per_seq = (N + 63) / 64;
  const int total_blocks = B * p.blocks_per_seq;
  // Token ranges: enough workgroups for the chip (one per CU), but ranges of at least eight token
  // blocks -- every range leaves an fp32 partial matrix that is written and read again.  The wide
  // tile is taken when it fills the chip with at most sixteen ranges.
  auto ranges = [&](int kx) {
    const int tiles = ((F + kWgRows - 1) / kWgRows) * (E / (64 * kx));
    return std::max(1, std::min(std::max(1, 256 / tiles), total_blocks / 8));
  };
  p.kx = (E % 256 == 0 && ((F + kWgRows - 1) / kWgRows) * (E / 256) * ranges(4) >= 192 && ranges(4) <= 16) ? 4 : 2;
  const int want = ranges(p.kx);
  p.per_split = (total_blocks + want - 1) / want;
  p.splits = (total_blocks + p.per_split - 1) / p.per_split;
  p.wt_off = 0;
  p.pad_off = align256(wt_elems * 2);
  p.part_off = p.pad_off + align256((size_t)total_blocks * 8);
  p.bias_off = p.part_off + (p.splits > 1 ? align256((size_t)p.splits * F * E * 4) : 0);
  p.total = p.bias_off + (p.splits > 1 ? align256((size_t)p.splits * F * 4) : 0);
  return p;
}

template <int KX>
hipError_t launch_wgrad(const WgradArgs& a, int splits, int kernel_id, hipStream_t stream) {
  using S = WgShape<KX>;
  const int tiles = ((a.F + kWgRows - 1) / kWgRows) * (a.E / S::kCols);
  const size_t lds_bytes = (size_t)S::kStagesW * S::kStageBytesW;
  hipError_t e0 = hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_wgrad_kernel<KX>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e0 != hipSuccess) return e0;
  ProfileScope prof(kernel_id, stream);
  hipLaunchKernelGGL(proj_wgrad_kernel<KX>, dim3(8 * ((tiles * splits + 7) / 8)), dim3(kWgThreads), lds_bytes,
                     stream, a);
  return hipGetLastError();
}

hipError_t run_wgrad(WgradArgs a, const BwdPlan& p, char* ws, int kernel_id, hipStream_t stream) {
  a.blocks_per_seq = p.blocks_per_seq;
  a.splits = p.splits;
  a.per_split = p.per_split;
  a.pad = reinterpret_cast<const unsigned long long*>(ws + p.pad_off);
  a.part = reinterpret_cast<float*>(ws + p.part_off);
  a.part_bias = reinterpret_cast<float*>(ws + p.bias_off);
  hipError_t e = p.kx == 4 ? launch_wgrad<4>(a, p.splits, kernel_id, stream)
                           : launch_wgrad<2>(a, p.splits, kernel_id, stream);
  if (e != hipSuccess || p.splits == 1) return e;
  hipLaunchKernelGGL(proj_wgrad_finalize_kernel, dim3(1024), dim3(256), 0, stream, a);
  return hipGetLastError();
}
}  // namespace

size_t qkv_project_bwd_workspace(int B, int N, int H, int E) {
  return plan_bwd(B, N, 3 * H * kD, E, (size_t)3 * H * kD * E).total;
}
size_t out_project_bwd_workspace(int B, int N, int H, int E) {
  return plan_bwd(B, N, E, H * kD, (size_t)E * H * kD).total;
}

hipError_t launch_qkv_project_bwd(const void* x, const void* w_qkv, const unsigned char* flags,
                                  const void* dq, const void* dk, const void* dv, int B, int N, int H,
                                  int E, void* dx, float* dw, float* dbias, void* workspace,
                                  hipStream_t stream) {
  const int F = 3 * H * kD;
  const BwdPlan p = plan_bwd(B, N, F, E, (size_t)F * E);
  char* ws = static_cast<char*>(workspace);
  unsigned short* wt = reinterpret_cast<unsigned short*>(ws + p.wt_off);
  const int n_tr = dx ? (F / 64) * (E / 64) : 0;
  hipLaunchKernelGGL(proj_bwd_prep_kernel, dim3(n_tr + 64), dim3(256), 0, stream,
                     static_cast<const unsigned short*>(w_qkv), dx ? wt : nullptr, F, E, flags, B, N,
                     reinterpret_cast<unsigned long long*>(ws + p.pad_off));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (dx) {  // dx[tok, :] = sum over the 3 H heads of dq, dk, dv [tok, head] . w_qkv[head rows, :]
    ProjArgs a = {};
    a.w = wt;                       // [E][F]
    a.tok3[0] = static_cast<const unsigned short*>(dq);
    a.tok3[1] = static_cast<const unsigned short*>(dk);
    a.tok3[2] = static_cast<const unsigned short*>(dv);
    a.flags = flags;
    a.out[0] = static_cast<unsigned short*>(dx);
    a.B = B; a.N = N; a.H = H; a.E = E;
    a.F = E;
    a.K = F;
    e = launch_proj_any<true>(a, 10, stream);
    if (e != hipSuccess) return e;
  }
  if (dw) {
    WgradArgs g = {};
    g.g.p[0] = static_cast<const unsigned short*>(dq);
    g.g.p[1] = static_cast<const unsigned short*>(dk);
    g.g.p[2] = static_cast<const unsigned short*>(dv);
    g.g.heads = 1;
    g.x.p[0] = static_cast<const unsigned short*>(x);
    g.x.heads = 0;
    g.x.ld = E;
    g.out = dw;
    g.out_bias = dbias;
    g.want_bias = dbias != nullptr;
    g.B = B; g.N = N; g.H = H; g.F = F; g.E = E;
    e = run_wgrad(g, p, ws, 11, stream);
  }
  return e;
}

hipError_t launch_out_project_bwd(const void* o, const void* w_o, const unsigned char* flags,
                                  const void* dy, int B, int N, int H, int E, void* d_o, float* dw,
                                  float* dbias, void* workspace, hipStream_t stream) {
  const int J = H * kD;
  const BwdPlan p = plan_bwd(B, N, E, J, (size_t)E * J);
  char* ws = static_cast<char*>(workspace);
  unsigned short* wt = reinterpret_cast<unsigned short*>(ws + p.wt_off);
  const int n_tr = d_o ? (E / 64) * (J / 64) : 0;
  hipLaunchKernelGGL(proj_bwd_prep_kernel, dim3(n_tr + 64), dim3(256), 0, stream,
                     static_cast<const unsigned short*>(w_o), d_o ? wt : nullptr, E, J, flags, B, N,
                     reinterpret_cast<unsigned long long*>(ws + p.pad_off));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (d_o) {  // d_o[tok, head i] = dy[tok, :] . w_o[:, head i columns], written head by head
    ProjArgs a = {};
    a.w = wt;                       // [H*64][E]
    a.tok = static_cast<const unsigned short*>(dy);
    a.flags = flags;
    a.out[0] = static_cast<unsigned short*>(d_o);
    a.B = B; a.N = N; a.H = H; a.E = E;
    a.F = J;
    a.K = E;
    e = launch_proj_any<false>(a, 12, stream);
    if (e != hipSuccess) return e;
  }
  if (dw) {
    WgradArgs g = {};
    g.g.p[0] = static_cast<const unsigned short*>(dy);
    g.g.heads = 0;
    g.g.ld = E;
    g.x.p[0] = static_cast<const unsigned short*>(o);
    g.x.heads = 1;
    g.out = dw;
    g.out_bias = dbias;
    g.want_bias = dbias != nullptr;
    g.B = B; g.N = N; g.H = H; g.F = E; g.E = J;
    e = run_wgrad(g, p, ws, 13, stream);
  }
  return e;
}

}  // namespace mate
