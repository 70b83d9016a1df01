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
  const unsigned short* tok;     // QKV: x [B*N][E];  out: o [B][H][N][64]
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
  if (kOut) {  // k step = one head of the attention output
    tok_base = reinterpret_cast<const char*>(a.tok + (((size_t)b * a.H) * a.N + n0) * kD);
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
    const char* tb = tok_base + (size_t)ks * tok_step;
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
  a.tok = static_cast<const unsigned short*>(o);
  a.bias = bias;
  a.flags = flags;
  a.out[0] = static_cast<unsigned short*>(y);
  a.B = B; a.N = N; a.H = H; a.E = E;
  a.F = E;
  a.K = H * kD;
  return launch_proj_any<true>(a, 9, stream);
}

}  // namespace mate
