// Dense-mask variant of the bf16 MFMA attention kernels for short sequences.
//
// Section 3.1 keeps two functionally equivalent implementations -- the reordered, windowed one and
// plain attention under the mask of Section 3 -- and picks the faster per use case, because at
// short lengths the cost of reordering outweighs the saved work.  Here the reordered path is
// mate_build_segments + mate_attn_fwd / mate_attn_bwd; this file is the other one: no segment
// tables, no sort, no gathers.  A workgroup owns 128 consecutive positions of one
// (sequence, head) and streams every 64-position tile of the sequence; each (query, key) pair is
// scored and then kept or dropped by comparing the two tokens' codes
//     code = row id (row heads) / column id (column heads) for a table token,
//            -1 for a question token, -2 for padding
//     allowed(a, b) = a > -2 and b > -2 and (a == b or a == -1 or b == -1)
// which is the attention pattern A^i_k of Section 3 written per pair.  The arithmetic (base-2
// online softmax, bf16 P and dS, fp32 accumulation, accumulators of the dK/dV kernel started at
// -lse / scale and -delta) is that of the segment kernels, so both paths meet the same oracle.
#include <hip/hip_runtime.h>

#include "d2l.h"
#include "launch.h"
#include "mfma_common.h"
#include "stream_plan.h"
#include "tile_bodies.h"

namespace mate {
namespace {

constexpr int kStage = 2 * kTileBytes;        // two tensors' tiles
constexpr int kDkvStageD = kStage + 512;      // ... plus -lse/scale[64], -delta[64]

struct DenseUnit {
  int b, bh, view, tile;  // tile: which 128 positions are owned
};

// Workgroup -> (sequence, head, owner tile); (sequence, head) pairs with equal index mod 8 share
// an XCD (consecutive workgroups go to consecutive XCDs), so their K / V tiles share an L2.
__device__ inline bool dense_unit(const DenseArgs& a, DenseUnit& u) {
  const int T = owner_slots(a.N), q = blockIdx.x & 7, r = blockIdx.x >> 3;
  u.tile = r % T;
  u.bh = (r / T) * 8 + q;
  if (u.bh >= a.B * a.H) return false;
  u.b = u.bh / a.H;
  u.view = a.head_kind[u.bh % a.H];
  return true;
}
inline int dense_grid(const DenseArgs& a) { return 8 * ((a.B * a.H + 7) / 8) * owner_slots(a.N); }

// Codes of all positions of the sequence (padded with -2 to a whole number of tiles) into LDS.
__device__ inline void load_codes(const DenseArgs& a, const DenseUnit& u, int* code) {
  const int N = a.N;
  const int* ids = (u.view == 0 ? a.row_ids : a.col_ids) + (size_t)u.b * N;
  const unsigned char* fl = a.flags + (size_t)u.b * N;
  for (int n = threadIdx.x; n < ((N + BN - 1) / BN) * BN; n += kThreads) {
    int c = -2;
    if (n < N) {
      const int f = fl[n];
      c = f == 0 ? ids[n] : f == 1 ? -1 : -2;
    }
    code[n] = c;
  }
}

// Owned row of a lane: position, code, and whether anything may be written for it.
struct DenseRow {
  int pos;     // clamped to N - 1
  bool in_range;
  int code;
  bool global;
};
__device__ inline DenseRow dense_row(const DenseArgs& a, const DenseUnit& u, const int* code, int wave, int m) {
  DenseRow r;
  const int p = u.tile * BM + wave * 32 + m;
  r.in_range = p < a.N;
  r.pos = min(p, a.N - 1);
  r.code = code[r.pos];
  r.global = r.code == -1;
  return r;
}

// May the owned row (code mc, global flag) meet a streamed row with code kc?  (Pad owners get
// arbitrary answers; their results are replaced by zeros.)
// Written with bitwise operators on purpose: as a conditional expression it compiled to a
// divergent branch per element.
__device__ inline bool allowed(int kc, int mc, bool owner_global) {
  return ((int)(kc == mc) | (int)(kc == -1) | ((int)owner_global & (int)(kc > -2))) != 0;
}

// Streams the sequence's 64-position tiles of two tensors through two LDS stages.
struct DenseStream {
  const unsigned short *X0, *X1;
  const float *rows0, *rows1;  // optional per-position floats (wavefront 0 / 1 load them)
  char* stages;
  int stage_bytes, N, wave, lane;
  LoadLane ll;
  __device__ void issue(int t) {
    char* st = stages + (t & 1) * stage_bytes;
    const int p0 = min(t * BN + ll.row0, N - 1), p1 = min(t * BN + ll.row0 + 8, N - 1);
    issue_tile(X0, p0, p1, ll, st, wave);
    issue_tile(X1, p0, p1, ll, st + kTileBytes, wave);
    const float* rs = wave == 0 ? rows0 : wave == 1 ? rows1 : nullptr;
    if (rs) issue_row_words(rs, min(t * BN + lane, N - 1), st + kStage + 256 * wave);
  }
  // tile t is complete for every wavefront and the other stage is free: start loading tile t + 1
  __device__ const char* acquire(int t, int n_tiles) {
    wait_vmcnt_le(0);
    barrier_no_fence();
    if (t + 1 < n_tiles) issue(t + 1);
    return stages + (t & 1) * stage_bytes;
  }
};

// The dense-mask rule as a Mask of tile_bodies.h: the pair is kept iff the two tokens' codes say
// so.  `codes` points at the tile's 64 codes in LDS, offset by this lane half's 4 hl.
struct CodeMask {
  static constexpr bool full = false;
  const int* codes;
  int my_code;
  bool my_global;
  int k[16];
  __device__ __forceinline__ CodeMask(const int* tile_codes, int hl, int code, bool global)
      : codes(tile_codes + 4 * hl), my_code(code), my_global(global) {}
  __device__ __forceinline__ void load(int blk) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int4 kc = *reinterpret_cast<const int4*>(codes + blk * 32 + 8 * g);
      k[4 * g] = kc.x; k[4 * g + 1] = kc.y; k[4 * g + 2] = kc.z; k[4 * g + 3] = kc.w;
    }
  }
  __device__ __forceinline__ bool skip(int) const { return false; }
  __device__ __forceinline__ bool in(int, int c) const { return allowed(k[c], my_code, my_global); }
};

// ======================================================================================
// forward
// ======================================================================================
__global__ __launch_bounds__(kThreads) void fwd_dense_kernel(DenseArgs a) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * kStage];
  __shared__ __attribute__((aligned(16))) int code[kDenseMaxN];
  __shared__ int q_tok[BM];
  DenseUnit u;
  if (!dense_unit(a, u)) return;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = lane & 31, hl = lane >> 5;
  const size_t bh = (size_t)u.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  unsigned short* O = static_cast<unsigned short*>(a.out) + bh * kD;

  DenseStream stream{K, V, nullptr, nullptr, lds, kStage, N, wave, lane, make_load_lane(wave, lane)};
  stream.issue(0);
  load_codes(a, u, code);
  if (tid < BM) q_tok[tid] = u.tile * BM + tid < N ? u.tile * BM + tid : -1;
  __syncthreads();
  const DenseRow me = dense_row(a, u, code, wave, m);
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + (size_t)me.pos * kD + ks * 16 + hl * 8));
  asm volatile("" ::"v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]));

  const float sc = a.scale * kLog2e;
  f32x16 o_acc[2] = {zero16(), zero16()};
  float m_run = -INFINITY, l_run = 0.f;
  int koff[4], voff[2][2];
  operand_offsets(lane, koff, voff);
  const bool wave_active = u.tile * BM + wave * 32 < N;

  const int n_tiles = (N + BN - 1) / BN;
  for (int t = 0; t < n_tiles; ++t) {
    const char* Kst = stream.acquire(t, n_tiles);
    const char* Vst = Kst + kTileBytes;
    if (!wave_active) continue;
    fwd_tile(Kst, Vst, qf, koff, voff, sc, 0.f, CodeMask(code + t * BN, hl, me.code, me.global), o_acc, m_run, l_run);
  }
  __syncthreads();
  const float l_tot = half_sum(l_run);
  const bool live = me.in_range && me.code > -2;  // pad positions: O = 0, LSE = 0
  if (hl == 0 && me.in_range)
    a.lse[bh + me.pos] = live ? (m_run * sc + __builtin_amdgcn_logf(l_tot)) * kLn2 : 0.f;
  const float inv = live ? 1.f / l_tot : 0.f;
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int c = 0; c < 16; ++c) o_acc[db][c] = live ? o_acc[db][c] * inv : 0.f;
  const f32x16 (*accs[1])[2] = {&o_acc};
  const float muls[1] = {1.f};
  unsigned short* const outs[1] = {O};
  store_owned_rows<1>(accs, muls, outs, lds, q_tok, wave, lane);
}

// ======================================================================================
// dQ (and -delta, -lse / scale for the dK/dV kernel)
// ======================================================================================
__global__ __launch_bounds__(kThreads) void bwd_dq_dense_kernel(DenseArgs a) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * kStage];
  __shared__ __attribute__((aligned(16))) int code[kDenseMaxN];
  __shared__ int q_tok[BM];
  DenseUnit u;
  if (!dense_unit(a, u)) return;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = lane & 31, hl = lane >> 5;
  const size_t bh = (size_t)u.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  const unsigned short* O = static_cast<const unsigned short*>(a.o) + bh * kD;
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dQ = static_cast<unsigned short*>(a.dq) + bh * kD;

  DenseStream stream{K, V, nullptr, nullptr, lds, kStage, N, wave, lane, make_load_lane(wave, lane)};
  stream.issue(0);
  load_codes(a, u, code);
  if (tid < BM) q_tok[tid] = u.tile * BM + tid < N ? u.tile * BM + tid : -1;
  __syncthreads();
  const DenseRow me = dense_row(a, u, code, wave, m);
  bf16x8 qf[4], gf[4], of[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)me.pos * kD + ks * 16 + hl * 8;
    qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + off));
    gf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(dO + off));
    of[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(O + off));
  }
  const float lse = a.lse[bh + me.pos];
  asm volatile("" ::"v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]), "v"(gf[0]), "v"(gf[1]),
               "v"(gf[2]), "v"(gf[3]), "v"(of[0]), "v"(of[1]), "v"(of[2]), "v"(of[3]), "v"(lse));
  float delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int e = 0; e < 8; ++e) delta = fmaf((float)gf[ks][e], (float)of[ks][e], delta);
  delta = half_sum(delta);
  if (hl == 0 && me.in_range) {
    a.delta[bh + me.pos] = -delta;
    a.nlse[bh + me.pos] = -lse / a.scale;
  }
  const float lse2 = lse * kLog2e, sc = a.scale * kLog2e;
  int koff[4], toff[2][2];
  operand_offsets(lane, koff, toff);
  const bool wave_active = u.tile * BM + wave * 32 < N;

  f32x16 dq_acc[2] = {zero16(), zero16()};
  const int n_tiles = (N + BN - 1) / BN;
  for (int t = 0; t < n_tiles; ++t) {
    const char* Kst = stream.acquire(t, n_tiles);
    const char* Vst = Kst + kTileBytes;
    if (!wave_active) continue;
    dq_tile(Kst, Vst, qf, gf, koff, toff, sc, lse2, delta, CodeMask(code + t * BN, hl, me.code, me.global), dq_acc);
  }
  __syncthreads();
  const float mul = me.in_range && me.code > -2 ? a.scale : 0.f;  // pad positions: zeros
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int c = 0; c < 16; ++c) dq_acc[db][c] = mul != 0.f ? dq_acc[db][c] * mul : 0.f;
  const f32x16 (*accs[1])[2] = {&dq_acc};
  const float muls[1] = {1.f};
  unsigned short* const outs[1] = {dQ};
  store_owned_rows<1>(accs, muls, outs, lds, q_tok, wave, lane);
}

// ======================================================================================
// dK, dV
// ======================================================================================
__global__ __launch_bounds__(kThreads) void bwd_dkv_dense_kernel(DenseArgs a) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * kDkvStageD];
  __shared__ __attribute__((aligned(16))) int code[kDenseMaxN];
  __shared__ int k_tok[BM];
  DenseUnit u;
  if (!dense_unit(a, u)) return;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = lane & 31, hl = lane >> 5;
  const size_t bh = (size_t)u.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dK = static_cast<unsigned short*>(a.dk) + bh * kD;
  unsigned short* dV = static_cast<unsigned short*>(a.dv) + bh * kD;

  DenseStream stream{Q, dO, a.nlse + bh, a.delta + bh, lds, kDkvStageD, N, wave, lane,
                     make_load_lane(wave, lane)};
  stream.issue(0);
  load_codes(a, u, code);
  if (tid < BM) k_tok[tid] = u.tile * BM + tid < N ? u.tile * BM + tid : -1;
  __syncthreads();
  const DenseRow me = dense_row(a, u, code, wave, m);  // this lane's key
  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)me.pos * kD + ks * 16 + hl * 8;
    kf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(K + off));
    vf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(V + off));
  }
  asm volatile("" ::"v"(kf[0]), "v"(kf[1]), "v"(kf[2]), "v"(kf[3]), "v"(vf[0]), "v"(vf[1]),
               "v"(vf[2]), "v"(vf[3]));
  const float sc = a.scale * kLog2e;
  int poff[4], toff[2][2];
  operand_offsets(lane, poff, toff);
  const bool wave_active = u.tile * BM + wave * 32 < N;

  f32x16 dk_acc[2] = {zero16(), zero16()}, dv_acc[2] = {zero16(), zero16()};
  const int n_tiles = (N + BN - 1) / BN;
  for (int t = 0; t < n_tiles; ++t) {
    const char* Qst = stream.acquire(t, n_tiles);
    const char* Gst = Qst + kTileBytes;
    const float* lse_row = reinterpret_cast<const float*>(Qst + kStage);
    const float* delta_row = lse_row + BN;
    if (!wave_active) continue;
    dkv_tile(Qst, Gst, lse_row, delta_row, kf, vf, poff, toff, sc, hl, CodeMask(code + t * BN, hl, me.code, me.global), dk_acc, dv_acc);
  }
  __syncthreads();
  const bool live = me.in_range && me.code > -2;  // pad positions: zeros
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      dk_acc[db][c] = live ? dk_acc[db][c] * a.scale : 0.f;
      dv_acc[db][c] = live ? dv_acc[db][c] : 0.f;
    }
  const f32x16 (*accs[2])[2] = {&dk_acc, &dv_acc};
  const float muls[2] = {1.f, 1.f};
  unsigned short* const outs[2] = {dK, dV};
  store_owned_rows<2>(accs, muls, outs, lds, k_tok, wave, lane);
}

}  // namespace

hipError_t launch_fwd_dense(const DenseArgs& a, hipStream_t stream) {
  ProfileScope prof(5, stream);
  hipLaunchKernelGGL(fwd_dense_kernel, dim3(dense_grid(a)), dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dense(const DenseArgs& a, hipStream_t stream) {
  {
    ProfileScope prof(6, stream);
    hipLaunchKernelGGL(bwd_dq_dense_kernel, dim3(dense_grid(a)), dim3(kThreads), 0, stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfileScope prof(7, stream);
  hipLaunchKernelGGL(bwd_dkv_dense_kernel, dim3(dense_grid(a)), dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace mate
