// bf16 MFMA backward for MATE attention: the derivative of the forward (Section 3 head
// equation restricted to the attention pattern A^i_k) with respect to Q, K and V.
//
// No floating-point atomics, so results are bit-reproducible:
//   dq kernel  -- a workgroup owns 128 queries (sorted order of the head kind, or question
//                 tokens) and streams the key tiles they see, exactly like the forward:
//                 P = exp(S - LSE), dP = dO V^T, dS = P (dP - delta), dQ += dS K.
//                 It also produces delta_k = dO_k . O_k for its queries and leaves -delta and
//                 -LSE / scale for the next kernel.
//   dkv kernel -- a workgroup owns 128 keys and streams the query tiles that see them: the
//                 question tokens plus the table tokens of the keys' own segments (every
//                 non-pad token when the keys are question tokens):
//                 dV += P^T dO, dK += dS^T Q.
//   finalize   -- question-token owners stream the whole sequence, so their stream is cut into
//                 chunks run by separate workgroups; this kernel adds the fp32 partials in
//                 chunk order.
// Pairs (table query, table key) are therefore recomputed once in each of the first two.
#include <hip/hip_runtime.h>

#include "d2l.h"
#include "launch.h"
#include "mfma_common.h"
#include "stream_plan.h"
#include "tile_bodies.h"
#include "tile_stream.h"

namespace mate {
namespace {

// ======================================================================================
// dQ (and delta)
// ======================================================================================
constexpr int kDqStage = 2 * kTileBytes;          // K tile, V tile
constexpr int kDqNS = 2, kDkvNS = 2;              // LDS stages of the two kernels
constexpr int kDkvStage = 2 * kTileBytes + 512;   // Q tile, dO tile, -lse/scale[64], -delta[64]

__device__ __forceinline__ void bwd_dq_unit(const AttnArgs& a, const Work& w) {
  __shared__ __attribute__((aligned(1024))) char lds[kDqNS * kDqStage];
  __shared__ int idx_ring[kIdxSlots][BN];
  __shared__ int q_tok[BM];

  const int b = w.bh / a.H;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
  const int m = lane & 31, hl = lane >> 5;
  const int view = w.view;
  const UnitPlan& u = w.u;

  const size_t bh = (size_t)w.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  const unsigned short* O = static_cast<const unsigned short*>(a.o) + bh * kD;
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dQ = static_cast<unsigned short*>(a.dq) + bh * kD;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  if (u.kind == UNIT_PAD) {
    unsigned short* const outs[1] = {dQ};
    zero_pad_rows<1>(outs, u, tid);
    return;
  }
  // First round trip: which rows this workgroup owns, and the token indices of the first tiles.
  // Second: the owned rows (registers) and the first K / V tiles (LDS), all in flight together.
  // K and V tiles stream through the LDS ring; K is read both plain (S^T = K Q^T) and
  // transposed (dQ^T += K^T dS^T), V plain (dP^T = V dO^T).
  TileStream<kDqStage, kDqNS> stream(u, global_idx, lds, idx_ring, K, V, nullptr, 0, wave, lane);
  stream.begin();
  const OwnedRow me = owned_row(u, a, b, view, wave, m);
  asm volatile("" ::"v"(me.pos), "v"(me.lo), "v"(me.hi), "v"(me.stage_tok));  // the owned rows are known from here on
  if (tid < BM) q_tok[tid] = me.stage_tok;
  stream.prime();

  // this lane's query row and dO row as B operands (column m, k = dims), and delta
  bf16x8 qf[4], gf[4], of[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)me.pos * kD + ks * 16 + hl * 8;
    qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + off));
    gf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(dO + off));
    of[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(O + off));
  }
  const float lse = a.lse[bh + me.pos];
  // Everything loaded into registers so far is pinned as complete here, so that no load with a
  // register destination is pending inside the loop.
  asm volatile("" ::"v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]), "v"(gf[0]), "v"(gf[1]),
               "v"(gf[2]), "v"(gf[3]), "v"(of[0]), "v"(of[1]), "v"(of[2]), "v"(of[3]), "v"(lse));
  float delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int e = 0; e < 8; ++e) delta = fmaf((float)gf[ks][e], (float)of[ks][e], delta);
  delta = half_sum(delta);
  // every chunk of a question-token owner computes the same delta; the first one stores it
  // (stored negated, with -lse / scale beside it: the dK/dV kernel starts its accumulators there)
  if (hl == 0 && me.valid && u.t_begin == 0) {
    a.delta[bh + me.pos] = -delta;
    a.nlse[bh + me.pos] = -lse / a.scale;
  }
  const float lse2 = lse * kLog2e;
  const float sc = a.scale * kLog2e;

  int koff[4], toff[2][2];
  operand_offsets(lane, koff, toff);

  f32x16 dq_acc[2] = {zero16(), zero16()};
  for (int t = u.t_begin; t < u.t_end; ++t) {
    const char* Kst = stream.acquire(t);
    const char* Vst = Kst + kTileBytes;
    const bool part0 = t < u.n_t0;
    const int base = part0 ? t * BN : u.s_lo + (t - u.n_t0) * BN;
    const bool skip = !me.wave_active || (!part0 && (base >= me.w_hi || base + BN <= me.w_lo));
    if (!skip) {
      const bool full = part0 ? (base + BN <= u.G) : (base >= me.a_lo && base + BN <= me.a_hi);
      dq_tile(Kst, Vst, qf, gf, koff, toff, sc, lse2, delta, WindowMask(full, base, hl, part0 ? 0 : me.lo, part0 ? u.G : me.hi, part0 ? 0 : me.w_lo, part0 ? u.G : me.w_hi), dq_acc);
    }
    stream.release();
  }
  __syncthreads();  // all wavefronts are done reading the stages; reuse them for the epilogue
  if (u.part >= 0) {
    const size_t slot = (size_t)w.bh * owner_slots(N) + u.part;
    store_partial(dq_acc, a.scale, a.part[0] + slot * BM * kD, wave, lane);
    return;
  }
  const f32x16 (*accs[1])[2] = {&dq_acc};
  const float muls[1] = {a.scale};
  unsigned short* const outs[1] = {dQ};
  store_owned_rows<1>(accs, muls, outs, lds, q_tok, wave, lane);
}

// (four workgroups per CU: with three, the column-head units of the benchmark shape do not all
// fit at once and the stragglers double the kernel's critical path)
__global__ __launch_bounds__(kThreads, 4) void bwd_dq_mfma_kernel(AttnArgs a) {
  Work w;
  if (!take_unit<true>(a, w)) return;
  bwd_dq_unit(a, w);
}

// ======================================================================================
// dK, dV
// ======================================================================================
__device__ __forceinline__ void bwd_dkv_unit(const AttnArgs& a, const Work& w) {
  __shared__ __attribute__((aligned(1024))) char lds[kDkvNS * kDkvStage];
  __shared__ int idx_ring[kIdxSlots][BN];
  __shared__ int k_tok[BM];

  const int b = w.bh / a.H;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
  const int m = lane & 31, hl = lane >> 5;
  const int view = w.view;
  const UnitPlan& u = w.u;

  const size_t bh = (size_t)w.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dK = static_cast<unsigned short*>(a.dk) + bh * kD;
  unsigned short* dV = static_cast<unsigned short*>(a.dv) + bh * kD;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  if (u.kind == UNIT_PAD) {
    unsigned short* const outs[2] = {dK, dV};
    zero_pad_rows<2>(outs, u, tid);
    return;
  }
  // Q and dO tiles of the streamed queries go through the LDS ring, each read plain
  // (S = Q K^T, dP = dO V^T) and transposed (dK^T += Q^T dS, dV^T += dO^T P); wavefront 0
  // also brings the queries' -lse / scale, wavefront 1 their -delta (one float per row).
  // First round trip: the owned rows' positions and the first tiles' token indices; second:
  // the owned K / V rows (registers) and the first tiles (LDS).
  const float* row_src = wave == 0 ? a.nlse + bh : wave == 1 ? a.delta + bh : nullptr;
  TileStream<kDkvStage, kDkvNS> stream(u, global_idx, lds, idx_ring, Q, dO, row_src,
                               2 * kTileBytes + 256 * wave, wave, lane);
  stream.begin();
  // `me` is this lane's key; its window is the set of query slots that see it
  const OwnedRow me = owned_row(u, a, b, view, wave, m);
  asm volatile("" ::"v"(me.pos), "v"(me.lo), "v"(me.hi), "v"(me.stage_tok));  // the owned rows are known from here on
  if (tid < BM) k_tok[tid] = me.stage_tok;
  stream.prime();

  bf16x8 kf[4], vf[4];  // this lane's key and value rows as B operands
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)me.pos * kD + ks * 16 + hl * 8;
    kf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(K + off));
    vf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(V + off));
  }
  const float sc = a.scale * kLog2e;
  asm volatile("" ::"v"(kf[0]), "v"(kf[1]), "v"(kf[2]), "v"(kf[3]), "v"(vf[0]), "v"(vf[1]),
               "v"(vf[2]), "v"(vf[3]));

  int poff[4], toff[2][2];
  operand_offsets(lane, poff, toff);

  f32x16 dk_acc[2] = {zero16(), zero16()}, dv_acc[2] = {zero16(), zero16()};
  for (int t = u.t_begin; t < u.t_end; ++t) {
    const char* Qst = stream.acquire(t);
    const char* Gst = Qst + kTileBytes;
    const float* lse_row = reinterpret_cast<const float*>(Qst + 2 * kTileBytes);
    const float* delta_row = lse_row + BN;
    const bool part0 = t < u.n_t0;
    const int base = part0 ? t * BN : u.s_lo + (t - u.n_t0) * BN;
    const bool skip = !me.wave_active || (!part0 && (base >= me.w_hi || base + BN <= me.w_lo));
    if (!skip) {
      const bool full = part0 ? (base + BN <= u.G) : (base >= me.a_lo && base + BN <= me.a_hi);
      dkv_tile(Qst, Gst, lse_row, delta_row, kf, vf, poff, toff, sc, hl, WindowMask(full, base, hl, part0 ? 0 : me.lo, part0 ? u.G : me.hi, part0 ? 0 : me.w_lo, part0 ? u.G : me.w_hi), dk_acc, dv_acc);
    }
    stream.release();
  }
  __syncthreads();  // all wavefronts are done reading the stages; reuse them for the epilogue
  if (u.part >= 0) {
    const size_t slot = (size_t)w.bh * owner_slots(N) + u.part;
    store_partial(dk_acc, a.scale, a.part[1] + slot * BM * kD, wave, lane);
    store_partial(dv_acc, 1.f, a.part[2] + slot * BM * kD, wave, lane);
    return;
  }
  const f32x16 (*accs[2])[2] = {&dk_acc, &dv_acc};
  const float muls[2] = {a.scale, 1.f};
  unsigned short* const outs[2] = {dK, dV};
  store_owned_rows<2>(accs, muls, outs, lds, k_tok, wave, lane);
}

__global__ __launch_bounds__(kThreads) void bwd_dkv_mfma_kernel(AttnArgs a) {
  Work w;
  if (!take_unit<true>(a, w)) return;
  bwd_dkv_unit(a, w);
}

// Adds the chunk partials of question-token rows in chunk order and stores dQ, dK, dV rows.
// blockIdx.z selects the tensor; 8 threads per row, 32 rows per workgroup.
__global__ __launch_bounds__(kThreads) void bwd_finalize_kernel(AttnArgs a) {
  const int bh_i = blockIdx.y, b = bh_i / a.H, N = a.N, which = blockIdx.z;
  // header and counts in one scalar round trip (both lie inside the table buffer whatever it holds)
  const int* cnt = a.seg.counts + (size_t)b * kCountWords;
  const int h_magic = a.seg.hdr[0], h_B = a.seg.hdr[1], h_N = a.seg.hdr[2];
  const int G = cnt[C_G], L = cnt[C_L];
  if (h_magic != kMagic || h_B != a.B || h_N != a.N) return;
  const GlobalSplit s = global_split(G, L, N);
  if (s.n_chunks <= 1) return;
  const int piece = threadIdx.x & 7;
  for (int x = blockIdx.x * 32 + (threadIdx.x >> 3); x < G; x += gridDim.x * 32) {
  const int gt = x / BM, r = x % BM;
  const size_t slot0 = (size_t)bh_i * owner_slots(N) + (size_t)gt * s.n_chunks;
  // chunks are read eight at a time, all loads issued before the first addition (the pin below:
  // left alone, the compiler keeps only a few in flight and the kernel becomes a chain of memory
  // round trips); the order of the additions is fixed, so the result is deterministic
  const int tok = a.seg.global_idx[(size_t)b * N + x];
  constexpr int kBatch = 8;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int c0 = 0; c0 < s.n_chunks; c0 += kBatch) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    f32x4 p0[kBatch], p1[kBatch];
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const int c = min(c0 + e, s.n_chunks - 1);
      const float* p = a.part[which] + ((slot0 + c) * BM + r) * kD + piece * 8;
      p0[e] = *reinterpret_cast<const f32x4*>(p);
      p1[e] = *reinterpret_cast<const f32x4*>(p + 4);
    }
    asm volatile("" ::"v"(p0[0]), "v"(p0[1]), "v"(p0[2]), "v"(p0[3]), "v"(p0[4]), "v"(p0[5]), "v"(p0[6]), "v"(p0[7]),
                 "v"(p1[0]), "v"(p1[1]), "v"(p1[2]), "v"(p1[3]), "v"(p1[4]), "v"(p1[5]), "v"(p1[6]), "v"(p1[7]));
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const float w = c0 + e < s.n_chunks ? 1.f : 0.f;
      acc[0] += w * p0[e].x; acc[1] += w * p0[e].y; acc[2] += w * p0[e].z; acc[3] += w * p0[e].w;
      acc[4] += w * p1[e].x; acc[5] += w * p1[e].y; acc[6] += w * p1[e].z; acc[7] += w * p1[e].w;
    }
  }
  void* dst = which == 0 ? a.dq : which == 1 ? a.dk : a.dv;
  uint4 w;
  w.x = f32_to_bf16_bits(acc[0]) | ((unsigned)f32_to_bf16_bits(acc[1]) << 16);
  w.y = f32_to_bf16_bits(acc[2]) | ((unsigned)f32_to_bf16_bits(acc[3]) << 16);
  w.z = f32_to_bf16_bits(acc[4]) | ((unsigned)f32_to_bf16_bits(acc[5]) << 16);
  w.w = f32_to_bf16_bits(acc[6]) | ((unsigned)f32_to_bf16_bits(acc[7]) << 16);
  *reinterpret_cast<uint4*>(static_cast<unsigned short*>(dst) + ((size_t)bh_i * N + tok) * kD +
                            piece * 8) = w;
  }
}

}  // namespace

hipError_t launch_bwd_mfma(const AttnArgs& a, hipStream_t stream) {
  const dim3 grid(unit_grid(a.B, a.H, a.N, a.n_col)), block(kThreads);
  hipError_t e;
  {
    ProfileScope prof(3, stream);
    hipLaunchKernelGGL(bwd_dq_mfma_kernel, grid, block, 0, stream, a);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfileScope prof(4, stream);
    hipLaunchKernelGGL(bwd_dkv_mfma_kernel, grid, block, 0, stream, a);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (owner_slots(a.N) >= 2)  // partials exist only while question tokens fill <= half the owner slots
    hipLaunchKernelGGL(bwd_finalize_kernel, dim3(kFinalizeBlocks, a.B * a.H, 3), block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace mate
