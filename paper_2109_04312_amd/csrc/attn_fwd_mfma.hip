// bf16 MFMA forward for MATE attention (Section 3: attention pattern and head equation;
// Section 3.1: per-head-kind ordering so that a token's keys are contiguous).
//
// A workgroup (4 wavefronts) owns 128 consecutive queries of one (sequence, head) in the head
// kind's sorted order -- or 128 question tokens, or 1024 pad tokens (zero fill).  It streams the
// keys those queries may see in 64-key tiles: first the question tokens (gathered through
// global_idx), then the sorted slots spanned by the queries' own row / column segments
// (gathered through perm; every table token for question-token owners, whose key stream is cut
// into chunks run by separate workgroups).  Each key tile goes straight from global memory
// into LDS once (K and V both as [key][dim]; V^T is produced by transposing LDS reads) and is
// used by all four wavefronts; scores are masked per element by "key slot inside this query's
// segment range", and one online softmax runs across
// the question-key and segment-key tiles, which is the single softmax over the union that the
// definition asks for.  Chunked owners leave (unnormalised O, max, sum) partials that the
// finalize kernel merges with the usual log-sum-exp rule.
#include <hip/hip_runtime.h>

#include "d2l.h"
#include "launch.h"
#include "mfma_common.h"
#include "stream_plan.h"
#include "tile_bodies.h"
#include "tile_stream.h"

namespace mate {
namespace {

constexpr int kStageBytes = 2 * kTileBytes;   // K tile, V tile
constexpr float kLazyBits = 8.f;
constexpr int NS = 2;  // LDS stages: small enough for four workgroups per CU

__device__ __forceinline__ void fwd_unit(const AttnArgs& a, const Work& w) {
  __shared__ __attribute__((aligned(1024))) char lds[NS * kStageBytes];
  __shared__ int idx_ring[kIdxSlots][BN];  // [tile & 7][row] token positions
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
  unsigned short* O = static_cast<unsigned short*>(a.out) + bh * kD;
  float* LSE = a.lse + bh;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  if (u.kind == UNIT_PAD) {  // pad positions: O = 0, LSE = 0
    unsigned short* const outs[1] = {O};
    zero_pad_rows<1>(outs, u, tid);
    int tok[kPadSlots / kThreads];
#pragma unroll
    for (int i = 0; i < kPadSlots / kThreads; ++i) {
      const int row = u.t0 + tid + i * kThreads;
      tok[i] = row < u.own_count ? u.own_list[row] : -1;
    }
#pragma unroll
    for (int i = 0; i < kPadSlots / kThreads; ++i)
      if (tok[i] >= 0) LSE[tok[i]] = 0.f;
    return;
  }

  // First round trip: which rows this workgroup owns, and the token indices of the first tiles.
  // Second: the owned query rows (registers) and the first K / V tiles (LDS), all in flight
  // together.
  TileStream<kStageBytes, NS> stream(u, global_idx, lds, idx_ring, K, V, nullptr, 0, wave, lane);
  stream.begin();
  const OwnedRow me = owned_row(u, a, b, view, wave, m);
  asm volatile("" ::"v"(me.pos), "v"(me.lo), "v"(me.hi), "v"(me.stage_tok));  // the owned rows are known from here on
  if (tid < BM) q_tok[tid] = me.stage_tok;
  stream.prime();

  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + (size_t)me.pos * kD + ks * 16 + hl * 8));

  const float sc = a.scale * kLog2e;  // scores are kept raw; exp2(s * sc - m * sc)
  const float lazy = kLazyBits / sc;   // in raw-score units
  f32x16 o_acc[2] = {zero16(), zero16()};
  float m_run = -INFINITY, l_run = 0.f;  // running max of raw scores; this lane-half's share of the sum

  const int tb = u.t_begin, te = u.t_end;
  // Everything loaded into registers so far is pinned as complete here, so that no load with a
  // register destination is pending inside the loop (the compiler would otherwise wait for
  // *all* outstanding loads, prefetches included, at the first use).
  asm volatile("" ::"v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]));

  int koff[4], voff[2][2];
  operand_offsets(lane, koff, voff);

  for (int t = tb; t < te; ++t) {
    const char* Kst = stream.acquire(t);
    const char* Vst = Kst + kTileBytes;

    // visible slot window for this tile: question keys [0,G), else this lane's segment range
    const bool part0 = t < u.n_t0;
    const int base = part0 ? t * BN : u.s_lo + (t - u.n_t0) * BN;
    const bool skip = !me.wave_active || (!part0 && (base >= me.w_hi || base + BN <= me.w_lo));
    if (!skip) {
      const bool full = part0 ? (base + BN <= u.G) : (base >= me.a_lo && base + BN <= me.a_hi);
      fwd_tile(Kst, Vst, qf, koff, voff, sc, lazy, WindowMask(full, base, hl, part0 ? 0 : me.lo, part0 ? u.G : me.hi, part0 ? 0 : me.w_lo, part0 ? u.G : me.w_hi), o_acc, m_run, l_run);
    }
    stream.release();
  }
  __syncthreads();  // all wavefronts are done reading the stages; reuse them for the epilogue

  const float l_tot = half_sum(l_run);
  if (u.part >= 0) {
    // chunk of a question-token owner: leave (unnormalised O, max, sum) for the finalize kernel
    const size_t slot = (size_t)w.bh * owner_slots(N) + u.part;
    store_partial(o_acc, 1.f, a.part[0] + slot * BM * kD, wave, lane);
    if (hl == 0)
      *reinterpret_cast<float2*>(a.part_ml + (slot * BM + wave * 32 + m) * 2) =
          make_float2(m_run == -INFINITY ? m_run : m_run * sc, l_tot);
    return;
  }
  if (hl == 0 && me.valid) LSE[me.pos] = (m_run * sc + __builtin_amdgcn_logf(l_tot)) * kLn2;
  const f32x16 (*accs[1])[2] = {&o_acc};
  const float muls[1] = {1.f / l_tot};
  unsigned short* const outs[1] = {O};
  store_owned_rows<1>(accs, muls, outs, lds, q_tok, wave, lane);
}

__global__ __launch_bounds__(kThreads, 4) void fwd_mfma_kernel(AttnArgs a) {
  Work w;
  if (!take_unit<false>(a, w)) return;
  fwd_unit(a, w);
}

// Merges the chunk partials of question-token queries: O = sum_c 2^(m_c - m) O_c / sum_c 2^(m_c - m) l_c.
// 8 threads per query row (8 dims each), 32 rows per workgroup.
__global__ __launch_bounds__(kThreads) void fwd_finalize_kernel(AttnArgs a) {
  const int bh_i = blockIdx.y, b = bh_i / a.H, N = a.N;
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
  const int tok = a.seg.global_idx[(size_t)b * N + x];
  const size_t slot0 = (size_t)bh_i * owner_slots(N) + (size_t)gt * s.n_chunks;
  // Chunks are read kBatch at a time with all loads of a batch issued before the first use (the
  // pin at the end of load_batch: left alone, the compiler keeps only a few in flight and the
  // kernel becomes a chain of memory round trips).  The chunk count is only known on the device;
  // the combination order is fixed, so the result is deterministic.  A first batch usually
  // covers every chunk: then each partial is read exactly once.
  constexpr int kBatch = 8;
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  float m = -INFINITY;
  f32x2 ml[kBatch];
  f32x4 p0[kBatch], p1[kBatch];
  auto load_batch = [&](int c0) {
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const int c = min(c0 + e, s.n_chunks - 1);
      ml[e] = *reinterpret_cast<const f32x2*>(a.part_ml + ((slot0 + c) * BM + r) * 2);
      const float* p = a.part[0] + ((slot0 + c) * BM + r) * kD + piece * 8;
      p0[e] = *reinterpret_cast<const f32x4*>(p);
      p1[e] = *reinterpret_cast<const f32x4*>(p + 4);
    }
    asm volatile("" ::"v"(p0[0]), "v"(p0[1]), "v"(p0[2]), "v"(p0[3]), "v"(p0[4]), "v"(p0[5]), "v"(p0[6]), "v"(p0[7]),
                 "v"(p1[0]), "v"(p1[1]), "v"(p1[2]), "v"(p1[3]), "v"(p1[4]), "v"(p1[5]), "v"(p1[6]), "v"(p1[7]),
                 "v"(ml[0]), "v"(ml[1]), "v"(ml[2]), "v"(ml[3]), "v"(ml[4]), "v"(ml[5]), "v"(ml[6]), "v"(ml[7]));
  };
  load_batch(0);
#pragma unroll
  for (int e = 0; e < kBatch; ++e) m = fmaxf(m, e < s.n_chunks ? ml[e].x : -INFINITY);
  for (int c0 = kBatch; c0 < s.n_chunks; c0 += 8) {  // more chunks than one batch: finish the maximum first
    float mv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      mv[e] = c0 + e < s.n_chunks ? a.part_ml[((slot0 + c0 + e) * BM + r) * 2] : -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) m = fmaxf(m, mv[e]);
  }
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, l = 0.f;
  for (int c0 = 0; c0 < s.n_chunks; c0 += kBatch) {
    if (c0) load_batch(c0);
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const float w = c0 + e < s.n_chunks ? __builtin_amdgcn_exp2f(ml[e].x - m) : 0.f;
      l += w * ml[e].y;
      acc[0] += w * p0[e].x; acc[1] += w * p0[e].y; acc[2] += w * p0[e].z; acc[3] += w * p0[e].w;
      acc[4] += w * p1[e].x; acc[5] += w * p1[e].y; acc[6] += w * p1[e].z; acc[7] += w * p1[e].w;
    }
  }
  const float inv = 1.f / l;
  const size_t bh = (size_t)bh_i * N;
  uint4 w;
  w.x = f32_to_bf16_bits(acc[0] * inv) | ((unsigned)f32_to_bf16_bits(acc[1] * inv) << 16);
  w.y = f32_to_bf16_bits(acc[2] * inv) | ((unsigned)f32_to_bf16_bits(acc[3] * inv) << 16);
  w.z = f32_to_bf16_bits(acc[4] * inv) | ((unsigned)f32_to_bf16_bits(acc[5] * inv) << 16);
  w.w = f32_to_bf16_bits(acc[6] * inv) | ((unsigned)f32_to_bf16_bits(acc[7] * inv) << 16);
  *reinterpret_cast<uint4*>(static_cast<unsigned short*>(a.out) + (bh + tok) * kD + piece * 8) = w;
  if (piece == 0) a.lse[bh + tok] = (m + __builtin_amdgcn_logf(l)) * kLn2;
  }
}

}  // namespace

hipError_t launch_fwd_mfma(const AttnArgs& a, hipStream_t stream) {
  {
    ProfileScope prof(2, stream);
    hipLaunchKernelGGL(fwd_mfma_kernel, dim3(unit_grid(a.B, a.H, a.N, a.n_col)), dim3(kThreads), 0, stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // partials exist only while question tokens fill at most half the owner slots; a few
  // workgroups per (b,h) stride over however many question tokens there are
  if (owner_slots(a.N) >= 2)
    hipLaunchKernelGGL(fwd_finalize_kernel, dim3(kFinalizeBlocks, a.B * a.H), dim3(kThreads), 0,
                       stream, a);
  return hipGetLastError();
}

}  // namespace mate
