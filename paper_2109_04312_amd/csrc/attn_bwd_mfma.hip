// bf16 MFMA backward for MATE attention: the derivative of the forward (Section 3 head
// equation restricted to the attention pattern A^i_k) with respect to Q, K and V.
//
// No floating-point atomics, so results are bit-reproducible:
//   dq kernel  -- a workgroup owns 128 queries (sorted order of the head kind, or question
//                 tokens) and streams the key tiles they see, exactly like the forward:
//                 P = exp(S - LSE), dP = dO V^T, dS = P (dP - delta), dQ += dS K.
//                 It also produces delta_k = dO_k . O_k for its queries.
//   dkv kernel -- a workgroup owns 128 keys and streams the query tiles that see them: the
//                 question tokens plus the table tokens of the keys' own segments (every
//                 non-pad token when the keys are question tokens):
//                 dV += P^T dO, dK += dS^T Q.
//   finalize   -- question-token owners stream the whole sequence, so their stream is cut into
//                 chunks run by separate workgroups; this kernel adds the fp32 partials in
//                 chunk order.
// Pairs (table query, table key) are therefore recomputed once in each of the first two.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_common.h"
#include "stream_plan.h"

namespace mate {
namespace {

// ======================================================================================
// dQ (and delta)
// ======================================================================================
__device__ __forceinline__ int bwd_dq_unit(const AttnArgs& a) {
  // per buffer: K [key][dim], V [key][dim], K^T [dim][key]
  __shared__ __attribute__((aligned(16))) unsigned short lds[2 * 3 * kTileElems];
  __shared__ int q_tok[BM];

  const TileId id = map_block(blockIdx.x, a.B * a.H);
  if (!id.valid || !tables_match(a)) return 0;
  const int b = id.bh / a.H, h = id.bh % a.H;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hl = lane >> 5;
  const int view = a.head_kind[h];
  const UnitPlan u = plan_unit(a, b, view, id.tile);
  if (u.kind == UNIT_NONE) return 0;

  const size_t bh = (size_t)id.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  const unsigned short* O = static_cast<const unsigned short*>(a.o) + bh * kD;
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dQ = static_cast<unsigned short*>(a.dq) + bh * kD;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  if (u.kind == UNIT_PAD) {
    zero_pad_rows(dQ, u, tid);
    return unit_info(u);
  }
  const OwnedRow me = owned_row(u, a, b, view, wave, m);
  if (tid < BM) q_tok[tid] = u.t0 + tid < u.own_count ? u.own_list[u.t0 + tid] : -1;

  // this lane's query row and dO row as B operands (column m, k = dims), and delta
  bf16x8 qf[4], gf[4];
  float delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)me.pos * kD + ks * 16 + hl * 8;
    qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + off));
    gf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(dO + off));
    const bf16x8 of = as_bf16x8(*reinterpret_cast<const uint4*>(O + off));
#pragma unroll
    for (int e = 0; e < 8; ++e) delta = fmaf((float)gf[ks][e], (float)of[e], delta);
  }
  delta += __shfl_xor(delta, 32, 64);
  // every chunk of a question-token owner computes the same delta; the first one stores it
  if (hl == 0 && me.valid && u.t_begin == 0) a.delta[bh + me.pos] = delta;
  const float lse2 = a.lse[bh + me.pos] * kLog2e;
  const float sc = a.scale * kLog2e;

  // wavefronts 0-1 stage K (natural + transposed), wavefronts 2-3 stage V (natural); token
  // indices are fetched two tiles ahead, rows one tile ahead
  const unsigned short* stage_src = tid < 128 ? K : V;
  const int sx = tid & 127;
  auto fetch_idx = [&](TileIdx& ix, int t) {
    const int* list; int base, last;
    tile_source(u, global_idx, t, list, base, last);
    load_tile_idx(ix, list, base, last, sx);
  };
  auto store = [&](const TileRegs& r, int buf) {
    unsigned short* Ks = lds + buf * 3 * kTileElems;
    if (tid < 128) store_block4x8(r, Ks, Ks + 2 * kTileElems, tid);
    else store_block4x8(r, Ks + kTileElems, nullptr, tid - 128);
  };

  f32x16 dq_acc[2] = {zero16(), zero16()};
  TileIdx idx;
  TileRegs regs;
  fetch_idx(idx, u.t_begin);
  load_tile_rows(regs, stage_src, idx, sx);
  if (u.t_begin + 1 < u.t_end) fetch_idx(idx, u.t_begin + 1);
  store(regs, 0);
  __syncthreads();

  const int k_off = rho(m) * kLdsRow + hl * 8, t_off = m * kLdsRow + hl * 8;
  for (int t = u.t_begin; t < u.t_end; ++t) {
    const int buf = (t - u.t_begin) & 1;
    const unsigned short* Kp = lds + buf * 3 * kTileElems + k_off;
    const unsigned short* Vp = Kp + kTileElems;
    const unsigned short* Ktp = lds + buf * 3 * kTileElems + 2 * kTileElems + t_off;
    if (t + 1 < u.t_end) {
      load_tile_rows(regs, stage_src, idx, sx);
      if (t + 2 < u.t_end) fetch_idx(idx, t + 2);
    }
    const bool part0 = t < u.n_t0;
    const int base = part0 ? t * BN : u.s_lo + (t - u.n_t0) * BN;
    const bool skip = !me.wave_active || (!part0 && (base >= me.w_hi || base + BN <= me.w_lo));
    if (!skip) {
      f32x16 s[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          s[jb] = mfma(lds_read8(Kp + jb * 32 * kLdsRow + ks * 16), qf[ks], s[jb]);     // S^T  = K Q^T
          dp[jb] = mfma(lds_read8(Vp + jb * 32 * kLdsRow + ks * 16), gf[ks], dp[jb]);   // dP^T = V dO^T
        }
      // P = exp2(S sc - lse2); dS = P (dP - delta)
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int c = 0; c < 16; ++c)
          s[jb][c] = __builtin_amdgcn_exp2f(fmaf(s[jb][c], sc, -lse2)) * (dp[jb][c] - delta);
      const bool full = part0 ? (base + BN <= u.G) : (base >= me.a_lo && base + BN <= me.a_hi);
      if (!full) {  // wave-uniform: zero the pairs outside the pattern
        const int lo = part0 ? 0 : me.lo, hi = part0 ? u.G : me.hi;
        const int d0 = base + 8 * hl - lo;
        const unsigned len = (unsigned)(hi - lo);
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int c = 0; c < 16; ++c) {
            const bool in = (unsigned)(d0 + jb * 32 + 16 * (c >> 3) + (c & 7)) < len;
            s[jb][c] = in ? s[jb][c] : 0.f;
          }
      }
      // dQ^T += K^T dS^T
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const bf16x8 ds8 = pack8(s[jb], 8 * tt);
#pragma unroll
          for (int db = 0; db < 2; ++db)
            dq_acc[db] = mfma(lds_read8(Ktp + db * 32 * kLdsRow + jb * 32 + tt * 16), ds8, dq_acc[db]);
        }
    }
    if (t + 1 < u.t_end) store(regs, buf ^ 1);
    __syncthreads();
  }
  if (u.part >= 0) {
    const size_t slot = (size_t)id.bh * owner_slots(N) + u.part;
    store_partial(dq_acc, a.scale, a.part[0] + slot * BM * kD, wave, lane);
    return unit_info(u);
  }
  store_owned_rows(dq_acc, a.scale, lds, dQ, q_tok, wave, lane);
  return unit_info(u);
}

__global__ __launch_bounds__(kThreads) void bwd_dq_mfma_kernel(AttnArgs a) {
  MATE_TRACE_KERNEL(bwd_dq_unit(a), 1)
}

// ======================================================================================
// dK, dV
// ======================================================================================
__device__ __forceinline__ int bwd_dkv_unit(const AttnArgs& a) {
  // per buffer: Q [query][dim], dO [query][dim], Q^T [dim][query], dO^T [dim][query]
  __shared__ __attribute__((aligned(16))) unsigned short lds[2 * 4 * kTileElems];
  __shared__ float row_stat[2][2][BN];  // [buffer][lse2 | delta][query]
  __shared__ int k_tok[BM];

  const TileId id = map_block(blockIdx.x, a.B * a.H);
  if (!id.valid || !tables_match(a)) return 0;
  const int b = id.bh / a.H, h = id.bh % a.H;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hl = lane >> 5;
  const int view = a.head_kind[h];
  const UnitPlan u = plan_unit(a, b, view, id.tile);
  if (u.kind == UNIT_NONE) return 0;

  const size_t bh = (size_t)id.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dK = static_cast<unsigned short*>(a.dk) + bh * kD;
  unsigned short* dV = static_cast<unsigned short*>(a.dv) + bh * kD;
  const float* LSE = a.lse + bh;
  const float* DELTA = a.delta + bh;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  if (u.kind == UNIT_PAD) {
    zero_pad_rows(dK, u, tid);
    zero_pad_rows(dV, u, tid);
    return unit_info(u);
  }
  // `me` is this lane's key; its window is the set of query slots that see it
  const OwnedRow me = owned_row(u, a, b, view, wave, m);
  if (tid < BM) k_tok[tid] = u.t0 + tid < u.own_count ? u.own_list[u.t0 + tid] : -1;

  bf16x8 kf[4], vf[4];  // this lane's key and value rows as B operands
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)me.pos * kD + ks * 16 + hl * 8;
    kf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(K + off));
    vf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(V + off));
  }
  const float sc = a.scale * kLog2e;

  // wavefronts 0-1 stage Q, wavefronts 2-3 stage dO (each natural + transposed);
  // threads 0..63 / 128..191 also fetch lse / delta of the 64 streamed queries.  Token indices
  // are fetched two tiles ahead, rows one tile ahead.
  const unsigned short* stage_src = tid < 128 ? Q : dO;
  const float* stat_src = tid < 128 ? LSE : DELTA;
  const float stat_mul = tid < 128 ? kLog2e : 1.f;
  const int sx = tid & 127;
  int stat_tok = 0;
  float stat = 0.f;
  auto fetch_idx = [&](TileIdx& ix, int t) {
    const int* list; int base, last;
    tile_source(u, global_idx, t, list, base, last);
    load_tile_idx(ix, list, base, last, sx);
    if (sx < BN) stat_tok = list[min(base + sx, last)];
  };
  auto fetch_rows = [&](TileRegs& r, const TileIdx& ix) {
    load_tile_rows(r, stage_src, ix, sx);
    if (sx < BN) stat = stat_src[stat_tok] * stat_mul;
  };
  auto store = [&](const TileRegs& r, int buf) {
    unsigned short* Qs = lds + buf * 4 * kTileElems;
    if (tid < 128) store_block4x8(r, Qs, Qs + 2 * kTileElems, tid);
    else store_block4x8(r, Qs + kTileElems, Qs + 3 * kTileElems, tid - 128);
    if (sx < BN) row_stat[buf][tid >> 7][sx] = stat;
  };

  f32x16 dk_acc[2] = {zero16(), zero16()}, dv_acc[2] = {zero16(), zero16()};
  TileIdx idx;
  TileRegs regs;
  fetch_idx(idx, u.t_begin);
  fetch_rows(regs, idx);
  if (u.t_begin + 1 < u.t_end) fetch_idx(idx, u.t_begin + 1);
  store(regs, 0);
  __syncthreads();

  const int n_off = rho(m) * kLdsRow + hl * 8, t_off = m * kLdsRow + hl * 8;
  for (int t = u.t_begin; t < u.t_end; ++t) {
    const int buf = (t - u.t_begin) & 1;
    const unsigned short* Qp = lds + buf * 4 * kTileElems + n_off;
    const unsigned short* Gp = Qp + kTileElems;
    const unsigned short* Qtp = lds + buf * 4 * kTileElems + 2 * kTileElems + t_off;
    const unsigned short* Gtp = Qtp + kTileElems;
    if (t + 1 < u.t_end) {
      fetch_rows(regs, idx);
      if (t + 2 < u.t_end) fetch_idx(idx, t + 2);
    }
    const bool part0 = t < u.n_t0;
    const int base = part0 ? t * BN : u.s_lo + (t - u.n_t0) * BN;
    const bool skip = !me.wave_active || (!part0 && (base >= me.w_hi || base + BN <= me.w_lo));
    if (!skip) {
      f32x16 s[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          s[ib] = mfma(lds_read8(Qp + ib * 32 * kLdsRow + ks * 16), kf[ks], s[ib]);     // S  = Q K^T
          dp[ib] = mfma(lds_read8(Gp + ib * 32 * kLdsRow + ks * 16), vf[ks], dp[ib]);   // dP = dO V^T
        }
      // rows of these tiles are the streamed queries: their lse / delta come from LDS, eight
      // consecutive rows per group of eight registers
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const int row0 = ib * 32 + tt * 16 + 8 * hl;
          const float4 l0 = *reinterpret_cast<const float4*>(&row_stat[buf][0][row0]);
          const float4 l1 = *reinterpret_cast<const float4*>(&row_stat[buf][0][row0 + 4]);
          const float4 d0 = *reinterpret_cast<const float4*>(&row_stat[buf][1][row0]);
          const float4 d1 = *reinterpret_cast<const float4*>(&row_stat[buf][1][row0 + 4]);
          const float ls[8] = {l0.x, l0.y, l0.z, l0.w, l1.x, l1.y, l1.z, l1.w};
          const float de[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int c = tt * 8 + e;
            const float p = __builtin_amdgcn_exp2f(fmaf(s[ib][c], sc, -ls[e]));
            s[ib][c] = p;                           // P
            dp[ib][c] = p * (dp[ib][c] - de[e]);    // dS
          }
        }
      const bool full = part0 ? (base + BN <= u.G) : (base >= me.a_lo && base + BN <= me.a_hi);
      if (!full) {  // wave-uniform: zero the pairs outside the pattern
        const int lo = part0 ? 0 : me.lo, hi = part0 ? u.G : me.hi;
        const int d0 = base + 8 * hl - lo;
        const unsigned len = (unsigned)(hi - lo);
#pragma unroll
        for (int ib = 0; ib < 2; ++ib)
#pragma unroll
          for (int c = 0; c < 16; ++c) {
            const bool in = (unsigned)(d0 + ib * 32 + 16 * (c >> 3) + (c & 7)) < len;
            s[ib][c] = in ? s[ib][c] : 0.f;
            dp[ib][c] = in ? dp[ib][c] : 0.f;
          }
      }
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const bf16x8 p8 = pack8(s[ib], 8 * tt), ds8 = pack8(dp[ib], 8 * tt);
#pragma unroll
          for (int db = 0; db < 2; ++db) {
            const int off = db * 32 * kLdsRow + ib * 32 + tt * 16;
            dv_acc[db] = mfma(lds_read8(Gtp + off), p8, dv_acc[db]);   // dV^T += dO^T P
            dk_acc[db] = mfma(lds_read8(Qtp + off), ds8, dk_acc[db]);  // dK^T += Q^T dS
          }
        }
    }
    if (t + 1 < u.t_end) store(regs, buf ^ 1);
    __syncthreads();
  }
  if (u.part >= 0) {
    const size_t slot = (size_t)id.bh * owner_slots(N) + u.part;
    store_partial(dk_acc, a.scale, a.part[1] + slot * BM * kD, wave, lane);
    store_partial(dv_acc, 1.f, a.part[2] + slot * BM * kD, wave, lane);
    return unit_info(u);
  }
  store_owned_rows(dk_acc, a.scale, lds, dK, k_tok, wave, lane);
  store_owned_rows(dv_acc, 1.f, lds, dV, k_tok, wave, lane);
  return unit_info(u);
}

__global__ __launch_bounds__(kThreads) void bwd_dkv_mfma_kernel(AttnArgs a) {
  MATE_TRACE_KERNEL(bwd_dkv_unit(a), 2)
}

// Adds the chunk partials of question-token rows in chunk order and stores dQ, dK, dV rows.
// blockIdx.z selects the tensor; 8 threads per row, 32 rows per workgroup.
__global__ __launch_bounds__(kThreads) void bwd_finalize_kernel(AttnArgs a) {
  const int bh_i = blockIdx.y, b = bh_i / a.H, N = a.N, which = blockIdx.z;
  if (!tables_match(a)) return;
  const int* cnt = a.seg.counts + (size_t)b * kCountWords;
  const int G = cnt[C_G], L = cnt[C_L];
  const GlobalSplit s = global_split(G, L, N);
  if (s.n_chunks <= 1) return;
  const int piece = threadIdx.x & 7;
  for (int x = blockIdx.x * 32 + (threadIdx.x >> 3); x < G; x += gridDim.x * 32) {
  const int gt = x / BM, r = x % BM;
  const size_t slot0 = (size_t)bh_i * owner_slots(N) + (size_t)gt * s.n_chunks;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int c = 0; c < s.n_chunks; ++c) {
    const float* p = a.part[which] + ((slot0 + c) * BM + r) * kD + piece * 8;
    const float4 p0 = *reinterpret_cast<const float4*>(p), p1 = *reinterpret_cast<const float4*>(p + 4);
    acc[0] += p0.x; acc[1] += p0.y; acc[2] += p0.z; acc[3] += p0.w;
    acc[4] += p1.x; acc[5] += p1.y; acc[6] += p1.z; acc[7] += p1.w;
  }
  const int tok = a.seg.global_idx[(size_t)b * N + x];
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
  const dim3 grid(grid_blocks(a.B * a.H, units_per_bh(a.N))), block(kThreads);
  hipLaunchKernelGGL(bwd_dq_mfma_kernel, grid, block, 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dkv_mfma_kernel, grid, block, 0, stream, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (owner_slots(a.N) >= 2)  // partials exist only while question tokens fill <= half the owner slots
    hipLaunchKernelGGL(bwd_finalize_kernel, dim3(kFinalizeBlocks, a.B * a.H, 3), block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace mate
