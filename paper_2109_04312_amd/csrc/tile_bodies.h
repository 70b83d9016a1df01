// What a wavefront does with ONE streamed 64-row tile, shared by the segment kernels and the
// dense-mask kernels: the arithmetic is the same in both (Section 3 head equation: scores,
// one softmax, weighted sum; and its derivative), only the rule that says which (owned row,
// streamed row) pairs belong to the attention pattern differs.  That rule is the Mask argument:
//
//   mask.full          wave-uniform: every pair of this tile belongs to the pattern (no masking)
//   mask.skip(blk)     wave-uniform: no pair of the 32-row block blk belongs to the pattern
//   mask.load(blk)     fetch what in() needs for the 32-row block blk of the tile
//   mask.in(blk, c)    does the pair (this lane's owned row, streamed row c_row(c) of block blk)
//                      belong to the pattern?  c = accumulator register 0..15
//
// Layout everywhere: C tiles have rows = streamed rows, columns = the wavefront's 32 owned rows
// (lane m = owned row, lane half hl), so per-owned-row quantities are per-lane scalars.
#pragma once
#include <hip/hip_runtime.h>

#include "d2l.h"
#include "mfma_common.h"

namespace mate {

// Per-lane LDS offsets of the operand reads: plain 16-byte reads for the four 16-wide k slices,
// transposing reads for the two 32-row blocks of the other operand (see d2l.h).
__device__ __forceinline__ void operand_offsets(int lane, int (&poff)[4], int (&toff)[2][2]) {
  const int m = lane & 31, hl = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) poff[ks] = plain_off(m, hl, ks);
#pragma unroll
  for (int db = 0; db < 2; ++db) {
    toff[db][0] = tr_off(lane, db, 0);
    toff[db][1] = tr_off(lane, db, 1);
  }
}

// Segment path: the owned row meets the streamed sorted slots [lo, hi); the tile's first row is
// slot `base`.  (For the question-token part of a stream lo = 0, hi = G.)
struct WindowMask {
  const bool full;
  const int d0;        // base + 4 hl - lo
  const unsigned len;  // hi - lo
  const int skip_lo, skip_hi;  // wave-uniform: block blk is outside every row's window iff
                               // 32 blk >= skip_hi or 32 blk + 32 <= skip_lo
  // [u_lo, u_hi) = union of the windows of the wavefront's rows, in the same slot numbering as base
  __device__ __forceinline__ WindowMask(bool full_, int base, int hl, int lo, int hi, int u_lo, int u_hi)
      : full(full_), d0(base + 4 * hl - lo), len((unsigned)(hi - lo)), skip_lo(u_lo - base),
        skip_hi(u_hi - base) {}
  __device__ __forceinline__ bool skip(int blk) const { return 32 * blk >= skip_hi || 32 * blk + 32 <= skip_lo; }
  __device__ __forceinline__ void load(int) const {}
  __device__ __forceinline__ bool in(int blk, int c) const {
    return (unsigned)(d0 + blk * 32 + 8 * (c >> 2) + (c & 3)) < len;
  }
};

// Forward: S^T = K Q^T, mask, online softmax in base 2 (running maximum m_run of the raw scores,
// this lane half's share l_run of the row sum, rescaled only when some row's maximum has risen
// by more than `lazy` raw-score units), P rounded to bf16, O^T += V^T P^T.
template <class Mask>
__device__ __forceinline__ void fwd_tile(const char* Kst, const char* Vst, const bf16x8 (&qf)[4],
                                         const int (&koff)[4], const int (&voff)[2][2], float sc,
                                         float lazy, Mask&& mask, f32x16 (&o_acc)[2], float& m_run,
                                         float& l_run) {
  // S^T = K Q^T : rows = keys of the tile, columns = this wave's queries.  (Both 32-key blocks
  // are always computed here: skipping invisible blocks, as the backward bodies do, made this
  // one slower -- the two blocks' instruction streams no longer interleave.)
  f32x16 s[2] = {zero16(), zero16()};
#pragma unroll
  for (int jb = 0; jb < 2; ++jb)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      s[jb] = mfma(read_plain(Kst + jb * 32 * 128, koff[ks]), qf[ks], s[jb]);
  if (!mask.full) {  // wave-uniform: some (query, key) pairs of this tile are outside the pattern
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
      mask.load(jb);
#pragma unroll
      for (int c = 0; c < 16; ++c) s[jb][c] = mask.in(jb, c) ? s[jb][c] : -INFINITY;
    }
  }
  float mx = s[0][0];
#pragma unroll
  for (int c = 1; c < 16; c += 2) mx = fmaxf(fmaxf(mx, s[0][c]), s[0][c + 1 < 16 ? c + 1 : 0]);
#pragma unroll
  for (int c = 0; c < 16; c += 2) mx = fmaxf(fmaxf(mx, s[1][c]), s[1][c + 1]);
  mx = half_max(mx);
  // Rescale only when some row's maximum has moved up by more than `lazy`.  Until then
  // probabilities may exceed 1 by that factor, which changes neither their relative rounding in
  // bf16 nor the fp32 sums' accuracy.
  if (__any(mx > m_run + lazy)) {
    const float m_new = fmaxf(m_run, mx);
    const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((m_run - m_new) * sc);
    l_run *= alpha;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int c = 0; c < 16; ++c) o_acc[db][c] *= alpha;
    m_run = m_new;
  }
  const float msc = m_run == -INFINITY ? 0.f : m_run * sc;
  // P^T = exp2(S^T sc - m sc), rounded to bf16;  O^T += V^T P^T;  l += sum of rounded P
#pragma unroll
  for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
    for (int c = 0; c < 16; ++c) s[jb][c] = __builtin_amdgcn_exp2f(fmaf(s[jb][c], sc, -msc));
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const bf16x8 pb = pack8(s[jb], 8 * tt);
      l_run = sum8(pb, l_run);
      const char* vt = Vst + (jb * 32 + tt * 16) * 128;
#pragma unroll
      for (int db = 0; db < 2; ++db)
        o_acc[db] = mfma(read_transposed(vt, voff[db][0], voff[db][1]), pb, o_acc[db]);
    }
  }
}

// dQ: P = exp2(S sc - lse2), dP^T = V dO^T, dS = P (dP - delta), dQ^T += K^T dS^T; one 32-key block
// at a time, so only one block's scores are live.
template <class Mask>
__device__ __forceinline__ void dq_tile(const char* Kst, const char* Vst, const bf16x8 (&qf)[4],
                                        const bf16x8 (&gf)[4], const int (&koff)[4],
                                        const int (&toff)[2][2], float sc, float lse2, float delta,
                                        Mask&& mask, f32x16 (&dq_acc)[2]) {
#pragma unroll
  for (int jb = 0; jb < 2; ++jb) {
    if (mask.skip(jb)) continue;
    f32x16 s = zero16(), dp = zero16();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      s = mfma(read_plain(Kst + jb * 32 * 128, koff[ks]), qf[ks], s);     // S^T  = K Q^T
      dp = mfma(read_plain(Vst + jb * 32 * 128, koff[ks]), gf[ks], dp);   // dP^T = V dO^T
    }
#pragma unroll
    for (int c = 0; c < 16; ++c)
      s[c] = __builtin_amdgcn_exp2f(fmaf(s[c], sc, -lse2)) * (dp[c] - delta);
    if (!mask.full) {  // wave-uniform: zero the pairs outside the pattern
      mask.load(jb);
#pragma unroll
      for (int c = 0; c < 16; ++c) s[c] = mask.in(jb, c) ? s[c] : 0.f;
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const bf16x8 ds8 = pack8(s, 8 * tt);
      const char* kt = Kst + (jb * 32 + tt * 16) * 128;
#pragma unroll
      for (int db = 0; db < 2; ++db)
        dq_acc[db] = mfma(read_transposed(kt, toff[db][0], toff[db][1]), ds8, dq_acc[db]);
    }
  }
}

// dK, dV: rows of the tile are the streamed queries.  The accumulators start at the rows'
// -lse / scale and -delta (from LDS, four consecutive rows per group of four registers), so the
// contractions deliver S - lse / scale and dP - delta directly: P = exp2(that sc), dS = P (dP - delta);
// dV^T += dO^T P, dK^T += Q^T dS.
template <class Mask>
__device__ __forceinline__ void dkv_tile(const char* Qst, const char* Gst, const float* lse_row,
                                         const float* delta_row, const bf16x8 (&kf)[4],
                                         const bf16x8 (&vf)[4], const int (&poff)[4],
                                         const int (&toff)[2][2], float sc, int hl, Mask&& mask,
                                         f32x16 (&dk_acc)[2], f32x16 (&dv_acc)[2]) {
#pragma unroll
  for (int ib = 0; ib < 2; ++ib) {
    if (mask.skip(ib)) continue;
    f32x16 s, dp;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int row0 = ib * 32 + 8 * g + 4 * hl;
      const float4 l4 = *reinterpret_cast<const float4*>(lse_row + row0);
      const float4 d4 = *reinterpret_cast<const float4*>(delta_row + row0);
      s[4 * g] = l4.x; s[4 * g + 1] = l4.y; s[4 * g + 2] = l4.z; s[4 * g + 3] = l4.w;
      dp[4 * g] = d4.x; dp[4 * g + 1] = d4.y; dp[4 * g + 2] = d4.z; dp[4 * g + 3] = d4.w;
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      s = mfma(read_plain(Qst + ib * 32 * 128, poff[ks]), kf[ks], s);     // S  = Q K^T
      dp = mfma(read_plain(Gst + ib * 32 * 128, poff[ks]), vf[ks], dp);   // dP = dO V^T
    }
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      s[c] = __builtin_amdgcn_exp2f(s[c] * sc);  // P
      dp[c] *= s[c];                             // dS
    }
    if (!mask.full) {  // wave-uniform: zero the pairs outside the pattern
      mask.load(ib);
#pragma unroll
      for (int c = 0; c < 16; ++c) {
        const bool in = mask.in(ib, c);
        s[c] = in ? s[c] : 0.f;
        dp[c] = in ? dp[c] : 0.f;
      }
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const bf16x8 p8 = pack8(s, 8 * tt), ds8 = pack8(dp, 8 * tt);
      const char* gt = Gst + (ib * 32 + tt * 16) * 128;
      const char* qt = Qst + (ib * 32 + tt * 16) * 128;
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        dv_acc[db] = mfma(read_transposed(gt, toff[db][0], toff[db][1]), p8, dv_acc[db]);   // dV^T += dO^T P
        dk_acc[db] = mfma(read_transposed(qt, toff[db][0], toff[db][1]), ds8, dk_acc[db]);  // dK^T += Q^T dS
      }
    }
  }
}

}  // namespace mate
