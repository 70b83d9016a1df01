// bf16 MFMA forward for MATE attention (Section 3: attention pattern and head equation;
// Section 3.1: per-head-kind ordering so that a token's keys are contiguous).
//
// A workgroup (4 wavefronts) owns 128 consecutive queries of one (sequence, head) in the head
// kind's sorted order -- or 128 question tokens, or 128 pad tokens (zero fill).  It streams the
// keys those queries may see in 64-key tiles: first the question tokens (gathered through
// global_idx), then the sorted slots spanned by the queries' own row / column segments
// (gathered through perm; every table token for a question-token tile).  Each key tile is
// staged in LDS once (K as [key][dim], V transposed to [dim][key]) and used by all four
// wavefronts; scores are masked per element by "key slot inside this query's segment range",
// and one online softmax runs across the question-key and segment-key tiles, which is the
// single softmax over the union that the definition asks for.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_common.h"

namespace mate {
namespace {

constexpr int BM = 128;  // queries per workgroup (32 per wavefront)
constexpr int BN = 64;   // keys per streamed tile
constexpr int kThreads = 256;
constexpr int kTileElems = BN * kLdsRow;  // one staged K (or V^T) tile, in bf16 elements

struct KeyTileRegs {
  uint4 r[4];
};

// Thread roles when staging a key tile: wavefronts 0-1 copy K rows (4 x 16 bytes each),
// wavefronts 2-3 take V, four keys x eight dims per thread, and write it transposed.
__device__ inline void load_key_tile(KeyTileRegs& t, const unsigned short* __restrict__ K,
                                     const unsigned short* __restrict__ V,
                                     const int* __restrict__ list, int base, int last, int tid) {
  if (tid < 128) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int piece = tid + 128 * u;  // 512 pieces of 16 bytes
      const int row = piece >> 3, col = piece & 7;
      const int tok = list[min(base + row, last)];
      t.r[u] = *reinterpret_cast<const uint4*>(K + (size_t)tok * kD + col * 8);
    }
  } else {
    const int x = tid - 128, jg = x & 15, dg = x >> 4;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int tok = list[min(base + jg * 4 + u, last)];
      t.r[u] = *reinterpret_cast<const uint4*>(V + (size_t)tok * kD + dg * 8);
    }
  }
}

__device__ inline void store_key_tile(const KeyTileRegs& t, unsigned short* Ks, unsigned short* Vt,
                                      int tid) {
  if (tid < 128) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int piece = tid + 128 * u;
      const int row = piece >> 3, col = piece & 7;
      *reinterpret_cast<uint4*>(Ks + row * kLdsRow + col * 8) = t.r[u];
    }
  } else {
    const int x = tid - 128, jg = x & 15, dg = x >> 4;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      *reinterpret_cast<uint2*>(Vt + (dg * 8 + e) * kLdsRow + jg * 4) = transpose_pick(t.r, e);
  }
}

__global__ __launch_bounds__(kThreads) void fwd_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned short lds[4 * kTileElems];  // 2 x (K, V^T)
  __shared__ int q_tok[BM];

  const TileId id = map_block(blockIdx.x, a.B * a.H);
  if (!id.valid) return;
  const int b = id.bh / a.H, h = id.bh % a.H;
  const int N = a.N, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hl = lane >> 5;
  const int view = a.head_kind[h];
  if (a.seg.hdr[0] != kMagic || a.seg.hdr[1] != a.B || a.seg.hdr[2] != N) return;

  const int* cnt = a.seg.counts + (size_t)b * kCountWords;
  const int G = cnt[C_G], L = cnt[C_L], P = cnt[C_P];
  const int n_gt = (G + BM - 1) / BM, n_lt = (L + BM - 1) / BM, n_pt = (P + BM - 1) / BM;
  const size_t bh = (size_t)id.bh * N;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q) + bh * kD;
  const unsigned short* K = static_cast<const unsigned short*>(a.k) + bh * kD;
  const unsigned short* V = static_cast<const unsigned short*>(a.v) + bh * kD;
  unsigned short* O = static_cast<unsigned short*>(a.out) + bh * kD;
  float* LSE = a.lse + bh;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  int tile = id.tile;
  if (tile >= n_gt + n_lt + n_pt) return;
  if (tile >= n_gt + n_lt) {  // pad positions: O = 0, LSE = 0
    const int t0 = (tile - n_gt - n_lt) * BM;
    const int* pad_idx = a.seg.pad_idx + (size_t)b * N;
    for (int x = tid; x < BM * 8; x += kThreads) {
      const int row = x >> 3, piece = x & 7;
      if (t0 + row < P) {
        const int tok = pad_idx[t0 + row];
        *reinterpret_cast<uint4*>(O + (size_t)tok * kD + piece * 8) = make_uint4(0, 0, 0, 0);
        if (piece == 0) LSE[tok] = 0.f;
      }
    }
    return;
  }

  // ---- which queries, which keys -------------------------------------------------------
  const bool is_global = tile < n_gt;
  const int* q_list;
  const int* k_list;
  int t0, q_count, k_lo, k_hi;
  if (is_global) {
    t0 = tile * BM;
    q_list = global_idx;
    q_count = G;
    k_list = a.seg.perm[0] + (size_t)b * N;  // all table tokens; row order is the contiguous one
    k_lo = 0;
    k_hi = L;
  } else {
    t0 = (tile - n_gt) * BM;
    q_list = a.seg.perm[view] + (size_t)b * N;
    q_count = L;
    k_list = q_list;
    const int2* rng = a.seg.slot_rng[view] + (size_t)b * N;
    k_lo = rng[t0].x;
    k_hi = rng[min(t0 + BM, L) - 1].y;
  }
  // This lane's query: row m of the wavefront's 32.  Rows past the end repeat the last query
  // (computed, never stored) so that every lane always has at least one visible key.
  const int q_slot = min(t0 + wave * 32 + m, q_count - 1);
  const int q_pos = q_list[q_slot];
  int my_lo = 0, my_hi = L;
  if (!is_global) {
    const int2 r = a.seg.slot_rng[view][(size_t)b * N + q_slot];
    my_lo = r.x;
    my_hi = r.y;
  }
  // Slot range any query of this wavefront can see (queries are sorted, ranges are monotone).
  const int w_lo = __shfl(my_lo, 0, 64), w_hi = __shfl(my_hi, 31, 64);
  // Slot range every query of this wavefront sees (no per-element mask needed inside it).
  const int w_lo_all = __shfl(my_lo, 31, 64), w_hi_all = __shfl(my_hi, 0, 64);
  if (tid < BM) q_tok[tid] = t0 + tid < q_count ? q_list[t0 + tid] : -1;

  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + (size_t)q_pos * kD + ks * 16 + hl * 8));

  const int n_t0 = (G + BN - 1) / BN;                      // question-key tiles
  const int n_t1 = k_hi > k_lo ? (k_hi - k_lo + BN - 1) / BN : 0;  // segment-key tiles
  const int n_tiles = n_t0 + n_t1;
  const float sc = a.scale * kLog2e;

  f32x16 o_acc[2] = {zero16(), zero16()};
  float m_run = -INFINITY, l_run = 0.f;

  auto tile_src = [&](int t, const int*& list, int& base, int& last) {
    if (t < n_t0) { list = global_idx; base = t * BN; last = G - 1; }
    else { list = k_list; base = k_lo + (t - n_t0) * BN; last = k_hi - 1; }
  };

  KeyTileRegs regs;
  {
    const int* list; int base, last;
    tile_src(0, list, base, last);
    load_key_tile(regs, K, V, list, base, last, tid);
    store_key_tile(regs, lds, lds + kTileElems, tid);
  }
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    unsigned short* Ks = lds + (t & 1) * 2 * kTileElems;
    unsigned short* Vt = Ks + kTileElems;
    if (t + 1 < n_tiles) {
      const int* list; int base, last;
      tile_src(t + 1, list, base, last);
      load_key_tile(regs, K, V, list, base, last, tid);
    }
    // visible slot window for this tile: question keys [0,G), else this lane's segment range
    const bool part0 = t < n_t0;
    const int base = part0 ? t * BN : k_lo + (t - n_t0) * BN;
    const int lo = part0 ? 0 : my_lo, hi = part0 ? G : my_hi;
    const bool skip = !part0 && (base >= w_hi || base + BN <= w_lo);
    if (!skip) {
      // S^T = K Q^T : rows = keys of the tile (permuted by rho), columns = this wave's queries
      f32x16 s[2] = {zero16(), zero16()};
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          s[jb] = mfma(lds_read8(Ks + (jb * 32 + rho(m)) * kLdsRow + ks * 16 + hl * 8), qf[ks], s[jb]);

      const bool full = part0 ? (base + BN <= G) : (base >= w_lo_all && base + BN <= w_hi_all);
      float mx = -INFINITY;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          float v = s[jb][c] * sc;
          if (!full) {
            const int slot = base + jb * 32 + tile_row(c, hl);
            if (slot < lo || slot >= hi) v = -INFINITY;
          }
          s[jb][c] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);       // finite from the first visible key on
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
      float psum = 0.f;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          const float p = __builtin_amdgcn_exp2f(s[jb][c] - m_use);
          s[jb][c] = p;
          psum += p;
        }
      l_run = l_run * alpha + psum;
      m_run = m_new;
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int c = 0; c < 16; ++c) o_acc[db][c] *= alpha;
      // O^T += V^T P^T
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const bf16x8 pb = pack8(s[jb], 8 * tt);
#pragma unroll
          for (int db = 0; db < 2; ++db)
            o_acc[db] = mfma(lds_read8(Vt + (db * 32 + m) * kLdsRow + jb * 32 + tt * 16 + hl * 8),
                             pb, o_acc[db]);
        }
    }
    if (t + 1 < n_tiles) {
      unsigned short* Kn = lds + ((t + 1) & 1) * 2 * kTileElems;
      store_key_tile(regs, Kn, Kn + kTileElems, tid);
    }
    __syncthreads();
  }

  // ---- epilogue: normalise, transpose through LDS, store rows of O in token order -------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  unsigned short* Os = lds;  // [BM][kLdsRow]; the loop ended on a barrier
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = f32_to_bf16_bits(o_acc[db][4 * g] * inv) |
            ((unsigned)f32_to_bf16_bits(o_acc[db][4 * g + 1] * inv) << 16);
      w.y = f32_to_bf16_bits(o_acc[db][4 * g + 2] * inv) |
            ((unsigned)f32_to_bf16_bits(o_acc[db][4 * g + 3] * inv) << 16);
      *reinterpret_cast<uint2*>(Os + (wave * 32 + m) * kLdsRow + db * 32 + 8 * g + 4 * hl) = w;
    }
  if (hl == 0 && t0 + wave * 32 + m < q_count) LSE[q_pos] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = wave * 32 + it * 8 + (lane >> 3), piece = lane & 7;
    const int tok = q_tok[row];
    if (tok >= 0)
      *reinterpret_cast<uint4*>(O + (size_t)tok * kD + piece * 8) =
          *reinterpret_cast<const uint4*>(Os + row * kLdsRow + piece * 8);
  }
}

}  // namespace

hipError_t launch_fwd_mfma(const AttnArgs& a, hipStream_t stream) {
  const int tiles = (a.N + BM - 1) / BM + 2;  // question + table + pad tiles, each rounded up
  hipLaunchKernelGGL(fwd_mfma_kernel, dim3(grid_blocks(a.B * a.H, tiles)), dim3(kThreads), 0,
                     stream, a);
  return hipGetLastError();
}

}  // namespace mate
