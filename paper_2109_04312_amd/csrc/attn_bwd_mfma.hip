// bf16 MFMA backward for MATE attention: the derivative of the forward (Section 3 head
// equation restricted to the attention pattern A^i_k) with respect to Q, K and V.
//
// Two kernels, no floating-point atomics, so results are bit-reproducible:
//   dq kernel  -- a workgroup owns 128 queries (sorted order of the head kind, or question
//                 tokens) and streams the key tiles they see, exactly like the forward:
//                 P = exp(S - LSE), dP = dO V^T, dS = P (dP - delta), dQ += dS K.
//                 It also produces delta_k = dO_k . O_k for its queries.
//   dkv kernel -- a workgroup owns 128 keys and streams the query tiles that see them: the
//                 question tokens plus the table tokens of the keys' own segments (every
//                 non-pad token when the keys are question tokens):
//                 dV += P^T dO, dK += dS^T Q.
// Pairs (table query, table key) are therefore recomputed once in each kernel.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_common.h"

namespace mate {
namespace {

constexpr int BM = 128;  // owned rows per workgroup (32 per wavefront)
constexpr int BN = 64;   // streamed rows per tile
constexpr int kThreads = 256;
constexpr int kTileElems = BN * kLdsRow;

struct TileRegs {
  uint4 r[4];
};

// 128 threads fetch a 64-row x 64-dim tile as (4 rows x 8 dims) blocks; x in [0,128).
__device__ inline void load_block4x8(TileRegs& t, const unsigned short* __restrict__ X,
                                     const int* __restrict__ list, int base, int last, int x) {
  const int jg = x & 15, dg = x >> 4;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int tok = list[min(base + jg * 4 + u, last)];
    t.r[u] = *reinterpret_cast<const uint4*>(X + (size_t)tok * kD + dg * 8);
  }
}
// ... and write it to LDS as [row][dim] and, transposed, as [dim][row].
__device__ inline void store_block4x8(const TileRegs& t, unsigned short* nat, unsigned short* tr,
                                      int x) {
  const int jg = x & 15, dg = x >> 4;
  if (nat) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
      *reinterpret_cast<uint4*>(nat + (jg * 4 + u) * kLdsRow + dg * 8) = t.r[u];
  }
  if (tr) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      *reinterpret_cast<uint2*>(tr + (dg * 8 + e) * kLdsRow + jg * 4) = transpose_pick(t.r, e);
  }
}

// Owned-row bookkeeping shared by both kernels: which list the 128 owned rows come from, and
// which sorted-slot window the streamed side covers.
struct Owner {
  bool is_global;
  const int* own_list;   // owned rows: global_idx or perm[view]
  int t0, own_count;
  const int* str_list;   // streamed table tokens: perm[view] (perm[0] for question-token owners)
  int s_lo, s_hi;        // streamed slot window
};

__device__ inline bool make_owner(Owner& w, const AttnArgs& a, int b, int view, int tile, int G,
                                  int L, int n_gt) {
  const int N = a.N;
  w.is_global = tile < n_gt;
  if (w.is_global) {
    w.t0 = tile * BM;
    w.own_list = a.seg.global_idx + (size_t)b * N;
    w.own_count = G;
    w.str_list = a.seg.perm[0] + (size_t)b * N;
    w.s_lo = 0;
    w.s_hi = L;
  } else {
    w.t0 = (tile - n_gt) * BM;
    w.own_list = a.seg.perm[view] + (size_t)b * N;
    w.own_count = L;
    w.str_list = w.own_list;
    const int2* rng = a.seg.slot_rng[view] + (size_t)b * N;
    w.s_lo = rng[w.t0].x;
    w.s_hi = rng[min(w.t0 + BM, L) - 1].y;
  }
  return true;
}

// Epilogue shared by both kernels: a C tile pair (columns = owned rows, registers = head dims)
// scaled, rounded to bf16, transposed through LDS and stored as whole 128-byte token rows.
__device__ inline void store_owned_rows(const f32x16 acc[2], float mul, unsigned short* stage,
                                        unsigned short* __restrict__ out, const int* row_tok,
                                        int wave, int lane) {
  const int m = lane & 31, hl = lane >> 5;
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = f32_to_bf16_bits(acc[db][4 * g] * mul) |
            ((unsigned)f32_to_bf16_bits(acc[db][4 * g + 1] * mul) << 16);
      w.y = f32_to_bf16_bits(acc[db][4 * g + 2] * mul) |
            ((unsigned)f32_to_bf16_bits(acc[db][4 * g + 3] * mul) << 16);
      *reinterpret_cast<uint2*>(stage + (wave * 32 + m) * kLdsRow + db * 32 + 8 * g + 4 * hl) = w;
    }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = wave * 32 + it * 8 + (lane >> 3), piece = lane & 7;
    const int tok = row_tok[row];
    if (tok >= 0)
      *reinterpret_cast<uint4*>(out + (size_t)tok * kD + piece * 8) =
          *reinterpret_cast<const uint4*>(stage + row * kLdsRow + piece * 8);
  }
  __syncthreads();
}

__device__ inline void zero_pad_rows(unsigned short* __restrict__ out, const int* pad_idx, int t0,
                                     int P, int tid) {
  for (int x = tid; x < BM * 8; x += kThreads) {
    const int row = x >> 3, piece = x & 7;
    if (t0 + row < P)
      *reinterpret_cast<uint4*>(out + (size_t)pad_idx[t0 + row] * kD + piece * 8) =
          make_uint4(0, 0, 0, 0);
  }
}

// ======================================================================================
// dQ (and delta)
// ======================================================================================
__global__ __launch_bounds__(kThreads) void bwd_dq_mfma_kernel(AttnArgs a) {
  // per buffer: K [key][dim], V [key][dim], K^T [dim][key]
  __shared__ __attribute__((aligned(16))) unsigned short lds[2 * 3 * kTileElems];
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
  const unsigned short* O = static_cast<const unsigned short*>(a.o) + bh * kD;
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dQ = static_cast<unsigned short*>(a.dq) + bh * kD;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  const int tile = id.tile;
  if (tile >= n_gt + n_lt + n_pt) return;
  if (tile >= n_gt + n_lt) {
    zero_pad_rows(dQ, a.seg.pad_idx + (size_t)b * N, (tile - n_gt - n_lt) * BM, P, tid);
    return;
  }
  Owner w;
  make_owner(w, a, b, view, tile, G, L, n_gt);

  const int q_slot = min(w.t0 + wave * 32 + m, w.own_count - 1);
  const int q_pos = w.own_list[q_slot];
  int my_lo = 0, my_hi = L;
  if (!w.is_global) {
    const int2 r = a.seg.slot_rng[view][(size_t)b * N + q_slot];
    my_lo = r.x;
    my_hi = r.y;
  }
  const int w_lo = __shfl(my_lo, 0, 64), w_hi = __shfl(my_hi, 31, 64);
  const int w_lo_all = __shfl(my_lo, 31, 64), w_hi_all = __shfl(my_hi, 0, 64);
  if (tid < BM) q_tok[tid] = w.t0 + tid < w.own_count ? w.own_list[w.t0 + tid] : -1;

  // this lane's query row and dO row as B operands (column m, k = dims), and delta
  bf16x8 qf[4], gf[4];
  float delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)q_pos * kD + ks * 16 + hl * 8;
    qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + off));
    gf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(dO + off));
    const bf16x8 of = as_bf16x8(*reinterpret_cast<const uint4*>(O + off));
#pragma unroll
    for (int e = 0; e < 8; ++e) delta = fmaf((float)gf[ks][e], (float)of[e], delta);
  }
  delta += __shfl_xor(delta, 32, 64);
  const bool row_ok = w.t0 + wave * 32 + m < w.own_count;
  if (hl == 0 && row_ok) a.delta[bh + q_pos] = delta;
  const float lse2 = a.lse[bh + q_pos] * kLog2e;
  const float sc = a.scale * kLog2e;

  const int n_t0 = (G + BN - 1) / BN;
  const int n_t1 = w.s_hi > w.s_lo ? (w.s_hi - w.s_lo + BN - 1) / BN : 0;
  const int n_tiles = n_t0 + n_t1;

  auto tile_src = [&](int t, const int*& list, int& base, int& last) {
    if (t < n_t0) { list = global_idx; base = t * BN; last = G - 1; }
    else { list = w.str_list; base = w.s_lo + (t - n_t0) * BN; last = w.s_hi - 1; }
  };
  // wavefronts 0-1 stage K (natural + transposed), wavefronts 2-3 stage V (natural)
  auto load = [&](TileRegs& r, int t) {
    const int* list; int base, last;
    tile_src(t, list, base, last);
    load_block4x8(r, tid < 128 ? K : V, list, base, last, tid & 127);
  };
  auto store = [&](const TileRegs& r, int buf) {
    unsigned short* Ks = lds + buf * 3 * kTileElems;
    if (tid < 128) store_block4x8(r, Ks, Ks + 2 * kTileElems, tid);
    else store_block4x8(r, Ks + kTileElems, nullptr, tid - 128);
  };

  f32x16 dq_acc[2] = {zero16(), zero16()};
  TileRegs regs;
  load(regs, 0);
  store(regs, 0);
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const unsigned short* Ks = lds + (t & 1) * 3 * kTileElems;
    const unsigned short* Vs = Ks + kTileElems;
    const unsigned short* Kt = Ks + 2 * kTileElems;
    if (t + 1 < n_tiles) load(regs, t + 1);
    const bool part0 = t < n_t0;
    const int base = part0 ? t * BN : w.s_lo + (t - n_t0) * BN;
    const int lo = part0 ? 0 : my_lo, hi = part0 ? G : my_hi;
    const bool skip = !part0 && (base >= w_hi || base + BN <= w_lo);
    if (!skip) {
      f32x16 s[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int off = (jb * 32 + rho(m)) * kLdsRow + ks * 16 + hl * 8;
          s[jb] = mfma(lds_read8(Ks + off), qf[ks], s[jb]);     // S^T  = K Q^T
          dp[jb] = mfma(lds_read8(Vs + off), gf[ks], dp[jb]);   // dP^T = V dO^T
        }
      const bool full = part0 ? (base + BN <= G) : (base >= w_lo_all && base + BN <= w_hi_all);
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          float p = __builtin_amdgcn_exp2f(s[jb][c] * sc - lse2);
          if (!full) {
            const int slot = base + jb * 32 + tile_row(c, hl);
            if (slot < lo || slot >= hi) p = 0.f;
          }
          s[jb][c] = p * (dp[jb][c] - delta);  // dS^T
        }
      // dQ^T += K^T dS^T
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const bf16x8 db8 = pack8(s[jb], 8 * tt);
#pragma unroll
          for (int db = 0; db < 2; ++db)
            dq_acc[db] = mfma(lds_read8(Kt + (db * 32 + m) * kLdsRow + jb * 32 + tt * 16 + hl * 8),
                              db8, dq_acc[db]);
        }
    }
    if (t + 1 < n_tiles) store(regs, (t + 1) & 1);
    __syncthreads();
  }
  store_owned_rows(dq_acc, a.scale, lds, dQ, q_tok, wave, lane);
}

// ======================================================================================
// dK, dV
// ======================================================================================
__global__ __launch_bounds__(kThreads) void bwd_dkv_mfma_kernel(AttnArgs a) {
  // per buffer: Q [query][dim], dO [query][dim], Q^T [dim][query], dO^T [dim][query]
  __shared__ __attribute__((aligned(16))) unsigned short lds[2 * 4 * kTileElems];
  __shared__ float row_stat[2][2][BN];  // [buffer][lse2 | delta][query]
  __shared__ int k_tok[BM];

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
  const unsigned short* dO = static_cast<const unsigned short*>(a.dout) + bh * kD;
  unsigned short* dK = static_cast<unsigned short*>(a.dk) + bh * kD;
  unsigned short* dV = static_cast<unsigned short*>(a.dv) + bh * kD;
  const float* LSE = a.lse + bh;
  const float* DELTA = a.delta + bh;
  const int* global_idx = a.seg.global_idx + (size_t)b * N;

  const int tile = id.tile;
  if (tile >= n_gt + n_lt + n_pt) return;
  if (tile >= n_gt + n_lt) {
    const int* pad_idx = a.seg.pad_idx + (size_t)b * N;
    zero_pad_rows(dK, pad_idx, (tile - n_gt - n_lt) * BM, P, tid);
    zero_pad_rows(dV, pad_idx, (tile - n_gt - n_lt) * BM, P, tid);
    return;
  }
  Owner w;
  make_owner(w, a, b, view, tile, G, L, n_gt);

  const int k_slot = min(w.t0 + wave * 32 + m, w.own_count - 1);
  const int k_pos = w.own_list[k_slot];
  int my_lo = 0, my_hi = L;  // query slots that see this key (its own segment, or everything)
  if (!w.is_global) {
    const int2 r = a.seg.slot_rng[view][(size_t)b * N + k_slot];
    my_lo = r.x;
    my_hi = r.y;
  }
  const int w_lo = __shfl(my_lo, 0, 64), w_hi = __shfl(my_hi, 31, 64);
  const int w_lo_all = __shfl(my_lo, 31, 64), w_hi_all = __shfl(my_hi, 0, 64);
  if (tid < BM) k_tok[tid] = w.t0 + tid < w.own_count ? w.own_list[w.t0 + tid] : -1;

  bf16x8 kf[4], vf[4];  // this lane's key and value rows as B operands
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const size_t off = (size_t)k_pos * kD + ks * 16 + hl * 8;
    kf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(K + off));
    vf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(V + off));
  }
  const float sc = a.scale * kLog2e;

  const int n_t0 = (G + BN - 1) / BN;
  const int n_t1 = w.s_hi > w.s_lo ? (w.s_hi - w.s_lo + BN - 1) / BN : 0;
  const int n_tiles = n_t0 + n_t1;

  auto tile_src = [&](int t, const int*& list, int& base, int& last) {
    if (t < n_t0) { list = global_idx; base = t * BN; last = G - 1; }
    else { list = w.str_list; base = w.s_lo + (t - n_t0) * BN; last = w.s_hi - 1; }
  };
  // wavefronts 0-1 stage Q, wavefronts 2-3 stage dO (each natural + transposed);
  // threads 0..63 / 128..191 also fetch lse / delta of the 64 streamed queries.
  float stat = 0.f;
  auto load = [&](TileRegs& r, int t) {
    const int* list; int base, last;
    tile_src(t, list, base, last);
    load_block4x8(r, tid < 128 ? Q : dO, list, base, last, tid & 127);
    if ((tid & 127) < BN) {
      const int tok = list[min(base + (tid & 127), last)];
      stat = tid < 128 ? LSE[tok] * kLog2e : DELTA[tok];
    }
  };
  auto store = [&](const TileRegs& r, int buf) {
    unsigned short* Qs = lds + buf * 4 * kTileElems;
    if (tid < 128) store_block4x8(r, Qs, Qs + 2 * kTileElems, tid);
    else store_block4x8(r, Qs + kTileElems, Qs + 3 * kTileElems, tid - 128);
    if ((tid & 127) < BN) row_stat[buf][tid >> 7][tid & 127] = stat;
  };

  f32x16 dk_acc[2] = {zero16(), zero16()}, dv_acc[2] = {zero16(), zero16()};
  TileRegs regs;
  load(regs, 0);
  store(regs, 0);
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int buf = t & 1;
    const unsigned short* Qs = lds + buf * 4 * kTileElems;
    const unsigned short* Gs = Qs + kTileElems;
    const unsigned short* Qt = Qs + 2 * kTileElems;
    const unsigned short* Gt = Qs + 3 * kTileElems;
    if (t + 1 < n_tiles) load(regs, t + 1);
    const bool part0 = t < n_t0;
    const int base = part0 ? t * BN : w.s_lo + (t - n_t0) * BN;
    const int lo = part0 ? 0 : my_lo, hi = part0 ? G : my_hi;
    const bool skip = !part0 && (base >= w_hi || base + BN <= w_lo);
    if (!skip) {
      f32x16 s[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int off = (ib * 32 + rho(m)) * kLdsRow + ks * 16 + hl * 8;
          s[ib] = mfma(lds_read8(Qs + off), kf[ks], s[ib]);     // S  = Q K^T  (rows = queries)
          dp[ib] = mfma(lds_read8(Gs + off), vf[ks], dp[ib]);   // dP = dO V^T
        }
      const bool full = part0 ? (base + BN <= G) : (base >= w_lo_all && base + BN <= w_hi_all);
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          const int row = ib * 32 + tile_row(c, hl);
          float p = __builtin_amdgcn_exp2f(s[ib][c] * sc - row_stat[buf][0][row]);
          if (!full) {
            const int slot = base + row;
            if (slot < lo || slot >= hi) p = 0.f;
          }
          s[ib][c] = p;                                            // P
          dp[ib][c] = p * (dp[ib][c] - row_stat[buf][1][row]);     // dS
        }
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const bf16x8 p8 = pack8(s[ib], 8 * tt), ds8 = pack8(dp[ib], 8 * tt);
#pragma unroll
          for (int db = 0; db < 2; ++db) {
            const int off = (db * 32 + m) * kLdsRow + ib * 32 + tt * 16 + hl * 8;
            dv_acc[db] = mfma(lds_read8(Gt + off), p8, dv_acc[db]);   // dV^T += dO^T P
            dk_acc[db] = mfma(lds_read8(Qt + off), ds8, dk_acc[db]);  // dK^T += Q^T dS
          }
        }
    }
    if (t + 1 < n_tiles) store(regs, (t + 1) & 1);
    __syncthreads();
  }
  store_owned_rows(dk_acc, a.scale, lds, dK, k_tok, wave, lane);
  store_owned_rows(dv_acc, 1.f, lds, dV, k_tok, wave, lane);
}

}  // namespace

hipError_t launch_bwd_mfma(const AttnArgs& a, hipStream_t stream) {
  const int tiles = (a.N + BM - 1) / BM + 2;
  const dim3 grid(grid_blocks(a.B * a.H, tiles)), block(kThreads);
  hipLaunchKernelGGL(bwd_dq_mfma_kernel, grid, block, 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dkv_mfma_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace mate
