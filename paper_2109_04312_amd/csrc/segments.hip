// Segment builder: the per-head-kind reordering of Section 3.1 (row-order / column-order
// traversal of the table tokens), computed as a stable sort by id plus run boundaries.
// Integer work only.  One 1024-thread workgroup per (sequence, view); the whole sort lives in
// LDS as a bitonic network over 64-bit keys (id << 32 | position): positions make all keys
// distinct, so any correct sort of them IS the stable sort by id.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "seg_layout.h"

namespace mate {

constexpr int kSegThreads = 1024;
constexpr int kSegWaves = kSegThreads / 64;

// Exclusive prefix sum of one int per thread across the workgroup; `total` gets the sum.
// `tmp` is kSegWaves + 1 ints of LDS.  Ends with a barrier so `tmp` can be reused at once.
__device__ inline int block_exclusive_scan(int v, int* tmp, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int up = __shfl_up(inc, d, 64);
    if (lane >= d) inc += up;
  }
  if (lane == 63) tmp[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSegWaves; ++w) {
    int s = tmp[w];
    if (w < wave) base += s;
    tot += s;
  }
  __syncthreads();
  total = tot;
  return base + inc - v;
}

template <int P2>
__global__ __launch_bounds__(kSegThreads) void build_segments_kernel(
    const int* __restrict__ row_ids, const int* __restrict__ col_ids,
    const unsigned char* __restrict__ flags, int B, int N, int* __restrict__ seg) {
  constexpr int PER = P2 / kSegThreads;  // consecutive elements owned by one thread
  static_assert(PER >= 1, "P2 must be at least the workgroup size");
  __shared__ unsigned long long keys[P2];
  __shared__ int scan_tmp[kSegWaves + 1];

  const int b = blockIdx.x, view = blockIdx.y, tid = threadIdx.x;
  const SegLayout lay(B, N);
  int* counts = seg + lay.counts + (size_t)b * kCountWords;
  int* global_idx = seg + lay.global_idx + (size_t)b * N;
  int* pad_idx = seg + lay.pad_idx + (size_t)b * N;
  int* vbase = seg + lay.view0 + (size_t)view * lay.view_stride;
  int* perm = vbase + lay.perm + (size_t)b * N;
  int* seg_off = vbase + lay.seg_off + (size_t)b * (N + 1);
  int* seg_of_tok = vbase + lay.seg_of_tok + (size_t)b * N;
  int2* slot_rng = reinterpret_cast<int2*>(vbase + lay.slot_rng) + (size_t)b * N;
  const int* ids = (view == 0 ? row_ids : col_ids) + (size_t)b * N;
  const unsigned char* fl = flags + (size_t)b * N;

  if (b == 0 && view == 0 && tid < kHdrWords)
    seg[tid] = tid == 0 ? kMagic : tid == 1 ? B : tid == 2 ? N : 0;

  // ---- classify: keys for table tokens, sentinel for everything else -------------------
  int n_g = 0, n_p = 0, n_l = 0, bad = 0;
  unsigned char my_flag[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int i = tid * PER + e;
    unsigned long long key = ~0ull;
    unsigned char f = 2;
    if (i < N) {
      f = fl[i];
      if (f > 2) { bad = 1; f = 2; }
      if (f == 0) {
        const int id = ids[i];
        if (id < 0) bad = 1;
        key = ((unsigned long long)(unsigned)id << 32) | (unsigned)i;
        ++n_l;
      } else {
        seg_of_tok[i] = -1;
        if (f == 1) ++n_g; else ++n_p;
      }
    }
    my_flag[e] = i < N ? f : (unsigned char)3;
    keys[i] = key;
  }
  int G, P, L;
  int g_at = block_exclusive_scan(n_g, scan_tmp, G);
  int p_at = block_exclusive_scan(n_p, scan_tmp, P);
  (void)block_exclusive_scan(n_l, scan_tmp, L);
  const int any_bad = __syncthreads_or(bad);
  if (view == 0) {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int i = tid * PER + e;
      if (my_flag[e] == 1) global_idx[g_at++] = i;
      if (my_flag[e] == 2) pad_idx[p_at++] = i;
    }
    for (int i = G + tid; i < N; i += kSegThreads) global_idx[i] = -1;
    for (int i = P + tid; i < N; i += kSegThreads) pad_idx[i] = -1;
    if (tid == 0) { counts[C_G] = G; counts[C_L] = L; counts[C_P] = P; counts[7] = 0; }
  }
  if (tid == 0) counts[5 + view] = any_bad;

  // ---- bitonic sort of keys[0..P2) ascending ------------------------------------------
  for (int k = 2; k <= P2; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      __syncthreads();
#pragma unroll
      for (int e = 0; e < (PER + 1) / 2; ++e) {
        const int t = tid + e * kSegThreads;  // pair index, P2/2 pairs
        if (PER == 1 && t >= P2 / 2) break;
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int p = i | j;
        const unsigned long long a = keys[i], c = keys[p];
        const bool asc = (i & k) == 0;
        if ((a > c) == asc) { keys[i] = c; keys[p] = a; }
      }
    }
  }
  __syncthreads();

  // ---- run boundaries -> segment index per slot ----------------------------------------
  unsigned long long mine[PER];
  int head[PER];
  int n_head = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int s = tid * PER + e;
    mine[e] = keys[s];
    head[e] = 0;
    if (s < L) {
      head[e] = (s == 0) || ((keys[s - 1] >> 32) != (mine[e] >> 32));
      n_head += head[e];
    }
  }
  int S;
  int seg_idx = block_exclusive_scan(n_head, scan_tmp, S) - 1;  // ends with a barrier
  // keys[] is dead now; reuse its bytes as two int arrays.
  int* seg_of_slot = reinterpret_cast<int*>(keys);       // [P2]
  int* seg_start = seg_of_slot + P2;                      // [P2], entry S (== L) is implied
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int s = tid * PER + e;
    if (s < L) {
      seg_idx += head[e];
      const int pos = (int)(unsigned)(mine[e] & 0xffffffffu);
      perm[s] = pos;
      seg_of_tok[pos] = seg_idx;
      seg_of_slot[s] = seg_idx;
      if (head[e]) { seg_start[seg_idx] = s; seg_off[seg_idx] = s; }
    } else if (s < N) {
      perm[s] = -1;
    }
  }
  if (tid == 0) { seg_off[S] = L; counts[C_SROW + view] = S; }
  for (int i = S + 1 + tid; i <= N; i += kSegThreads) seg_off[i] = -1;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int s = tid * PER + e;
    if (s < N) {
      int2 r = make_int2(0, 0);
      if (s < L) {
        const int g = seg_of_slot[s];
        r.x = seg_start[g];
        r.y = (g + 1 < S) ? seg_start[g + 1] : L;
      }
      slot_rng[s] = r;
    }
  }
}

hipError_t launch_build_segments(const int* row_ids, const int* col_ids,
                                 const unsigned char* flags, int B, int N, int* seg,
                                 hipStream_t stream) {
  dim3 grid(B, 2), block(kSegThreads);
  ProfileScope prof(1, stream);
#define MATE_SEG_CASE(P2)                                                                  \
  if (N <= P2) {                                                                            \
    hipLaunchKernelGGL(build_segments_kernel<P2>, grid, block, 0, stream, row_ids, col_ids, \
                       flags, B, N, seg);                                                   \
    return hipGetLastError();                                                               \
  }
  MATE_SEG_CASE(1024)
  MATE_SEG_CASE(4096)
  MATE_SEG_CASE(8192)
  MATE_SEG_CASE(16384)
#undef MATE_SEG_CASE
  return hipErrorInvalidValue;
}

}  // namespace mate
