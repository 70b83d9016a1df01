// Positional index that restarts at the beginning of each cell (Section 3.2: for sequences
// longer than 512 tokens the index of the positional embedding is reset per cell, so that no
// embeddings for large indices have to be learnt).  Integer work only.
//
// A cell is a maximal run of consecutive table tokens with the same (row, column).  A table
// token's index is its distance from the first token of its cell: position minus the largest
// "cell start" position at or before it, i.e. an inclusive running maximum over the sequence.
// Question tokens keep their absolute position, pads get 0.
//
// One 1024-thread workgroup per sequence.  A wavefront owns a contiguous block and walks it in
// batches of 64 with lane = consecutive element, so loads and stores are unit-stride; the
// running maximum is a shuffle scan inside a batch, a scalar carry between the batches of a
// wavefront, and one LDS exchange between wavefronts.
#include <hip/hip_runtime.h>

#include "launch.h"

namespace mate {

constexpr int kPosThreads = 1024;
constexpr int kPosWaves = kPosThreads / 64;
constexpr int kPosMaxBatches = 16;  // 16384 positions / 1024 threads

__global__ __launch_bounds__(kPosThreads) void cell_positions_kernel(
    const int* __restrict__ row_ids, const int* __restrict__ col_ids,
    const unsigned char* __restrict__ flags, int N, int* __restrict__ out) {
  __shared__ int wave_last[kPosWaves];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int* row = row_ids + (size_t)b * N;
  const int* col = col_ids + (size_t)b * N;
  const unsigned char* fl = flags + (size_t)b * N;
  int* dst = out + (size_t)b * N;

  const int nb = (N + kPosThreads - 1) / kPosThreads;  // batches per wavefront (uniform)
  const int w0 = wave * nb * 64;
  int start[kPosMaxBatches];        // latest cell start at or before my element, inside my wavefront's block
  unsigned char kind[kPosMaxBatches];
  // All inputs of the wavefront's block first, so that the loads travel together.  The previous
  // position's values are loaded rather than shuffled: the first lane's neighbour belongs to
  // another batch or wavefront.
  bool head[kPosMaxBatches];
#pragma unroll
  for (int e = 0; e < kPosMaxBatches; ++e) {
    if (e >= nb) continue;  // uniform; the loops are fully unrolled so that the arrays stay in registers
    const int i = w0 + e * 64 + lane;
    const int ic = min(i, N - 1), ip = max(ic - 1, 0);
    const unsigned char f = fl[ic], fp = fl[ip];
    const int r = row[ic], rp = row[ip], c = col[ic], cp = col[ip];
    kind[e] = i < N ? f : (unsigned char)2;
    head[e] = i < N && f == 0 && (i == 0 || fp != 0 || rp != r || cp != c);
  }
  int carry = -1;
#pragma unroll
  for (int e = 0; e < kPosMaxBatches; ++e) {
    if (e >= nb) continue;
    const int i = w0 + e * 64 + lane;
    int s = head[e] ? i : -1;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(s, d, 64);
      if (lane >= d) s = max(s, up);
    }
    s = max(s, carry);
    carry = __shfl(s, 63, 64);
    start[e] = s;
  }
  if (lane == 0) wave_last[wave] = carry;
  __syncthreads();
  int before = -1;  // latest cell start in the blocks of the wavefronts before mine
  for (int w = 0; w < wave; ++w) before = max(before, wave_last[w]);
#pragma unroll
  for (int e = 0; e < kPosMaxBatches; ++e) {
    if (e >= nb) continue;
    const int i = w0 + e * 64 + lane;
    if (i < N) {
      // a table token always has a cell start at or before it (position 0 at the latest)
      const int s = max(start[e], before);
      dst[i] = kind[e] == 0 ? i - s : kind[e] == 1 ? i : 0;
    }
  }
}

hipError_t launch_cell_positions(const int* row_ids, const int* col_ids, const unsigned char* flags,
                                 int B, int N, int* out, hipStream_t stream) {
  if (N > kPosThreads * kPosMaxBatches) return hipErrorInvalidValue;
  hipLaunchKernelGGL(cell_positions_kernel, dim3(B), dim3(kPosThreads), 0, stream, row_ids, col_ids,
                     flags, N, out);
  return hipGetLastError();
}

}  // namespace mate
