// Plan kernel: counts the units of every (sequence, head), decides which head kind's
// table-token units are the longer ones, lays the units out in eight work queues (one per XCD)
// and zeroes the queues' ticket counters.  One workgroup; integer work only.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "launch.h"
#include "stream_plan.h"

namespace mate {
namespace {

__global__ __launch_bounds__(256) void plan_kernel(AttnArgs a) {
  __shared__ unsigned long long cost[2];
  __shared__ int first_view;
  const int tid = threadIdx.x, B = a.B, H = a.H, N = a.N, BH = B * H;
  const int nq = plan_nq(BH);
  if (tid < 16) a.plan[kPlanCounters + tid] = 0;
  if (!tables_match(a)) {  // tables built for another shape: leave every queue empty
    if (tid < 8) a.plan[kPlanTotal + tid] = 0;
    return;
  }
  if (tid < 2) cost[tid] = 0;
  __syncthreads();
  // streamed tiles of all table-token units per view (counted by the segment builder)
  unsigned long long c0 = 0, c1 = 0;
  for (int b = tid; b < B; b += 256) {
    c0 += (unsigned)a.seg.counts[(size_t)b * kCountWords + C_COST_ROW];
    c1 += (unsigned)a.seg.counts[(size_t)b * kCountWords + C_COST_COL];
  }
  if (c0) atomicAdd(&cost[0], c0);
  if (c1) atomicAdd(&cost[1], c1);
  __syncthreads();
  if (tid == 0) {
    int n_col = 0;
    for (int h = 0; h < H; ++h) n_col += a.head_kind[h];
    const unsigned long long w0 = cost[0] * (unsigned)(H - n_col), w1 = cost[1] * (unsigned)n_col;
    first_view = w1 > w0 ? 1 : 0;  // the kind with more work goes first
    a.plan[kPlanFirstView] = first_view;
  }
  __syncthreads();

  if (tid < 8) {
    // queue tid: its pairs bh = tid + 8 j, those of the heavier head kind first
    const int q = tid, fv = first_view;
    int* pref = a.plan + kPlanPref + q * (nq + 1);
    int* list = a.plan + plan_list(BH) + q * nq;
    int n = 0, run = 0;
    for (int pass = 0; pass < 2; ++pass)
      for (int j = 0; j < nq; ++j) {
        const int bh = q + 8 * j;
        if (bh >= BH) break;
        if ((a.head_kind[bh % H] == fv) != (pass == 0)) continue;
        const int* cnt = a.seg.counts + (size_t)(bh / H) * kCountWords;
        const GlobalSplit s = global_split(cnt[C_G], cnt[C_L], N);
        list[n] = bh;
        pref[n++] = run;
        run += (cnt[C_L] + BM - 1) / BM + s.n_gt * s.n_chunks + (cnt[C_P] + BM - 1) / BM;
      }
    for (int j = n; j <= nq; ++j) pref[j] = run;
    for (int j = n; j < nq; ++j) list[j] = 0;
    a.plan[kPlanTotal + q] = run;
  }
}

}  // namespace

hipError_t launch_plan(const AttnArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, stream, a);
  return hipGetLastError();
}

int persistent_grid() {
#ifdef MATE_TRACE
  if (const char* e = std::getenv("MATE_GRID")) return std::atoi(e);
#endif
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 512;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    cached[dev] = 2 * cus;
  }
  return cached[dev];
}

}  // namespace mate
