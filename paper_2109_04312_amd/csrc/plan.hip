// Plan kernel: counts the units of every (sequence, head), decides which head kind's
// table-token units are the longer ones, lays the units out in eight work queues (one per XCD)
// and zeroes the queues' ticket counters.  One workgroup; integer work only.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "launch.h"
#include "stream_plan.h"

namespace mate {
namespace {

__global__ __launch_bounds__(64) void plan_kernel(AttnArgs a) {
  const int tid = threadIdx.x, B = a.B, H = a.H, N = a.N, BH = B * H;
  const int nq = plan_nq(BH);
  if (tid < 16) a.plan[kPlanCounters + tid] = 0;
  if (!tables_match(a)) {  // tables built for another shape: leave every queue empty
    if (tid < 8) a.plan[kPlanTotal + tid] = 0;
    return;
  }
  if (tid < 8) {
    const int q = tid;
    int* pref_pad = a.plan + kPlanPref + 2 * q * (nq + 1);
    int* pref_glob = pref_pad + nq + 1;
    int pairs = 0, most = 0, pads = 0, globs = 0;
    for (int j = 0; j < nq; ++j) {
      pref_pad[j] = pads;
      pref_glob[j] = globs;
      const int bh = q + 8 * j;
      if (bh >= BH) continue;
      const int* cnt = a.seg.counts + (size_t)(bh / H) * kCountWords;
      const GlobalSplit s = global_split(cnt[C_G], cnt[C_L], N);
      ++pairs;
      most = max(most, (cnt[C_L] + BM - 1) / BM);
      pads += (cnt[C_P] + BM - 1) / BM;
      globs += s.n_gt * s.n_chunks;
    }
    pref_pad[nq] = pads;
    pref_glob[nq] = globs;
    a.plan[kPlanPairs + q] = max(pairs, 1);
    a.plan[kPlanMost + q] = most;
    a.plan[kPlanTotal + q] = pairs * most + pads + globs;
  }
}

}  // namespace

hipError_t launch_plan(const AttnArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace mate
