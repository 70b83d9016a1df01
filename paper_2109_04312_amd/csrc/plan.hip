// Plan kernel: counts the units of every (sequence, head), decides which head kind's
// table-token units are the longer ones, lays the units out in eight work queues (one per XCD)
// and zeroes the queues' ticket counters.  One workgroup; integer work only.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "stream_plan.h"

namespace mate {
namespace {

__global__ __launch_bounds__(256) void plan_kernel(AttnArgs a) {
  __shared__ unsigned long long cost[2];
  __shared__ int band_total[8][4];
  __shared__ int first_view;
  const int tid = threadIdx.x, B = a.B, H = a.H, N = a.N, BH = B * H;
  const int UG = owner_slots(N), nq = plan_nq(BH);
  if (!tables_match(a)) {  // tables built for another shape: leave every queue empty
    if (tid < 16) a.plan[kPlanCounters + tid] = 0;
    if (tid < 64) a.plan[kPlanCum + tid] = 0;
    return;
  }
  if (tid < 2) cost[tid] = 0;
  if (tid < 16) a.plan[kPlanCounters + tid] = 0;
  __syncthreads();

  // streamed tiles of all table-token units, per view
  unsigned long long c0 = 0, c1 = 0;
  for (int idx = tid; idx < B * UG; idx += 256) {
    const int b = idx / UG, t0 = (idx % UG) * BM;
    const int L = a.seg.counts[(size_t)b * kCountWords + C_L];
    if (t0 >= L) continue;
    const int last = min(t0 + BM, L) - 1;
    const int2* r0 = a.seg.slot_rng[0] + (size_t)b * N;
    const int2* r1 = a.seg.slot_rng[1] + (size_t)b * N;
    c0 += (unsigned)(r0[last].y - r0[t0].x + BN - 1) / BN;
    c1 += (unsigned)(r1[last].y - r1[t0].x + BN - 1) / BN;
  }
  atomicAdd(&cost[0], c0);
  atomicAdd(&cost[1], c1);
  __syncthreads();
  if (tid == 0) {
    int n_col = 0;
    for (int h = 0; h < H; ++h) n_col += a.head_kind[h];
    const unsigned long long w0 = cost[0] * (unsigned)(H - n_col), w1 = cost[1] * (unsigned)n_col;
    // longer units first; with equal work (or no column heads) rows go first
    first_view = w1 > w0 ? 1 : 0;
    a.plan[kPlanFirstView] = first_view;
  }
  __syncthreads();

  if (tid < 32) {
    const int q = tid >> 2, band = tid & 3, fv = first_view;
    int* pref = a.plan + kPlanPref + (4 * q + band) * (nq + 1);
    int run = 0;
    for (int j = 0; j < nq; ++j) {
      pref[j] = run;
      const int bh = q + 8 * j;
      if (bh >= BH) continue;
      const int b = bh / H, h = bh % H;
      const int* cnt = a.seg.counts + (size_t)b * kCountWords;
      const int G = cnt[C_G], L = cnt[C_L], P = cnt[C_P];
      int n = 0;
      if (band < 2) {
        if ((a.head_kind[h] == fv) == (band == 0)) n = (L + BM - 1) / BM;
      } else if (band == 2) {
        const GlobalSplit s = global_split(G, L, N);
        n = s.n_gt * s.n_chunks;
      } else {
        n = (P + BM - 1) / BM;
      }
      run += n;
    }
    pref[nq] = run;
    band_total[q][band] = run;
  }
  __syncthreads();
  if (tid < 8) {
    int run = 0;
    for (int band = 0; band < 4; ++band) {
      run += band_total[tid][band];
      a.plan[kPlanCum + 8 * tid + band] = run;
    }
  }
}

}  // namespace

hipError_t launch_plan(const AttnArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, stream, a);
  return hipGetLastError();
}

int persistent_grid() {
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
