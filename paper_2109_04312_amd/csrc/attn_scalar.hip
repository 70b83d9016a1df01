// Scalar (non-MFMA) MATE attention, fp32 arithmetic throughout: the path for dtype f32.
//
// One wavefront owns one query (forward, dQ) or one key (dK/dV) and walks the two key
// (query) lists the attention pattern of Section 3 gives it: the question tokens, and the
// sorted slots of its own row / column segment -- or every table token if it is itself a
// question token.  Lanes take 64 list entries at a time for the score dot products and the
// 64 head dimensions for the accumulations, so accumulation order is fixed and results are
// bit-reproducible.
#include <hip/hip_runtime.h>

#include "launch.h"

namespace mate {
namespace {

constexpr int D = 64;
constexpr int kWavesPerBlock = 4;

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(unsigned short x) { return __uint_as_float((unsigned)x << 16); }
__device__ inline void from_f32(float& d, float x) { d = x; }
__device__ inline void from_f32(unsigned short& d, float x) {
  unsigned u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
  d = (unsigned short)(u >> 16);
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// What one wavefront works on: token position `pos` and the two index lists to walk.
struct Item {
  int pos;          // token position, -1 = nothing to do
  bool pad;
  const int* list0; int n0;          // question tokens: global_idx[0..G)
  const int* list1; int lo1, hi1;    // sorted table tokens: perm[lo1..hi1)
};

// x in [0,N): first the G question tokens, then the L table tokens in the head's sorted
// order, then the pads.
__device__ inline Item make_item(const SegTables& t, int b, int N, int view, int x) {
  const int* c = t.counts + (size_t)b * kCountWords;
  const int G = c[C_G], L = c[C_L];
  Item it;
  it.pad = false;
  it.list0 = t.global_idx + (size_t)b * N;
  it.n0 = G;
  if (x < G) {
    it.pos = it.list0[x];
    it.list1 = t.perm[0] + (size_t)b * N;  // any view lists all table tokens; rows are contiguous
    it.lo1 = 0;
    it.hi1 = L;
  } else if (x < G + L) {
    const int s = x - G;
    it.list1 = t.perm[view] + (size_t)b * N;
    it.pos = it.list1[s];
    const int2 r = t.slot_rng[view][(size_t)b * N + s];
    it.lo1 = r.x;
    it.hi1 = r.y;
  } else {
    it.pos = t.pad_idx[(size_t)b * N + (x - G - L)];
    it.pad = true;
    it.list1 = it.list0;
    it.lo1 = it.hi1 = 0;
    it.n0 = 0;
  }
  return it;
}

// Tables built for another (B, N), or never built: every wavefront leaves before reading them.
__device__ inline bool tables_ok(const AttnArgs& a) {
  return a.seg.hdr[0] == kMagic && a.seg.hdr[1] == a.B && a.seg.hdr[2] == a.N;
}

template <typename T>
__device__ inline float dot_row(const float* __restrict__ a, const T* __restrict__ row) {
  float acc = 0.f;
#pragma unroll
  for (int d = 0; d < D; ++d) acc = fmaf(a[d], to_f32(row[d]), acc);
  return acc;
}

template <typename T>
__global__ __launch_bounds__(64 * kWavesPerBlock) void fwd_scalar_kernel(AttnArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, h = blockIdx.y, x = blockIdx.x * kWavesPerBlock + wave;
  if (x >= a.N || !tables_ok(a)) return;
  const Item it = make_item(a.seg, b, a.N, a.head_kind[h], x);
  const size_t bh = ((size_t)b * a.H + h) * a.N;
  const T* Q = static_cast<const T*>(a.q) + bh * D;
  const T* K = static_cast<const T*>(a.k) + bh * D;
  const T* V = static_cast<const T*>(a.v) + bh * D;
  T* O = static_cast<T*>(a.out) + bh * D;
  if (it.pad) {
    from_f32(O[(size_t)it.pos * D + lane], 0.f);
    if (lane == 0) a.lse[bh + it.pos] = 0.f;
    return;
  }
  float qv[D];
#pragma unroll
  for (int d = 0; d < D; ++d) qv[d] = to_f32(Q[(size_t)it.pos * D + d]);
  float m = -INFINITY, l = 0.f, o = 0.f;
  for (int part = 0; part < 2; ++part) {
    const int* list = part ? it.list1 : it.list0;
    const int lo = part ? it.lo1 : 0, hi = part ? it.hi1 : it.n0;
    for (int c0 = lo; c0 < hi; c0 += 64) {
      const bool valid = c0 + lane < hi;
      const int kp = valid ? list[c0 + lane] : 0;
      const float s = valid ? a.scale * dot_row(qv, K + (size_t)kp * D) : -INFINITY;
      const float m_new = fmaxf(m, wave_max(s));
      const float alpha = expf(m - m_new);
      const float p = valid ? expf(s - m_new) : 0.f;
      l = l * alpha + wave_sum(p);
      o *= alpha;
      const int n = min(64, hi - c0);
      for (int j = 0; j < n; ++j) {
        const float pj = __shfl(p, j, 64);
        const int kj = __shfl(kp, j, 64);
        o = fmaf(pj, to_f32(V[(size_t)kj * D + lane]), o);
      }
      m = m_new;
    }
  }
  from_f32(O[(size_t)it.pos * D + lane], o / l);
  if (lane == 0) a.lse[bh + it.pos] = m + logf(l);
}

// dQ for one query per wavefront; also stores delta_k = dO_k . O_k for the dK/dV kernel.
template <typename T>
__global__ __launch_bounds__(64 * kWavesPerBlock) void bwd_dq_scalar_kernel(AttnArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, h = blockIdx.y, x = blockIdx.x * kWavesPerBlock + wave;
  if (x >= a.N || !tables_ok(a)) return;
  const Item it = make_item(a.seg, b, a.N, a.head_kind[h], x);
  const size_t bh = ((size_t)b * a.H + h) * a.N;
  const T* Q = static_cast<const T*>(a.q) + bh * D;
  const T* K = static_cast<const T*>(a.k) + bh * D;
  const T* V = static_cast<const T*>(a.v) + bh * D;
  const T* O = static_cast<const T*>(a.o) + bh * D;
  const T* dO = static_cast<const T*>(a.dout) + bh * D;
  T* dQ = static_cast<T*>(a.dq) + bh * D;
  if (it.pad) {
    from_f32(dQ[(size_t)it.pos * D + lane], 0.f);
    if (lane == 0) a.delta[bh + it.pos] = 0.f;
    return;
  }
  float qv[D], gv[D];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    qv[d] = to_f32(Q[(size_t)it.pos * D + d]);
    gv[d] = to_f32(dO[(size_t)it.pos * D + d]);
  }
  const float delta =
      wave_sum(to_f32(dO[(size_t)it.pos * D + lane]) * to_f32(O[(size_t)it.pos * D + lane]));
  if (lane == 0) a.delta[bh + it.pos] = delta;
  const float lse = a.lse[bh + it.pos];
  float acc = 0.f;
  for (int part = 0; part < 2; ++part) {
    const int* list = part ? it.list1 : it.list0;
    const int lo = part ? it.lo1 : 0, hi = part ? it.hi1 : it.n0;
    for (int c0 = lo; c0 < hi; c0 += 64) {
      const bool valid = c0 + lane < hi;
      const int kp = valid ? list[c0 + lane] : 0;
      float ds = 0.f;
      if (valid) {
        const float p = expf(a.scale * dot_row(qv, K + (size_t)kp * D) - lse);
        ds = p * (dot_row(gv, V + (size_t)kp * D) - delta);
      }
      const int n = min(64, hi - c0);
      for (int j = 0; j < n; ++j) {
        const float dsj = __shfl(ds, j, 64);
        const int kj = __shfl(kp, j, 64);
        acc = fmaf(dsj, to_f32(K[(size_t)kj * D + lane]), acc);
      }
    }
  }
  from_f32(dQ[(size_t)it.pos * D + lane], a.scale * acc);
}

// dK and dV for one key per wavefront.  The queries that see a table key are the question
// tokens plus the table tokens of its own segment; a question key is seen by every non-pad
// token -- the same two lists as in the forward, read the other way round.
template <typename T>
__global__ __launch_bounds__(64 * kWavesPerBlock) void bwd_dkv_scalar_kernel(AttnArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, h = blockIdx.y, x = blockIdx.x * kWavesPerBlock + wave;
  if (x >= a.N || !tables_ok(a)) return;
  const Item it = make_item(a.seg, b, a.N, a.head_kind[h], x);
  const size_t bh = ((size_t)b * a.H + h) * a.N;
  const T* Q = static_cast<const T*>(a.q) + bh * D;
  const T* K = static_cast<const T*>(a.k) + bh * D;
  const T* V = static_cast<const T*>(a.v) + bh * D;
  const T* dO = static_cast<const T*>(a.dout) + bh * D;
  T* dK = static_cast<T*>(a.dk) + bh * D;
  T* dV = static_cast<T*>(a.dv) + bh * D;
  if (it.pad) {
    from_f32(dK[(size_t)it.pos * D + lane], 0.f);
    from_f32(dV[(size_t)it.pos * D + lane], 0.f);
    return;
  }
  float kv[D], vv[D];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    kv[d] = to_f32(K[(size_t)it.pos * D + d]);
    vv[d] = to_f32(V[(size_t)it.pos * D + d]);
  }
  float acc_k = 0.f, acc_v = 0.f;
  for (int part = 0; part < 2; ++part) {
    const int* list = part ? it.list1 : it.list0;
    const int lo = part ? it.lo1 : 0, hi = part ? it.hi1 : it.n0;
    for (int c0 = lo; c0 < hi; c0 += 64) {
      const bool valid = c0 + lane < hi;
      const int qp = valid ? list[c0 + lane] : 0;
      float p = 0.f, ds = 0.f;
      if (valid) {
        p = expf(a.scale * dot_row(kv, Q + (size_t)qp * D) - a.lse[bh + qp]);
        ds = p * (dot_row(vv, dO + (size_t)qp * D) - a.delta[bh + qp]);
      }
      const int n = min(64, hi - c0);
      for (int j = 0; j < n; ++j) {
        const float pj = __shfl(p, j, 64);
        const float dsj = __shfl(ds, j, 64);
        const int qj = __shfl(qp, j, 64);
        acc_v = fmaf(pj, to_f32(dO[(size_t)qj * D + lane]), acc_v);
        acc_k = fmaf(dsj, to_f32(Q[(size_t)qj * D + lane]), acc_k);
      }
    }
  }
  from_f32(dK[(size_t)it.pos * D + lane], a.scale * acc_k);
  from_f32(dV[(size_t)it.pos * D + lane], acc_v);
}

inline dim3 scalar_grid(const AttnArgs& a) {
  return dim3((a.N + kWavesPerBlock - 1) / kWavesPerBlock, a.H, a.B);
}

}  // namespace

hipError_t launch_fwd_scalar(const AttnArgs& a, bool bf16, hipStream_t stream) {
  const dim3 block(64 * kWavesPerBlock);
  if (bf16)
    hipLaunchKernelGGL(fwd_scalar_kernel<unsigned short>, scalar_grid(a), block, 0, stream, a);
  else
    hipLaunchKernelGGL(fwd_scalar_kernel<float>, scalar_grid(a), block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_bwd_scalar(const AttnArgs& a, bool bf16, hipStream_t stream) {
  const dim3 block(64 * kWavesPerBlock);
  if (bf16) {
    hipLaunchKernelGGL(bwd_dq_scalar_kernel<unsigned short>, scalar_grid(a), block, 0, stream, a);
    hipLaunchKernelGGL(bwd_dkv_scalar_kernel<unsigned short>, scalar_grid(a), block, 0, stream, a);
  } else {
    hipLaunchKernelGGL(bwd_dq_scalar_kernel<float>, scalar_grid(a), block, 0, stream, a);
    hipLaunchKernelGGL(bwd_dkv_scalar_kernel<float>, scalar_grid(a), block, 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace mate
