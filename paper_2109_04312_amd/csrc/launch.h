// Host-side launchers, one per kernel family.  Everything is enqueued on `stream`.
#pragma once
#include <hip/hip_runtime.h>

#include "seg_layout.h"

namespace mate {

struct AttnArgs {
  const void *q, *k, *v;    // [B,H,N,64]
  const void *o, *dout;     // backward only
  void *out;                // forward only
  float* lse;               // forward: written; backward: read (const in spirit)
  void *dq, *dk, *dv;       // backward only
  float* delta;             // backward scratch [B,H,N]: rowsum(dO * O), negated in the bf16 path
  float* nlse;              // backward scratch [B,H,N] of the bf16 path: -lse / scale
  float* part[3];           // partial results of chunked question-token owners, per (b,h):
                            //   forward: [0] unnormalised O;  backward: dQ, dK, dV
  float* part_ml;           // forward: running max (log2 domain) and sum per partial row
  SegTables seg;
  unsigned char head_kind[256];
  alignas(4) unsigned char head_order[256];  // heads sorted column heads first (stable);
                                             // read as 32-bit words by the kernels
  int n_col;                      // number of column heads
  int B, H, N;
  float scale;
};

// Arguments of the dense-mask variant (no segment tables: ids and flags directly).
constexpr int kDenseMaxN = 1024;
struct DenseArgs {
  const void *q, *k, *v, *o, *dout;
  void* out;
  float* lse;
  void *dq, *dk, *dv;
  float *delta, *nlse;      // backward scratch [B,H,N]: -rowsum(dO * O), -lse / scale
  const int *row_ids, *col_ids;
  const unsigned char* flags;
  unsigned char head_kind[256];
  int B, H, N;
  float scale;
};

// Measurement hook: when `kernel` matches the kernel about to be launched, record `start`
// before and `stop` after that one launch on its stream, then disarm.
struct ProfileHook {
  int kernel;
  hipEvent_t start, stop;
};
extern thread_local ProfileHook g_profile_hook;
struct ProfileScope {
  hipStream_t stream;
  bool armed;
  ProfileScope(int kernel, hipStream_t s) : stream(s), armed(g_profile_hook.kernel == kernel) {
    if (armed) (void)hipEventRecord(g_profile_hook.start, stream);
  }
  ~ProfileScope() {
    if (armed) {
      (void)hipEventRecord(g_profile_hook.stop, stream);
      g_profile_hook.kernel = 0;
    }
  }
};

// max_global >= N and radius = 0: the pattern of Section 3; otherwise the bucketed approximation
// of Section 3.1 (global part of at most max_global tokens, windows of three buckets of radius).
hipError_t launch_build_segments(const int* row_ids, const int* col_ids,
                                 const unsigned char* flags, int B, int N, int max_global,
                                 int radius, int* seg, hipStream_t stream);

// Positional index restarting at each cell (Section 3.2); out is [B, N] int32.
hipError_t launch_cell_positions(const int* row_ids, const int* col_ids, const unsigned char* flags,
                                 int B, int N, int* out, hipStream_t stream);

// Projections either side of the attention (bf16): x [B,N,E] -> q, k, v [B,H,N,64] with
// w_qkv [3*H*64, E]; o [B,H,N,64] -> y [B,N,E] with w_o [E, H*64].  bias may be null.
// H even, E a multiple of 128.
hipError_t launch_qkv_project(const void* x, const void* w_qkv, const float* bias,
                              const unsigned char* flags, int B, int N, int H, int E, void* q,
                              void* k, void* v, hipStream_t stream);
hipError_t launch_out_project(const void* o, const void* w_o, const float* bias,
                              const unsigned char* flags, int B, int N, int H, int E, void* y,
                              hipStream_t stream);

// Backward of the two projections.  dx / d_o, dw, dbias may each be null (not wanted); dw and
// dbias are float32.  `workspace` holds *_project_bwd_workspace(...) bytes.
size_t qkv_project_bwd_workspace(int B, int N, int H, int E);
size_t out_project_bwd_workspace(int B, int N, int H, int E);
hipError_t launch_qkv_project_bwd(const void* x, const void* w_qkv, const unsigned char* flags,
                                  const void* dq, const void* dk, const void* dv, int B, int N, int H,
                                  int E, void* dx, float* dw, float* dbias, void* workspace,
                                  hipStream_t stream);
hipError_t launch_out_project_bwd(const void* o, const void* w_o, const unsigned char* flags,
                                  const void* dy, int B, int N, int H, int E, void* d_o, float* dw,
                                  float* dbias, void* workspace, hipStream_t stream);

// Measurement aid: `workgroups` x 4 wavefronts each issue `iters` x 8 independent 32x32x16 bf16
// MFMAs and write one float per thread to `sink` (workgroups * 256 floats).
hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, hipStream_t stream);
double mfma_probe_flop(int workgroups, int iters);

// Scalar (non-MFMA) kernels: fp32 arithmetic throughout, one wavefront per query / key.
// They serve dtype f32 and are the fallback-free reference-quality path for it.
hipError_t launch_fwd_scalar(const AttnArgs& a, bool bf16, hipStream_t stream);
hipError_t launch_bwd_scalar(const AttnArgs& a, bool bf16, hipStream_t stream);

// bf16 MFMA kernels.
hipError_t launch_fwd_mfma(const AttnArgs& a, hipStream_t stream);
hipError_t launch_bwd_mfma(const AttnArgs& a, hipStream_t stream);
hipError_t launch_fwd_dense(const DenseArgs& a, hipStream_t stream);
hipError_t launch_bwd_dense(const DenseArgs& a, hipStream_t stream);

}  // namespace mate
