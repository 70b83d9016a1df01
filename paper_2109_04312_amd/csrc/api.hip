// C ABI entry points: argument validation on the host, then kernel launches on the caller's
// stream.  No allocation, no global state.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>

#include "../../include/mate.h"
#include "launch.h"
#include "seg_layout.h"
#include "stream_plan.h"

using namespace mate;

// Scratch of mate_attn_bwd_dense_static: one copy per GPU, held until the process ends.  In host
// code this name is only a stand-in; the device address comes from hipGetSymbolAddress (below),
// once per device, and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[MATE_STATIC_SCRATCH_BYTES];

namespace mate {
// Measurement hook (see mate_profile_kernel): events to record around the next launch of one
// kernel.  Thread-local, cleared when used.
thread_local ProfileHook g_profile_hook = {0, nullptr, nullptr};
}  // namespace mate

namespace {

bool shape_ok(int B, int N) { return B >= 1 && N >= 1 && N <= MATE_MAX_N; }

size_t align16(size_t n) { return (n + 15) & ~size_t(15); }
size_t delta_bytes(int B, int H, int N) { return align16((size_t)B * H * N * sizeof(float)); }
// partial results of chunked question-token owners (bf16 MFMA path only)
size_t part_bytes(int B, int H, int N) { return (size_t)B * H * part_words_per_bh(N) * sizeof(float); }
size_t stat_bytes(int B, int H, int N) { return (size_t)B * H * stat_words_per_bh(N) * sizeof(float); }

mate_status fill_args(AttnArgs& a, const void* segments, const uint8_t* head_kind, int B, int H,
                      int N, int D, mate_dtype t, float scale) {
  if (!segments || !head_kind) return MATE_ERR_NULL;
  if (!shape_ok(B, N) || H < 1 || H > MATE_MAX_HEADS) return MATE_ERR_SHAPE;
  if (D != MATE_HEAD_DIM || (t != MATE_F32 && t != MATE_BF16)) return MATE_ERR_UNSUPPORTED;
  if (!(scale > 0.f) || !(scale < 3.0e38f)) return MATE_ERR_UNSUPPORTED;
  std::memset(&a, 0, sizeof(a));
  int n_sorted = 0;
  for (int h = 0; h < H; ++h) {
    if (head_kind[h] > MATE_HEAD_COL) return MATE_ERR_UNSUPPORTED;
    a.head_kind[h] = head_kind[h];
  }
  for (int kind = MATE_HEAD_COL; kind >= MATE_HEAD_ROW; --kind)
    for (int h = 0; h < H; ++h)
      if (head_kind[h] == kind) a.head_order[n_sorted++] = (unsigned char)h;
  a.n_col = 0;
  for (int h = 0; h < H; ++h) a.n_col += head_kind[h] == MATE_HEAD_COL;
  a.seg = make_tables(segments, B, N);
  a.B = B;
  a.H = H;
  a.N = N;
  a.scale = scale;
  return MATE_OK;
}

}  // namespace

extern "C" {

size_t mate_segments_bytes(int B, int N) {
  if (!shape_ok(B, N)) return 0;
  return SegLayout(B, N).total * sizeof(int);
}

size_t mate_workspace_bytes(int B, int H, int N, int D, mate_dtype t, int for_bwd) {
  if (!shape_ok(B, N) || H < 1 || H > MATE_MAX_HEADS || D != MATE_HEAD_DIM) return 0;
  if (t == MATE_F32) return for_bwd ? delta_bytes(B, H, N) : 0;
  if (t != MATE_BF16) return 0;
  return for_bwd ? 2 * delta_bytes(B, H, N) + 3 * part_bytes(B, H, N)
                 : part_bytes(B, H, N) + stat_bytes(B, H, N);
}

mate_status mate_build_segments(const int32_t* row_ids, const int32_t* col_ids,
                                const uint8_t* flags, int B, int N, void* segments,
                                void* stream) {
  if (!row_ids || !col_ids || !flags || !segments) return MATE_ERR_NULL;
  if (!shape_ok(B, N)) return MATE_ERR_SHAPE;
  hipError_t e = launch_build_segments(row_ids, col_ids, flags, B, N, N, 0,
                                       static_cast<int*>(segments),
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_build_segments_bucketed(const int32_t* row_ids, const int32_t* col_ids,
                                         const uint8_t* flags, int B, int N, int global_length,
                                         int radius, void* segments, void* stream) {
  if (!row_ids || !col_ids || !flags || !segments) return MATE_ERR_NULL;
  if (!shape_ok(B, N)) return MATE_ERR_SHAPE;
  if (global_length < 0 || radius < 1) return MATE_ERR_UNSUPPORTED;
  // a sequence has at most N question tokens and N slots: larger values change nothing
  hipError_t e = launch_build_segments(row_ids, col_ids, flags, B, N, std::min(global_length, N),
                                       std::min(radius, N), static_cast<int*>(segments),
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_segments_export_windows(const void* segments, int B, int N, int view,
                                         int32_t* window, void* stream) {
  if (!segments || !window) return MATE_ERR_NULL;
  if (!shape_ok(B, N) || view < 0 || view > 1) return MATE_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const SegLayout lay(B, N);
  const int* w = static_cast<const int*>(segments);
  int head[kHdrWords];
  if (hipMemcpyAsync(head, w, sizeof(head), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipMemcpyAsync(window, w + lay.view0 + (size_t)view * lay.view_stride + lay.slot_rng,
                     (size_t)B * N * 2 * sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return MATE_ERR_HIP;
  return head[0] == kMagic && head[1] == B && head[2] == N ? MATE_OK : MATE_ERR_SHAPE;
}

mate_status mate_cell_positions(const int32_t* row_ids, const int32_t* col_ids,
                                const uint8_t* flags, int B, int N, int32_t* positions,
                                void* stream) {
  if (!row_ids || !col_ids || !flags || !positions) return MATE_ERR_NULL;
  if (!shape_ok(B, N)) return MATE_ERR_SHAPE;
  hipError_t e = launch_cell_positions(row_ids, col_ids, flags, B, N, positions,
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_segments_export(const void* segments, int B, int N, int view, int32_t* perm,
                                 int32_t* seg_off, int32_t* seg_of_tok, int32_t* global_idx,
                                 int32_t* counts, void* stream) {
  if (!segments) return MATE_ERR_NULL;
  if (!shape_ok(B, N) || view < 0 || view > 1) return MATE_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const SegLayout lay(B, N);
  const int* w = static_cast<const int*>(segments);
  const int* vb = w + lay.view0 + (size_t)view * lay.view_stride;
  int head[kHdrWords];
#define MATE_D2H(dst, src, words)                                                             \
  if (hipMemcpyAsync(dst, src, (size_t)(words) * sizeof(int), hipMemcpyDeviceToHost, s) !=    \
      hipSuccess)                                                                             \
    return MATE_ERR_HIP;
  MATE_D2H(head, w, kHdrWords);
  if (perm) MATE_D2H(perm, vb + lay.perm, (size_t)B * N);
  if (seg_off) MATE_D2H(seg_off, vb + lay.seg_off, (size_t)B * (N + 1));
  if (seg_of_tok) MATE_D2H(seg_of_tok, vb + lay.seg_of_tok, (size_t)B * N);
  if (global_idx) MATE_D2H(global_idx, w + lay.global_idx, (size_t)B * N);
  if (hipStreamSynchronize(s) != hipSuccess) return MATE_ERR_HIP;
  if (head[0] != kMagic || head[1] != B || head[2] != N) return MATE_ERR_SHAPE;
  // per-sequence counts, a few sequences per copy through a fixed buffer (no allocation)
  constexpr int kBatch = 64;
  int cnt[kBatch * kCountWords];
  int bad = 0;
  for (int b0 = 0; b0 < B; b0 += kBatch) {
    const int nb = std::min(kBatch, B - b0);
    MATE_D2H(cnt, w + lay.counts + (size_t)b0 * kCountWords, (size_t)nb * kCountWords);
    if (hipStreamSynchronize(s) != hipSuccess) return MATE_ERR_HIP;
    for (int b = b0; b < b0 + nb; ++b) {
      const int* c = cnt + (size_t)(b - b0) * kCountWords;
      // the builder writes the valid part of each list only: the rest is -1 by this function's contract
      if (perm) std::fill(perm + (size_t)b * N + c[C_L], perm + (size_t)(b + 1) * N, -1);
      if (global_idx) std::fill(global_idx + (size_t)b * N + c[C_G], global_idx + (size_t)(b + 1) * N, -1);
      if (seg_off)
        std::fill(seg_off + (size_t)b * (N + 1) + c[C_SROW + view] + 1, seg_off + (size_t)(b + 1) * (N + 1), -1);
      if (counts) {
        counts[3 * b + 0] = c[C_G];
        counts[3 * b + 1] = c[C_L];
        counts[3 * b + 2] = c[C_SROW + view];
      }
      bad |= c[5] | c[6];  // per-view "bad id or flag seen" words
    }
  }
#undef MATE_D2H
  return bad ? MATE_ERR_BAD_ID : MATE_OK;
}

mate_status mate_segments_status(const void* segments, int B, int N, void* stream) {
  if (!segments) return MATE_ERR_NULL;
  if (!shape_ok(B, N)) return MATE_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int* w = static_cast<const int*>(segments);
  int head[kHdrWords];
  if (hipMemcpyAsync(head, w, sizeof(head), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return MATE_ERR_HIP;
  if (head[0] != kMagic || head[1] != B || head[2] != N) return MATE_ERR_SHAPE;
  // the per-sequence words, a few sequences per copy through a fixed buffer (no allocation)
  constexpr int kBatch = 64;
  int cnt[kBatch * kCountWords];
  int bad = 0;
  for (int b0 = 0; b0 < B; b0 += kBatch) {
    const int n = std::min(kBatch, B - b0);
    if (hipMemcpyAsync(cnt, w + SegLayout(B, N).counts + (size_t)b0 * kCountWords,
                       (size_t)n * kCountWords * sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
      return MATE_ERR_HIP;
    for (int b = 0; b < n; ++b) bad |= cnt[b * kCountWords + 5] | cnt[b * kCountWords + 6];
  }
  return bad ? MATE_ERR_BAD_ID : MATE_OK;
}

int mate_attn_prefers_dense(int B, int H, int N, mate_dtype t) {
  (void)B;
  (void)H;
  // Measured on MI355X with tables shaped like the short benchmark configuration (B = 32,
  // H = 12): build + forward + backward of the segment path against forward + backward of the
  // dense-mask variant.  Dense wins up to N = 256 and loses from N = 384 on; the batch and head
  // counts scale both sides alike, so they do not enter.
  return t == MATE_BF16 && N >= 1 && N <= MATE_DENSE_PREFERRED_MAX_N;
}

namespace {
mate_status proj_args_ok(int B, int N, int H, int E, mate_dtype t) {
  if (!shape_ok(B, N) || H < 1 || H > MATE_MAX_HEADS || E < 1) return MATE_ERR_SHAPE;
  if (t != MATE_BF16 || (H & 1) || E % 128 != 0 || E > 65536) return MATE_ERR_UNSUPPORTED;
  return MATE_OK;
}
}  // namespace

mate_status mate_qkv_project(const void* x, const void* w_qkv, const float* bias,
                             const uint8_t* flags, int B, int N, int H, int E, mate_dtype t,
                             void* q, void* k, void* v, void* stream) {
  if (!x || !w_qkv || !flags || !q || !k || !v) return MATE_ERR_NULL;
  const mate_status st = proj_args_ok(B, N, H, E, t);
  if (st != MATE_OK) return st;
  hipError_t e = launch_qkv_project(x, w_qkv, bias, flags, B, N, H, E, q, k, v,
                                    static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_out_project(const void* o, const void* w_o, const float* bias,
                             const uint8_t* flags, int B, int N, int H, int E, mate_dtype t,
                             void* y, void* stream) {
  if (!o || !w_o || !flags || !y) return MATE_ERR_NULL;
  const mate_status st = proj_args_ok(B, N, H, E, t);
  if (st != MATE_OK) return st;
  hipError_t e = launch_out_project(o, w_o, bias, flags, B, N, H, E, y,
                                    static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

size_t mate_project_bwd_workspace_bytes(int B, int N, int H, int E) {
  if (proj_args_ok(B, N, H, E, MATE_BF16) != MATE_OK) return 0;
  return std::max(qkv_project_bwd_workspace(B, N, H, E), out_project_bwd_workspace(B, N, H, E));
}

mate_status mate_qkv_project_bwd(const void* x, const void* w_qkv, const uint8_t* flags,
                                 const void* dq, const void* dk, const void* dv, int B, int N,
                                 int H, int E, mate_dtype t, void* dx, float* dw_qkv, float* dbias,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || !w_qkv || !flags || !dq || !dk || !dv) return MATE_ERR_NULL;
  const mate_status st = proj_args_ok(B, N, H, E, t);
  if (st != MATE_OK) return st;
  if (dbias && !dw_qkv) return MATE_ERR_NULL;  // the bias gradient rides on the weight gradient
  if (!workspace || workspace_bytes < qkv_project_bwd_workspace(B, N, H, E)) return MATE_ERR_WORKSPACE;
  hipError_t e = launch_qkv_project_bwd(x, w_qkv, flags, dq, dk, dv, B, N, H, E, dx, dw_qkv, dbias,
                                        workspace, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_out_project_bwd(const void* o, const void* w_o, const uint8_t* flags,
                                 const void* dy, int B, int N, int H, int E, mate_dtype t,
                                 void* d_o, float* dw_o, float* dbias, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (!o || !w_o || !flags || !dy) return MATE_ERR_NULL;
  const mate_status st = proj_args_ok(B, N, H, E, t);
  if (st != MATE_OK) return st;
  if (dbias && !dw_o) return MATE_ERR_NULL;
  if (!workspace || workspace_bytes < out_project_bwd_workspace(B, N, H, E)) return MATE_ERR_WORKSPACE;
  hipError_t e = launch_out_project_bwd(o, w_o, flags, dy, B, N, H, E, d_o, dw_o, dbias, workspace,
                                        static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_attn_fwd(const void* q, const void* k, const void* v, const void* segments,
                          const uint8_t* head_kind, int B, int H, int N, int D, mate_dtype t,
                          float scale, void* out, float* lse, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!q || !k || !v || !out || !lse) return MATE_ERR_NULL;
  AttnArgs a;
  mate_status st = fill_args(a, segments, head_kind, B, H, N, D, t, scale);
  if (st != MATE_OK) return st;
  const size_t need = mate_workspace_bytes(B, H, N, D, t, 0);
  if (need && (!workspace || workspace_bytes < need)) return MATE_ERR_WORKSPACE;
  a.q = q; a.k = k; a.v = v; a.out = out; a.lse = lse;
  if (t == MATE_BF16) {
    char* p = static_cast<char*>(workspace);
    a.part[0] = reinterpret_cast<float*>(p);
    a.part_ml = reinterpret_cast<float*>(p + part_bytes(B, H, N));
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = (t == MATE_BF16) ? launch_fwd_mfma(a, s) : launch_fwd_scalar(a, false, s);
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                          const float* lse, const void* dout, const void* segments,
                          const uint8_t* head_kind, int B, int H, int N, int D, mate_dtype t,
                          float scale, void* dq, void* dk, void* dv, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return MATE_ERR_NULL;
  AttnArgs a;
  mate_status st = fill_args(a, segments, head_kind, B, H, N, D, t, scale);
  if (st != MATE_OK) return st;
  const size_t need = mate_workspace_bytes(B, H, N, D, t, 1);
  if (need && (!workspace || workspace_bytes < need)) return MATE_ERR_WORKSPACE;
  a.q = q; a.k = k; a.v = v; a.o = out; a.dout = dout;
  a.lse = const_cast<float*>(lse);
  a.dq = dq; a.dk = dk; a.dv = dv;
  a.delta = static_cast<float*>(workspace);
  if (t == MATE_BF16) {
    a.nlse = reinterpret_cast<float*>(static_cast<char*>(workspace) + delta_bytes(B, H, N));
    char* p = static_cast<char*>(workspace) + 2 * delta_bytes(B, H, N);
    for (int i = 0; i < 3; ++i) a.part[i] = reinterpret_cast<float*>(p + i * part_bytes(B, H, N));
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = (t == MATE_BF16) ? launch_bwd_mfma(a, s) : launch_bwd_scalar(a, false, s);
  return e == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

namespace {
mate_status fill_dense(DenseArgs& a, const int32_t* row_ids, const int32_t* col_ids,
                       const uint8_t* flags, const uint8_t* head_kind, int B, int H, int N, int D,
                       mate_dtype t, float scale) {
  if (!row_ids || !col_ids || !flags || !head_kind) return MATE_ERR_NULL;
  if (!shape_ok(B, N) || H < 1 || H > MATE_MAX_HEADS) return MATE_ERR_SHAPE;
  if (D != MATE_HEAD_DIM || t != MATE_BF16 || N > MATE_DENSE_MAX_N) return MATE_ERR_UNSUPPORTED;
  if (!(scale > 0.f) || !(scale < 3.0e38f)) return MATE_ERR_UNSUPPORTED;
  static_assert(MATE_DENSE_MAX_N == kDenseMaxN, "header and kernels disagree");
  std::memset(&a, 0, sizeof(a));
  for (int h = 0; h < H; ++h) {
    if (head_kind[h] > MATE_HEAD_COL) return MATE_ERR_UNSUPPORTED;
    a.head_kind[h] = head_kind[h];
  }
  a.row_ids = row_ids; a.col_ids = col_ids; a.flags = flags;
  a.B = B; a.H = H; a.N = N; a.scale = scale;
  return MATE_OK;
}
}  // namespace

size_t mate_dense_workspace_bytes(int B, int H, int N) {
  if (!shape_ok(B, N) || N > MATE_DENSE_MAX_N || H < 1 || H > MATE_MAX_HEADS) return 0;
  return 2 * delta_bytes(B, H, N);
}

mate_status mate_attn_fwd_dense(const void* q, const void* k, const void* v,
                                const int32_t* row_ids, const int32_t* col_ids,
                                const uint8_t* flags, const uint8_t* head_kind, int B, int H,
                                int N, int D, mate_dtype t, float scale, void* out, float* lse,
                                void* stream) {
  if (!q || !k || !v || !out || !lse) return MATE_ERR_NULL;
  DenseArgs a;
  mate_status st = fill_dense(a, row_ids, col_ids, flags, head_kind, B, H, N, D, t, scale);
  if (st != MATE_OK) return st;
  a.q = q; a.k = k; a.v = v; a.out = out; a.lse = lse;
  return launch_fwd_dense(a, static_cast<hipStream_t>(stream)) == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_attn_bwd_dense(const void* q, const void* k, const void* v, const void* out,
                                const float* lse, const void* dout, const int32_t* row_ids,
                                const int32_t* col_ids, const uint8_t* flags,
                                const uint8_t* head_kind, int B, int H, int N, int D,
                                mate_dtype t, float scale, void* dq, void* dk, void* dv,
                                void* workspace, size_t workspace_bytes, void* stream) {
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return MATE_ERR_NULL;
  DenseArgs a;
  mate_status st = fill_dense(a, row_ids, col_ids, flags, head_kind, B, H, N, D, t, scale);
  if (st != MATE_OK) return st;
  const size_t need = mate_dense_workspace_bytes(B, H, N);
  if (!workspace || workspace_bytes < need) return MATE_ERR_WORKSPACE;
  a.q = q; a.k = k; a.v = v; a.o = out; a.dout = dout;
  a.lse = const_cast<float*>(lse);
  a.dq = dq; a.dk = dk; a.dv = dv;
  a.delta = static_cast<float*>(workspace);
  a.nlse = reinterpret_cast<float*>(static_cast<char*>(workspace) + delta_bytes(B, H, N));
  return launch_bwd_dense(a, static_cast<hipStream_t>(stream)) == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, or null

// Address of the current device's copy of `scratch`; looked up on the first call on that device.
mate_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MATE_ERR_HIP;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MATE_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // racing threads store the same value
  }
  *out = p;
  return MATE_OK;
}
}  // namespace

mate_status mate_attn_bwd_dense_static(const void* q, const void* k, const void* v, const void* out,
                                       const float* lse, const void* dout, const int32_t* row_ids,
                                       const int32_t* col_ids, const uint8_t* flags,
                                       const uint8_t* head_kind, int B, int H, int N, int D,
                                       mate_dtype t, float scale, void* dq, void* dk, void* dv,
                                       void* stream) {
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return MATE_ERR_NULL;
  DenseArgs a;
  mate_status st = fill_dense(a, row_ids, col_ids, flags, head_kind, B, H, N, D, t, scale);
  if (st != MATE_OK) return st;
  if (mate_dense_workspace_bytes(B, H, N) > (size_t)MATE_STATIC_SCRATCH_BYTES) return MATE_ERR_WORKSPACE;
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != MATE_OK) return st;
  a.q = q; a.k = k; a.v = v; a.o = out; a.dout = dout;
  a.lse = const_cast<float*>(lse);
  a.dq = dq; a.dk = dk; a.dv = dv;
  // Nothing has to be cleared: the dQ kernel writes both arrays at every position before the
  // dK/dV kernel reads them, for this call's (B, H, N); what an earlier call left behind lies
  // beyond that or is overwritten.
  a.delta = static_cast<float*>(ws);
  a.nlse = reinterpret_cast<float*>(static_cast<char*>(ws) + delta_bytes(B, H, N));
  return launch_bwd_dense(a, static_cast<hipStream_t>(stream)) == hipSuccess ? MATE_OK : MATE_ERR_HIP;
}

mate_status mate_profile_kernel(int kernel, void* start_event, void* stop_event) {
  if (kernel < MATE_KERNEL_NONE || kernel > MATE_KERNEL_OUT_PROJECT_WGRAD) return MATE_ERR_UNSUPPORTED;
  if (kernel != MATE_KERNEL_NONE && (!start_event || !stop_event)) return MATE_ERR_NULL;
  g_profile_hook.kernel = kernel;
  g_profile_hook.start = static_cast<hipEvent_t>(start_event);
  g_profile_hook.stop = static_cast<hipEvent_t>(stop_event);
  return MATE_OK;
}

mate_status mate_probe_mfma(float* sink, size_t sink_bytes, int workgroups, int iters,
                            double* flop, void* stream) {
  if (!sink) return MATE_ERR_NULL;
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24)) return MATE_ERR_SHAPE;
  if (sink_bytes < (size_t)workgroups * 256 * sizeof(float)) return MATE_ERR_WORKSPACE;
  if (flop) *flop = mfma_probe_flop(workgroups, iters);
  return launch_mfma_probe(sink, workgroups, iters, static_cast<hipStream_t>(stream)) == hipSuccess
             ? MATE_OK : MATE_ERR_HIP;
}

const char* mate_status_string(mate_status s) {
  switch (s) {
    case MATE_OK: return "ok";
    case MATE_ERR_NULL: return "a required pointer is NULL";
    case MATE_ERR_SHAPE: return "shape out of range, or segment tables built for another (B, N)";
    case MATE_ERR_UNSUPPORTED: return "unsupported head size, dtype or head kind";
    case MATE_ERR_WORKSPACE: return "workspace too small";
    case MATE_ERR_BAD_ID: return "negative id on a table token, or flag value above 2";
    case MATE_ERR_HIP: return "HIP call or kernel launch failed";
  }
  return "unknown status";
}

}  // extern "C"
