/*
 * mate.h -- C ABI of the MI355X (gfx950) implementation of MATE multi-view sparse
 * self-attention (arXiv 2109.04312, "MATE: Multi-view Attention for Table Transformer
 * Efficiency").
 *
 * The operation (Section 3 of the paper).  Every token k of a sequence carries a row
 * number r_k and a column number c_k, and is either a table token, a question token
 * (member of the set Q; attends to and from everything) or padding.  Head i of kind ROW
 * lets table token k attend to  Q U {j : r_j = r_k};  a head of kind COLUMN to
 * Q U {j : c_j = c_k};  a question token attends to every non-pad token (the three-case
 * definition of the attention pattern A^i_k).  The output at position k is the softmax
 * over A^i_k of scale * q_k . k_j applied to the values v_j (the head equation of the same
 * section, after the Q/K/V projections).  The result equals the mask-based implementation
 * exactly; it is computed the way Section 3.1 proposes -- each head kind reorders the table
 * tokens (row order / column order) so that its keys are contiguous -- but with exact
 * variable-length segments in place of fixed-radius buckets.
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers unless the comment says HOST.  The caller owns every
 *     buffer (inputs, outputs, segment tables, workspace); the library allocates nothing
 *     and keeps no state between calls.
 *   - Tensors are contiguous, row-major.  Q, K, V, O, dO, dQ, dK, dV are [B, H, N, D];
 *     LSE is [B, H, N] float; row_ids / col_ids are [B, N] int32; flags is [B, N] uint8.
 *   - D must be 64.  1 <= N <= MATE_MAX_N.  1 <= H <= MATE_MAX_HEADS.  B >= 1.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; only the calls documented as synchronising wait for it.
 *   - Return value: MATE_OK or a negative mate_status.  Argument errors are detected on the
 *     host before anything is launched; nothing is written in that case.
 *   - Base pointers must be 16-byte aligned (any hipMalloc / torch allocation is).
 */
#ifndef MATE_H_
#define MATE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MATE_OK = 0,
  MATE_ERR_NULL = -1,        /* a required pointer is NULL                                */
  MATE_ERR_SHAPE = -2,       /* B, H, N out of range, or tables built for another (B, N)  */
  MATE_ERR_UNSUPPORTED = -3, /* D != 64, unknown dtype or head kind, scale not positive   */
  MATE_ERR_WORKSPACE = -4,   /* workspace_bytes smaller than mate_workspace_bytes(...)    */
  MATE_ERR_BAD_ID = -5,      /* a table token has a negative id, or a flag value > 2      */
  MATE_ERR_HIP = -6          /* a HIP call or kernel launch failed                        */
} mate_status;

typedef enum { MATE_F32 = 0, MATE_BF16 = 1 } mate_dtype;

/* flags[b, n]: what kind of token sits at position n */
enum { MATE_TOK_LOCAL = 0, MATE_TOK_GLOBAL = 1, MATE_TOK_PAD = 2 };
/* head_kind[h] */
enum { MATE_HEAD_ROW = 0, MATE_HEAD_COL = 1 };

enum { MATE_MAX_N = 16384, MATE_MAX_HEADS = 256, MATE_HEAD_DIM = 64,
       MATE_DENSE_MAX_N = 1024 /* longest sequence of the dense-mask variant */,
       MATE_DENSE_PREFERRED_MAX_N = 256 /* measured on MI355X: up to here the dense-mask
                                           variant is the faster of the two */ };

/* Device bytes needed for the segment tables of B sequences of length N (0 if out of range). */
size_t mate_segments_bytes(int B, int N);

/* Device bytes of scratch needed by mate_attn_fwd (for_bwd = 0) or mate_attn_bwd
 * (for_bwd = 1) for this shape; may be 0.  The contents need no initialisation and are
 * undefined afterwards. */
size_t mate_workspace_bytes(int B, int H, int N, int D, mate_dtype t, int for_bwd);

/*
 * Segment builder -- the data-dependent but deterministic per-head-kind reordering of
 * Section 3.1 ("row order traversal" / "column order traversal"), which the paper notes can
 * be computed once per input (caption of the complexity table).  Integer work only.
 *
 * For every sequence b it classifies positions by flag, lists GLOBAL positions in ascending
 * order, and for each view (0 = rows, 1 = columns) stable-sorts the LOCAL positions by their
 * id (row_ids for view 0, col_ids for view 1; ties keep ascending position), numbers the
 * runs of equal id 0..S-1 ("segments") and records where each run starts.  Ids of GLOBAL
 * and PAD tokens are ignored.  A LOCAL token with id 0 shares a segment only with other
 * LOCAL tokens of id 0.
 *
 *   row_ids, col_ids  [B, N] int32, >= 0 for LOCAL tokens
 *   flags             [B, N] uint8, MATE_TOK_*
 *   segments          mate_segments_bytes(B, N) bytes; the valid part of every table is
 *                     overwritten (entries past a list's length are left as they were)
 *
 * Asynchronous on `stream`.  A negative id on a LOCAL token or a flag > 2 does not stop the
 * build (the id is ordered as an unsigned number, the token is treated as padding) but sets
 * a status word that mate_segments_export reports as MATE_ERR_BAD_ID.
 */
mate_status mate_build_segments(const int32_t* row_ids, const int32_t* col_ids,
                                const uint8_t* flags, int B, int N, void* segments,
                                void* stream);

/*
 * Segment builder of the bucketed mode -- the approximation of Section 3.1 ("Efficient
 * implementation"): after each head kind has ordered its input, a global part of at most G
 * tokens attends to and from everything, the rest is grouped in buckets of R consecutive
 * tokens of that order, and a token attends to the global part and to the tokens of its own
 * and the two adjacent buckets that share its row / column.  The appendix gives G = 116,
 * R = 42 for the published models.  With G >= the number of question tokens and R >= the
 * longest row / column the tables equal those of mate_build_segments (last sentence of the
 * section's description).  The paper leaves out the code that fills the global part and builds
 * the windows; this library reads it as:
 *   - the global part is the first `global_length` GLOBAL tokens of a sequence by position;
 *     the GLOBAL tokens after them are treated as LOCAL tokens with the ids they carry
 *     (the paper gives question tokens row = column = 0), so their ids must be >= 0;
 *   - bucket j is sorted slots [j R, (j + 1) R) of the head kind's order of LOCAL tokens;
 *   - the first bucket has no left neighbour and the last no right neighbour (no wrap-around).
 * mate_attn_fwd / mate_attn_bwd given these tables compute the bucketed attention; nothing
 * else changes.  (The dense-mask variant has no bucketed form.)
 *
 *   global_length  G >= 0;  radius  R >= 1;  otherwise MATE_ERR_UNSUPPORTED
 * Everything else as for mate_build_segments.
 */
mate_status mate_build_segments_bucketed(const int32_t* row_ids, const int32_t* col_ids,
                                         const uint8_t* flags, int B, int N, int global_length,
                                         int radius, void* segments, void* stream);

/*
 * Positional index with a restart per cell -- Section 3.2: for sequences longer than 512
 * tokens the index of the positional embedding is reset at the beginning of each cell.
 * Integer work only; independent of the segment tables.
 *
 * A cell is a maximal run of consecutive LOCAL positions with equal (row id, column id).
 *   positions[b, k] = k - (first position of k's cell)   for LOCAL tokens
 *                   = k                                   for GLOBAL tokens
 *                   = 0                                   for PAD tokens (and flags > 2)
 *
 *   row_ids, col_ids, flags   [B, N] as for mate_build_segments
 *   positions                 [B, N] int32, overwritten
 * Asynchronous on `stream`.
 */
mate_status mate_cell_positions(const int32_t* row_ids, const int32_t* col_ids,
                                const uint8_t* flags, int B, int N, int32_t* positions,
                                void* stream);

/*
 * Copies the tables of one view to HOST arrays (test and inspection hook; waits for
 * `stream`).  Any output pointer may be NULL.  Entries past the valid length are -1.
 *
 *   perm        HOST [B, N]    sorted slot -> token position, first L_b valid
 *   seg_off     HOST [B, N+1]  first slot of segment i, then L_b at index S_b
 *   seg_of_tok  HOST [B, N]    token position -> segment index, -1 for GLOBAL / PAD
 *   global_idx  HOST [B, N]    ascending GLOBAL positions, first G_b valid
 *   counts      HOST [B, 3]    G_b, L_b, S_b (of this view)
 *
 * Returns MATE_ERR_BAD_ID if the builder met an invalid id or flag, MATE_ERR_SHAPE if the
 * buffer was built for another (B, N).
 */
mate_status mate_segments_export(const void* segments, int B, int N, int view, int32_t* perm,
                                 int32_t* seg_off, int32_t* seg_of_tok, int32_t* global_idx,
                                 int32_t* counts, void* stream);

/*
 * Status of a table buffer (waits for `stream`; copies a few words per sequence to the host,
 * allocates nothing): MATE_OK, MATE_ERR_SHAPE if the buffer does not hold tables built for this
 * (B, N) -- never built, or built for another shape -- or MATE_ERR_BAD_ID if the builder met a
 * negative id on a LOCAL token or a flag above 2.  This is the call that reports what the
 * asynchronous builder and attention calls cannot return themselves.
 */
mate_status mate_segments_status(const void* segments, int B, int N, void* stream);

/*
 * Copies the attention windows of one view to a HOST array (test and inspection hook; waits
 * for `stream`): window[b][s] = {lo, hi}, the sorted slots [lo, hi) whose tokens slot s attends
 * to besides the global part -- its segment, in bucketed mode cut to buckets j - 1 .. j + 1 of
 * its own bucket j (Section 3.1).  Entries past L_b are {0, 0}.
 *
 *   window      HOST [B, N, 2] int32
 */
mate_status mate_segments_export_windows(const void* segments, int B, int N, int view,
                                         int32_t* window, void* stream);

/*
 * Forward pass: O[b,h,k,:] = sum_{j in A} softmax_j(scale * q_k . k_j) v_j with A the
 * attention pattern of Section 3 for head kind head_kind[h]; one softmax over the union
 * of question keys and own-row (own-column) keys.  LSE[b,h,k] = log sum_{j in A}
 * exp(scale * q_k . k_j), kept for the backward pass.  PAD positions get O = 0, LSE = 0.
 *
 *   q, k, v     [B, H, N, D] of dtype t (bf16: accumulate and softmax in fp32, probabilities
 *               rounded to bf16 before multiplying V; f32: fp32 throughout)
 *   segments    tables from mate_build_segments for the same (B, N)
 *   head_kind   HOST [H] uint8, MATE_HEAD_*
 *   scale       softmax scale, positive and finite (the appendix listing uses 1/sqrt(D));
 *               anything else is MATE_ERR_UNSUPPORTED
 *   out         [B, H, N, D] dtype t;  lse [B, H, N] float
 *   workspace   mate_workspace_bytes(..., 0) bytes (may be NULL if that is 0)
 *
 * Asynchronous on `stream`, so what only the device can see is not in the return value:
 *   - `segments` must point to mate_segments_bytes(B, N) bytes.  If they do not hold tables
 *     built for this (B, N) (never built, or built for another shape) every workgroup leaves
 *     before using them: `out`, `lse` (and dq, dk, dv in the backward) are left exactly as
 *     they were.  mate_segments_status reports MATE_ERR_SHAPE for such a buffer.
 *   - Tables built from invalid ids or flags (MATE_ERR_BAD_ID from mate_segments_status) are
 *     still consistent tables -- the builder orders a negative id as an unsigned number and
 *     treats a flag above 2 as padding -- so the attention runs on them and its results are
 *     those of that reading of the input.
 */
mate_status mate_attn_fwd(const void* q, const void* k, const void* v, const void* segments,
                          const uint8_t* head_kind, int B, int H, int N, int D, mate_dtype t,
                          float scale, void* out, float* lse, void* workspace,
                          size_t workspace_bytes, void* stream);

/*
 * Backward pass: gradients of sum(O * dO) with respect to Q, K, V (the derivative of the
 * forward above; the paper trains through it but does not write it out).  `out` and `lse`
 * are the forward's results for the same inputs.  dO at PAD positions is ignored; PAD
 * positions of dq, dk, dv are written 0.  Deterministic: no floating-point atomics, two
 * runs give identical bits.
 *
 *   dout        [B, H, N, D] dtype t
 *   dq, dk, dv  [B, H, N, D] dtype t (overwritten)
 *   workspace   mate_workspace_bytes(..., 1) bytes
 */
mate_status mate_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                          const float* lse, const void* dout, const void* segments,
                          const uint8_t* head_kind, int B, int H, int N, int D, mate_dtype t,
                          float scale, void* dq, void* dk, void* dv, void* workspace,
                          size_t workspace_bytes, void* stream);

/*
 * Dense-mask variant for short sequences.  Section 3.1 keeps two functionally equivalent
 * implementations (the reordered one above and plain attention under the mask of Section 3) and
 * uses whichever is faster for the sequence length at hand.  These two calls are the second
 * one: same results as mate_attn_fwd / mate_attn_bwd, no segment tables -- every (query, key)
 * pair is scored and kept or dropped by comparing the tokens' ids and flags.
 *
 *   row_ids, col_ids, flags   [B, N] as for mate_build_segments (ids of table tokens must be
 *                             >= 0; nothing checks that here)
 *   t           MATE_BF16 only;  N <= MATE_DENSE_MAX_N;  otherwise MATE_ERR_UNSUPPORTED
 *   workspace   backward only: mate_dense_workspace_bytes(B, H, N) bytes
 * Everything else as above.  Asynchronous on `stream`; deterministic.
 */
size_t mate_dense_workspace_bytes(int B, int H, int N);
/* The choice Section 3.1 describes ("the best of the two functionally equivalent
 * implementations"): non-zero if the dense-mask variant is the faster one for this shape and
 * dtype on MI355X (measured break-even: bf16, N <= MATE_DENSE_PREFERRED_MAX_N), zero if the
 * segment path is (always for MATE_F32, which the dense variant does not support). */
int mate_attn_prefers_dense(int B, int H, int N, mate_dtype t);
mate_status mate_attn_fwd_dense(const void* q, const void* k, const void* v,
                                const int32_t* row_ids, const int32_t* col_ids,
                                const uint8_t* flags, const uint8_t* head_kind, int B, int H,
                                int N, int D, mate_dtype t, float scale, void* out, float* lse,
                                void* stream);
mate_status mate_attn_bwd_dense(const void* q, const void* k, const void* v, const void* out,
                                const float* lse, const void* dout, const int32_t* row_ids,
                                const int32_t* col_ids, const uint8_t* flags,
                                const uint8_t* head_kind, int B, int H, int N, int D,
                                mate_dtype t, float scale, void* dq, void* dk, void* dv,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * mate_attn_bwd_dense for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments without the workspace, same kernels, same results bit for bit.  The scratch
 * (two floats per (b, h, position)) lives in a static device array of MATE_STATIC_SCRATCH_BYTES
 * inside the library, one copy per GPU, held until the process ends; its address is looked up
 * on the first call on each device.  The call allocates and frees nothing.
 *
 *   mate_dense_workspace_bytes(B, H, N) > MATE_STATIC_SCRATCH_BYTES  ->  MATE_ERR_WORKSPACE
 *   (the limit is B * H * N <= 524288, e.g. 32 x 16 x 1024); nothing is launched then.
 *
 * Every call on a GPU uses that GPU's one array: two calls that overlap on the same GPU (on
 * different streams, or from different threads) race on it and must be serialised by the
 * caller.  Calls that follow each other on one stream are safe, whatever their sizes.
 */
enum { MATE_STATIC_SCRATCH_BYTES = 4 * 1024 * 1024 };
mate_status mate_attn_bwd_dense_static(const void* q, const void* k, const void* v, const void* out,
                                       const float* lse, const void* dout, const int32_t* row_ids,
                                       const int32_t* col_ids, const uint8_t* flags,
                                       const uint8_t* head_kind, int B, int H, int N, int D,
                                       mate_dtype t, float scale, void* dq, void* dk, void* dv,
                                       void* stream);

/*
 * The projections either side of the attention, bf16 on the matrix cores.
 *
 * mate_qkv_project: q[b,i,k,:] = W_Q^i x[b,k,:] (+ bias), likewise K and V -- the products
 * W_Q^i X_k, W_K^i X_j, W_V^i X_j of the head equation of Section 3 for all heads at once,
 * written directly in the [B, H, N, 64] layout mate_attn_fwd reads.
 * mate_out_project: y[b,k,:] = W_O concat_i o[b,i,k,:] (+ bias), the output projection of a
 * standard Transformer layer (the paper's equation stops at the head), reading the attention
 * output in the layout mate_attn_fwd writes.
 * Rows of PAD tokens are written as zeros (token tiles of padding only are not computed).
 *
 *   x       [B, N, E] bf16            w_qkv  [3*H*64, E] bf16: the 64 rows of W_Q^0 .. W_Q^{H-1},
 *                                            then of W_K^i, then of W_V^i
 *   o       [B, H, N, 64] bf16        w_o    [E, H*64] bf16
 *   bias    [3*H*64] / [E] float, DEVICE, may be NULL
 *   flags   [B, N] uint8, MATE_TOK_*
 *   q,k,v   [B, H, N, 64] bf16        y      [B, N, E] bf16
 *   t       MATE_BF16 only; H even; E a multiple of 128; otherwise MATE_ERR_UNSUPPORTED
 * fp32 accumulation, one rounding to bf16 on store.  Asynchronous on `stream`; deterministic.
 */
mate_status mate_qkv_project(const void* x, const void* w_qkv, const float* bias,
                             const uint8_t* flags, int B, int N, int H, int E, mate_dtype t,
                             void* q, void* k, void* v, void* stream);
mate_status mate_out_project(const void* o, const void* w_o, const float* bias,
                             const uint8_t* flags, int B, int N, int H, int E, mate_dtype t,
                             void* y, void* stream);

/*
 * Backward of the two projections (the derivative of the calls above; the paper trains through
 * them but does not write them out), bf16 on the matrix cores with fp32 accumulation.
 *
 * mate_qkv_project_bwd:  with G[b,k,:] = the rows of dq, dk, dv at token (b,k) in the feature order
 * of w_qkv (rows of PAD tokens count as zero, whatever they hold),
 *     dx[b,k,:]  = G[b,k,:] w_qkv                      [B, N, E] bf16, rows of PAD tokens written 0
 *     dw_qkv     = sum over non-pad tokens of G^T x    [3*H*64, E] float
 *     dbias      = sum over non-pad tokens of G        [3*H*64] float
 *   dq, dk, dv are read in the [B, H, N, 64] layout mate_attn_bwd writes them in.
 * mate_out_project_bwd:  with G = dy [B, N, E] (rows of PAD tokens count as zero),
 *     d_o[b,i,k,:] = (G[b,k,:] w_o)[64 i .. 64 i + 63] [B, H, N, 64] bf16, the layout mate_attn_bwd
 *                                                      reads dout in; rows of PAD tokens written 0
 *     dw_o       = sum over non-pad tokens of G^T concat_i o[b,i,k,:]    [E, H*64] float
 *     dbias      = sum over non-pad tokens of G        [E] float
 *
 *   dx / d_o, dw_*, dbias   any of them may be NULL (not computed); dbias needs dw_*
 *   workspace   mate_project_bwd_workspace_bytes(B, N, H, E) bytes (a transposed copy of the
 *               weights, one 64-bit pad mask per 64 tokens, partial sums of the weight gradient)
 *   t, H, E     as for the forward calls
 * Asynchronous on `stream`; deterministic (partial sums are added in a fixed order, no atomics).
 */
size_t mate_project_bwd_workspace_bytes(int B, int N, int H, int E);
mate_status mate_qkv_project_bwd(const void* x, const void* w_qkv, const uint8_t* flags,
                                 const void* dq, const void* dk, const void* dv, int B, int N,
                                 int H, int E, mate_dtype t, void* dx, float* dw_qkv, float* dbias,
                                 void* workspace, size_t workspace_bytes, void* stream);
mate_status mate_out_project_bwd(const void* o, const void* w_o, const uint8_t* flags,
                                 const void* dy, int B, int N, int H, int E, mate_dtype t,
                                 void* d_o, float* dw_o, float* dbias, void* workspace,
                                 size_t workspace_bytes, void* stream);

/*
 * Measurement hook, not part of the computation: arms the calling thread so that the next
 * launch of the named kernel (inside mate_build_segments / mate_attn_fwd* / mate_attn_bwd* /
 * mate_*_project) is
 * bracketed by hipEventRecord(start_event) and hipEventRecord(stop_event) on the stream of that
 * call; the hook disarms itself once used.  The events are hipEvent_t handles passed as void*,
 * created with timing enabled and owned by the caller.  kernel = MATE_KERNEL_NONE disarms.
 * This is the only state the library keeps (per host thread).
 */
enum { MATE_KERNEL_NONE = 0, MATE_KERNEL_BUILD = 1, MATE_KERNEL_FWD = 2, MATE_KERNEL_BWD_DQ = 3,
       MATE_KERNEL_BWD_DKV = 4, MATE_KERNEL_FWD_DENSE = 5, MATE_KERNEL_BWD_DQ_DENSE = 6,
       MATE_KERNEL_BWD_DKV_DENSE = 7, MATE_KERNEL_QKV_PROJECT = 8, MATE_KERNEL_OUT_PROJECT = 9,
       MATE_KERNEL_QKV_PROJECT_DGRAD = 10, MATE_KERNEL_QKV_PROJECT_WGRAD = 11,
       MATE_KERNEL_OUT_PROJECT_DGRAD = 12, MATE_KERNEL_OUT_PROJECT_WGRAD = 13 };
mate_status mate_profile_kernel(int kernel, void* start_event, void* stop_event);

/*
 * Measurement aid, not part of the computation: launches a kernel that only issues independent
 * 32x32x16 bf16 matrix instructions (`workgroups` x 4 wavefronts x `iters` x 8 of them), so a
 * benchmark can time what the matrix cores of this machine sustain, beside the nominal peak.
 *   sink        workgroups * 256 floats, overwritten (keeps the work alive)
 *   flop        HOST, may be NULL: receives the number of floating-point operations launched
 * Asynchronous on `stream`.
 */
mate_status mate_probe_mfma(float* sink, size_t sink_bytes, int workgroups, int iters,
                            double* flop, void* stream);

/* Static, NUL-terminated description of a status code (HOST pointer, never NULL). */
const char* mate_status_string(mate_status s);

#ifdef __cplusplus
}
#endif
#endif /* MATE_H_ */
