"""CPU oracle for MATE multi-view sparse attention.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file.
It shares no code with the HIP library and never calls it.  Everything is float64 numpy,
written as the plain definition: an explicit N x N 0/1 mask, a dense masked softmax, and
the textbook derivative of that.  There is no tiling, sorting trick, online softmax or
fusion here; `numpy.matmul`, `numpy.exp` and `sorted` are the only library steps.

What each function follows in the paper (arXiv 2109.04312):
  * attention_mask      -- the attention-pattern equation of Section 3 (the three-case
                           definition of A^i_k), with "all positions (except padding)".
  * attn_forward        -- the head equation of Section 3 (gather over A^i_k, softmax of
                           key.query scores, weighted sum of values), realised as the
                           mask-based implementation the same section describes.
  * attn_backward       -- not in the paper: the derivative of attn_forward w.r.t. Q, K, V.
  * build_segments      -- the per-head data-dependent, deterministic reordering of
                           Section 3.1 (row-order / column-order traversal), stated as a
                           stable sort plus run boundaries.
  * bucketed_flags, bucketed_attention_mask
                        -- the approximation of Section 3.1 ("Efficient implementation"):
                           a global part of at most G tokens, the rest of each head's
                           ordered input in buckets of R, a bucket attending to itself and
                           to its two neighbours, further restricted by the row / column
                           mask.  Every function below takes `bucketed=(G, R)` for it.
                           PARITY UNPINNED for the readings listed under "bucketed" below:
                           the paper leaves out the code that would decide them.
  * cell_positions      -- Section 3.2: for long sequences the index of the positional
                           embedding restarts at the beginning of each cell.
  * project_qkv, project_out
                        -- the projections either side of the attention: W_Q^i X_k, W_K^i X_j,
                           W_V^i X_j of the head equation of Section 3 for all heads at once,
                           and the usual output projection over the concatenated heads (the
                           equation stops at the head; the model is a standard Transformer
                           layer otherwise).
  * project_qkv_backward, project_out_backward
                        -- not in the paper: the derivatives of the two projections with
                           respect to their input, weights and bias.

Readings taken where the paper is silent (listed again in the design notes):
  * the softmax scale is an explicit argument (the equation has none, the appendix
    listing divides by sqrt(head size));
  * Q is given by a per-token GLOBAL flag, not inferred from row = column = 0;
  * a table token with id 0 shares a segment only with other *table* tokens of id 0;
  * padding is a third flag value: pad keys get exactly zero weight, pad queries
    produce zero output and zero gradients;
  * local rows use ONE softmax over (global keys U own row/column keys).
  * positional index: a cell is a maximal run of consecutive table tokens with the same
    (row, column); question tokens keep their absolute position, pads get 0.
Bucketed mode (Section 3.1 and the description of the views in the appendix):
  * the global part is the first G question tokens by position; question tokens beyond
    it join the long part with the ids they carry (the section's claim that the two
    implementations agree once G covers the question part holds exactly this way);
  * the long part is the head's sorted order of table tokens (pads excluded), bucket j =
    sorted slots [jR, (j+1)R); the last bucket may be short;
  * "adjacent" does not wrap around: the first bucket has no left neighbour, the last no
    right neighbour (a rotation would pair them; the row / column mask hides that pair
    unless one segment spans the whole long part).

Pins: tests/test_oracle_*.py (brute force from set notation, library SDPA special
cases, closed forms, finite differences, permutation / relabelling invariants,
brute-force ranks for the segment tables).
"""
from __future__ import annotations

import numpy as np

TOK_LOCAL, TOK_GLOBAL, TOK_PAD = 0, 1, 2
HEAD_ROW, HEAD_COL = 0, 1


# --------------------------------------------------------------------------------------
# Attention pattern (Section 3, definition of A^i_k)
# --------------------------------------------------------------------------------------
def attention_mask(row_ids, col_ids, flags, kind) -> np.ndarray:
    """mask[k, j] = 1 iff query position k may attend to key position j (one sequence).

    k in Q (GLOBAL)  -> every non-pad j
    else, row head   -> Q  U  {j : r_j = r_k}
    else, column head-> Q  U  {j : c_j = c_k}
    Pad keys are never attended; pad queries attend to nothing.  The sets {j : r_j = r_k}
    range over table tokens only (a question token enters once, through Q).
    """
    row_ids = np.asarray(row_ids)
    col_ids = np.asarray(col_ids)
    flags = np.asarray(flags)
    ids = row_ids if kind == HEAD_ROW else col_ids
    is_g = flags == TOK_GLOBAL
    is_l = flags == TOK_LOCAL
    nonpad = is_g | is_l
    same = (ids[:, None] == ids[None, :]) & is_l[:, None] & is_l[None, :]
    m = same | (is_g[:, None] & nonpad[None, :]) | (is_l[:, None] & is_g[None, :])
    return m.astype(np.uint8)


def useful_pairs(row_ids, col_ids, flags, kind, bucketed=None) -> int:
    """Number of (query, key) pairs with non-zero weight for one sequence and head kind."""
    return int(_mask(row_ids, col_ids, flags, kind, bucketed).sum(dtype=np.int64))


# --------------------------------------------------------------------------------------
# Bucketed approximation (Section 3.1)
# --------------------------------------------------------------------------------------
def bucketed_flags(flags, global_length) -> np.ndarray:
    """Flags of one sequence after the global part is cut at `global_length` tokens: the
    question tokens past the first G (in position order) become table tokens."""
    flags = np.array(flags, np.uint8, copy=True)
    seen = 0
    for p in range(flags.shape[0]):
        if flags[p] == TOK_GLOBAL:
            if seen >= global_length:
                flags[p] = TOK_LOCAL
            seen += 1
    return flags


def bucket_of_token(ids, flags, radius) -> np.ndarray:
    """Bucket index of every table token of one sequence in one view (-1 for the others):
    tokens ordered by id, ties by position; slot s of that order lies in bucket s // R."""
    N = len(flags)
    loc = [p for p in range(N) if flags[p] == TOK_LOCAL]
    order = sorted(loc, key=lambda p: int(ids[p]))
    bucket = np.full(N, -1, np.int64)
    for slot, p in enumerate(order):
        bucket[p] = slot // radius
    return bucket


def bucketed_attention_mask(row_ids, col_ids, flags, kind, global_length, radius) -> np.ndarray:
    """mask[k, j] of Section 3.1 for one sequence: the pattern of Section 3 on the flags cut at
    G, with a table-token pair kept only if the two buckets are equal or adjacent."""
    fl = bucketed_flags(flags, global_length)
    m = attention_mask(row_ids, col_ids, fl, kind).astype(bool)
    ids = np.asarray(row_ids if kind == HEAD_ROW else col_ids)
    bucket = bucket_of_token(ids, fl, radius)
    is_l = fl == TOK_LOCAL
    both_local = is_l[:, None] & is_l[None, :]
    near = np.abs(bucket[:, None] - bucket[None, :]) <= 1
    return (m & (~both_local | near)).astype(np.uint8)


def _mask(row_ids, col_ids, flags, kind, bucketed):
    if bucketed is None:
        return attention_mask(row_ids, col_ids, flags, kind)
    return bucketed_attention_mask(row_ids, col_ids, flags, kind, *bucketed)


# --------------------------------------------------------------------------------------
# Forward (Section 3, head equation; mask-based implementation)
# --------------------------------------------------------------------------------------
def _head_forward(q, k, v, mask, scale):
    """One (sequence, head): q,k,v [N,D] float64, mask [N,N] -> O [N,D], LSE [N], P [N,N]."""
    s = scale * (q @ k.T)
    allowed = mask.astype(bool)
    has = allowed.any(axis=1)
    s_m = np.where(allowed, s, -np.inf)
    m = np.where(has, s_m.max(axis=1, initial=-np.inf), 0.0)
    e = np.where(allowed, np.exp(s_m - m[:, None]), 0.0)
    z = e.sum(axis=1)
    p = e / np.where(has, z, 1.0)[:, None]
    o = p @ v
    lse = np.where(has, m + np.log(np.where(has, z, 1.0)), 0.0)
    return o, lse, p


def attn_forward(q, k, v, row_ids, col_ids, flags, head_kind, scale, bucketed=None):
    """q,k,v [B,H,N,D] -> (O [B,H,N,D] float64, LSE [B,H,N] float64).

    LSE_k = log sum_{j in A_k} exp(scale * q_k.k_j); rows of pad queries are 0 in both.
    bucketed = (G, R) selects the pattern of Section 3.1 instead of Section 3's.
    """
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    B, H, N, D = q.shape
    o = np.zeros((B, H, N, D), np.float64)
    lse = np.zeros((B, H, N), np.float64)
    for b in range(B):
        masks = {}
        for h in range(H):
            kind = int(head_kind[h])
            if kind not in masks:
                masks[kind] = _mask(row_ids[b], col_ids[b], flags[b], kind, bucketed)
            o[b, h], lse[b, h], _ = _head_forward(q[b, h], k[b, h], v[b, h], masks[kind], scale)
    return o, lse


# --------------------------------------------------------------------------------------
# Backward (derivative of the above; loss gradient dO is the only incoming gradient)
# --------------------------------------------------------------------------------------
def _head_backward(q, k, v, do, mask, scale):
    o, _, p = _head_forward(q, k, v, mask, scale)
    delta = (do * o).sum(axis=1)             # delta_k = dO_k . O_k
    dv = p.T @ do                            # dV_j = sum_k P[k,j] dO_k
    dp = do @ v.T                            # dP[k,j] = dO_k . V_j
    ds = p * (dp - delta[:, None])           # softmax Jacobian, row by row
    dq = scale * (ds @ k)                    # dQ_k = scale sum_j dS[k,j] K_j
    dk = scale * (ds.T @ q)                  # dK_j = scale sum_k dS[k,j] Q_k
    return dq, dk, dv


def attn_backward(q, k, v, do, row_ids, col_ids, flags, head_kind, scale, bucketed=None):
    """Gradients (dQ, dK, dV) [B,H,N,D] float64 of sum(O * dO); dO at pad queries is ignored."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    do = np.asarray(do, np.float64)
    B, H, N, D = q.shape
    dq = np.zeros_like(q)
    dk = np.zeros_like(q)
    dv = np.zeros_like(q)
    for b in range(B):
        masks = {}
        nonpad = (np.asarray(flags[b]) != TOK_PAD)[:, None]
        for h in range(H):
            kind = int(head_kind[h])
            if kind not in masks:
                masks[kind] = _mask(row_ids[b], col_ids[b], flags[b], kind, bucketed)
            dq[b, h], dk[b, h], dv[b, h] = _head_backward(
                q[b, h], k[b, h], v[b, h], do[b, h] * nonpad, masks[kind], scale)
    return dq, dk, dv


# --------------------------------------------------------------------------------------
# Segment tables (Section 3.1: per-head reordering of the table tokens)
# --------------------------------------------------------------------------------------
def build_segments(row_ids, col_ids, flags, bucketed=None):
    """Per-sequence integer tables, fixed-size arrays filled with -1 past their valid length.
    bucketed = (G, R): the tables of the flags cut at G (Section 3.1), windows limited to the
    neighbouring buckets.

    Returns a dict with
      counts      [B,4]  int32 : G (global), L (table), S_row, S_col
      global_idx  [B,N]  int32 : ascending positions of GLOBAL tokens
      perm        [2,B,N]  int32 : view 0 = rows, 1 = columns; table-token positions sorted by
                                   (id, position) -- i.e. a stable sort by id
      seg_off     [2,B,N+1] int32: first sorted slot of each segment, then L
      seg_of_tok  [2,B,N]  int32 : segment index of each table token, -1 for others
      window      [2,B,N,2] int32: per sorted slot, the range [lo, hi) of sorted slots whose
                                   tokens it attends to: its segment, in bucketed mode cut
                                   to buckets j-1 .. j+1 of its own bucket j; 0,0 past L
    """
    row_ids = np.asarray(row_ids)
    col_ids = np.asarray(col_ids)
    flags = np.asarray(flags)
    B, N = flags.shape
    counts = np.zeros((B, 4), np.int32)
    global_idx = np.full((B, N), -1, np.int32)
    perm = np.full((2, B, N), -1, np.int32)
    seg_off = np.full((2, B, N + 1), -1, np.int32)
    seg_of_tok = np.full((2, B, N), -1, np.int32)
    window = np.zeros((2, B, N, 2), np.int32)
    if bucketed is not None:
        flags = np.stack([bucketed_flags(flags[b], bucketed[0]) for b in range(B)])
    for b in range(B):
        glob = [p for p in range(N) if flags[b, p] == TOK_GLOBAL]
        loc = [p for p in range(N) if flags[b, p] == TOK_LOCAL]
        counts[b, 0] = len(glob)
        counts[b, 1] = len(loc)
        global_idx[b, : len(glob)] = glob
        for view, ids in enumerate((row_ids[b], col_ids[b])):
            order = sorted(loc, key=lambda p: int(ids[p]))   # Python's sort is stable
            perm[view, b, : len(order)] = order
            n_seg = 0
            for slot, p in enumerate(order):
                if slot == 0 or ids[p] != ids[order[slot - 1]]:
                    seg_off[view, b, n_seg] = slot
                    n_seg += 1
                seg_of_tok[view, b, p] = n_seg - 1
            seg_off[view, b, n_seg] = len(order)
            counts[b, 2 + view] = n_seg
            for slot, p in enumerate(order):
                g = seg_of_tok[view, b, p]
                lo, hi = int(seg_off[view, b, g]), int(seg_off[view, b, g + 1])
                if bucketed is not None:
                    j, R = slot // bucketed[1], bucketed[1]
                    lo, hi = max(lo, (j - 1) * R), min(hi, (j + 2) * R)
                window[view, b, slot] = (lo, hi)
    return dict(counts=counts, global_idx=global_idx, perm=perm, seg_off=seg_off,
                seg_of_tok=seg_of_tok, window=window)


# --------------------------------------------------------------------------------------
# Positional index with a restart per cell (Section 3.2)
# --------------------------------------------------------------------------------------
def cell_positions(row_ids, col_ids, flags):
    """[B,N] int32: index fed to the positional embedding.  A table token gets its offset from
    the first token of its cell (a cell = consecutive table tokens sharing row and column), a
    question token its position in the sequence, a pad 0."""
    row_ids = np.asarray(row_ids)
    col_ids = np.asarray(col_ids)
    flags = np.asarray(flags)
    B, N = flags.shape
    out = np.zeros((B, N), np.int32)
    for b in range(B):
        start = 0
        for p in range(N):
            if flags[b, p] == TOK_GLOBAL:
                out[b, p] = p
            elif flags[b, p] == TOK_LOCAL:
                same_cell = (p > 0 and flags[b, p - 1] == TOK_LOCAL
                             and row_ids[b, p - 1] == row_ids[b, p] and col_ids[b, p - 1] == col_ids[b, p])
                if not same_cell:
                    start = p
                out[b, p] = p - start
    return out


# --------------------------------------------------------------------------------------
# Projections either side of the attention (head equation of Section 3)
# --------------------------------------------------------------------------------------
def project_qkv(x, w_qkv, bias, flags, n_heads):
    """x [B,N,E];  w_qkv [3*H*m, E] holds the rows of W_Q^0 .. W_Q^{H-1}, then W_K^i, then W_V^i
    (m rows per head);  bias [3*H*m] or None.  Returns q, k, v [B,H,N,m] float64 with
    q[b,i,k,:] = W_Q^i x[b,k,:] (+ bias); rows of pad tokens are 0."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w_qkv, np.float64)
    B, N, E = x.shape
    m = w.shape[0] // (3 * n_heads)
    y = x @ w.T
    if bias is not None:
        y = y + np.asarray(bias, np.float64)
    y = y * (np.asarray(flags) != TOK_PAD)[:, :, None]
    y = y.reshape(B, N, 3, n_heads, m)
    return tuple(np.ascontiguousarray(y[:, :, t].transpose(0, 2, 1, 3)) for t in range(3))


def project_out(o, w_o, bias, flags):
    """o [B,H,N,m];  w_o [E, H*m];  bias [E] or None.  y[b,k,:] = w_o . concat_i o[b,i,k,:]
    (+ bias), float64 [B,N,E]; rows of pad tokens are 0."""
    o = np.asarray(o, np.float64)
    B, H, N, m = o.shape
    cat = o.transpose(0, 2, 1, 3).reshape(B, N, H * m)
    y = cat @ np.asarray(w_o, np.float64).T
    if bias is not None:
        y = y + np.asarray(bias, np.float64)
    return y * (np.asarray(flags) != TOK_PAD)[:, :, None]


def project_qkv_backward(x, w_qkv, flags, dq, dk, dv, n_heads):
    """Derivative of project_qkv: with Y = [q | k | v] (all heads, feature order as the rows of
    w_qkv) and G = dL/dY assembled from dq, dk, dv [B,H,N,m] (rows of pad tokens ignored: the
    forward writes zeros there whatever x is), returns
      dx [B,N,E]      = G w_qkv           (0 at pad tokens)
      dw [3*H*m, E]   = sum over non-pad tokens of G^T x
      dbias [3*H*m]   = sum over non-pad tokens of G."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w_qkv, np.float64)
    B, N, E = x.shape
    keep = (np.asarray(flags) != TOK_PAD)[:, :, None]
    g = np.concatenate([np.asarray(t, np.float64).transpose(0, 2, 1, 3).reshape(B, N, -1) for t in (dq, dk, dv)],
                       axis=-1) * keep                                  # [B,N,3*H*m]
    dx = g @ w
    g2 = g.reshape(B * N, -1)
    dw = g2.T @ x.reshape(B * N, E)
    return dx, dw, g2.sum(axis=0)


def project_out_backward(o, w_o, flags, dy):
    """Derivative of project_out: with G = dy [B,N,E] (rows of pad tokens ignored), returns
      d_o [B,H,N,m]  = G w_o, split back into heads (0 at pad tokens)
      dw [E, H*m]    = sum over non-pad tokens of G^T concat_i o[:, i]
      dbias [E]      = sum over non-pad tokens of G."""
    o = np.asarray(o, np.float64)
    w = np.asarray(w_o, np.float64)
    B, H, N, m = o.shape
    g = np.asarray(dy, np.float64) * (np.asarray(flags) != TOK_PAD)[:, :, None]
    cat = o.transpose(0, 2, 1, 3).reshape(B, N, H * m)
    d_cat = g @ w                                                        # [B,N,H*m]
    d_o = np.ascontiguousarray(d_cat.reshape(B, N, H, m).transpose(0, 2, 1, 3))
    g2 = g.reshape(B * N, -1)
    dw = g2.T @ cat.reshape(B * N, H * m)
    return d_o, dw, g2.sum(axis=0)
