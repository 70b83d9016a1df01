// Segment builder: the per-head-kind reordering of Section 3.1 (row-order / column-order
// traversal of the table tokens), computed as a stable sort of the table-token positions by id
// plus run boundaries.  Integer work only.  1024-thread workgroups; all sorting lives in LDS.
//
// Two ways, chosen on the device from the ids themselves:
//   * sequences of more than 1024 positions whose ids are all below 512 (every row and column
//     number of a real table): the order is a counting
//     sort, slot(p) = first slot of id_p + number of earlier table tokens with the same id, and
//     everything else (segments, windows, work units) follows from the histogram of ids.  Up to
//     eight workgroups share a (sequence, view): each reads the whole sequence (a few KB),
//     builds the histogram and the part of it that lies before its own chunk of positions, and
//     ranks and writes only its chunk; one more workgroup has no chunk and lists the work units
//     instead (the longest single piece of work after the histogram).  Nothing is exchanged
//     between workgroups.
//   * otherwise (short sequences, where one workgroup is as fast; large ids): workgroup 0 of the
//     (sequence, view) sorts alone, as described next.
//
// Sort: table-token positions are first compacted in ascending order, then reordered by a
// least-significant-digit radix sort on their id, 9 bits per pass.  Each pass is stable (every
// wavefront owns a contiguous block of the current order, counts its digits, and ranks equal
// digits inside a 64-element batch in lane order with ballots), so ties keep ascending position.
// Passes whose digit is zero for every id are skipped: ids below 512 cost one pass.
//
// The kernel also lists the work units of the attention kernels per (sequence, view): pieces of
// up to 128 slots of the sorted order (cut so that none straddles the boundary of a long
// segment, listed longest streamed side first) with the window of sorted slots their segments
// span, then the pad tiles, and per sequence the chunks of the question-token owners.  The
// attention kernels map a workgroup index to one of these records with arithmetic alone.
//
// Bucketed mode (the approximation of Section 3.1: a global part of at most G tokens, the rest
// of the head's order in buckets of R, a bucket meeting itself and its two neighbours): the
// question tokens past the first `max_global` are classified as table tokens, and every slot's
// window is its segment cut to the slots of buckets j - 1 .. j + 1 of its own bucket j.  The
// attention kernels read windows only, so the mode lives entirely in these tables.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "launch.h"
#include "seg_layout.h"

namespace mate {

constexpr int kSegThreads = 1024;
constexpr int kSegWaves = kSegThreads / 64;
constexpr int kDigitBits = 9;               // radix digit: ids below 512 sort in one pass
constexpr unsigned kBins = 1u << kDigitBits;

// Workgroup barrier for data exchanged through LDS only: waits for this wavefront's LDS traffic,
// not for its global stores (a full fence would stall every phase on store round trips; nothing
// the kernel writes to global memory is read back inside it).
__device__ inline void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

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
  lds_barrier();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSegWaves; ++w) {
    int s = tmp[w];
    if (w < wave) base += s;
    tot += s;
  }
  lds_barrier();
  total = tot;
  return base + inc - v;
}

// Number of set bits of `mask` that belong to lanes before this one (v_mbcnt).
__device__ inline int lanes_before(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
}

// Exclusive prefix count of one flag per thread across the workgroup (ballots instead of a
// shuffle chain); `total` gets the number of set flags.  Same contract as block_exclusive_scan.
__device__ inline int block_flag_scan(bool flag, int* tmp, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long m = __ballot(flag);
  if (lane == 0) tmp[wave] = __popcll(m);
  lds_barrier();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSegWaves; ++w) {
    const int c = tmp[w];
    if (w < wave) base += c;
    tot += c;
  }
  lds_barrier();
  total = tot;
  return base + lanes_before(m);
}

// The value of the previous lane (lane 0 keeps its own): a DPP move, no LDS round trip.
__device__ inline int from_previous_lane(int v) {
  return __builtin_amdgcn_update_dpp(v, v, 0x138 /* wave_shr:1 */, 0xf, 0xf, false);
}

// Lanes of the wavefront that hold the same digit as this lane (valid lanes only).  Only the
// bits of `vary` (wave-uniform: the bits in which the digits of this batch differ at all) need a
// ballot each.
__device__ inline unsigned long long match_digit(unsigned digit, bool valid, unsigned vary) {
  unsigned long long same = __ballot(valid);
  for (unsigned v = vary; v; v &= v - 1u) {
    const bool one = (digit >> (__ffs(v) - 1)) & 1u;
    const unsigned long long m = __ballot(one);
    same &= one ? m : ~m;
  }
  return same;
}
// Bits in which the digits of the valid lanes differ (wave-uniform).
__device__ inline unsigned varying_bits(unsigned digit, bool valid) {
  const unsigned long long vm = __ballot(valid);
  if (vm == 0) return 0u;
  const unsigned first = __builtin_amdgcn_readlane(digit, __ffsll((long long)vm) - 1);
  unsigned d = valid ? digit ^ first : 0u;
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) d |= __shfl_xor(d, s, 64);
  return __builtin_amdgcn_readfirstlane(d);
}

template <int P2>
__global__ __launch_bounds__(kSegThreads) void build_segments_kernel(
    const int* __restrict__ row_ids, const int* __restrict__ col_ids,
    const unsigned char* __restrict__ flags, int B, int N, int max_global, int radius,
    int* __restrict__ seg) {
  constexpr int CHUNK = P2 / kSegWaves;  // consecutive elements owned by one wavefront
  constexpr int NB = CHUNK / 64;         // 64-element batches per wavefront
  static_assert(NB >= 1, "P2 must be at least the workgroup size");
  __shared__ int ids[P2];                  // id by token position; later: segment starts (ushort)
  __shared__ unsigned short buf_a[P2];     // current order of table-token positions
  __shared__ unsigned short buf_b[P2];     // next order; later: segment index by slot
  __shared__ unsigned short hist[kSegWaves][kBins];  // per-wavefront digit counts -> first output slots
  __shared__ int scan_tmp[kSegWaves + 1];
  __shared__ int wave_tot[5][kSegWaves];
  __shared__ int s_or, s_bad;
  // counting-sort path: ids seen anywhere / before this workgroup's chunk (they live in the two
  // order buffers, which only the general path uses, and later); first slot and segment index
  // of every id; scratch for the work-unit list
  int* const full_h = reinterpret_cast<int*>(buf_b);
  int* const before_h = reinterpret_cast<int*>(buf_a);
  __shared__ int start_v[kBins + 1];
  __shared__ int seg_i[kBins];
  __shared__ int seg_tmp[2][kBins + 8];
  static_assert(P2 * sizeof(unsigned short) >= kBins * sizeof(int), "histograms must fit the order buffers");

  const int b = blockIdx.x, view = blockIdx.y, tid = threadIdx.x;
  // Several workgroups per (sequence, view): K of them take a chunk of the positions each, one
  // more (k == K, no chunk) lists the work units.
  const int k = blockIdx.z, K = gridDim.z > 1 ? (int)gridDim.z - 1 : 1;
  const int chunk = (((N + K - 1) / K) + 63) & ~63, c0 = k < K ? k * chunk : 0, c1 = min(N, c0 + chunk);
  const int lane = tid & 63, wave = tid >> 6;
  const SegLayout lay(B, N);
  int* counts = seg + lay.counts + (size_t)b * kCountWords;
  int* global_idx = seg + lay.global_idx + (size_t)b * N;
  int* pad_idx = seg + lay.pad_idx + (size_t)b * N;
  int* vbase = seg + lay.view0 + (size_t)view * lay.view_stride;
  int* perm = vbase + lay.perm + (size_t)b * N;
  int* seg_off = vbase + lay.seg_off + (size_t)b * (N + 1);
  int* seg_of_tok = vbase + lay.seg_of_tok + (size_t)b * N;
  int2* slot_rng = reinterpret_cast<int2*>(vbase + lay.slot_rng) + (size_t)b * N;
  int4* unit = reinterpret_cast<int4*>(vbase + lay.unit) + (size_t)b * lay.units * 2;
  int4* gunit = reinterpret_cast<int4*>(seg + lay.gunit) + (size_t)b * lay.tiles * 2;
  const int* id_src = (view == 0 ? row_ids : col_ids) + (size_t)b * N;
  const unsigned char* fl = flags + (size_t)b * N;

  if (b == 0 && view == 0 && k == 0 && tid < kHdrWords)
    seg[tid] = tid == 0 ? kMagic : tid == 1 ? B : tid == 2 ? N : tid == 4 ? max_global : tid == 5 ? radius : 0;
  if (tid == 0) { s_or = 0; s_bad = 0; }
  if (tid < kBins) { full_h[tid] = 0; before_h[tid] = 0; }
  lds_barrier();

  // Element order everywhere below: a wavefront owns CHUNK consecutive elements and walks them in
  // batches of 64, lane = consecutive element, so that LDS and global accesses are unit-stride
  // and ranks inside a batch come from ballots.
  const int w0 = wave * CHUNK;

  // All of this wavefront's inputs first, in one go: the loads travel together instead of one
  // dependent round trip per batch (the compiler does not move them across the stores below).
  unsigned char in_flag[NB];
  int in_id[NB];
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    const int i = w0 + e * 64 + lane;
    in_flag[e] = i < N ? fl[i] : (unsigned char)3;
    in_id[e] = i < N ? id_src[i] : 0;
  }

  // ---- bucketed mode: question tokens past the first max_global join the table tokens ----------
  unsigned demote = 0;  // bit e: my element of batch e is such a token
  if (max_global < N) {  // uniform; a sequence has at most N question tokens
    int n_q = 0;
#pragma unroll
    for (int e = 0; e < NB; ++e) {
      n_q += __popcll(__ballot(in_flag[e] == 1));
    }
    if (lane == 0) wave_tot[1][wave] = n_q;
    lds_barrier();
    int q_at = 0;
#pragma unroll
    for (int w = 0; w < kSegWaves; ++w)
      if (w < wave) q_at += wave_tot[1][w];
    lds_barrier();  // wave_tot is written again below
#pragma unroll
    for (int e = 0; e < NB; ++e) {
      const bool is_q = in_flag[e] == 1;
      const unsigned long long mq = __ballot(is_q);
      if (is_q && q_at + lanes_before(mq) >= max_global) demote |= 1u << e;
      q_at += __popcll(mq);
    }
  }

  // ---- classify; count the three kinds of position per wavefront ---------------------------
  unsigned char my_flag[NB];
  int n_g = 0, n_p = 0, n_l = 0, bad = 0, my_or = 0;
  int g_bef = 0, p_bef = 0;  // question / pad tokens before this workgroup's chunk (this wavefront's share)
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    const int i = w0 + e * 64 + lane;
    unsigned char f = 3;
    int id = 0;
    if (i < N) {
      f = in_flag[e];
      if (f > 2) { bad = 1; f = 2; }
      if ((demote >> e) & 1u) f = 0;
      id = in_id[e];
      if (f == 0) {
        if (id < 0) bad = 1;
        my_or |= id;
      }
      ids[i] = f == 0 ? id : -(int)f;   // table token: its id; question token -1; pad -2
    }
    my_flag[e] = f;
    const unsigned long long ml = __ballot(f == 0), mg = __ballot(f == 1), mp = __ballot(f == 2);
    n_l += __popcll(ml);
    n_g += __popcll(mg);
    n_p += __popcll(mp);
    if (w0 + e * 64 < c0) { g_bef += __popcll(mg); p_bef += __popcll(mp); }   // (c0 is a multiple of 64)
    // histogram of the low digit, one LDS add per run of equal ids inside the batch (ids of a
    // flattened table come in runs); only meaningful if every id turns out to be below kBins
    const int key = f == 0 ? (id & (int)(kBins - 1u)) : -1;
    const int prev = from_previous_lane(key);
    const bool head = lane == 0 || key != prev;
    const unsigned long long mh = __ballot(head);
    if (head && key >= 0) {
      const unsigned long long later = lane == 63 ? 0ull : mh >> (lane + 1);
      const int run = later ? __ffsll((long long)later) : 64 - lane;
      atomicAdd(&full_h[key], run);
      if (w0 + e * 64 < c0) atomicAdd(&before_h[key], run);
    }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) my_or |= __shfl_xor(my_or, d, 64);
  if (lane == 0) {
    wave_tot[0][wave] = n_l;
    wave_tot[1][wave] = n_g;
    wave_tot[2][wave] = n_p;
    wave_tot[3][wave] = g_bef;
    wave_tot[4][wave] = p_bef;
    if (my_or) atomicOr(&s_or, my_or);
  }
  if (bad) s_bad = 1;
  lds_barrier();
  int L = 0, G = 0, P = 0, l_at = 0, g_at = 0, p_at = 0, g_before = 0, p_before = 0;
#pragma unroll
  for (int w = 0; w < kSegWaves; ++w) {
    const int cl = wave_tot[0][w], cg = wave_tot[1][w], cp = wave_tot[2][w];
    if (w < wave) { l_at += cl; g_at += cg; p_at += cp; }
    L += cl; G += cg; P += cp;
    g_before += wave_tot[3][w];
    p_before += wave_tot[4][w];
  }
  const unsigned all_bits = (unsigned)s_or;
  const float inv_radius = radius > 0 ? 1.0f / (float)radius : 0.f;
  const int n_pt = (P + kPadSlots - 1) / kPadSlots;
  const int n_t0 = (G + BN - 1) / BN;
  constexpr int kMaxUnits = kMaxTiles + kMaxTiles / 2 + 2;
  __shared__ unsigned short head_pos[kMaxUnits];
  __shared__ unsigned short unit_len[kMaxUnits];

  if (K > 1 && (all_bits & ~(kBins - 1u)) == 0) {
    // ============ counting-sort path: every id is below kBins, several workgroups ============
    constexpr int NBC = P2 > 8 * kSegThreads ? 2 : 1;   // 64-position batches of the chunk per wavefront
    // first slot and segment index of every id
    const int c_id = tid < (int)kBins ? full_h[tid] : 0;
    int tot_l, S;
    const int first_slot = block_exclusive_scan(c_id, scan_tmp, tot_l);
    const int seg_index = block_flag_scan(c_id > 0, scan_tmp, S);
    if (tid < (int)kBins) {
      start_v[tid] = first_slot;
      seg_i[tid] = seg_index;
      if (c_id > 0) seg_tmp[0][seg_index] = first_slot;   // first slot of every segment, compact
    }
    if (tid == 0) { start_v[kBins] = L; seg_tmp[0][S] = L; }
    for (int i = tid; i < kSegWaves * (int)kBins / 2; i += kSegThreads) reinterpret_cast<int*>(&hist[0][0])[i] = 0;
    lds_barrier();
    // window of slot s: the slots of its id (binary search over the first slots), in bucketed
    // mode cut to the neighbouring buckets.  Slots are below 2^14, so the bucket index comes
    // exactly from one float multiply: (s + 0.5) / radius is at least 0.5 / radius away from an
    // integer and the rounding error is below 2e-7 s / radius.
    auto window = [&](int s) {
      int lo_i = 0, hi_i = kBins;   // smallest i in (0, kBins] with start_v[i] > s
      while (hi_i - lo_i > 1) {
        const int mid = (lo_i + hi_i) >> 1;
        if (start_v[mid] > s) hi_i = mid; else lo_i = mid;
      }
      int lo = start_v[hi_i - 1], hi = start_v[hi_i];
      if (radius > 0) {
        const int first = (int)(((float)s + 0.5f) * inv_radius) * radius;  // first slot of s's bucket
        lo = max(lo, first - radius);
        hi = min(hi, first + 2 * radius);
      }
      return make_int2(lo, hi);
    };

    // ---- this workgroup's chunk of positions: rank among equal ids, kind lists ----------------
    if (k < K) {
      int code[NBC], rank_w[NBC], g_rank[NBC], p_rank[NBC];
      int g_w = 0, p_w = 0;
#pragma unroll
      for (int j = 0; j < NBC; ++j) {
        const int p = c0 + (wave * NBC + j) * 64 + lane;
        code[j] = p < c1 ? ids[p] : -3;
        const bool local = code[j] >= 0;
        const unsigned dg = local ? (unsigned)code[j] : 0u;
        const unsigned long long same = match_digit(dg, local, varying_bits(dg, local));
        const int before = lanes_before(same);
        int old = 0;
        if (local && before == 0) {  // first lane of a group of equal ids
          old = hist[wave][dg];
          hist[wave][dg] = (unsigned short)(old + __popcll(same));
        }
        old = __shfl(old, local ? __ffsll((long long)same) - 1 : lane, 64);
        rank_w[j] = old + before;
        const unsigned long long mg = __ballot(code[j] == -1), mp = __ballot(code[j] == -2);
        g_rank[j] = g_w + lanes_before(mg);
        p_rank[j] = p_w + lanes_before(mp);
        g_w += __popcll(mg);
        p_w += __popcll(mp);
      }
      if (lane == 0) { wave_tot[1][wave] = g_w; wave_tot[2][wave] = p_w; }
      lds_barrier();
      // (id, wavefront) counts -> tokens with that id before the wavefront's block
      if (tid < (int)kBins) {
        int running = before_h[tid];
#pragma unroll
        for (int w = 0; w < kSegWaves; ++w) {
          const int c = hist[w][tid];
          hist[w][tid] = (unsigned short)running;
          running += c;
        }
      }
      int g_at_c = g_before, p_at_c = p_before;
#pragma unroll
      for (int w = 0; w < kSegWaves; ++w)
        if (w < wave) { g_at_c += wave_tot[1][w]; p_at_c += wave_tot[2][w]; }
      lds_barrier();
#pragma unroll
      for (int j = 0; j < NBC; ++j) {
        const int p = c0 + (wave * NBC + j) * 64 + lane;
        if (p < c1) {
          if (code[j] >= 0) {
            const int slot = start_v[code[j]] + hist[wave][code[j]] + rank_w[j];
            perm[slot] = p;
            seg_of_tok[p] = seg_i[code[j]];
          } else {
            seg_of_tok[p] = -1;
            if (view == 0) {
              if (code[j] == -1) global_idx[g_at_c + g_rank[j]] = p;
              else pad_idx[p_at_c + p_rank[j]] = p;
            }
          }
          // the same index range, read as sorted slots: their windows
          slot_rng[p] = p < L ? window(p) : make_int2(0, 0);
        }
      }
    }
    // ---- per-sequence and per-segment tables (first workgroup) -----------------------------------
    if (k == 0) {
      if (tid < (int)kBins && c_id > 0) seg_off[seg_index] = first_slot;
      if (tid == 0) {
        seg_off[S] = L;
        counts[C_SROW + view] = S;
        counts[5 + view] = s_bad;
        if (view == 0) { counts[C_G] = G; counts[C_L] = L; counts[C_P] = P; }
      }
    }
    if (k != K) return;
    // ---- work units of the attention kernels (the workgroup without a chunk) ---------------------
    // A run is a segment of at least kBigSegment slots, or the shorter segments between two such
    // segments; units are 128-slot pieces of runs (see the general path below for why).
    const int* sstart = seg_tmp[0];
    int* run_start = seg_tmp[1];
    bool cut = false;
    if (tid < S) {
      const int size = sstart[tid + 1] - sstart[tid];
      cut = tid == 0 || size >= kBigSegment || sstart[tid] - sstart[tid - 1] >= kBigSegment;
    }
    int n_runs;
    const int run_index = block_flag_scan(cut, scan_tmp, n_runs);
    if (cut) run_start[run_index] = sstart[tid];
    if (tid == 0) run_start[n_runs] = L;
    lds_barrier();
    const int run_units = tid < n_runs ? (run_start[tid + 1] - run_start[tid] + kTileSlots - 1) / kTileSlots : 0;
    int n_units;
    const int unit_base = block_exclusive_scan(run_units, scan_tmp, n_units);
    if (n_units + n_pt <= lay.units) {
      for (int i = 0; i < run_units; ++i) head_pos[unit_base + i] = (unsigned short)(run_start[tid] + i * kTileSlots);
    } else {  // more records than the buffer has: every 128 slots regardless of segments
      n_units = (L + kTileSlots - 1) / kTileSlots;
      if (tid < n_units) head_pos[tid] = (unsigned short)(tid * kTileSlots);
    }
    lds_barrier();
    int4 r0 = make_int4(UNIT_NONE, 0, 0, 0), r1 = make_int4(0, 0, -1, 0);
    if (tid < n_units) {
      const int t0 = min((int)head_pos[tid], L - 1);
      const int end = min(max(tid + 1 < n_units ? (int)head_pos[tid + 1] : L, t0 + 1), min(L, t0 + kTileSlots));
      const int lo = window(t0).x, hi = window(end - 1).y;
      r0 = make_int4(UNIT_LOCAL, t0, lo, hi);
      r1.y = n_t0 + (hi - lo + BN - 1) / BN;
      r1.w = end;
      unit_len[tid] = (unsigned short)r1.y;
    }
    lds_barrier();
    if (tid < lay.units) {
      int place = tid;
      if (tid < n_units) {   // longest streamed side first, ties in slot order
        place = 0;
        const int mine = r1.y;
#pragma unroll 8
        for (int j = 0; j < n_units; ++j) {
          const int other = unit_len[j];
          place += other > mine || (other == mine && j < tid);
        }
      } else if (tid < n_units + n_pt) {
        r0 = make_int4(UNIT_PAD, (tid - n_units) * kPadSlots, 0, 0);
      }
      unit[2 * place] = r0;
      unit[2 * place + 1] = r1;
    }
    if (view == 0 && tid < lay.tiles) {  // question-token owners (the same for both views)
      const GlobalSplit gs = global_split(G, L, N);
      int4 q0 = make_int4(UNIT_NONE, 0, 0, 0), q1 = make_int4(0, 0, -1, 0);
      if (tid < gs.n_gt * gs.n_chunks) {
        const int gt = tid / gs.n_chunks, c = tid % gs.n_chunks;
        q0 = make_int4(UNIT_GLOBAL, gt * BM, 0, L);
        q1.x = c * gs.per;
        q1.y = min(gs.n_st, q1.x + gs.per);
        if (gs.n_chunks > 1) q1.z = tid;
      }
      gunit[2 * tid] = q0;
      gunit[2 * tid + 1] = q1;
    }
    return;
  }
  if (k != 0) return;   // ids of 512 and more: the first workgroup sorts alone

  // ======================= general path: LSD radix sort in this workgroup =======================
  // ---- compact the three kinds in ascending position order ------------------------------------
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    const int i = w0 + e * 64 + lane;
    const unsigned long long ml = __ballot(my_flag[e] == 0), mg = __ballot(my_flag[e] == 1),
                             mp = __ballot(my_flag[e] == 2);
    if (my_flag[e] == 0) buf_a[l_at + lanes_before(ml)] = (unsigned short)i;
    else if (i < N) seg_of_tok[i] = -1;
    if (view == 0) {
      if (my_flag[e] == 1) global_idx[g_at + lanes_before(mg)] = i;
      if (my_flag[e] == 2) pad_idx[p_at + lanes_before(mp)] = i;
    }
    l_at += __popcll(ml);
    g_at += __popcll(mg);
    p_at += __popcll(mp);
  }
  if (view == 0) {
    // entries past G and P stay unwritten: nothing reads them (the export hook masks them)
    if (tid == 0) { counts[C_G] = G; counts[C_L] = L; counts[C_P] = P; }
  }
  if (tid == 0) counts[5 + view] = s_bad;
  lds_barrier();

  // ---- stable LSD radix sort of buf_a[0..L) by ids[position] --------------------------------
  unsigned short* cur = buf_a;
  unsigned short* nxt = buf_b;
  for (int shift = 0; shift < 32; shift += kDigitBits) {
    if (((all_bits >> shift) & (kBins - 1u)) == 0) continue;  // digit 0 everywhere: order unchanged
    for (int i = tid; i < kSegWaves * kBins / 2; i += kSegThreads) reinterpret_cast<int*>(&hist[0][0])[i] = 0;
    lds_barrier();
    // count digits per wavefront; every element learns its rank among the equal digits of its
    // wavefront's block (batches in order, lanes in order inside a batch)
    int pos[NB], rank_w[NB];
    unsigned dig[NB];
#pragma unroll
    for (int e = 0; e < NB; ++e) {
      const int s = w0 + e * 64 + lane;
      pos[e] = s < L ? cur[s] : 0;
      dig[e] = s < L ? ((unsigned)ids[pos[e]] >> shift) & (kBins - 1u) : 0u;
    }
#pragma unroll
    for (int e = 0; e < NB; ++e) {
      const bool valid = w0 + e * 64 + lane < L;
      const unsigned long long same = match_digit(dig[e], valid, varying_bits(dig[e], valid));
      const int before = lanes_before(same);
      int old = 0;
      if (valid && before == 0) {  // first lane of a group of equal digits
        old = hist[wave][dig[e]];
        hist[wave][dig[e]] = (unsigned short)(old + __popcll(same));
      }
      old = __shfl(old, valid ? __ffsll((long long)same) - 1 : lane, 64);
      rank_w[e] = old + before;
    }
    lds_barrier();
    // counts -> first output slot of (digit, wavefront): digits ascending, wavefronts ascending
    int first[kSegWaves], tot = 0;
    if (tid < kBins) {
#pragma unroll
      for (int w = 0; w < kSegWaves; ++w) first[w] = hist[w][tid];
#pragma unroll
      for (int w = 0; w < kSegWaves; ++w) {
        const int c = first[w];
        first[w] = tot;
        tot += c;
      }
    }
    int all;
    const int digit_base = block_exclusive_scan(tot, scan_tmp, all);
    if (tid < kBins) {
#pragma unroll
      for (int w = 0; w < kSegWaves; ++w) hist[w][tid] = (unsigned short)(first[w] + digit_base);
    }
    lds_barrier();
#pragma unroll
    for (int e = 0; e < NB; ++e)
      if (w0 + e * 64 + lane < L) nxt[hist[wave][dig[e]] + rank_w[e]] = (unsigned short)pos[e];
    lds_barrier();
    unsigned short* t = cur; cur = nxt; nxt = t;
  }

  // ---- run boundaries -> segment index per slot ----------------------------------------------
  unsigned head_bits = 0;  // bit e: my slot of batch e starts a segment
  int my_pos[NB];
  int n_head = 0;
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    const int s = w0 + e * 64 + lane;
    my_pos[e] = s < L ? cur[s] : 0;
    const bool head = s < L && (s == 0 || ids[cur[s - 1]] != ids[my_pos[e]]);
    head_bits |= (unsigned)head << e;
    n_head += __popcll(__ballot(head));
  }
  if (lane == 0) wave_tot[0][wave] = n_head;
  lds_barrier();  // also: every wavefront is done reading ids[]
  int S = 0, seg_at = 0;
#pragma unroll
  for (int w = 0; w < kSegWaves; ++w) {
    const int c = wave_tot[0][w];
    if (w < wave) seg_at += c;
    S += c;
  }
  // ids[] and the spare order buffer are dead now: reuse them
  unsigned short* seg_start = reinterpret_cast<unsigned short*>(ids);  // [P2], entry S (== L) implied
  unsigned short* seg_of_slot = nxt;                                    // [P2]
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    const int s = w0 + e * 64 + lane;
    const bool head = (head_bits >> e) & 1u;
    const unsigned long long mh = __ballot(head);
    const int seg_idx = seg_at + lanes_before(mh) + (head ? 1 : 0) - 1;  // heads up to and including me
    if (s < L) {
      perm[s] = my_pos[e];
      seg_of_tok[my_pos[e]] = seg_idx;
      seg_of_slot[s] = (unsigned short)seg_idx;
      if (head) { seg_start[seg_idx] = (unsigned short)s; seg_off[seg_idx] = s; }
    }  // perm past L, like seg_off past S, stays unwritten (masked by the export hook)
    seg_at += __popcll(mh);
  }
  if (tid == 0) { seg_off[S] = L; counts[C_SROW + view] = S; }
  lds_barrier();
  // window of slot s: its segment, in bucketed mode cut to the neighbouring buckets.  Slots are
  // below 2^14, so the bucket index comes exactly from one float multiply: (s + 0.5) / radius is
  // at least 0.5 / radius away from an integer and the rounding error is below 2e-7 s / radius.
  auto window = [&](int s) {
    const int g = seg_of_slot[s];
    int lo = seg_start[g], hi = g + 1 < S ? (int)seg_start[g + 1] : L;
    if (radius > 0) {
      const int first = (int)(((float)s + 0.5f) * inv_radius) * radius;  // first slot of s's bucket
      lo = max(lo, first - radius);
      hi = min(hi, first + 2 * radius);
    }
    return make_int2(lo, hi);
  };
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    const int s = w0 + e * 64 + lane;
    if (s < N) slot_rng[s] = s < L ? window(s) : make_int2(0, 0);
  }

  // ---- work units of the attention kernels -------------------------------------------------
  // Table-token owners: up to 128 consecutive sorted slots each, streaming the question tokens
  // and then the slot window spanned by the segments those slots touch; pad owners after them.
  // A segment of at least kBigSegment slots starts a unit of its own ("cut"), and so does the
  // first slot after it, so no unit straddles the boundary of a long segment; if that would
  // need more records than the buffer has, the slots are cut every 128 regardless.
  auto seg_size = [&](int g) { return (g + 1 < S ? (int)seg_start[g + 1] : L) - (int)seg_start[g]; };
  unsigned cut_bits = 0;  // bit e: my slot of batch e is a cut
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    const int s = w0 + e * 64 + lane;
    bool cut = false;
    if (s < L) {
      const int g = seg_of_slot[s];
      cut = s == (int)seg_start[g] &&
            (g == 0 || seg_size(g) >= kBigSegment || seg_size(g - 1) >= kBigSegment);
    }
    cut_bits |= (unsigned)cut << e;
  }
  int n_units = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {  // 0: with cuts; 1: every 128 slots (rare)
    const bool use_cuts = attempt == 0;
    // last cut inside each wavefront's block -> the cut in force at the start of the next ones
    int last = -1;
#pragma unroll
    for (int e = 0; e < NB; ++e) {
      const unsigned long long m = __ballot(use_cuts && ((cut_bits >> e) & 1u));
      if (m) last = w0 + e * 64 + 63 - __clzll((long long)m);
    }
    if (lane == 0) wave_tot[1][wave] = last;
    lds_barrier();
    int running = 0;
#pragma unroll
    for (int w = 0; w < kSegWaves; ++w)
      if (w < wave) running = max(running, wave_tot[1][w]);
    unsigned hbits = 0;  // bit e: my slot of batch e starts a unit
    int n_head_w = 0;
#pragma unroll
    for (int e = 0; e < NB; ++e) {
      const int s = w0 + e * 64 + lane;
      const unsigned long long m = __ballot(use_cuts && ((cut_bits >> e) & 1u));
      const unsigned long long upto = m & (~0ull >> (63 - lane));  // cuts at lanes <= mine
      const int base = upto ? w0 + e * 64 + 63 - __clzll((long long)upto) : running;
      const bool head = s < L && ((s - base) & (kTileSlots - 1)) == 0;
      hbits |= (unsigned)head << e;
      n_head_w += __popcll(__ballot(head));
      if (m) running = w0 + e * 64 + 63 - __clzll((long long)m);
    }
    if (lane == 0) wave_tot[0][wave] = n_head_w;
    lds_barrier();
    int head_at = 0;
    n_units = 0;
#pragma unroll
    for (int w = 0; w < kSegWaves; ++w) {
      const int c = wave_tot[0][w];
      if (w < wave) head_at += c;
      n_units += c;
    }
    const bool fits = n_units + n_pt <= lay.units;  // always true without cuts
    if (fits) {
#pragma unroll
      for (int e = 0; e < NB; ++e) {
        const bool head = (hbits >> e) & 1u;
        const unsigned long long mh = __ballot(head);
        if (head) head_pos[head_at + lanes_before(mh)] = (unsigned short)(w0 + e * 64 + lane);
        head_at += __popcll(mh);
      }
    }
    lds_barrier();  // head_pos is complete; wave_tot may be written again
    if (fits) break;
  }
  // streamed length of every unit, then its place in the list: longest first (ties in slot
  // order), so that across a launch the long units start first and the short ones fill the end
  int4 r0 = make_int4(UNIT_NONE, 0, 0, 0), r1 = make_int4(0, 0, -1, 0);
  if (tid < n_units) {
    // (clamped so that a record can never name a slot outside [0, L), whatever else goes wrong)
    const int t0 = min((int)head_pos[tid], L - 1);
    const int end = min(max(tid + 1 < n_units ? (int)head_pos[tid + 1] : L, t0 + 1), min(L, t0 + kTileSlots));
    const int lo = window(t0).x, hi = window(end - 1).y;
    r0 = make_int4(UNIT_LOCAL, t0, lo, hi);
    r1.y = n_t0 + (hi - lo + BN - 1) / BN;
    r1.w = end;
    unit_len[tid] = (unsigned short)r1.y;
  }
  lds_barrier();
  if (tid < lay.units) {
    int place = tid;
    if (tid < n_units) {
      place = 0;
      const int mine = r1.y;
      for (int j = 0; j < n_units; ++j) {
        const int other = unit_len[j];
        place += other > mine || (other == mine && j < tid);
      }
    } else if (tid < n_units + n_pt) {
      r0 = make_int4(UNIT_PAD, (tid - n_units) * kPadSlots, 0, 0);
    }
    unit[2 * place] = r0;
    unit[2 * place + 1] = r1;
  }
  // question-token owners (the same for both views; written by the row view's workgroup)
  if (view == 0 && tid < lay.tiles) {
    const GlobalSplit gs = global_split(G, L, N);
    int4 r0 = make_int4(UNIT_NONE, 0, 0, 0), r1 = make_int4(0, 0, -1, 0);
    if (tid < gs.n_gt * gs.n_chunks) {
      const int gt = tid / gs.n_chunks, c = tid % gs.n_chunks;
      r0 = make_int4(UNIT_GLOBAL, gt * BM, 0, L);
      r1.x = c * gs.per;
      r1.y = min(gs.n_st, r1.x + gs.per);
      if (gs.n_chunks > 1) r1.z = tid;
    }
    gunit[2 * tid] = r0;
    gunit[2 * tid + 1] = r1;
  }
}

hipError_t launch_build_segments(const int* row_ids, const int* col_ids,
                                 const unsigned char* flags, int B, int N, int max_global,
                                 int radius, int* seg, hipStream_t stream) {
  // up to eight workgroups per (sequence, view) with at least 1024 positions each, and with more
  // than one of them a further one for the work-unit list
  const int chunks = std::min(8, (N + kSegThreads - 1) / kSegThreads);
  dim3 grid(B, 2, chunks > 1 ? chunks + 1 : 1), block(kSegThreads);
  ProfileScope prof(1, stream);
#define MATE_SEG_CASE(P2)                                                                  \
  if (N <= P2) {                                                                            \
    hipLaunchKernelGGL(build_segments_kernel<P2>, grid, block, 0, stream, row_ids, col_ids, \
                       flags, B, N, max_global, radius, seg);                               \
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
