// Step 2 of the paper's Sec. 3.2.1 read literally: the candidate set T_rho of a window is made of the k lowest-FD EDGES
// of the complete bipartite graph between its node sets A and B -- not one edge per A node.  An A node then owns as
// many edges as rank that low (it is averaged into each of those B nodes with its full weight, Eq. "message-passing"
// with several ones in a row of M) and leaves if it owns at least one, so the number of tokens that go depends on
// the data: between ceil(k / |B|) and min(k, |A|) per window.
//
//   edge_select_kernel : one workgroup per window.  Reads the partial inner-product tiles that fd_partial_kernel left
//                        (lk_score_fd.hip), forms FD of every (a, b) pair into LDS as an order-preserving integer key,
//                        finds the k-th smallest key by a 4-pass radix select (8 bits per pass, LDS histogram; integer
//                        counts, so the result does not depend on the order of the atomics), breaks a tie AT the
//                        threshold by (A position, B position), and writes
//                          dst[a]      the B token of a's lowest selected edge, -1 if a stays
//                          src_rank[a] position of a among the sources of that B token
//                          cnt[b]      number of selected edges into b
//                          best_fd / best_dst  of every A node, as the default selection reports them
//                        plus the window's edge list (a, b, position of a among b's sources) at a fixed offset
//                        (the k of the windows before it) for edge_fill_kernel; every window writes all of its slots.
//   select_scan_kernel : unchanged (lk_select.hip): new_index from dst, grp_offsets from cnt.
//   edge_fill_kernel   : grp_src[grp_offsets[b] + position] = a for every edge.
//
// Windows of more than 2 * EDGE_MAX_SIDE tokens (up to the library's 4096) do not fit that kernel's LDS; for them
//   edge_keys_kernel       : one workgroup per 32 x 32 partial tile: FD of its pairs as order-preserving keys into a
//                            |A| x |B| matrix per window in the workspace (row-major, pitch |B|)
//   edge_select_big_kernel : one workgroup of 1024 threads per window works on that matrix: the k-th smallest of the
//                            composite keys (FD key, pair index) by a radix select of 11 + 11 + 10 bits over the FD key
//                            and, only if the threshold value is shared by more pairs than are still wanted, 11 + 11 bits
//                            over the pair index (row-major, so a tie at the threshold goes by (A position, B position)
//                            exactly as in the small kernel, without an ordered pass); then one pass by rows (best edge
//                            and lowest selected edge of every A node) and one by columns (sources of every B node, edge
//                            list).  The slots of the edge list are handed out by an LDS counter: the list is scratch,
//                            and what edge_fill_kernel makes of it does not depend on the slot order.
// The passes re-read the matrix from L2 / memory; one workgroup per window keeps this simple and is adequate for
// the 300- to 600-token windows of the coarse stages (a 2880-token window takes a few hundred microseconds).
#include <atomic>
#include "lk_fd_body.h"

namespace lk {

constexpr int EDGE_THREADS = 256;
constexpr int EDGE_WAVES = EDGE_THREADS / 64;
constexpr int EDGE_UNROLL = 4;
constexpr int EDGE_ITEMS = EDGE_MAX_SIDE * EDGE_MAX_SIDE / EDGE_THREADS;   // keys per thread, at most

struct EdgeArgs {
  const int32_t *win_remove;   // k per window
  int32_t *dst, *cnt, *src_rank;
  int32_t *edges;              // [3][sum_k]: A token, B token, position among the B token's sources
  int sum_k;                   // slots of the edge list
  int key_capacity;            // 32-bit keys the launch reserved LDS for
  int clamp_v;                 // counts come from the device alone: a window's k is also bounded by its tokens, so that
                               // sum_k = the tokens of the batch always suffices
  uint32_t *big_keys;          // large windows: [n_windows][big_stride] FD keys
  size_t big_stride;
  int max_a, max_b;            // the caller's bound on the sides of a window
};

// The k a window really gets: what was asked, at most its pairs (and its tokens, see clamp_v).
__device__ __forceinline__ int edge_count(int k_asked, int nA, int nB, int clamp_v) {
  int k = k_asked < 0 ? 0 : k_asked;
  const int E = nA * nB;
  k = k > E ? E : k;
  if (clamp_v && k > nA + nB) k = nA + nB;
  return k;
}
// Slots of the windows before window w.
__device__ __forceinline__ int edge_slots_before(const FdArgs &g, const EdgeArgs &q, int w, int first, int step) {
  int before = 0;
  for (int i = first; i < w; i += step) {
    const int v = g.win_offsets[i + 1] - g.win_offsets[i];
    before += edge_count(q.win_remove[i], side_a(v, 0), side_b(v, 0), q.clamp_v);
  }
  return before;
}

// Workgroup-wide sum of one int per thread; every thread gets the total.
__device__ __forceinline__ int edge_block_sum(int v, int *wsum) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();   // wsum may still be read from the call before
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int w = 0; w < EDGE_WAVES; ++w) t += wsum[w];
  return t;
}

// Sum of the KS slices of one partial sum, in slice order (fp64), all loads issued together.
template <int KS>
__device__ __forceinline__ double edge_sum_slices(const float *p, int64_t ks_stride) {
  float v[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) v[ks] = p[ks * ks_stride];
  double s = 0.0;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) s += (double)v[ks];
  return s;
}

// KS: slices of the hidden axis the partial tiles were computed in (g.ksplit)
template <int KS>
__global__ __launch_bounds__(EDGE_THREADS) void edge_select_kernel(FdArgs g, EdgeArgs q) {
  extern __shared__ uint32_t keys[];   // [nA][pitch]
  __shared__ double na2[EDGE_MAX_SIDE], nb2[EDGE_MAX_SIDE];
  __shared__ int hist[256];
  __shared__ int col_cnt[EDGE_MAX_SIDE], col_start[EDGE_MAX_SIDE];
  __shared__ int wsum[EDGE_WAVES];
  __shared__ int pick[2];
  __shared__ int tok[2 * EDGE_MAX_SIDE];   // the window's tokens (checked), in list order: a token lookup inside a loop
                                           // must not be a trip to global memory
  const int w = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const WinInfo wi = win_info(g, w);
  const int nA = wi.nA, nB = wi.nB;
  // the host refuses such windows, and sizes the LDS from its own bound on the window: a device-side list that breaks
  // either is left alone
  if (nA > EDGE_MAX_SIDE || nB > EDGE_MAX_SIDE || nA * (nB | 1) > q.key_capacity) return;
  const int E = nA * nB;
  const int k = edge_count(q.win_remove[w], nA, nB, q.clamp_v);

  for (int i = tid; i < nA + nB; i += EDGE_THREADS) tok[i] = checked_token(g, wi.off + i);
  // slots of this window in the edge list: the k of the windows before it (the barriers inside also publish tok[]).
  // Slots no window uses (the list is sized from an upper bound) were marked empty by the launcher's fill.
  const int edge_base = edge_block_sum(edge_slots_before(g, q, w, tid, EDGE_THREADS), wsum);
  if (nB == 0) {   // a window of one token (or none): no pair, nothing leaves
    for (int i = tid; i < nA; i += EDGE_THREADS) {
      const int t = tok[i];
      if (t >= 0) {
        q.dst[t] = -1; q.cnt[t] = 0; q.src_rank[t] = 0;
        g.best_fd[t] = __uint_as_float(0x7f800000u);
        g.best_dst[t] = -1;
      }
    }
    return;
  }

  // ---- where the sums of pair (la, lb) lie in the partial tiles
  const int64_t ks_stride = (int64_t)g.n_tiles * FD_TILE_FLOATS;
  const int per = g.mt * g.nt;
  const int grp_s = (g.group > 1) ? w % g.group : 0;
  const int row_shift = grp_s * g.slot;                 // rows and columns of this window inside a packed tile
  const int tile0 = (g.group > 1) ? w / g.group : w * per;
  auto tile_of = [&](int la, int lb) { return (g.group > 1) ? tile0 : tile0 + (la >> 5) * g.nt + (lb >> 5); };
  for (int i = tid; i < nA + nB; i += EDGE_THREADS) {
    if (i < nA) {
      const int r = (g.group > 1) ? row_shift + i : (i & 31);
      na2[i] = edge_sum_slices<KS>(g.partial + (int64_t)tile_of(i, 0) * FD_TILE_FLOATS + 32 * 32 + r, ks_stride);
    } else {
      const int lb = i - nA;
      const int c = (g.group > 1) ? row_shift + lb : (lb & 31);
      nb2[lb] = edge_sum_slices<KS>(g.partial + (int64_t)tile_of(0, lb) * FD_TILE_FLOATS + 32 * 32 + 32 + c, ks_stride);
    }
  }
  __syncthreads();

  // ---- FD of every pair -> order-preserving key in LDS.  EDGE_UNROLL pairs per thread and round: the loads of all
  // of them (every slice) are issued before the first is used; a round is one trip to memory, so this loop is as long
  // as its number of rounds
  const int pitch = nB | 1;   // odd: a thread per row and a thread per column both walk the array without bank conflicts
  // pair index -> (A position, B position) without a division per pair: a step of EDGE_THREADS pairs moves the position
  // by (step_a, step_b) with at most one carry
  const int step_a = EDGE_THREADS / nB, step_b = EDGE_THREADS - step_a * nB;
  const int la0 = tid / nB, lb0 = tid - la0 * nB;   // this thread's first pair
  {
    int la_n = la0, lb_n = lb0;
    for (int e0 = tid; e0 < E; e0 += EDGE_THREADS * EDGE_UNROLL) {
      double dot[EDGE_UNROLL];
      int la[EDGE_UNROLL], lb[EDGE_UNROLL];
#pragma unroll
      for (int u = 0; u < EDGE_UNROLL; ++u) {
        const bool ok = e0 + u * EDGE_THREADS < E;
        la[u] = ok ? la_n : nA - 1;   // surplus pairs re-read the last one and are dropped
        lb[u] = ok ? lb_n : nB - 1;
        lb_n += step_b; la_n += step_a;
        if (lb_n >= nB) { lb_n -= nB; ++la_n; }
        const int r = (g.group > 1) ? row_shift + la[u] : (la[u] & 31);
        const int c = (g.group > 1) ? row_shift + lb[u] : (lb[u] & 31);
        dot[u] = edge_sum_slices<KS>(g.partial + (int64_t)tile_of(la[u], lb[u]) * FD_TILE_FLOATS + r * 32 + c, ks_stride);
      }
#pragma unroll
      for (int u = 0; u < EDGE_UNROLL; ++u) {
        float f = (float)divergence(g.metric, dot[u], na2[la[u]], nb2[lb[u]]);
        if (!(f >= 0.f)) f = __uint_as_float(0x7f800000u);   // NaN ranks last, like +inf
        if (e0 + u * EDGE_THREADS < E) keys[la[u] * pitch + lb[u]] = f32_order_key(f);
      }
    }
  }
  __syncthreads();

  // ---- every thread takes its keys into registers (pair e = it * EDGE_THREADS + tid): the passes below then touch
  // LDS for the histogram only
  uint32_t kreg[EDGE_ITEMS];
  {
    int la = la0, lb = lb0;
#pragma unroll
    for (int it = 0; it < EDGE_ITEMS; ++it) {
      if (it * EDGE_THREADS >= E) break;   // uniform over the workgroup
      kreg[it] = (it * EDGE_THREADS + tid < E) ? keys[la * pitch + lb] : 0u;
      lb += step_b; la += step_a;
      if (lb >= nB) { lb -= nB; ++la; }
    }
  }

  // ---- k-th smallest key: radix select, most significant byte first
  uint32_t prefix = 0, mask = 0;
  int remaining = k;   // how many of the keys that match the prefix so far are wanted
  int n_equal = 0;     // keys equal to the threshold (after the last pass)
  static_assert(EDGE_THREADS == 256 && EDGE_MAX_SIDE == 128, "one thread per histogram bin; a half of the workgroup per node set");
  for (int shift = 24; k > 0 && shift >= 0; shift -= 8) {   // k is uniform over the workgroup
    hist[tid] = 0;
    __syncthreads();
    // FD lies in [0, 2], so most keys share their leading bytes and plain atomics would queue on one LDS word: a thread
    // adds a run of equal digits once
    int run_digit = -1, run = 0;
#pragma unroll
    for (int it = 0; it < EDGE_ITEMS; ++it) {
      if (it * EDGE_THREADS >= E) break;
      const uint32_t key = kreg[it];
      const bool in = it * EDGE_THREADS + tid < E && (key & mask) == prefix;
      const int digit = in ? (int)((key >> shift) & 255u) : run_digit;
      if (digit != run_digit) {
        if (run > 0) atomicAdd(&hist[run_digit], run);
        run_digit = digit;
        run = 0;
      }
      run += in ? 1 : 0;
    }
    if (run > 0) atomicAdd(&hist[run_digit], run);
    __syncthreads();
    // inclusive scan of the 256 bins, one per thread
    const int h = hist[tid];
    int inc = h;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    for (int w2 = 0; w2 < wave; ++w2) inc += wsum[w2];
    const int exc = inc - h;
    if (exc < remaining && remaining <= inc) { pick[0] = tid; pick[1] = remaining - exc; }   // exactly one bin
    __syncthreads();
    prefix |= (uint32_t)pick[0] << shift;
    mask |= 255u << shift;
    remaining = pick[1];
    n_equal = hist[pick[0]];
    __syncthreads();
  }
  // k == 0: no key is selected (a flag rather than a sentinel threshold)
  const bool any = k > 0;
  const uint32_t threshold = prefix;
  // `remaining` of the n_equal keys AT the threshold are wanted: the first ones in (A position, B position) order.
  // The others are pushed past every real key (the largest real key is that of +inf), so that afterwards
  // "selected" simply means key <= threshold.
  if (any && remaining < n_equal) {
    int base = 0;
    int la = la0, lb = lb0;
#pragma unroll
    for (int it = 0; it < EDGE_ITEMS; ++it) {
      if (it * EDGE_THREADS >= E) break;
      const bool eq = it * EDGE_THREADS + tid < E && kreg[it] == threshold;
      const unsigned long long bal = __ballot(eq);
      const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
      __syncthreads();
      if (lane == 0) wsum[wave] = __popcll(bal);
      __syncthreads();
      int before_me = base + in_wave, all = 0;
#pragma unroll
      for (int w2 = 0; w2 < EDGE_WAVES; ++w2) {
        before_me += (w2 < wave) ? wsum[w2] : 0;
        all += wsum[w2];
      }
      if (eq && before_me >= remaining) {
        kreg[it] = 0xffffffffu;
        keys[la * pitch + lb] = 0xffffffffu;
      }
      base += all;
      lb += step_b; la += step_a;
      if (lb >= nB) { lb -= nB; ++la; }
    }
  }
  // ---- per B node: number of selected edges (every thread adds those among its own keys)
  if (tid < EDGE_MAX_SIDE) col_cnt[tid] = 0;
  __syncthreads();   // also publishes the keys changed above
  if (any) {
    int lb = lb0;   // only the column of a pair matters here
#pragma unroll
    for (int it = 0; it < EDGE_ITEMS; ++it) {
      if (it * EDGE_THREADS >= E) break;
      if (it * EDGE_THREADS + tid < E && kreg[it] <= threshold) atomicAdd(&col_cnt[lb], 1);
      lb += step_b;
      if (lb >= nB) lb -= nB;
    }
  }
  __syncthreads();

  // ---- slots of every B node's edges inside the window's edge list
  const int my_cnt = tid < nB ? col_cnt[tid] : 0;
  if (tid < 64) {   // exclusive prefix over at most 128 columns: two per lane
    const int c0 = col_cnt[2 * tid], c1 = col_cnt[2 * tid + 1];
    int inc = c0 + c1;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    col_start[2 * tid] = inc - c0 - c1;
    col_start[2 * tid + 1] = inc - c1;
  }
  __syncthreads();
  if (tid < nB) {
    const int b_tok = tok[2 * tid + 1];
    if (b_tok >= 0) {
      q.dst[b_tok] = -1; q.cnt[b_tok] = my_cnt; q.src_rank[b_tok] = 0;
      g.best_fd[b_tok] = __uint_as_float(0x7f800000u);
      g.best_dst[b_tok] = -1;
    }
    int pos = 0;
    for (int la = 0; la < nA; ++la) {
      if (any && keys[la * pitch + tid] <= threshold) {
        const int slot = edge_base + col_start[tid] + pos;
        if (slot < q.sum_k) {
          q.edges[slot] = tok[2 * la];
          q.edges[q.sum_k + slot] = b_tok;
          q.edges[2 * q.sum_k + slot] = pos;
        }
        ++pos;
      }
    }
  }
  // ---- per A node (the upper half of the workgroup): lowest selected edge, and the best edge whether selected or not
  if (tid >= EDGE_MAX_SIDE && tid - EDGE_MAX_SIDE < nA) {
    const int la = tid - EDGE_MAX_SIDE;
    uint32_t best = 0xffffffffu, best_sel = 0xffffffffu;
    int best_c = -1, sel_c = -1;
    for (int lb = 0; lb < nB; ++lb) {
      const uint32_t key = keys[la * pitch + lb];
      // a key pushed past the threshold above was equal to it before
      const uint32_t real = key == 0xffffffffu ? threshold : key;
      if (real < best) { best = real; best_c = lb; }            // columns ascend: strict < keeps the first minimum
      if (any && key <= threshold && key < best_sel) { best_sel = key; sel_c = lb; }
    }
    int rank = 0;
    if (sel_c >= 0)
      for (int l2 = 0; l2 < la; ++l2) rank += keys[l2 * pitch + sel_c] <= threshold ? 1 : 0;   // sel_c >= 0 implies any
    const int a_tok = tok[2 * la];
    if (a_tok >= 0) {
      q.dst[a_tok] = sel_c >= 0 ? tok[2 * sel_c + 1] : -1;
      q.src_rank[a_tok] = rank;
      q.cnt[a_tok] = 0;
      // order key back to the float it came from
      const uint32_t u = (best & 0x80000000u) ? (best & 0x7fffffffu) : ~best;
      g.best_fd[a_tok] = __uint_as_float(u);
      g.best_dst[a_tok] = best_c >= 0 ? tok[2 * best_c + 1] : -1;
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------------
// Large windows: FD keys of every pair in a matrix per window (global memory), selection by one workgroup per window.
constexpr int EB_THREADS = 1024;
constexpr int EB_WAVES = EB_THREADS / 64;
constexpr int EB_MAX_SIDE = 2048;   // |A| and |B| of the library's largest window
constexpr int EB_BINS = 2048;       // 11-bit digits

// One workgroup per 32 x 32 partial tile of fd_partial_kernel (one window per tile: group == 1).
template <int KS>
__global__ __launch_bounds__(256) void edge_keys_kernel(FdArgs g, EdgeArgs q) {
  __shared__ double na2[32], nb2[32];
  __shared__ int rtok[64];
  const int per = g.mt * g.nt;
  const int tile = blockIdx.x, tid = threadIdx.x;
  const int w = tile / per, rem = tile - w * per, mt = rem / g.nt, nt = rem - mt * g.nt;
  const WinInfo wi = win_info(g, w);
  const int row0 = mt * 32, col0 = nt * 32;
  if (row0 >= wi.nA || col0 >= wi.nB || wi.nA > q.max_a || wi.nB > q.max_b) return;   // uniform
  const int64_t ks_stride = (int64_t)g.n_tiles * FD_TILE_FLOATS;
  const float *base = g.partial + (int64_t)tile * FD_TILE_FLOATS;
  if (tid < 64) {
    // |a|^2 was accumulated by the first tile of this row of tiles, |b|^2 by the first tile of this column of tiles
    const int i = tid & 31;
    if (tid < 32) na2[i] = edge_sum_slices<KS>(g.partial + (int64_t)(w * per + mt * g.nt) * FD_TILE_FLOATS + 32 * 32 + i, ks_stride);
    else nb2[i] = edge_sum_slices<KS>(g.partial + (int64_t)(w * per + nt) * FD_TILE_FLOATS + 32 * 32 + 32 + i, ks_stride);
    rtok[tid] = reinterpret_cast<const int32_t *>(base + FD_TOK_OFFSET)[tid];   // tokens of the 32 rows, then of the 32 columns
  }
  __syncthreads();
  uint32_t *M = q.big_keys + (size_t)w * q.big_stride;
  const int pitch = wi.nB;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int e = u * 256 + tid, r = e >> 5, c = e & 31;
    const int la = row0 + r, lb = col0 + c;
    const double dot = edge_sum_slices<KS>(base + e, ks_stride);
    float f = (float)divergence(g.metric, dot, na2[r], nb2[c]);
    if (!(f >= 0.f) || rtok[r] < 0 || rtok[32 + c] < 0) f = __uint_as_float(0x7f800000u);   // NaN ranks last, like +inf
    if (la < wi.nA && lb < wi.nB) M[(size_t)la * pitch + lb] = f32_order_key(f);
  }
}

constexpr int EB_LOADS = 16;   // keys a thread keeps in flight per step of the radix and column passes
constexpr int EB_ROWS = 4;     // rows a wave takes at a time in the row pass
__global__ __launch_bounds__(EB_THREADS) void edge_select_big_kernel(FdArgs g, EdgeArgs q) {
  __shared__ int hist[EB_BINS];
  __shared__ int tok[2 * EB_MAX_SIDE];
  __shared__ uint16_t selcol[EB_MAX_SIDE];   // lowest selected edge of every A node (0xffff: none)
  __shared__ int wsum[EB_WAVES];
  __shared__ int pick[3];
  __shared__ int slot_counter;
  const int w = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const WinInfo wi = win_info(g, w);
  const int nA = wi.nA, nB = wi.nB;
  if (nA > q.max_a || nB > q.max_b || nA > EB_MAX_SIDE || nB > EB_MAX_SIDE) return;   // refused by the host; left alone
  const int E = nA * nB;
  const int k = edge_count(q.win_remove[w], nA, nB, q.clamp_v);
  for (int i = tid; i < nA + nB; i += EB_THREADS) tok[i] = checked_token(g, wi.off + i);
  if (tid == 0) slot_counter = 0;
  // slots of this window in the edge list (the barriers inside also publish tok[] and the counter)
  int before = edge_slots_before(g, q, w, tid, EB_THREADS);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) before += __shfl_xor(before, o, 64);
  if (lane == 0) wsum[wave] = before;
  __syncthreads();
  int edge_base = 0;
#pragma unroll
  for (int i = 0; i < EB_WAVES; ++i) edge_base += wsum[i];
  __syncthreads();
  if (nB == 0) {   // a window of one token (or none): no pair, nothing leaves
    for (int i = tid; i < nA; i += EB_THREADS) {
      const int t = tok[i];
      if (t >= 0) {
        q.dst[t] = -1; q.cnt[t] = 0; q.src_rank[t] = 0;
        g.best_fd[t] = __uint_as_float(0x7f800000u);
        g.best_dst[t] = -1;
      }
    }
    return;
  }
  const uint32_t *M = q.big_keys + (size_t)w * q.big_stride;

  // ---- the k-th smallest composite key (FD key, pair index): radix select, most significant digit first.
  // Passes 0..2 take the FD key (11, 11, 10 bits), passes 3..4 the pair index (11, 11 bits: E <= 2^22).
  uint32_t kprefix = 0, kmask = 0, eprefix = 0, emask = 0;
  int remaining = k, n_equal = 0;
  for (int pass = 0; pass < 5 && k > 0; ++pass) {   // uniform
    if (pass == 3 && remaining == n_equal) break;   // every pair at the threshold value is wanted: no tie to break
    for (int i = tid; i < EB_BINS; i += EB_THREADS) hist[i] = 0;
    __syncthreads();
    int run_digit = -1, run = 0;   // FD lies in a narrow range: a thread adds a run of equal digits once
    for (int e0 = tid; e0 < E; e0 += EB_LOADS * EB_THREADS) {
      uint32_t key[EB_LOADS];
#pragma unroll
      for (int u = 0; u < EB_LOADS; ++u) { const int e = e0 + u * EB_THREADS; key[u] = M[e < E ? e : E - 1]; }
#pragma unroll
      for (int u = 0; u < EB_LOADS; ++u) {
        const uint32_t e = (uint32_t)(e0 + u * EB_THREADS);
        const bool in = e < (uint32_t)E && (key[u] & kmask) == kprefix && (e & emask) == eprefix;
        int digit;
        if (pass == 0) digit = (int)(key[u] >> 21);
        else if (pass == 1) digit = (int)((key[u] >> 10) & 2047u);
        else if (pass == 2) digit = (int)(key[u] & 1023u);
        else if (pass == 3) digit = (int)((e >> 11) & 2047u);
        else digit = (int)(e & 2047u);
        digit = in ? digit : run_digit;
        if (digit != run_digit) {
          if (run > 0) atomicAdd(&hist[run_digit], run);
          run_digit = digit;
          run = 0;
        }
        run += in ? 1 : 0;
      }
    }
    if (run > 0) atomicAdd(&hist[run_digit], run);
    __syncthreads();
    // the bin that holds the remaining-th key: inclusive scan over the bins, two per thread
    const int h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
    int inc = h0 + h1;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    for (int w2 = 0; w2 < wave; ++w2) inc += wsum[w2];
    const int exc = inc - h0 - h1;
    if (exc < remaining && remaining <= exc + h0) { pick[0] = 2 * tid; pick[1] = remaining - exc; pick[2] = h0; }              // exactly one bin
    else if (exc + h0 < remaining && remaining <= inc) { pick[0] = 2 * tid + 1; pick[1] = remaining - exc - h0; pick[2] = h1; }
    __syncthreads();
    const uint32_t digit = (uint32_t)pick[0];
    if (pass == 0) { kprefix |= digit << 21; kmask |= 2047u << 21; }
    else if (pass == 1) { kprefix |= digit << 10; kmask |= 2047u << 10; }
    else if (pass == 2) { kprefix |= digit; kmask |= 1023u; }
    else if (pass == 3) { eprefix |= digit << 11; emask |= 2047u << 11; }
    else { eprefix |= digit; emask |= 2047u; }
    remaining = pick[1];
    n_equal = pick[2];
    __syncthreads();
  }
  const bool any = k > 0;
  const uint32_t T = kprefix;
  const uint32_t Te = emask ? eprefix : 0xffffffffu;   // at the threshold value: the pairs up to this index are taken
  auto selected = [&](uint32_t key, uint32_t e) { return any && (key < T || (key == T && e <= Te)); };

  // ---- by rows: best edge and lowest selected edge of every A node (a wave takes EB_ROWS rows at a time, so that
  // their loads are in flight together; lanes stride the columns)
  for (int la0 = wave * EB_ROWS; la0 < nA; la0 += EB_WAVES * EB_ROWS) {
    unsigned long long best_r[EB_ROWS], best_sel_r[EB_ROWS];   // (key << 32 | column): the minimum is the first minimum
#pragma unroll
    for (int r = 0; r < EB_ROWS; ++r) { best_r[r] = ~0ull; best_sel_r[r] = ~0ull; }
    for (int lb0 = lane; lb0 < nB; lb0 += 4 * 64) {
      uint32_t key[EB_ROWS][4];
#pragma unroll
      for (int r = 0; r < EB_ROWS; ++r) {
        const uint32_t *row = M + (size_t)(la0 + r < nA ? la0 + r : nA - 1) * nB;
#pragma unroll
        for (int u = 0; u < 4; ++u) { const int lb = lb0 + u * 64; key[r][u] = row[lb < nB ? lb : nB - 1]; }
      }
#pragma unroll
      for (int r = 0; r < EB_ROWS; ++r) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int lb = lb0 + u * 64;
          if (lb < nB && la0 + r < nA) {
            const unsigned long long c = ((unsigned long long)key[r][u] << 32) | (unsigned)lb;
            best_r[r] = c < best_r[r] ? c : best_r[r];
            if (selected(key[r][u], (uint32_t)((la0 + r) * nB + lb))) best_sel_r[r] = c < best_sel_r[r] ? c : best_sel_r[r];
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < EB_ROWS; ++r) {
      unsigned long long best = best_r[r], best_sel = best_sel_r[r];
      const int la = la0 + r;
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        const unsigned long long ob = __shfl_xor(best, o, 64), os = __shfl_xor(best_sel, o, 64);
        best = ob < best ? ob : best;
        best_sel = os < best_sel ? os : best_sel;
      }
      if (lane == 0 && la < nA) {
        const int sel_c = best_sel == ~0ull ? -1 : (int)(best_sel & 0xffffffffu);
        selcol[la] = sel_c < 0 ? (uint16_t)0xffffu : (uint16_t)sel_c;
        const int a_tok = tok[2 * la];
        if (a_tok >= 0) {
          const uint32_t bk = (uint32_t)(best >> 32);
          const uint32_t u = (bk & 0x80000000u) ? (bk & 0x7fffffffu) : ~bk;   // order key back to the float it came from
          g.best_fd[a_tok] = __uint_as_float(u);
          g.best_dst[a_tok] = tok[2 * (int)(best & 0xffffffffu) + 1];
          q.dst[a_tok] = sel_c >= 0 ? tok[2 * sel_c + 1] : -1;
          q.cnt[a_tok] = 0;
          if (sel_c < 0) q.src_rank[a_tok] = 0;   // (a node that leaves gets its rank from the column pass below)
        }
      }
    }
  }
  __syncthreads();
  // ---- by columns: the sources of every B node in ascending A position, edge list, rank of every leaving A node
  for (int lb = tid; lb < nB; lb += EB_THREADS) {
    const int b_tok = tok[2 * lb + 1];
    int pos = 0;
    for (int la0 = 0; la0 < nA; la0 += EB_LOADS) {
      uint32_t key[EB_LOADS];
#pragma unroll
      for (int u = 0; u < EB_LOADS; ++u) { const int la = la0 + u; key[u] = M[(size_t)(la < nA ? la : nA - 1) * nB + lb]; }
#pragma unroll
      for (int u = 0; u < EB_LOADS; ++u) {
        const int la = la0 + u;
        if (la < nA && selected(key[u], (uint32_t)(la * nB + lb))) {
          const int a_tok = tok[2 * la];
          if (selcol[la] == (uint16_t)lb && a_tok >= 0) q.src_rank[a_tok] = pos;
          const int slot = edge_base + atomicAdd(&slot_counter, 1);
          if (slot < q.sum_k) {
            q.edges[slot] = a_tok;
            q.edges[q.sum_k + slot] = b_tok;
            q.edges[2 * q.sum_k + slot] = pos;
          }
          ++pos;
        }
      }
    }
    if (b_tok >= 0) {
      q.dst[b_tok] = -1; q.cnt[b_tok] = pos; q.src_rank[b_tok] = 0;
      g.best_fd[b_tok] = __uint_as_float(0x7f800000u);
      g.best_dst[b_tok] = -1;
    }
  }
}

__global__ __launch_bounds__(256) void edge_clear_kernel(int32_t *edges, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) edges[i] = -1;
}

__global__ __launch_bounds__(256) void edge_fill_kernel(EdgeArgs q, const int32_t *grp_offsets, int32_t *grp_src, int sum_n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= q.sum_k) return;
  const int a = q.edges[i], b = q.edges[q.sum_k + i], pos = q.edges[2 * q.sum_k + i];
  if ((unsigned)a >= (unsigned)sum_n || (unsigned)b >= (unsigned)sum_n) return;
  const int slot = grp_offsets[b] + pos;
  if (slot >= 0 && slot < q.sum_k) grp_src[slot] = a;
}

hipError_t launch_edge_select(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows,
                              int max_window, int sum_n, int sum_k, const int32_t *win_offsets,
                              const int32_t *win_tokens, const int32_t *win_remove, float *partial, float *best_fd,
                              int32_t *best_dst, int32_t *dst, int32_t *cnt, int32_t *src_rank, int32_t *edges,
                              bool device_counts, uint32_t *big_keys, hipStream_t stream) {
  if (n_windows == 0 || plan.n_tiles == 0) return hipSuccess;
  const int maxA = (max_window + 1) / 2, maxB = max_window / 2;
  if (maxA > EB_MAX_SIDE || (maxA > EDGE_MAX_SIDE && (!big_keys || plan.group != 1))) return hipErrorInvalidValue;
  hipError_t e;
  if (device_counts && sum_k > 0) {   // the list is sized from a bound: slots no window uses must read as empty
    hipLaunchKernelGGL(edge_clear_kernel, dim3((unsigned)((2 * (size_t)sum_k + 255) / 256)), dim3(256), 0, stream, edges, 2 * sum_k);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  e = launch_fd_partial(plan, dtype, X, ldx, d, n_windows, sum_n, win_offsets, win_tokens, partial, stream);
  if (e != hipSuccess) return e;
  const FdArgs g = make_fd_args(plan, dtype, X, ldx, d, n_windows, sum_n, win_offsets, win_tokens, partial, best_fd, best_dst);
  EdgeArgs q{};
  q.win_remove = win_remove; q.dst = dst; q.cnt = cnt; q.src_rank = src_rank; q.edges = edges; q.sum_k = sum_k;
  q.key_capacity = maxA * (maxB | 1); q.clamp_v = device_counts ? 1 : 0;
  q.big_keys = big_keys; q.big_stride = (size_t)maxA * (size_t)(maxB > 0 ? maxB : 1); q.max_a = maxA; q.max_b = maxB;
  if (maxA > EDGE_MAX_SIDE) {   // windows beyond the one-kernel path
    const dim3 tiles((unsigned)plan.n_tiles);
    switch (plan.ksplit) {
      case 1: hipLaunchKernelGGL(edge_keys_kernel<1>, tiles, dim3(256), 0, stream, g, q); break;
      case 2: hipLaunchKernelGGL(edge_keys_kernel<2>, tiles, dim3(256), 0, stream, g, q); break;
      case 4: hipLaunchKernelGGL(edge_keys_kernel<4>, tiles, dim3(256), 0, stream, g, q); break;
      case 8: hipLaunchKernelGGL(edge_keys_kernel<8>, tiles, dim3(256), 0, stream, g, q); break;
      case 16: hipLaunchKernelGGL(edge_keys_kernel<16>, tiles, dim3(256), 0, stream, g, q); break;
      default: return hipErrorInvalidValue;   // make_fd_plan doubles from 1 up to 16
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(edge_select_big_kernel, dim3((unsigned)n_windows), dim3(EB_THREADS), 0, stream, g, q);
    return hipGetLastError();
  }
  const size_t lds = (size_t)maxA * (size_t)(maxB | 1) * sizeof(uint32_t);
  static std::atomic<bool> allowed[64];   // up to 66 KB of dynamic LDS: above the 64 KB default, set once per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!allowed[dev].load(std::memory_order_acquire)) {
    const int max_lds = (int)((size_t)EDGE_MAX_SIDE * (EDGE_MAX_SIDE | 1) * sizeof(uint32_t));
    const void *kernels[5] = {reinterpret_cast<const void *>(edge_select_kernel<1>), reinterpret_cast<const void *>(edge_select_kernel<2>),
                              reinterpret_cast<const void *>(edge_select_kernel<4>), reinterpret_cast<const void *>(edge_select_kernel<8>),
                              reinterpret_cast<const void *>(edge_select_kernel<16>)};
    for (const void *kf : kernels) {
      e = hipFuncSetAttribute(kf, hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
      if (e != hipSuccess) return e;
    }
    allowed[dev].store(true, std::memory_order_release);
  }
  const dim3 grid((unsigned)n_windows), block(EDGE_THREADS);
  switch (plan.ksplit) {
    case 1: hipLaunchKernelGGL(edge_select_kernel<1>, grid, block, lds, stream, g, q); break;
    case 2: hipLaunchKernelGGL(edge_select_kernel<2>, grid, block, lds, stream, g, q); break;
    case 4: hipLaunchKernelGGL(edge_select_kernel<4>, grid, block, lds, stream, g, q); break;
    case 8: hipLaunchKernelGGL(edge_select_kernel<8>, grid, block, lds, stream, g, q); break;
    case 16: hipLaunchKernelGGL(edge_select_kernel<16>, grid, block, lds, stream, g, q); break;
    default: return hipErrorInvalidValue;   // make_fd_plan doubles from 1 up to 16
  }
  return hipGetLastError();
}

size_t edge_big_key_count(int n_windows, int max_window) {
  const int maxA = (max_window + 1) / 2, maxB = max_window / 2;
  if (maxA <= EDGE_MAX_SIDE) return 0;
  return (size_t)n_windows * (size_t)maxA * (size_t)(maxB > 0 ? maxB : 1);
}

hipError_t launch_edge_fill(int sum_k, int sum_n, const int32_t *edges, const int32_t *grp_offsets, int32_t *grp_src,
                            hipStream_t stream) {
  if (sum_k <= 0) return hipSuccess;
  EdgeArgs q{};
  q.edges = const_cast<int32_t *>(edges);
  q.sum_k = sum_k;
  hipLaunchKernelGGL(edge_fill_kernel, dim3((unsigned)((sum_k + 255) / 256)), dim3(256), 0, stream, q, grp_offsets, grp_src, sum_n);
  return hipGetLastError();
}

}  // namespace lk
