// Edge selection (paper Sec. 3.2.1 Step 2) and the index structures of the merge.
//
// In every window the r A nodes with the lowest best-edge FD are merged into their B node; the order
// is fixed by the key (order-preserving bits of FD, then local position), so equal FDs go to the
// earlier token.  Selection is by counting, not sorting: the rank of an A node is the number of
// smaller keys in its window, and the rank of a merged node inside its group is the number of
// earlier merged nodes with the same destination, which makes the inverse map (grp_offsets /
// grp_src) deterministic without atomics on the output.
//
//   select_window_kernel : per window -> dst[], per-token source counts, per-source ranks (up to 256 A nodes), by
//                          counting smaller keys inside one workgroup
//   select_rank_kernel   : the same results for larger windows, the counting spread over several workgroups
//   select_scan_kernel   : one workgroup (per sequence, for larger batches) -> exclusive scans (new_index, grp_offsets),
//                          cu_vis_out, grp_src
#include <atomic>
#include "lk_xi_body.h"

namespace lk {

struct SelArgs {
  int n_windows, batch, sum_n;
  const int32_t *cu_vis, *win_offsets, *win_tokens, *win_remove;
  float *best_fd;            // inputs of the selection -- or, when best_key is given, outputs derived from the keys
  int32_t *best_dst;
  const unsigned long long *best_key;   // optional: packed keys of the tiled FD kernel, [column tile][list position]
  int key_mt, key_nt;                   // tiles per window that kernel was planned with
  int32_t *dst, *new_index, *grp_offsets, *grp_src, *cu_vis_out, *cnt, *src_rank;
  int cap;   // power of two >= the larger side of the largest window
  int dir;   // 0: even list positions propose, 1: odd ones (side_a / pos_a)
  int per_seq;   // scan: one workgroup per sequence (0: one workgroup for the whole batch)
};


// Score and proposal of the A node at list position `pos`, local position `la` (token `tok`, a valid index): from
// best_fd / best_dst, or from the packed keys the tiled FD kernel leaves per column tile (n_col of them for this window).
__device__ __forceinline__ void proposal_of(const SelArgs &g, int tok, int pos, int la, int n_col, float &fd, int &prop) {
  if (g.best_key) {
    const unsigned long long key =
        la < g.key_mt * FD_BIG_TILE ? fd_big_best_key(g.best_key, g.sum_n, pos, n_col) : ~0ull;   // else: beyond the tiles
    fd = key == ~0ull ? __uint_as_float(0x7f800000u) : __uint_as_float((unsigned)(key >> 32));
    prop = key == ~0ull ? -1 : (int)(key & 0xffffffffu);
  } else {
    fd = g.best_fd[tok];
    prop = g.best_dst[tok];
  }
}
// With keys as the input, the selection also writes best_fd / best_dst (the outputs of the score step).
__device__ __forceinline__ void publish(const SelArgs &g, int tok, float fd, int prop) {
  if (g.best_key && tok >= 0) { g.best_fd[tok] = fd; g.best_dst[tok] = prop; }
}

// Windows of up to COUNT_MAX_A A nodes: one workgroup per window.  The rank of an A node among the keys of its window
// is the number of smaller keys (earlier position first among equal keys); a merged node's rank inside its group is
// the number of earlier merged nodes with the same target, and a B node's source count the number of merged nodes
// that name it.  Three short counting loops over LDS: no sort, and every token of the window is written exactly once.
// SEGS threads share a position (A node t and B node t) and split the window's list between them: the loops are
// chains of dependent LDS reads and compares, so longer lists want more waves rather than longer loops.
constexpr int COUNT_MAX_A = 256;

template <int SEGS>
__global__ __launch_bounds__(COUNT_MAX_A * SEGS) void select_window_kernel(SelArgs g) {
  // order-preserving FD bits of every A node, then the target of every merged A node; all-ones beyond |A| (never
  // smaller than a key, never a valid target), padded to whole groups of four
  __shared__ __attribute__((aligned(16))) uint32_t key[COUNT_MAX_A + 4];
  __shared__ __attribute__((aligned(16))) uint32_t tgt[COUNT_MAX_A + 4];
  __shared__ int part[3][SEGS][COUNT_MAX_A];
  const int w = blockIdx.x;
  const int off = g.win_offsets[w];
  const int v = g.win_offsets[w + 1] - off;
  const int cap = g.cap < COUNT_MAX_A ? g.cap : COUNT_MAX_A;
  const int v_in = v < 2 * cap ? v : 2 * cap;   // window larger than the caller's bound: the surplus tokens stay
  const int nA = side_a(v_in, g.dir), nB = side_b(v_in, g.dir);
  int r = g.win_remove[w];
  r = r < 0 ? 0 : (r > nA ? nA : r);
  if (nB == 0) r = 0;
  const int la = threadIdx.x % COUNT_MAX_A, seg = threadIdx.x / COUNT_MAX_A;
  for (int t = v_in + (int)threadIdx.x; t < v; t += COUNT_MAX_A * SEGS) {
    const int tok = g.win_tokens[off + t];
    if ((unsigned)tok < (unsigned)g.sum_n) {
      g.dst[tok] = -1; g.cnt[tok] = 0; g.src_rank[tok] = 0;
      publish(g, tok, __uint_as_float(0x7f800000u), -1);
    }
  }
  const bool has_a = la < nA, has_b = la < nB;
  const int a_pos = has_a ? pos_a(la, g.dir) : 0;
  int a_tok = g.win_tokens[off + a_pos];
  int b_tok = g.win_tokens[off + (has_b ? pos_b(la, g.dir) : 0)];
  const int first_b = g.win_tokens[off + (nB > 0 ? pos_b(0, g.dir) : 0)];
  if (!has_a || (unsigned)a_tok >= (unsigned)g.sum_n) a_tok = -1;
  if (!has_b || (unsigned)b_tok >= (unsigned)g.sum_n) b_tok = -1;
  float fd;
  int prop;   // the proposal of this A node, or the first B node of the window
  proposal_of(g, a_tok >= 0 ? a_tok : 0, off + a_pos, has_a ? la : 0, fd_big_col_tiles(nB, g.key_nt), fd, prop);
  if (seg == 0) {
    publish(g, a_tok, fd, prop);
    publish(g, b_tok, __uint_as_float(0x7f800000u), -1);
  }
  if (a_tok < 0 || !(fd >= 0.f)) fd = __uint_as_float(0x7f800000u);   // NaN or negative never wins
  if (a_tok < 0) prop = -1;
  else if ((unsigned)prop >= (unsigned)g.sum_n) prop = (nB > 0 && (unsigned)first_b < (unsigned)g.sum_n) ? first_b : -1;
  const int n4 = (nA + 3) & ~3;
  const int seg_len = ((n4 / 4 + SEGS - 1) / SEGS) * 4;   // entries per segment, a multiple of 4
  const int o_begin = seg * seg_len, o_end = min(n4, o_begin + seg_len);
  const uint32_t mine = has_a ? f32_order_key(fd) : 0xffffffffu;
  if (seg == 0 && la < n4) key[la] = mine;
  __syncthreads();
  int c0 = 0;
#pragma unroll 4
  for (int o = o_begin; o < o_end; o += 4) {
    const uint4 k = *reinterpret_cast<const uint4 *>(&key[o]);
    c0 += (k.x < mine || (k.x == mine && o < la)) ? 1 : 0;
    c0 += (k.y < mine || (k.y == mine && o + 1 < la)) ? 1 : 0;
    c0 += (k.z < mine || (k.z == mine && o + 2 < la)) ? 1 : 0;
    c0 += (k.w < mine || (k.w == mine && o + 3 < la)) ? 1 : 0;
  }
  if (SEGS > 1) {
    part[0][seg][la] = c0;
    __syncthreads();
    c0 = 0;
#pragma unroll
    for (int q = 0; q < SEGS; ++q) c0 += part[0][q][la];
  }
  const bool merged = has_a && c0 < r && prop >= 0;   // a selected node without a usable target stays
  const uint32_t mine_t = merged ? (uint32_t)prop : 0xffffffffu;
  if (seg == 0 && la < n4) tgt[la] = mine_t;
  __syncthreads();
  const uint32_t self = (uint32_t)b_tok;
  int c1 = 0, c2 = 0;
#pragma unroll 4
  for (int o = o_begin; o < o_end; o += 4) {
    const uint4 d = *reinterpret_cast<const uint4 *>(&tgt[o]);
    c1 += (d.x == mine_t && o < la) ? 1 : 0;
    c1 += (d.y == mine_t && o + 1 < la) ? 1 : 0;
    c1 += (d.z == mine_t && o + 2 < la) ? 1 : 0;
    c1 += (d.w == mine_t && o + 3 < la) ? 1 : 0;
    c2 += (d.x == self) ? 1 : 0;
    c2 += (d.y == self) ? 1 : 0;
    c2 += (d.z == self) ? 1 : 0;
    c2 += (d.w == self) ? 1 : 0;
  }
  if (SEGS > 1) {
    part[1][seg][la] = c1;
    part[2][seg][la] = c2;
    __syncthreads();
    c1 = c2 = 0;
#pragma unroll
    for (int q = 0; q < SEGS; ++q) { c1 += part[1][q][la]; c2 += part[2][q][la]; }
  }
  if (seg != 0) return;
  if (a_tok >= 0) {
    g.dst[a_tok] = merged ? prop : -1;
    g.src_rank[a_tok] = merged ? c1 : 0;
    g.cnt[a_tok] = 0;
  }
  if (b_tok >= 0) {
    g.dst[b_tok] = -1;
    g.src_rank[b_tok] = 0;
    g.cnt[b_tok] = c2;
  }
}

// ---------------------------------------------------------------------------------------------------------
// Large windows (more than 256 A nodes): selection by counting instead of sorting.  The rank of an A node among the
// keys of its window is the number of smaller keys -- |A|^2 comparisons, but they spread over many workgroups and
// need no barrier ladder, where a 2048-key bitonic sort in one workgroup is 66 dependent passes.
//   MODE 0: rank of every A node -> dst (and the default dst of the B nodes)
//   MODE 1: from dst: rank of every merged A node among the earlier sources of its target, sources per B node
// One workgroup = 32 A positions (and the 32 B positions beside them) of one window; 8 threads share a position and
// split the window's key list between them.
constexpr int RANK_ROWS = 32;
constexpr int RANK_SEGS = 8;
constexpr int RANK_MAX_A = 2048;   // |A| of the largest window the library accepts (4096 tokens)

template <int MODE>
__global__ __launch_bounds__(RANK_ROWS * RANK_SEGS) void select_rank_kernel(SelArgs g, int blocks_per_window) {
  // MODE 0: order-preserving FD bits; MODE 1: dst of every A node.  Padded with all-ones up to whole 4-entry groups
  // per segment: an all-ones entry is never smaller than a key and never a valid target.
  __shared__ __attribute__((aligned(16))) uint32_t vals[RANK_MAX_A + 4 * RANK_SEGS];
  __shared__ int part[2][RANK_SEGS][RANK_ROWS];
  const int w = blockIdx.x / blocks_per_window, rb = blockIdx.x - w * blocks_per_window;
  const int off = g.win_offsets[w];
  const int v = g.win_offsets[w + 1] - off;
  const int v_in = v < 2 * g.cap ? v : 2 * g.cap;
  const int nA = side_a(v_in, g.dir), nB = side_b(v_in, g.dir);
  if (rb * RANK_ROWS >= (nA > nB ? nA : nB)) return;
  if (MODE == 0 && rb == 0) {   // tokens of a window beyond the caller's bound stay
    for (int t = v_in + (int)threadIdx.x; t < v; t += RANK_ROWS * RANK_SEGS) {
      const int tok = g.win_tokens[off + t];
      if ((unsigned)tok < (unsigned)g.sum_n) {
        g.dst[tok] = -1; g.cnt[tok] = 0; g.src_rank[tok] = 0;
        publish(g, tok, __uint_as_float(0x7f800000u), -1);
      }
    }
  }
  int r = g.win_remove[w];
  r = r < 0 ? 0 : (r > nA ? nA : r);
  if (nB == 0) r = 0;
  const int tid = threadIdx.x;

  // the window's list: one value per A node
  const int seg_len = ((nA + RANK_SEGS - 1) / RANK_SEGS + 3) & ~3;   // entries per segment, a multiple of 4
  for (int la0 = 0; la0 < seg_len * RANK_SEGS; la0 += RANK_ROWS * RANK_SEGS) {
    const int la = la0 + tid;
    const int lc = la < nA ? la : (nA > 0 ? nA - 1 : 0);
    const int lpos = nA > 0 ? pos_a(lc, g.dir) : 0;   // (a window without a proposing node: position 0, value unused)
    const int tok = g.win_tokens[off + lpos];
    const bool ok = (unsigned)tok < (unsigned)g.sum_n;
    uint32_t val;
    if (MODE == 0) {
      float fd;
      int unused;
      proposal_of(g, ok ? tok : 0, off + lpos, lc, fd_big_col_tiles(nB, g.key_nt), fd, unused);
      if (!ok || !(fd >= 0.f)) fd = __uint_as_float(0x7f800000u);   // NaN or negative never wins
      val = f32_order_key(fd);
    } else {
      const int d = g.dst[ok ? tok : 0];
      val = ok ? (uint32_t)d : 0xffffffffu;
    }
    if (la < seg_len * RANK_SEGS) vals[la] = la < nA ? val : 0xffffffffu;
  }
  // this thread's position and the tokens there
  const int row = tid & (RANK_ROWS - 1), seg = tid / RANK_ROWS;
  const int la = rb * RANK_ROWS + row;
  const bool has_a = la < nA, has_b = la < nB;
  const int a_pos = has_a ? pos_a(la, g.dir) : 0;
  int a_tok = g.win_tokens[off + a_pos];
  int b_tok = g.win_tokens[off + (has_b ? pos_b(la, g.dir) : 0)];
  if (!has_a || (unsigned)a_tok >= (unsigned)g.sum_n) a_tok = -1;
  if (!has_b || (unsigned)b_tok >= (unsigned)g.sum_n) b_tok = -1;
  int prop = -1;
  if (MODE == 0 && seg == 0) {   // the proposal of this A node, or the first B node of the window
    float fd;
    proposal_of(g, a_tok >= 0 ? a_tok : 0, off + a_pos, has_a ? la : 0, fd_big_col_tiles(nB, g.key_nt), fd, prop);
    publish(g, a_tok, fd, prop);
    publish(g, b_tok, __uint_as_float(0x7f800000u), -1);
    const int first_b = g.win_tokens[off + (nB > 0 ? pos_b(0, g.dir) : 0)];
    if (a_tok < 0) prop = -1;
    else if ((unsigned)prop >= (unsigned)g.sum_n) prop = (nB > 0 && (unsigned)first_b < (unsigned)g.sum_n) ? first_b : -1;
  }
  __syncthreads();

  const int o_begin = seg * seg_len;
  int c0 = 0, c1 = 0;
  if (MODE == 0) {
    const uint32_t mine = vals[has_a ? la : 0];
#pragma unroll 4
    for (int o = o_begin; o < o_begin + seg_len; o += 4) {
      const uint4 k = *reinterpret_cast<const uint4 *>(&vals[o]);
      c0 += (k.x < mine || (k.x == mine && o < la)) ? 1 : 0;
      c0 += (k.y < mine || (k.y == mine && o + 1 < la)) ? 1 : 0;
      c0 += (k.z < mine || (k.z == mine && o + 2 < la)) ? 1 : 0;
      c0 += (k.w < mine || (k.w == mine && o + 3 < la)) ? 1 : 0;
    }
  } else {
    const uint32_t mine = has_a ? vals[la] : 0xffffffffu;    // target of this A node (all-ones: stays)
    const uint32_t self = (uint32_t)b_tok;                   // this B node as a target
#pragma unroll 4
    for (int o = o_begin; o < o_begin + seg_len; o += 4) {
      const uint4 d = *reinterpret_cast<const uint4 *>(&vals[o]);
      c0 += (d.x == mine && o < la) ? 1 : 0;
      c0 += (d.y == mine && o + 1 < la) ? 1 : 0;
      c0 += (d.z == mine && o + 2 < la) ? 1 : 0;
      c0 += (d.w == mine && o + 3 < la) ? 1 : 0;
      c1 += (d.x == self) ? 1 : 0;
      c1 += (d.y == self) ? 1 : 0;
      c1 += (d.z == self) ? 1 : 0;
      c1 += (d.w == self) ? 1 : 0;
    }
  }
  part[0][seg][row] = c0;
  part[1][seg][row] = c1;
  __syncthreads();
  if (seg == 0) {
    int s0 = 0, s1 = 0;
#pragma unroll
    for (int q = 0; q < RANK_SEGS; ++q) { s0 += part[0][q][row]; s1 += part[1][q][row]; }
    if (MODE == 0) {
      if (a_tok >= 0) g.dst[a_tok] = (s0 < r) ? prop : -1;
      if (b_tok >= 0) g.dst[b_tok] = -1;
    } else {
      if (a_tok >= 0) {
        const bool merged = vals[la] != 0xffffffffu;
        g.src_rank[a_tok] = merged ? s0 : 0;
        g.cnt[a_tok] = 0;
      }
      if (b_tok >= 0) {
        g.src_rank[b_tok] = 0;
        g.cnt[b_tok] = s1;
      }
    }
  }
}

// Scans over all tokens of the batch.  Every thread owns a run of consecutive tokens, so one pass needs a single
// workgroup scan (two values at once) instead of one per 1024 tokens; all loads of a pass are issued together.
// One workgroup does the whole batch, or (per_seq, for batches of some size) one workgroup per sequence: it first
// counts what stays and what is merged in the sequences before its own -- re-reading a few KB is cheaper than any
// exchange between workgroups -- and then scans its own tokens from those bases.  A token's target lies in its own
// window, hence in its own sequence, so the inverse map needs nothing from another workgroup either.
constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_ITEMS = 10;     // tokens per thread and pass (10240 tokens per pass)
constexpr int FILL_UNROLL = 4;
constexpr int SCAN_PER_SEQ_MIN_TOKENS = 2048;   // batches with fewer tokens: one workgroup for all (a single short pass)
constexpr int SCAN_PER_SEQ_MAX_BATCH = 256;
constexpr size_t SCAN_LDS_BYTES = (size_t)2 * SCAN_THREADS * SCAN_ITEMS * sizeof(int);   // 80 KB: above the 64 KB default

// WITH_HEADS: the first n_head_blocks workgroups of the launch do something else entirely -- they sum the per-head xi
// partials (last pass of the xi computation, lk_xi_body.h), which is independent of the scan and as short; the scan
// is the last workgroup.  (The scan stays written out in the kernel: as an inlined function it costs eight more
// registers at the 128-register limit of a 1024-thread workgroup and spills.)
template <bool WITH_HEADS>
__global__ __launch_bounds__(SCAN_THREADS) void select_scan_kernel(SelArgs g, XiArgs x, int n_head_blocks) {
  if (WITH_HEADS && (int)blockIdx.x < n_head_blocks) {
    xi_heads_body(x, blockIdx.x * SCAN_THREADS + threadIdx.x);
    return;
  }
  extern __shared__ int scan_lds[];               // SCAN_LDS_BYTES
  int *kb = scan_lds;                              // staying tokens before each token of the pass
  int *gb = scan_lds + SCAN_THREADS * SCAN_ITEMS;  // sources before each token of the pass (= its group's first slot)
  __shared__ int2 wsum[SCAN_THREADS / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s_first = g.cu_vis[tid <= g.batch ? tid : g.batch];   // sequence start handled by this thread (first round)
  // the tokens of this workgroup: [t0, t1)
  const int seq = (int)blockIdx.x - (WITH_HEADS ? n_head_blocks : 0);
  int t0 = 0, t1 = g.sum_n;
  if (g.per_seq) {
    t0 = g.cu_vis[seq]; t1 = g.cu_vis[seq + 1];
    t0 = t0 < 0 ? 0 : (t0 > g.sum_n ? g.sum_n : t0);
    t1 = t1 < t0 ? t0 : (t1 > g.sum_n ? g.sum_n : t1);
  }
  int keep_base = 0, cnt_base = 0;
  if (g.per_seq) {   // staying tokens and sources before this sequence
    int ks = 0, cs = 0;
    for (int i = tid; i < t0; i += 4 * SCAN_THREADS) {   // uniform trip count per wave is not needed: plain loads
      int dv[4], cv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int ii = i + j * SCAN_THREADS;
        const int ic = ii < t0 ? ii : 0;
        dv[j] = g.dst[ic]; cv[j] = g.cnt[ic];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = i + j * SCAN_THREADS < t0;
        ks += (ok && dv[j] < 0) ? 1 : 0;
        cs += ok ? cv[j] : 0;
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) { ks += __shfl_xor(ks, o, 64); cs += __shfl_xor(cs, o, 64); }
    if (lane == 0) wsum[wave] = make_int2(ks, cs);
    __syncthreads();
#pragma unroll
    for (int w2 = 0; w2 < SCAN_THREADS / 64; ++w2) { keep_base += wsum[w2].x; cnt_base += wsum[w2].y; }
    __syncthreads();   // wsum is written again by the first pass
  }
  const int keep_first = keep_base;
  const int n_loc = t1 - t0;
  int per = (n_loc + SCAN_THREADS - 1) / SCAN_THREADS;
  per = per < 1 ? 1 : (per > SCAN_ITEMS ? SCAN_ITEMS : per);
  if (per < SCAN_ITEMS && per > 1 && !(per & 1)) ++per;   // an odd run length: thread t's slots in kb[] start at bank t * per
  const int pass_tokens = per * SCAN_THREADS;
  const bool one_pass = n_loc <= pass_tokens;   // then dst / src_rank stay in registers for the inverse map below
  int d[SCAN_ITEMS], c[SCAN_ITEMS], sr[SCAN_ITEMS];
  for (int pass_base = t0; pass_base < t1; pass_base += pass_tokens) {
    const int i0 = pass_base + tid * per;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
      const bool ok = k < per && i0 + k < t1;
      const int ic = ok ? i0 + k : 0;            // unconditional loads from a clamped index
      const int dv = g.dst[ic], cv = g.cnt[ic], sv = g.src_rank[ic];
      d[k] = ok ? dv : 0;
      c[k] = ok ? cv : 0;
      sr[k] = sv;
    }
    int ks = 0, cs = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
      const bool ok = k < per && i0 + k < t1;
      ks += (ok && d[k] < 0) ? 1 : 0;
      cs += c[k];
    }
    int ik = ks, ic2 = cs;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int tk = __shfl_up(ik, o, 64), tc = __shfl_up(ic2, o, 64);
      if (lane >= o) { ik += tk; ic2 += tc; }
    }
    if (lane == 63) wsum[wave] = make_int2(ik, ic2);
    __syncthreads();
    int wk = 0, wc = 0, tot_k = 0, tot_c = 0;
#pragma unroll
    for (int w2 = 0; w2 < SCAN_THREADS / 64; ++w2) {
      const int2 v = wsum[w2];
      wk += (w2 < wave) ? v.x : 0;
      wc += (w2 < wave) ? v.y : 0;
      tot_k += v.x;
      tot_c += v.y;
    }
    int ek = keep_base + wk + ik - ks, ec = cnt_base + wc + ic2 - cs;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
      const bool ok = k < per && i0 + k < t1;
      if (ok) {
        const int keep = d[k] < 0 ? 1 : 0;
        kb[tid * per + k] = ek;
        gb[tid * per + k] = ec;
        g.new_index[i0 + k] = keep ? ek : -1;
        g.grp_offsets[i0 + k] = ec;
        ek += keep;
        ec += c[k];
      }
    }
    // a single pass reads nothing back from global memory (the group starts come from LDS below): then the barrier need
    // not wait for the stores above
    if (one_pass) lds_barrier(); else __syncthreads();
    // vision offsets after the step: staying tokens before each sequence start that falls into this pass
    const int pass_end = min(pass_base + pass_tokens, t1);
    for (int b = tid; b <= (g.per_seq ? -1 : g.batch); b += SCAN_THREADS) {
      const int s = (b == tid) ? s_first : g.cu_vis[b];
      if (s >= pass_base && s < pass_end) g.cu_vis_out[b] = kb[s - pass_base];
    }
    keep_base += tot_k;
    cnt_base += tot_c;
    if (!one_pass) __syncthreads();
  }
  for (int b = tid; b <= (g.per_seq ? -1 : g.batch); b += SCAN_THREADS) {
    const int s = (b == tid) ? s_first : g.cu_vis[b];
    if (s >= g.sum_n) g.cu_vis_out[b] = keep_base;
  }
  if (g.per_seq && tid == 0) {   // the offset of the own sequence; the last workgroup also closes both arrays
    g.cu_vis_out[seq] = keep_first;
    if (seq == g.batch - 1) g.cu_vis_out[g.batch] = keep_base;
  }
  if (tid == 0 && (!g.per_seq || seq == g.batch - 1)) g.grp_offsets[g.sum_n] = cnt_base;
  // inverse map: source a goes to slot grp_offsets[dst[a]] + (its rank among the sources of that target).  In a single
  // pass the group starts of all tokens are in LDS (written before the barrier above); otherwise they are read back
  // from global memory after the barrier below.
  // (a target outside [t0, t1) cannot come from the selection kernels; it is dropped rather than followed)
  if (one_pass) {
    const int i0 = t0 + tid * per;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {   // c[] is free now: it takes the group starts
      const bool ok = k < per && i0 + k < t1 && d[k] >= t0 && d[k] < t1;
      c[k] = gb[ok ? d[k] - t0 : 0];
      d[k] = ok ? d[k] : -1;
    }
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
      if (d[k] >= 0) g.grp_src[c[k] + sr[k]] = i0 + k;
  }
  __syncthreads();
  for (int a0 = t0; a0 < (one_pass ? t0 : t1); a0 += FILL_UNROLL * SCAN_THREADS) {
    int b[FILL_UNROLL], r2[FILL_UNROLL], go[FILL_UNROLL];
#pragma unroll
    for (int j = 0; j < FILL_UNROLL; ++j) {
      const int a = a0 + j * SCAN_THREADS + tid;
      const int ac = a < t1 ? a : 0;
      const int bv = g.dst[ac], sv = g.src_rank[ac];
      b[j] = (a < t1 && bv >= t0 && bv < t1) ? bv : -1;
      r2[j] = sv;
    }
#pragma unroll
    for (int j = 0; j < FILL_UNROLL; ++j) go[j] = g.grp_offsets[b[j] >= 0 ? b[j] : 0];
#pragma unroll
    for (int j = 0; j < FILL_UNROLL; ++j)
      if (b[j] >= 0) g.grp_src[go[j] + r2[j]] = a0 + j * SCAN_THREADS + tid;
  }
}



// The scan kernels take more dynamic LDS than the default limit: a property of a kernel as loaded on a device, set once
// per device (setting it twice is harmless: the flag only has to be free of data races).
static hipError_t allow_scan_lds() {
  static std::atomic<bool> done[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(select_scan_kernel<false>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)SCAN_LDS_BYTES);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(select_scan_kernel<true>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)SCAN_LDS_BYTES);
  if (e != hipSuccess) return e;
  done[dev].store(true, std::memory_order_release);
  return hipSuccess;
}

hipError_t launch_select_scan(int batch, int sum_n, const int32_t *cu_vis, const int32_t *dst, int32_t *new_index,
                              int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out, const int32_t *cnt,
                              const int32_t *src_rank, hipStream_t stream) {
  SelArgs g{};
  g.batch = batch; g.sum_n = sum_n; g.cu_vis = cu_vis;
  g.dst = const_cast<int32_t *>(dst); g.new_index = new_index; g.grp_offsets = grp_offsets; g.grp_src = grp_src;
  g.cu_vis_out = cu_vis_out; g.cnt = const_cast<int32_t *>(cnt); g.src_rank = const_cast<int32_t *>(src_rank);
  // one workgroup per sequence once a batch is large enough for the single workgroup's serial passes to show, as long
  // as all of them fit the chip at once (one workgroup of this kernel fills a CU)
  g.per_seq = (batch > 1 && batch <= SCAN_PER_SEQ_MAX_BATCH && sum_n >= SCAN_PER_SEQ_MIN_TOKENS) ? 1 : 0;
  hipError_t e = allow_scan_lds();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(select_scan_kernel<false>, dim3(g.per_seq ? (unsigned)batch : 1u), dim3(SCAN_THREADS), SCAN_LDS_BYTES,
                     stream, g, XiArgs{}, 0);
  return hipGetLastError();
}

hipError_t launch_select_scan_heads(int batch, int sum_n, const int32_t *cu_vis, const int32_t *dst, int32_t *new_index,
                                    int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out, const int32_t *cnt,
                                    const int32_t *src_rank, const XiArgs &x, hipStream_t stream) {
  SelArgs g{};
  g.batch = batch; g.sum_n = sum_n; g.cu_vis = cu_vis;
  g.dst = const_cast<int32_t *>(dst); g.new_index = new_index; g.grp_offsets = grp_offsets; g.grp_src = grp_src;
  g.cu_vis_out = cu_vis_out; g.cnt = const_cast<int32_t *>(cnt); g.src_rank = const_cast<int32_t *>(src_rank);
  const int n_head_blocks = (sum_n + SCAN_THREADS - 1) / SCAN_THREADS;
  hipError_t e = allow_scan_lds();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(select_scan_kernel<true>, dim3((unsigned)(n_head_blocks + 1)), dim3(SCAN_THREADS), SCAN_LDS_BYTES,
                     stream, g, x, n_head_blocks);
  return hipGetLastError();
}

hipError_t launch_select(int n_windows, int max_window_tokens, int batch, int sum_n, const int32_t *cu_vis,
                         const int32_t *win_offsets, const int32_t *win_tokens, const int32_t *win_remove,
                         const unsigned long long *keys, int key_mt, int key_nt, float *best_fd, int32_t *best_dst,
                         int32_t *dst, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out,
                         int32_t *cnt, int32_t *src_rank, int dir, hipStream_t stream) {
  SelArgs g{};
  g.best_key = keys; g.key_mt = key_mt; g.key_nt = key_nt; g.dir = dir;
  g.n_windows = n_windows; g.batch = batch; g.sum_n = sum_n;
  g.cu_vis = cu_vis; g.win_offsets = win_offsets; g.win_tokens = win_tokens; g.win_remove = win_remove;
  g.best_fd = best_fd; g.best_dst = best_dst;
  g.dst = dst; g.new_index = new_index; g.grp_offsets = grp_offsets; g.grp_src = grp_src;
  g.cu_vis_out = cu_vis_out; g.cnt = cnt; g.src_rank = src_rank;
  const int maxA = (max_window_tokens + 1) / 2;   // (dir 1: the caller hands in an even bound, so this covers both sides)
  g.cap = maxA > 1 ? maxA : 1;
  if (n_windows > 0) {
    hipError_t e;
    if (g.cap <= COUNT_MAX_A) {
      if (g.cap > 96) hipLaunchKernelGGL(select_window_kernel<4>, dim3(n_windows), dim3(COUNT_MAX_A * 4), 0, stream, g);
      else hipLaunchKernelGGL(select_window_kernel<1>, dim3(n_windows), dim3(COUNT_MAX_A), 0, stream, g);
      e = hipGetLastError();
    } else {
      // counting selection; a window beyond the library's limit keeps its surplus A nodes, as everywhere else
      g.cap = maxA < RANK_MAX_A ? maxA : RANK_MAX_A;
      const int bpw = (g.cap + RANK_ROWS - 1) / RANK_ROWS;
      const dim3 grid((unsigned)(n_windows * bpw)), block(RANK_ROWS * RANK_SEGS);
      hipLaunchKernelGGL(select_rank_kernel<0>, grid, block, 0, stream, g, bpw);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(select_rank_kernel<1>, grid, block, 0, stream, g, bpw);
      e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
  }
  return launch_select_scan(batch, sum_n, cu_vis, dst, new_index, grp_offsets, grp_src, cu_vis_out, cnt, src_rank, stream);
}

}  // namespace lk
