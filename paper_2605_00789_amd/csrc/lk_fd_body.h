// Device-side bodies of the small-window feature-divergence kernels (paper Sec. 3.2.1 Steps 1-2).  They take the
// workgroup index and a block of LDS as arguments so that a launch can run them next to the bodies of another step
// (lk_fused.hip) as well as on their own (lk_score_fd.hip, where the algorithm is described).
#pragma once
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {


constexpr int FD_THREADS = 256;
constexpr int FD_WAVES = 4;
constexpr int FD_CHUNKS = 4;   // 16-byte chunks per lane and span
constexpr double NORM_EPS = 1e-12;

struct FdArgs {
  const void *X;
  int64_t ldx;
  int d, n_windows, sum_n;
  const int32_t *win_offsets, *win_tokens;
  float *partial;
  float *best_fd;
  int32_t *best_dst;
  int slot, group, mt, nt, n_tiles, ksplit, n_spans, spans_per_wg;
  int metric;   // 0: 1 - cos, 1: |a - b|, 2: |a - b|^2
  int dir;      // 0: even list positions propose, 1: odd ones (side_a / pos_a)
};

// Divergence of a pair from its inner product and squared norms (fp64).  The distances use
// |a - b|^2 = |a|^2 + |b|^2 - 2 <a, b>; the three sums of a pair come from the same instruction sequence, so identical
// rows give exactly 0.
__device__ __forceinline__ double divergence(int metric, double dot, double a2, double b2) {
  if (metric == 0) {
    double den;
    if (a2 >= NORM_EPS * NORM_EPS && b2 >= NORM_EPS * NORM_EPS) den = sqrt(a2 * b2);
    else den = fmax(sqrt(a2), NORM_EPS) * fmax(sqrt(b2), NORM_EPS);
    const double fd = 1.0 - dot / den;
    return fd < 0.0 ? 0.0 : fd;   // (a NaN stays a NaN: fmax would turn it into the best possible score)
  }
  const double d2 = a2 + b2 - 2.0 * dot;
  return metric == 1 ? sqrt(d2 < 0.0 ? 0.0 : d2) : (d2 < 0.0 ? 0.0 : d2);
}

constexpr int FD_PARTIAL_LDS = FD_WAVES * (32 * 32 + 2 * 32) * (int)sizeof(float);   // bytes of LDS fd_partial_body needs

struct WinInfo { int off, nA, nB; };

__device__ __forceinline__ WinInfo win_info(const FdArgs &g, int w) {
  WinInfo wi{0, 0, 0};
  if (w < g.n_windows) {
    wi.off = g.win_offsets[w];
    const int v = g.win_offsets[w + 1] - wi.off;
    wi.nA = side_a(v, g.dir);
    wi.nB = side_b(v, g.dir);
  }
  return wi;
}

__device__ __forceinline__ int checked_token(const FdArgs &g, int idx) {
  const int t = g.win_tokens[idx];
  return ((unsigned)t < (unsigned)g.sum_n) ? t : -1;
}

template <typename T>
__device__ __forceinline__ void fd_partial_body(const FdArgs &g, int block_id, char *lds) {
  using E = Elem<T>;
  constexpr int EPC = E::PER_CHUNK;
  constexpr int LANE_ELEMS = FD_CHUNKS * EPC;   // contiguous elements of one lane in a span
  constexpr int SPAN = 2 * LANE_ELEMS;          // elements of a row covered by one span

  float (*red)[32 * 32] = reinterpret_cast<float (*)[32 * 32]>(lds);                                  // [FD_WAVES][32 * 32]
  float (*rnorm)[2][32] = reinterpret_cast<float (*)[2][32]>(lds + FD_WAVES * 32 * 32 * sizeof(float));   // [FD_WAVES][2][32]

  const int tile = block_id % g.n_tiles;
  const int ks = block_id / g.n_tiles;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, half = lane >> 5;

  // rows of this tile
  int a_tok = -1, b_tok = -1;
  bool need_na = true, need_nb = true;
  if (g.group > 1) {
    const int s = r / g.slot, l = r - s * g.slot;
    const WinInfo wi = win_info(g, tile * g.group + s);
    if (l < wi.nA) a_tok = checked_token(g, wi.off + pos_a(l, g.dir));
    if (l < wi.nB) b_tok = checked_token(g, wi.off + pos_b(l, g.dir));
  } else {
    const int per = g.mt * g.nt;
    const int w = tile / per, rem = tile - w * per;
    const int mt = rem / g.nt, nt = rem - mt * g.nt;
    const WinInfo wi = win_info(g, w);
    const int la = mt * 32 + r, lb = nt * 32 + r;
    if (la < wi.nA) a_tok = checked_token(g, wi.off + pos_a(la, g.dir));
    if (lb < wi.nB) b_tok = checked_token(g, wi.off + pos_b(lb, g.dir));
    need_na = (nt == 0);
    need_nb = (mt == 0);
  }
  // slice 0 leaves the tile's token lists (rows, then columns) for the kernel that finishes the tile
  if (ks == 0 && wave == 0)
    reinterpret_cast<int32_t *>(g.partial + (int64_t)tile * FD_TILE_FLOATS + FD_TOK_OFFSET)[lane] = half ? b_tok : a_tok;
  // a tile without A rows or without B rows is never read by the epilogue
  if (__ballot(a_tok >= 0) == 0ull || __ballot(b_tok >= 0) == 0ull) return;

  // padding rows of the tile read token 0: their products land in rows/columns nobody reads
  const char *pa = static_cast<const char *>(g.X) + (int64_t)(a_tok < 0 ? 0 : a_tok) * g.ldx * E::BYTES;
  const char *pb = static_cast<const char *>(g.X) + (int64_t)(b_tok < 0 ? 0 : b_tok) * g.ldx * E::BYTES;

  f32x16 acc = {0}, na = {0}, nb = {0};
  const int s_begin = ks * g.spans_per_wg;
  const int s_end = min(s_begin + g.spans_per_wg, g.n_spans);

  uint4 ca[FD_CHUNKS], cb[FD_CHUNKS];
  auto load_span = [&](int s, uint4 *va, uint4 *vb) {
    const int e0 = s * SPAN + half * LANE_ELEMS;
#pragma unroll
    for (int c = 0; c < FD_CHUNKS; ++c) {
      const int e = e0 + c * EPC;
      const bool ok = (e + EPC <= g.d);
      const int ec = ok ? e : g.d - EPC;   // unconditional load from a clamped address, zeroed below
      const uint4 ta = ld16(pa + (int64_t)ec * E::BYTES), tb = ld16(pb + (int64_t)ec * E::BYTES);
      va[c] = ok ? ta : make_uint4(0, 0, 0, 0);
      vb[c] = ok ? tb : make_uint4(0, 0, 0, 0);
    }
  };

  int s = s_begin + wave;
  if (s < s_end) load_span(s, ca, cb);
  while (s < s_end) {
    uint4 na_next[FD_CHUNKS], nb_next[FD_CHUNKS];
    const int sn = s + FD_WAVES;
    if (sn < s_end) load_span(sn, na_next, nb_next);
#pragma unroll
    for (int c = 0; c < FD_CHUNKS; ++c) {
      E::mma32(ca[c], cb[c], acc);
      if (need_na) E::mma32(ca[c], ca[c], na);
      if (need_nb) E::mma32(cb[c], cb[c], nb);
    }
    if (sn < s_end) {
#pragma unroll
      for (int c = 0; c < FD_CHUNKS; ++c) { ca[c] = na_next[c]; cb[c] = nb_next[c]; }
    }
    s = sn;
  }

  // cross-wave sum through LDS
#pragma unroll
  for (int i = 0; i < 16; ++i) red[wave][acc_row(i, lane) * 32 + r] = acc[i];
  if (((r >> 2) & 1) == half) {   // this lane holds the diagonal element (r, r)
    const int idx = 4 * (r >> 3) + (r & 3);
    float da = 0.f, db = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      da = (i == idx) ? na[i] : da;
      db = (i == idx) ? nb[i] : db;
    }
    rnorm[wave][0][r] = da;
    rnorm[wave][1][r] = db;
  }
  __syncthreads();
  float *out = g.partial + ((int64_t)ks * g.n_tiles + tile) * FD_TILE_FLOATS;
  for (int e = threadIdx.x; e < 32 * 32; e += FD_THREADS)
    out[e] = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
  if (threadIdx.x < 64) {
    const int which = threadIdx.x >> 5, i = threadIdx.x & 31;
    out[32 * 32 + threadIdx.x] = (rnorm[0][which][i] + rnorm[1][which][i]) + (rnorm[2][which][i] + rnorm[3][which][i]);
  }
}

// One workgroup per 32 A rows.  Phase 1: squared norms of the block's rows and of its window's columns
// into LDS.  Phase 2: thread (row group t/32, column lane t%32) sweeps 4 rows x the column tiles; all
// loads of the partial slices are issued together (the slice loop is unrolled), the sum order is fixed.
constexpr int FD_MAX_KSPLIT = 16;

__device__ __forceinline__ double sum_slices(const float *p, int64_t ks_stride, int ksplit) {
  // every load is unconditional (surplus slices re-read the last one and are dropped afterwards): the
  // compiler then issues all of them before the first wait instead of one load per branch
  float v[FD_MAX_KSPLIT];
#pragma unroll
  for (int ks = 0; ks < FD_MAX_KSPLIT; ++ks) v[ks] = p[(ks < ksplit ? ks : ksplit - 1) * ks_stride];
#pragma unroll
  for (int ks = 0; ks < FD_MAX_KSPLIT; ++ks) v[ks] = (ks < ksplit) ? v[ks] : 0.f;
  double s = 0.0;
#pragma unroll
  for (int ks = 0; ks < FD_MAX_KSPLIT; ++ks) s += (double)v[ks];
  return s;
}

// ---------------------------------------------------------------------------------------------------------
// Windows that fit one 32 x 32 tile (at most 64 tokens): the epilogue AND the per-window selection (paper Step 2:
// the r A nodes with the lowest FD) in one kernel.  fd_partial_kernel leaves the partial tiles; one workgroup per
// tile sums them in their fixed order and finishes the tile in LDS: cosines, first minimum per row, rank of every
// A node among the keys (FD bits, position) of its window, then dst / per-target source counts / rank of each
// source in its group -- exactly what select_window_kernel derives from best_fd and best_dst.
// (Handing the tile to "the last workgroup to arrive" inside fd_partial_kernel was tried and dropped: the
// device-scope fence it needs writes back the L2 of the whole XCD and costs far more than a launch.)
struct SmallSelArgs {
  const int32_t *win_remove;
  int32_t *dst, *cnt, *src_rank;
};

struct SmallTileLds {
  double tile[32 * 32];
  double n2[2][32];             // |a|^2 per tile row, |b|^2 per tile column
  uint32_t row_key[32];         // order-preserving bits of the row's best FD (as stored in fp32)
  int row_col[32];              // best tile column (-1: none)
  int row_tok[32], col_tok[32]; // token of tile row / column, -1 for padding
  int slot_r[32];               // r of the window in slot s (clamped)
  uint32_t col_mask;            // bit c set: tile column c holds a B node
};

// One workgroup per tile: partial tiles summed in slice order, then the tile is finished in LDS.
// Every global load of the kernel is independent of the others (the token lists of the tile come from the
// record fd_partial_kernel left with slice 0), so all of them are in flight together.
__device__ __forceinline__ void fd_tail_select_body(const FdArgs &g, const SmallSelArgs &q, int tile, char *lds) {
  SmallTileLds &L = *reinterpret_cast<SmallTileLds *>(lds);
  const int tid = threadIdx.x;
  const int64_t ks_stride = (int64_t)g.n_tiles * FD_TILE_FLOATS;
  const float *base = g.partial + (int64_t)tile * FD_TILE_FLOATS;
  const int shift = (g.group > 1) ? (g.slot == 8 ? 3 : 4) : 5;   // tile row or column >> shift = its window slot

  // ---- metadata (wave 0) and partial sums (everyone)
  int m_tok = -1, m_off = 0, m_end = 0, m_rem = 0;
  if (tid < 64) {
    m_tok = reinterpret_cast<const int32_t *>(base + FD_TOK_OFFSET)[tid];   // rows 0..31, then columns 0..31
    const int rr = tid & 31;
    const int w = tile * g.group + (rr >> shift);
    const int wc = w < g.n_windows ? w : g.n_windows - 1;
    m_off = g.win_offsets[wc]; m_end = g.win_offsets[wc + 1]; m_rem = q.win_remove[wc];
    if (w >= g.n_windows) { m_end = m_off; m_rem = 0; }
  }
  // a tile without A rows or without B rows has no sums from fd_partial_kernel: they are not used either
  for (int e = tid; e < 32 * 32; e += FD_THREADS) L.tile[e] = sum_slices(base + e, ks_stride, g.ksplit);
  if (tid < 64) {
    L.n2[tid >> 5][tid & 31] = sum_slices(base + 32 * 32 + tid, ks_stride, g.ksplit);
    if (tid < 32) L.row_tok[tid] = m_tok; else L.col_tok[tid - 32] = m_tok;
    const unsigned long long cm = __ballot(tid >= 32 && m_tok >= 0);
    if (tid == 0) L.col_mask = (uint32_t)(cm >> 32);
    if (tid < 32 && (tid & ((1 << shift) - 1)) == 0) {   // first row of a window slot: its removal count
      const int v = m_end - m_off;
      const int cap = (g.group > 1) ? g.slot : 32;
      int nA = side_a(v, g.dir);
      nA = nA < cap ? nA : cap;
      int rr = m_rem < 0 ? 0 : (m_rem > nA ? nA : m_rem);
      if (side_b(v, g.dir) == 0) rr = 0;
      L.slot_r[tid >> shift] = rr;
    }
  }
  __syncthreads();

  // ---- FD and first minimum per row: 8 threads per row, 4 columns each
  constexpr int TPR = FD_THREADS / 32;
  constexpr int CPT = 32 / TPR;
  {
    const int rr = tid / TPR, cl = tid % TPR;
    const int ta = L.row_tok[rr];
    const int sw = rr >> shift;
    const uint32_t cols = L.col_mask & ((shift == 5) ? 0xffffffffu : (((1u << (1 << shift)) - 1u) << (sw << shift)));
    double best = __longlong_as_double(0x7ff0000000000000ll);
    int best_c = 0x7fffffff;
    const double a2 = L.n2[0][rr];
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = cl + TPR * k;
      const double dot = L.tile[rr * 32 + c];
      const double fd = divergence(g.metric, dot, a2, L.n2[1][c]);
      const bool live = ta >= 0 && ((cols >> c) & 1u);
      if (live && fd < best) { best = fd; best_c = c; }   // columns ascend: strict < keeps the first minimum
    }
#pragma unroll
    for (int m = TPR / 2; m >= 1; m >>= 1) {
      const double ob = __shfl_xor(best, m, 64);
      const int oc = __shfl_xor(best_c, m, 64);
      if (ob < best || (ob == best && oc < best_c)) { best = ob; best_c = oc; }
    }
    if (cl == 0) {
      const bool has = best_c != 0x7fffffff;
      float f = has ? (float)best : __uint_as_float(0x7f800000u);
      // a row without any finite score falls back to the first B node of its window
      const int first_c = cols ? __ffs((int)cols) - 1 : -1;
      const int bc = has ? best_c : first_c;
      if (!(f >= 0.f)) f = __uint_as_float(0x7f800000u);
      L.row_key[rr] = f32_order_key(f);
      L.row_col[rr] = bc;
      if (ta >= 0) {
        g.best_fd[ta] = f;
        g.best_dst[ta] = bc >= 0 ? L.col_tok[bc] : -1;
      }
    }
    if (cl == 1 && L.col_tok[rr] >= 0) {   // B rows carry no proposal
      g.best_fd[L.col_tok[rr]] = __uint_as_float(0x7f800000u);
      g.best_dst[L.col_tok[rr]] = -1;
    }
  }
  __syncthreads();

  // ---- selection by wave 0, row data in registers: lanes 0..31 act for the tile rows (A nodes), lanes 32..63
  // for the tile columns (B nodes).  Values of other rows are read with constant-lane broadcasts.
  if (tid < 64) {
    const int rr = tid & 31;
    const int tok = L.row_tok[rr], col = L.row_col[rr];
    const uint32_t key = L.row_key[rr];
    const int win = rr >> shift;
    const int valid = tok >= 0 ? 1 : 0;
    int rank = 0;
#pragma unroll
    for (int o = 0; o < 32; ++o) {
      const uint32_t ko = (uint32_t)__builtin_amdgcn_readlane((int)key, o);
      const int vo = __builtin_amdgcn_readlane(valid, o);
      rank += (vo && (o >> shift) == win && (ko < key || (ko == key && o < rr))) ? 1 : 0;
    }
    const bool sel = valid && col >= 0 && rank < L.slot_r[win];
    const uint32_t selmask = (uint32_t)__ballot(sel);   // lanes 0..31
    // rows: rank among the earlier sources of the same destination; columns: number of sources
    const bool is_col = tid >= 32;
    const int target = is_col ? rr : col;
    const int limit = is_col ? 32 : rr;
    int n = 0;
#pragma unroll
    for (int o = 0; o < 32; ++o) {
      const int co = __builtin_amdgcn_readlane(col, o);
      n += (((selmask >> o) & 1u) && (o >> shift) == win && co == target && o < limit) ? 1 : 0;
    }
    if (!is_col) {
      if (tok >= 0) {
        q.dst[tok] = sel ? L.col_tok[col] : -1;
        q.src_rank[tok] = sel ? n : 0;
        q.cnt[tok] = 0;
      }
    } else {
      const int tb = L.col_tok[rr];
      if (tb >= 0) {
        q.dst[tb] = -1;
        q.src_rank[tb] = 0;
        q.cnt[tb] = n;
      }
    }
  }
}

// Arguments of the small-window kernels from a plan and the caller's tensors (host side).
inline FdArgs make_fd_args(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                           const int32_t *win_offsets, const int32_t *win_tokens, float *partial, float *best_fd,
                           int32_t *best_dst) {
  FdArgs g{};
  g.X = X; g.ldx = ldx; g.d = d; g.n_windows = n_windows; g.sum_n = sum_n;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens;
  g.partial = partial; g.best_fd = best_fd; g.best_dst = best_dst;
  g.slot = plan.slot; g.group = plan.group; g.mt = plan.mt; g.nt = plan.nt;
  g.n_tiles = plan.n_tiles; g.ksplit = plan.ksplit; g.metric = plan.metric; g.dir = plan.dir;
  const int span = (dtype == 1) ? 64 : 32;
  g.n_spans = (d + span - 1) / span;
  g.spans_per_wg = (g.n_spans + plan.ksplit - 1) / plan.ksplit;
  return g;
}

}  // namespace lk
