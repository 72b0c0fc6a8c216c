// Feature divergence and the best edge of every A node (paper Sec. 3.2.1 Steps 1-2, Eq. "similarity").
//
// For every window the |A| x |B| block of inner products <x_a, x_b> is a dense contraction over the
// hidden dimension and runs on the matrix cores (bf16 -> v_mfma_f32_32x32x16_bf16, fp32 ->
// v_mfma_f32_32x32x2_f32), fp32 accumulation.  The squared norms come from the same instruction
// (a tile times itself: the diagonal is |x|^2), so a token identical to another one gets cos == 1 exactly.
// The FD matrix is never written: an epilogue reduces each A row to (min FD, arg min) directly.
//
//   fd_partial_kernel : one workgroup = one 32x32 tile x one slice of the hidden axis; the four waves of
//                       the workgroup take interleaved 128-byte runs of that slice straight from global
//                       memory into MFMA operands (no LDS staging: nothing is reused across waves), are
//                       summed through LDS and stored as a partial tile.
//   fd_epilogue_kernel: sums the partial tiles over the slices in a fixed order (fp64), forms
//                       cos = dot / sqrt(|a|^2 |b|^2), FD = max(1 - cos, 0) and keeps the first minimum per row.
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
};

struct WinInfo { int off, nA, nB; };

__device__ __forceinline__ WinInfo win_info(const FdArgs &g, int w) {
  WinInfo wi{0, 0, 0};
  if (w < g.n_windows) {
    wi.off = g.win_offsets[w];
    const int v = g.win_offsets[w + 1] - wi.off;
    wi.nA = (v + 1) >> 1;
    wi.nB = v >> 1;
  }
  return wi;
}

__device__ __forceinline__ int checked_token(const FdArgs &g, int idx) {
  const int t = g.win_tokens[idx];
  return ((unsigned)t < (unsigned)g.sum_n) ? t : -1;
}

template <typename T>
__global__ __launch_bounds__(FD_THREADS) void fd_partial_kernel(FdArgs g) {
  using E = Elem<T>;
  constexpr int EPC = E::PER_CHUNK;
  constexpr int LANE_ELEMS = FD_CHUNKS * EPC;   // contiguous elements of one lane in a span
  constexpr int SPAN = 2 * LANE_ELEMS;          // elements of a row covered by one span

  __shared__ float red[FD_WAVES][32 * 32];
  __shared__ float rnorm[FD_WAVES][2][32];

  const int tile = blockIdx.x % g.n_tiles;
  const int ks = blockIdx.x / g.n_tiles;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, half = lane >> 5;

  // rows of this tile
  int a_tok = -1, b_tok = -1;
  bool need_na = true, need_nb = true;
  if (g.group > 1) {
    const int s = r / g.slot, l = r - s * g.slot;
    const WinInfo wi = win_info(g, tile * g.group + s);
    if (l < wi.nA) a_tok = checked_token(g, wi.off + 2 * l);
    if (l < wi.nB) b_tok = checked_token(g, wi.off + 2 * l + 1);
  } else {
    const int per = g.mt * g.nt;
    const int w = tile / per, rem = tile - w * per;
    const int mt = rem / g.nt, nt = rem - mt * g.nt;
    const WinInfo wi = win_info(g, w);
    const int la = mt * 32 + r, lb = nt * 32 + r;
    if (la < wi.nA) a_tok = checked_token(g, wi.off + 2 * la);
    if (lb < wi.nB) b_tok = checked_token(g, wi.off + 2 * lb + 1);
    need_na = (nt == 0);
    need_nb = (mt == 0);
  }
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

__global__ __launch_bounds__(FD_THREADS) void fd_epilogue_kernel(FdArgs g) {
  __shared__ double nb2[FD_MAX_COLS];
  __shared__ double na2[32];
  const int rb = blockIdx.x;
  const int c32 = threadIdx.x & 31, rgrp = threadIdx.x >> 5;   // 8 row groups
  const int64_t ks_stride = (int64_t)g.n_tiles * FD_TILE_FLOATS;
  const int per = g.mt * g.nt;

  int tile_row0;            // tile holding the dots of (this row block, column tile 0)
  int tile_col0;            // tile holding |b|^2 of column tile 0
  int w_single = 0, m_single = 0;
  if (g.group > 1) {
    tile_row0 = tile_col0 = rb;
  } else {
    w_single = rb / g.mt;
    m_single = rb - w_single * g.mt;
    tile_row0 = w_single * per + m_single * g.nt;
    tile_col0 = w_single * per;
  }
  const int ncol_tiles = (g.group > 1) ? 1 : g.nt;
  for (int c = threadIdx.x; c < ncol_tiles * 32 + 32; c += FD_THREADS) {
    if (c < ncol_tiles * 32)
      nb2[c] = sum_slices(g.partial + (int64_t)(tile_col0 + (c >> 5)) * FD_TILE_FLOATS + 32 * 32 + 32 + (c & 31),
                          ks_stride, g.ksplit);
    else
      na2[c - ncol_tiles * 32] = sum_slices(g.partial + (int64_t)tile_row0 * FD_TILE_FLOATS + 32 * 32 + (c - ncol_tiles * 32),
                                            ks_stride, g.ksplit);
  }
  __syncthreads();

  const int col_cap = (g.group > 1) ? g.slot : g.nt * 32;   // columns this launch really tiled
#pragma unroll
  for (int rp = 0; rp < 4; ++rp) {
    const int r = rp * 8 + rgrp;
    WinInfo wi;
    int l, col_base;   // local A position; first tile column of this row's window
    if (g.group > 1) {
      const int s = r / g.slot;
      l = r - s * g.slot;
      wi = win_info(g, rb * g.group + s);
      col_base = s * g.slot;
    } else {
      wi = win_info(g, w_single);
      l = m_single * 32 + r;
      col_base = 0;
    }
    const bool a_valid = l < wi.nA;
    if (wi.nB > col_cap) wi.nB = col_cap;
    double best = __longlong_as_double(0x7ff0000000000000ll);   // +inf
    int best_c = 0x7fffffff;
    if (a_valid && wi.nB > 0) {
      const double a2 = na2[r];
      for (int c = c32; c < wi.nB; c += 32) {
        const int tc = col_base + c;   // column inside this row block's tile row
        const double dot = sum_slices(g.partial + (int64_t)(tile_row0 + (tc >> 5)) * FD_TILE_FLOATS + r * 32 + (tc & 31),
                                      ks_stride, g.ksplit);
        const double b2 = nb2[tc];
        double den;
        if (a2 >= NORM_EPS * NORM_EPS && b2 >= NORM_EPS * NORM_EPS) den = sqrt(a2 * b2);
        else den = fmax(sqrt(a2), NORM_EPS) * fmax(sqrt(b2), NORM_EPS);
        const double fd = fmax(1.0 - dot / den, 0.0);
        if (fd < best) { best = fd; best_c = c; }   // columns ascend: strict < keeps the first minimum
      }
    }
    // reduce over the 32 lanes of the half-wave that share this row
#pragma unroll
    for (int m = 16; m >= 1; m >>= 1) {
      const double ob = __shfl_xor(best, m, 64);
      const int oc = __shfl_xor(best_c, m, 64);
      if (ob < best || (ob == best && oc < best_c)) { best = ob; best_c = oc; }
    }
    if (c32 == 0 && a_valid) {
      const int a_tok = checked_token(g, wi.off + 2 * l);
      if (a_tok >= 0) {
        // no finite score at all (NaN rows): propose the first B node with FD = +inf, so that counts stay exact
        const bool has = best_c != 0x7fffffff;
        g.best_fd[a_tok] = has ? (float)best : __uint_as_float(0x7f800000u);
        g.best_dst[a_tok] = (wi.nB > 0) ? checked_token(g, wi.off + 2 * (has ? best_c : 0) + 1) : -1;
      }
    }
    if (c32 == 1 && l < wi.nB) {   // B rows carry no proposal
      const int b_tok = checked_token(g, wi.off + 2 * l + 1);
      if (b_tok >= 0) {
        g.best_fd[b_tok] = __uint_as_float(0x7f800000u);
        g.best_dst[b_tok] = -1;
      }
    }
  }
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
  int row_col[32], row_sel[32]; // best tile column (-1: none), 1 if the row is merged away
  int row_tok[32], col_tok[32]; // token of tile row / column, -1 for padding
  int row_win[32], col_win[32]; // window slot of tile row / column
  int slot_r[32];               // r of the window in slot s (clamped)
};

// Finishes one tile from its summed dots and squared norms (in L.tile / L.n2).  Called by a whole workgroup.
template <int THREADS>
__device__ __forceinline__ void small_tile_tail(const FdArgs &g, const SmallSelArgs &q, int tile, SmallTileLds &L) {
  const int tid = threadIdx.x;
  if (tid < 32) {
    const int r = tid;
    int a_tok = -1, b_tok = -1, my_slot = 0, l = r;
    WinInfo wi;
    if (g.group > 1) {
      my_slot = r / g.slot;
      l = r - my_slot * g.slot;
      wi = win_info(g, tile * g.group + my_slot);
    } else {
      wi = win_info(g, tile);
    }
    if (l < wi.nA) a_tok = checked_token(g, wi.off + 2 * l);
    if (l < wi.nB) b_tok = checked_token(g, wi.off + 2 * l + 1);
    L.row_tok[r] = a_tok; L.col_tok[r] = b_tok; L.row_win[r] = my_slot; L.col_win[r] = my_slot;
    if (l == 0) {   // first row of a window slot: its removal count
      const int w = (g.group > 1) ? tile * g.group + my_slot : tile;
      int rr = (w < g.n_windows) ? q.win_remove[w] : 0;
      const int cap = (g.group > 1) ? g.slot : 32;
      const int nA = wi.nA < cap ? wi.nA : cap;
      rr = rr < 0 ? 0 : (rr > nA ? nA : rr);
      if (wi.nB == 0) rr = 0;
      L.slot_r[my_slot] = rr;
    }
  }
  __syncthreads();
  // FD and first minimum per row: THREADS/32 threads per row
  constexpr int TPR = THREADS / 32;          // threads per row (8 or 16)
  constexpr int CPT = 32 / TPR;              // columns per thread
  {
    const int rr = tid / TPR, cl = tid % TPR;
    const int ta = L.row_tok[rr];
    const int sw = L.row_win[rr];
    double best = __longlong_as_double(0x7ff0000000000000ll);
    int best_c = 0x7fffffff;
    const double a2 = L.n2[0][rr];
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = cl + TPR * k;
      if (ta >= 0 && L.col_tok[c] >= 0 && L.col_win[c] == sw) {
        const double dot = L.tile[rr * 32 + c];
        const double b2 = L.n2[1][c];
        double den;
        if (a2 >= NORM_EPS * NORM_EPS && b2 >= NORM_EPS * NORM_EPS) den = sqrt(a2 * b2);
        else den = fmax(sqrt(a2), NORM_EPS) * fmax(sqrt(b2), NORM_EPS);
        const double fd = fmax(1.0 - dot / den, 0.0);
        if (fd < best) { best = fd; best_c = c; }   // columns ascend: strict < keeps the first minimum
      }
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
      // first column of the row's window: the fall-back partner of a row without any finite score
      int first_c = -1;
      for (int c = 0; c < 32; ++c)
        if (first_c < 0 && L.col_tok[c] >= 0 && L.col_win[c] == sw) first_c = c;
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
  // selection: rank of every A node among the keys (FD, position) of its window
  if (tid < 32) {
    const int rr = tid;
    int sel = 0;
    if (L.row_tok[rr] >= 0 && L.row_col[rr] >= 0) {
      const uint64_t key = ((uint64_t)L.row_key[rr] << 32) | (uint32_t)rr;
      int rank = 0;
      for (int o = 0; o < 32; ++o)
        if (L.row_tok[o] >= 0 && L.row_win[o] == L.row_win[rr] && ((((uint64_t)L.row_key[o]) << 32) | (uint32_t)o) < key) ++rank;
      sel = rank < L.slot_r[L.row_win[rr]];
    }
    L.row_sel[rr] = sel;
  }
  __syncthreads();
  if (tid < 32) {            // A rows: destination and rank among the sources of that destination
    const int rr = tid, ta = L.row_tok[rr];
    if (ta >= 0) {
      int rank = 0;
      if (L.row_sel[rr])
        for (int o = 0; o < rr; ++o)
          if (L.row_sel[o] && L.row_win[o] == L.row_win[rr] && L.row_col[o] == L.row_col[rr]) ++rank;
      q.dst[ta] = L.row_sel[rr] ? L.col_tok[L.row_col[rr]] : -1;
      q.src_rank[ta] = rank;
      q.cnt[ta] = 0;
    }
  } else if (tid < 64) {     // B columns: number of sources
    const int cc = tid - 32, tb = L.col_tok[cc];
    if (tb >= 0) {
      int n = 0;
      for (int o = 0; o < 32; ++o)
        if (L.row_sel[o] && L.row_win[o] == L.col_win[cc] && L.row_col[o] == cc) ++n;
      q.dst[tb] = -1;
      q.src_rank[tb] = 0;
      q.cnt[tb] = n;
    }
  }
}

// One workgroup per tile: partial tiles summed in slice order, then the tile is finished in LDS.
__global__ __launch_bounds__(FD_THREADS) void fd_tail_select_kernel(FdArgs g, SmallSelArgs q) {
  __shared__ SmallTileLds L;
  const int tile = blockIdx.x, tid = threadIdx.x;
  const int64_t ks_stride = (int64_t)g.n_tiles * FD_TILE_FLOATS;
  const float *base = g.partial + (int64_t)tile * FD_TILE_FLOATS;
  // a tile without A rows or without B rows was never written by fd_partial_kernel: its sums are not used either
  for (int e = tid; e < 32 * 32; e += FD_THREADS) L.tile[e] = sum_slices(base + e, ks_stride, g.ksplit);
  if (tid < 64) L.n2[tid >> 5][tid & 31] = sum_slices(base + 32 * 32 + tid, ks_stride, g.ksplit);
  __syncthreads();
  small_tile_tail<FD_THREADS>(g, q, tile, L);
}

FdPlan make_fd_small_fused_plan(int n_windows, int max_window_tokens, int d, int dtype_bytes) {
  FdPlan p{};
  const int maxA = (max_window_tokens + 1) / 2;
  if (maxA > 32) return p;   // n_tiles == 0: not applicable
  return make_fd_plan(n_windows, max_window_tokens, d, dtype_bytes);   // single-tile windows: mt == nt == 1
}

hipError_t launch_fd_select_small(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows,
                                  int sum_n, const int32_t *win_offsets, const int32_t *win_tokens,
                                  const int32_t *win_remove, float *partial, float *best_fd, int32_t *best_dst,
                                  int32_t *dst, int32_t *cnt, int32_t *src_rank, hipStream_t stream) {
  if (n_windows == 0 || plan.n_tiles == 0) return hipSuccess;
  FdArgs g{};
  g.X = X; g.ldx = ldx; g.d = d; g.n_windows = n_windows; g.sum_n = sum_n;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens;
  g.partial = partial; g.best_fd = best_fd; g.best_dst = best_dst;
  g.slot = plan.slot; g.group = plan.group; g.mt = 1; g.nt = 1; g.n_tiles = plan.n_tiles; g.ksplit = plan.ksplit;
  const int span = (dtype == 1) ? 64 : 32;
  g.n_spans = (d + span - 1) / span;
  g.spans_per_wg = (g.n_spans + plan.ksplit - 1) / plan.ksplit;
  const dim3 grid((unsigned)(plan.n_tiles * plan.ksplit));
  if (dtype == 1) hipLaunchKernelGGL(fd_partial_kernel<bf16_t>, grid, dim3(FD_THREADS), 0, stream, g);
  else hipLaunchKernelGGL(fd_partial_kernel<float>, grid, dim3(FD_THREADS), 0, stream, g);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  SmallSelArgs q{win_remove, dst, cnt, src_rank};
  hipLaunchKernelGGL(fd_tail_select_kernel, dim3((unsigned)plan.n_tiles), dim3(FD_THREADS), 0, stream, g, q);
  return hipGetLastError();
}

FdPlan make_fd_plan(int n_windows, int max_window_tokens, int d, int dtype_bytes) {
  FdPlan p{};
  const int maxA = (max_window_tokens + 1) / 2, maxB = max_window_tokens / 2;
  if (maxA <= 16) {
    p.slot = maxA <= 8 ? 8 : 16;
    p.group = 32 / p.slot;
    p.mt = p.nt = 1;
    p.n_tiles = (n_windows + p.group - 1) / p.group;
    p.n_rowblocks = p.n_tiles;
  } else {
    p.slot = 0;
    p.group = 1;
    p.mt = (maxA + 31) / 32;
    p.nt = maxB > 0 ? (maxB + 31) / 32 : 1;
    p.n_tiles = n_windows * p.mt * p.nt;
    p.n_rowblocks = n_windows * p.mt;
  }
  const int span = (dtype_bytes == 2) ? 64 : 32;
  const int n_spans = (d + span - 1) / span;
  const int max_ks = n_spans / FD_WAVES > 0 ? n_spans / FD_WAVES : 1;
  int ks = 1;
  while ((int64_t)p.n_tiles * ks < 1024 && ks * 2 <= max_ks && ks * 2 <= 16) ks *= 2;   // 16 = FD_MAX_KSPLIT
  p.ksplit = ks;
  p.partial_floats = (size_t)p.n_tiles * ks * FD_TILE_FLOATS;
  return p;
}

hipError_t launch_fd(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                     const int32_t *win_offsets, const int32_t *win_tokens, float *partial, float *best_fd,
                     int32_t *best_dst, hipStream_t stream) {
  if (n_windows == 0 || plan.n_tiles == 0) return hipSuccess;
  FdArgs g{};
  g.X = X; g.ldx = ldx; g.d = d; g.n_windows = n_windows; g.sum_n = sum_n;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens;
  g.partial = partial; g.best_fd = best_fd; g.best_dst = best_dst;
  g.slot = plan.slot; g.group = plan.group; g.mt = plan.mt; g.nt = plan.nt;
  g.n_tiles = plan.n_tiles; g.ksplit = plan.ksplit;
  const int span = (dtype == 1) ? 64 : 32;
  g.n_spans = (d + span - 1) / span;
  g.spans_per_wg = (g.n_spans + plan.ksplit - 1) / plan.ksplit;
  const dim3 grid((unsigned)(plan.n_tiles * plan.ksplit));
  if (dtype == 1) hipLaunchKernelGGL(fd_partial_kernel<bf16_t>, grid, dim3(FD_THREADS), 0, stream, g);
  else hipLaunchKernelGGL(fd_partial_kernel<float>, grid, dim3(FD_THREADS), 0, stream, g);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fd_epilogue_kernel, dim3((unsigned)plan.n_rowblocks), dim3(FD_THREADS), 0, stream, g);
  return hipGetLastError();
}

}  // namespace lk
