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
#include "lk_fd_body.h"

namespace lk {

template <typename T>
__global__ __launch_bounds__(FD_THREADS, 3) void fd_partial_kernel(FdArgs g) {
  __shared__ __attribute__((aligned(16))) char lds[FD_PARTIAL_LDS];
  fd_partial_body<T>(g, blockIdx.x, lds);
}

__global__ __launch_bounds__(FD_THREADS) void fd_tail_select_kernel(FdArgs g, SmallSelArgs q) {
  __shared__ __attribute__((aligned(16))) char lds[sizeof(SmallTileLds)];
  fd_tail_select_body(g, q, blockIdx.x, lds);
}

__global__ __launch_bounds__(FD_THREADS) void fd_epilogue_kernel(FdArgs g) {
  __shared__ double nb2[FD_MAX_COLS];
  __shared__ double na2[32];
  const int rb = blockIdx.x;
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
  // Eight threads share a row of the block; a thread takes four neighbouring columns of every column tile, so the
  // slices of a tile arrive as ksplit 16-byte loads per thread, all in flight together (one round trip per column tile).
  const int r = threadIdx.x >> 3, sub = threadIdx.x & 7;
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
  const int nB = wi.nB < col_cap ? wi.nB : col_cap;
  double best = __longlong_as_double(0x7ff0000000000000ll);   // +inf
  int best_c = 0x7fffffff;
  const double a2 = na2[r];
  for (int t = 0; t < ncol_tiles; ++t) {
    const int tc0 = t * 32 + sub * 4;   // first of this thread's columns inside the block's tile row
    if (tc0 + 3 < col_base || tc0 >= col_base + nB) continue;   // none of the four belongs to this row's window
    const float *p = g.partial + (int64_t)(tile_row0 + t) * FD_TILE_FLOATS + r * 32 + sub * 4;
    f32x4 v[FD_MAX_KSPLIT];
#pragma unroll
    for (int ks = 0; ks < FD_MAX_KSPLIT; ++ks)   // surplus slices re-read the last one and are dropped
      v[ks] = *reinterpret_cast<const f32x4 *>(p + (ks < g.ksplit ? ks : g.ksplit - 1) * ks_stride);
    double dot[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int ks = 0; ks < FD_MAX_KSPLIT; ++ks) {
#pragma unroll
      for (int j = 0; j < 4; ++j) dot[j] += (ks < g.ksplit) ? (double)v[ks][j] : 0.0;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = tc0 + j - col_base;   // column inside the window
      if (a_valid && c >= 0 && c < nB) {
        const double fd = divergence(g.metric, dot[j], a2, nb2[tc0 + j]);
        if (fd < best) { best = fd; best_c = c; }   // columns ascend: strict < keeps the first minimum
      }
    }
  }
  // reduce over the eight lanes that share this row
#pragma unroll
  for (int m = 4; m >= 1; m >>= 1) {
    const double ob = __shfl_xor(best, m, 64);
    const int oc = __shfl_xor(best_c, m, 64);
    if (ob < best || (ob == best && oc < best_c)) { best = ob; best_c = oc; }
  }
  if (sub == 0 && a_valid) {
    const int a_tok = checked_token(g, wi.off + pos_a(l, g.dir));
    if (a_tok >= 0) {
      // no finite score at all (NaN rows): propose the first B node with FD = +inf, so that counts stay exact
      const bool has = best_c != 0x7fffffff;
      g.best_fd[a_tok] = has ? (float)best : __uint_as_float(0x7f800000u);
      g.best_dst[a_tok] = (wi.nB > 0) ? checked_token(g, wi.off + pos_b(has ? best_c : 0, g.dir)) : -1;
    }
  }
  if (sub == 1 && l < wi.nB) {   // B rows carry no proposal
    const int b_tok = checked_token(g, wi.off + pos_b(l, g.dir));
    if (b_tok >= 0) {
      g.best_fd[b_tok] = __uint_as_float(0x7f800000u);
      g.best_dst[b_tok] = -1;
    }
  }
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
  const FdArgs g = make_fd_args(plan, dtype, X, ldx, d, n_windows, sum_n, win_offsets, win_tokens, partial, best_fd, best_dst);
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

hipError_t launch_fd_partial(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                             const int32_t *win_offsets, const int32_t *win_tokens, float *partial, hipStream_t stream) {
  if (n_windows == 0 || plan.n_tiles == 0) return hipSuccess;
  const FdArgs g = make_fd_args(plan, dtype, X, ldx, d, n_windows, sum_n, win_offsets, win_tokens, partial, nullptr, nullptr);
  const dim3 grid((unsigned)(plan.n_tiles * plan.ksplit));
  if (dtype == 1) hipLaunchKernelGGL(fd_partial_kernel<bf16_t>, grid, dim3(FD_THREADS), 0, stream, g);
  else hipLaunchKernelGGL(fd_partial_kernel<float>, grid, dim3(FD_THREADS), 0, stream, g);
  return hipGetLastError();
}

hipError_t launch_fd(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                     const int32_t *win_offsets, const int32_t *win_tokens, float *partial, float *best_fd,
                     int32_t *best_dst, hipStream_t stream) {
  if (n_windows == 0 || plan.n_tiles == 0) return hipSuccess;
  const FdArgs g = make_fd_args(plan, dtype, X, ldx, d, n_windows, sum_n, win_offsets, win_tokens, partial, best_fd, best_dst);
  const dim3 grid((unsigned)(plan.n_tiles * plan.ksplit));
  if (dtype == 1) hipLaunchKernelGGL(fd_partial_kernel<bf16_t>, grid, dim3(FD_THREADS), 0, stream, g);
  else hipLaunchKernelGGL(fd_partial_kernel<float>, grid, dim3(FD_THREADS), 0, stream, g);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fd_epilogue_kernel, dim3((unsigned)plan.n_rowblocks), dim3(FD_THREADS), 0, stream, g);
  return hipGetLastError();
}

}  // namespace lk
