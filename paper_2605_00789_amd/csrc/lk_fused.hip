// Scores and selection of one step in three launches on ONE stream (paper Sec. 3.2.1 Steps 1-3).
//
// The prompt-guidance weight xi (two passes over the keys, then a sum over heads) and the feature divergence with
// its selection (partial tiles, tile tail, index scan) are two chains of three short kernels each; neither depends
// on the other until the merge.  Run on two streams they overlap, but every fork and join of the streams costs about
// as much as one of these kernels.  Here the k-th kernels of the two chains share a launch instead: the first
// workgroups of a launch run the xi pass, the rest the FD step (device bodies from lk_xi_body.h / lk_fd_body.h;
// the LDS block is the larger of the two needs, registers likewise).
//
//   launch 1   xi pass 1 (row statistics)      |  FD partial tiles               (workgroups of the two kinds alternate)
//   launch 2   xi pass 2 (column sums)         |  tile tail: epilogue + per-window selection     (tails first)
//   launch 3   xi heads summed                 |  index scan                     (select_scan_kernel<true>)
//
// Applies to windows of at most 64 tokens (one tile per window); results are bit-identical to the separate kernels.
#include "lk_fd_body.h"
#include "lk_xi_body.h"

namespace lk {

template <int A, int B> struct MaxOf { static constexpr int value = A > B ? A : B; };

template <typename T, int DH, int RW>
__global__ __launch_bounds__(XI_THREADS, 3) void rowstat_partial_kernel(XiArgs x, int n_xi_blocks, FdArgs f) {
  static_assert(XI_THREADS == FD_THREADS, "both bodies are written for 256 threads");
  __shared__ __attribute__((aligned(16))) char lds[MaxOf<XiStage<T, DH, RW>::LDS_ROWSTAT, FD_PARTIAL_LDS>::value];
  // the two kinds of workgroup alternate, so that both chains get the chip from the start of the launch
  const int n_fd_blocks = f.n_tiles * f.ksplit;
  const int paired = 2 * (n_xi_blocks < n_fd_blocks ? n_xi_blocks : n_fd_blocks);
  const int i = blockIdx.x;
  bool is_xi;
  int id;
  if (i < paired) { is_xi = (i & 1) == 0; id = i >> 1; }
  else { is_xi = n_xi_blocks > n_fd_blocks; id = i - paired / 2; }
  if (is_xi) xi_rowstat_body<T, DH, RW>(x, id, lds);
  else fd_partial_body<T>(f, id, lds);
}

template <typename T, int DH, int RW, bool VISION_LSE>
__global__ __launch_bounds__(XI_THREADS) void colsum_tail_kernel(XiArgs x, int n_xi_blocks, FdArgs f, SmallSelArgs q) {
  __shared__ __attribute__((aligned(16))) char lds[MaxOf<XiStage<T, DH, RW>::LDS_COLSUM, (int)sizeof(SmallTileLds)>::value];
  // the few tile tails go first: they are the longer dependency chain and must not wait for a free slot
  if ((int)blockIdx.x < f.n_tiles) fd_tail_select_body(f, q, blockIdx.x, lds);
  else xi_colsum_body<T, DH, RW, VISION_LSE>(x, blockIdx.x - f.n_tiles, lds);
}

template <typename T, int DH, int RW>
static hipError_t launch_two(const XiArgs &x, int n_xi_blocks, bool pass1, bool vision_lse, const FdArgs &f,
                             const SmallSelArgs &q, hipStream_t stream) {
  const unsigned g1 = (unsigned)((pass1 ? n_xi_blocks : 0) + f.n_tiles * f.ksplit);
  hipLaunchKernelGGL((rowstat_partial_kernel<T, DH, RW>), dim3(g1), dim3(XI_THREADS), 0, stream, x,
                     pass1 ? n_xi_blocks : 0, f);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const unsigned g2 = (unsigned)(n_xi_blocks + f.n_tiles);
  if (vision_lse)
    hipLaunchKernelGGL((colsum_tail_kernel<T, DH, RW, true>), dim3(g2), dim3(XI_THREADS), 0, stream, x, n_xi_blocks, f, q);
  else
    hipLaunchKernelGGL((colsum_tail_kernel<T, DH, RW, false>), dim3(g2), dim3(XI_THREADS), 0, stream, x, n_xi_blocks, f, q);
  return hipGetLastError();
}

template <typename T, int DH>
static hipError_t launch_two_t(const XiArgs &x, int n_xi_blocks, bool pass1, bool vision_lse, int max_t, const FdArgs &f,
                               const SmallSelArgs &q, hipStream_t stream) {
  if constexpr (xi_long_chunks_fit<T, DH>()) {
    if (max_t > 64) return launch_two<T, DH, 128>(x, n_xi_blocks, pass1, vision_lse, f, q, stream);
  }
  return launch_two<T, DH, 64>(x, n_xi_blocks, pass1, vision_lse, f, q, stream);
}

hipError_t launch_score_select_fused(const XiPlan &xp, const FdPlan &fp, int dtype, int xi_mode, int batch, int heads,
                                     int head_dim, int d, int n_windows, int sum_n, int sum_t, const int32_t *cu_vis,
                                     const int32_t *cu_txt, const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                     const void *K, int64_t k_tok_stride, int64_t k_head_stride, const float *lse,
                                     float scale, float *stats, float *xi_part, float *xi, const void *X, int64_t ldx,
                                     const int32_t *win_offsets, const int32_t *win_tokens, const int32_t *win_remove,
                                     float *partial, float *best_fd, int32_t *best_dst, int32_t *dst, int32_t *cnt,
                                     int32_t *src_rank, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                                     int32_t *cu_vis_out, hipStream_t stream) {
  const XiArgs x = make_xi_args(xp, xi_mode, batch, heads, sum_n, sum_t, cu_vis, cu_txt, Q, q_tok_stride, q_head_stride, K,
                                k_tok_stride, k_head_stride, lse, scale, stats, xi_part, xi);
  const FdArgs f = make_fd_args(fp, dtype, X, ldx, d, n_windows, sum_n, win_offsets, win_tokens, partial, best_fd, best_dst);
  const SmallSelArgs q{win_remove, dst, cnt, src_rank};
  const int n_xi_blocks = batch * heads * xp.max_vis_blocks;
  const bool pass1 = (xi_mode == 0 && lse == nullptr);
  const bool vision_lse = (xi_mode == 1);
  const int max_t = xp.max_text_tiles * 32;
  hipError_t e = hipErrorInvalidValue;
#define LK_CASE(TT, DHV) e = launch_two_t<TT, DHV>(x, n_xi_blocks, pass1, vision_lse, max_t, f, q, stream)
  if (dtype == 1) {
    if (head_dim == 128) LK_CASE(bf16_t, 128);
    else if (head_dim == 64) LK_CASE(bf16_t, 64);
    else if (head_dim == 32) LK_CASE(bf16_t, 32);
  } else {
    if (head_dim == 128) LK_CASE(float, 128);
    else if (head_dim == 64) LK_CASE(float, 64);
    else if (head_dim == 32) LK_CASE(float, 32);
  }
#undef LK_CASE
  if (e != hipSuccess) return e;
  return launch_select_scan_heads(batch, sum_n, cu_vis, dst, new_index, grp_offsets, grp_src, cu_vis_out, cnt, src_rank, x,
                                  stream);
}

}  // namespace lk
