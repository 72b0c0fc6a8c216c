// Prompt-guidance weight xi (paper Sec. 3.2.1 Step 3, Eq. "attention-factor"):
//   xi_i = sum over heads h and prompt tokens j of the attention weight between vision token i and j.
// The logits q.k * scale of one head are a (prompt x vision x head_dim) contraction and run on the
// matrix cores; nothing of the attention matrix is ever written to memory.
//
//   text-query mode, no lse handed in:
//     pass 1  per (sequence, head, 128 vision tokens): for every prompt row the maximum and the sum of
//             exponentials over those vision keys, one (max, sum) pair per block.
//     pass 2  per (sequence, head, 128 vision tokens): merges the pairs of its prompt rows, recomputes the
//             logits and adds exp(logit - max) / sum over the prompt rows -> per-head partial xi.
//   lse handed in (either mode): pass 2 only.
//   pass 3  sums the heads in a fixed order and applies the floor.
// Batches with enough (sequence, head) pairs run passes 1 and 2 as one launch with one workgroup per pair
// (lk_xi_seq.hip); pass 3 is the same.
// The operand whose index must be reduced inside a lane is always fed as the MFMA row operand:
// accumulator registers run over rows, lanes over columns, so both reductions stay in registers.
#include "lk_xi_body.h"

namespace lk {

template <typename T, int DH, int RW>
__global__ __launch_bounds__(XI_THREADS) void xi_rowstat_kernel(XiArgs g) {
  __shared__ __attribute__((aligned(16))) char lds[XiStage<T, DH, RW>::LDS_ROWSTAT];
  xi_rowstat_body<T, DH, RW>(g, blockIdx.x, lds);
}

template <typename T, int DH, int RW, bool VISION_LSE>
__global__ __launch_bounds__(XI_THREADS) void xi_colsum_kernel(XiArgs g) {
  __shared__ __attribute__((aligned(16))) char lds[XiStage<T, DH, RW>::LDS_COLSUM];
  xi_colsum_body<T, DH, RW, VISION_LSE>(g, blockIdx.x, lds);
}

__global__ __launch_bounds__(64) void xi_heads_kernel(XiArgs g) { xi_heads_body(g, blockIdx.x * 64 + threadIdx.x); }

XiPlan make_xi_plan(int batch, const int32_t *h_cu_vis, const int32_t *h_cu_txt, int heads, int xi_mode) {
  XiPlan p{};
  if (xi_mode == 2 || !h_cu_txt) return p;
  int max_t = 0, max_n = 0;
  for (int b = 0; b < batch; ++b) {
    max_t = h_cu_txt[b + 1] - h_cu_txt[b] > max_t ? h_cu_txt[b + 1] - h_cu_txt[b] : max_t;
    max_n = h_cu_vis[b + 1] - h_cu_vis[b] > max_n ? h_cu_vis[b + 1] - h_cu_vis[b] : max_n;
  }
  p.max_text_tiles = (max_t + 31) / 32;
  p.max_vis_blocks = (max_n + 127) / 128;
  p.stat_floats = (size_t)heads * (size_t)h_cu_txt[batch] * (size_t)p.max_vis_blocks * 2;
  p.part_floats = (size_t)heads * (size_t)h_cu_vis[batch];
  return p;
}

template <typename T, int DH, int RW>
static hipError_t launch_xi_rw(const XiPlan &plan, const XiArgs &g, int xi_mode, hipStream_t stream) {
  const bool vision_lse = (xi_mode == 1);
  const unsigned grid = (unsigned)(g.batch * g.heads * plan.max_vis_blocks);
  if (xi_mode == 0 && g.lse == nullptr) {
    if (grid) hipLaunchKernelGGL((xi_rowstat_kernel<T, DH, RW>), dim3(grid), dim3(XI_THREADS), 0, stream, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (grid) {
    if (vision_lse)
      hipLaunchKernelGGL((xi_colsum_kernel<T, DH, RW, true>), dim3(grid), dim3(XI_THREADS), 0, stream, g);
    else
      hipLaunchKernelGGL((xi_colsum_kernel<T, DH, RW, false>), dim3(grid), dim3(XI_THREADS), 0, stream, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (g.sum_n) hipLaunchKernelGGL(xi_heads_kernel, dim3((unsigned)((g.sum_n + 63) / 64)), dim3(64), 0, stream, g);
  return hipGetLastError();
}

template <typename T, int DH>
static hipError_t launch_xi_t(const XiPlan &plan, const XiArgs &g, int xi_mode, int max_t, hipStream_t stream) {
  if constexpr (xi_long_chunks_fit<T, DH>()) {
    if (max_t > 64) return launch_xi_rw<T, DH, 128>(plan, g, xi_mode, stream);
  }
  return launch_xi_rw<T, DH, 64>(plan, g, xi_mode, stream);
}

hipError_t launch_xi(const XiPlan &plan, int dtype, int xi_mode, int batch, int heads, int head_dim, int sum_n,
                     int sum_t, const int32_t *cu_vis, const int32_t *cu_txt, const void *Q, int64_t q_tok_stride,
                     int64_t q_head_stride, const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                     const float *lse, float scale, float *stats, float *xi_part, float *xi, hipStream_t stream) {
  const XiArgs g = make_xi_args(plan, xi_mode, batch, heads, sum_n, sum_t, cu_vis, cu_txt, Q, q_tok_stride, q_head_stride, K,
                                k_tok_stride, k_head_stride, lse, scale, stats, xi_part, xi);
  const int max_t = plan.max_text_tiles * 32;
  if (xi_seq_applies(plan, xi_mode, lse, batch, heads)) {
    const hipError_t e = launch_xi_seq(g, dtype, head_dim, stream);
    if (e != hipSuccess) return e;
    if (g.sum_n) hipLaunchKernelGGL(xi_heads_kernel, dim3((unsigned)((g.sum_n + 63) / 64)), dim3(64), 0, stream, g);
    return hipGetLastError();
  }
#define LK_XI_CASE(TT, DHV) return launch_xi_t<TT, DHV>(plan, g, xi_mode, max_t, stream)
  if (dtype == 1) {
    if (head_dim == 128) LK_XI_CASE(bf16_t, 128);
    if (head_dim == 64) LK_XI_CASE(bf16_t, 64);
    if (head_dim == 32) LK_XI_CASE(bf16_t, 32);
  } else {
    if (head_dim == 128) LK_XI_CASE(float, 128);
    if (head_dim == 64) LK_XI_CASE(float, 64);
    if (head_dim == 32) LK_XI_CASE(float, 32);
  }
#undef LK_XI_CASE
  return hipErrorInvalidValue;
}

}  // namespace lk
