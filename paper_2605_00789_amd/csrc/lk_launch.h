// Host-side launch plans and launcher declarations (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lk {

// The bipartite split of a window's list (Sec. 3.2.1 Step 1) and the direction of the merge (message-passing
// paragraph: the reverse direction is defined analogously).  dir 0: the tokens at list positions 0, 2, 4, ... propose
// and merge into the tokens at positions 1, 3, 5, ...; dir 1: the odd positions propose, the even ones receive.  In
// the kernels "A" is always the proposing side and "B" the receiving side.
__host__ __device__ __forceinline__ int side_a(int v, int dir) { return (v + 1 - dir) >> 1; }
__host__ __device__ __forceinline__ int side_b(int v, int dir) { return (v + dir) >> 1; }
__host__ __device__ __forceinline__ int pos_a(int i, int dir) { return 2 * i + dir; }
__host__ __device__ __forceinline__ int pos_b(int j, int dir) { return 2 * j + 1 - dir; }

// ---- feature divergence (Steps 1-2) ------------------------------------------------------
// The |A_w| x |B_w| cosine blocks are cut into 32x32 tiles.  Small windows are packed several to
// a tile (block diagonal): `slot` rows/cols per window, `group` windows per tile.  Large windows
// get mt x nt tiles each.  The d axis is split over `ksplit` workgroups (and the 4 waves of each);
// partial tiles are summed in a fixed order by the epilogue.
struct FdPlan {
  int slot;         // rows (and cols) reserved per window in a packed tile; 0 when group == 1
  int group;        // windows per tile
  int mt, nt;       // tiles per window along A and B (group == 1)
  int n_tiles;      // tile jobs
  int n_rowblocks;  // epilogue jobs (one per 32 A rows)
  int ksplit;
  size_t partial_floats;   // n_tiles * ksplit * FD_TILE_FLOATS
  int metric;              // 0 cosine FD, 1 Euclidean, 2 squared L2 (set by the caller after planning)
  int dir;                 // 0: even list positions propose, 1: odd ones (set by the caller after planning; a plan for
                           // dir 1 is made with the window bound rounded up to even, so that both sides fit)
};
constexpr int FD_TOK_OFFSET = 32 * 32 + 32 + 32;    // dots, |a|^2 partials, |b|^2 partials ...
constexpr int FD_TILE_FLOATS = FD_TOK_OFFSET + 64;  // ... then (slice 0 only) the tokens of the 32 rows and 32 columns
constexpr int FD_MAX_COLS = 2048;                   // |B| of the largest supported window

FdPlan make_fd_plan(int n_windows, int max_window_tokens, int d, int dtype_bytes);

// cu_target / win_remove / status / dir / counts_done (all optional): the per-window counts of a token budget
// (launch_window_counts, mode 2) in the same launch where the kernel allows it; *counts_done says whether it did.
hipError_t launch_build_windows(const int32_t *cu_vis, const int32_t *pos, const int32_t *new_index,
                                const int32_t *cu_out, int batch, int max_seq, int tiles,
                                int grid_h, int grid_w, int w, int32_t *win_offsets, int32_t *win_tokens,
                                const int32_t *cu_target, int32_t *win_remove, int32_t *status, int dir, bool *counts_done,
                                hipStream_t stream);

// windows + their counts from per-sequence target lengths, in one launch where possible (lk_api.hip); a lightkv_status
int build_windows_with_counts(int32_t batch, const int32_t *h_cu_vis, const int32_t *cu_vis, const int32_t *pos,
                              const int32_t *new_index, const int32_t *cu_vis_out, int32_t tiles, int32_t grid_h,
                              int32_t grid_w, int32_t w, int32_t *win_offsets, int32_t *win_tokens, int32_t n_windows,
                              int32_t direction, const int32_t *cu_target, int32_t *win_remove, int32_t *status,
                              void *stream);

// per-window counts from a ratio (mode 0: tokens, 1: edges) or from per-sequence target lengths (mode 2)
hipError_t launch_window_counts(int batch, int win_per_seq, const int32_t *win_offsets, int mode, int dir, double rho,
                                const int32_t *cu_vis, const int32_t *cu_target, int32_t *win_remove, int32_t *status,
                                hipStream_t stream);

hipError_t launch_fd(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                     const int32_t *win_offsets, const int32_t *win_tokens, float *partial, float *best_fd,
                     int32_t *best_dst, hipStream_t stream);

// Windows of at most 64 tokens: partial tiles, then epilogue + per-window selection in one kernel
// (n_tiles == 0: not applicable).
FdPlan make_fd_small_fused_plan(int n_windows, int max_window_tokens, int d, int dtype_bytes);
hipError_t launch_fd_select_small(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows,
                                  int sum_n, const int32_t *win_offsets, const int32_t *win_tokens,
                                  const int32_t *win_remove, float *partial, float *best_fd, int32_t *best_dst,
                                  int32_t *dst, int32_t *cnt, int32_t *src_rank, hipStream_t stream);

// Step 2 read literally (lk_select_edges.hip): the k lowest-FD edges of every window.  Windows of at most
// 2 * EDGE_MAX_SIDE tokens are ranked in LDS by one kernel; larger ones through a key matrix in `big_keys`.
// `edges` is scratch of 3 * sum_k ints (sum_k = the k of all windows, or a bound on it with device_counts, where a
// window's k is also bounded by its tokens).
constexpr int EDGE_MAX_SIDE = 128;
hipError_t launch_fd_partial(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                             const int32_t *win_offsets, const int32_t *win_tokens, float *partial, hipStream_t stream);
hipError_t launch_edge_select(const FdPlan &plan, int dtype, const void *X, int64_t ldx, int d, int n_windows,
                              int max_window, int sum_n, int sum_k, const int32_t *win_offsets,
                              const int32_t *win_tokens, const int32_t *win_remove, float *partial, float *best_fd,
                              int32_t *best_dst, int32_t *dst, int32_t *cnt, int32_t *src_rank, int32_t *edges,
                              bool device_counts, uint32_t *big_keys, hipStream_t stream);
// the FD keys of every pair of every window, for windows beyond the one-kernel path: 32-bit keys (0 if not needed)
size_t edge_big_key_count(int n_windows, int max_window);
hipError_t launch_edge_fill(int sum_k, int sum_n, const int32_t *edges, const int32_t *grp_offsets, int32_t *grp_src,
                            hipStream_t stream);

// Debug dump of the FD of every pair (lk_fd_dump.hip); at most 65535 windows.
hipError_t launch_fd_dump(int dtype, const void *X, int64_t ldx, int d, int n_windows, int max_window, int sum_n,
                          int metric, int dir, const int32_t *win_offsets, const int32_t *win_tokens, float *out,
                          long long capacity, hipStream_t stream);

// Large windows (compute bound): LDS-tiled MFMA GEMM with the row arg-min fused into its epilogue.
struct FdBigPlan {
  int wb;            // MFMA blocks (16 x 16) per edge of the workgroup tile
  int mt, nt;        // workgroup tiles per window along A and B
  int max_window;    // the caller's bound on the tokens of a window
  size_t norm_floats;   // |x|^2 per token (used when the caller does not hand them in)
  int nt_store;      // column tiles that keep keys of their own: nt, or 1 (all tiles of a window share one key per row)
  size_t key_bytes;  // [nt_store][sum_n] packed keys (FD bits << 32 | B token): per column tile, the best key of the A
                     // row at every position of the window lists; all-ones where nothing was offered
  int metric;        // as in FdPlan
  int dir;           // as in FdPlan
};
constexpr int FD_BIG_TILE = 96;            // rows and columns of a workgroup tile
constexpr int FD_BIG_KEYS_PER_TILE_MAX_NT = 4;   // up to this many column tiles per window, each keeps keys of its own
constexpr int FD_BIG_MIN_WINDOW = 128;   // windows bounded by fewer tokens use the small-tile path, and so do
constexpr int FD_BIG_MIN_TILES = 32;     // problems that make up fewer workgroup tiles than this
FdBigPlan make_fd_big_plan(int n_windows, int max_window_tokens, int sum_n);
hipError_t launch_fd_big(const FdBigPlan &plan, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                         const int32_t *win_offsets, const int32_t *win_tokens, const float *x_sqnorm, float *sq_ws,
                         unsigned long long *keys, float *best_fd, int32_t *best_dst, bool finalize,
                         hipStream_t stream);
// Full pairwise matching (every two tokens of a window): one packed key per list position in `keys`
// (FD bits << 32 | position of the nearest neighbour in the window list).  bf16, d a multiple of 64.
// best_fd / best_dst: written from the keys if not NULL (every token's nearest neighbour).
hipError_t launch_fd_pair(const void *X, int64_t ldx, int d, int n_windows, int max_window, int sum_n, int metric,
                          const int32_t *win_offsets, const int32_t *win_tokens, const float *x_sqnorm, float *sq_ws,
                          unsigned long long *keys, float *best_fd, int32_t *best_dst, hipStream_t stream);
// ... and the selection on those keys (lk_select_pair.hip): dst, source counts and ranks, best_fd / best_dst
hipError_t launch_pair_select(int n_windows, int max_window, int sum_n, const int32_t *win_offsets,
                              const int32_t *win_tokens, const int32_t *win_remove, const unsigned long long *keys,
                              float *best_fd, int32_t *best_dst, int32_t *dst, int32_t *cnt, int32_t *src_rank,
                              hipStream_t stream);

// ---- scores + selection in three launches on one stream (lk_fused.hip); windows of at most 64 tokens
struct XiArgs;
struct XiPlan;
hipError_t launch_score_select_fused(const XiPlan &xp, const FdPlan &fp, int dtype, int xi_mode, int batch, int heads,
                                     int head_dim, int d, int n_windows, int sum_n, int sum_t, const int32_t *cu_vis,
                                     const int32_t *cu_txt, const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                     const void *K, int64_t k_tok_stride, int64_t k_head_stride, const float *lse,
                                     float scale, float *stats, float *xi_part, float *xi, const void *X, int64_t ldx,
                                     const int32_t *win_offsets, const int32_t *win_tokens, const int32_t *win_remove,
                                     float *partial, float *best_fd, int32_t *best_dst, int32_t *dst, int32_t *cnt,
                                     int32_t *src_rank, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                                     int32_t *cu_vis_out, hipStream_t stream);
// index scan with the head sum of xi in the same launch (x: arguments of the xi passes)
hipError_t launch_select_scan_heads(int batch, int sum_n, const int32_t *cu_vis, const int32_t *dst, int32_t *new_index,
                                    int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out, const int32_t *cnt,
                                    const int32_t *src_rank, const XiArgs &x, hipStream_t stream);

// ---- prompt-guidance weight xi (Step 3) ----------------------------------------------------
struct XiPlan {
  int max_text_tiles;  // ceil(max T_b / 32)
  int max_vis_blocks;  // ceil(max N_b / 128): pass 1 leaves one (max, sum) pair per prompt row and block
  size_t stat_floats;  // pass-1 partial (max, sum) pairs: heads * sumT * max_vis_blocks * 2
  size_t part_floats;  // per-head partial xi: heads * sumN
};
XiPlan make_xi_plan(int batch, const int32_t *h_cu_vis, const int32_t *h_cu_txt, int heads, int xi_mode);

hipError_t launch_xi(const XiPlan &plan, int dtype, int xi_mode, int batch, int heads, int head_dim, int sum_n,
                     int sum_t, const int32_t *cu_vis, const int32_t *cu_txt, const void *Q, int64_t q_tok_stride,
                     int64_t q_head_stride, const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                     const float *lse, float scale, float *stats, float *xi_part, float *xi, hipStream_t stream);

// Batches: one workgroup per (sequence, head) pair, both softmax sweeps in one launch (lk_xi_seq.hip).  Applies to
// text-query mode without a given lse, prompts of at most 256 tokens and at least XI_SEQ_MIN_PAIRS pairs.
constexpr int XI_SEQ_MIN_PAIRS = 256;
bool xi_seq_applies(const XiPlan &plan, int xi_mode, const float *lse, int batch, int heads);
hipError_t launch_xi_seq(const XiArgs &g, int dtype, int head_dim, hipStream_t stream);

// ---- selection (Step 2) ----------------------------------------------------------------------
// keys == nullptr: best_fd / best_dst are the inputs.  Otherwise the packed keys of launch_fd_big(..., finalize = false)
// are (planned with key_mt row tiles and key_nt stored column tiles per window), and best_fd / best_dst are written from them on the way (one
// launch less than finalizing first).
hipError_t launch_select(int n_windows, int max_window_tokens, int batch, int sum_n, const int32_t *cu_vis,
                         const int32_t *win_offsets, const int32_t *win_tokens, const int32_t *win_remove,
                         const unsigned long long *keys, int key_mt, int key_nt, float *best_fd, int32_t *best_dst, int32_t *dst,
                         int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out, int32_t *cnt,
                         int32_t *src_rank, int dir, hipStream_t stream);

// the scan half of lightkv_select alone (dst, cnt, src_rank already written)
hipError_t launch_select_scan(int batch, int sum_n, const int32_t *cu_vis, const int32_t *dst, int32_t *new_index,
                              int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out, const int32_t *cnt,
                              const int32_t *src_rank, hipStream_t stream);

// ---- message passing + compaction (Steps 3-5) ---------------------------------------------------
struct RowTensors {
  const void *in[3];
  void *out[3];
  int64_t ld_in[3];
  int64_t ld_out[3];
};
// mode 0: aggregate in place (out == in, only rows with sources are written)
// mode 1: compact (copy staying rows to new_index)      mode 2: aggregate + compact
// x_sqnorm_out (optional, modes 1 and 2): |x|^2 of every output row of the first tensor, fp32
hipError_t launch_rows(int mode, int dtype, int d, int sum_n, const RowTensors &t, const int32_t *new_index,
                       const int32_t *grp_offsets, const int32_t *grp_src, const float *xi, const int32_t *pos,
                       int32_t *pos_out, float *x_sqnorm_out, int64_t out_rows, hipStream_t stream);

// rows behind the vision span (modes 1 and 2): input row sum_n + j -> output row cu_vis_out[batch] + j
hipError_t launch_tail_rows(int dtype, int d, int sum_n, int batch, const RowTensors &t, const int32_t *pos,
                            int32_t *pos_out, const int32_t *cu_vis_out, int64_t tail_rows, int64_t out_rows,
                            hipStream_t stream);

}  // namespace lk
