// C ABI of the LightKV compression step: argument validation, workspace layout, launches.
// Nothing here allocates, synchronises or reads device memory.
#include "../../include/lightkv.h"
#include "lk_launch.h"
#include "lk_helpers.h"

#include <math.h>
#include <mutex>

namespace {

using namespace lk;

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Checked {
  int sum_n = 0, sum_t = 0, max_seq = 0, max_window = 0, elem_bytes = 0;
  int64_t sum_remove = 0;   // sum of h_win_remove (when given); edge lists without host counts: the slots reserved
  bool edge_device_counts = false;   // LIGHTKV_MATCH_EDGE_TOPK without h_win_remove: the counts are on the device only
};

// The window bound the launch plans are made with.  In the reverse direction the receiving side of an odd window is
// the larger one; planning with the bound rounded up to even makes room for either side (the library's largest
// window, 4096 tokens, is even).
int plan_bound(const lightkv_problem *p, int max_window) {
  return p->direction == LIGHTKV_DIRECTION_B_TO_A ? ((max_window + 1) & ~1) : max_window;
}

lightkv_status check_problem(const lightkv_problem *p, bool need_windows, bool need_txt, Checked &c) {
  if (!p || !p->h_cu_vis || !p->cu_vis) return LIGHTKV_ERR_NULL;
  if (p->batch < 1 || p->d < 1 || p->heads < 1 || p->head_dim < 1 || p->n_windows < 0) return LIGHTKV_ERR_SHAPE;
  if (p->dtype != LIGHTKV_F32 && p->dtype != LIGHTKV_BF16) return LIGHTKV_ERR_UNSUPPORTED;
  if (p->metric < LIGHTKV_METRIC_COSINE || p->metric > LIGHTKV_METRIC_L2SQ) return LIGHTKV_ERR_UNSUPPORTED;
  if (p->match < LIGHTKV_MATCH_BEST_PER_A || p->match > LIGHTKV_MATCH_FULL_PAIRWISE) return LIGHTKV_ERR_UNSUPPORTED;
  if (p->direction != LIGHTKV_DIRECTION_A_TO_B && p->direction != LIGHTKV_DIRECTION_B_TO_A) return LIGHTKV_ERR_UNSUPPORTED;
  // the reverse direction is defined for the best edge of every proposing node; an edge list and the full pairwise
  // visit have no proposing side
  if (p->direction != LIGHTKV_DIRECTION_A_TO_B && p->match != LIGHTKV_MATCH_BEST_PER_A) return LIGHTKV_ERR_UNSUPPORTED;
  // full pairwise matching runs on the tiled matrix-core kernel only: bf16 rows of whole 64-element k-steps
  if (p->match == LIGHTKV_MATCH_FULL_PAIRWISE && (p->dtype != LIGHTKV_BF16 || p->d % 64 != 0))
    return LIGHTKV_ERR_UNSUPPORTED;
  c.elem_bytes = p->dtype == LIGHTKV_BF16 ? 2 : 4;
  if (p->d % (16 / c.elem_bytes) != 0) return LIGHTKV_ERR_UNSUPPORTED;
  if ((int64_t)p->heads * p->head_dim != p->d) return LIGHTKV_ERR_SHAPE;
  if (p->head_dim != 32 && p->head_dim != 64 && p->head_dim != 128) return LIGHTKV_ERR_UNSUPPORTED;
  if (p->h_cu_vis[0] != 0) return LIGHTKV_ERR_SHAPE;
  for (int b = 0; b < p->batch; ++b) {
    const int n = p->h_cu_vis[b + 1] - p->h_cu_vis[b];
    if (n < 0) return LIGHTKV_ERR_SHAPE;
    if (n > LIGHTKV_MAX_SEQ_TOKENS) return LIGHTKV_ERR_UNSUPPORTED;
    c.max_seq = n > c.max_seq ? n : c.max_seq;
  }
  c.sum_n = p->h_cu_vis[p->batch];
  if (need_txt) {
    if (!p->h_cu_txt || !p->cu_txt) return LIGHTKV_ERR_NULL;
    if (p->h_cu_txt[0] != 0) return LIGHTKV_ERR_SHAPE;
    for (int b = 0; b < p->batch; ++b) {
      const int t = p->h_cu_txt[b + 1] - p->h_cu_txt[b];
      if (t < 0) return LIGHTKV_ERR_SHAPE;
      if (t > LIGHTKV_MAX_TEXT_TOKENS) return LIGHTKV_ERR_UNSUPPORTED;
    }
    c.sum_t = p->h_cu_txt[p->batch];
  }
  if (need_windows) {
    if (!p->win_offsets || !p->win_tokens) return LIGHTKV_ERR_NULL;
    int maxw = 0;
    if (p->h_win_offsets) {
      if (p->n_windows > 0 && p->h_win_offsets[0] != 0) return LIGHTKV_ERR_WINDOWS;
      for (int w = 0; w < p->n_windows; ++w) {
        const int v = p->h_win_offsets[w + 1] - p->h_win_offsets[w];
        if (v < 0) return LIGHTKV_ERR_WINDOWS;
        maxw = v > maxw ? v : maxw;
      }
      if (p->n_windows > 0 && p->h_win_offsets[p->n_windows] != c.sum_n) return LIGHTKV_ERR_WINDOWS;
      if (p->n_windows == 0 && c.sum_n != 0) return LIGHTKV_ERR_WINDOWS;
      if (p->max_window_tokens > 0 && p->max_window_tokens < maxw) return LIGHTKV_ERR_WINDOWS;
      if (p->h_win_remove) {
        for (int w = 0; w < p->n_windows; ++w) {
          const int v = p->h_win_offsets[w + 1] - p->h_win_offsets[w];
          const int r = p->h_win_remove[w];
          // tokens of A at most; with the k lowest edges, pairs of the window at most
          const int cap = (v < 2) ? 0 : (p->match == LIGHTKV_MATCH_EDGE_TOPK ? ((v + 1) / 2) * (v / 2) : side_a(v, p->direction));
          if (r < 0 || r > cap) return LIGHTKV_ERR_REMOVE_COUNT;
          c.sum_remove += r;
        }
      }
      c.max_window = p->max_window_tokens > 0 ? p->max_window_tokens : maxw;
    } else {
      if (p->max_window_tokens <= 0) return LIGHTKV_ERR_NULL;
      c.max_window = p->max_window_tokens;
    }
    if (c.max_window > LIGHTKV_MAX_WINDOW_TOKENS) return LIGHTKV_ERR_UNSUPPORTED;
    c.max_window = plan_bound(p, c.max_window);
    if (p->match == LIGHTKV_MATCH_EDGE_TOPK) {
      // the edge list is sized from the host's counts (validated against the host's window sizes) or, without them,
      // for one slot per token: a window's k is then bounded by its tokens as well as by its pairs
      if (p->h_win_remove && !p->h_win_offsets) return LIGHTKV_ERR_NULL;
      if (!p->h_win_remove) { c.sum_remove = c.sum_n; c.edge_device_counts = true; }
      if (c.max_window > LIGHTKV_EDGE_MAX_WINDOW_TOKENS || c.sum_remove >= (1ll << 28)) return LIGHTKV_ERR_UNSUPPORTED;
      // windows beyond the one-kernel path keep the keys of all their pairs in the workspace
      if (edge_big_key_count(p->n_windows, c.max_window) >= (1ull << 31)) return LIGHTKV_ERR_UNSUPPORTED;
    }
  }
  return LIGHTKV_OK;
}

// The two halves of lightkv_score (xi from Q/K, FD from X) share no data, so they are enqueued as a fork/join:
// xi on a helper stream, FD on the caller's stream, joined by events before the call returns.  Under stream capture
// the fork/join becomes two parallel branches of the graph.  Helper sets come from a per-device pool (lk_helpers.h);
// without one the work runs serially on the caller's stream.
using Fork = HelperSet<1, 2>;   // stream[0]: xi; event[0]: fork, event[1]: join

struct WsLayout {
  size_t fd_partial = 0, fd_norm = 0, fd_keys = 0, xi_stats = 0, xi_part = 0, sel_cnt = 0,
         sel_rank = 0, edges = 0, total = 0;
};

bool edge_topk(const lightkv_problem *p) { return p->match == LIGHTKV_MATCH_EDGE_TOPK; }
bool full_pairwise(const lightkv_problem *p) { return p->match == LIGHTKV_MATCH_FULL_PAIRWISE; }
// ints of scratch for the edge list (A token, B token, position among the B token's sources)
// ... followed by the key matrices of windows beyond the one-kernel path
size_t edge_ints(const lightkv_problem *p, const Checked &c) {
  return edge_topk(p) ? (size_t)3 * (size_t)c.sum_remove + edge_big_key_count(p->n_windows, c.max_window) : 0;
}

bool use_big_fd(const lightkv_problem *p, const Checked &c) {
  if (full_pairwise(p)) return true;   // squared norms and one packed key per position, as on the tiled bipartite path
  if (edge_topk(p)) return false;   // every pair's FD is ranked: the small tiles keep them all, the tiled kernel only row minima
  // the large-window kernel wants whole pairs of 128-element k-steps; other shapes take the small-tile path
  if (p->dtype != LIGHTKV_BF16 || p->d % 256 != 0 || c.max_window < FD_BIG_MIN_WINDOW) return false;
  // ... and enough 96 x 96 tiles to give the chip work: with few, its long k loop per tile is all latency.  Measured per
  // step: one window of 387 tokens (9 tiles) 169 us tiled against 165 us on the small-tile path; 64 windows of 144
  // tokens (64 tiles) 109 against 123 us per score call; one window of 2880 tokens is 225 tiles.
  const FdBigPlan big = make_fd_big_plan(p->n_windows, c.max_window, c.sum_n);
  return (int64_t)p->n_windows * big.mt * big.nt >= FD_BIG_MIN_TILES;
}

WsLayout ws_layout(const FdPlan &fd, const FdBigPlan &big, bool use_big, const XiPlan &xi, int sum_n, size_t n_edge_ints) {
  // (full pairwise matching needs at most what the tiled bipartite path lays out: norms and one key plane or more)
  WsLayout l;
  size_t off = 0;
  l.fd_partial = off; off = align_up(off + (use_big ? 0 : fd.partial_floats * sizeof(float)));
  l.fd_norm = off;    off = align_up(off + (use_big ? big.norm_floats * sizeof(float) : 0));
  l.fd_keys = off;    off = align_up(off + (use_big ? big.key_bytes : 0));
  l.xi_stats = off;   off = align_up(off + xi.stat_floats * sizeof(float));
  l.xi_part = off;    off = align_up(off + xi.part_floats * sizeof(float));
  l.sel_cnt = off;    off = align_up(off + (size_t)sum_n * sizeof(int32_t));
  l.sel_rank = off;   off = align_up(off + (size_t)sum_n * sizeof(int32_t));
  l.edges = off;      off = align_up(off + n_edge_ints * sizeof(int32_t));
  l.total = off + ALIGN;
  return l;
}

bool row_tensor_ok(const void *p, int64_t ld, int d, int elem_bytes, lightkv_status &st) {
  if (!p) return true;
  if (!aligned16(p) || ld % (16 / elem_bytes) != 0) { st = LIGHTKV_ERR_UNSUPPORTED; return false; }
  if (ld < d) { st = LIGHTKV_ERR_SHAPE; return false; }
  return true;
}

// from_keys: the scores are the packed keys the tiled FD kernel left in the workspace (best_fd / best_dst are then
// outputs, written by the selection kernels); otherwise best_fd / best_dst are the inputs.
lightkv_status select_impl(const lightkv_problem *p, bool from_keys, float *best_fd, int32_t *best_dst,
                           int32_t *dst, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                           int32_t *cu_vis_out, void *ws, size_t ws_bytes, void *stream) {
  Checked c;
  lightkv_status st = check_problem(p, true, false, c);
  if (st != LIGHTKV_OK) return st;
  if (!p->win_remove || !best_fd || !best_dst || !dst || !new_index || !grp_offsets || !grp_src || !cu_vis_out)
    return LIGHTKV_ERR_NULL;
  const FdPlan fd = make_fd_plan(p->n_windows, c.max_window, p->d, c.elem_bytes);
  const bool have_txt = p->h_cu_txt && p->cu_txt;
  const XiPlan xp = make_xi_plan(p->batch, p->h_cu_vis, have_txt ? p->h_cu_txt : nullptr, p->heads, 0);
  const FdBigPlan big = make_fd_big_plan(p->n_windows, c.max_window, c.sum_n);
  if (edge_topk(p) || full_pairwise(p)) return LIGHTKV_ERR_UNSUPPORTED;   // scores of another kind: lightkv_score_select only
  const WsLayout l = ws_layout(fd, big, use_big_fd(p, c), xp, c.sum_n, 0);
  // only the selection scratch (and the keys) are used here; accept a workspace that covers the layout
  if (!ws || (reinterpret_cast<uintptr_t>(ws) % ALIGN) != 0 || ws_bytes < l.total) return LIGHTKV_ERR_WORKSPACE;
  char *wsb = static_cast<char *>(ws);
  const unsigned long long *keys = from_keys ? reinterpret_cast<const unsigned long long *>(wsb + l.fd_keys) : nullptr;
  if (launch_select(p->n_windows, c.max_window, p->batch, c.sum_n, p->cu_vis, p->win_offsets, p->win_tokens,
                    p->win_remove, keys, big.mt, big.nt_store, best_fd, best_dst, dst, new_index, grp_offsets, grp_src, cu_vis_out,
                    reinterpret_cast<int32_t *>(wsb + l.sel_cnt), reinterpret_cast<int32_t *>(wsb + l.sel_rank),
                    p->direction, static_cast<hipStream_t>(stream)) != hipSuccess)
    return LIGHTKV_ERR_LAUNCH;
  return LIGHTKV_OK;
}
}  // namespace

extern "C" {

const char *lightkv_status_string(int status) {
  switch (status) {
    case LIGHTKV_OK: return "ok";
    case LIGHTKV_ERR_NULL: return "a required pointer is NULL";
    case LIGHTKV_ERR_SHAPE: return "inconsistent sizes, strides or offsets";
    case LIGHTKV_ERR_WINDOWS: return "window lists are not a partition of the tokens";
    case LIGHTKV_ERR_REMOVE_COUNT: return "a window is asked to remove more tokens than its set A holds";
    case LIGHTKV_ERR_UNSUPPORTED: return "unsupported dtype, head size, alignment or size limit";
    case LIGHTKV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LIGHTKV_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

int lightkv_version(void) { return 320; }   // 0.3.2: lightkv_compress_schedule_ratio (0.3.1: lightkv_problem.direction,
                                            // direction argument of lightkv_window_counts, edge lists for windows of
                                            // up to 4096 tokens)

lightkv_status lightkv_workspace_size(const lightkv_problem *p, size_t *bytes) {
  if (!bytes) return LIGHTKV_ERR_NULL;
  Checked c;
  // prompt offsets are optional here: without them the xi scratch is not counted (XI_GIVEN callers)
  const bool have_txt = p && p->h_cu_txt && p->cu_txt;
  lightkv_status st = check_problem(p, true, have_txt, c);
  if (st != LIGHTKV_OK) return st;
  const FdPlan fd = make_fd_plan(p->n_windows, c.max_window, p->d, c.elem_bytes);
  const XiPlan xi = make_xi_plan(p->batch, p->h_cu_vis, have_txt ? p->h_cu_txt : nullptr, p->heads, 0);
  const FdBigPlan big = make_fd_big_plan(p->n_windows, c.max_window, c.sum_n);
  *bytes = ws_layout(fd, big, use_big_fd(p, c), xi, c.sum_n, edge_ints(p, c)).total;
  return LIGHTKV_OK;
}

static lightkv_status build_windows_impl(int32_t batch, const int32_t *h_cu_vis, const int32_t *cu_vis,
                                         const int32_t *pos, const int32_t *new_index, const int32_t *cu_vis_out,
                                         int32_t tiles, int32_t grid_h, int32_t grid_w, int32_t w,
                                         int32_t *win_offsets, int32_t *win_tokens, void *stream,
                                         const int32_t *cu_target = nullptr, int32_t *win_remove = nullptr,
                                         int32_t *status = nullptr, int dir = 0, bool *counts_done = nullptr) {
  if (!h_cu_vis || !cu_vis || !pos || !win_offsets || !win_tokens) return LIGHTKV_ERR_NULL;
  if (batch < 1 || tiles < 1 || grid_h < 1 || grid_w < 1 || w < 0 || h_cu_vis[0] != 0) return LIGHTKV_ERR_SHAPE;
  int max_seq = 0;
  for (int b = 0; b < batch; ++b) {
    const int n = h_cu_vis[b + 1] - h_cu_vis[b];
    if (n < 0) return LIGHTKV_ERR_SHAPE;
    max_seq = n > max_seq ? n : max_seq;
  }
  if (max_seq > LIGHTKV_MAX_SEQ_TOKENS) return LIGHTKV_ERR_UNSUPPORTED;
  if ((int64_t)tiles * w * w > (1 << 17) || (int64_t)tiles * grid_h * grid_w > (1ll << 30)) return LIGHTKV_ERR_UNSUPPORTED;
  if (launch_build_windows(cu_vis, pos, new_index, cu_vis_out, batch, max_seq, tiles, grid_h, grid_w, w, win_offsets,
                           win_tokens, cu_target, win_remove, status, dir, counts_done,
                           static_cast<hipStream_t>(stream)) != hipSuccess)
    return LIGHTKV_ERR_LAUNCH;
  return LIGHTKV_OK;
}

lightkv_status lightkv_build_windows(int32_t batch, const int32_t *h_cu_vis, const int32_t *cu_vis,
                                     const int32_t *pos, int32_t tiles, int32_t grid_h, int32_t grid_w,
                                     int32_t w, int32_t *win_offsets, int32_t *win_tokens, void *stream) {
  return build_windows_impl(batch, h_cu_vis, cu_vis, pos, nullptr, nullptr, tiles, grid_h, grid_w, w, win_offsets,
                            win_tokens, stream);
}

lightkv_status lightkv_build_windows_next(int32_t batch, const int32_t *h_cu_vis, const int32_t *cu_vis,
                                          const int32_t *pos, const int32_t *new_index, const int32_t *cu_vis_out,
                                          int32_t tiles, int32_t grid_h, int32_t grid_w, int32_t w,
                                          int32_t *win_offsets, int32_t *win_tokens, void *stream) {
  if (!new_index || !cu_vis_out) return LIGHTKV_ERR_NULL;
  return build_windows_impl(batch, h_cu_vis, cu_vis, pos, new_index, cu_vis_out, tiles, grid_h, grid_w, w, win_offsets,
                            win_tokens, stream);
}

int32_t lightkv_windows_per_sequence(int32_t tiles, int32_t w) {
  if (tiles < 1 || w < 0 || (int64_t)tiles * w * w > (1 << 17)) return -1;
  return w == 0 ? 1 : tiles * w * w;
}

int32_t lightkv_max_window_cells(int32_t tiles, int32_t grid_h, int32_t grid_w, int32_t w) {
  if (tiles < 1 || grid_h < 1 || grid_w < 1 || w < 0 || (int64_t)tiles * grid_h * grid_w > (1ll << 30)) return -1;
  if (w == 0) return tiles * grid_h * grid_w;
  // window k of an axis of g cells holds the cells c with floor(c * w / g) == k
  auto widest = [](int g, int w_) {
    int best = 0, run = 0, prev = -1;
    for (int c = 0; c < g; ++c) {
      const int k = (int)((int64_t)c * w_ / g);
      run = k == prev ? run + 1 : 1;
      prev = k;
      best = run > best ? run : best;
    }
    return best;
  };
  return widest(grid_h, w) * widest(grid_w, w);
}

lightkv_status lightkv_window_counts(int32_t batch, int32_t n_windows, const int32_t *win_offsets, int32_t mode,
                                     int32_t direction, double rho, const int32_t *cu_vis, const int32_t *cu_vis_target,
                                     int32_t *win_remove, int32_t *status, void *stream) {
  if (direction != LIGHTKV_DIRECTION_A_TO_B && direction != LIGHTKV_DIRECTION_B_TO_A) return LIGHTKV_ERR_UNSUPPORTED;
  if (direction != LIGHTKV_DIRECTION_A_TO_B && mode == LIGHTKV_COUNT_EDGES) return LIGHTKV_ERR_UNSUPPORTED;
  if (!win_offsets || !win_remove) return LIGHTKV_ERR_NULL;
  if (batch < 1 || n_windows < 0 || n_windows % batch != 0) return LIGHTKV_ERR_SHAPE;
  if (mode < LIGHTKV_COUNT_RATIO || mode > LIGHTKV_COUNT_TARGET) return LIGHTKV_ERR_UNSUPPORTED;
  if (mode == LIGHTKV_COUNT_TARGET && (!cu_vis || !cu_vis_target)) return LIGHTKV_ERR_NULL;
  if (mode != LIGHTKV_COUNT_TARGET && !(rho >= 0.0 && rho <= 1e6)) return LIGHTKV_ERR_SHAPE;   // also refuses NaN
  if (n_windows == 0) return LIGHTKV_OK;
  if (launch_window_counts(batch, n_windows / batch, win_offsets, mode, direction, rho, cu_vis, cu_vis_target, win_remove,
                           status, static_cast<hipStream_t>(stream)) != hipSuccess)
    return LIGHTKV_ERR_LAUNCH;
  return LIGHTKV_OK;
}

}  // extern "C"

// Windows and their counts for lightkv_compress_schedule: lightkv_build_windows (or _next) followed by
// lightkv_window_counts(LIGHTKV_COUNT_TARGET) on the windows just built -- in ONE launch where the partition kernel
// allows it (the window sizes are in its LDS at the end), in two otherwise.  Same validation, same results.
int lk::build_windows_with_counts(int32_t batch, const int32_t *h_cu_vis, const int32_t *cu_vis, const int32_t *pos,
                                  const int32_t *new_index, const int32_t *cu_vis_out, int32_t tiles, int32_t grid_h,
                                  int32_t grid_w, int32_t w, int32_t *win_offsets, int32_t *win_tokens, int32_t n_windows,
                                  int32_t direction, const int32_t *cu_target, int32_t *win_remove, int32_t *status,
                                  void *stream) {
  if ((new_index == nullptr) != (cu_vis_out == nullptr)) return LIGHTKV_ERR_NULL;
  if (!cu_target || !win_remove) return LIGHTKV_ERR_NULL;
  if (direction != LIGHTKV_DIRECTION_A_TO_B && direction != LIGHTKV_DIRECTION_B_TO_A) return LIGHTKV_ERR_UNSUPPORTED;
  const int32_t wps = lightkv_windows_per_sequence(tiles, w);
  if (batch < 1 || wps < 0 || (int64_t)wps * batch != n_windows) return LIGHTKV_ERR_SHAPE;
  bool done = false;
  const lightkv_status st = build_windows_impl(batch, h_cu_vis, cu_vis, pos, new_index, cu_vis_out, tiles, grid_h, grid_w, w,
                                               win_offsets, win_tokens, stream, cu_target, win_remove, status, direction, &done);
  if (st != LIGHTKV_OK || done) return st;
  // the current lengths of the sequences: after the previous stage's compaction in the "next" form
  return lightkv_window_counts(batch, n_windows, win_offsets, LIGHTKV_COUNT_TARGET, direction, 0.0,
                               cu_vis_out ? cu_vis_out : cu_vis, cu_target, win_remove, status, stream);
}

namespace {
struct SelectOut {   // outputs of lightkv_select, present when selection is to be fused behind the scores
  int32_t *dst, *new_index, *grp_offsets, *grp_src, *cu_vis_out;
};

// sel == nullptr: plain lightkv_score.  Otherwise the caller guarantees that make_fd_small_fused_plan applies.
// keys_only: on the tiled MFMA path, leave the packed keys in the workspace and do not write best_fd / best_dst
// (the caller's selection reads the keys and writes them).
lightkv_status score_impl(const lightkv_problem *p, const void *X, int64_t ldx, const float *x_sqnorm,
                          const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                          const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                          int32_t xi_mode, const float *lse, float softmax_scale,
                          float *xi, float *best_fd, int32_t *best_dst, const SelectOut *sel, bool keys_only,
                          float *fd_dump, int64_t fd_dump_floats, void *ws, size_t ws_bytes, void *stream) {
  if (xi_mode < LIGHTKV_XI_TEXT_QUERY || xi_mode > LIGHTKV_XI_GIVEN) return LIGHTKV_ERR_UNSUPPORTED;
  const bool need_xi = xi_mode != LIGHTKV_XI_GIVEN;
  const bool need_fd = X != nullptr;   // X == NULL: only xi is wanted (the two halves may be enqueued separately)
  if (!need_fd && !need_xi) return LIGHTKV_ERR_NULL;
  Checked c;
  lightkv_status st = check_problem(p, need_fd, need_xi, c);
  if (st != LIGHTKV_OK) return st;
  if (!xi || (need_fd && (!best_fd || !best_dst))) return LIGHTKV_ERR_NULL;
  if (need_fd && !row_tensor_ok(X, ldx, p->d, c.elem_bytes, st)) return st;
  if (x_sqnorm && (reinterpret_cast<uintptr_t>(x_sqnorm) & 3)) return LIGHTKV_ERR_UNSUPPORTED;
  if (fd_dump) {
    if (!need_fd) return LIGHTKV_ERR_NULL;
    if (fd_dump_floats < 0) return LIGHTKV_ERR_SHAPE;
    // (the dump holds the bipartite |A| x |B| blocks: not defined for full pairwise matching)
    if ((reinterpret_cast<uintptr_t>(fd_dump) & 3) || p->n_windows > 65535 || p->match == LIGHTKV_MATCH_FULL_PAIRWISE)
      return LIGHTKV_ERR_UNSUPPORTED;
  }
  if (need_xi) {
    if (!Q || !K) return LIGHTKV_ERR_NULL;
    if (xi_mode == LIGHTKV_XI_VISION_QUERY && !lse) return LIGHTKV_ERR_NULL;
    const int64_t m = 16 / c.elem_bytes;
    if (!aligned16(Q) || !aligned16(K) || q_tok_stride % m || q_head_stride % m || k_tok_stride % m || k_head_stride % m)
      return LIGHTKV_ERR_UNSUPPORTED;
    if (q_tok_stride < 0 || q_head_stride < 0 || k_tok_stride < 0 || k_head_stride < 0) return LIGHTKV_ERR_SHAPE;
  }
  // the workspace layout is the same whichever halves are requested, so that an xi-only call and an FD-only call
  // on two streams can share one workspace (their regions are disjoint)
  int max_window = c.max_window;
  if (!need_fd) {   // windows were not validated: take the bound as given, clamped, just to lay the workspace out
    max_window = p->max_window_tokens > 0 ? p->max_window_tokens : 0;
    if (max_window > LIGHTKV_MAX_WINDOW_TOKENS) max_window = LIGHTKV_MAX_WINDOW_TOKENS;
    if (max_window == 0 && p->h_win_offsets)
      for (int w = 0; w < p->n_windows; ++w) {
        const int v = p->h_win_offsets[w + 1] - p->h_win_offsets[w];
        max_window = v > max_window ? v : max_window;
      }
    c.max_window = plan_bound(p, max_window);
  }
  FdPlan fd = make_fd_plan(p->n_windows, c.max_window, p->d, c.elem_bytes);
  const XiPlan xp = make_xi_plan(p->batch, p->h_cu_vis, p->h_cu_txt && p->cu_txt ? p->h_cu_txt : nullptr, p->heads, 0);
  FdBigPlan big = make_fd_big_plan(p->n_windows, c.max_window, c.sum_n);
  fd.metric = big.metric = p->metric;
  fd.dir = big.dir = p->direction;
  const bool use_big = use_big_fd(p, c);
  const bool edge = sel && need_fd && edge_topk(p);
  const bool pairwise = need_fd && full_pairwise(p);
  if (pairwise && (uint64_t)c.sum_n * (uint64_t)ldx * 2u >= (1ull << 32)) return LIGHTKV_ERR_UNSUPPORTED;   // 32-bit row offsets
  const WsLayout l = ws_layout(fd, big, use_big, xp, c.sum_n, need_fd ? edge_ints(p, c) : 0);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) % ALIGN) != 0 || ws_bytes < l.total) return LIGHTKV_ERR_WORKSPACE;
  char *wsb = static_cast<char *>(ws);
  hipStream_t s = static_cast<hipStream_t>(stream);

  if (use_big && (uint64_t)c.sum_n * (uint64_t)ldx * 2u >= (1ull << 32)) return LIGHTKV_ERR_UNSUPPORTED;   // 32-bit row offsets
  // Both halves and the selection, single-tile windows, a small step: three launches on the caller's stream, each
  // running a step of the xi chain next to a step of the FD chain (no helper stream, no fork/join).  Larger steps fill
  // the chip with either chain alone; there the shared launches take as long as the two in a row and the helper
  // stream is the better arrangement (measured: 2880 tokens 248 vs 237 us per three stages, 576 tokens 190 vs 199).
  // (only layouts of the small-tile path hold the partial tiles these launches write: never with use_big)
  if (need_xi && need_fd && sel && !edge && !pairwise && !use_big && fd.n_tiles > 0 && c.sum_n > 0 &&
      c.sum_n <= LIGHTKV_ONE_STREAM_MAX_TOKENS && p->n_windows > 0) {
    const float scale = softmax_scale != 0.f ? softmax_scale : 1.0f / sqrtf((float)p->head_dim);
    int32_t *cnt = reinterpret_cast<int32_t *>(wsb + l.sel_cnt), *rank = reinterpret_cast<int32_t *>(wsb + l.sel_rank);
    const hipError_t e = launch_score_select_fused(
        xp, fd, p->dtype, xi_mode, p->batch, p->heads, p->head_dim, p->d, p->n_windows, c.sum_n, c.sum_t, p->cu_vis,
        p->cu_txt, Q, q_tok_stride, q_head_stride, K, k_tok_stride, k_head_stride, lse, scale,
        reinterpret_cast<float *>(wsb + l.xi_stats), reinterpret_cast<float *>(wsb + l.xi_part), xi, X, ldx,
        p->win_offsets, p->win_tokens, p->win_remove, reinterpret_cast<float *>(wsb + l.fd_partial), best_fd, best_dst,
        sel->dst, cnt, rank, sel->new_index, sel->grp_offsets, sel->grp_src, sel->cu_vis_out, s);
    return e == hipSuccess ? LIGHTKV_OK : LIGHTKV_ERR_LAUNCH;
  }
  Fork *fk = nullptr;
  std::unique_lock<std::mutex> fork_guard;   // released when this call returns, i.e. after the join has been enqueued
  if (need_xi) {
    if (need_fd) fk = acquire_helpers<1, 2>(s, fork_guard);
    hipStream_t xs = s;
    if (fk) {
      if (hipEventRecord(fk->event[0], s) == hipSuccess && hipStreamWaitEvent(fk->stream[0], fk->event[0], 0) == hipSuccess) xs = fk->stream[0];
      else { (void)hipGetLastError(); fk = nullptr; }
    }
    const float scale = softmax_scale != 0.f ? softmax_scale : 1.0f / sqrtf((float)p->head_dim);
    const hipError_t e = launch_xi(xp, p->dtype, xi_mode, p->batch, p->heads, p->head_dim, c.sum_n, c.sum_t, p->cu_vis,
                                   p->cu_txt, Q, q_tok_stride, q_head_stride, K, k_tok_stride, k_head_stride, lse, scale,
                                   reinterpret_cast<float *>(wsb + l.xi_stats),
                                   reinterpret_cast<float *>(wsb + l.xi_part), xi, xs);
    if (fk && hipEventRecord(fk->event[1], fk->stream[0]) != hipSuccess) return LIGHTKV_ERR_LAUNCH;
    if (e != hipSuccess) {   // the helper stream must rejoin the caller's stream whatever happened on it
      if (fk) (void)hipStreamWaitEvent(s, fk->event[1], 0);
      return LIGHTKV_ERR_LAUNCH;
    }
  }
  lightkv_status fd_status = LIGHTKV_OK;
  if (!need_fd) {
    // xi only
  } else if (pairwise) {
    // every two tokens of a window: nearest neighbour per token on the matrix cores, the visit in rank order, index scan
    int32_t *cnt = reinterpret_cast<int32_t *>(wsb + l.sel_cnt), *rank = reinterpret_cast<int32_t *>(wsb + l.sel_rank);
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(wsb + l.fd_keys);
    if (!sel) {   // scores only: every token's nearest neighbour
      if (launch_fd_pair(X, ldx, p->d, p->n_windows, c.max_window, c.sum_n, p->metric, p->win_offsets, p->win_tokens,
                         x_sqnorm, reinterpret_cast<float *>(wsb + l.fd_norm), keys, best_fd, best_dst, s) != hipSuccess)
        fd_status = LIGHTKV_ERR_LAUNCH;
    } else if (launch_fd_pair(X, ldx, p->d, p->n_windows, c.max_window, c.sum_n, p->metric, p->win_offsets, p->win_tokens,
                       x_sqnorm, reinterpret_cast<float *>(wsb + l.fd_norm), keys, nullptr, nullptr, s) != hipSuccess ||
        launch_pair_select(p->n_windows, c.max_window, c.sum_n, p->win_offsets, p->win_tokens, p->win_remove, keys,
                           best_fd, best_dst, sel->dst, cnt, rank, s) != hipSuccess ||
        launch_select_scan(p->batch, c.sum_n, p->cu_vis, sel->dst, sel->new_index, sel->grp_offsets, sel->grp_src,
                           sel->cu_vis_out, cnt, rank, s) != hipSuccess)
      fd_status = LIGHTKV_ERR_LAUNCH;
  } else if (edge) {
    // the k lowest edges of every window: partial tiles, ranking per window, index scan, group lists from the edge list
    int32_t *cnt = reinterpret_cast<int32_t *>(wsb + l.sel_cnt), *rank = reinterpret_cast<int32_t *>(wsb + l.sel_rank);
    int32_t *edges = reinterpret_cast<int32_t *>(wsb + l.edges);
    const int sum_k = (int)c.sum_remove;
    if (launch_edge_select(fd, p->dtype, X, ldx, p->d, p->n_windows, c.max_window, c.sum_n, sum_k, p->win_offsets,
                           p->win_tokens, p->win_remove, reinterpret_cast<float *>(wsb + l.fd_partial), best_fd,
                           best_dst, sel->dst, cnt, rank, edges, c.edge_device_counts,
                           reinterpret_cast<uint32_t *>(edges + (size_t)3 * (size_t)sum_k), s) != hipSuccess ||
        launch_select_scan(p->batch, c.sum_n, p->cu_vis, sel->dst, sel->new_index, sel->grp_offsets, sel->grp_src,
                           sel->cu_vis_out, cnt, rank, s) != hipSuccess ||
        launch_edge_fill(sum_k, c.sum_n, edges, sel->grp_offsets, sel->grp_src, s) != hipSuccess)
      fd_status = LIGHTKV_ERR_LAUNCH;
  } else if (sel) {
    int32_t *cnt = reinterpret_cast<int32_t *>(wsb + l.sel_cnt), *rank = reinterpret_cast<int32_t *>(wsb + l.sel_rank);
    if (launch_fd_select_small(fd, p->dtype, X, ldx, p->d, p->n_windows, c.sum_n, p->win_offsets, p->win_tokens,
                               p->win_remove, reinterpret_cast<float *>(wsb + l.fd_partial), best_fd, best_dst,
                               sel->dst, cnt, rank, s) != hipSuccess ||
        launch_select_scan(p->batch, c.sum_n, p->cu_vis, sel->dst, sel->new_index, sel->grp_offsets, sel->grp_src,
                           sel->cu_vis_out, cnt, rank, s) != hipSuccess)
      fd_status = LIGHTKV_ERR_LAUNCH;
  } else if (use_big) {
    if (launch_fd_big(big, X, ldx, p->d, p->n_windows, c.sum_n, p->win_offsets, p->win_tokens,
                      x_sqnorm, reinterpret_cast<float *>(wsb + l.fd_norm),
                      reinterpret_cast<unsigned long long *>(wsb + l.fd_keys), best_fd, best_dst, !keys_only,
                      s) != hipSuccess)
      fd_status = LIGHTKV_ERR_LAUNCH;
  } else if (launch_fd(fd, p->dtype, X, ldx, p->d, p->n_windows, c.sum_n, p->win_offsets, p->win_tokens,
                       reinterpret_cast<float *>(wsb + l.fd_partial), best_fd, best_dst, s) != hipSuccess) {
    fd_status = LIGHTKV_ERR_LAUNCH;
  }
  if (fd_dump && fd_status == LIGHTKV_OK &&
      launch_fd_dump(p->dtype, X, ldx, p->d, p->n_windows, c.max_window, c.sum_n, p->metric, p->direction, p->win_offsets,
                     p->win_tokens, fd_dump, (long long)fd_dump_floats, s) != hipSuccess)
    fd_status = LIGHTKV_ERR_LAUNCH;
  if (fk && hipStreamWaitEvent(s, fk->event[1], 0) != hipSuccess) return LIGHTKV_ERR_LAUNCH;   // join
  return fd_status;
}
}  // namespace

extern "C" {

lightkv_status lightkv_score(const lightkv_problem *p, const void *X, int64_t ldx, const float *x_sqnorm,
                             const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                             const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                             int32_t xi_mode, const float *lse, float softmax_scale,
                             float *xi, float *best_fd, int32_t *best_dst, float *fd_dump, int64_t fd_dump_floats,
                             void *ws, size_t ws_bytes, void *stream) {
  return score_impl(p, X, ldx, x_sqnorm, Q, q_tok_stride, q_head_stride, K, k_tok_stride, k_head_stride, xi_mode, lse,
                    softmax_scale, xi, best_fd, best_dst, nullptr, false, fd_dump, fd_dump_floats, ws, ws_bytes, stream);
}

lightkv_status lightkv_score_select(const lightkv_problem *p, const void *X, int64_t ldx, const float *x_sqnorm,
                                    const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                    const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                                    int32_t xi_mode, const float *lse, float softmax_scale,
                                    float *xi, float *best_fd, int32_t *best_dst,
                                    int32_t *dst, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                                    int32_t *cu_vis_out, void *ws, size_t ws_bytes, void *stream) {
  if (!X || !dst || !new_index || !grp_offsets || !grp_src || !cu_vis_out) return LIGHTKV_ERR_NULL;
  Checked c;
  lightkv_status st = check_problem(p, true, false, c);
  if (st != LIGHTKV_OK) return st;
  if (!p->win_remove) return LIGHTKV_ERR_NULL;
  const FdPlan small = make_fd_small_fused_plan(p->n_windows, c.max_window, p->d, c.elem_bytes);
  if ((small.n_tiles > 0 && !use_big_fd(p, c)) || p->n_windows == 0 || edge_topk(p) || full_pairwise(p)) {
    const SelectOut sel{dst, new_index, grp_offsets, grp_src, cu_vis_out};
    return score_impl(p, X, ldx, x_sqnorm, Q, q_tok_stride, q_head_stride, K, k_tok_stride, k_head_stride, xi_mode, lse,
                      softmax_scale, xi, best_fd, best_dst, &sel, false, nullptr, 0, ws, ws_bytes, stream);
  }
  // the tiled MFMA path leaves packed keys: the selection reads them directly and writes best_fd / best_dst itself
  const bool from_keys = use_big_fd(p, c);
  st = score_impl(p, X, ldx, x_sqnorm, Q, q_tok_stride, q_head_stride, K, k_tok_stride, k_head_stride, xi_mode, lse,
                  softmax_scale, xi, best_fd, best_dst, nullptr, from_keys, nullptr, 0, ws, ws_bytes, stream);
  if (st != LIGHTKV_OK) return st;
  return select_impl(p, from_keys, best_fd, best_dst, dst, new_index, grp_offsets, grp_src, cu_vis_out, ws, ws_bytes,
                     stream);
}

lightkv_status lightkv_select(const lightkv_problem *p, const float *best_fd, const int32_t *best_dst,
                              int32_t *dst, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                              int32_t *cu_vis_out, void *ws, size_t ws_bytes, void *stream) {
  // without keys, best_fd / best_dst are only read
  return select_impl(p, false, const_cast<float *>(best_fd), const_cast<int32_t *>(best_dst), dst, new_index,
                     grp_offsets, grp_src, cu_vis_out, ws, ws_bytes, stream);
}

static lightkv_status rows_call(int mode, const lightkv_problem *p, const int32_t *new_index,
                                const int32_t *grp_offsets, const int32_t *grp_src, const float *xi,
                                const void *X, int64_t ldx, const void *K, int64_t ldk, const void *V, int64_t ldv,
                                const int32_t *pos, void *Xo, void *Ko, void *Vo, int32_t *pos_out,
                                float *x_sqnorm_out, int64_t out_rows, int64_t tail_rows, const int32_t *cu_vis_out,
                                void *stream) {
  Checked c;
  lightkv_status st = check_problem(p, false, false, c);
  if (st != LIGHTKV_OK) return st;
  if (tail_rows < 0 || (uint64_t)tail_rows > (1ull << 31)) return LIGHTKV_ERR_SHAPE;
  if (tail_rows > 0 && !cu_vis_out) return LIGHTKV_ERR_NULL;
  if (mode != 1 && (!grp_offsets || !grp_src || !xi)) return LIGHTKV_ERR_NULL;
  if (mode != 0 && !new_index) return LIGHTKV_ERR_NULL;
  if (mode != 0 && out_rows < 0) return LIGHTKV_ERR_SHAPE;
  if (mode != 0 && out_rows > c.sum_n + tail_rows) out_rows = c.sum_n + tail_rows;
  const void *in[3] = {X, K, V};
  void *out[3] = {Xo, Ko, Vo};
  const int64_t ld[3] = {ldx, ldk, ldv};
  RowTensors t{};
  for (int i = 0; i < 3; ++i) {
    if (mode != 0 && ((in[i] == nullptr) != (out[i] == nullptr))) return LIGHTKV_ERR_NULL;
    if (!row_tensor_ok(in[i], ld[i], p->d, c.elem_bytes, st)) return st;
    if (mode != 0 && in[i]) {
      if (!aligned16(out[i])) return LIGHTKV_ERR_UNSUPPORTED;
      const char *a = static_cast<const char *>(in[i]);
      const char *b = static_cast<const char *>(out[i]);
      const size_t in_bytes = ((size_t)c.sum_n + (size_t)tail_rows) * (size_t)ld[i] * c.elem_bytes;
      const size_t out_bytes = (size_t)out_rows * (size_t)p->d * c.elem_bytes;
      if (a == b || (b > a && b < a + in_bytes) || (a > b && a < b + out_bytes)) return LIGHTKV_ERR_SHAPE;
    }
    t.in[i] = in[i];
    t.out[i] = mode == 0 ? const_cast<void *>(in[i]) : out[i];
    t.ld_in[i] = ld[i];
    t.ld_out[i] = mode == 0 ? ld[i] : p->d;
  }
  if (mode != 0 && ((pos == nullptr) != (pos_out == nullptr))) return LIGHTKV_ERR_NULL;
  if (mode != 0 && pos && pos == pos_out) return LIGHTKV_ERR_SHAPE;
  if (x_sqnorm_out && (!X || (reinterpret_cast<uintptr_t>(x_sqnorm_out) & 3))) return LIGHTKV_ERR_NULL;
  if (launch_rows(mode, p->dtype, p->d, c.sum_n, t, new_index, grp_offsets, grp_src, xi, pos, pos_out, x_sqnorm_out,
                  out_rows, static_cast<hipStream_t>(stream)) != hipSuccess)
    return LIGHTKV_ERR_LAUNCH;
  if (tail_rows > 0 && launch_tail_rows(p->dtype, p->d, c.sum_n, p->batch, t, pos, pos_out, cu_vis_out, tail_rows, out_rows,
                                        static_cast<hipStream_t>(stream)) != hipSuccess)
    return LIGHTKV_ERR_LAUNCH;
  return LIGHTKV_OK;
}

lightkv_status lightkv_aggregate(const lightkv_problem *p, const int32_t *grp_offsets, const int32_t *grp_src,
                                 const float *xi, void *X, int64_t ldx, void *K, int64_t ldk,
                                 void *V, int64_t ldv, void *stream) {
  return rows_call(0, p, nullptr, grp_offsets, grp_src, xi, X, ldx, K, ldk, V, ldv, nullptr, nullptr, nullptr,
                   nullptr, nullptr, nullptr, 0, 0, nullptr, stream);
}

lightkv_status lightkv_compact(const lightkv_problem *p, const int32_t *new_index,
                               const void *X, int64_t ldx, const void *K, int64_t ldk,
                               const void *V, int64_t ldv, const int32_t *pos,
                               void *X_out, void *K_out, void *V_out, int32_t *pos_out, float *x_sqnorm_out,
                               int64_t out_rows, int64_t tail_rows, const int32_t *cu_vis_out, void *stream) {
  return rows_call(1, p, new_index, nullptr, nullptr, nullptr, X, ldx, K, ldk, V, ldv, pos, X_out, K_out, V_out,
                   pos_out, x_sqnorm_out, out_rows, tail_rows, cu_vis_out, stream);
}

lightkv_status lightkv_aggregate_compact(const lightkv_problem *p, const int32_t *new_index,
                                         const int32_t *grp_offsets, const int32_t *grp_src, const float *xi,
                                         const void *X, int64_t ldx, const void *K, int64_t ldk,
                                         const void *V, int64_t ldv, const int32_t *pos,
                                         void *X_out, void *K_out, void *V_out, int32_t *pos_out,
                                         float *x_sqnorm_out, int64_t out_rows, int64_t tail_rows,
                                         const int32_t *cu_vis_out, void *stream) {
  return rows_call(2, p, new_index, grp_offsets, grp_src, xi, X, ldx, K, ldk, V, ldv, pos, X_out, K_out, V_out,
                   pos_out, x_sqnorm_out, out_rows, tail_rows, cu_vis_out, stream);
}

}  // extern "C"

// ---- lightkv_select without a workspace argument ---------------------------------------------------------------
// For callers that can neither allocate nor carry a workspace (code under graph capture, serving loops with a fixed
// memory plan): the selection's two per-token scratch arrays live in a static device array of this library.  Each
// device holds its own copy of the array at its own address; the address is looked up once per device and used from
// then on -- the array's name itself is only a host-side stand-in.
constexpr int STATIC_SELECT_MAX_TOKENS = LIGHTKV_SELECT_STATIC_MAX_TOKENS;
static __device__ __align__(256) int32_t scratch[2 * STATIC_SELECT_MAX_TOKENS];   // [0, MAX): source counts, [MAX, 2 MAX): source ranks

namespace {

__global__ __launch_bounds__(256) void clear_scratch_kernel(int32_t *a, int32_t *b, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) { a[i] = 0; b[i] = 0; }
}

// device address of `scratch` on the current device (nullptr if it cannot be had)
int32_t *static_scratch_for_current_device() {
  static int32_t *ptr[64] = {};
  static std::mutex mu;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
    ptr[dev] = static_cast<int32_t *>(p);
  }
  return ptr[dev];
}
}  // namespace

extern "C" lightkv_status lightkv_select_static(const lightkv_problem *p, const float *best_fd, const int32_t *best_dst,
                                                int32_t *dst, int32_t *new_index, int32_t *grp_offsets,
                                                int32_t *grp_src, int32_t *cu_vis_out, void *stream) {
  Checked c;
  lightkv_status st = check_problem(p, true, false, c);
  if (st != LIGHTKV_OK) return st;
  if (!p->win_remove || !best_fd || !best_dst || !dst || !new_index || !grp_offsets || !grp_src || !cu_vis_out)
    return LIGHTKV_ERR_NULL;
  if (edge_topk(p) || full_pairwise(p)) return LIGHTKV_ERR_UNSUPPORTED;
  if (c.sum_n > STATIC_SELECT_MAX_TOKENS) return LIGHTKV_ERR_UNSUPPORTED;   // beyond the static array
  int32_t *base = static_scratch_for_current_device();
  if (!base) return LIGHTKV_ERR_LAUNCH;
  int32_t *cnt = base, *rank = base + STATIC_SELECT_MAX_TOKENS;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (c.sum_n > 0) {
    // the array keeps the previous call's contents: what this call reads starts from zero (a fill kernel rather than
    // a memset node, so that the call can be captured into a graph)
    hipLaunchKernelGGL(clear_scratch_kernel, dim3((unsigned)((c.sum_n + 255) / 256)), dim3(256), 0, s, cnt, rank, c.sum_n);
    if (hipGetLastError() != hipSuccess) return LIGHTKV_ERR_LAUNCH;
  }
  if (launch_select(p->n_windows, c.max_window, p->batch, c.sum_n, p->cu_vis, p->win_offsets, p->win_tokens,
                    p->win_remove, nullptr, 0, 0, const_cast<float *>(best_fd), const_cast<int32_t *>(best_dst), dst,
                    new_index, grp_offsets, grp_src, cu_vis_out, cnt, rank, p->direction, s) != hipSuccess)
    return LIGHTKV_ERR_LAUNCH;
  return LIGHTKV_OK;
}
