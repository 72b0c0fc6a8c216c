// The hierarchical schedule (paper Sec. 3.2.2) as one call: every stage's windows, scores, selection and merge are
// enqueued through the library's own entry points, arranged over the caller's stream and two helper streams so that
//   - xi (needs only Q and the stage's K rows) runs next to the feature-divergence chain and the selection,
//   - the next stage's windows (need only pos and the selection) are built next to the merge of the rows.
// Nothing here launches a kernel itself or allocates device memory.  lightkv_compress_schedule never synchronises;
// lightkv_compress_schedule_ratio (token counts that depend on the data) waits for the stream once per stage, to read
// the sequence offsets the stage left.
#include "../../include/lightkv.h"

#include "lk_helpers.h"
#include "lk_launch.h"

#include <hip/hip_runtime.h>
#include <mutex>
#include <algorithm>

namespace {

// Helper streams and events of one call: stream[0] runs xi, stream[1] builds the next stage's windows; event[0..3] =
// fork_xi, join_xi, fork_win, join_win.  Sets come from a per-device pool (lk_helpers.h), distinct from the one
// lightkv_score uses for its own fork.
using Helpers = lk::HelperSet<2, 4>;
enum { EV_FORK_XI = 0, EV_JOIN_XI = 1, EV_FORK_WIN = 2, EV_JOIN_WIN = 3 };

// `to` waits for everything enqueued on `from` so far
bool order_after(hipStream_t to, hipStream_t from, hipEvent_t ev) {
  return hipEventRecord(ev, from) == hipSuccess && hipStreamWaitEvent(to, ev, 0) == hipSuccess;
}

}  // namespace

extern "C" lightkv_status lightkv_compress_schedule(const lightkv_stage *stages, int32_t n_stages,
                                                    int32_t tiles, int32_t grid_h, int32_t grid_w,
                                                    const void *X, int64_t ldx, const void *K, int64_t ldk,
                                                    const void *V, int64_t ldv, const int32_t *pos,
                                                    const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                                    float softmax_scale, void *ws, size_t ws_bytes, void *stream) {
  if (!stages || !X || !K || !V || !pos || !Q) return LIGHTKV_ERR_NULL;
  if (n_stages < 1) return LIGHTKV_ERR_SHAPE;
  for (int s = 0; s < n_stages; ++s) {
    const lightkv_stage &st = stages[s];
    if (st.reserved != 0 || st.problem.match != LIGHTKV_MATCH_BEST_PER_A) return LIGHTKV_ERR_UNSUPPORTED;
    if (!st.win_offsets || !st.win_tokens || !st.xi || !st.best_fd || !st.best_dst || !st.dst || !st.new_index ||
        !st.grp_offsets || !st.grp_src || !st.cu_vis_out || !st.X_out || !st.K_out || !st.V_out || !st.pos_out)
      return LIGHTKV_ERR_NULL;
    if (st.problem.win_offsets != st.win_offsets || st.problem.win_tokens != st.win_tokens) return LIGHTKV_ERR_SHAPE;
    if (!st.problem.h_cu_vis || !st.problem.cu_vis) return LIGHTKV_ERR_NULL;
    if (st.problem.batch != stages[0].problem.batch || st.problem.d != stages[0].problem.d) return LIGHTKV_ERR_SHAPE;
    if (st.cu_vis_target) {   // counts from the token budget: the schedule writes the array the descriptor points to
      if (!st.win_remove) return LIGHTKV_ERR_NULL;
      if (st.problem.win_remove != st.win_remove || st.problem.n_windows % st.problem.batch != 0) return LIGHTKV_ERR_SHAPE;
    }
    size_t need = 0;
    const lightkv_status ws_st = lightkv_workspace_size(&st.problem, &need);
    if (ws_st != LIGHTKV_OK) return ws_st;
    if (!ws || ws_bytes < need) return LIGHTKV_ERR_WORKSPACE;
  }
  hipStream_t main = static_cast<hipStream_t>(stream);
  std::unique_lock<std::mutex> guard;
  Helpers *h = lk::acquire_helpers<2, 4>(main, guard);

  const int d = stages[0].problem.d, head_dim = stages[0].problem.head_dim;
  const void *Xi = X, *Ki = K, *Vi = V;
  int64_t ldxi = ldx, ldki = ldk, ldvi = ldv;
  const int32_t *posi = pos;
  const float *sq = nullptr;          // squared norms of Xi, once a stage has produced them
  bool windows_pending = false;       // this stage's windows are being built on the window stream
  lightkv_status rc = LIGHTKV_OK;
  bool xi_forked = false, win_forked = false;
  for (int s = 0; s < n_stages && rc == LIGHTKV_OK; ++s) {
    const lightkv_stage &st = stages[s];
    const lightkv_problem *p = &st.problem;
    const int sum_n = p->h_cu_vis[p->batch];
    const bool one_stream = p->max_window_tokens > 0 && p->max_window_tokens <= 64 &&
                            sum_n <= LIGHTKV_ONE_STREAM_MAX_TOKENS;
    // ---- xi on its helper stream (or, if there is none, first on the caller's)
    xi_forked = false;
    if (!one_stream) {
      hipStream_t xs = main;
      if (h && order_after(h->stream[0], main, h->event[EV_FORK_XI])) { xs = h->stream[0]; xi_forked = true; }
      else if (h) (void)hipGetLastError();
      rc = lightkv_score(p, nullptr, 0, nullptr, Q, q_tok_stride, q_head_stride, Ki, ldki, head_dim, LIGHTKV_XI_TEXT_QUERY,
                         nullptr, softmax_scale, st.xi, nullptr, nullptr, nullptr, 0, ws, ws_bytes, xs);
      if (xi_forked && hipEventRecord(h->event[EV_JOIN_XI], h->stream[0]) != hipSuccess) rc = rc == LIGHTKV_OK ? LIGHTKV_ERR_LAUNCH : rc;
    }
    // ---- windows: built by the previous stage's tail, or here
    if (windows_pending) {
      if (win_forked && hipStreamWaitEvent(main, h->event[EV_JOIN_WIN], 0) != hipSuccess) rc = rc == LIGHTKV_OK ? LIGHTKV_ERR_LAUNCH : rc;
    } else if (rc == LIGHTKV_OK) {
      if (st.cu_vis_target)   // windows and their counts (one launch where the partition kernel allows it)
        rc = (lightkv_status)lk::build_windows_with_counts(p->batch, p->h_cu_vis, p->cu_vis, posi, nullptr, nullptr, tiles,
                                                           grid_h, grid_w, st.w, st.win_offsets, st.win_tokens, p->n_windows,
                                                           p->direction, st.cu_vis_target, st.win_remove, st.status, main);
      else
        rc = lightkv_build_windows(p->batch, p->h_cu_vis, p->cu_vis, posi, tiles, grid_h, grid_w, st.w, st.win_offsets,
                                   st.win_tokens, main);
    }
    windows_pending = false;
    // ---- feature divergence + selection
    if (rc == LIGHTKV_OK) {
      if (one_stream)
        rc = lightkv_score_select(p, Xi, ldxi, sq, Q, q_tok_stride, q_head_stride, Ki, ldki, head_dim,
                                  LIGHTKV_XI_TEXT_QUERY, nullptr, softmax_scale, st.xi, st.best_fd, st.best_dst, st.dst,
                                  st.new_index, st.grp_offsets, st.grp_src, st.cu_vis_out, ws, ws_bytes, main);
      else
        rc = lightkv_score_select(p, Xi, ldxi, sq, nullptr, 0, 0, nullptr, 0, 0, LIGHTKV_XI_GIVEN, nullptr, softmax_scale,
                                  st.xi, st.best_fd, st.best_dst, st.dst, st.new_index, st.grp_offsets, st.grp_src,
                                  st.cu_vis_out, ws, ws_bytes, main);
    }
    // ---- the next stage's windows, next to the merge
    win_forked = false;
    if (rc == LIGHTKV_OK && s + 1 < n_stages) {
      const lightkv_stage &nx = stages[s + 1];
      hipStream_t wsx = main;
      if (h && order_after(h->stream[1], main, h->event[EV_FORK_WIN])) { wsx = h->stream[1]; win_forked = true; }
      else if (h) (void)hipGetLastError();
      // ... with their counts: the next stage's budget over the windows as they now are (cu_vis_out of this stage is
      // the next stage's cu_vis)
      if (nx.cu_vis_target)
        rc = (lightkv_status)lk::build_windows_with_counts(p->batch, p->h_cu_vis, p->cu_vis, posi, st.new_index, st.cu_vis_out,
                                                           tiles, grid_h, grid_w, nx.w, nx.win_offsets, nx.win_tokens,
                                                           nx.problem.n_windows, nx.problem.direction, nx.cu_vis_target,
                                                           nx.win_remove, nx.status, wsx);
      else
        rc = lightkv_build_windows_next(p->batch, p->h_cu_vis, p->cu_vis, posi, st.new_index, st.cu_vis_out, tiles, grid_h,
                                        grid_w, nx.w, nx.win_offsets, nx.win_tokens, wsx);
      if (win_forked && hipEventRecord(h->event[EV_JOIN_WIN], h->stream[1]) != hipSuccess) rc = rc == LIGHTKV_OK ? LIGHTKV_ERR_LAUNCH : rc;
      windows_pending = true;
    }
    // ---- join xi, merge and compact
    if (xi_forked && hipStreamWaitEvent(main, h->event[EV_JOIN_XI], 0) != hipSuccess) rc = rc == LIGHTKV_OK ? LIGHTKV_ERR_LAUNCH : rc;
    xi_forked = false;
    if (rc == LIGHTKV_OK)
      rc = lightkv_aggregate_compact(p, st.new_index, st.grp_offsets, st.grp_src, st.xi, Xi, ldxi, Ki, ldki, Vi, ldvi,
                                     posi, st.X_out, st.K_out, st.V_out, st.pos_out, st.x_sqnorm_out, st.out_rows, 0, nullptr, main);
    Xi = st.X_out; Ki = st.K_out; Vi = st.V_out;
    ldxi = ldki = ldvi = d;
    posi = st.pos_out;
    sq = st.x_sqnorm_out;
  }
  // whatever happened, nothing stays forked: the helper streams rejoin the caller's
  if (xi_forked) (void)hipStreamWaitEvent(main, h->event[EV_JOIN_XI], 0);
  if (win_forked) (void)hipStreamWaitEvent(main, h->event[EV_JOIN_WIN], 0);
  return rc;
}

// The schedule when a stage's token count depends on the data (the k lowest edges of a window, the full pairwise
// visit, or any matching driven by the ratio of Sec. 3.2.2 instead of fixed budgets): per-window counts come from the
// window sizes on the device, and the batch + 1 sequence offsets a stage leaves are read back before the next stage is
// laid out -- the one synchronisation per stage.
extern "C" lightkv_status lightkv_compress_schedule_ratio(const lightkv_stage *stages, int32_t n_stages, const double *rho,
                                                          int32_t tiles, int32_t grid_h, int32_t grid_w,
                                                          const void *X, int64_t ldx, const void *K, int64_t ldk,
                                                          const void *V, int64_t ldv, const int32_t *pos,
                                                          const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                                          float softmax_scale, void *ws, size_t ws_bytes,
                                                          int32_t *h_cu_vis_out, void *stream) {
  if (!stages || !rho || !X || !K || !V || !pos || !Q || !h_cu_vis_out) return LIGHTKV_ERR_NULL;
  if (n_stages < 1) return LIGHTKV_ERR_SHAPE;
  const int batch = stages[0].problem.batch;
  if (batch < 1) return LIGHTKV_ERR_SHAPE;
  for (int s = 0; s < n_stages; ++s) {
    const lightkv_stage &st = stages[s];
    if (st.reserved != 0 || st.cu_vis_target) return LIGHTKV_ERR_UNSUPPORTED;
    if (!st.win_offsets || !st.win_tokens || !st.win_remove || !st.xi || !st.best_fd || !st.best_dst || !st.dst ||
        !st.new_index || !st.grp_offsets || !st.grp_src || !st.cu_vis_out || !st.X_out || !st.K_out || !st.V_out ||
        !st.pos_out)
      return LIGHTKV_ERR_NULL;
    if (st.problem.win_offsets != st.win_offsets || st.problem.win_tokens != st.win_tokens ||
        st.problem.win_remove != st.win_remove)
      return LIGHTKV_ERR_SHAPE;
    // counts and window sizes are the device's alone here
    if (st.problem.h_win_offsets || st.problem.h_win_remove) return LIGHTKV_ERR_UNSUPPORTED;
    if (st.problem.batch != batch || st.problem.d != stages[0].problem.d || st.problem.max_window_tokens <= 0 ||
        st.problem.n_windows % batch != 0)
      return LIGHTKV_ERR_SHAPE;
    if (!(rho[s] >= 0.0 && rho[s] <= 1e6)) return LIGHTKV_ERR_SHAPE;
  }
  if (!stages[0].problem.h_cu_vis || !stages[0].problem.cu_vis) return LIGHTKV_ERR_NULL;
  hipStream_t main = static_cast<hipStream_t>(stream);
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(main, &cs) != hipSuccess) { (void)hipGetLastError(); return LIGHTKV_ERR_LAUNCH; }
  if (cs != hipStreamCaptureStatusNone) return LIGHTKV_ERR_UNSUPPORTED;   // the call waits for the stream: not capturable
  std::unique_lock<std::mutex> guard;
  Helpers *h = lk::acquire_helpers<2, 4>(main, guard);

  const int d = stages[0].problem.d, head_dim = stages[0].problem.head_dim;
  const void *Xi = X, *Ki = K, *Vi = V;
  int64_t ldxi = ldx, ldki = ldk, ldvi = ldv;
  const int32_t *posi = pos;
  const float *sq = nullptr;
  const int32_t *h_cu = stages[0].problem.h_cu_vis;   // offsets of the stage's input: on the host ...
  const int32_t *d_cu = stages[0].problem.cu_vis;     // ... and on the device
  bool windows_pending = false, win_forked = false;
  lightkv_status rc = LIGHTKV_OK;
  for (int s = 0; s < n_stages && rc == LIGHTKV_OK; ++s) {
    const lightkv_stage &st = stages[s];
    lightkv_problem q = st.problem;
    q.h_cu_vis = h_cu;
    q.cu_vis = d_cu;
    int max_seq = 0;
    for (int b = 0; b < batch; ++b) max_seq = std::max(max_seq, h_cu[b + 1] - h_cu[b]);
    // a window holds no more tokens than its sequence: the tighter bound picks the cheaper launch plans; the plans are
    // not monotone in it, so if that one wants more workspace than there is, the stage's own bound is used
    const int bound = st.problem.max_window_tokens;
    q.max_window_tokens = std::max(1, std::min(bound, max_seq));
    size_t need = 0;
    rc = lightkv_workspace_size(&q, &need);
    if (rc == LIGHTKV_OK && (!ws || ws_bytes < need) && q.max_window_tokens != bound) {
      q.max_window_tokens = bound;
      rc = lightkv_workspace_size(&q, &need);
    }
    if (rc == LIGHTKV_OK && (!ws || ws_bytes < need)) rc = LIGHTKV_ERR_WORKSPACE;
    const int count_mode = q.match == LIGHTKV_MATCH_EDGE_TOPK ? LIGHTKV_COUNT_EDGES : LIGHTKV_COUNT_RATIO;
    // ---- windows and their counts: built next to the previous stage's merge, or here
    if (windows_pending) {
      if (win_forked && hipStreamWaitEvent(main, h->event[EV_JOIN_WIN], 0) != hipSuccess) rc = rc == LIGHTKV_OK ? LIGHTKV_ERR_LAUNCH : rc;
      win_forked = false;
    } else if (rc == LIGHTKV_OK) {
      rc = lightkv_build_windows(batch, h_cu, d_cu, posi, tiles, grid_h, grid_w, st.w, st.win_offsets, st.win_tokens, main);
      if (rc == LIGHTKV_OK)
        rc = lightkv_window_counts(batch, q.n_windows, st.win_offsets, count_mode, q.direction, rho[s], nullptr, nullptr,
                                   st.win_remove, nullptr, main);
    }
    windows_pending = false;
    // ---- scores (xi and feature divergence) and selection
    if (rc == LIGHTKV_OK)
      rc = lightkv_score_select(&q, Xi, ldxi, sq, Q, q_tok_stride, q_head_stride, Ki, ldki, head_dim, LIGHTKV_XI_TEXT_QUERY,
                                nullptr, softmax_scale, st.xi, st.best_fd, st.best_dst, st.dst, st.new_index, st.grp_offsets,
                                st.grp_src, st.cu_vis_out, ws, ws_bytes, main);
    // ---- the next stage's windows and counts follow from the selection alone: next to the merge
    if (rc == LIGHTKV_OK && s + 1 < n_stages) {
      const lightkv_stage &nx = stages[s + 1];
      const int nx_mode = nx.problem.match == LIGHTKV_MATCH_EDGE_TOPK ? LIGHTKV_COUNT_EDGES : LIGHTKV_COUNT_RATIO;
      hipStream_t wsx = main;
      if (h && order_after(h->stream[1], main, h->event[EV_FORK_WIN])) { wsx = h->stream[1]; win_forked = true; }
      else if (h) (void)hipGetLastError();
      rc = lightkv_build_windows_next(batch, h_cu, d_cu, posi, st.new_index, st.cu_vis_out, tiles, grid_h, grid_w, nx.w,
                                      nx.win_offsets, nx.win_tokens, wsx);
      if (rc == LIGHTKV_OK)
        rc = lightkv_window_counts(batch, nx.problem.n_windows, nx.win_offsets, nx_mode, nx.problem.direction, rho[s + 1],
                                   nullptr, nullptr, nx.win_remove, nullptr, wsx);
      if (win_forked && hipEventRecord(h->event[EV_JOIN_WIN], h->stream[1]) != hipSuccess) rc = rc == LIGHTKV_OK ? LIGHTKV_ERR_LAUNCH : rc;
      windows_pending = true;
    }
    // ---- merge and compact
    if (rc == LIGHTKV_OK)
      rc = lightkv_aggregate_compact(&q, st.new_index, st.grp_offsets, st.grp_src, st.xi, Xi, ldxi, Ki, ldki, Vi, ldvi, posi,
                                     st.X_out, st.K_out, st.V_out, st.pos_out, st.x_sqnorm_out, st.out_rows, 0, nullptr, main);
    // ---- the offsets the stage left: the next stage's descriptor
    int32_t *h_out = h_cu_vis_out + (size_t)s * (batch + 1);
    if (rc == LIGHTKV_OK &&
        (hipMemcpyAsync(h_out, st.cu_vis_out, sizeof(int32_t) * (batch + 1), hipMemcpyDeviceToHost, main) != hipSuccess ||
         hipStreamSynchronize(main) != hipSuccess)) {
      (void)hipGetLastError();
      rc = LIGHTKV_ERR_LAUNCH;
    }
    if (rc == LIGHTKV_OK) {
      // a sequence never grows, and everything that stays must have found room in the stage's outputs
      bool ok = h_out[0] == 0;
      for (int b = 0; ok && b < batch; ++b) {
        const int n = h_out[b + 1] - h_out[b];
        ok = n >= 0 && n <= h_cu[b + 1] - h_cu[b];
      }
      if (!ok || h_out[batch] > st.out_rows) rc = LIGHTKV_ERR_SHAPE;
    }
    Xi = st.X_out; Ki = st.K_out; Vi = st.V_out;
    ldxi = ldki = ldvi = d;
    posi = st.pos_out;
    sq = st.x_sqnorm_out;
    h_cu = h_out;
    d_cu = st.cu_vis_out;
  }
  if (win_forked) (void)hipStreamWaitEvent(main, h->event[EV_JOIN_WIN], 0);   // nothing stays forked
  return rc;
}
