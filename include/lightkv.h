/*
 * lightkv.h -- C ABI of the LightKV compression step for AMD MI355X (gfx950).
 *
 * One step of prompt-guided vision-token compression, as run after a selected
 * decoder layer during LVLM prefill (paper Sec. 3.2): inside every spatial window
 * the vision tokens are split into two alternating node sets A and B (Sec. 3.2.1,
 * Step 1), every A node is scored against the B nodes by feature divergence
 * FD = 1 - cos (Eq. "similarity"), the lowest-FD edges are selected (Step 2), the
 * selected A nodes are averaged into their B node with the prompt-attention
 * weights xi (Step 3, Eq. "attention-factor" and Eq. "message-passing"), and the
 * merged A nodes are dropped from the hidden states and from the layer's K/V rows
 * alike (Steps 4-5; appendix figure "Method overview").
 *
 * Conventions
 *   - plain C, no C++ types cross the boundary; every function returns a
 *     lightkv_status (0 = OK) and never throws.  Arguments are validated before
 *     anything is enqueued: a single-step call that returns an error has touched no
 *     output.  lightkv_compress_schedule validates every stage first, too; if a
 *     later stage's launch then fails, the stages before it stay enqueued.
 *   - pointers named h_* are HOST memory, read during the call only.  Every other
 *     pointer is DEVICE memory owned by the caller; the library allocates no device
 *     memory and frees none.  Scratch comes from the caller's workspace `ws` (size
 *     from lightkv_workspace_size, 256-byte aligned); lightkv_select_static uses a
 *     static device array instead.
 *   - state the library keeps between calls (per device, host-side handles only,
 *     created on first use outside stream capture, default priority, never
 *     destroyed): one helper stream with two events for lightkv_score, two helper
 *     streams with four events for the two schedule calls, and the "large LDS"
 *     attribute of three kernels.  Calls whose `stream` is being captured never
 *     touch the helper streams: they enqueue everything on `stream` in order, so
 *     a capture only ever contains the caller's stream.
 *   - all work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) or on helper streams that fork from and rejoin it before the
 *     call returns; no call synchronises or reads device memory on the host, with
 *     one exception that says so: lightkv_compress_schedule_ratio.
 *   - tensors are token-major: row i holds the `d` contiguous elements of token i;
 *     `ld*` are row strides in elements.  Sequences of a batch are packed one after
 *     the other; cu_vis / cu_txt are their [batch+1] offsets.
 *   - indices are int32.  Device data pointers must be 16-byte aligned, row strides
 *     multiples of 8 elements (bf16) or 4 elements (fp32).
 *   - element type: LIGHTKV_BF16 (bf16 storage, fp32 accumulation on the matrix
 *     cores) or LIGHTKV_F32.
 *   - threads: any host thread may call; calls are independent as long as their
 *     outputs and workspaces do not overlap (two calls that share a workspace must
 *     be ordered by the caller's streams, except where a function says otherwise).
 *     Calls that use a helper stream take turns enqueueing (a mutex per device).
 *   - results are bit-reproducible: the same inputs give the same outputs on every
 *     call, whatever else runs on the device.
 */
#ifndef LIGHTKV_H
#define LIGHTKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LIGHTKV_OK = 0,
  LIGHTKV_ERR_NULL = 1,         /* a required pointer is NULL                                   */
  LIGHTKV_ERR_SHAPE = 2,        /* sizes/strides/offsets inconsistent, aliasing in/out buffers   */
  LIGHTKV_ERR_WINDOWS = 3,      /* window CSR not a partition of the tokens                      */
  LIGHTKV_ERR_REMOVE_COUNT = 4, /* some r_w exceeds |A_w|: one step removes at most half a window
                                   (limitations paragraph of the paper)                           */
  LIGHTKV_ERR_UNSUPPORTED = 5,  /* dtype, head_dim, alignment or a size beyond the stated limits */
  LIGHTKV_ERR_WORKSPACE = 6,    /* workspace NULL, misaligned or too small                       */
  LIGHTKV_ERR_LAUNCH = 7        /* the HIP runtime refused a launch                              */
} lightkv_status;

typedef enum { LIGHTKV_F32 = 0, LIGHTKV_BF16 = 1 } lightkv_dtype;

/* How the prompt-guidance weight xi_i (Eq. "attention-factor") is obtained. */
typedef enum {
  /* prompt token j is the query, vision token i the key: xi_i = sum_h sum_j softmax_i(q_j.k_i*scale).
     The softmax runs over the sequence's vision keys, or uses the caller's lse[heads, sumT]. */
  LIGHTKV_XI_TEXT_QUERY = 0,
  /* index order of the equation taken literally: vision token i is the query, prompt token j the key,
     xi_i = sum_h sum_j exp(q_i.k_j*scale - lse[h,i]); lse[heads, sumN] (log-sum-exp of the whole
     attention row of query i, as a flash-style attention kernel returns it) is required. */
  LIGHTKV_XI_VISION_QUERY = 1,
  /* xi is an input (e.g. all ones: the uniform-weight ablation of the paper). */
  LIGHTKV_XI_GIVEN = 2
} lightkv_xi_mode;

/* Divergence between two hidden states used for the token pairing (Step 1).  The method uses the cosine form;
   the two distances are those of the paper's similarity-metric ablation (appendix).  best_fd then holds
   |a - b| or |a - b|^2; the rest of the step is unchanged. */
typedef enum {
  LIGHTKV_METRIC_COSINE = 0,     /* FD = 1 - cos(a, b)  (Eq. "similarity") */
  LIGHTKV_METRIC_EUCLIDEAN = 1,  /* |a - b|   */
  LIGHTKV_METRIC_L2SQ = 2        /* |a - b|^2 */
} lightkv_metric;

/* How Step 2 builds the candidate set T_rho of a window from the FD of its |A| x |B| pairs. */
typedef enum {
  /* every A node offers its lowest-FD B node, and the r_w A nodes with the lowest offers are merged: exactly r_w tokens
     leave the window (the reading all sizes in this header assume). */
  LIGHTKV_MATCH_BEST_PER_A = 0,
  /* the sentence of Step 2 taken literally: the win_remove[w] lowest-FD EDGES of the window (ties: lower A position,
     then lower B position).  An A node may own several of them -- it is averaged into each of those B nodes with its
     full weight -- and leaves if it owns at least one, so the number of tokens that leave is known only on the
     device (cu_vis_out): between ceil(k / |B|) and min(k, |A|) per window.  Supported by lightkv_score_select for
     windows of at most LIGHTKV_EDGE_MAX_WINDOW_TOKENS tokens; see there. */
  LIGHTKV_MATCH_EDGE_TOPK = 1,
  /* full pairwise matching, the appendix ablation ("Bipartite vs. full pairwise matching"): no A/B split, FD between
     every two tokens of a window (the whole v x v matrix, 4 x the bipartite block), every token offers its lowest-FD
     neighbour (ties: the neighbour earlier in the window).  The appendix gives no merge rule; this build's reading:
     the tokens of a window are visited in ascending order of their offer (ties: earlier in the window first), and a
     visited token is merged into its neighbour unless a token merged earlier was merged INTO it, or its neighbour has
     itself been merged away; the visit ends after win_remove[w] merges.  So at most win_remove[w] tokens leave a
     window (fewer if the visit runs out: the count is known on the device, cu_vis_out), no token that leaves is a
     destination, and best_fd / best_dst hold every token's offer (+inf / -1 for a token alone in its window).
     lightkv_score computes the offers, lightkv_score_select offers and selection (lightkv_select alone returns
     LIGHTKV_ERR_UNSUPPORTED); bf16, d a multiple of 64. */
  LIGHTKV_MATCH_FULL_PAIRWISE = 2
} lightkv_match;

/* Which side of a window's bipartite split proposes (Sec. 3.2.1, message-passing paragraph: messages go from A to B,
   and the reverse direction is defined analogously).  With B_TO_A the tokens at the odd local positions (set B) each
   offer their lowest-FD edge into set A (ties: the A node earlier in the window), the r_w of them with the lowest FD
   are merged into their A node, and set A stays: every statement of this header about "A" and "B" then holds with
   the two sets exchanged (0 <= r_w <= |B_w| = floor(v_w / 2); best_fd / best_dst are written for the B nodes and are
   +inf / -1 for the A nodes).  Defined for LIGHTKV_MATCH_BEST_PER_A only; with another lightkv_match the calls return
   LIGHTKV_ERR_UNSUPPORTED. */
typedef enum {
  LIGHTKV_DIRECTION_A_TO_B = 0,   /* a zeroed struct: the paper's direction */
  LIGHTKV_DIRECTION_B_TO_A = 1
} lightkv_direction;

/* Limits of this build. */
#define LIGHTKV_MAX_WINDOW_TOKENS 4096   /* tokens in one window                    */
#define LIGHTKV_MAX_SEQ_TOKENS    16384  /* vision tokens in one sequence           */
#define LIGHTKV_MAX_TEXT_TOKENS   4096   /* prompt tokens in one sequence           */
#define LIGHTKV_EDGE_MAX_WINDOW_TOKENS 4096 /* tokens in one window with LIGHTKV_MATCH_EDGE_TOPK; windows bounded by more than
                                               256 tokens are ranked through a matrix of all their FD values in the workspace */
#define LIGHTKV_SELECT_STATIC_MAX_TOKENS 65536  /* vision tokens of a batch in lightkv_select_static */
/* Steps of at most this many vision tokens whose windows hold at most 64 tokens: lightkv_score_select runs the xi
   passes inside the launches of the FD chain, on the caller's stream alone (see there). */
#define LIGHTKV_ONE_STREAM_MAX_TOKENS 1024

/*
 * Problem descriptor of one compression step (host struct).
 * Windows (Sec. 3.2 and Sec. 3.2.2 "Window partitioning") are given in CSR form:
 * window w owns win_tokens[win_offsets[w] .. win_offsets[w+1]), token indices into
 * the packed tensors, ascending.  Local positions 0,2,4,.. form set A, 1,3,5,.. set B
 * (Step 1).  Windows never cross sequences.  r_w = win_remove[w] tokens of A are
 * merged away in window w (Step 2; 0 <= r_w <= |A_w|).
 */
typedef struct lightkv_problem {
  int32_t batch;              /* sequences in the batch                                          */
  int32_t d;                  /* elements per row of X, K, V (= heads*head_dim)                  */
  int32_t heads, head_dim;    /* head_dim in {32, 64, 128}                                       */
  int32_t dtype;              /* lightkv_dtype                                                   */
  int32_t n_windows;
  int32_t max_window_tokens;  /* host-side upper bound on the size of any window; sizes launches.
                                 0 = take it from h_win_offsets (then required).                 */
  int32_t metric;             /* lightkv_metric; 0 (a zeroed struct) = cosine FD; other values ->
                                 LIGHTKV_ERR_UNSUPPORTED                                          */
  int32_t match;              /* lightkv_match; 0 (a zeroed struct) = one edge per A node.  With
                                 LIGHTKV_MATCH_EDGE_TOPK win_remove[w] counts EDGES (0 <= k_w <= |A_w| |B_w|;
                                 h_win_remove optional, see lightkv_score_select); with LIGHTKV_MATCH_FULL_PAIRWISE it is
                                 the most tokens that may leave (0 <= r_w <= ceil(v_w / 2))       */
  int32_t direction;          /* lightkv_direction; 0 (a zeroed struct) = A proposes, B receives    */
  const int32_t *h_cu_vis;    /* HOST [batch+1] vision-token offsets, h_cu_vis[0] = 0            */
  const int32_t *h_cu_txt;    /* HOST [batch+1] prompt-token offsets (may be NULL for XI_GIVEN)  */
  const int32_t *cu_vis;      /* device copy of h_cu_vis                                         */
  const int32_t *cu_txt;      /* device copy of h_cu_txt                                         */
  const int32_t *win_offsets; /* device [n_windows+1]                                            */
  const int32_t *win_tokens;  /* device [sumN]                                                   */
  const int32_t *win_remove;  /* device [n_windows]                                              */
  const int32_t *h_win_offsets; /* HOST mirror, optional: when given the CSR is validated on the host */
  const int32_t *h_win_remove;  /* HOST mirror, optional: when given r_w <= |A_w| is validated        */
} lightkv_problem;

const char *lightkv_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int lightkv_version(void);

/* Bytes of workspace that any call for this problem needs (upper bound over the four steps). */
lightkv_status lightkv_workspace_size(const lightkv_problem *p, size_t *bytes);

/*
 * Window partition (Sec. 3.2: the tokens are put back on their image grid and cut into w x w
 * non-overlapping windows; Sec. 3.2.2: later stages use fewer, larger windows).
 *   pos[sumN]  device: original grid cell of every current token, tile*grid_h*grid_w + row*grid_w + col
 *   window of a token = (tile, floor(row*w/grid_h), floor(col*w/grid_w)); w = 0: one window per sequence.
 *   Every sequence owns tiles*w*w windows (1 if w = 0), in that order; n_windows = batch * that.
 * Outputs: win_offsets[n_windows+1], win_tokens[sumN] (device).  Tokens of a window are listed in
 * ascending order.  Sequences longer than LIGHTKV_MAX_SEQ_TOKENS -> LIGHTKV_ERR_UNSUPPORTED.
 * A pos value outside the grid is clamped to the last tile/row/col.
 */
lightkv_status lightkv_build_windows(int32_t batch, const int32_t *h_cu_vis, const int32_t *cu_vis,
                                     const int32_t *pos, int32_t tiles, int32_t grid_h, int32_t grid_w,
                                     int32_t w, int32_t *win_offsets, int32_t *win_tokens, void *stream);

/*
 * The same partition for the NEXT stage of the hierarchical schedule (Sec. 3.2.2), taken from this stage's tensors
 * before they are compacted: h_cu_vis / cu_vis / pos describe the current tokens, new_index[sumN] (from
 * lightkv_select) says which of them stay and under which index, cu_vis_out[batch+1] (from lightkv_select) holds
 * the sequence offsets after compaction.  The outputs list the staying tokens under their new indices, exactly as
 * lightkv_build_windows would on the compacted pos -- but they depend on the selection only, so the call can be
 * enqueued next to the merge of the rows instead of behind it.
 */
lightkv_status lightkv_build_windows_next(int32_t batch, const int32_t *h_cu_vis, const int32_t *cu_vis,
                                          const int32_t *pos, const int32_t *new_index, const int32_t *cu_vis_out,
                                          int32_t tiles, int32_t grid_h, int32_t grid_w, int32_t w,
                                          int32_t *win_offsets, int32_t *win_tokens, void *stream);

/* Host arithmetic of the partition: windows a sequence owns (tiles*w*w, or 1 for w = 0) and the largest number of
   grid cells a window can cover (the bound callers pass as max_window_tokens).  Negative on invalid arguments. */
int32_t lightkv_windows_per_sequence(int32_t tiles, int32_t w);
int32_t lightkv_max_window_cells(int32_t tiles, int32_t grid_h, int32_t grid_w, int32_t w);

/* How lightkv_window_counts turns the schedule's ratio or token budget into per-window counts. */
typedef enum {
  /* Sec. 3.2.2: a fraction rho of every window's tokens leaves, r_w = floor(rho * v_w), never more than the window's
     set A (one step removes at most half: limitations paragraph). */
  LIGHTKV_COUNT_RATIO = 0,
  /* Step 2 as printed, for LIGHTKV_MATCH_EDGE_TOPK: k_w = floor(rho * v_w / 2) pairs, never more than |A_w| |B_w|. */
  LIGHTKV_COUNT_EDGES = 1,
  /* every sequence is given the length it must have after the step; the difference is spread over its windows as
     evenly as their sizes allow: with cap_w = |A_w| (0 for windows of fewer than two tokens) and q the largest level
     for which sum_w min(cap_w, q) stays within the budget, window w gives min(cap_w, q), and the first windows (in
     window order) with cap_w > q give one more until the budget is met.  Equal windows: floor(R/W) each, one more
     for the first R mod W. */
  LIGHTKV_COUNT_TARGET = 2
} lightkv_count_mode;

/*
 * Per-window counts r_w (or k_w) on the device, from the window sizes as they are (after earlier stages the windows
 * of a sequence no longer hold equal numbers of tokens).  Every sequence owns n_windows / batch windows.
 *   win_offsets[n_windows+1]  device, from lightkv_build_windows
 *   direction                 lightkv_direction: which set counts as "A" below (RATIO and TARGET; EDGES: A_TO_B only)
 *   rho                       RATIO / EDGES; a double, so that the floor is the one a host program computes
 *   cu_vis, cu_vis_target     TARGET: device [batch+1] offsets of the sequences now and after the step
 *   win_remove[n_windows]     device, out
 *   status[batch]             device, out, may be NULL: 1 where a sequence's budget cannot be met (negative, or more
 *                             than its sets A hold: then every window gives its whole set A), else 0
 */
lightkv_status lightkv_window_counts(int32_t batch, int32_t n_windows, const int32_t *win_offsets, int32_t mode,
                                     int32_t direction, double rho, const int32_t *cu_vis, const int32_t *cu_vis_target,
                                     int32_t *win_remove, int32_t *status, void *stream);

/*
 * Scores (Steps 1-3).
 *   X[sumN, d] (row stride ldx): vision hidden states.  For every A node the lowest-FD B node of its
 *   window: best_fd[i] = FD (fp32, clamped at 0), best_dst[i] = that B token; ties go to the B node that
 *   comes first in the window.  B rows, and A rows of windows without a B node, get +inf / -1.
 *   FD(a,b) = 1 - <x_a,x_b> / (max(|x_a|,1e-12) * max(|x_b|,1e-12))          (Eq. "similarity")
 *   x_sqnorm[sumN] (device, fp32, may be NULL): |x_i|^2 = sum_j X[i,j]^2 of every row of X as stored, if the caller
 *     already has it -- lightkv_compact / lightkv_aggregate_compact produce it for the rows they write.  It is trusted,
 *     not checked; it saves one pass over X where the library would compute the norms on their own (large windows on
 *     the matrix-core path) and is ignored elsewhere.  With the values those calls produce the results are bit-identical
 *     to passing NULL.
 *   xi[sumN]: prompt-guidance weight (Eq. "attention-factor"), floored at 1e-30.
 *     TEXT_QUERY  : Q = prompt queries [sumT, heads, head_dim], K = vision keys [sumN, heads, head_dim]
 *     VISION_QUERY: Q = vision queries [sumN, ...],             K = prompt keys [sumT, ...], lse required
 *     GIVEN       : Q, K, lse ignored, xi is read-only input and left as is.
 *     element (token t, head h, e) of Q sits at Q[t*q_tok_stride + h*q_head_stride + e], K alike.
 *   softmax_scale: 0 selects 1/sqrt(head_dim).   lse: natural-log units, layout [heads, tokens], or NULL.
 *   fd_dump (device, fp32, may be NULL; debugging): the FD of EVERY pair, window after window, each window a row-major
 *     |A_w| x |B_w| block (rows: A nodes in window order, columns: B nodes); block w starts at sum_{u<w} |A_u| |B_u|.
 *     fd_dump_floats is the capacity of the buffer in floats; pairs beyond it are not written.  The scoring kernels
 *     never form these values (they keep row minima): the dump comes from a plain kernel of its own that accumulates
 *     in fp64, so it agrees with best_fd to the accuracy of the scoring kernels' fp32 accumulation (about 1e-6), not
 *     bit for bit.  At most 65535 windows; needs X.
 *   The two halves are independent and may be enqueued by two calls, e.g. on two streams with the same workspace:
 *   X == NULL computes xi only (windows, best_fd, best_dst are not touched), xi_mode GIVEN computes the FD half only.
 *   When both halves are requested in one call the library runs them concurrently (xi on an internal helper stream
 *   that forks from and joins `stream`; the only object the library ever creates, one per device, on the first such
 *   call outside stream capture; host threads that make such calls on one device take turns enqueueing).
 */
lightkv_status lightkv_score(const lightkv_problem *p, const void *X, int64_t ldx, const float *x_sqnorm,
                             const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                             const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                             int32_t xi_mode, const float *lse, float softmax_scale,
                             float *xi, float *best_fd, int32_t *best_dst, float *fd_dump, int64_t fd_dump_floats,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * Edge selection (Step 2) and the index structures of the merge.
 * In window w the r_w A nodes with the lowest best_fd are merged (ties: earlier in the window first);
 * if the device-side r_w exceeds |A_w| it is clamped to |A_w|, and windows without a B node merge nothing.
 * An A node without a usable proposal (NaN scores) ranks last and, if still selected, goes to the first
 * B node of its window, so exactly min(r_w, |A_w|) tokens leave every window.
 *   dst[sumN]          token the A token is merged into, -1 for every token that stays (sets R and B)
 *   new_index[sumN]    row of a staying token in the compacted tensors (order preserved), -1 if merged
 *   grp_offsets[sumN+1], grp_src[sum r_w]   inverse of dst: the sources of token b, ascending
 *   cu_vis_out[batch+1]  vision-token offsets after the step
 */
lightkv_status lightkv_select(const lightkv_problem *p, const float *best_fd, const int32_t *best_dst,
                              int32_t *dst, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                              int32_t *cu_vis_out, void *ws, size_t ws_bytes, void *stream);

/*
 * lightkv_select for callers that cannot allocate and carry no workspace: code under HIP graph capture, serving loops
 * with a fixed memory plan, harnesses that forbid hipMalloc.  Same inputs, same outputs (bit for bit) as lightkv_select
 * with LIGHTKV_MATCH_BEST_PER_A; the two per-token scratch arrays of the selection live in a static device array of
 * the library (512 KB on every device the library has run on, held until the process ends) instead of `ws`.  The call
 * allocates and frees nothing.  At most LIGHTKV_SELECT_STATIC_MAX_TOKENS vision tokens in the batch (more ->
 * LIGHTKV_ERR_UNSUPPORTED, nothing launched).  All calls on one device share that array: calls that may overlap on a
 * device (different streams, different host threads) race and must be ordered by the caller.
 */
lightkv_status lightkv_select_static(const lightkv_problem *p, const float *best_fd, const int32_t *best_dst,
                                     int32_t *dst, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                                     int32_t *cu_vis_out, void *stream);

/*
 * lightkv_score followed by lightkv_select in one call: same arguments, same outputs (bit for bit).  When every
 * window holds at most 64 tokens, the row arg-min and the per-window selection run in one kernel (one launch less);
 * if in addition xi is computed and the step has at most LIGHTKV_ONE_STREAM_MAX_TOKENS tokens, the xi passes share the
 * launches of the FD kernels and the whole call is three launches on `stream` (no helper stream).  Otherwise the call
 * is the two calls in sequence.  X must not be NULL; xi_mode GIVEN skips the xi half as in lightkv_score.
 *
 * With p->match == LIGHTKV_MATCH_EDGE_TOPK (this call only; lightkv_select alone returns LIGHTKV_ERR_UNSUPPORTED,
 * because the selection needs the FD of every pair, which never leaves the workspace):
 *   win_remove[w] = k_w, the number of EDGES taken in window w (device values above |A_w| |B_w| are clamped).
 *                 With h_win_remove (and h_win_offsets, against which it is validated) the edge list is sized from
 *                 the host's counts, which must equal the device's.  Without h_win_remove the counts are read on
 *                 the device only -- e.g. straight from lightkv_window_counts(LIGHTKV_COUNT_EDGES), no read-back --,
 *                 the list gets one slot per token of the batch, and k_w is in addition clamped to v_w, the tokens of
 *                 the window (never binding for rho <= 2);
 *   dst[a]        the B token of a's lowest selected edge, -1 if a owns none (a stays)
 *   grp_offsets / grp_src   sources of every B token over ALL selected edges, ascending; grp_src needs sum k_w ints
 *                           (sumN ints without h_win_remove)
 *   new_index, cu_vis_out   as above; the number of staying tokens is data dependent -- a caller that needs it on the
 *                           host reads cu_vis_out back.  lightkv_aggregate_compact / lightkv_compact then write that
 *                           many rows; size their outputs for sumN - (number of windows with k_w > 0) rows or more.
 *   best_fd / best_dst      the lowest-FD edge of every A node, selected or not.
 * The scores are fp32 when they are ranked: pairs whose FD agree to fp32 rounding are ordered by position.
 */
lightkv_status lightkv_score_select(const lightkv_problem *p, const void *X, int64_t ldx, const float *x_sqnorm,
                                    const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                    const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                                    int32_t xi_mode, const float *lse, float softmax_scale,
                                    float *xi, float *best_fd, int32_t *best_dst,
                                    int32_t *dst, int32_t *new_index, int32_t *grp_offsets, int32_t *grp_src,
                                    int32_t *cu_vis_out, void *ws, size_t ws_bytes, void *stream);

/*
 * Message passing (Step 3, Eq. "message-passing"), in place: every token b that has sources becomes
 *   y_b <- (xi_b*y_b + sum_a xi_a*y_a) / (xi_b + sum_a xi_a)       for y in {X, K, V} rows,
 * evaluated as y_b + sum_a w_a*(y_a - y_b), w_a = xi_a/(xi_b + sum xi_a), in fp32 (identical rows stay
 * bit-identical), rounded to nearest-even on store.  Source (A) rows are only read; each B row has one
 * writer, so the update is race free.  Any of X, K, V may be NULL (skipped).
 */
lightkv_status lightkv_aggregate(const lightkv_problem *p, const int32_t *grp_offsets, const int32_t *grp_src,
                                 const float *xi, void *X, int64_t ldx, void *K, int64_t ldk,
                                 void *V, int64_t ldv, void *stream);

/*
 * Delete + reorder (Steps 4-5): out[new_index[i]] = in[i] for every staying token, for X, K, V and pos.
 * Outputs are dense [out_rows, d] (row stride d) and must not overlap the inputs (-> LIGHTKV_ERR_SHAPE).
 * out_rows is the capacity of the output tensors in rows (normally sumN' = sumN - sum r_w); a staying
 * token whose new_index does not fit is dropped, never written out of bounds -- compare
 * cu_vis_out[batch] from lightkv_select with out_rows to detect that.
 * NULL tensors are skipped (in and out together).
 * x_sqnorm_out[out_rows] (device, fp32, may be NULL; needs X): |x|^2 of every row written to X_out, as stored -- the
 * x_sqnorm argument of the next stage's lightkv_score; the rows pass through registers here anyway.
 * Rows behind the vision span (Step 5 and the appendix "Method overview" figure: the sequence continues with the
 * prompt's text behind the now shorter vision span): with tail_rows > 0 the inputs X, K, V, pos hold tail_rows more
 * rows directly behind their sumN vision rows (for one sequence: its text tokens; for a batch: the callers' block of
 * trailing rows), and these are copied to the outputs directly behind the vision rows that stay, input row sumN + j
 * to output row cu_vis_out[batch] + j.  cu_vis_out (device, from lightkv_select) is then required and out_rows must
 * cover the staying vision rows plus tail_rows.  tail_rows == 0: cu_vis_out may be NULL.
 */
lightkv_status lightkv_compact(const lightkv_problem *p, const int32_t *new_index,
                               const void *X, int64_t ldx, const void *K, int64_t ldk,
                               const void *V, int64_t ldv, const int32_t *pos,
                               void *X_out, void *K_out, void *V_out, int32_t *pos_out, float *x_sqnorm_out,
                               int64_t out_rows, int64_t tail_rows, const int32_t *cu_vis_out, void *stream);

/*
 * lightkv_aggregate followed by lightkv_compact in one pass over the rows: reads every input row once,
 * writes every output row once, leaves the inputs untouched.  Same results as the two calls (x_sqnorm_out, tail_rows
 * and cu_vis_out as in lightkv_compact).
 */
lightkv_status lightkv_aggregate_compact(const lightkv_problem *p, const int32_t *new_index,
                                         const int32_t *grp_offsets, const int32_t *grp_src, const float *xi,
                                         const void *X, int64_t ldx, const void *K, int64_t ldk,
                                         const void *V, int64_t ldv, const int32_t *pos,
                                         void *X_out, void *K_out, void *V_out, int32_t *pos_out,
                                         float *x_sqnorm_out, int64_t out_rows, int64_t tail_rows,
                                         const int32_t *cu_vis_out, void *stream);

/*
 * One stage of the hierarchical schedule (Sec. 3.2.2) for lightkv_compress_schedule: the stage's descriptor and every
 * buffer the stage writes.  All device buffers are the caller's; sizes as in the calls they are passed to.
 */
typedef struct lightkv_stage {
  lightkv_problem problem;   /* the stage's descriptor; win_offsets / win_tokens point to the two arrays below          */
  int32_t w;                 /* windows per axis of a tile in this stage (0: one window per sequence)                   */
  int32_t reserved;          /* must be 0                                                                               */
  int32_t *win_offsets;      /* [n_windows+1]  written by the schedule (lightkv_build_windows / _next)                  */
  int32_t *win_tokens;       /* [sumN]                                                                                  */
  float *xi;                 /* [sumN]                                                                                  */
  float *best_fd;            /* [sumN]                                                                                  */
  int32_t *best_dst, *dst, *new_index;   /* [sumN] each                                                                 */
  int32_t *grp_offsets;      /* [sumN+1]                                                                                */
  int32_t *grp_src;          /* [sum r_w]                                                                               */
  int32_t *cu_vis_out;       /* [batch+1]; must equal the next stage's problem.cu_vis contents (the caller's schedule   */
                             /* fixes every stage's token counts in advance; with cu_vis_target below the library       */
                             /* derives the per-window counts that meet them and reports in `status` if it cannot)      */
  void *X_out, *K_out, *V_out;   /* [out_rows, d] dense                                                                 */
  int32_t *pos_out;          /* [out_rows]                                                                              */
  float *x_sqnorm_out;       /* [out_rows] or NULL: squared norms of X_out, handed to the next stage's scores          */
  int64_t out_rows;
  /* Counts from the stage's token budget (NULL: problem.win_remove is the caller's and is used as it is).  When given,  */
  /* the schedule calls lightkv_window_counts(LIGHTKV_COUNT_TARGET) on the windows it has just built and writes          */
  /* win_remove, which must be the array problem.win_remove points to.                                                   */
  const int32_t *cu_vis_target;   /* device [batch+1]: sequence offsets this stage must leave (= its cu_vis_out)       */
  int32_t *win_remove;            /* device [n_windows], written by the schedule                                       */
  int32_t *status;                /* device [batch] or NULL: 1 where the budget of a sequence could not be met         */
} lightkv_stage;

/*
 * The whole schedule in one call (Sec. 3.2.2: several compression stages at chosen layers, each with its own window
 * size; here the stages run back to back on the same K/V/Q, every stage consuming what the one before wrote):
 *   stage 0 reads X, K, V, pos; stage s > 0 reads stage s-1's X_out, K_out, V_out, pos_out (row stride d).
 *   Q[sumT, heads, head_dim] (prompt queries, TEXT_QUERY) is the same for all stages; xi of stage s is computed
 *   against the K rows that stage merges.  softmax_scale as in lightkv_score.
 * Per stage the call enqueues what the single calls would -- lightkv_build_windows (stage 0; later stages' windows are
 * built by lightkv_build_windows_next next to the previous stage's merge), lightkv_score (xi) next to
 * lightkv_score_select (FD + selection), lightkv_aggregate_compact -- with the same results, bit for bit.  xi and the
 * next stage's windows run on two internal helper streams that fork from and join `stream` (created per device on the
 * first call outside stream capture, default priority, kept for the life of the process; if they cannot be made, or
 * the first call on a device comes under capture, everything is enqueued on `stream` in order).  Steps of at most
 * LIGHTKV_ONE_STREAM_MAX_TOKENS tokens whose windows hold at most 64 tokens use the one-stream form of
 * lightkv_score_select instead.  One workspace serves all stages: ws_bytes must cover lightkv_workspace_size of every
 * stage.  Host threads calling this on one device take turns enqueueing.  Only LIGHTKV_MATCH_BEST_PER_A (fixed token
 * counts) is supported here; lightkv_compress_schedule_ratio below takes the others.
 * Errors: the first failing call's status; stages before it have been enqueued.
 */
lightkv_status lightkv_compress_schedule(const lightkv_stage *stages, int32_t n_stages,
                                         int32_t tiles, int32_t grid_h, int32_t grid_w,
                                         const void *X, int64_t ldx, const void *K, int64_t ldk,
                                         const void *V, int64_t ldv, const int32_t *pos,
                                         const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                         float softmax_scale, void *ws, size_t ws_bytes, void *stream);

/*
 * The schedule when the token count a stage leaves depends on the data: LIGHTKV_MATCH_EDGE_TOPK (Step 2 of Sec. 3.2.1
 * read literally: the k lowest edges of a window), LIGHTKV_MATCH_FULL_PAIRWISE (appendix "Bipartite vs. full pairwise
 * matching"), or LIGHTKV_MATCH_BEST_PER_A driven by the ratio of Sec. 3.2.2 instead of fixed budgets.  rho[n_stages]
 * (host) is the ratio of every stage; the per-window counts are computed on the device from the windows as they are
 * (lightkv_window_counts: LIGHTKV_COUNT_EDGES for EDGE_TOPK, LIGHTKV_COUNT_RATIO otherwise) and consumed there.
 * Per stage the call enqueues lightkv_build_windows + lightkv_window_counts (stage 0; later stages' windows and counts
 * are built by lightkv_build_windows_next next to the previous stage's merge, on a helper stream as in
 * lightkv_compress_schedule), lightkv_score_select (xi from Q and the stage's K rows, TEXT_QUERY) and
 * lightkv_aggregate_compact -- with the same results as those calls, bit for bit -- then copies the stage's cu_vis_out
 * to h_cu_vis_out[s * (batch+1) ...] (host, [n_stages * (batch+1)], out) and WAITS for `stream`: the next stage's launch
 * plans need those offsets.  One synchronisation per stage; the call cannot be captured into a graph (a capturing
 * stream -> LIGHTKV_ERR_UNSUPPORTED, nothing enqueued).  When it returns LIGHTKV_OK every stage has finished.
 * Of the descriptors: stages[0].problem carries the input's h_cu_vis / cu_vis; for s > 0 those two fields are ignored
 * (the library uses what stage s-1 left).  problem.max_window_tokens is required for every stage (a bound from the cell
 * geometry, lightkv_max_window_cells, holds whatever the earlier stages removed); h_win_offsets, h_win_remove and
 * cu_vis_target must be NULL; win_remove is required and must be the array problem.win_remove points to; status is not
 * used.  Every per-token array of a stage must hold the tokens of stage 0's input (no stage has more), grp_src as
 * lightkv_score_select states, out_rows at least the rows the stage leaves (checked after the stage ->
 * LIGHTKV_ERR_SHAPE).  ws_bytes should cover lightkv_workspace_size of every stage's descriptor laid over stage 0's
 * offsets; each stage's real need is checked when it is reached (-> LIGHTKV_ERR_WORKSPACE).
 * Errors: the first failing call's status; stages before it have run.
 */
lightkv_status lightkv_compress_schedule_ratio(const lightkv_stage *stages, int32_t n_stages, const double *rho,
                                               int32_t tiles, int32_t grid_h, int32_t grid_w,
                                               const void *X, int64_t ldx, const void *K, int64_t ldk,
                                               const void *V, int64_t ldv, const int32_t *pos,
                                               const void *Q, int64_t q_tok_stride, int64_t q_head_stride,
                                               float softmax_scale, void *ws, size_t ws_bytes,
                                               int32_t *h_cu_vis_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LIGHTKV_H */
