// Edge selection (paper Sec. 3.2.1 Step 2) and the index structures of the merge.
//
// In every window the r A nodes with the lowest best-edge FD are merged into their B node; the order
// is fixed by the 64-bit key (order-preserving bits of FD, local position), so equal FDs go to the
// earlier token.  Selection is an LDS bitonic sort of the window's keys by one workgroup; a second
// sort of (destination, source) pairs yields each source's rank inside its group, which makes the
// inverse map (grp_offsets / grp_src) deterministic without atomics on the output.
//
//   select_window_kernel : per window -> dst[], per-token source counts, per-source ranks
//   select_scan_kernel   : one workgroup -> exclusive scans (new_index, grp_offsets), cu_vis_out, grp_src
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {

struct SelArgs {
  int n_windows, batch, sum_n;
  const int32_t *cu_vis, *win_offsets, *win_tokens, *win_remove;
  const float *best_fd;
  const int32_t *best_dst;
  int32_t *dst, *new_index, *grp_offsets, *grp_src, *cu_vis_out, *cnt, *src_rank;
  int cap;   // power of two >= the largest |A|
};

template <int THREADS>
__global__ __launch_bounds__(THREADS) void select_window_kernel(SelArgs g) {
  extern __shared__ uint64_t keys[];          // cap entries
  int *start = reinterpret_cast<int *>(keys + g.cap);   // cap entries: scan buffer
  const int w = blockIdx.x;
  const int off = g.win_offsets[w];
  const int v = g.win_offsets[w + 1] - off;
  int nA = (v + 1) >> 1;
  const int nB = v >> 1;
  if (nA > g.cap) nA = g.cap;                 // window larger than the caller's bound: surplus rows stay
  int r = g.win_remove[w];
  r = r < 0 ? 0 : (r > nA ? nA : r);
  if (nB == 0) r = 0;

  // every token of the window starts as "stays, no sources"
  for (int t = threadIdx.x; t < v; t += THREADS) {
    const int tok = g.win_tokens[off + t];
    if ((unsigned)tok < (unsigned)g.sum_n) {
      g.dst[tok] = -1;
      g.cnt[tok] = 0;
      g.src_rank[tok] = 0;
    }
  }
  if (r == 0) return;

  const int p2 = next_pow2(nA);
  for (int la = threadIdx.x; la < p2; la += THREADS) {
    uint64_t key = ~0ull;
    if (la < nA) {
      const int tok = g.win_tokens[off + 2 * la];
      float fd = __uint_as_float(0x7f800000u);
      if ((unsigned)tok < (unsigned)g.sum_n) fd = g.best_fd[tok];
      if (!(fd >= 0.f)) fd = __uint_as_float(0x7f800000u);   // NaN or negative never wins
      key = ((uint64_t)f32_order_key(fd) << 32) | (uint32_t)la;
    }
    keys[la] = key;
  }
  bitonic_sort_lds(keys, p2);

  // the first r keys are the merged A nodes; rebuild keys as (destination token, source token)
  uint64_t pair[(2048 + THREADS - 1) / THREADS];
  int np = 0;
  for (int k = threadIdx.x; k < p2; k += THREADS, ++np) {
    uint64_t pk = ~0ull;
    if (k < r) {
      const int la = (int)(keys[k] & 0xffffffffu);
      const int a_tok = g.win_tokens[off + 2 * la];
      int b_tok = -1;
      if ((unsigned)a_tok < (unsigned)g.sum_n) b_tok = g.best_dst[a_tok];
      if ((unsigned)b_tok >= (unsigned)g.sum_n) b_tok = g.win_tokens[off + 1];   // no usable proposal: first B node
      if ((unsigned)b_tok < (unsigned)g.sum_n && (unsigned)a_tok < (unsigned)g.sum_n)
        pk = ((uint64_t)(uint32_t)b_tok << 32) | (uint32_t)a_tok;
    }
    pair[np] = pk;
  }
  __syncthreads();
  np = 0;
  for (int k = threadIdx.x; k < p2; k += THREADS, ++np) keys[k] = pair[np];
  const int p2r = next_pow2(r);
  bitonic_sort_lds(keys, p2r <= p2 ? p2r : p2);   // entries >= r are all ~0 and already in place

  // group starts: inclusive max-scan of (k where the destination changes)
  for (int k = threadIdx.x; k < p2r; k += THREADS) {
    const bool head = (k == 0) || ((keys[k] >> 32) != (keys[k - 1] >> 32));
    start[k] = head ? k : 0;
  }
  __syncthreads();
  for (int step = 1; step < p2r; step <<= 1) {
    int val[(2048 + THREADS - 1) / THREADS];
    int n = 0;
    for (int k = threadIdx.x; k < p2r; k += THREADS, ++n) val[n] = (k >= step) ? max(start[k], start[k - step]) : start[k];
    __syncthreads();
    n = 0;
    for (int k = threadIdx.x; k < p2r; k += THREADS, ++n) start[k] = val[n];
    __syncthreads();
  }
  for (int k = threadIdx.x; k < r; k += THREADS) {
    const uint64_t pk = keys[k];
    if (pk == ~0ull) continue;               // an A node without a valid proposal stays
    const int b_tok = (int)(pk >> 32), a_tok = (int)(pk & 0xffffffffu);
    g.dst[a_tok] = b_tok;
    g.src_rank[a_tok] = k - start[k];
    const bool last = (k == r - 1) || ((keys[k + 1] >> 32) != (pk >> 32));
    if (last) g.cnt[b_tok] = k - start[k] + 1;
  }
}

// Single workgroup: scans over all tokens of the batch.  Every thread owns a run of consecutive tokens, so one
// pass needs a single workgroup scan (two values at once) instead of one per 1024 tokens; all loads of a pass are
// issued together.
constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_ITEMS = 12;     // tokens per thread and pass (12288 tokens per pass)
constexpr int FILL_UNROLL = 4;

__global__ __launch_bounds__(SCAN_THREADS) void select_scan_kernel(SelArgs g) {
  __shared__ int kb[SCAN_THREADS * SCAN_ITEMS];   // staying tokens before each token of the pass
  __shared__ int2 wsum[SCAN_THREADS / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s_first = g.cu_vis[tid <= g.batch ? tid : g.batch];   // sequence start handled by this thread (first round)
  int per = (g.sum_n + SCAN_THREADS - 1) / SCAN_THREADS;
  per = per < 1 ? 1 : (per > SCAN_ITEMS ? SCAN_ITEMS : per);
  const int pass_tokens = per * SCAN_THREADS;
  int keep_base = 0, cnt_base = 0;
  for (int pass_base = 0; pass_base < g.sum_n; pass_base += pass_tokens) {
    const int i0 = pass_base + tid * per;
    int d[SCAN_ITEMS], c[SCAN_ITEMS];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
      const bool ok = k < per && i0 + k < g.sum_n;
      const int ic = ok ? i0 + k : 0;            // unconditional loads from a clamped index
      const int dv = g.dst[ic], cv = g.cnt[ic];
      d[k] = ok ? dv : 0;
      c[k] = ok ? cv : 0;
    }
    int ks = 0, cs = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
      const bool ok = k < per && i0 + k < g.sum_n;
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
      const bool ok = k < per && i0 + k < g.sum_n;
      if (ok) {
        const int keep = d[k] < 0 ? 1 : 0;
        kb[tid * per + k] = ek;
        g.new_index[i0 + k] = keep ? ek : -1;
        g.grp_offsets[i0 + k] = ec;
        ek += keep;
        ec += c[k];
      }
    }
    __syncthreads();
    // vision offsets after the step: staying tokens before each sequence start that falls into this pass
    const int pass_end = min(pass_base + pass_tokens, g.sum_n);
    for (int b = tid; b <= g.batch; b += SCAN_THREADS) {
      const int s = (b == tid) ? s_first : g.cu_vis[b];
      if (s >= pass_base && s < pass_end) g.cu_vis_out[b] = kb[s - pass_base];
    }
    keep_base += tot_k;
    cnt_base += tot_c;
    __syncthreads();
  }
  for (int b = tid; b <= g.batch; b += SCAN_THREADS) {
    const int s = (b == tid) ? s_first : g.cu_vis[b];
    if (s >= g.sum_n) g.cu_vis_out[b] = keep_base;
  }
  if (tid == 0) g.grp_offsets[g.sum_n] = cnt_base;
  __syncthreads();   // grp_offsets written by this workgroup are visible to it below
  for (int a0 = 0; a0 < g.sum_n; a0 += FILL_UNROLL * SCAN_THREADS) {
    int b[FILL_UNROLL], sr[FILL_UNROLL], go[FILL_UNROLL];
#pragma unroll
    for (int j = 0; j < FILL_UNROLL; ++j) {
      const int a = a0 + j * SCAN_THREADS + tid;
      const int ac = a < g.sum_n ? a : 0;
      const int bv = g.dst[ac], sv = g.src_rank[ac];
      b[j] = a < g.sum_n ? bv : -1;
      sr[j] = sv;
    }
#pragma unroll
    for (int j = 0; j < FILL_UNROLL; ++j) go[j] = g.grp_offsets[b[j] >= 0 ? b[j] : 0];
#pragma unroll
    for (int j = 0; j < FILL_UNROLL; ++j)
      if (b[j] >= 0) g.grp_src[go[j] + sr[j]] = a0 + j * SCAN_THREADS + tid;
  }
}

hipError_t launch_select_scan(int batch, int sum_n, const int32_t *cu_vis, const int32_t *dst, int32_t *new_index,
                              int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out, const int32_t *cnt,
                              const int32_t *src_rank, hipStream_t stream) {
  SelArgs g{};
  g.batch = batch; g.sum_n = sum_n; g.cu_vis = cu_vis;
  g.dst = const_cast<int32_t *>(dst); g.new_index = new_index; g.grp_offsets = grp_offsets; g.grp_src = grp_src;
  g.cu_vis_out = cu_vis_out; g.cnt = const_cast<int32_t *>(cnt); g.src_rank = const_cast<int32_t *>(src_rank);
  hipLaunchKernelGGL(select_scan_kernel, dim3(1), dim3(SCAN_THREADS), 0, stream, g);
  return hipGetLastError();
}

hipError_t launch_select(int n_windows, int max_window_tokens, int batch, int sum_n, const int32_t *cu_vis,
                         const int32_t *win_offsets, const int32_t *win_tokens, const int32_t *win_remove,
                         const float *best_fd, const int32_t *best_dst, int32_t *dst, int32_t *new_index,
                         int32_t *grp_offsets, int32_t *grp_src, int32_t *cu_vis_out, int32_t *cnt,
                         int32_t *src_rank, hipStream_t stream) {
  SelArgs g{};
  g.n_windows = n_windows; g.batch = batch; g.sum_n = sum_n;
  g.cu_vis = cu_vis; g.win_offsets = win_offsets; g.win_tokens = win_tokens; g.win_remove = win_remove;
  g.best_fd = best_fd; g.best_dst = best_dst;
  g.dst = dst; g.new_index = new_index; g.grp_offsets = grp_offsets; g.grp_src = grp_src;
  g.cu_vis_out = cu_vis_out; g.cnt = cnt; g.src_rank = src_rank;
  const int maxA = (max_window_tokens + 1) / 2;
  g.cap = next_pow2(maxA > 1 ? maxA : 1);
  const size_t lds = (size_t)g.cap * (sizeof(uint64_t) + sizeof(int));
  if (n_windows > 0) {
    if (g.cap <= 256) hipLaunchKernelGGL(select_window_kernel<256>, dim3(n_windows), dim3(256), lds, stream, g);
    else hipLaunchKernelGGL(select_window_kernel<1024>, dim3(n_windows), dim3(1024), lds, stream, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(select_scan_kernel, dim3(1), dim3(SCAN_THREADS), 0, stream, g);
  return hipGetLastError();
}

}  // namespace lk
