// Window partition of the vision tokens (paper Sec. 3.2 and Sec. 3.2.2 "Window partitioning"):
// every token is assigned to a window by its cell in the original image grid, and the tokens of
// each window are listed in ascending sequence order (CSR).  One workgroup per sequence.
//
// Fast path (count table fits LDS): a stable multi-bin partition.  Every wave-sized run of 64
// consecutive tokens counts its tokens per window with ballots; a prefix over the runs and a scan
// over the windows give each token its slot directly -- no sort, no atomics, order preserved.
// Fallback: LDS bitonic sort of (window id, local index) keys.
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {

constexpr int WIN_THREADS = 1024;
constexpr int LOCAL_BITS = 14;             // local token index < 16384
constexpr size_t WIN_TABLE_LDS_MAX = 56 * 1024;   // bytes of LDS the (run, window) count table may take
constexpr int WIN_KEEP = 4;                // passes of 1024 tokens whose window and rank stay in registers between phases
constexpr int WIN_RUN_PARTS = 4;           // threads sharing a window's prefix over the runs (up to 256 windows per sequence)

struct WinArgs {
  const int32_t *cu_vis, *pos;
  // "next stage" form: the tokens are those of the PREVIOUS stage (cu_vis, pos); a token takes part if
  // new_index[i] >= 0 and is listed under that index; cu_out holds the sequence offsets after compaction.
  // Both NULL: the plain form (every token takes part under its own index).
  const int32_t *new_index, *cu_out;
  int batch, tiles, grid_h, grid_w, w, win_per_seq;
  int32_t *win_offsets, *win_tokens;
  // optional (table kernel only): the per-window counts of the sequences' token budgets in the same launch -- the
  // window sizes are in LDS at the end of the kernel anyway.  cu_target NULL: no counts.
  const int32_t *cu_target;   // [batch + 1] offsets of the sequences after the step the windows are built for
  int32_t *win_remove, *status;
  int dir;
};

// index under which token i is listed, or -1 if it does not take part
__device__ __forceinline__ int listed_as(const WinArgs &g, int i) { return g.new_index ? g.new_index[i] : i; }

__device__ __forceinline__ int window_of(const WinArgs &g, int p) {
  if (g.w == 0) return 0;
  const int cells = g.grid_h * g.grid_w;
  p = p < 0 ? 0 : p;
  int tile = p / cells;
  const int cell = p - tile * cells;
  tile = tile >= g.tiles ? g.tiles - 1 : tile;
  int row = cell / g.grid_w;
  const int col = cell - row * g.grid_w;
  row = row >= g.grid_h ? g.grid_h - 1 : row;
  return tile * g.w * g.w + (row * g.w / g.grid_h) * g.w + (col * g.w / g.grid_w);
}

// rank of this lane among the lanes of its wave that share its window id, and the size of that group
__device__ __forceinline__ void wave_bin_rank(int wid, bool valid, int lane, int &rank, int &group_size, bool &is_leader) {
  unsigned long long remaining = __ballot(valid);
  rank = 0; group_size = 0; is_leader = false;
  while (remaining) {
    const int leader = __ffsll((long long)remaining) - 1;
    const int lw = __shfl(wid, leader, 64);
    const unsigned long long m = __ballot(valid && wid == lw);
    if (valid && wid == lw) {
      rank = __popcll(m & ((1ull << lane) - 1ull));
      group_size = __popcll(m);
      is_leader = (lane == leader);
    }
    remaining &= ~m;
  }
}

// ---- the token budget of a sequence spread over its windows (Sec. 3.2.2: the ratios P given as target lengths) ----
// With cap_w the most a window can give and q the largest level for which sum_w min(cap_w, q) stays within the budget,
// window w gives min(cap_w, q), and the first windows (in order) that can give more than q give one more until the
// budget is met.  A budget that cannot be met (negative, or above sum_w cap_w): every window gives its cap (nothing for
// a negative budget) and the status word is set.  Integer work; run by all NT threads of a workgroup.
// red, wave_tot: NT / 64 ints of LDS each.
template <int NT>
__device__ __forceinline__ int block_sum(int v, int *red) {
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();                              // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) t += red[i];
  return t;
}

template <int NT, typename CapFn>
__device__ __forceinline__ void counts_target_body(int W, int budget, CapFn cap_of, int32_t *win_remove, int32_t *status,
                                                   int *red, int *wave_tot) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int total = 0, maxcap = 0;
  for (int w = tid; w < W; w += NT) { const int c = cap_of(w); total += c; maxcap = c > maxcap ? c : maxcap; }
  total = block_sum<NT>(total, red);
  for (int o = 32; o >= 1; o >>= 1) { const int t = __shfl_xor(maxcap, o, 64); maxcap = t > maxcap ? t : maxcap; }
  __syncthreads();
  if (lane == 0) red[wave] = maxcap;
  __syncthreads();
  maxcap = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) maxcap = red[i] > maxcap ? red[i] : maxcap;
  const bool infeasible = budget < 0 || budget > total;
  if (status && tid == 0) *status = infeasible ? 1 : 0;
  if (infeasible) {   // more than every set A holds: all of them go; a negative budget: nothing goes
    for (int w = tid; w < W; w += NT) win_remove[w] = budget < 0 ? 0 : cap_of(w);
    return;
  }
  // largest level q in [0, maxcap + 1] with sum_w min(cap_w, q) <= budget
  int lo = 0, hi = maxcap + 1;
  while (lo < hi) {   // uniform
    const int mid = (lo + hi + 1) >> 1;
    int f = 0;
    for (int w = tid; w < W; w += NT) { const int c = cap_of(w); f += c < mid ? c : mid; }
    f = block_sum<NT>(f, red);
    if (f <= budget) lo = mid; else hi = mid - 1;
  }
  const int q = lo;
  int given = 0;
  for (int w = tid; w < W; w += NT) { const int c = cap_of(w); given += c < q ? c : q; }
  given = block_sum<NT>(given, red);
  const int missing = budget - given;
  // one more from the first `missing` windows (in order) whose cap exceeds q
  int carry = 0;
  for (int wb = 0; wb < W; wb += NT) {   // uniform
    const int w = wb + tid;
    const int c = w < W ? cap_of(w) : 0;
    const int more = (w < W && c > q) ? 1 : 0;
    int inc = more;
    for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(inc, o, 64); if (lane >= o) inc += t; }
    __syncthreads();
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int before = carry, all = 0;
#pragma unroll
    for (int k = 0; k < NT / 64; ++k) { before += (k < wave) ? wave_tot[k] : 0; all += wave_tot[k]; }
    const int excl = before + inc - more;
    if (w < W) win_remove[w] = (c < q ? c : q) + ((more && excl < missing) ? 1 : 0);
    carry += all;
  }
}

__global__ __launch_bounds__(WIN_THREADS) void build_windows_table_kernel(WinArgs g) {
  extern __shared__ uint16_t table[];   // [runs][win_per_seq] counts, then exclusive prefixes over the runs
  __shared__ int scan_lds[64];
  __shared__ int part_sum[WIN_RUN_PARTS][WIN_THREADS / WIN_RUN_PARTS];
  const int b = blockIdx.x;
  const int base = g.cu_vis[b];
  const int n = g.cu_vis[b + 1] - base;
  const int out_base = g.cu_out ? g.cu_out[b] : base;                 // first listed index of the sequence
  const int out_n = g.cu_out ? g.cu_out[b + 1] - out_base : n;        // tokens that take part
  const int wps = g.win_per_seq;
  const int wbase = b * wps;
  const int runs = (n + 63) >> 6;
  int *winbase = reinterpret_cast<int *>(table + (size_t)runs * wps + ((runs * wps) & 1));   // [wps] after the table
  const int lane = threadIdx.x & 63;

  for (int e = threadIdx.x; e < runs * wps; e += WIN_THREADS) table[e] = 0;
  __syncthreads();
  // phase 1: per-run counts.  The first WIN_KEEP passes keep (listed index, window, rank inside the run's group) in
  // registers for phase 3; longer sequences recompute them there.
  int k_id[WIN_KEEP], k_wid[WIN_KEEP], k_rank[WIN_KEEP];
#pragma unroll
  for (int p = 0; p < WIN_KEEP; ++p) {
    k_id[p] = -1; k_wid[p] = 0; k_rank[p] = 0;
    const int i = p * WIN_THREADS + (int)threadIdx.x;
    if (p * WIN_THREADS < n) {   // uniform
      const int id = i < n ? listed_as(g, base + i) : -1;
      const bool valid = id >= 0;
      const int wid = valid ? window_of(g, g.pos[base + i]) : -1;
      int rank, gs; bool leader;
      wave_bin_rank(wid, valid, lane, rank, gs, leader);
      if (leader) table[(i >> 6) * wps + wid] = (uint16_t)gs;
      k_id[p] = id; k_wid[p] = wid; k_rank[p] = rank;
    }
  }
  for (int i0 = WIN_KEEP * WIN_THREADS; i0 < n; i0 += WIN_THREADS) {
    const int i = i0 + threadIdx.x;
    const bool valid = i < n && listed_as(g, base + (i < n ? i : 0)) >= 0;
    const int wid = valid ? window_of(g, g.pos[base + i]) : -1;
    int rank, gs; bool leader;
    wave_bin_rank(wid, valid, lane, rank, gs, leader);
    if (leader) table[(i >> 6) * wps + wid] = (uint16_t)gs;
  }
  __syncthreads();
  // phase 2: exclusive prefix over the runs for every window, then a scan over the windows
  int carry = 0;
  const bool split_runs = wps <= WIN_THREADS / WIN_RUN_PARTS;   // uniform: WIN_RUN_PARTS threads share a window's runs
  for (int w0 = 0; w0 < wps; w0 += WIN_THREADS) {
    const int w = split_runs ? (int)threadIdx.x % (WIN_THREADS / WIN_RUN_PARTS) : w0 + (int)threadIdx.x;
    int total = 0;
    if (split_runs) {
      // the runs of a window in WIN_RUN_PARTS contiguous parts: part sums, then every part rewrites its own counts
      // as prefixes -- a quarter of the dependent LDS steps of one thread per window
      const int part = (int)threadIdx.x / (WIN_THREADS / WIN_RUN_PARTS);
      const int per_part = (runs + WIN_RUN_PARTS - 1) / WIN_RUN_PARTS;
      const int r_begin = min(part * per_part, runs), r_end = min(r_begin + per_part, runs);
      int mine = 0;
      if (w < wps)
        for (int r = r_begin; r < r_end; ++r) mine += table[r * wps + w];
      part_sum[part][w & (WIN_THREADS / WIN_RUN_PARTS - 1)] = mine;
      __syncthreads();
      int before = 0;
#pragma unroll
      for (int q = 0; q < WIN_RUN_PARTS; ++q) {
        const int v = part_sum[q][w & (WIN_THREADS / WIN_RUN_PARTS - 1)];
        before += (q < part) ? v : 0;
        total += v;
      }
      if (w < wps) {
        int running = before;
        for (int r = r_begin; r < r_end; ++r) {
          const int c = table[r * wps + w];
          table[r * wps + w] = (uint16_t)running;
          running += c;
        }
      }
      total = (part == 0 && w < wps) ? total : 0;   // one thread per window enters the scan over the windows
    } else if (w < wps) {
      for (int r = 0; r < runs; ++r) {
        const int c = table[r * wps + w];
        table[r * wps + w] = (uint16_t)total;
        total += c;
      }
    }
    // block exclusive scan of `total`
    const int wave = threadIdx.x >> 6;
    int inc = total;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) scan_lds[wave] = inc;
    __syncthreads();
    if (wave == 0) {
      int ws = (lane < WIN_THREADS / 64) ? scan_lds[lane] : 0;
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) {
        const int t = __shfl_up(ws, o, 64);
        if (lane >= o) ws += t;
      }
      if (lane < WIN_THREADS / 64) scan_lds[32 + lane] = ws;
    }
    __syncthreads();
    const int excl = carry + (wave ? scan_lds[32 + wave - 1] : 0) + inc - total;
    if (w < wps && (!split_runs || (int)threadIdx.x < WIN_THREADS / WIN_RUN_PARTS)) {
      winbase[w] = excl;
      g.win_offsets[wbase + w] = out_base + excl;
    }
    carry += scan_lds[32 + WIN_THREADS / 64 - 1];
    __syncthreads();
  }
  if (threadIdx.x == 0 && b == g.batch - 1) g.win_offsets[wbase + wps] = out_base + out_n;
  // phase 3: slots
#pragma unroll
  for (int p = 0; p < WIN_KEEP; ++p) {
    const int i = p * WIN_THREADS + (int)threadIdx.x;
    if (k_id[p] >= 0)
      g.win_tokens[out_base + winbase[k_wid[p]] + table[(i >> 6) * wps + k_wid[p]] + k_rank[p]] = k_id[p];
  }
  for (int i0 = WIN_KEEP * WIN_THREADS; i0 < n; i0 += WIN_THREADS) {
    const int i = i0 + threadIdx.x;
    const int id = i < n ? listed_as(g, base + i) : -1;
    const bool valid = id >= 0;
    const int wid = valid ? window_of(g, g.pos[base + i]) : -1;
    int rank, gs; bool leader;
    wave_bin_rank(wid, valid, lane, rank, gs, leader);
    if (valid) g.win_tokens[out_base + winbase[wid] + table[(i >> 6) * wps + wid] + rank] = id;
  }
  if (g.cu_target) {
    // the sizes of this sequence's windows are the differences of winbase[] (LDS; the end of the last window is out_n)
    auto cap_of = [&](int w) {
      const int v = (w + 1 < wps ? winbase[w + 1] : out_n) - winbase[w];
      const int c = v >= 2 ? side_a(v, g.dir) : 0;   // the proposing side; a single token has nobody to merge into
      return c < 65535 ? c : 65535;
    };
    const int budget = out_n - (g.cu_target[b + 1] - g.cu_target[b]);
    counts_target_body<WIN_THREADS>(wps, budget, cap_of, g.win_remove + wbase, g.status ? g.status + b : nullptr, scan_lds,
                                    scan_lds + 32);
  }
}

__global__ __launch_bounds__(WIN_THREADS) void build_windows_sort_kernel(WinArgs g) {
  extern __shared__ uint32_t keys[];
  const int b = blockIdx.x;
  const int base = g.cu_vis[b];
  const int n_all = g.cu_vis[b + 1] - base;                            // tokens looked at
  const int out_base = g.cu_out ? g.cu_out[b] : base;
  const int n = g.cu_out ? g.cu_out[b + 1] - out_base : n_all;         // tokens that take part: they sort to the front
  const int wbase = b * g.win_per_seq;
  const int p2 = next_pow2(n_all > 1 ? n_all : 1);
  for (int i = threadIdx.x; i < p2; i += blockDim.x) {
    const bool in = i < n_all && listed_as(g, base + (i < n_all ? i : 0)) >= 0;
    keys[i] = in ? (((uint32_t)window_of(g, g.pos[base + i]) << LOCAL_BITS) | (uint32_t)i) : 0xffffffffu;
  }
  bitonic_sort_lds(keys, p2);
  // sorted position k holds the k-th token of the window-major order
  for (int k = threadIdx.x; k <= n; k += blockDim.x) {
    const int prev = (k == 0) ? -1 : (int)(keys[k - 1] >> LOCAL_BITS);
    int cur;
    if (k < n) {
      cur = (int)(keys[k] >> LOCAL_BITS);
      g.win_tokens[out_base + k] = listed_as(g, base + (int)(keys[k] & ((1u << LOCAL_BITS) - 1u)));
    } else {
      cur = (b == g.batch - 1) ? g.win_per_seq : g.win_per_seq - 1;   // the next sequence writes its own first offset
    }
    for (int id = prev + 1; id <= cur; ++id) g.win_offsets[wbase + id] = out_base + k;
  }
}

// ---- per-window counts (Sec. 3.2.1 Step 2, Sec. 3.2.2: the ratios P of the schedule) -----------------------------
// One workgroup per sequence.  mode 0: r_w = min(floor(rho v_w), ceil(v_w / 2)) tokens; mode 1: k_w = min(floor(rho v_w / 2),
// |A_w| |B_w|) edges; mode 2: the sequence has to go from its current length to a target length, and the difference
// is spread over its windows as evenly as their sizes allow (no window gives more than its set A): with q the largest
// level for which sum_w min(cap_w, q) stays within the budget, window w gives min(cap_w, q), and the first windows
// that can give more than q give one more until the budget is met.  Integer work throughout; rho is a double so that
// the floor is taken in the precision a host program would use.
constexpr int CNT_THREADS = 256;
constexpr int CNT_CACHE = 8192;   // window caps kept in LDS (16 KB)

struct CountArgs {
  const int32_t *win_offsets, *cu_vis, *cu_target;
  int32_t *win_remove, *status;
  int win_per_seq, mode, dir;
  double rho;
};

__global__ __launch_bounds__(CNT_THREADS) void window_counts_kernel(CountArgs g) {
  __shared__ int red[4];
  __shared__ int wave_tot[4];
  const int b = blockIdx.x, W = g.win_per_seq, w0 = b * W;
  const int tid = threadIdx.x;
  if (g.mode != 2) {
    for (int w = tid; w < W; w += CNT_THREADS) {
      const long long v = g.win_offsets[w0 + w + 1] - g.win_offsets[w0 + w];
      long long r, cap;
      if (g.mode == 0) { r = (long long)floor(g.rho * (double)v + 1e-9); cap = side_a((int)v, g.dir); }
      else             { r = (long long)floor(g.rho * (double)v / 2.0 + 1e-9); cap = ((v + 1) / 2) * (v / 2); }
      r = r < 0 ? 0 : (r > cap ? cap : r);
      g.win_remove[w0 + w] = (int)r;
    }
    if (g.status && tid == 0) g.status[b] = 0;
    return;
  }
  const int budget = (g.cu_vis[b + 1] - g.cu_vis[b]) - (g.cu_target[b + 1] - g.cu_target[b]);
  // the caps are looked at a dozen times: the first CNT_CACHE of them are kept in LDS (one trip to memory instead of
  // one per pass, which is what this small kernel's time consists of); longer lists re-read the rest
  __shared__ uint16_t cap_lds[CNT_CACHE];
  auto cap_mem = [&](int w) {
    const int v = g.win_offsets[w0 + w + 1] - g.win_offsets[w0 + w];
    const int c = v >= 2 ? side_a(v, g.dir) : 0;   // the proposing side; a single token has nobody to merge into
    return c < 65535 ? c : 65535;
  };
  for (int w = tid; w < W && w < CNT_CACHE; w += CNT_THREADS) cap_lds[w] = (uint16_t)cap_mem(w);
  __syncthreads();
  auto cap_of = [&](int w) { return w < CNT_CACHE ? (int)cap_lds[w] : cap_mem(w); };
  counts_target_body<CNT_THREADS>(W, budget, cap_of, g.win_remove + w0, g.status ? g.status + b : nullptr, red, wave_tot);
}

hipError_t launch_window_counts(int batch, int win_per_seq, const int32_t *win_offsets, int mode, int dir, double rho,
                                const int32_t *cu_vis, const int32_t *cu_target, int32_t *win_remove, int32_t *status,
                                hipStream_t stream) {
  CountArgs g{};
  g.win_offsets = win_offsets; g.cu_vis = cu_vis; g.cu_target = cu_target; g.win_remove = win_remove; g.status = status;
  g.win_per_seq = win_per_seq; g.mode = mode; g.dir = dir; g.rho = rho;
  hipLaunchKernelGGL(window_counts_kernel, dim3(batch), dim3(CNT_THREADS), 0, stream, g);
  return hipGetLastError();
}

hipError_t launch_build_windows(const int32_t *cu_vis, const int32_t *pos, const int32_t *new_index,
                                const int32_t *cu_out, int batch, int max_seq, int tiles,
                                int grid_h, int grid_w, int w, int32_t *win_offsets, int32_t *win_tokens,
                                const int32_t *cu_target, int32_t *win_remove, int32_t *status, int dir, bool *counts_done,
                                hipStream_t stream) {
  if (counts_done) *counts_done = false;
  WinArgs g{};
  g.cu_vis = cu_vis; g.pos = pos; g.new_index = new_index; g.cu_out = cu_out; g.batch = batch; g.tiles = tiles; g.grid_h = grid_h; g.grid_w = grid_w; g.w = w;
  g.win_per_seq = (w == 0) ? 1 : tiles * w * w;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens;
  const int runs = (max_seq + 63) / 64;
  const int64_t entries = (int64_t)runs * g.win_per_seq;
  const size_t lds = (size_t)(entries + (entries & 1)) * sizeof(uint16_t) + (size_t)g.win_per_seq * sizeof(int);
  if (lds <= WIN_TABLE_LDS_MAX) {
    if (cu_target && win_remove && counts_done) {   // the counts ride along (the sort fallback leaves them to the caller)
      g.cu_target = cu_target; g.win_remove = win_remove; g.status = status; g.dir = dir;
      *counts_done = true;
    }
    hipLaunchKernelGGL(build_windows_table_kernel, dim3(batch), dim3(WIN_THREADS), lds, stream, g);
  } else {
    const int p2 = next_pow2(max_seq > 1 ? max_seq : 1);
    hipLaunchKernelGGL(build_windows_sort_kernel, dim3(batch), dim3(WIN_THREADS), p2 * sizeof(uint32_t), stream, g);
  }
  return hipGetLastError();
}

}  // namespace lk
