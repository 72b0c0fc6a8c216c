// Selection under full pairwise matching (appendix, "Bipartite vs. full pairwise matching").  The appendix reports
// accuracy and cost of matching every token against every other token of its window but gives no merge rule; the
// reading implemented here (and in the test oracle): the tokens of a window are visited in ascending order of their
// nearest-neighbour FD (ties: earlier in the window first); a visited token is merged into its nearest neighbour
// unless a token merged earlier was merged INTO it (a token that has received others stays) or its nearest neighbour
// has itself been merged away already; the visit ends after r_w merges.  At most r_w tokens leave a window.
//
// One workgroup per window (at most 4096 tokens), everything in LDS:
//   1. rank of every token among the (FD bits, position) keys of the window, by counting smaller keys
//   2. the visit, which is sequential by definition, as a fixed point: a token can be decided as soon as every token
//      visited before it that could affect it is decided -- the earlier-ranked tokens that name it as their nearest
//      neighbour (any of them leaving makes it a destination) and its own nearest neighbour if that one ranks
//      earlier (it may be gone).  Every round decides at least the lowest-ranked undecided token, so the loop ends
//      after at most v rounds (in practice a handful: chains of nearest neighbours are short); it is bounded by v.
//   3. the first r_w of the tokens that may leave, in rank order (a scan over ranks)
//   4. dst, the number of sources of every destination, and the rank of every source among the sources of its
//      destination in ascending token order -- what select_scan_kernel turns into new_index and the inverse map.
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {

constexpr int PS_THREADS = 1024;
constexpr int PS_MAX = 4096;              // tokens of the largest window
constexpr int PS_ITEMS = PS_MAX / PS_THREADS;

struct PairSelArgs {
  int n_windows, sum_n, cap;              // cap: the caller's bound on the tokens of a window
  const int32_t *win_offsets, *win_tokens, *win_remove;
  const unsigned long long *keys;         // [sum_n] by list position
  float *best_fd;
  int32_t *best_dst, *dst, *cnt, *src_rank;
};

enum : unsigned char { PS_UNDECIDED = 0, PS_LEAVES = 1, PS_STAYS = 2 };

__global__ __launch_bounds__(PS_THREADS) void pair_select_kernel(PairSelArgs g) {
  // order-preserving FD bits (step 1); then, per position, the lowest rank among the undecided tokens that name it
  // (step 2); then the number of its sources (step 4)
  __shared__ __attribute__((aligned(16))) uint32_t key[PS_MAX];
  uint32_t *minpend = key;
  __shared__ __attribute__((aligned(16))) uint16_t nbr[PS_MAX];     // nearest neighbour (list position), 0xffff: none
  __shared__ uint16_t rnk[PS_MAX];
  __shared__ uint16_t by_rank[PS_MAX];                              // token at every rank; later: leavers before every rank
  __shared__ unsigned char state[PS_MAX];
  __shared__ unsigned char received[PS_MAX];
  __shared__ int wave_tot[PS_THREADS / 64];
  __shared__ int n_undecided;
  const int w = blockIdx.x;
  const int off = g.win_offsets[w];
  int v = g.win_offsets[w + 1] - off;
  const int v_all = v;
  v = v < g.cap ? v : g.cap;
  v = v < PS_MAX ? v : PS_MAX;
  int r = g.win_remove[w];
  r = r < 0 ? 0 : r;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // tokens of a window beyond the bound are neither scored nor merged
  for (int l = v + tid; l < v_all; l += PS_THREADS) {
    const int t = g.win_tokens[off + l];
    if ((unsigned)t < (unsigned)g.sum_n) {
      g.dst[t] = -1; g.cnt[t] = 0; g.src_rank[t] = 0;
      g.best_fd[t] = __uint_as_float(0x7f800000u); g.best_dst[t] = -1;
    }
  }
  // ---- 0. keys -> LDS, best_fd / best_dst
  int tok[PS_ITEMS];
#pragma unroll
  for (int k = 0; k < PS_ITEMS; ++k) {
    const int l = k * PS_THREADS + tid;
    tok[k] = -1;
    if (l < PS_MAX) { key[l] = 0xffffffffu; nbr[l] = 0xffffu; state[l] = PS_STAYS; received[l] = 0; }
    if (l < v) {
      const int t = g.win_tokens[off + l];
      const unsigned long long kk = g.keys[off + l];
      const bool okt = (unsigned)t < (unsigned)g.sum_n;
      const unsigned nb = (unsigned)(kk & 0xffffffffu);
      const float fd = __uint_as_float((unsigned)(kk >> 32));
      const bool has = okt && kk != ~0ull && nb < (unsigned)v && fd >= 0.f;   // NaN or negative never competes
      tok[k] = okt ? t : -1;
      key[l] = has ? f32_order_key(fd) : 0xffffffffu;
      nbr[l] = has ? (uint16_t)nb : (uint16_t)0xffffu;
      state[l] = has ? PS_UNDECIDED : PS_STAYS;
      if (okt) {
        const int nt = has ? g.win_tokens[off + (int)nb] : -1;
        g.best_fd[t] = has ? fd : __uint_as_float(0x7f800000u);
        g.best_dst[t] = ((unsigned)nt < (unsigned)g.sum_n) ? nt : -1;
        if (has && (unsigned)nt >= (unsigned)g.sum_n) { nbr[l] = 0xffffu; state[l] = PS_STAYS; key[l] = 0xffffffffu; }
      }
    }
  }
  __syncthreads();
  // ---- 1. ranks by counting (keys beyond v are all-ones: never smaller)
  const int v4 = (v + 3) & ~3;
#pragma unroll
  for (int k = 0; k < PS_ITEMS; ++k) {
    const int l = k * PS_THREADS + tid;
    if (k * PS_THREADS < v) {   // uniform
      const uint32_t mine = l < v ? key[l] : 0xffffffffu;
      int c = 0;
      for (int o = 0; o < v4; o += 4) {
        const uint4 q = *reinterpret_cast<const uint4 *>(&key[o]);
        c += (q.x < mine || (q.x == mine && o < l)) ? 1 : 0;
        c += (q.y < mine || (q.y == mine && o + 1 < l)) ? 1 : 0;
        c += (q.z < mine || (q.z == mine && o + 2 < l)) ? 1 : 0;
        c += (q.w < mine || (q.w == mine && o + 3 < l)) ? 1 : 0;
      }
      if (l < v) { rnk[l] = (uint16_t)c; by_rank[c] = (uint16_t)l; }
    }
  }
  __syncthreads();
  // ---- 2. the visit as a fixed point
  for (int round = 0; round <= v; ++round) {   // bounded: every round decides at least one token
    if (tid == 0) n_undecided = 0;
    for (int l = tid; l < v; l += PS_THREADS) minpend[l] = 0xffffffffu;
    __syncthreads();
    for (int l = tid; l < v; l += PS_THREADS)
      if (state[l] == PS_UNDECIDED) atomicMin(&minpend[nbr[l]], (uint32_t)rnk[l]);
    __syncthreads();
    unsigned char decided[PS_ITEMS];
    int left = 0;
#pragma unroll
    for (int k = 0; k < PS_ITEMS; ++k) {
      const int l = k * PS_THREADS + tid;
      decided[k] = PS_UNDECIDED;
      if (l < v && state[l] == PS_UNDECIDED) {
        const int b = nbr[l];
        const uint32_t my_rank = rnk[l];
        const unsigned char sb = state[b];
        const bool ready = minpend[l] >= my_rank && (sb != PS_UNDECIDED || rnk[b] > my_rank);
        if (ready) decided[k] = (received[l] || sb == PS_LEAVES) ? PS_STAYS : PS_LEAVES;
        else ++left;
      }
    }
    __syncthreads();   // every thread has read the states of this round before any is changed
#pragma unroll
    for (int k = 0; k < PS_ITEMS; ++k) {
      const int l = k * PS_THREADS + tid;
      if (decided[k] != PS_UNDECIDED) {
        state[l] = decided[k];
        if (decided[k] == PS_LEAVES) received[nbr[l]] = 1;
      }
    }
    if (left) atomicAdd(&n_undecided, left);
    __syncthreads();
    if (n_undecided == 0) break;   // uniform
    __syncthreads();               // n_undecided is reset at the top of the next round
  }
  // ---- 3. the first r leavers in rank order: by_rank[q] -> leavers before rank q (exclusive scan over ranks)
  {
    int carry = 0;
    for (int q0 = 0; q0 < v; q0 += PS_THREADS) {   // uniform
      const int q = q0 + tid;
      const int flag = (q < v && state[by_rank[q]] == PS_LEAVES) ? 1 : 0;
      int inc = flag;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(inc, o, 64); if (lane >= o) inc += t; }
      __syncthreads();
      if (lane == 63) wave_tot[wave] = inc;
      __syncthreads();
      int before = carry;
      for (int k = 0; k < wave; ++k) before += wave_tot[k];
      if (q < v && flag && before + inc - flag >= r) state[by_rank[q]] = PS_STAYS;   // beyond the r-th merge: stays after all
      int total = 0;
      for (int k = 0; k < PS_THREADS / 64; ++k) total += wave_tot[k];
      carry += total;
    }
  }
  __syncthreads();
  // ---- 4. destinations, source counts, source ranks.  key[] now counts the sources of every position; nbr of a token
  // that stays is set to "none" so that the rank loop only compares neighbours.
  for (int l = tid; l < v4; l += PS_THREADS) {
    key[l] = 0;
    if (l >= v || state[l] != PS_LEAVES) nbr[l] = 0xffffu;
  }
  __syncthreads();
  for (int l = tid; l < v; l += PS_THREADS)
    if (nbr[l] != 0xffffu) atomicAdd(&key[nbr[l]], 1u);
  __syncthreads();
#pragma unroll
  for (int k = 0; k < PS_ITEMS; ++k) {
    const int l = k * PS_THREADS + tid;
    if (k * PS_THREADS < v) {   // uniform
      const uint16_t mine = l < v ? nbr[l] : (uint16_t)0xffffu;
      int c = 0;
      if (__any(mine != 0xffffu)) {   // waves without a leaver skip the loop
        for (int o = 0; o < v4; o += 8) {
          const uint4 q = *reinterpret_cast<const uint4 *>(&nbr[o]);
          const uint32_t ww[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            c += ((ww[e] & 0xffffu) == mine && o + 2 * e < l) ? 1 : 0;
            c += ((ww[e] >> 16) == mine && o + 2 * e + 1 < l) ? 1 : 0;
          }
        }
      }
      if (l < v && tok[k] >= 0) {
        const bool leaves = mine != 0xffffu;
        const int bt = leaves ? g.win_tokens[off + mine] : -1;
        g.dst[tok[k]] = leaves ? bt : -1;
        g.src_rank[tok[k]] = leaves ? c : 0;
        g.cnt[tok[k]] = (int)key[l];
      }
    }
  }
}

hipError_t launch_pair_select(int n_windows, int max_window, int sum_n, const int32_t *win_offsets,
                              const int32_t *win_tokens, const int32_t *win_remove, const unsigned long long *keys,
                              float *best_fd, int32_t *best_dst, int32_t *dst, int32_t *cnt, int32_t *src_rank,
                              hipStream_t stream) {
  if (n_windows == 0 || sum_n == 0) return hipSuccess;
  PairSelArgs g{};
  g.n_windows = n_windows; g.sum_n = sum_n; g.cap = max_window;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens; g.win_remove = win_remove; g.keys = keys;
  g.best_fd = best_fd; g.best_dst = best_dst; g.dst = dst; g.cnt = cnt; g.src_rank = src_rank;
  hipLaunchKernelGGL(pair_select_kernel, dim3((unsigned)n_windows), dim3(PS_THREADS), 0, stream, g);
  return hipGetLastError();
}

}  // namespace lk
