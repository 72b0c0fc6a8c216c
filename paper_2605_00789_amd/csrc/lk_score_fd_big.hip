// Feature divergence for LARGE windows (paper Sec. 3.2.1 Steps 1-2, Eq. "similarity"; the global stage of
// the hierarchical schedule, Sec. 3.2.2): here the |A| x |B| x d contraction is compute bound and is run as a
// classic LDS-tiled MFMA GEMM with the row arg-min fused into its epilogue.
//
//   row_norms_kernel : |x|^2 of every token (fp32) -- skipped when the caller hands the squared norms in (the kernel
//                      that wrote X can produce them on the way).
//   fd_big_kernel    : workgroup tile 96 x 96, four waves, v_mfma_f32_16x16x32_bf16.  Rows are gathered through the
//                      window's token list; 128-element k-steps travel global -> register ring (2 steps in flight)
//                      -> double-buffered LDS (rows padded to 272 bytes: conflict-free 16-byte operand reads).
//                      Every wave accumulates the whole tile over its quarter of each k-step; the partial tiles are
//                      merged through LDS (fixed order), which also gives a two-level fp32 summation (error of a
//                      4096-long dot product near 2e-7 relative).
//                      Epilogue: cos = dot * (1/|a|) * (1/|b|) in fp64 (inverse roots in fp64, once per tile row and
//                      column), FD = max(1 - cos, 0) rounded to fp32, row minimum over the tile's columns by shuffles
//                      and an LDS integer min on the key (FD bits << 32 | B token): integer min is order independent,
//                      so the result is bit-reproducible and equal FDs go to the earlier B token.  With up to four
//                      column tiles per window the tile's key of every row is stored per column tile and whoever
//                      reads the scores takes the minimum over them (no atomics on global memory, nothing to
//                      initialise); with more, the column tiles meet in one key per row by a 64-bit atomicMin.
//   fd_big_finalize_kernel: keys -> best_fd / best_dst (the selection kernels can read the keys themselves).
#include <atomic>
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {

constexpr int BIG_THREADS = 256;
constexpr int BIG_BK = 128;                    // elements per k-step
constexpr int BIG_PITCH = BIG_BK * 2 + 16;     // bytes per staged row
constexpr int BIG_DEPTH = 2;                   // k-steps of global loads in flight per thread (even)

struct BigArgs {
  const void *X;
  int64_t ldx;
  int d, n_windows, sum_n;
  const int32_t *win_offsets, *win_tokens;
  const float *sq;               // [sum_n] |x|^2 of every token (fp32)
  float *sq_out;                 // row_norms_kernel: where it writes them
  unsigned long long *cand;      // [nt_store][sum_n]: per column tile, the best key of the A row at every list position
  int nt_store;                  // nt: every column tile stores its own keys; 1: all column tiles of a window meet in one
                                 // key per position by atomicMin (the keys are reset first)
  int reset_keys;                // row_norms_kernel: also reset the keys
  float *best_fd;
  int32_t *best_dst;
  int mt, nt;
  int metric;                    // 0: 1 - cos, 1: |a - b|, 2: |a - b|^2
  int mt2, nt2;                  // fd_pair_kernel: 192 x 192 tiles per window along rows and columns
  int dir;                       // bipartite kernels: 0 even list positions propose, 1 odd ones (side_a / pos_a)
};

// ---- |x|^2 per token, summed in fp32 ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void row_norms_kernel(BigArgs g) {
  const int lane = threadIdx.x & 63;
  const int tok = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tok >= g.sum_n) return;
  const char *row = static_cast<const char *>(g.X) + (int64_t)tok * g.ldx * 2;
  const int n_chunks = g.d >> 3;
  float s = 0.f;
  for (int c0 = 0; c0 < n_chunks; c0 += 64 * 8) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int c = c0 + u * 64 + lane;
      v[u] = ld16(row + (int64_t)(c < n_chunks ? c : n_chunks - 1) * 16);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int c = c0 + u * 64 + lane;
      const float t = sumsq_chunk_bf16(v[u]);
      s += (c < n_chunks) ? t : 0.f;
    }
  }
  s = wave_sum_butterfly(s);
  if (lane == 0) {
    g.sq_out[tok] = s;
    if (g.reset_keys) g.cand[tok] = ~0ull;
  }
}

__global__ __launch_bounds__(256) void reset_keys_kernel(BigArgs g) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < g.sum_n) g.cand[i] = ~0ull;
}

// Workgroup tile 96 x 96, four waves.  The waves do NOT split the tile: each one accumulates the whole 96 x 96
// block (6 x 6 MFMA blocks of 16 x 16) over its own quarter of every 128-element k-step.  Per MFMA this halves the
// LDS operand traffic of a 2 x 2 wave arrangement (48 flop per LDS byte instead of 24), and the four partial sums
// give a two-level fp32 summation for free.  The partial tiles are merged through LDS at the end.
constexpr int BIG_TM = FD_BIG_TILE;
constexpr int BIG_NB = BIG_TM / 16;            // 6 blocks per edge
constexpr int BIG_OWN = BIG_NB * BIG_NB / 4;   // 9 blocks per wave in the epilogue
constexpr int BIG_STAGE = 2 * BIG_TM * BIG_PITCH;

__global__ __launch_bounds__(BIG_THREADS) void fd_big_kernel(BigArgs g) {
  constexpr int PASSES = BIG_TM / 16;          // 16 rows x 16 chunks of 16 bytes are staged per pass
  extern __shared__ __attribute__((aligned(16))) char lds[];

  // Workgroups are dealt to the 8 XCDs round robin; give every XCD a contiguous run of logical tiles, and order the
  // tiles of a window in column panels of 4, so that the tiles sharing an L2 touch few distinct row/column blocks.
  const int per = g.mt * g.nt;
  const int n_tiles = g.n_windows * per;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int lid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lid >= n_tiles) return;
  const int w = lid / per;
  const int rem = lid - w * per;
  constexpr int PW = 4;
  const int panel = rem / (g.mt * PW);
  const int in_panel = rem - panel * g.mt * PW;
  const int pw = min(PW, g.nt - panel * PW);
  const int mt = in_panel / pw, nt = panel * PW + (in_panel - mt * pw);
  const int off = g.win_offsets[w];
  const int v = g.win_offsets[w + 1] - off;
  const int nA = side_a(v, g.dir), nB = side_b(v, g.dir);
  const int row0 = mt * BIG_TM, col0 = nt * BIG_TM;
  if (row0 >= nA || col0 >= nB) return;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l16 = lane & 15, kg = lane >> 4;

  // rows this thread stages: 16 rows per pass, 16 threads per row.  Row offsets are 32-bit (the tensor is far
  // below 4 GB, checked by the launcher) so that every load is "uniform base + per-lane offset": the k position
  // advances on the scalar unit and the loop body carries no address arithmetic on the vector unit.
  const int srow = tid >> 4, schunk = tid & 15;
  uint32_t offa[PASSES], offb[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    int la = row0 + p * 16 + srow, lb = col0 + p * 16 + srow;
    la = la < nA ? la : nA - 1;                 // padding rows repeat the last valid one; never read back
    lb = lb < nB ? lb : nB - 1;
    int ta = g.win_tokens[off + pos_a(la, g.dir)], tb = g.win_tokens[off + pos_b(lb, g.dir)];
    ta = ((unsigned)ta < (unsigned)g.sum_n) ? ta : 0;
    tb = ((unsigned)tb < (unsigned)g.sum_n) ? tb : 0;
    offa[p] = (uint32_t)ta * (uint32_t)g.ldx * 2u + (uint32_t)schunk * 16u;
    offb[p] = (uint32_t)tb * (uint32_t)g.ldx * 2u + (uint32_t)schunk * 16u;
  }
  // token and |x|^2 of the tile row / column this thread publishes for the epilogue (threads 0..191), fetched now so
  // that the latency hides behind the k loop
  int e_tok = -1;
  float e_sq = 0.f;
  if (tid < 2 * BIG_TM) {
    const bool is_b = tid >= BIG_TM;
    const int l = (is_b ? col0 : row0) + (is_b ? tid - BIG_TM : tid);
    const int lim = is_b ? nB : nA;
    const int lc = l < lim ? l : lim - 1;
    const int t = g.win_tokens[off + (is_b ? pos_b(lc, g.dir) : pos_a(lc, g.dir))];
    const bool ok = l < lim && (unsigned)t < (unsigned)g.sum_n;
    e_sq = g.sq[ok ? t : 0];
    e_tok = ok ? t : -1;
  }

  f32x4 acc[BIG_NB][BIG_NB];
#pragma unroll
  for (int i = 0; i < BIG_NB; ++i)
#pragma unroll
    for (int j = 0; j < BIG_NB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // d is a multiple of 2 * BIG_BK (checked by the launcher): an even number of whole k-steps, no tails.
  const int n_ksteps = g.d / BIG_BK;
  const char *xbase = static_cast<const char *>(g.X);
  // Global -> register ring (BIG_DEPTH k-steps in flight) -> LDS (double buffered) -> MFMA operands.
  uint4 ring[BIG_DEPTH][2 * PASSES];
  auto gload = [&](int ks, uint4 *r) {   // unconditional: steps past the end re-read the last one
    const char *kb = xbase + (size_t)(ks < n_ksteps ? ks : n_ksteps - 1) * (BIG_BK * 2);   // scalar
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      r[p] = ld16(kb + offa[p]);
      r[PASSES + p] = ld16(kb + offb[p]);
    }
  };
  char *lds_w = lds + srow * BIG_PITCH + schunk * 16;
  auto lstore = [&](int stage, const uint4 *r) {
    char *base = lds_w + stage * BIG_STAGE;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      *reinterpret_cast<uint4 *>(base + p * 16 * BIG_PITCH) = r[p];
      *reinterpret_cast<uint4 *>(base + BIG_TM * BIG_PITCH + p * 16 * BIG_PITCH) = r[PASSES + p];
    }
  };
  const char *lds_r = lds + l16 * BIG_PITCH + wave * 64 + kg * 16;
  // One k-step: the operand fragments of `stage` are read first; then the 36 MFMAs are issued with the 12 LDS stores
  // that move step ks + 1 from its ring slot into the other stage slotted between them (3 MFMAs, 1 store, ...), so
  // the matrix pipe runs while the LDS port takes the stores, and the global loads feeding those stores get the
  // whole fragment-read time on top of their two k-steps to arrive.  Each ring register is refilled right after its store.
  auto step = [&](int stage, uint4 *r, int ks_refill) {
    const char *abase = lds_r + stage * BIG_STAGE;
    const char *bbase = abase + BIG_TM * BIG_PITCH;
    char *wbase = lds_w + (stage ^ 1) * BIG_STAGE;
    bf16x8 fa[BIG_NB], fb[BIG_NB];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < BIG_NB; ++i) fb[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(bbase + i * 16 * BIG_PITCH));
#pragma unroll
    for (int i = 0; i < BIG_NB; ++i) fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(abase + i * 16 * BIG_PITCH));
#pragma unroll
    for (int i = 0; i < BIG_NB; ++i)
#pragma unroll
      for (int j = 0; j < BIG_NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      *reinterpret_cast<uint4 *>(wbase + p * 16 * BIG_PITCH) = r[p];
      *reinterpret_cast<uint4 *>(wbase + BIG_TM * BIG_PITCH + p * 16 * BIG_PITCH) = r[PASSES + p];
    }
    gload(ks_refill, r);
    // issue order for the block above: 12 LDS reads, then (3 MFMA, 1 LDS write, the refill of that register) x 12
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * BIG_NB, 0);
#pragma unroll
    for (int q = 0; q < 2 * PASSES; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, BIG_NB * BIG_NB / (2 * PASSES), 0);
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // sched_barrier(0) pins the issue order: loads complete in order, so the wait before an LDS store only has to
  // cover the oldest slot while the younger ones stay in flight.
#pragma unroll
  for (int j = 0; j < BIG_DEPTH; ++j) {
    gload(j, ring[j]);
    __builtin_amdgcn_sched_barrier(0);
  }
  lstore(0, ring[0]);
  __builtin_amdgcn_sched_barrier(0);
  gload(BIG_DEPTH, ring[0]);
  __builtin_amdgcn_sched_barrier(0);
  lds_barrier();
  // The body is branch free: with control flow inside, the compiler's wait-count bookkeeping falls back to waiting
  // for every load in flight.  Step ks computes from LDS stage ks & 1 while the data of step ks + 1 moves from its
  // ring slot to the other stage (after the last step that copy is a harmless repeat).
  // (an empty statement that ties every accumulator to the accumulation registers at this point: without it the
  // register allocator rotates the accumulators through other registers inside the k loop, ~100 copies per step)
#pragma unroll
  for (int i = 0; i < BIG_NB; ++i)
#pragma unroll
    for (int j = 0; j < BIG_NB; ++j) asm volatile("" : "+a"(acc[i][j]));
  for (int ks0 = 0; ks0 < n_ksteps; ks0 += BIG_DEPTH) {
#pragma unroll
    for (int u = 0; u < BIG_DEPTH; ++u) {
      const int ks = ks0 + u;
      const int slot = (u + 1) % BIG_DEPTH;        // ring slot of step ks + 1
      step(u & 1, ring[slot], ks + 1 + BIG_DEPTH);   // BIG_DEPTH is even: the stage parity is static
      lds_barrier();
    }
  }

  // (an empty statement that ties every accumulator to the accumulation registers at this point: without it the
  // register allocator rotates the accumulators through other registers inside the k loop, ~100 copies per step)
#pragma unroll
  for (int i = 0; i < BIG_NB; ++i)
#pragma unroll
    for (int j = 0; j < BIG_NB; ++j) asm volatile("" : "+a"(acc[i][j]));
  // ---- merge the four partial tiles: wave w ends up owning the blocks whose linear id is w mod 4.
  // LDS is free now: [0, 1536) bytes hold 1/|a| and 1/|b| of the tile, [1536, 2304) the tokens, [2304, 3072) the row
  // keys, then from 4096 on the 4 x 12 KB exchange buffers.
  double *e_rnorm = reinterpret_cast<double *>(lds);              // [96] rows then [96] cols
  int *e_token = reinterpret_cast<int *>(lds + 2 * BIG_TM * 8);   // [96] row tokens then [96] col tokens
  float *xbuf = reinterpret_cast<float *>(lds + 4096);            // [4 waves][12 blocks][256 floats]
  unsigned long long *row_key = reinterpret_cast<unsigned long long *>(lds + 2 * BIG_TM * 8 + 2 * BIG_TM * 4);   // [96]
  if (tid < 2 * BIG_TM) {
    // the only fp64 sqrt/div of the cosine path: once per tile row and column
    e_rnorm[tid] = e_sq != e_sq ? (double)e_sq : (g.metric == 0 ? 1.0 / fmax(sqrt((double)e_sq), 1e-12) : (double)e_sq);   // NaN rows keep a NaN norm
    e_token[tid] = e_tok;
  }
  if (tid < BIG_TM) row_key[tid] = ~0ull;
  // Three rounds of 12 blocks: every wave leaves its partials of the round's blocks in LDS, the owner of a block
  // (wave w owns blocks 12 t + 3 w + 0..2 of round t) adds the four partials in a fixed order.  Register indices
  // are static everywhere -- only LDS addresses depend on the wave -- so the accumulators stay in place in the k loop.
  f32x4 own[BIG_OWN];
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 3; ++t) {
#pragma unroll
    for (int k = 0; k < 12; ++k) {
      const int b = 12 * t + k;
      *reinterpret_cast<f32x4 *>(xbuf + ((wave * 12 + k) * 64 + lane) * 4) = acc[b / BIG_NB][b % BIG_NB];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const float *src = xbuf + ((3 * wave + k) * 64 + lane) * 4;
      const f32x4 p0 = *reinterpret_cast<const f32x4 *>(src);
      const f32x4 p1 = *reinterpret_cast<const f32x4 *>(src + 12 * 256);
      const f32x4 p2 = *reinterpret_cast<const f32x4 *>(src + 2 * 12 * 256);
      const f32x4 p3 = *reinterpret_cast<const f32x4 *>(src + 3 * 12 * 256);
      own[3 * t + k] = (p0 + p1) + (p2 + p3);
    }
    __syncthreads();
  }

  // ---- epilogue on the owned blocks.  Round t, wave w: blocks (i, j) = (2 t + w / 2, 3 (w % 2) + k), k = 0..2 --
  // three neighbours in one block row, so a lane first takes the minimum over its three columns, and only 12 keys
  // per lane go through the 16-lane reduction.  The reductions run side by side (all shuffles of a step are issued
  // before the first is used): with one wave per SIMD a chain of dependent shuffles would expose every latency.
  // Accumulator layout of a 16x16 block: lane holds column (lane % 16) and rows 4*(lane/16) + 0..3.
  unsigned long long kmin[12];
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    const int bi = 2 * t + (wave >> 1);
#pragma unroll
    for (int q = 0; q < 4; ++q) kmin[4 * t + q] = ~0ull;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int cl = (3 * (wave & 1) + k) * 16 + l16;
      const double rb = e_rnorm[BIG_TM + cl];
      const int tb = e_token[BIG_TM + cl];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int rl = bi * 16 + kg * 4 + q;
        const double ra = e_rnorm[rl];
        const int ta = e_token[rl];
        const double dot = (double)own[3 * t + k][q];
        float fd;
        if (g.metric == 0) {
          { const double c1 = 1.0 - dot * ra * rb; fd = (float)(c1 < 0.0 ? 0.0 : c1); }   // (a NaN stays a NaN: fmax would drop it)
        } else {   // |a - b|^2 = |a|^2 + |b|^2 - 2 <a, b>
          double d2 = ra + rb - 2.0 * dot;
          d2 = d2 < 0.0 ? 0.0 : d2;   // (keeps a NaN)
          fd = (float)(g.metric == 1 ? sqrt(d2) : d2);
        }
        // key = (FD bits, B token): tokens of a window ascend with their local position, so the smaller token is the
        // earlier column; NaN never competes
        unsigned long long key = ((unsigned long long)__float_as_uint(fd) << 32) | (unsigned)tb;
        key = (ta >= 0 && tb >= 0 && fd == fd) ? key : ~0ull;
        kmin[4 * t + q] = key < kmin[4 * t + q] ? key : kmin[4 * t + q];
      }
    }
  }
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) {   // the 16 lanes with the same lane/16 hold the same rows
    unsigned long long other[12];
#pragma unroll
    for (int e = 0; e < 12; ++e) other[e] = __shfl_xor(kmin[e], m, 64);
#pragma unroll
    for (int e = 0; e < 12; ++e) kmin[e] = other[e] < kmin[e] ? other[e] : kmin[e];
  }
  if (l16 == 0) {   // LDS: minimum over the tile's 6 column blocks (two waves contribute to every row)
#pragma unroll
    for (int e = 0; e < 12; ++e) {
      const int rl = (2 * (e >> 2) + (wave >> 1)) * 16 + kg * 4 + (e & 3);
      if (kmin[e] != ~0ull) atomicMin(&row_key[rl], kmin[e]);
    }
  }
  __syncthreads();
  // the tile's best key of every row, filed under the row's position in the window list and this column tile: the
  // reader takes the minimum over the window's column tiles (integer min: equal FDs go to the earlier B token)
  // With many column tiles per window that minimum is taken here instead, by one integer atomicMin per row and tile
  // on a single key per position (order independent, so still bit-reproducible).
  if (tid < BIG_TM && row0 + tid < nA) {
    const size_t pos = (size_t)(off + pos_a(row0 + tid, g.dir));
    if (g.nt_store > 1 || g.nt == 1) g.cand[(size_t)nt * (size_t)g.sum_n + pos] = row_key[tid];
    else if (row_key[tid] != ~0ull) atomicMin(&g.cand[pos], row_key[tid]);
  }
}

// Keys -> best_fd / best_dst for every token, window by window (the keys are filed by list position).  A token no
// key was offered for (B nodes, A nodes of windows without a B node, rows of NaNs, rows beyond the caller's window
// bound) gets +inf / -1.
__global__ __launch_bounds__(256) void fd_big_finalize_kernel(BigArgs g, int chunks_per_window) {
  const int w = blockIdx.x / chunks_per_window, c = blockIdx.x - w * chunks_per_window;
  const int off = g.win_offsets[w];
  const int v = g.win_offsets[w + 1] - off;
  const int n_col = fd_big_col_tiles(side_b(v, g.dir), g.nt_store);
  for (int t = c * 256 + (int)threadIdx.x; t < v; t += chunks_per_window * 256) {
    const int tok = g.win_tokens[off + t];
    if ((unsigned)tok >= (unsigned)g.sum_n) continue;
    const bool scored = (t & 1) == g.dir && (t >> 1) < g.mt * FD_BIG_TILE;
    const unsigned long long key = scored ? fd_big_best_key(g.cand, g.sum_n, off + t, n_col) : ~0ull;
    g.best_fd[tok] = key == ~0ull ? __uint_as_float(0x7f800000u) : __uint_as_float((unsigned)(key >> 32));
    g.best_dst[tok] = key == ~0ull ? -1 : (int)(key & 0xffffffffu);
  }
}


// ---------------------------------------------------------------------------------------------------------------------
// Full pairwise matching (appendix, "Bipartite vs. full pairwise matching"): FD between every two tokens of a window,
// the whole v x v matrix (what the appendix FLOPs table counts: 4 x the bipartite block), and for every token its
// lowest-FD neighbour.  For the 2880-token window that is a 2880 x 2880 x 4096 contraction, 68 GFLOP.
//
// What bounds these kernels is operand delivery, not the matrix pipe: every operand byte a workgroup consumes comes
// out of L2 (nothing is reused through L1), the chip's L2s hand over about 19.5 TB/s in total (measured with the
// loads of this very loop alone), and a T x T tile needs 2 * 2T bytes per k for 2 T^2 flop per k.  With 96 x 96 tiles
// the loads alone take longer than the MFMAs; here the output is large enough for 192 x 192 tiles to fill the chip
// (15 x 15 = 225 workgroups), which halves the bytes per flop.  A workgroup is 2 x 2 waves of 96 x 96 each, a wave's
// tile a 3 x 3 grid of 32 x 32 accumulators.  (Bare loops of independent MFMAs on this chip: v_mfma_f32_32x32x16_bf16
// sustains 2.0-2.1 PFLOP/s on constant operands and 1.33-1.5 PFLOP/s on random bf16 operands -- the clocks drop
// with the switching activity -- and v_mfma_f32_16x16x32_bf16 1.4-1.5 even on constant ones.  So about 1.5 PFLOP/s,
// 60 % of the nominal 2.5, is what the matrix pipes give on real data.  Measured on this kernel, 2880 x 2880 x 4096:
// 89 us in all; without its LDS stores 75; MFMAs and barriers alone 66, of which about 10 are launch, the dependent
// index loads in front of the loop and the epilogue; the global loads cost nothing on top.)  Per
// k-step of 64: 384 rows x 128 bytes staged (12 loads and 12 LDS stores per thread), 24 fragment reads and 36 MFMAs
// per wave; register ring of two k-steps, two LDS stages, one LDS-only barrier per step, branch-free body.
// Epilogue per wave on its own quadrant: FD in fp64 from the stored norms, diagonal masked, minimum over the three
// column blocks per lane, 32-lane reductions by shuffles, one integer atomicMin per row and wave on the row's key
// (FD bits << 32 | position of the neighbour in the window list): order independent, so bit-reproducible, and equal
// FDs go to the earlier neighbour.
constexpr int T2_NB = 3;                          // 32 x 32 blocks per edge of a wave's tile
constexpr int T2_WT = 32 * T2_NB;                 // 96
constexpr int T2_TM = 2 * T2_WT;                  // 192: rows and columns of a workgroup tile
constexpr int T2_BK = 64;                         // elements per k-step
constexpr int T2_PITCH = T2_BK * 2 + 16;          // 144 bytes per staged row: 16 rows of one k-chunk fall on 16 distinct 16-byte slots
constexpr int T2_STAGE = 2 * T2_TM * T2_PITCH;    // row panel, then column panel
constexpr int T2_PASSES = T2_TM / 32;             // 32 rows x 8 chunks of 16 bytes are staged per pass

// (window, tile) of a workgroup.  Workgroups are dealt to the 8 XCDs round robin, each XCD with an L2 of its own.  One
// window: the tile grid is cut into 2 x 4 blocks, one per XCD, so that an XCD's tiles touch as few distinct row and
// column panels as possible (what an XCD's L2 has to fetch from the fabric).  Several windows: every XCD takes a
// contiguous run of (window, tile) jobs, tiles row-major.
struct T2Job { int w, mt, nt; bool ok; };
__device__ __forceinline__ T2Job t2_job(const BigArgs &g, int block) {
  T2Job j{0, 0, 0, false};
  const int xcd = block & 7, local = block >> 3;
  if (g.n_windows == 1) {
    const int bi = xcd >> 2, bj = xcd & 3;
    const int r0 = bi * g.mt2 / 2, r1 = (bi + 1) * g.mt2 / 2;
    const int c0 = bj * g.nt2 / 4, c1 = (bj + 1) * g.nt2 / 4;
    const int wd = c1 - c0;
    if (wd <= 0 || local >= wd * (r1 - r0)) return j;
    j.mt = r0 + local / wd;
    j.nt = c0 + local - (local / wd) * wd;
    j.ok = true;
    return j;
  }
  const int per = g.mt2 * g.nt2;
  const int n_jobs = g.n_windows * per;
  const int per_xcd = (n_jobs + 7) >> 3;
  const int lid = xcd * per_xcd + local;
  if (local >= per_xcd || lid >= n_jobs) return j;
  j.w = lid / per;
  const int rem = lid - j.w * per;
  j.mt = rem / g.nt2;
  j.nt = rem - j.mt * g.nt2;
  j.ok = true;
  return j;
}
// workgroups to launch so that every job of t2_job has one
static unsigned t2_grid(int n_windows, int mt2, int nt2) {
  if (n_windows == 1) {
    int biggest = 0;
    for (int x = 0; x < 8; ++x) {
      const int bi = x >> 2, bj = x & 3;
      const int h = (bi + 1) * mt2 / 2 - bi * mt2 / 2, wd = (bj + 1) * nt2 / 4 - bj * nt2 / 4;
      biggest = h * wd > biggest ? h * wd : biggest;
    }
    return 8u * (unsigned)biggest;
  }
  const unsigned n_jobs = (unsigned)n_windows * (unsigned)(mt2 * nt2);
  return (n_jobs + 7u) / 8u * 8u;
}

__global__ __launch_bounds__(BIG_THREADS) void fd_pair_kernel(BigArgs g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const T2Job job = t2_job(g, blockIdx.x);
  if (!job.ok) return;
  const int off = g.win_offsets[job.w];
  int v = g.win_offsets[job.w + 1] - off;
  v = v < g.mt2 * T2_TM ? v : g.mt2 * T2_TM;       // a window beyond the caller's bound: its surplus tokens are not scored
  const int row0 = job.mt * T2_TM, col0 = job.nt * T2_TM;
  if (v < 2 || row0 >= v || col0 >= v) return;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, kg = lane >> 5;    // MFMA operand layout: row (column) l32, k-slice kg of a 16-element sub-step
  const int wm = wave >> 1, wn = wave & 1;

  // rows this thread stages: 32 rows per pass, 8 threads per row (128 bytes).  Inside a wave the row order is
  // 0, 8, 1, 9, ...: two rows that are 8 apart lie 8 * 144 = 128 (mod 256) bytes apart, so the 16 lanes of a quarter
  // wave store to 256 distinct bytes of a 256-byte bank row (in natural order neighbouring rows overlap by 16 bytes).
  // 32-bit offsets (checked by the launcher): every load is "uniform base + per-lane offset", the k position
  // advances on the scalar unit.
  const int sg = tid >> 3, schunk = tid & 7;
  const int srow = (sg & ~15) | ((sg & 1) << 3) | ((sg & 15) >> 1);
  uint32_t offa[T2_PASSES], offb[T2_PASSES];
#pragma unroll
  for (int p = 0; p < T2_PASSES; ++p) {
    int la = row0 + p * 32 + srow, lb = col0 + p * 32 + srow;
    la = la < v ? la : v - 1;                   // padding rows repeat the last valid one; their results are never used
    lb = lb < v ? lb : v - 1;
    int ta = g.win_tokens[off + la], tb = g.win_tokens[off + lb];
    ta = ((unsigned)ta < (unsigned)g.sum_n) ? ta : 0;
    tb = ((unsigned)tb < (unsigned)g.sum_n) ? tb : 0;
    offa[p] = (uint32_t)ta * (uint32_t)g.ldx * 2u + (uint32_t)schunk * 16u;
    offb[p] = (uint32_t)tb * (uint32_t)g.ldx * 2u + (uint32_t)schunk * 16u;
  }
  // |x|^2 of the tile rows / columns this thread publishes for the epilogue (384 entries over 256 threads), fetched now
  // so that the latency hides behind the k loop
  float e_sq[2];
  bool e_ok[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int e = tid + u * BIG_THREADS;          // 0..191: rows, 192..383: columns
    const int l = e < T2_TM ? row0 + e : col0 + e - T2_TM;
    const int t = g.win_tokens[off + (l < v ? l : v - 1)];
    e_ok[u] = e < 2 * T2_TM && l < v && (unsigned)t < (unsigned)g.sum_n;
    e_sq[u] = g.sq[e_ok[u] ? t : 0];
  }

  f32x16 acc[T2_NB][T2_NB];
#pragma unroll
  for (int i = 0; i < T2_NB; ++i)
#pragma unroll
    for (int j = 0; j < T2_NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int n_my = g.d / T2_BK;                   // k-steps (d is a multiple of 64, at least 64: checked by the launcher)
  const char *xbase = static_cast<const char *>(g.X);
  uint4 ring[2][2 * T2_PASSES];
  auto gload = [&](int ks, uint4 *r) {   // unconditional: steps past the end re-read the last one
    const char *kb = xbase + (size_t)(ks < n_my ? ks : n_my - 1) * (T2_BK * 2);   // scalar
#pragma unroll
    for (int p = 0; p < T2_PASSES; ++p) {
      r[p] = ld16(kb + offa[p]);
      r[T2_PASSES + p] = ld16(kb + offb[p]);
    }
  };
  char *lds_w = lds + srow * T2_PITCH + schunk * 16;
  auto lstore = [&](int stage, const uint4 *r) {
    char *base = lds_w + stage * T2_STAGE;
#pragma unroll
    for (int p = 0; p < T2_PASSES; ++p) {
      *reinterpret_cast<uint4 *>(base + p * 32 * T2_PITCH) = r[p];
      *reinterpret_cast<uint4 *>(base + T2_TM * T2_PITCH + p * 32 * T2_PITCH) = r[T2_PASSES + p];
    }
  };
  const char *lds_ra = lds + (wm * T2_WT + l32) * T2_PITCH + kg * 16;
  const char *lds_rb = lds + (T2_TM + wn * T2_WT + l32) * T2_PITCH + kg * 16;
  // operand fragments of one 32-element half of a k-step: two 16-element sub-steps x (3 row blocks + 3 column blocks)
  struct Frag { bf16x8 a[2][T2_NB], b[2][T2_NB]; };
  auto fread = [&](int stage, int h, Frag &f) {
    const char *abase = lds_ra + stage * T2_STAGE + h * 64;
    const char *bbase = lds_rb + stage * T2_STAGE + h * 64;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int i = 0; i < T2_NB; ++i) f.b[u][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(bbase + i * 32 * T2_PITCH + u * 32));
#pragma unroll
      for (int i = 0; i < T2_NB; ++i) f.a[u][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(abase + i * 32 * T2_PITCH + u * 32));
    }
  };
  auto mma = [&](const Frag &f) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < T2_NB; ++i)
#pragma unroll
        for (int j = 0; j < T2_NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[u][i], f.b[u][j], acc[i][j], 0, 0, 0);
  };
  // One k-step = two halves of 32 elements, and the operand fragments of a half are fetched from LDS while the
  // MFMAs of the half before it run, so that (with one wave per SIMD) the matrix pipe never waits for an LDS round trip:
  //   first half : 18 MFMAs on f0 | 12 fragment reads (second half of this stage -> f1) | the 12 LDS stores that move
  //                the next step's data from its ring slot into the other stage | 6 of the 12 global loads that refill
  //                the ring slot
  //   barrier    : the other stage is complete (LDS traffic only; global loads stay in flight)
  //   second half: 18 MFMAs on f1 | 12 fragment reads (first half of the other stage -> f0) | the other 6 refills
  // Issue order is pinned with sched_group_barrier: one MFMA, then one LDS or memory instruction, and so on.
  Frag f0, f1;
  auto step = [&](int stage, uint4 *r, int ks_refill) {
    char *wbase = lds_w + (stage ^ 1) * T2_STAGE;
    const char *kb = xbase + (size_t)(ks_refill < n_my ? ks_refill : n_my - 1) * (T2_BK * 2);   // scalar
    __builtin_amdgcn_sched_barrier(0);
    fread(stage, 1, f1);
    mma(f0);
#pragma unroll
    for (int p = 0; p < T2_PASSES; ++p) {
      *reinterpret_cast<uint4 *>(wbase + p * 32 * T2_PITCH) = r[p];
      *reinterpret_cast<uint4 *>(wbase + T2_TM * T2_PITCH + p * 32 * T2_PITCH) = r[T2_PASSES + p];
    }
#pragma unroll
    for (int p = 0; p < T2_PASSES / 2; ++p) {
      r[p] = ld16(kb + offa[p]);
      r[T2_PASSES + p] = ld16(kb + offb[p]);
    }
    // 12 reads first (they feed the second half and have the whole first half to arrive), then 12 x (1 MFMA, 1 store),
    // then 6 x (1 MFMA, 1 load)
    __builtin_amdgcn_sched_group_barrier(0x100, 4 * T2_NB, 0);
#pragma unroll
    for (int q = 0; q < 2 * T2_PASSES; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
    }
#pragma unroll
    for (int q = 0; q < T2_PASSES; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();
    __builtin_amdgcn_sched_barrier(0);
    fread(stage ^ 1, 0, f0);
    mma(f1);
#pragma unroll
    for (int p = T2_PASSES / 2; p < T2_PASSES; ++p) {
      r[p] = ld16(kb + offa[p]);
      r[T2_PASSES + p] = ld16(kb + offb[p]);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 4 * T2_NB, 0);
#pragma unroll
    for (int q = 0; q < T2_PASSES; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  gload(0, ring[0]);
  __builtin_amdgcn_sched_barrier(0);
  gload(1, ring[1]);
  __builtin_amdgcn_sched_barrier(0);
  lstore(0, ring[0]);
  __builtin_amdgcn_sched_barrier(0);
  gload(2, ring[0]);
  __builtin_amdgcn_sched_barrier(0);
  lds_barrier();
  fread(0, 0, f0);
  // (an empty statement that ties every accumulator to the accumulation registers: without it the register allocator
  // rotates the accumulators through other registers inside the k loop)
#pragma unroll
  for (int i = 0; i < T2_NB; ++i)
#pragma unroll
    for (int j = 0; j < T2_NB; ++j) asm volatile("" : "+a"(acc[i][j]));
  // Step ks computes from LDS stage ks & 1 while the data of step ks + 1 moves from its ring slot to the other stage
  // (after the last step that copy is a harmless repeat, and so is the fragment fetch at its end).  Steps come in
  // pairs so that stage and ring slot are static.  No barrier is needed between two steps: a step only stores to the
  // stage whose last reads (this wave's and, through the mid-step barrier of the step before, everybody's) are complete.
  int ks = 0;
  for (; ks + 1 < n_my; ks += 2) {
    step(0, ring[1], ks + 3);
    step(1, ring[0], ks + 4);
  }
  if (ks < n_my) step(0, ring[1], ks + 3);   // an odd number of steps: the last one, from stage 0
#pragma unroll
  for (int i = 0; i < T2_NB; ++i)
#pragma unroll
    for (int j = 0; j < T2_NB; ++j) asm volatile("" : "+a"(acc[i][j]));
  __syncthreads();   // every wave is through with the operand stages before the epilogue reuses LDS

  // ---- epilogue.  LDS is free now: 1/|x| (or |x|^2 for the distances) of the 192 rows, then of the 192 columns.
  double *e_rnorm = reinterpret_cast<double *>(lds);
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int e = tid + u * BIG_THREADS;
    if (e < 2 * T2_TM)   // a negative entry marks a row or column that does not exist (norms are never negative)
      e_rnorm[e] = !e_ok[u] ? -1.0 : (e_sq[u] != e_sq[u] || g.metric != 0 ? (double)e_sq[u] : 1.0 / fmax(sqrt((double)e_sq[u]), 1e-12));   // NaN rows keep a NaN norm
  }
  __syncthreads();
  // Accumulator layout of a 32 x 32 block: a lane holds column lane % 32 and the 16 rows acc_row(e, lane).
#pragma unroll
  for (int i = 0; i < T2_NB; ++i) {
    unsigned long long kmin[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) kmin[e] = ~0ull;
#pragma unroll
    for (int j = 0; j < T2_NB; ++j) {
      const int cl = wn * T2_WT + j * 32 + l32;
      const double rb = e_rnorm[T2_TM + cl];
      const int lb = col0 + cl;                     // position of the column token in the window list
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rl = wm * T2_WT + i * 32 + acc_row(e, lane);
        const double ra = e_rnorm[rl];
        const double dot = (double)acc[i][j][e];
        float fd;
        if (g.metric == 0) {
          { const double c1 = 1.0 - dot * ra * rb; fd = (float)(c1 < 0.0 ? 0.0 : c1); }   // (a NaN stays a NaN: fmax would drop it)
        } else {   // |a - b|^2 = |a|^2 + |b|^2 - 2 <a, b>
          double d2 = ra + rb - 2.0 * dot;
          d2 = d2 < 0.0 ? 0.0 : d2;   // (keeps a NaN)
          fd = (float)(g.metric == 1 ? sqrt(d2) : d2);
        }
        unsigned long long key = ((unsigned long long)__float_as_uint(fd) << 32) | (unsigned)lb;
        key = (ra >= 0.0 && rb >= 0.0 && row0 + rl != lb && fd == fd) ? key : ~0ull;   // no self pairs, NaN never competes
        kmin[e] = key < kmin[e] ? key : kmin[e];
      }
    }
#pragma unroll
    for (int m = 16; m >= 1; m >>= 1) {   // the 32 lanes with the same lane / 32 hold the same rows
      unsigned long long other[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) other[e] = __shfl_xor(kmin[e], m, 64);
#pragma unroll
      for (int e = 0; e < 16; ++e) kmin[e] = other[e] < kmin[e] ? other[e] : kmin[e];
    }
    if (l32 == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int la = row0 + wm * T2_WT + i * 32 + acc_row(e, lane);
        if (la < v && kmin[e] != ~0ull) atomicMin(&g.cand[(size_t)(off + la)], kmin[e]);
      }
    }
  }
}

FdBigPlan make_fd_big_plan(int n_windows, int max_window_tokens, int sum_n) {
  FdBigPlan p{};
  const int maxA = (max_window_tokens + 1) / 2, maxB = max_window_tokens / 2;
  p.wb = BIG_NB;   // 96 x 96 workgroup tiles: 15 x 15 = 225 tiles for the 1440 x 1440 case, one round on 256 CUs
  p.mt = (maxA + BIG_TM - 1) / BIG_TM;
  p.nt = maxB > 0 ? (maxB + BIG_TM - 1) / BIG_TM : 1;
  p.metric = 0;
  p.max_window = max_window_tokens;
  p.norm_floats = (size_t)sum_n;
  p.nt_store = p.nt <= FD_BIG_KEYS_PER_TILE_MAX_NT ? p.nt : 1;
  p.key_bytes = (size_t)sum_n * 8 * (size_t)p.nt_store;
  return p;
}

// kernels that ask for more dynamic LDS than the 64 KB default: a property of a kernel as loaded on a device, set once
// per device (setting it twice is harmless: the flag only has to be free of data races)
static hipError_t allow_big_lds(int which, const void *kernel, size_t lds) {
  static std::atomic<bool> attr_set[2][64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[which][dev].load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set[which][dev].store(true, std::memory_order_release);
  }
  return hipSuccess;
}

hipError_t launch_fd_big(const FdBigPlan &plan, const void *X, int64_t ldx, int d, int n_windows, int sum_n,
                         const int32_t *win_offsets, const int32_t *win_tokens, const float *x_sqnorm, float *sq_ws,
                         unsigned long long *keys, float *best_fd, int32_t *best_dst, bool finalize,
                         hipStream_t stream) {
  if (n_windows == 0 || sum_n == 0) return hipSuccess;
  BigArgs g{};
  g.X = X; g.ldx = ldx; g.d = d; g.n_windows = n_windows; g.sum_n = sum_n;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens;
  g.cand = keys; g.best_fd = best_fd; g.best_dst = best_dst;
  g.mt = plan.mt; g.nt = plan.nt; g.metric = plan.metric; g.dir = plan.dir;
  g.sq = x_sqnorm ? x_sqnorm : sq_ws; g.sq_out = sq_ws;
  g.nt_store = plan.nt_store;
  g.reset_keys = plan.nt_store == 1 && plan.nt > 1;   // one key per position, reached by atomicMin: start from all-ones
  hipError_t e;
  if (!x_sqnorm) {   // nobody computed the squared norms on the way: one pass over X (which also resets the keys)
    hipLaunchKernelGGL(row_norms_kernel, dim3((unsigned)((sum_n + 3) / 4)), dim3(256), 0, stream, g);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  } else if (g.reset_keys) {
    hipLaunchKernelGGL(reset_keys_kernel, dim3((unsigned)((sum_n + 255) / 256)), dim3(256), 0, stream, g);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const unsigned n_tiles = (unsigned)(n_windows * plan.mt * plan.nt);
  const unsigned grid = (n_tiles + 7u) / 8u * 8u;   // whole rounds over the XCDs; surplus workgroups exit at once
  constexpr size_t lds = (size_t)2 * BIG_STAGE;      // 102 KB: above the 64 KB default
  e = allow_big_lds(0, reinterpret_cast<const void *>(fd_big_kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fd_big_kernel, dim3(grid), dim3(BIG_THREADS), lds, stream, g);
  e = hipGetLastError();
  if (e != hipSuccess || !finalize) return e;   // without it the caller's selection reads the keys
  const int cpw = (plan.max_window + 255) / 256 > 0 ? (plan.max_window + 255) / 256 : 1;
  hipLaunchKernelGGL(fd_big_finalize_kernel, dim3((unsigned)(n_windows * cpw)), dim3(256), 0, stream, g, cpw);
  return hipGetLastError();
}

// Keys of fd_pair_kernel -> best_fd / best_dst (every token's nearest neighbour), for callers of lightkv_score; the
// selection of lightkv_score_select reads the keys itself.
__global__ __launch_bounds__(256) void fd_pair_finalize_kernel(BigArgs g, int chunks_per_window) {
  const int w = blockIdx.x / chunks_per_window, c = blockIdx.x - w * chunks_per_window;
  const int off = g.win_offsets[w];
  const int v = g.win_offsets[w + 1] - off;
  const int scored = v < g.mt2 * T2_TM ? v : g.mt2 * T2_TM;
  for (int l = c * 256 + (int)threadIdx.x; l < v; l += chunks_per_window * 256) {
    const int tok = g.win_tokens[off + l];
    if ((unsigned)tok >= (unsigned)g.sum_n) continue;
    const unsigned long long key = l < scored ? g.cand[off + l] : ~0ull;
    const unsigned nb = (unsigned)(key & 0xffffffffu);
    const int nt = (key != ~0ull && nb < (unsigned)scored) ? g.win_tokens[off + (int)nb] : -1;
    const bool has = (unsigned)nt < (unsigned)g.sum_n;
    g.best_fd[tok] = has ? __uint_as_float((unsigned)(key >> 32)) : __uint_as_float(0x7f800000u);
    g.best_dst[tok] = has ? nt : -1;
  }
}

// Full pairwise matching: squared norms (unless handed in) and key reset, then the 192 x 192 tiled kernel.  Leaves one
// packed key per list position in `keys` (FD bits << 32 | position of the nearest neighbour in the window list; all
// ones where there is none); the selection reads them.  d must be a multiple of 64.
hipError_t launch_fd_pair(const void *X, int64_t ldx, int d, int n_windows, int max_window, int sum_n, int metric,
                          const int32_t *win_offsets, const int32_t *win_tokens, const float *x_sqnorm, float *sq_ws,
                          unsigned long long *keys, float *best_fd, int32_t *best_dst, hipStream_t stream) {
  if (n_windows == 0 || sum_n == 0) return hipSuccess;
  BigArgs g{};
  g.X = X; g.ldx = ldx; g.d = d; g.n_windows = n_windows; g.sum_n = sum_n;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens;
  g.cand = keys; g.metric = metric; g.best_fd = best_fd; g.best_dst = best_dst;
  g.sq = x_sqnorm ? x_sqnorm : sq_ws; g.sq_out = sq_ws;
  g.reset_keys = 1;
  g.mt2 = g.nt2 = (max_window + T2_TM - 1) / T2_TM;
  hipError_t e;
  if (!x_sqnorm) hipLaunchKernelGGL(row_norms_kernel, dim3((unsigned)((sum_n + 3) / 4)), dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(reset_keys_kernel, dim3((unsigned)((sum_n + 255) / 256)), dim3(256), 0, stream, g);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  constexpr size_t lds = (size_t)2 * T2_STAGE;   // 108 KB
  e = allow_big_lds(1, reinterpret_cast<const void *>(fd_pair_kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fd_pair_kernel, dim3(t2_grid(n_windows, g.mt2, g.nt2)), dim3(BIG_THREADS), lds, stream, g);
  e = hipGetLastError();
  if (e != hipSuccess || !best_fd) return e;   // without outputs of its own the caller's selection reads the keys
  const int cpw = max_window > 256 ? (max_window + 255) / 256 : 1;
  hipLaunchKernelGGL(fd_pair_finalize_kernel, dim3((unsigned)(n_windows * cpw)), dim3(256), 0, stream, g, cpw);
  return hipGetLastError();
}

}  // namespace lk
