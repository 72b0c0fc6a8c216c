// Device-side bodies of the xi kernels (paper Sec. 3.2.1 Step 3, Eq. "attention-factor").  They take the workgroup
// index and a block of LDS as arguments so that a launch can run them next to the bodies of another step
// (lk_fused.hip) as well as on their own (lk_score_xi.hip, where the algorithm is described).
#pragma once
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {


constexpr int XI_THREADS = 256;
constexpr float XI_FLOOR = 1e-30f;
constexpr float LOG2E = 1.4426950408889634f;

// 2^x on the hardware unit directly (v_exp_f32).  The library routine wraps it in a range reduction that keeps denormal
// results; a probability below 2^-126 is zero for every purpose here, and the wrapper is five more instructions on each
// of the H*T*N exponentials.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct XiArgs {
  const void *vis, *txt;                 // vision-side and prompt-side tensors of the contraction
  int64_t vis_ts, vis_hs, txt_ts, txt_hs;   // token / head strides in elements
  const int32_t *cu_vis, *cu_txt;
  const float *lse;                      // optional, natural log
  float scale_log2;                      // softmax scale * log2(e)
  float *stats;                          // [heads][sum_t][max_vis_blocks][2]  (max, sum) in the exp2 domain
  float *xi_part;                        // [heads][sum_n]
  float *xi;                             // [sum_n]
  int batch, heads, sum_n, sum_t, max_text_tiles, max_vis_blocks;
  int lse_per_vision;                    // 1: lse indexed [h][vision token] (vision-query mode)
};

template <typename T, int DH> struct XiShape {
  using E = Elem<T>;
  static constexpr int NCH = DH / 2 / E::PER_CHUNK;   // 16-byte chunks per lane: half a head row
};

// Loads half a head row of token (first + min(idx, count - 1)): always a valid address, never a branch, so
// the loads of a whole tile are in flight together.  Rows past `count` repeat the last one; callers mask them.
template <typename T, int DH>
__device__ __forceinline__ void load_half_row(const void *base, int first, int idx, int count, int64_t tok_stride,
                                              int64_t head_off, int half, uint4 *v) {
  using E = Elem<T>;
  const int tok = first + (idx < count ? idx : count - 1);
  const char *p = static_cast<const char *>(base) + ((int64_t)tok * tok_stride + head_off + half * (DH / 2)) * E::BYTES;
#pragma unroll
  for (int c = 0; c < XiShape<T, DH>::NCH; ++c) v[c] = ld16(p + c * 16);
}

// Prompt rows of one head are shared by the four waves of a workgroup: they are staged through LDS once per
// workgroup (coalesced 16-byte loads, rows padded by 16 bytes so that the MFMA operand reads are conflict free)
// instead of being fetched by every wave on its own.
// RW = prompt rows per staged chunk: 64 for short prompts, 128 otherwise (half as many barrier rounds per workgroup;
// 34 KB of LDS for bf16 heads of 128, still four workgroups per CU).
template <typename T, int DH, int RW> struct XiStage {
  static constexpr int ROW_BYTES = DH * Elem<T>::BYTES;
  static constexpr int PITCH = ROW_BYTES + 16;
  static constexpr int ROWS = RW;
  static constexpr int TILES = ROWS / 32;
  static constexpr int CPR = ROW_BYTES / 16;                // 16-byte chunks per row
  static constexpr int LDS_ROWSTAT = ROWS * PITCH + 4 * ROWS * 8;   // bytes of LDS pass 1 needs
  static constexpr int LDS_COLSUM = ROWS * PITCH + ROWS * 8;        // pass 2
};

// Copies prompt rows [j0, j0 + ROWS) of head h into LDS (rows past nT repeat the last one).
template <typename T, int DH, int RW>
__device__ __forceinline__ void stage_prompt_rows(const XiArgs &g, char *q_lds, int t0, int nT, int j0, int64_t txt_ho) {
  using S = XiStage<T, DH, RW>;
  constexpr int BYTES = Elem<T>::BYTES;
  constexpr int PER_PASS = XI_THREADS / S::CPR;             // rows covered by one pass of the workgroup
  const int c = threadIdx.x % S::CPR, r0 = threadIdx.x / S::CPR;
#pragma unroll
  for (int p = 0; p < S::ROWS / PER_PASS; ++p) {
    const int r = p * PER_PASS + r0;
    const int j = j0 + r;
    const int tok = t0 + (j < nT ? j : nT - 1);
    const uint4 v = ld16(static_cast<const char *>(g.txt) + ((int64_t)tok * g.txt_ts + txt_ho) * BYTES + c * 16);
    *reinterpret_cast<uint4 *>(q_lds + r * S::PITCH + c * 16) = v;
  }
}

// The same copy in two halves, so that other loads can be issued between the global loads and the LDS stores that wait
// for them.
template <typename T, int DH, int RW>
__device__ __forceinline__ void load_prompt_rows(const XiArgs &g, int t0, int nT, int j0, int64_t txt_ho,
                                                 uint4 (&v)[XiStage<T, DH, RW>::ROWS / (XI_THREADS / XiStage<T, DH, RW>::CPR)]) {
  using S = XiStage<T, DH, RW>;
  constexpr int BYTES = Elem<T>::BYTES;
  constexpr int PER_PASS = XI_THREADS / S::CPR;
  const int c = threadIdx.x % S::CPR, r0 = threadIdx.x / S::CPR;
#pragma unroll
  for (int p = 0; p < S::ROWS / PER_PASS; ++p) {
    const int j = j0 + p * PER_PASS + r0;
    const int tok = t0 + (j < nT ? j : nT - 1);
    v[p] = ld16(static_cast<const char *>(g.txt) + ((int64_t)tok * g.txt_ts + txt_ho) * BYTES + c * 16);
  }
}
template <typename T, int DH, int RW>
__device__ __forceinline__ void store_prompt_rows(char *q_lds,
                                                  const uint4 (&v)[XiStage<T, DH, RW>::ROWS / (XI_THREADS / XiStage<T, DH, RW>::CPR)]) {
  using S = XiStage<T, DH, RW>;
  constexpr int PER_PASS = XI_THREADS / S::CPR;
  const int c = threadIdx.x % S::CPR, r0 = threadIdx.x / S::CPR;
#pragma unroll
  for (int p = 0; p < S::ROWS / PER_PASS; ++p)
    *reinterpret_cast<uint4 *>(q_lds + (p * PER_PASS + r0) * S::PITCH + c * 16) = v[p];
}

template <typename T, int DH>
__device__ __forceinline__ void read_prompt_frag(const char *q_lds, int row, int half, uint4 *v) {
  using S = XiStage<T, DH, 64>;   // pitch and row size do not depend on the chunk length
  const char *p = q_lds + row * S::PITCH + half * (S::ROW_BYTES / 2);
#pragma unroll
  for (int c = 0; c < XiShape<T, DH>::NCH; ++c) v[c] = *reinterpret_cast<const uint4 *>(p + c * 16);
}

// ---- pass 1: (max, sum of exponentials) of every prompt row over one block of 128 vision keys ----------
// Workgroup = (sequence, head, vision block); wave w owns the 32 vision tokens blk*128 + w*32 .. +32 and keeps
// their key rows in registers as the MFMA row operand; the prompt rows come from LDS as the column operand.
template <typename T, int DH, int RW>
__device__ __forceinline__ void xi_rowstat_body(const XiArgs &g, int block_id, char *lds) {
  using E = Elem<T>;
  using S = XiStage<T, DH, RW>;
  constexpr int NCH = XiShape<T, DH>::NCH;
  char *q_lds = lds;                                                     // [ROWS * PITCH]
  float2 (*part)[S::ROWS] = reinterpret_cast<float2 (*)[S::ROWS]>(lds + S::ROWS * S::PITCH);   // [4][ROWS]

  int id = block_id;
  const int blk = id % g.max_vis_blocks; id /= g.max_vis_blocks;
  const int h = id % g.heads;
  const int b = id / g.heads;
  const int t0 = g.cu_txt[b], nT = g.cu_txt[b + 1] - t0;
  const int v0 = g.cu_vis[b], nV = g.cu_vis[b + 1] - v0;
  if (blk * 128 >= nV || nT == 0) return;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, half = lane >> 5;
  const float NEG_INF = __uint_as_float(0xff800000u);
  const int vt = blk * 4 + wave;
  const int64_t vis_ho = (int64_t)h * g.vis_hs, txt_ho = (int64_t)h * g.txt_hs;

  uint4 k[NCH];
  load_half_row<T, DH>(g.vis, v0, vt * 32 + r, nV, g.vis_ts, vis_ho, half, k);
  bool row_ok[16];
#pragma unroll
  for (int x = 0; x < 16; ++x) row_ok[x] = (vt * 32 + acc_row(x, lane)) < nV;
  const bool partial_block = blk * 128 + 128 > nV;          // uniform: only the last block of a sequence masks rows
  const bool neg_scale = g.scale_log2 < 0.f;
  const float pad = neg_scale ? __uint_as_float(0x7f800000u) : NEG_INF;   // product whose logit is -inf

  for (int j0 = 0; j0 < nT; j0 += S::ROWS) {
    __syncthreads();   // the previous chunk has been consumed
    stage_prompt_rows<T, DH, RW>(g, q_lds, t0, nT, j0, txt_ho);
    __syncthreads();
    const int n_tt = min(S::TILES, (nT - j0 + 31) >> 5);
    for (int tt = 0; tt < n_tt; ++tt) {
      uint4 q[NCH];
      read_prompt_frag<T, DH>(q_lds, tt * 32 + r, half, q);
      f32x16 acc = {0};
#pragma unroll
      for (int c = 0; c < NCH; ++c) E::mma32(k[c], q[c], acc);   // rows: vision tokens, cols: prompt rows
      // logits are acc * scale_log2; the extreme is taken on the raw products (maximum for a positive scale, minimum
      // for a negative one), the scale goes into the exponent's multiply-add
      if (partial_block) {
#pragma unroll
        for (int x = 0; x < 16; ++x) acc[x] = row_ok[x] ? acc[x] : pad;
      }
      float e = acc[0];
#pragma unroll
      for (int x = 1; x < 16; ++x) e = neg_scale ? fminf(e, acc[x]) : fmaxf(e, acc[x]);
      const float eo = __shfl_xor(e, 32, 64);   // both half-waves hold rows of the same column
      e = neg_scale ? fminf(e, eo) : fmaxf(e, eo);
      const float m = e * g.scale_log2;
      float s = 0.f;
#pragma unroll
      for (int x = 0; x < 16; ++x) s += fast_exp2(fmaf(acc[x], g.scale_log2, -m));   // padded rows: exp2(-inf) = 0
      s = (m > NEG_INF) ? s : 0.f;              // a tile of padded rows only: (-inf, 0), as the merge expects
      s += __shfl_xor(s, 32, 64);
      if (half == 0) part[wave][tt * 32 + r] = make_float2(m, s);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < n_tt * 32; idx += XI_THREADS) {
      const int j = j0 + idx;
      if (j < nT) {
        float m = NEG_INF;
#pragma unroll
        for (int w = 0; w < 4; ++w) m = fmaxf(m, part[w][idx].x);
        float s = 0.f;
        if (m > NEG_INF) {
#pragma unroll
          for (int w = 0; w < 4; ++w) s += part[w][idx].y * exp2f(part[w][idx].x - m);
        }
        reinterpret_cast<float2 *>(g.stats)[((int64_t)h * g.sum_t + t0 + j) * g.max_vis_blocks + blk] = make_float2(m, s);
      }
    }
  }
}

// ---- pass 2: column sums of exp(logit - lse) over the prompt rows -----------------------------------
// Same decomposition; the key rows of the wave's 32 vision tokens are now the MFMA column operand, so the sum
// over prompt rows runs over accumulator registers.
template <typename T, int DH, int RW, bool VISION_LSE>
__device__ __forceinline__ void xi_colsum_body(const XiArgs &g, int block_id, char *lds) {
  using E = Elem<T>;
  using S = XiStage<T, DH, RW>;
  constexpr int NCH = XiShape<T, DH>::NCH;
  char *q_lds = lds;                                                     // [ROWS * PITCH]
  float2 *rowstat = reinterpret_cast<float2 *>(lds + S::ROWS * S::PITCH);   // [ROWS] (max in exp2 domain, 1/sum)

  int id = block_id;
  const int blk = id % g.max_vis_blocks; id /= g.max_vis_blocks;
  const int h = id % g.heads;
  const int b = id / g.heads;
  const int t0 = g.cu_txt[b], nT = g.cu_txt[b + 1] - t0;
  const int v0 = g.cu_vis[b], nV = g.cu_vis[b + 1] - v0;
  if (blk * 128 >= nV) return;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, half = lane >> 5;
  const float NEG_INF = __uint_as_float(0xff800000u);

  const int i = blk * 128 + wave * 32 + r;   // vision token of this lane's column
  if (nT == 0) {   // no prompt tokens: xi is zero before the floor
    if (half == 0 && i < nV) g.xi_part[(int64_t)h * g.sum_n + v0 + i] = 0.f;
    return;
  }
  const int64_t vis_ho = (int64_t)h * g.vis_hs, txt_ho = (int64_t)h * g.txt_hs;
  uint4 k[NCH];
  load_half_row<T, DH>(g.vis, v0, i, nV, g.vis_ts, vis_ho, half, k);
  float col_m = 0.f;
  if (VISION_LSE) col_m = (i < nV) ? g.lse[(int64_t)h * g.sum_n + v0 + i] * LOG2E : 0.f;
  const int nblk = (nV + 127) >> 7;

  float colsum = 0.f;
  for (int j0 = 0; j0 < nT; j0 += S::ROWS) {
    __syncthreads();   // the previous chunk has been consumed
    // the prompt rows' loads go out first; the row statistics below issue their own loads behind them, and the LDS
    // stores that have to wait for the prompt rows come after both (one trip to memory instead of two in a row)
    uint4 staged[S::ROWS / (XI_THREADS / S::CPR)];
    load_prompt_rows<T, DH, RW>(g, t0, nT, j0, txt_ho, staged);
    if (VISION_LSE) store_prompt_rows<T, DH, RW>(q_lds, staged);
    if (!VISION_LSE) {
      // (max, 1/sum) of every prompt row of the chunk.  TPR threads share a row: each merges every TPR-th
      // per-block pair of pass 1 (its loads in flight together), then the partial results are merged by
      // shuffles -- a fixed order, and a dependent chain of nblk / TPR + log2(TPR) instead of nblk.
      constexpr int TPR = XI_THREADS / S::ROWS;   // threads per prompt row of a chunk: 4 or 2
      static_assert(TPR == 4 || TPR == 2, "chunk of 64 or 128 prompt rows");
      const int idx = threadIdx.x / TPR, part = threadIdx.x % TPR;
      const int j = j0 + idx;
      float m = 3.0e38f, inv = 0.f;   // rows past nT: exp2(x - huge) = 0, times 0
      if (g.lse) {
        if (j < nT) { m = g.lse[(int64_t)h * g.sum_t + t0 + j] * LOG2E; inv = 1.f; }
      } else {
        const float2 *p = reinterpret_cast<const float2 *>(g.stats) +
                          ((int64_t)h * g.sum_t + t0 + (j < nT ? j : nT - 1)) * g.max_vis_blocks;
        float pm = NEG_INF, psum = 0.f;
        for (int s0 = 0; s0 < nblk; s0 += 8 * TPR) {   // eight pairs per thread in flight; merged in index order
          float2 a[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int sb = s0 + TPR * u + part;
            a[u] = p[sb < nblk ? sb : nblk - 1];
            if (sb >= nblk) a[u] = make_float2(NEG_INF, 0.f);
          }
          float mn = pm;
#pragma unroll
          for (int u = 0; u < 8; ++u) mn = fmaxf(mn, a[u].x);
          if (mn > NEG_INF) {
            float acc = psum * exp2f(pm - mn);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += a[u].y * exp2f(a[u].x - mn);   // a pair of (-inf, 0) adds 0
            psum = acc;
            pm = mn;
          }
        }
#pragma unroll
        for (int o = 1; o < TPR; o <<= 1) {   // the threads of a row are neighbouring lanes
          const float om = __shfl_xor(pm, o, 64), os = __shfl_xor(psum, o, 64);
          const float mn = fmaxf(pm, om);
          // lower lane's pair first, so that both lanes of a pair compute the same bits
          const float lo_m = (threadIdx.x & o) ? om : pm, lo_s = (threadIdx.x & o) ? os : psum;
          const float hi_m = (threadIdx.x & o) ? pm : om, hi_s = (threadIdx.x & o) ? psum : os;
          psum = (mn > NEG_INF) ? lo_s * exp2f(lo_m - mn) + hi_s * exp2f(hi_m - mn) : 0.f;
          pm = mn;
        }
        if (j < nT) { m = pm; inv = 1.f / psum; }
      }
      store_prompt_rows<T, DH, RW>(q_lds, staged);
      if (part == 0) rowstat[idx] = make_float2(m, inv);   // rows past nT get weight 0
    }
    __syncthreads();
    const int n_tt = min(S::TILES, (nT - j0 + 31) >> 5);
    for (int tt = 0; tt < n_tt; ++tt) {
      uint4 q[NCH];
      read_prompt_frag<T, DH>(q_lds, tt * 32 + r, half, q);
      f32x16 acc = {0};
#pragma unroll
      for (int c = 0; c < NCH; ++c) E::mma32(q[c], k[c], acc);   // rows: prompt tokens, cols: vision tokens
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int row = tt * 32 + acc_row(x, lane);
        if (VISION_LSE) {
          colsum += (j0 + row < nT) ? fast_exp2(fmaf(acc[x], g.scale_log2, -col_m)) : 0.f;
        } else {
          const float2 st = rowstat[row];
          colsum = fmaf(fast_exp2(fmaf(acc[x], g.scale_log2, -st.x)), st.y, colsum);
        }
      }
    }
  }
  colsum += __shfl_xor(colsum, 32, 64);
  if (half == 0 && i < nV) g.xi_part[(int64_t)h * g.sum_n + v0 + i] = colsum;
}

// ---- pass 3: heads summed in a fixed order, floor applied ---------------------------------------------
__device__ __forceinline__ void xi_heads_body(const XiArgs &g, int i) {
  if (i >= g.sum_n) return;
  float s = 0.f;
  int h = 0;
  for (; h + 8 <= g.heads; h += 8) {   // eight loads in flight, summed in head order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = g.xi_part[(int64_t)(h + u) * g.sum_n + i];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; h < g.heads; ++h) s += g.xi_part[(int64_t)h * g.sum_n + i];
  g.xi[i] = fmaxf(s, XI_FLOOR);
}


// Arguments of the three passes from the caller's tensors (host side).
inline XiArgs make_xi_args(const XiPlan &plan, int xi_mode, int batch, int heads, int sum_n, int sum_t,
                           const int32_t *cu_vis, const int32_t *cu_txt, const void *Q, int64_t q_tok_stride,
                           int64_t q_head_stride, const void *K, int64_t k_tok_stride, int64_t k_head_stride,
                           const float *lse, float scale, float *stats, float *xi_part, float *xi) {
  XiArgs g{};
  if (xi_mode == 0) {   // prompt queries against vision keys
    g.vis = K; g.vis_ts = k_tok_stride; g.vis_hs = k_head_stride;
    g.txt = Q; g.txt_ts = q_tok_stride; g.txt_hs = q_head_stride;
  } else {              // vision queries against prompt keys
    g.vis = Q; g.vis_ts = q_tok_stride; g.vis_hs = q_head_stride;
    g.txt = K; g.txt_ts = k_tok_stride; g.txt_hs = k_head_stride;
  }
  g.cu_vis = cu_vis; g.cu_txt = cu_txt; g.lse = lse;
  g.scale_log2 = scale * LOG2E;
  g.stats = stats; g.xi_part = xi_part; g.xi = xi;
  g.batch = batch; g.heads = heads; g.sum_n = sum_n; g.sum_t = sum_t;
  g.max_text_tiles = plan.max_text_tiles; g.max_vis_blocks = plan.max_vis_blocks;
  g.lse_per_vision = (xi_mode == 1);
  return g;
}

// Prompt chunks of 128 rows for longer prompts, where the layout fits the LDS budget of four workgroups per CU
// (fp32 heads of 128 would need 67 KB: they keep the short chunk, and the long variant is never instantiated).
template <typename T, int DH> constexpr bool xi_long_chunks_fit() { return XiStage<T, DH, 128>::PITCH * 128 <= 40 * 1024; }

}  // namespace lk
