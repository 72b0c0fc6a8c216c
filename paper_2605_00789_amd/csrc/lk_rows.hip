// Message passing (paper Sec. 3.2.1 Step 3, Eq. "message-passing") and delete + reorder (Steps 4-5)
// on the row tensors X, K, V.  Pure HBM streaming: one wave per (token, tensor) row, 16-byte
// loads and stores, fp32 arithmetic, round-to-nearest-even on store.
//
// A token b with sources a_1..a_m becomes  y_b + sum_a w_a (y_a - y_b),  w_a = xi_a / (xi_b + sum xi_a),
// which equals the xi-weighted mean of the equation and returns y_b bit for bit when all rows are equal.
// Sources are visited in ascending token order (grp_src), so results are reproducible run to run.
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {

constexpr int ROW_THREADS = 256;

struct RowArgs {
  RowTensors t;
  const int32_t *new_index, *grp_offsets, *grp_src, *pos;
  int32_t *pos_out;
  float *x_sqnorm_out;   // optional: |x|^2 of every output row of tensor 0 (as stored), fp32
  const float *xi;
  int d, sum_n, mode;
  int64_t out_rows;   // capacity of the compacted outputs; rows beyond it are dropped
};

template <typename T> struct RowIO;
template <> struct RowIO<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4 &v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
    uint4 v;
    v.x = f32_to_bf16_rne(f[0]) | (f32_to_bf16_rne(f[1]) << 16);
    v.y = f32_to_bf16_rne(f[2]) | (f32_to_bf16_rne(f[3]) << 16);
    v.z = f32_to_bf16_rne(f[4]) | (f32_to_bf16_rne(f[5]) << 16);
    v.w = f32_to_bf16_rne(f[6]) | (f32_to_bf16_rne(f[7]) << 16);
    return v;
  }
};
template <> struct RowIO<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4 &v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};

// One wave = one row of one tensor (4 rows per workgroup).  Index loads go out together, then the whole row
// (8 x 16 bytes per lane for an 8 KB row) is in flight before anything is consumed; all loads are
// unconditional (clamped addresses) so that the compiler never has to wait inside a branch.
constexpr int ROWS_PER_WG = ROW_THREADS / WAVE;
constexpr int ROW_UNROLL = 8;   // 16-byte chunks per lane and pass
constexpr int64_t ROWS_STREAM_OUT_BYTES = 128ll << 20;   // inputs beyond this: nontemporal output stores

// MODE 0: aggregate in place   1: compact   2: aggregate + compact
//
// Dependent loads are what this kernel waits for, so they are arranged in as few rounds as possible:
//   round 1  the row itself, xi of the row, new_index and the group bounds (all depend on the row number only)
//   round 2  the source list of the group
//   round 3  xi of the sources and the rows of the first two sources, together
// A row without sources is stored after round 1.  Third and later sources of a group (rare) are fetched one by one.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// STREAM: the output rows are stored nontemporally (a template parameter: as a run-time choice between two stores of
// the same value the compiler merges them into one plain store)
template <typename T, int MODE, bool STREAM>
__global__ __launch_bounds__(ROW_THREADS) void rows_kernel(RowArgs g) {
  using IO = RowIO<T>;
  constexpr int N = IO::N;
  constexpr int BYTES = Elem<T>::BYTES;
  constexpr int HU = ROW_UNROLL / 2;
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
  const int which = blockIdx.y;
  if (b >= g.sum_n) return;
  const char *in = static_cast<const char *>(g.t.in[which]);
  char *out = static_cast<char *>(g.t.out[which]);
  const int64_t ld_in = g.t.ld_in[which] * BYTES;
  const int n_chunks = g.d / N;
  const bool single_pass = n_chunks <= WAVE * ROW_UNROLL;

  // round 1 (the in-place mode touches few rows: it looks at the group bounds first instead of fetching every row)
  uint4 v[ROW_UNROLL];
  const char *row_in = in ? in + (int64_t)b * ld_in : nullptr;
  if (MODE == 0 && g.grp_offsets[b + 1] == g.grp_offsets[b]) return;
  // A row that is merged away is fetched by its own wave as well as by its target's (8-11 % more bytes read): looking
  // at new_index first would save those bytes but puts one more dependent load in front of every row, and the longer
  // life of every wave costs more than the bytes (single launch on 2880 tokens: 26.8 -> 23.9 us without the look).
  // Large outputs are stored nontemporally: they cannot stay cached until the next stage reads them, and kept out of
  // the caches they leave them to the kernels that run next (batch of 16: step -3.6 %; on the cache-resident sizes the
  // same stores cost +2.4 %: the next stage's kernels then find their inputs in HBM).
  if (in != nullptr) {
#pragma unroll
    for (int u = 0; u < ROW_UNROLL; ++u) {
      const int c = u * WAVE + lane;
      v[u] = ld16(row_in + (int64_t)(c < n_chunks ? c : n_chunks - 1) * 16);
    }
  }
  float xb = 0.f;
  if (MODE != 1) xb = g.xi[b];
  int out_row = b, s0 = 0, s1 = 0;
  if (MODE != 0) out_row = g.new_index[b];
  if (MODE != 1) { s0 = g.grp_offsets[b]; s1 = g.grp_offsets[b + 1]; }
  const int m = s1 - s0;
  if (MODE != 0 && (out_row < 0 || out_row >= g.out_rows)) return;   // merged away, or no room in the output
  if (MODE == 0 && m == 0) return;                                    // in place: nothing to do for this row
  if (MODE != 0 && which == 0 && lane == 0 && g.pos && g.pos_out) g.pos_out[out_row] = g.pos[b];
  if (in == nullptr) return;
  char *row_out = out + (int64_t)out_row * g.t.ld_out[which] * BYTES;

  // rounds 2 and 3: lane s holds source s and its weight (groups beyond 64 sources take the slow loop)
  int a_l = b;
  float w_l = 0.f;
  const char *row_a0 = row_in, *row_a1 = row_in;
  if (MODE != 1 && m > 0) {
    const int mm = m < WAVE ? m : WAVE;
    a_l = g.grp_src[s0 + (lane < mm ? lane : mm - 1)];
    row_a0 = in + (int64_t)__shfl(a_l, 0, 64) * ld_in;
    row_a1 = in + (int64_t)__shfl(a_l, mm > 1 ? 1 : 0, 64) * ld_in;
  }

  // |x|^2 of the row as it is stored (tensor 0 only, on request): the next stage's feature divergence wants it, and
  // here the row is in registers anyway.  Same order of summation as the stand-alone pass over X.
  const bool want_sq = MODE != 0 && which == 0 && g.x_sqnorm_out != nullptr;
  float sq = 0.f;
  for (int c0 = 0; c0 < n_chunks; c0 += WAVE * ROW_UNROLL) {
    if (c0 > 0) {   // rows longer than one pass: later passes reload
#pragma unroll
      for (int u = 0; u < ROW_UNROLL; ++u) {
        const int c = c0 + u * WAVE + lane;
        v[u] = ld16(row_in + (int64_t)(c < n_chunks ? c : n_chunks - 1) * 16);
      }
    }
    if (MODE != 1 && m > 0) {
      // first half of the pass: its source chunks go out together with the xi loads below
      uint4 va0[HU], va1[HU];
#pragma unroll
      for (int u = 0; u < HU; ++u) {
        const int c = c0 + u * WAVE + lane;
        const int64_t o = (int64_t)(c < n_chunks ? c : n_chunks - 1) * 16;
        va0[u] = ld16(row_a0 + o);
        va1[u] = ld16(row_a1 + o);
      }
      if (c0 == 0) {
        const int mm = m < WAVE ? m : WAVE;
        float x_l = g.xi[a_l];
        x_l = lane < mm ? x_l : 0.f;
        float den = x_l;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) den += __shfl_xor(den, o, 64);   // fixed butterfly: reproducible
        den += xb;
        for (int s = s0 + WAVE; s < s1; ++s) den += g.xi[g.grp_src[s]];
        w_l = x_l / den;
        if (m > WAVE) w_l = 1.f / den;   // slow path keeps 1/den instead
      }
      const float w0 = (m <= WAVE) ? __shfl(w_l, 0, 64) : g.xi[__shfl(a_l, 0, 64)] * __shfl(w_l, 0, 64);
      const float w1 = (m <= 1) ? 0.f : ((m <= WAVE) ? __shfl(w_l, 1, 64) : g.xi[g.grp_src[s0 + 1]] * __shfl(w_l, 0, 64));
#pragma unroll
      for (int hb = 0; hb < ROW_UNROLL; hb += HU) {
        if (hb > 0) {
#pragma unroll
          for (int u = 0; u < HU; ++u) {
            const int c = c0 + (hb + u) * WAVE + lane;
            const int64_t o = (int64_t)(c < n_chunks ? c : n_chunks - 1) * 16;
            va0[u] = ld16(row_a0 + o);
            va1[u] = ld16(row_a1 + o);
          }
        }
        float acc[HU][N];   // y_b stays packed in v[] and is unpacked where it is used
#pragma unroll
        for (int u = 0; u < HU; ++u) {
          float y0[N], y1[N], yb[N];
          IO::unpack(v[hb + u], yb);
          IO::unpack(va0[u], y0);
          IO::unpack(va1[u], y1);
#pragma unroll
          for (int e = 0; e < N; ++e) acc[u][e] = fmaf(w1, y1[e] - yb[e], fmaf(w0, y0[e] - yb[e], yb[e]));
        }
        for (int s = 2; s < m; ++s) {   // third and later sources
          int a;
          float w;
          if (m <= WAVE) {
            a = __shfl(a_l, s, 64);
            w = __shfl(w_l, s, 64);
          } else {
            a = g.grp_src[s0 + s];
            w = g.xi[a] * __shfl(w_l, 0, 64);
          }
          const char *row_a = in + (int64_t)a * ld_in;
          uint4 va[HU];
#pragma unroll
          for (int u = 0; u < HU; ++u) {
            const int c = c0 + (hb + u) * WAVE + lane;
            va[u] = ld16(row_a + (int64_t)(c < n_chunks ? c : n_chunks - 1) * 16);
          }
#pragma unroll
          for (int u = 0; u < HU; ++u) {
            float ya[N], yb[N];
            IO::unpack(va[u], ya);
            IO::unpack(v[hb + u], yb);
#pragma unroll
            for (int e = 0; e < N; ++e) acc[u][e] = fmaf(w, ya[e] - yb[e], acc[u][e]);
          }
        }
#pragma unroll
        for (int u = 0; u < HU; ++u) v[hb + u] = IO::pack(acc[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < ROW_UNROLL; ++u) {
      const int c = c0 + u * WAVE + lane;
      if (c < n_chunks) {
        u32x4 *dst = reinterpret_cast<u32x4 *>(row_out + (int64_t)c * 16);
        const u32x4 t4 = {v[u].x, v[u].y, v[u].z, v[u].w};
        if (STREAM) __builtin_nontemporal_store(t4, dst);
        else *dst = t4;
      }
    }
    if (want_sq) {
#pragma unroll
      for (int u = 0; u < ROW_UNROLL; ++u) {
        const int c = c0 + u * WAVE + lane;
        const float t = BYTES == 2 ? sumsq_chunk_bf16(v[u]) : sumsq_chunk_f32(v[u]);
        sq += (c < n_chunks) ? t : 0.f;
      }
    }
  }
  if (want_sq) {
    sq = wave_sum_butterfly(sq);
    if (lane == 0) g.x_sqnorm_out[out_row] = sq;
  }
  (void)single_pass;
}

// Rows that trail the vision span in the caller's tensors (the prompt's text behind the image, Steps 4-5: the sequence
// is rebuilt behind the shorter vision span): row sum_n + j of the input moves to row n' + j of the output, n' being
// the number of vision rows that stay, read from the device (cu_vis_out[batch]).  One wave per (row, tensor).
struct TailArgs {
  RowTensors t;
  const int32_t *pos, *cu_vis_out;
  int32_t *pos_out;
  int d, sum_n, batch, elem_bytes;
  int64_t tail_rows, out_rows;
};

__global__ __launch_bounds__(ROW_THREADS) void tail_rows_kernel(TailArgs g) {
  const int lane = threadIdx.x & 63;
  const int64_t j = (int64_t)blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
  const int which = blockIdx.y;
  if (j >= g.tail_rows) return;
  int n_keep = g.cu_vis_out[g.batch];
  n_keep = n_keep < 0 ? 0 : (n_keep > g.sum_n ? g.sum_n : n_keep);
  const int64_t out_row = (int64_t)n_keep + j;
  if (out_row >= g.out_rows) return;   // no room in the output: dropped, never written out of bounds
  if (which == 0 && lane == 0 && g.pos && g.pos_out) g.pos_out[out_row] = g.pos[g.sum_n + j];
  const char *in = static_cast<const char *>(g.t.in[which]);
  char *out = static_cast<char *>(g.t.out[which]);
  if (!in) return;
  const char *row_in = in + ((int64_t)g.sum_n + j) * g.t.ld_in[which] * g.elem_bytes;
  char *row_out = out + out_row * g.t.ld_out[which] * g.elem_bytes;
  const int n_chunks = g.d * g.elem_bytes / 16;
  for (int c0 = 0; c0 < n_chunks; c0 += WAVE * ROW_UNROLL) {
    uint4 v[ROW_UNROLL];
#pragma unroll
    for (int u = 0; u < ROW_UNROLL; ++u) {
      const int c = c0 + u * WAVE + lane;
      v[u] = ld16(row_in + (int64_t)(c < n_chunks ? c : n_chunks - 1) * 16);
    }
#pragma unroll
    for (int u = 0; u < ROW_UNROLL; ++u) {
      const int c = c0 + u * WAVE + lane;
      if (c < n_chunks) *reinterpret_cast<uint4 *>(row_out + (int64_t)c * 16) = v[u];
    }
  }
}

hipError_t launch_tail_rows(int dtype, int d, int sum_n, int batch, const RowTensors &t, const int32_t *pos,
                            int32_t *pos_out, const int32_t *cu_vis_out, int64_t tail_rows, int64_t out_rows,
                            hipStream_t stream) {
  if (tail_rows <= 0) return hipSuccess;
  TailArgs g{};
  g.t = t; g.pos = pos; g.pos_out = pos_out; g.cu_vis_out = cu_vis_out; g.d = d; g.sum_n = sum_n; g.batch = batch;
  g.elem_bytes = dtype == 1 ? 2 : 4; g.tail_rows = tail_rows; g.out_rows = out_rows;
  const dim3 grid((unsigned)((tail_rows + ROWS_PER_WG - 1) / ROWS_PER_WG), 3);
  hipLaunchKernelGGL(tail_rows_kernel, grid, dim3(ROW_THREADS), 0, stream, g);
  return hipGetLastError();
}

hipError_t launch_rows(int mode, int dtype, int d, int sum_n, const RowTensors &t, const int32_t *new_index,
                       const int32_t *grp_offsets, const int32_t *grp_src, const float *xi, const int32_t *pos,
                       int32_t *pos_out, float *x_sqnorm_out, int64_t out_rows, hipStream_t stream) {
  if (sum_n == 0) return hipSuccess;
  RowArgs g{};
  g.x_sqnorm_out = x_sqnorm_out;
  g.t = t; g.new_index = new_index; g.grp_offsets = grp_offsets; g.grp_src = grp_src; g.pos = pos;
  g.pos_out = pos_out; g.xi = xi; g.d = d; g.sum_n = sum_n; g.mode = mode; g.out_rows = out_rows;
  int n_tensors = 0;
  for (int i = 0; i < 3; ++i) n_tensors += t.in[i] != nullptr;
  // nontemporal output stores once the tensors are far beyond what stays cached until the next stage reads them
  const bool stream_out = mode != 0 && (int64_t)sum_n * d * (dtype == 1 ? 2 : 4) * n_tensors > ROWS_STREAM_OUT_BYTES;
  const dim3 grid((unsigned)((sum_n + ROWS_PER_WG - 1) / ROWS_PER_WG), 3);
#define LK_ROWS(TT)                                                                                                \
  do {                                                                                                             \
    if (mode == 0) hipLaunchKernelGGL((rows_kernel<TT, 0, false>), grid, dim3(ROW_THREADS), 0, stream, g);        \
    else if (mode == 1 && stream_out) hipLaunchKernelGGL((rows_kernel<TT, 1, true>), grid, dim3(ROW_THREADS), 0, stream, g);  \
    else if (mode == 1) hipLaunchKernelGGL((rows_kernel<TT, 1, false>), grid, dim3(ROW_THREADS), 0, stream, g);   \
    else if (stream_out) hipLaunchKernelGGL((rows_kernel<TT, 2, true>), grid, dim3(ROW_THREADS), 0, stream, g);   \
    else hipLaunchKernelGGL((rows_kernel<TT, 2, false>), grid, dim3(ROW_THREADS), 0, stream, g);                  \
  } while (0)
  if (dtype == 1) LK_ROWS(bf16_t);
  else LK_ROWS(float);
#undef LK_ROWS
  return hipGetLastError();
}

}  // namespace lk
