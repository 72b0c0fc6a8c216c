// Message passing (paper Sec. 3.2.1 Step 3, Eq. "message-passing") and delete + reorder (Steps 4-5)
// on the row tensors X, K, V.  Pure HBM streaming: one workgroup per (token, tensor) row, 16-byte
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

template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void rows_kernel(RowArgs g) {
  using IO = RowIO<T>;
  constexpr int N = IO::N;
  constexpr int BYTES = Elem<T>::BYTES;
  const int b = blockIdx.x;
  const int which = blockIdx.y;
  const char *in = static_cast<const char *>(g.t.in[which]);
  char *out = static_cast<char *>(g.t.out[which]);

  int out_row = b;
  if (g.mode != 0) {
    out_row = g.new_index[b];
    if (out_row < 0 || out_row >= g.out_rows) return;   // merged away (or no room: the caller under-sized the output)
    if (which == 0 && threadIdx.x == 0 && g.pos && g.pos_out) g.pos_out[out_row] = g.pos[b];
  }
  if (in == nullptr) return;
  int s0 = 0, s1 = 0;
  if (g.mode != 1) { s0 = g.grp_offsets[b]; s1 = g.grp_offsets[b + 1]; }
  const int m = s1 - s0;
  if (g.mode == 0 && m == 0) return;   // in place: rows without sources are left alone

  const char *row_in = in + (int64_t)b * g.t.ld_in[which] * BYTES;
  char *row_out = out + (int64_t)out_row * g.t.ld_out[which] * BYTES;
  const int n_chunks = g.d / N;

  if (m == 0) {
    for (int c = threadIdx.x; c < n_chunks; c += ROW_THREADS)
      *reinterpret_cast<uint4 *>(row_out + (int64_t)c * 16) = ld16(row_in + (int64_t)c * 16);
    return;
  }

  // weights
  float den = g.xi[b];
  for (int s = s0; s < s1; ++s) den += g.xi[g.grp_src[s]];
  const float inv = 1.f / den;

  for (int c = threadIdx.x; c < n_chunks; c += ROW_THREADS) {
    float yb[N], acc[N];
    IO::unpack(ld16(row_in + (int64_t)c * 16), yb);
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] = yb[e];
    for (int s = s0; s < s1; ++s) {
      const int a = g.grp_src[s];
      const float w = g.xi[a] * inv;
      float ya[N];
      IO::unpack(ld16(in + (int64_t)a * g.t.ld_in[which] * BYTES + (int64_t)c * 16), ya);
#pragma unroll
      for (int e = 0; e < N; ++e) acc[e] = fmaf(w, ya[e] - yb[e], acc[e]);
    }
    *reinterpret_cast<uint4 *>(row_out + (int64_t)c * 16) = IO::pack(acc);
  }
}

hipError_t launch_rows(int mode, int dtype, int d, int sum_n, const RowTensors &t, const int32_t *new_index,
                       const int32_t *grp_offsets, const int32_t *grp_src, const float *xi, const int32_t *pos,
                       int32_t *pos_out, int64_t out_rows, hipStream_t stream) {
  if (sum_n == 0) return hipSuccess;
  RowArgs g{};
  g.t = t; g.new_index = new_index; g.grp_offsets = grp_offsets; g.grp_src = grp_src; g.pos = pos;
  g.pos_out = pos_out; g.xi = xi; g.d = d; g.sum_n = sum_n; g.mode = mode; g.out_rows = out_rows;
  const dim3 grid((unsigned)sum_n, 3);
  if (dtype == 1) hipLaunchKernelGGL(rows_kernel<bf16_t>, grid, dim3(ROW_THREADS), 0, stream, g);
  else hipLaunchKernelGGL(rows_kernel<float>, grid, dim3(ROW_THREADS), 0, stream, g);
  return hipGetLastError();
}

}  // namespace lk
