// Debug output of lightkv_score: the feature divergence of EVERY pair of every window (paper Sec. 3.2.1, Eq.
// "similarity"; the distances of the appendix ablation alike), as concatenated row-major |A_w| x |B_w| blocks in
// window order.  The scoring kernels never write these values -- they keep row minima only -- so the dump is computed
// here by a plain kernel of its own: one thread per pair, inner product and squared norms accumulated in fp64 over
// the hidden axis in index order, the same finishing formula, rounded to fp32 once.  It is a reference to debug
// against: it agrees with best_fd to the accuracy of the fp32 accumulation of the scoring kernels (about 1e-6), not
// bit for bit.  Speed does not matter here.
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {

struct DumpArgs {
  const void *X;
  int64_t ldx;
  int d, n_windows, sum_n, metric, dir, tiles_b;
  const int32_t *win_offsets, *win_tokens;
  float *out;
  long long capacity;   // floats the caller's buffer holds
};

template <typename T>
__global__ __launch_bounds__(256) void fd_dump_kernel(DumpArgs g) {
  __shared__ long long part[256];
  const int w = blockIdx.z;
  const int off = g.win_offsets[w];
  const int v = g.win_offsets[w + 1] - off;
  const int nA = side_a(v, g.dir), nB = side_b(v, g.dir);
  const int a0 = blockIdx.y * 16, b0 = blockIdx.x * 16;
  if (a0 >= nA || b0 >= nB) return;   // uniform
  // where this window's block starts: the pairs of the windows before it
  long long mine = 0;
  for (int u = threadIdx.x; u < w; u += 256) {
    const long long vu = g.win_offsets[u + 1] - g.win_offsets[u];
    mine += ((vu + 1) / 2) * (vu / 2);
  }
  part[threadIdx.x] = mine;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  const long long base = part[0];
  const int la = a0 + (int)(threadIdx.x >> 4), lb = b0 + (int)(threadIdx.x & 15);
  if (la >= nA || lb >= nB) return;
  const int ta = g.win_tokens[off + pos_a(la, g.dir)], tb = g.win_tokens[off + pos_b(lb, g.dir)];
  const long long idx = base + (long long)la * nB + lb;
  if (idx >= g.capacity) return;
  if ((unsigned)ta >= (unsigned)g.sum_n || (unsigned)tb >= (unsigned)g.sum_n) { g.out[idx] = __uint_as_float(0x7fc00000u); return; }
  const char *ra = static_cast<const char *>(g.X) + (int64_t)ta * g.ldx * Elem<T>::BYTES;
  const char *rb = static_cast<const char *>(g.X) + (int64_t)tb * g.ldx * Elem<T>::BYTES;
  double dot = 0.0, sa = 0.0, sb = 0.0;
  const int n_chunks = g.d / Elem<T>::PER_CHUNK;
  for (int c = 0; c < n_chunks; ++c) {
    const uint4 qa = ld16(ra + (int64_t)c * 16), qb = ld16(rb + (int64_t)c * 16);
    const uint32_t wa[4] = {qa.x, qa.y, qa.z, qa.w}, wb[4] = {qb.x, qb.y, qb.z, qb.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (Elem<T>::BYTES == 2) {
        const double a_lo = (double)__uint_as_float(wa[q] << 16), a_hi = (double)__uint_as_float(wa[q] & 0xffff0000u);
        const double b_lo = (double)__uint_as_float(wb[q] << 16), b_hi = (double)__uint_as_float(wb[q] & 0xffff0000u);
        dot = fma(a_lo, b_lo, dot); sa = fma(a_lo, a_lo, sa); sb = fma(b_lo, b_lo, sb);
        dot = fma(a_hi, b_hi, dot); sa = fma(a_hi, a_hi, sa); sb = fma(b_hi, b_hi, sb);
      } else {
        const double a = (double)__uint_as_float(wa[q]), b = (double)__uint_as_float(wb[q]);
        dot = fma(a, b, dot); sa = fma(a, a, sa); sb = fma(b, b, sb);
      }
    }
  }
  double fd;
  if (g.metric == 0) {
    fd = 1.0 - dot / (fmax(sqrt(sa), 1e-12) * fmax(sqrt(sb), 1e-12));
    fd = fd < 0.0 ? 0.0 : fd;   // (a NaN stays a NaN: fmax would drop it)
  } else {
    double d2 = sa + sb - 2.0 * dot;
    d2 = d2 < 0.0 ? 0.0 : d2;
    fd = g.metric == 1 ? sqrt(d2) : d2;
  }
  g.out[idx] = (float)fd;
}

hipError_t launch_fd_dump(int dtype, const void *X, int64_t ldx, int d, int n_windows, int max_window, int sum_n,
                          int metric, int dir, const int32_t *win_offsets, const int32_t *win_tokens, float *out,
                          long long capacity, hipStream_t stream) {
  if (n_windows == 0 || sum_n == 0 || max_window < 2) return hipSuccess;
  DumpArgs g{};
  g.X = X; g.ldx = ldx; g.d = d; g.n_windows = n_windows; g.sum_n = sum_n; g.metric = metric; g.dir = dir;
  g.win_offsets = win_offsets; g.win_tokens = win_tokens; g.out = out; g.capacity = capacity;
  const int ta = ((max_window + 1) / 2 + 15) / 16, tb = (max_window / 2 + 15) / 16;
  if (n_windows > 65535) return hipErrorInvalidValue;   // windows ride in the z dimension of the grid
  const dim3 grid((unsigned)tb, (unsigned)ta, (unsigned)n_windows);
  if (dtype == 1) hipLaunchKernelGGL(fd_dump_kernel<bf16_t>, grid, dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(fd_dump_kernel<float>, grid, dim3(256), 0, stream, g);
  return hipGetLastError();
}

}  // namespace lk
