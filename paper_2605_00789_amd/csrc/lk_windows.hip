// Window partition of the vision tokens (paper Sec. 3.2 and Sec. 3.2.2 "Window partitioning"):
// every token is assigned to a window by its cell in the original image grid, and the tokens of
// each window are listed in ascending sequence order (CSR).  One workgroup per sequence; the
// stable grouping is an LDS bitonic sort of (window id, local index) keys.
#include "lk_common.h"
#include "lk_launch.h"

namespace lk {

constexpr int WIN_THREADS = 1024;
constexpr int LOCAL_BITS = 14;   // local token index < 16384

__global__ __launch_bounds__(WIN_THREADS) void build_windows_kernel(
    const int32_t *__restrict__ cu_vis, const int32_t *__restrict__ pos, int batch, int tiles, int grid_h,
    int grid_w, int w, int win_per_seq, int32_t *__restrict__ win_offsets, int32_t *__restrict__ win_tokens) {
  extern __shared__ uint32_t keys[];
  const int b = blockIdx.x;
  const int base = cu_vis[b];
  const int n = cu_vis[b + 1] - base;
  const int wbase = b * win_per_seq;
  const int p2 = next_pow2(n > 1 ? n : 1);
  const int cells = grid_h * grid_w;
  for (int i = threadIdx.x; i < p2; i += blockDim.x) {
    uint32_t key = 0xffffffffu;
    if (i < n) {
      int wid = 0;
      if (w > 0) {
        int p = pos[base + i];
        p = p < 0 ? 0 : p;
        int tile = p / cells;
        int cell = p - tile * cells;
        tile = tile >= tiles ? tiles - 1 : tile;
        int row = cell / grid_w;
        int col = cell - row * grid_w;
        row = row >= grid_h ? grid_h - 1 : row;
        wid = tile * w * w + (row * w / grid_h) * w + (col * w / grid_w);
      }
      key = ((uint32_t)wid << LOCAL_BITS) | (uint32_t)i;
    }
    keys[i] = key;
  }
  bitonic_sort_lds(keys, p2);
  // sorted position k holds the k-th token of the window-major order
  for (int k = threadIdx.x; k <= n; k += blockDim.x) {
    const int prev = (k == 0) ? -1 : (int)(keys[k - 1] >> LOCAL_BITS);
    int cur;
    if (k < n) {
      cur = (int)(keys[k] >> LOCAL_BITS);
      win_tokens[base + k] = base + (int)(keys[k] & ((1u << LOCAL_BITS) - 1u));
    } else {
      cur = (b == batch - 1) ? win_per_seq : win_per_seq - 1;   // the next sequence writes its own first offset
    }
    for (int id = prev + 1; id <= cur; ++id) win_offsets[wbase + id] = base + k;
  }
}

hipError_t launch_build_windows(const int32_t *cu_vis, const int32_t *pos, int batch, int max_seq, int tiles,
                                int grid_h, int grid_w, int w, int32_t *win_offsets, int32_t *win_tokens,
                                hipStream_t stream) {
  const int win_per_seq = (w == 0) ? 1 : tiles * w * w;
  const int p2 = next_pow2(max_seq > 1 ? max_seq : 1);
  hipLaunchKernelGGL(build_windows_kernel, dim3(batch), dim3(WIN_THREADS), p2 * sizeof(uint32_t), stream, cu_vis,
                     pos, batch, tiles, grid_h, grid_w, w, win_per_seq, win_offsets, win_tokens);
  return hipGetLastError();
}

}  // namespace lk
