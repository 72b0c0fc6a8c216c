// Device-side helpers shared by the LightKV kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lk_launch.h"

namespace lk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct bf16_t { uint16_t bits; };   // storage tag for bf16 tensors

constexpr int WAVE = 64;

// ---- element traits --------------------------------------------------------------------
// A "chunk" is one 16-byte load of a lane.  One call of mma32() consumes one chunk of the
// A operand and one of the B operand per lane and adds a 32x32 outer-product block:
//   lane l supplies row (l % 32) and the k-slice (l / 32) of the chunk pair.
// The assignment of k indices to lanes is the same for both operands, which is all a dot
// product needs, so lanes may fetch any contiguous run of the row.
template <typename T> struct Elem;

template <> struct Elem<bf16_t> {
  static constexpr int BYTES = 2;
  static constexpr int PER_CHUNK = 8;
  static __device__ __forceinline__ void mma32(const uint4 &a, const uint4 &b, f32x16 &c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_float(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
};

template <> struct Elem<float> {
  static constexpr int BYTES = 4;
  static constexpr int PER_CHUNK = 4;
  static __device__ __forceinline__ void mma32(const uint4 &a, const uint4 &b, f32x16 &c) {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
  }
};

// Row held by accumulator register `idx` (0..15) of a 32x32 block in lane `lane`; its column is lane % 32.
__device__ __forceinline__ int acc_row(int idx, int lane) { return 8 * (idx >> 2) + 4 * (lane >> 5) + (idx & 3); }

// fp32 -> bf16 bits, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Monotone map float -> uint32 (a < b  <=>  key(a) < key(b)), -0 < +0.
__device__ __forceinline__ uint32_t f32_order_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint4 ld16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }

// In-place ascending bitonic sort of n (a power of two) keys in LDS by the whole workgroup.
template <typename KeyT>
__device__ __forceinline__ void bitonic_sort_lds(KeyT *keys, int n) {
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      __syncthreads();
      for (int t = threadIdx.x; t < (n >> 1); t += blockDim.x) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int l = i | j;
        const bool up = ((i & k) == 0);
        const KeyT a = keys[i], b = keys[l];
        if ((a > b) == up) { keys[i] = b; keys[l] = a; }
      }
    }
  }
  __syncthreads();
}

// Workgroup barrier that orders LDS traffic only: waits for this wave's outstanding LDS operations, then
// s_barrier.  Unlike __syncthreads() it does not wait for global loads, so prefetches stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// |x|^2 of the eight bf16 values of one 16-byte chunk, in a fixed order.  Every kernel that produces squared row
// norms uses this, the same chunk-to-lane assignment (chunk c of a row belongs to lane c % 64, chunks in ascending
// order) and the same butterfly over the wave, so that their results agree bit for bit.
__device__ __forceinline__ float sumsq_chunk_bf16(const uint4 &v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float t = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float lo = __uint_as_float(w[q] << 16), hi = __uint_as_float(w[q] & 0xffff0000u);
    t = fmaf(lo, lo, t);
    t = fmaf(hi, hi, t);
  }
  return t;
}
__device__ __forceinline__ float sumsq_chunk_f32(const uint4 &v) {
  float t = 0.f;
  t = fmaf(__uint_as_float(v.x), __uint_as_float(v.x), t);
  t = fmaf(__uint_as_float(v.y), __uint_as_float(v.y), t);
  t = fmaf(__uint_as_float(v.z), __uint_as_float(v.z), t);
  t = fmaf(__uint_as_float(v.w), __uint_as_float(v.w), t);
  return t;
}
__device__ __forceinline__ float wave_sum_butterfly(float s) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
  return s;
}

// Packed keys of the tiled FD kernel, [column tile][list position]: column tiles a window of nB B nodes really has,
// and the minimum over them for one position.
__device__ __forceinline__ int fd_big_col_tiles(int nB, int plan_nt) {
  const int n = (nB + 95) / 96;   // FD_BIG_TILE columns per tile
  return n < plan_nt ? n : plan_nt;
}
__device__ __forceinline__ unsigned long long fd_big_best_key(const unsigned long long *cand, int sum_n, int pos,
                                                              int n_col_tiles) {
  unsigned long long best = ~0ull;
  int n = 0;
  for (; n + 4 <= n_col_tiles; n += 4) {   // four loads in flight
    unsigned long long c[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) c[u] = cand[(size_t)(n + u) * (size_t)sum_n + (size_t)pos];
#pragma unroll
    for (int u = 0; u < 4; ++u) best = c[u] < best ? c[u] : best;
  }
  for (; n < n_col_tiles; ++n) {
    const unsigned long long c = cand[(size_t)n * (size_t)sum_n + (size_t)pos];
    best = c < best ? c : best;
  }
  return best;
}

__host__ __device__ __forceinline__ int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

}  // namespace lk
