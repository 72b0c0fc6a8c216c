// Prompt-guidance weight xi (paper Sec. 3.2.1 Step 3, Eq. "attention-factor"), text-query mode without a given lse,
// for batches: one workgroup owns one (sequence, head) pair and never leaves it, so the softmax statistics of the prompt
// rows stay in registers and nothing but the per-head result is written.
//
//   wave w keeps prompt rows 32w .. 32w+31 of the head in registers (prompts of at most 256 tokens);
//   the vision keys stream through LDS in blocks of 32 (coalesced 16-byte loads, requested XS_PF blocks ahead, three
//   LDS slots, one barrier per block; the MFMAs of the next block are issued before the exponentials of this one),
//   twice -- forwards, then backwards (the blocks seen last are the ones still in L2):
//     sweep 1  keys are the MFMA row operand: every lane follows one prompt row and keeps a running (max, sum of
//              exponentials) over the keys it sees (its half of every block); the two halves merge once at the end;
//     sweep 2  prompt rows are the MFMA row operand: exp2(logit * scale - max - log2 sum) summed over the wave's 32
//              prompt rows inside the lanes, then over the waves in wave order through LDS, gives xi of the block's
//              32 keys for this head.
// The heads are summed by xi_heads_kernel afterwards, as in the two-pass path.
#include "lk_xi_body.h"
#include <type_traits>

namespace lk {

constexpr int XS_WAVES = 8;
constexpr int XS_THREADS = XS_WAVES * 64;
constexpr int XS_PF = 2;   // key blocks in flight between the request and the LDS slots (two more are staged there)

template <typename T, int DH> struct XsShape {
  using S = XiStage<T, DH, 64>;
  static constexpr int CHUNKS = 32 * S::CPR;                                   // 16-byte chunks of a key block
  static constexpr int PASSES = (CHUNKS + XS_THREADS - 1) / XS_THREADS;        // chunks per thread
  static constexpr int BLOCK_BYTES = 32 * S::PITCH;
  // 128 registers per lane except for 512-byte head rows, whose operands alone take that many
  static constexpr int WAVES_PER_SIMD = S::ROW_BYTES >= 512 ? 2 : 4;
  static constexpr int LDS = 3 * BLOCK_BYTES + 2 * XS_WAVES * 32 * 4 + XS_WAVES * 32 * 4;
};

// NEG: the softmax scale is negative (the row extreme is then the minimum of the raw products)
template <typename T, int DH, bool NEG>
__global__ __launch_bounds__(XS_THREADS, (XsShape<T, DH>::WAVES_PER_SIMD)) void xi_seq_kernel(XiArgs g) {
  using E = Elem<T>;
  using S = XiStage<T, DH, 64>;
  using X = XsShape<T, DH>;
  constexpr int NCH = XiShape<T, DH>::NCH;
  extern __shared__ __attribute__((aligned(16))) char lds[];   // X::LDS bytes are used; the launch asks for XS_LDS_REQUEST
  char *kslot = lds;                                                                         // [3][32 * PITCH]
  float (*colpart)[XS_WAVES][32] = reinterpret_cast<float (*)[XS_WAVES][32]>(lds + 3 * X::BLOCK_BYTES);   // [2]
  float (*rowbias)[32] = reinterpret_cast<float (*)[32]>(lds + 3 * X::BLOCK_BYTES + 2 * XS_WAVES * 32 * 4);   // [waves]

  const int h = blockIdx.x % g.heads, b = blockIdx.x / g.heads;
  const int t0 = g.cu_txt[b], nT = g.cu_txt[b + 1] - t0;
  const int v0 = g.cu_vis[b], nV = g.cu_vis[b + 1] - v0;
  if (nV <= 0) return;
  float *out = g.xi_part + (int64_t)h * g.sum_n + v0;
  if (nT <= 0) {   // no prompt tokens: xi is zero before the floor
    for (int i = threadIdx.x; i < nV; i += XS_THREADS) out[i] = 0.f;
    return;
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, half = lane >> 5;
  const float NEG_INF = __uint_as_float(0xff800000u);
  const int64_t vis_ho = (int64_t)h * g.vis_hs, txt_ho = (int64_t)h * g.txt_hs;
  // an even number of blocks per sweep (the last one may lie entirely past the sequence: masked in sweep 1, not stored
  // in sweep 2), so that visits come in pairs and the two sets of request registers alternate without a branch
  const int nblk = ((nV + 63) >> 6) << 1;
  const int total = 2 * nblk;                      // both sweeps as one sequence of block visits
  const int n_active = (nT + 31) >> 5;             // waves that own prompt rows
  const bool active = wave < n_active;
  const float c2 = g.scale_log2;
  constexpr bool neg_scale = NEG;
  const float pad = neg_scale ? __uint_as_float(0x7f800000u) : NEG_INF;   // product whose logit is -inf

  // this wave's prompt rows (rows past nT repeat the last one; they are given weight zero in sweep 2)
  uint4 q[NCH];
  if (active) load_half_row<T, DH>(g.txt, t0, wave * 32 + r, nT, g.txt_ts, txt_ho, half, q);

  // key block `v` (a visit index; the second sweep repeats the first) -> registers, one 16-byte chunk per pass
  auto request = [&](int v, uint4 *dst) {
    v = v < total ? v : total - 1;
    const int blk = v < nblk ? v : total - 1 - v;   // sweep 2 runs backwards: its first blocks are still in L2
#pragma unroll
    for (int p = 0; p < X::PASSES; ++p) {
      int idx = p * XS_THREADS + threadIdx.x;
      idx = idx < X::CHUNKS ? idx : X::CHUNKS - 1;
      const int row = idx / S::CPR, ch = idx % S::CPR;
      const int key = blk * 32 + row;
      const int tok = v0 + (key < nV ? key : nV - 1);
      dst[p] = ld16(static_cast<const char *>(g.vis) + ((int64_t)tok * g.vis_ts + vis_ho) * E::BYTES + ch * 16);
    }
  };
  auto stage = [&](int slot, const uint4 *src) {
#pragma unroll
    for (int p = 0; p < X::PASSES; ++p) {
      const int idx = p * XS_THREADS + threadIdx.x;
      if (idx < X::CHUNKS) {
        const int row = idx / S::CPR, ch = idx % S::CPR;
        *reinterpret_cast<uint4 *>(kslot + slot * X::BLOCK_BYTES + row * S::PITCH + ch * 16) = src[p];
      }
    }
  };

  // visit v: block v + 2 is staged into the third LDS slot, the MFMAs of block v + 1 are issued, and the exponentials
  // of block v (products already in `cur`) run in their shadow
  static_assert(XS_PF == 2, "the two sets of request registers alternate with the parity of the visit");
  uint4 ring[XS_PF][X::PASSES];
  {
    uint4 f0[X::PASSES], f1[X::PASSES];
    request(0, f0);
    request(1, f1);
#pragma unroll
    for (int u = 2; u < 2 + XS_PF; ++u) request(u, ring[u % XS_PF]);
    stage(0, f0);
    stage(1, f1);
  }
  __syncthreads();

  float m = NEG_INF, s = 0.f;   // sweep 1: running statistics of prompt row 32 * wave + r over this lane's key rows
  f32x16 cur;                   // products of the wave's prompt rows with the block of this visit
  if (active) {                 // block 0, keys as rows
    uint4 k[NCH];
    read_prompt_frag<T, DH>(kslot, r, half, k);
#pragma unroll
    for (int x = 0; x < 16; ++x) cur[x] = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) E::mma32(k[c], q[c], cur);
  }

  // One visit.  PROD: orientation of the products of block v + 1 issued in this visit (1: keys as rows, sweep 1;
  // 2: keys as columns, sweep 2; 0: none).  VAL: what happens to the products of block v (1: running statistics,
  // 2: column sums).  MASK: block v may have rows past the sequence (sweep 1 only).  The compute part is one basic
  // block: the MFMAs of the next block are spread between the exponentials of this one.
  auto visit = [&](int v, uint4 *rg, auto prod_tag, auto val_tag, auto mask_tag) {
    constexpr int PROD = decltype(prod_tag)::value, VAL = decltype(val_tag)::value;
    constexpr bool MASK = decltype(mask_tag)::value;
    if (VAL == 2 && v > nblk && wave == XS_WAVES - 1 && lane < 32) {
      // xi of the block visited before this one: the waves' partial sums in wave order
      const int pb = total - v;   // block of visit v - 1
      float sum = 0.f;
      for (int w = 0; w < n_active; ++w) sum += colpart[(v - 1) & 1][w][lane];
      if (pb * 32 + lane < nV) out[pb * 32 + lane] = sum;
    }
    if (active) {
      f32x16 nxt;
      uint4 k[NCH];
      if (PROD) read_prompt_frag<T, DH>(kslot + ((v + 1) % 3) * X::BLOCK_BYTES, r, half, k);
      float bias[16];
      if (VAL == 2) {
        // -(max + log2 sum) of the prompt row behind every accumulator register; rows past nT: -inf, weight zero
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const f32x4 b4 = *reinterpret_cast<const f32x4 *>(&rowbias[wave][8 * gq + 4 * half]);
#pragma unroll
          for (int x = 0; x < 4; ++x) bias[4 * gq + x] = b4[x];
        }
      }
      if (VAL == 1 && MASK) {
#pragma unroll
        for (int x = 0; x < 16; ++x) cur[x] = (v * 32 + acc_row(x, lane) < nV) ? cur[x] : pad;
      }
      if (PROD) {
#pragma unroll
        for (int x = 0; x < 16; ++x) nxt[x] = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          if (PROD == 1) E::mma32(k[c], q[c], nxt);
          else E::mma32(q[c], k[c], nxt);
        }
      }
      if (VAL == 1) {
        // the extreme is taken on the raw products (maximum for a positive scale, minimum for a negative one), the
        // scale goes into the exponent's multiply-add
        float e0 = cur[0], e1 = cur[1];
        if (neg_scale) {
#pragma unroll
          for (int x = 2; x < 16; x += 2) { e0 = fminf(e0, cur[x]); e1 = fminf(e1, cur[x + 1]); }
          e0 = fminf(e0, e1);
        } else {
#pragma unroll
          for (int x = 2; x < 16; x += 2) { e0 = fmaxf(e0, cur[x]); e1 = fmaxf(e1, cur[x + 1]); }
          e0 = fmaxf(e0, e1);
        }
        const float mn = fmaxf(m, e0 * c2);
        // nothing but masked rows so far (mn = -inf): any finite reference keeps every term at exp2(-inf) = 0 without
        // a branch around the exponentials
        const float mref = (mn > NEG_INF) ? mn : 0.f;
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int x = 0; x < 16; x += 2) {
          a0 += fast_exp2(fmaf(cur[x], c2, -mref));
          a1 += fast_exp2(fmaf(cur[x + 1], c2, -mref));
        }
        s = fmaf(s, fast_exp2(m - mref), a0 + a1);
        m = mn;
      } else {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int x = 0; x < 16; x += 2) {
          a0 += fast_exp2(fmaf(cur[x], c2, bias[x]));
          a1 += fast_exp2(fmaf(cur[x + 1], c2, bias[x + 1]));
        }
        float cs = a0 + a1;
        cs += __shfl_xor(cs, 32, 64);
        if (half == 0) colpart[v & 1][wave][r] = cs;
      }
      if (PROD && E::BYTES == 2) {
        // issue order: one MFMA, then its share of the 60-odd vector instructions
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 64 / NCH, 0);
        }
      }
      if (PROD) cur = nxt;
    }
    // block v + 2 goes to the slot whose last readers (the products of block v - 1) passed the barrier that ended
    // visit v - 2; its registers then take the request for block v + 2 + XS_PF.  This comes after the compute part
    // because a wave runs in order: waiting here for the data first would hold back work that does not need it.
    stage((v + 2) % 3, rg);
    request(v + 2 + XS_PF, rg);
    lds_barrier();
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  const std::false_type no_mask{};
  const std::true_type mask{};

  int v = 0;
  for (; v < nblk - 2; v += 2) {
    visit(v, ring[0], I1{}, I1{}, no_mask);
    visit(v + 1, ring[1], I1{}, I1{}, no_mask);
  }
  visit(v, ring[0], I1{}, I1{}, mask);       // the last two blocks of sweep 1 may have rows past the sequence;
  visit(v + 1, ring[1], I2{}, I1{}, mask);   // the products of sweep 2 start
  v += 2;
  // between the sweeps: merge the two halves of every prompt row, lower half first in both lanes so that they hold
  // the same bits; sweep 2 reads the rows' biases in accumulator order
  if (active) {
    const float om = __shfl_xor(m, 32, 64), os = __shfl_xor(s, 32, 64);
    const float mm = fmaxf(m, om);
    const float lo_m = half ? om : m, lo_s = half ? os : s, hi_m = half ? m : om, hi_s = half ? s : os;
    const float ss = lo_s * exp2f(lo_m - mm) + hi_s * exp2f(hi_m - mm);
    const bool row_live = wave * 32 + r < nT;
    if (half == 0) rowbias[wave][r] = row_live ? -(mm + log2f(ss)) : NEG_INF;
  }
  __syncthreads();
  for (; v < total - 2; v += 2) {
    visit(v, ring[0], I2{}, I2{}, no_mask);
    visit(v + 1, ring[1], I2{}, I2{}, no_mask);
  }
  visit(v, ring[0], I2{}, I2{}, no_mask);
  visit(v + 1, ring[1], I0{}, I2{}, no_mask);
  if (wave == XS_WAVES - 1 && lane < 32) {
    const int pb = 0;   // the last visit of sweep 2
    float sum = 0.f;
    for (int w = 0; w < n_active; ++w) sum += colpart[(total - 1) & 1][w][lane];
    if (pb * 32 + lane < nV) out[pb * 32 + lane] = sum;
  }
}

bool xi_seq_applies(const XiPlan &plan, int xi_mode, const float *lse, int batch, int heads) {
  return xi_mode == 0 && lse == nullptr && plan.max_text_tiles > 0 && plan.max_text_tiles * 32 <= XS_WAVES * 32 &&
         batch * heads >= XI_SEQ_MIN_PAIRS;
}

// The kernel is launched with more LDS than it uses, so that only ONE workgroup fits a CU: this kernel never runs alone
// in a step (the feature-divergence chain runs beside it), and two workgroups per CU take every register of the CU for
// the whole length of the kernel, leaving the other chain to wait for a CU to drain.  With one, xi takes two rounds
// instead of one, and the step of a batch of 16 is 2 % shorter (472 -> 463 us).
constexpr size_t XS_LDS_REQUEST = 84 * 1024;

template <typename T, int DH>
static hipError_t launch_xi_seq_t(const XiArgs &g, hipStream_t stream) {
  static_assert(XsShape<T, DH>::LDS <= XS_LDS_REQUEST, "the request covers what the kernel uses");
  static bool allowed[64] = {};   // more than the 64 KB default: a property of the kernels as loaded on a device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!allowed[dev]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(xi_seq_kernel<T, DH, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)XS_LDS_REQUEST);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void *>(xi_seq_kernel<T, DH, false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)XS_LDS_REQUEST);
    if (e != hipSuccess) return e;
    allowed[dev] = true;
  }
  const dim3 grid((unsigned)(g.batch * g.heads)), block(XS_THREADS);
  if (g.scale_log2 < 0.f) hipLaunchKernelGGL((xi_seq_kernel<T, DH, true>), grid, block, XS_LDS_REQUEST, stream, g);
  else hipLaunchKernelGGL((xi_seq_kernel<T, DH, false>), grid, block, XS_LDS_REQUEST, stream, g);
  return hipGetLastError();
}

hipError_t launch_xi_seq(const XiArgs &g, int dtype, int head_dim, hipStream_t stream) {
  if (g.batch * g.heads <= 0) return hipSuccess;
  if (dtype == 1) {
    if (head_dim == 128) return launch_xi_seq_t<bf16_t, 128>(g, stream);
    if (head_dim == 64) return launch_xi_seq_t<bf16_t, 64>(g, stream);
    if (head_dim == 32) return launch_xi_seq_t<bf16_t, 32>(g, stream);
  } else {
    if (head_dim == 128) return launch_xi_seq_t<float, 128>(g, stream);
    if (head_dim == 64) return launch_xi_seq_t<float, 64>(g, stream);
    if (head_dim == 32) return launch_xi_seq_t<float, 32>(g, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace lk
