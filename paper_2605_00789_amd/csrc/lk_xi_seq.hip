// Prompt-guidance weight xi (paper Sec. 3.2.1 Step 3, Eq. "attention-factor"), text-query mode without a given lse,
// for batches: one workgroup owns one (sequence, head) pair and never leaves it, so the softmax statistics of the prompt
// rows stay in registers and nothing but the per-head result is written.
//
//   the prompt (at most 256 tokens) is cut into chunks of 32 rows; a wave keeps ONE chunk in registers, and when the
//   prompt has fewer chunks than the workgroup has waves, several waves (`groups`, up to GMAX) hold the same chunk and
//   share the keys among them: a visit then covers `groups` key blocks at once and the sequence of visits -- each
//   ending in a barrier, which is what the kernel's time is made of -- is that much shorter;
//   the vision keys stream through LDS in blocks of 32 (coalesced 16-byte loads, requested XS_PF visits ahead, three
//   LDS slots, one barrier per visit; the MFMAs of the next visit are issued before the exponentials of this one),
//   twice -- forwards, then backwards (the blocks seen last are the ones still in L2):
//     sweep 1  keys are the MFMA row operand: every lane follows one prompt row and keeps a running (max, sum of
//              exponentials) over the keys it sees (its half of every block of its group); the halves, then the groups
//              in group order, merge once at the end;
//     sweep 2  prompt rows are the MFMA row operand: exp2(logit * scale - max - log2 sum) summed over the wave's 32
//              prompt rows inside the lanes, then over the waves in wave order through LDS, gives xi of the block's
//              32 keys for this head.
// The heads are summed by xi_heads_kernel afterwards, as in the two-pass path.
#include <atomic>
#include "lk_xi_body.h"
#include <type_traits>

namespace lk {

constexpr int XS_MAX_CHUNKS = 8;   // prompt chunks of 32 rows: prompts of at most 256 tokens
constexpr int XS_PF = 2;   // visits in flight between the request and the LDS slots (two more are staged there)

template <typename T, int DH> struct XsShape {
  using S = XiStage<T, DH, 64>;
  // head rows of 256 bytes or more: operands, products and request registers do not fit 128 registers per lane, so
  // eight waves with 256 each; otherwise sixteen waves with 128
  static constexpr int WAVES = S::ROW_BYTES >= 256 ? 8 : 16;
  static constexpr int THREADS = WAVES * 64;
  static constexpr int WAVES_PER_SIMD = WAVES / 4;
  static constexpr int GMAX = S::ROW_BYTES >= 256 ? 2 : 4;                     // key blocks per visit, at most (LDS)
  static constexpr int RED_WAVES = GMAX * 32 / 64;                             // waves that add up a visit's column sums
  static constexpr int CHUNKS = 32 * S::CPR;                                   // 16-byte chunks of a key block
  static constexpr int passes(int groups) { return (groups * CHUNKS + THREADS - 1) / THREADS; }   // per thread and visit
  static constexpr int BLOCK_BYTES = 32 * S::PITCH;
  static constexpr int SLOT_BYTES = GMAX * BLOCK_BYTES;
  static constexpr int COLPART_OFF = 3 * SLOT_BYTES;                           // float [2][WAVES][32]
  static constexpr int ROWBIAS_OFF = COLPART_OFF + 2 * WAVES * 32 * 4;         // float [XS_MAX_CHUNKS][32]
  static constexpr int STATS_OFF = ROWBIAS_OFF + XS_MAX_CHUNKS * 32 * 4;       // float2 [WAVES][32]
  static constexpr int LDS = STATS_OFF + WAVES * 32 * 8;
  // One workgroup per CU: the launch asks for more than half of a CU's LDS whatever the shape uses.  This kernel never
  // runs alone in a step (the feature-divergence chain runs beside it), and a second workgroup would take the CU's
  // remaining registers for the whole length of the kernel, leaving the other chain to wait for a CU to drain.
  static constexpr int LDS_REQUEST = LDS > 84 * 1024 ? LDS : 84 * 1024;
};

// NEG: the softmax scale is negative (the row extreme is then the minimum of the raw products)
// G: waves that share a prompt chunk = key blocks per visit
template <typename T, int DH, bool NEG, int G>
__device__ __forceinline__ void xi_seq_body(const XiArgs &g) {
  using E = Elem<T>;
  using S = XiStage<T, DH, 64>;
  using X = XsShape<T, DH>;
  constexpr int NCH = XiShape<T, DH>::NCH;
  constexpr int WAVES = X::WAVES, THREADS = X::THREADS;
  extern __shared__ __attribute__((aligned(16))) char lds[];   // X::LDS bytes are used; the launch asks for X::LDS_REQUEST
  char *kslot = lds;                                                                         // [3][GMAX][32 * PITCH]
  float (*colpart)[WAVES][32] = reinterpret_cast<float (*)[WAVES][32]>(lds + X::COLPART_OFF);   // [2]
  float (*rowbias)[32] = reinterpret_cast<float (*)[32]>(lds + X::ROWBIAS_OFF);                 // [chunks]
  float2 (*stats)[32] = reinterpret_cast<float2 (*)[32]>(lds + X::STATS_OFF);                   // [waves]

  const int h = blockIdx.x % g.heads, b = blockIdx.x / g.heads;
  const int t0 = g.cu_txt[b], nT = g.cu_txt[b + 1] - t0;
  const int v0 = g.cu_vis[b], nV = g.cu_vis[b + 1] - v0;
  if (nV <= 0) return;
  float *out = g.xi_part + (int64_t)h * g.sum_n + v0;
  if (nT <= 0) {   // no prompt tokens: xi is zero before the floor
    for (int i = threadIdx.x; i < nV; i += THREADS) out[i] = 0.f;
    return;
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 31, half = lane >> 5;
  const float NEG_INF = __uint_as_float(0xff800000u);
  const int64_t vis_ho = (int64_t)h * g.vis_hs, txt_ho = (int64_t)h * g.txt_hs;
  // waves -> (group, chunk)
  constexpr int groups = G, CW = WAVES / G, PASSES = X::passes(G);
  static_assert(G <= X::GMAX && CW * G == WAVES && CW <= XS_MAX_CHUNKS, "groups x chunks = waves");
  const int n_active = (nT + 31) >> 5;             // prompt chunks: at most CW (the caller's choice of G)
  const int chunk = wave % CW, grp = wave / CW;
  const bool active = chunk < n_active;
  // a visit covers `groups` key blocks; both sweeps as one sequence of 2 * nvis visits (an even number, so that the
  // two sets of request registers alternate without a branch).  Blocks past the sequence (in the last visit of sweep 1
  // = the first of sweep 2 only) are masked in sweep 1 and not stored in sweep 2.
  const int nvis = ((nV + 31) / 32 + groups - 1) / groups;
  const int total = 2 * nvis;
  const float c2 = g.scale_log2;
  constexpr bool neg_scale = NEG;
  const float pad = neg_scale ? __uint_as_float(0x7f800000u) : NEG_INF;   // product whose logit is -inf

  // this wave's prompt rows (rows past nT repeat the last one; they are given weight zero in sweep 2)
  uint4 q[NCH];
  if (active) load_half_row<T, DH>(g.txt, t0, chunk * 32 + r, nT, g.txt_ts, txt_ho, half, q);

  // the key blocks of visit `v` (the second sweep repeats the first, backwards: its first blocks are still in L2)
  // -> registers, one 16-byte chunk per pass
  auto request = [&](int v, uint4 *dst) {
    v = v < total ? v : total - 1;
    const int step = v < nvis ? v : total - 1 - v;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      int idx = p * THREADS + threadIdx.x;
      idx = idx < G * X::CHUNKS ? idx : G * X::CHUNKS - 1;
      const int row = idx / S::CPR, ch = idx % S::CPR;   // row within the visit's G * 32 keys
      const int key = step * (G * 32) + row;
      const int tok = v0 + (key < nV ? key : nV - 1);
      dst[p] = ld16(static_cast<const char *>(g.vis) + ((int64_t)tok * g.vis_ts + vis_ho) * E::BYTES + ch * 16);
    }
  };
  auto stage = [&](int slot, const uint4 *src) {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int idx = p * THREADS + threadIdx.x;
      if (idx < G * X::CHUNKS) {
        const int row = idx / S::CPR, ch = idx % S::CPR;   // the blocks of a slot lie back to back
        *reinterpret_cast<uint4 *>(kslot + slot * X::SLOT_BYTES + row * S::PITCH + ch * 16) = src[p];
      }
    }
  };
  const char *my_blocks = kslot + grp * X::BLOCK_BYTES;   // this wave's block inside a slot

  // visit v: the blocks of visit v + 2 are staged into the third LDS slot, the MFMAs of visit v + 1 are issued, and the
  // exponentials of visit v (products already in `cur`) run in their shadow
  static_assert(XS_PF == 2, "the two sets of request registers alternate with the parity of the visit");
  uint4 ring[XS_PF][PASSES];
  {
    uint4 f0[PASSES], f1[PASSES];
    request(0, f0);
    request(1, f1);
#pragma unroll
    for (int u = 2; u < 2 + XS_PF; ++u) request(u, ring[u % XS_PF]);
    stage(0, f0);
    stage(1, f1);
  }
  __syncthreads();

  float m = NEG_INF, s = 0.f;   // sweep 1: running statistics of prompt row 32 * chunk + r over this lane's key rows
  f32x16 cur;                   // products of the wave's prompt rows with its block of this visit
  if (active) {                 // visit 0, keys as rows
    uint4 k[NCH];
    read_prompt_frag<T, DH>(my_blocks, r, half, k);
#pragma unroll
    for (int x = 0; x < 16; ++x) cur[x] = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) E::mma32(k[c], q[c], cur);
  }

  // xi of the blocks of sweep-2 visit `pv`: the chunks' partial sums in chunk order
  auto reduce_columns = [&](int pv) {
    if (wave >= WAVES - X::RED_WAVES) {
      const int idx = (wave - (WAVES - X::RED_WAVES)) * 64 + lane;
      const int gi = idx >> 5, kk = idx & 31;
      if (gi < groups) {
        float sum = 0.f;
        for (int c = 0; c < n_active; ++c) sum += colpart[pv & 1][gi * CW + c][kk];
        const int key = ((total - 1 - pv) * groups + gi) * 32 + kk;
        if (key < nV) out[key] = sum;
      }
    }
  };

  // One visit.  PROD: orientation of the products of visit v + 1 issued in this visit (1: keys as rows, sweep 1;
  // 2: keys as columns, sweep 2; 0: none).  VAL: what happens to the products of visit v (1: running statistics,
  // 2: column sums).  MASK: the blocks of visit v may have rows past the sequence (sweep 1 only).  The compute part is
  // one basic block: the MFMAs of the next visit are spread between the exponentials of this one.
  auto visit = [&](int v, uint4 *rg, auto prod_tag, auto val_tag, auto mask_tag) {
    constexpr int PROD = decltype(prod_tag)::value, VAL = decltype(val_tag)::value;
    constexpr bool MASK = decltype(mask_tag)::value;
    if (VAL == 2 && v > nvis) reduce_columns(v - 1);
    if (active) {
      f32x16 nxt;
      uint4 k[NCH];
      if (PROD) read_prompt_frag<T, DH>(my_blocks + ((v + 1) % 3) * X::SLOT_BYTES, r, half, k);
      float bias[16];
      if (VAL == 2) {
        // -(max + log2 sum) of the prompt row behind every accumulator register; rows past nT: -inf, weight zero
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const f32x4 b4 = *reinterpret_cast<const f32x4 *>(&rowbias[chunk][8 * gq + 4 * half]);
#pragma unroll
          for (int x = 0; x < 4; ++x) bias[4 * gq + x] = b4[x];
        }
      }
      if (VAL == 1 && MASK) {
        const int key0 = (v * groups + grp) * 32;
#pragma unroll
        for (int x = 0; x < 16; ++x) cur[x] = (key0 + acc_row(x, lane) < nV) ? cur[x] : pad;
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
    // the blocks of visit v + 2 go to the slot whose last readers (the products of visit v - 1) passed the barrier that
    // ended visit v - 2; its registers then take the request for visit v + 2 + XS_PF.  This comes after the compute
    // part because a wave runs in order: waiting here for the data first would hold back work that does not need it.
    stage((v + 2) % 3, rg);
    request(v + 2 + XS_PF, rg);
    lds_barrier();
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  const std::false_type no_mask{};
  const std::true_type mask{};

  // between the sweeps: merge the two halves of every prompt row (lower half first in both lanes so that they hold
  // the same bits), then the groups in group order; sweep 2 reads the rows' biases in accumulator order
  auto between_sweeps = [&]() {
    if (active) {
      const float om = __shfl_xor(m, 32, 64), os = __shfl_xor(s, 32, 64);
      const float mm = fmaxf(m, om);
      const float ref = (mm > NEG_INF) ? mm : 0.f;   // a group that saw nothing but masked rows: sum 0, maximum -inf
      const float lo_m = half ? om : m, lo_s = half ? os : s, hi_m = half ? m : om, hi_s = half ? s : os;
      const float ss = lo_s * exp2f(lo_m - ref) + hi_s * exp2f(hi_m - ref);
      if (half == 0) stats[wave][r] = make_float2(mm, ss);
    }
    __syncthreads();
    if (active && grp == 0 && half == 0) {
      float mm = NEG_INF;   // group 0 saw key 0: finite
      for (int gi = 0; gi < groups; ++gi) mm = fmaxf(mm, stats[gi * CW + chunk][r].x);
      float ss = 0.f;
      for (int gi = 0; gi < groups; ++gi) {
        const float2 st = stats[gi * CW + chunk][r];
        ss += st.y * exp2f(st.x - mm);
      }
      const bool row_live = chunk * 32 + r < nT;
      rowbias[chunk][r] = row_live ? -(mm + log2f(ss)) : NEG_INF;
    }
    __syncthreads();
  };

  // visits 0 .. nvis-2: sweep 1; nvis-1: its last (masked; the products of sweep 2 start); nvis .. total-2: sweep 2;
  // total-1: the last (no more products).  Pairs (even visit, odd visit) use the two sets of request registers in turn.
  int v = 0;
  for (; v + 2 <= nvis - 1; v += 2) {
    visit(v, ring[0], I1{}, I1{}, no_mask);
    visit(v + 1, ring[1], I1{}, I1{}, no_mask);
  }
  if (nvis - 1 - v == 1) {   // an even number of visits per sweep
    visit(v, ring[0], I1{}, I1{}, no_mask);
    visit(v + 1, ring[1], I2{}, I1{}, mask);
    between_sweeps();
  } else {                   // an odd number: the pair straddles the sweeps
    visit(v, ring[0], I2{}, I1{}, mask);
    between_sweeps();
    if (nvis == 1) visit(v + 1, ring[1], I0{}, I2{}, no_mask);
    else visit(v + 1, ring[1], I2{}, I2{}, no_mask);
  }
  v += 2;
  for (; v + 2 < total; v += 2) {
    visit(v, ring[0], I2{}, I2{}, no_mask);
    visit(v + 1, ring[1], I2{}, I2{}, no_mask);
  }
  if (v < total) {
    visit(v, ring[0], I2{}, I2{}, no_mask);
    visit(v + 1, ring[1], I0{}, I2{}, no_mask);
  }
  reduce_columns(total - 1);
}

// Every workgroup takes the largest group count that leaves a wave to each 32-row chunk of ITS prompt.
template <typename T, int DH, bool NEG>
__global__ __launch_bounds__((XsShape<T, DH>::THREADS), (XsShape<T, DH>::WAVES_PER_SIMD)) void xi_seq_kernel(XiArgs g) {
  using X = XsShape<T, DH>;
  const int b = blockIdx.x / g.heads;
  const int chunks = (g.cu_txt[b + 1] - g.cu_txt[b] + 31) >> 5;
  if constexpr (X::GMAX >= 4) {
    if (chunks * 4 <= X::WAVES) return xi_seq_body<T, DH, NEG, 4>(g);
  }
  if (chunks * 2 <= X::WAVES) return xi_seq_body<T, DH, NEG, 2>(g);
  if constexpr (X::WAVES <= XS_MAX_CHUNKS) xi_seq_body<T, DH, NEG, 1>(g);   // sixteen waves: two groups always fit
}

bool xi_seq_applies(const XiPlan &plan, int xi_mode, const float *lse, int batch, int heads) {
  return xi_mode == 0 && lse == nullptr && plan.max_text_tiles > 0 && plan.max_text_tiles <= XS_MAX_CHUNKS &&
         batch * heads >= XI_SEQ_MIN_PAIRS;
}

template <typename T, int DH>
static hipError_t launch_xi_seq_t(const XiArgs &g, hipStream_t stream) {
  constexpr int XS_LDS_REQUEST = XsShape<T, DH>::LDS_REQUEST;
  static std::atomic<bool> allowed[64];   // more than the 64 KB default: a property of the kernels as loaded on a device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!allowed[dev].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(xi_seq_kernel<T, DH, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)XS_LDS_REQUEST);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void *>(xi_seq_kernel<T, DH, false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)XS_LDS_REQUEST);
    if (e != hipSuccess) return e;
    allowed[dev].store(true, std::memory_order_release);
  }
  const dim3 grid((unsigned)(g.batch * g.heads)), block((XsShape<T, DH>::THREADS));
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
