// Top2Gating (Algorithm 1 of the paper, for G independent groups) in three kernels:
//
//   gate_topk_kernel    per token: logits x.wg, softmax, top-2, renormalised gates,
//                       the random-routing decision; per 64-token chunk: histogram of
//                       first choices / sampled second choices and the gate sums
//   gate_scan_kernel    per group: exclusive scan of the chunk histograms over the
//                       chunks (the running counters c_E of Algorithm 1 at chunk
//                       boundaries), c1, mean gates m_E, fill, empty slots
//   gate_slots_kernel   per chunk: stable rank of every token among the earlier
//                       tokens of its chunk with the same expert + the chunk base
//                       = position in the expert buffer; capacity test; combine
//                       weights; inverse map slot -> token; l_aux
//
// bf16 activations take the MFMA form of the first kernel (gate_mfma_*): x is
// exactly bf16, so with wg split into three bf16 terms (hi + mid + lo = all 24
// mantissa bits) every product is exact in fp32 and only the accumulation order
// differs from a plain fp32 dot product.  wg is repacked (by the caller once per
// weight update, else once per call) into the lane order of the
// v_mfma_f32_32x32x16_bf16 B operand, so each B load is one contiguous 1 KB read.
// Gates wider than 512 experts and fp32 activations with GEMM-friendly shapes get
// their logits from the persistent GEMM kernel; everything else keeps the plain FMA
// kernel.
//
// Positions never come from atomics: they are exact counts of earlier tokens, so
// the result equals the sequential two-pass loop of Algorithm 1 bit for bit.
#include <limits.h>
#include <math.h>
#include "common.h"

namespace moe {

namespace {

__device__ __forceinline__ void argmax_merge(float& bv, int& bi, float ov, int oi) {
  if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
}
__device__ __forceinline__ void wave_argmax(float& bv, int& bi) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(bv, o, 64);
    int oi = __shfl_xor(bi, o, 64);
    argmax_merge(bv, bi, ov, oi);
  }
}

// One block = one chunk of 64 tokens of one group; wave w takes tokens w, w+4, ...
// Lane l owns experts l, l+64, ... (EPL of them).
// PRE: the logits were computed beforehand on the matrix cores (very wide gates): zpre
// [tokens, cols] holds, for expert e, the three partial logits x . (hi, mid, lo term of wg) in
// columns 3e, 3e+1, 3e+2; they are added smallest term first.
template <typename T, int EPL, bool PRE>
__global__ __launch_bounds__(256) void gate_topk_kernel(
    const T* __restrict__ x, const float* __restrict__ wg, const float* __restrict__ u,
    const float* __restrict__ zpre, int cols, int S, int M, int E, int nch,
    int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot, float* __restrict__ weight,
    float* __restrict__ gates_opt,
    int32_t* __restrict__ hist1, int32_t* __restrict__ hist2, float* __restrict__ msum) {
  extern __shared__ unsigned char smem[];
  const int g = blockIdx.x / nch, ch = blockIdx.x % nch;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* xs = reinterpret_cast<float*>(smem) + (size_t)wave * M;  // this wave's token row
  float* msum_l = reinterpret_cast<float*>(smem) + (PRE ? 0 : (size_t)4 * M);  // [4][E]
  int* h1 = reinterpret_cast<int*>(msum_l + (size_t)4 * E);
  int* h2 = h1 + E;
  for (int e = threadIdx.x; e < E; e += 256) { h1[e] = 0; h2[e] = 0; }

  float macc[EPL];
#pragma unroll
  for (int j = 0; j < EPL; ++j) macc[j] = 0.f;

  for (int it = 0; it < kChunk / 4; ++it) {
    const int s = ch * kChunk + it * 4 + wave;
    const bool valid = s < S;
    const size_t n = (size_t)g * S + (valid ? s : 0);
    __syncthreads();  // previous row fully consumed (also orders the histogram zeroing)
    if (!PRE)
      for (int m = lane; m < M; m += 64) xs[m] = Elt<T>::load(x + n * M + m);
    __syncthreads();
    if (!valid) continue;  // both barriers of the next iteration are still reached

    float z[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) z[j] = 0.f;
    if (PRE) {
      const float* zp = zpre + n * cols;
#pragma unroll
      for (int j = 0; j < EPL; ++j) {
        const int e = lane + 64 * j;
        if (e < E) z[j] = (zp[3 * e + 2] + zp[3 * e + 1]) + zp[3 * e];
      }
    } else {
      for (int m = 0; m < M; ++m) {
        const float xv = xs[m];
        const float* wrow = wg + (size_t)m * E;
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
          const int e = lane + 64 * j;
          if (e < E) z[j] = fmaf(xv, wrow[e], z[j]);
        }
      }
    }
    // top-2 on the logits (softmax is monotone); ties go to the lowest index
    float v1 = -INFINITY; int e1 = INT_MAX;
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      const int e = lane + 64 * j;
      if (e < E) argmax_merge(v1, e1, z[j], e);
    }
    wave_argmax(v1, e1);
    float v2 = -INFINITY; int e2 = INT_MAX;
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      const int e = lane + 64 * j;
      if (e < E && e != e1) argmax_merge(v2, e2, z[j], e);
    }
    wave_argmax(v2, e2);

    // softmax over all experts (needed for the mean gates m_E)
    float p[EPL], psum = 0.f;
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      const int e = lane + 64 * j;
      p[j] = (e < E) ? expf(z[j] - v1) : 0.f;
      psum += p[j];
    }
    psum = wave_sum(psum);
    const float inv = 1.0f / psum;
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      const int e = lane + 64 * j;
      const float gate = p[j] * inv;
      macc[j] += gate;
      if (gates_opt != nullptr && e < E) gates_opt[n * E + e] = gate;
    }
    // g1/(g1+g2) and g2/(g1+g2): the softmax denominator cancels
    const float p2 = expf(v2 - v1);
    const float g1n = 1.0f / (1.0f + p2);
    const float g2n = p2 / (1.0f + p2);
    const bool sampled = 2.0f * g2n > u[n];
    if (lane == 0) {
      expert_idx[2 * n] = e1;
      expert_idx[2 * n + 1] = e2;
      weight[2 * n] = g1n;          // provisional: zeroed later if the slot is lost
      weight[2 * n + 1] = g2n;
      slot[2 * n + 1] = sampled ? 0 : MOE_SLOT_NOT_SAMPLED;
      atomicAdd(&h1[e1], 1);
      if (sampled) atomicAdd(&h2[e2], 1);
    }
  }

#pragma unroll
  for (int j = 0; j < EPL; ++j) {
    const int e = lane + 64 * j;
    if (e < E) msum_l[(size_t)wave * E + e] = macc[j];
  }
  __syncthreads();
  const size_t base = ((size_t)g * nch + ch) * E;
  for (int e = threadIdx.x; e < E; e += 256) {
    msum[base + e] = ((msum_l[e] + msum_l[E + e]) + msum_l[2 * (size_t)E + e]) + msum_l[3 * (size_t)E + e];
    hist1[base + e] = h1[e];
    hist2[base + e] = h2[e];
  }
}

// ----------------------------------------------------------------------------
// MFMA form for bf16 activations
// ----------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// K order inside a block of 64 model features: MFMA step j (0..3), lane half h,
// element i  <->  feature 32 h + 8 j + i.  A lane of the A operand then owns 64
// contiguous bytes of its token row per block (four 16-byte loads).
//
// wgP[ks][t][split][lane] (uint4 = 8 bf16): B operand of step ks = 4 kb + j for
// the 32 experts of column tile t; lane = 32 h + c holds expert 32 t + c.
__global__ __launch_bounds__(256) void gate_pack_wg_kernel(
    const float* __restrict__ wg, uint4* __restrict__ wgP, int M, int E, int T, int total) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int lane = idx & 63, t = (idx >> 6) % T, ks = (idx >> 6) / T;
  const int h = lane >> 5, col = 32 * t + (lane & 31);
  const int m0 = (ks >> 2) * 64 + 32 * h + 8 * (ks & 3);
  uint32_t w[3][4];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int m = m0 + i;
    const float v = (m < M && col < E) ? wg[(size_t)m * E + col] : 0.f;
    const bf16_t hi = f32_to_bf16(v);
    const float r1 = v - bf16_to_f32(hi);          // exact
    const bf16_t mid = f32_to_bf16(r1);
    const float r2 = r1 - bf16_to_f32(mid);        // exact
    const bf16_t lo = f32_to_bf16(r2);
    const bf16_t parts[3] = {hi, mid, lo};
#pragma unroll
    for (int sp = 0; sp < 3; ++sp) {
      if (i & 1) w[sp][i >> 1] |= (uint32_t)parts[sp] << 16;
      else w[sp][i >> 1] = parts[sp];
    }
  }
#pragma unroll
  for (int sp = 0; sp < 3; ++sp)
    wgP[((size_t)(ks * T + t) * 3 + sp) * 64 + lane] = uint4{w[sp][0], w[sp][1], w[sp][2], w[sp][3]};
}

struct Top2 { float v1; int e1; float v2; int e2; };

__device__ __forceinline__ bool better(float a, int ia, float b, int ib) {
  return a > b || (a == b && ia < ib);
}
__device__ __forceinline__ Top2 top2_merge(const Top2& a, const Top2& b) {
  // winner = better first entry; runner-up = better of the loser's first and the winner's second
  const bool bw = better(b.v1, b.e1, a.v1, a.e1);
  const float wv1 = bw ? b.v1 : a.v1, lv1 = bw ? a.v1 : b.v1, wv2 = bw ? b.v2 : a.v2;
  const int we1 = bw ? b.e1 : a.e1, le1 = bw ? a.e1 : b.e1, we2 = bw ? b.e2 : a.e2;
  const bool lb = better(lv1, le1, wv2, we2);
  Top2 r;
  r.v1 = wv1; r.e1 = we1;
  r.v2 = lb ? lv1 : wv2; r.e2 = lb ? le1 : we2;
  return r;
}

// Softmax / top-2 / random routing / chunk statistics for the 64 tokens of one chunk whose
// logits sit in LDS (zs, row pitch `pitch` floats, pitch = 8 mod 64).  NT threads, TPT = NT/64
// per token; a wavefront holds 64/TPT tokens (lane % (64/TPT)) and thread `sub` = lane / (64/TPT)
// of a token owns the 4-expert groups sub, sub + TPT, ...: its 16-byte reads and those of the
// 15 lanes around it fall into different banks.  A token's logits are processed in registers
// and its gates written back for the column sums.  Must be called by all threads of the block;
// ends with a barrier.
template <int NT, int EPAD>
__device__ __forceinline__ void gate_chunk_epilogue(
    float* zs, int pitch, int g, int ch, int S, int E, int nch, const float* __restrict__ u,
    int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot, float* __restrict__ weight,
    float* __restrict__ gates_opt, int32_t* __restrict__ hist1, int32_t* __restrict__ hist2,
    float* __restrict__ msum, int* h1, int* h2) {
  constexpr int TPT = NT / 64, TPW = 64 / TPT, EPT = EPAD / TPT, NG = EPT / 4;
  static_assert(EPT % 4 == 0 && EPT >= 4, "whole 4-expert groups per thread");
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  __shared__ float mpart[8 * EPAD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tk = wave * TPW + lane % TPW, sub = lane / TPW;
  const int s = ch * kChunk + tk;
  const bool valid = s < S;
  const size_t n = (size_t)g * S + (valid ? s : 0);
  const float u_n = u[n];                              // needed last: its latency hides below
  for (int e = tid; e < E; e += NT) { h1[e] = 0; h2[e] = 0; }
  float* zr = zs + (size_t)tk * pitch;
  float z[EPT];
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    const f32x4_t v = *reinterpret_cast<const f32x4_t*>(zr + 4 * (sub + TPT * i));
#pragma unroll
    for (int k = 0; k < 4; ++k) z[4 * i + k] = v[k];
  }
  Top2 t2{-INFINITY, INT_MAX, -INFINITY, INT_MAX};
#pragma unroll
  for (int i = 0; i < NG; ++i)
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int e = 4 * (sub + TPT * i) + k;
      const float zv = z[4 * i + k];
      if (e < E) {   // a thread meets its experts in ascending order: strict > keeps the lowest index of a tie
        if (zv > t2.v1) { t2.v2 = t2.v1; t2.e2 = t2.e1; t2.v1 = zv; t2.e1 = e; }
        else if (zv > t2.v2) { t2.v2 = zv; t2.e2 = e; }
      }
    }
#pragma unroll
  for (int o = TPW; o < 64; o <<= 1) {
    Top2 other;
    other.v1 = __shfl_xor(t2.v1, o, 64); other.e1 = __shfl_xor(t2.e1, o, 64);
    other.v2 = __shfl_xor(t2.v2, o, 64); other.e2 = __shfl_xor(t2.e2, o, 64);
    t2 = top2_merge(t2, other);
  }
  // softmax (bulk exponentials: the hardware exp2 path, relative error ~1e-6 at most over the
  // range a softmax tail can reach); rows past the end of the group count as zeros
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < NG; ++i)
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float p = 4 * (sub + TPT * i) + k < E ? __expf(z[4 * i + k] - t2.v1) : 0.f;
      z[4 * i + k] = p;
      psum += p;
    }
#pragma unroll
  for (int o = TPW; o < 64; o <<= 1) psum += __shfl_xor(psum, o, 64);
  const float inv = valid ? 1.0f / psum : 0.f;
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    f32x4_t v;
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = z[4 * i + k] * inv;
    *reinterpret_cast<f32x4_t*>(zr + 4 * (sub + TPT * i)) = v;
    if (gates_opt != nullptr && valid) {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (4 * (sub + TPT * i) + k < E) gates_opt[n * E + 4 * (sub + TPT * i) + k] = v[k];
    }
  }
  __syncthreads();                                     // histograms cleared, gates in LDS
  if (sub == 0 && valid) {
    const float p2 = expf(t2.v2 - t2.v1);
    const float g1n = 1.0f / (1.0f + p2);
    const float g2n = p2 / (1.0f + p2);
    const bool sampled = 2.0f * g2n > u_n;
    expert_idx[2 * n] = t2.e1;
    expert_idx[2 * n + 1] = t2.e2;
    weight[2 * n] = g1n;            // provisional: zeroed later if the slot is lost
    weight[2 * n + 1] = g2n;
    slot[2 * n + 1] = sampled ? 0 : MOE_SLOT_NOT_SAMPLED;
    atomicAdd(&h1[t2.e1], 1);
    if (sampled) atomicAdd(&h2[t2.e2], 1);
  }
  const size_t base = ((size_t)g * nch + ch) * E;
  // Gate sums of the chunk in a fixed order: eight interleaved partial sums over the 64 rows
  // (partial q takes rows q, q + 8, ...), then a tree.  tpe = 8, 4, 2 or 1 threads share the
  // partial sums of one expert.
  int tpe = 8;
  while (tpe * E > NT) tpe >>= 1;
  {
    const int e = tid / tpe, j = tid - e * tpe;
    if (e < E)
      for (int q = j; q < 8; q += tpe) {
        float part = 0.f;
#pragma unroll
        for (int r0 = 0; r0 < kChunk; r0 += 8) part += zs[(size_t)(r0 + q) * pitch + e];
        mpart[8 * e + q] = part;
      }
  }
  __syncthreads();
  for (int e = tid; e < E; e += NT) {
    const float* pp = mpart + 8 * e;
    msum[base + e] = ((pp[0] + pp[1]) + (pp[2] + pp[3])) + ((pp[4] + pp[5]) + (pp[6] + pp[7]));
    hist1[base + e] = h1[e];
    hist2[base + e] = h2[e];
  }
  __syncthreads();
}

#define MOE_GATE_MFMA(A, B, C) __builtin_amdgcn_mfma_f32_32x32x16_bf16( \
    __builtin_bit_cast(bf16x8_t, A), __builtin_bit_cast(bf16x8_t, B), C, 0, 0, 0)

// Narrow gates (E <= 64), two chunks per block: 128 tokens, wavefront w owns quarter w of the feature
// dimension and all four 32-token row tiles, so that one fetch of a packed weight fragment
// (3 KB per MFMA step from L2) feeds 12 MFMAs instead of 3: with one chunk per block the
// weight fragments cost three times the L2 traffic of x itself.  x goes from global memory
// straight into the A operand, two 64-feature blocks ahead, re-requested row tile by row tile
// as the MFMAs free the registers; the four partial sums meet in LDS.  The epilogue works in
// registers: two lanes per token read the four partial sums of half a row each (added in a fixed
// order), so softmax, top-2 and the routing decision need no further pass over LDS; the chunk's
// gate sums are wavefront butterflies over the 32 tokens of a wavefront, then one addition of
// the chunk's two wavefronts.
template <int ET>
__global__ __launch_bounds__(256) void gate_mfma_rows_kernel(
    const bf16_t* __restrict__ x, const uint4* __restrict__ wgP, const float* __restrict__ u,
    int S, int M, int E, int nch,
    int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot, float* __restrict__ weight,
    float* __restrict__ gates_opt,
    int32_t* __restrict__ hist1, int32_t* __restrict__ hist2, float* __restrict__ msum) {
  // pitch = 4 mod 32 floats: the 16-byte reads of 16 lanes (16 token rows, same columns) fall
  // into 16 different bank groups
  constexpr int Epad = 32 * ET, pitch = Epad + 4, PD = 2, EPT = Epad / 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char gate_smem[];
  float* part = reinterpret_cast<float*>(gate_smem);            // [4][128 * pitch]
  float* msw = part + 4 * 128 * pitch;                           // [4 wavefronts][Epad] gate sums
  int* hh = reinterpret_cast<int*>(msw + 4 * Epad);              // [2 chunks][2][Epad] histograms
  const int npair = (nch + 1) / 2;
  const int g = blockIdx.x / npair, pr = blockIdx.x % npair;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, h = lane >> 5;
  // epilogue role: token 32 wave + (lane % 16) + 16 (lane / 32), half (lane / 16) % 2 of its experts;
  // its random number is requested before everything else
  const int tk = 32 * wave + (lane & 15) + 16 * (lane >> 5), sub = (lane >> 4) & 1;
  const int s_ep = pr * 128 + tk;
  const bool valid = s_ep < S;
  const size_t n_ep = (size_t)g * S + (valid ? s_ep : 0);
  const float u_n = u[n_ep];
  for (int i = threadIdx.x; i < 4 * Epad; i += 256) hh[i] = 0;   // ordered by the barrier after the K loop

  const bf16_t* xrow[4];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt) {
    int s = pr * 128 + 32 * rt + r;
    s = s < S ? s : S - 1;                            // clamp: surplus rows are ignored later
    xrow[rt] = x + ((size_t)g * S + s) * M;
  }
  const int KB = (M + 63) / 64, KBq = (KB + 3) / 4;
  const int kb0 = wave * KBq < KB ? wave * KBq : KB;
  const int kb1 = kb0 + KBq < KB ? kb0 + KBq : KB;

  f32x16_t acc[4][ET];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int t = 0; t < ET; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rt][t][i] = 0.f;

  // Loads are unconditional: a block index past this wavefront's range is clamped (its
  // data is never multiplied) and features past M read the row start instead (they meet
  // zero weights in the packed operand).
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  u32x4_t a[PD][4][4];
#define MOE_GATE_LOAD_XROW(P, KBI, rt)                                                \
  {                                                                                   \
    int kbc_ = (KBI) < kb1 ? (KBI) : kb1 - 1;                                         \
    kbc_ = kbc_ < 0 ? 0 : kbc_;                                                       \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                   \
      const int col_ = kbc_ * 64 + 32 * h + 8 * j;                                    \
      a[P][rt][j] = *reinterpret_cast<const u32x4_t*>(xrow[rt] + (col_ < M ? col_ : 0)); \
    }                                                                                 \
  }
  // (two column tiles leave no registers for a pinned schedule: the compiler places the loads)
#define MOE_GATE_FENCE if (ET == 1) __builtin_amdgcn_sched_barrier(0);
  // Vector loads come back in the order they were issued, so a weight fragment requested
  // just before its MFMA would wait behind every x row requested earlier (HBM latency each
  // time).  The weight fragments of a whole super-block of SB feature blocks are therefore
  // requested first (they hit in L2), then the x rows, PD blocks ahead of their use.  The
  // fences keep the compiler from moving the loads to their uses.
  constexpr int SB = 4 / ET;
  for (int sb0 = kb0; sb0 < kb1; sb0 += SB) {
    u32x4_t b[SB][4][ET * 3];
#pragma unroll
    for (int q = 0; q < SB; ++q) {
      const int cur = sb0 + q < kb1 ? sb0 + q : kb1 - 1;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32x4_t* bp = reinterpret_cast<const u32x4_t*>(wgP) + (size_t)((cur * 4 + j) * ET) * 3 * 64 + lane;
#pragma unroll
        for (int t = 0; t < ET * 3; ++t) b[q][j][t] = bp[t * 64];
      }
    }
#pragma unroll
    for (int p = 0; p < PD; ++p)
#pragma unroll
      for (int rt = 0; rt < 4; ++rt) MOE_GATE_LOAD_XROW(p, sb0 + p, rt)
    MOE_GATE_FENCE
#pragma unroll
    for (int q = 0; q < SB; ++q) {
      const bool live = sb0 + q < kb1;                // wave-uniform
#pragma unroll
      for (int rt = 0; rt < 4; ++rt) {
        if (live) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int t = 0; t < ET; ++t) {
              acc[rt][t] = MOE_GATE_MFMA(a[q % PD][rt][j], b[q][j][t * 3 + 2], acc[rt][t]);
              acc[rt][t] = MOE_GATE_MFMA(a[q % PD][rt][j], b[q][j][t * 3 + 1], acc[rt][t]);
              acc[rt][t] = MOE_GATE_MFMA(a[q % PD][rt][j], b[q][j][t * 3 + 0], acc[rt][t]);
            }
        }
        MOE_GATE_FENCE
        if (q + PD < SB) MOE_GATE_LOAD_XROW(q % PD, sb0 + q + PD, rt)
        MOE_GATE_FENCE
      }
    }
  }
#undef MOE_GATE_LOAD_XROW
#undef MOE_GATE_FENCE
  // acc[rt][t][i]: token row 32 rt + 8 (i/4) + 4 h + i%4, expert 32 t + r
  float* dst = part + (size_t)wave * 128 * pitch;
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int t = 0; t < ET; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        dst[(32 * rt + 8 * (i >> 2) + 4 * h + (i & 3)) * pitch + 32 * t + r] = acc[rt][t][i];
  __syncthreads();

  // ---- epilogue: logits of experts [EPT sub, EPT sub + EPT) of token tk, in registers
  float z[EPT];
  {
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    const float* zr = part + (size_t)tk * pitch + EPT * sub;
#pragma unroll
    for (int i4 = 0; i4 < EPT / 4; ++i4) {
      const f32x4_t p0 = *reinterpret_cast<const f32x4_t*>(zr + 4 * i4);
      const f32x4_t p1 = *reinterpret_cast<const f32x4_t*>(zr + 128 * pitch + 4 * i4);
      const f32x4_t p2 = *reinterpret_cast<const f32x4_t*>(zr + 2 * 128 * pitch + 4 * i4);
      const f32x4_t p3 = *reinterpret_cast<const f32x4_t*>(zr + 3 * 128 * pitch + 4 * i4);
#pragma unroll
      for (int k = 0; k < 4; ++k) z[4 * i4 + k] = (p0[k] + p1[k]) + (p2[k] + p3[k]);
    }
  }
  const int ebase = EPT * sub;
  Top2 t2{-INFINITY, INT_MAX, -INFINITY, INT_MAX};
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int e = ebase + k;
    if (e < E) {     // ascending order: strict > keeps the lowest index of a tie
      if (z[k] > t2.v1) { t2.v2 = t2.v1; t2.e2 = t2.e1; t2.v1 = z[k]; t2.e1 = e; }
      else if (z[k] > t2.v2) { t2.v2 = z[k]; t2.e2 = e; }
    }
  }
  {
    Top2 other;
    other.v1 = __shfl_xor(t2.v1, 16, 64); other.e1 = __shfl_xor(t2.e1, 16, 64);
    other.v2 = __shfl_xor(t2.v2, 16, 64); other.e2 = __shfl_xor(t2.e2, 16, 64);
    t2 = top2_merge(t2, other);
  }
  // softmax numerators (bulk exponentials: the hardware exp2 path, relative error ~1e-6 at most
  // over the range a softmax tail can reach)
  float psum = 0.f;
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    z[k] = ebase + k < E ? __expf(z[k] - t2.v1) : 0.f;
    psum += z[k];
  }
  psum += __shfl_xor(psum, 16, 64);
  const float inv = valid ? 1.0f / psum : 0.f;        // rows past the end of the group count as zeros
#pragma unroll
  for (int k = 0; k < EPT; ++k) z[k] *= inv;          // the gates
  if (gates_opt != nullptr && valid) {
#pragma unroll
    for (int k = 0; k < EPT; ++k)
      if (ebase + k < E) gates_opt[n_ep * E + ebase + k] = z[k];
  }
  int* h1 = hh + (wave >> 1) * 2 * Epad;              // the histograms of this wavefront's chunk
  int* h2 = h1 + Epad;
  if (sub == 0 && valid) {
    const float p2 = expf(t2.v2 - t2.v1);
    const float g1n = 1.0f / (1.0f + p2);
    const float g2n = p2 / (1.0f + p2);
    const bool sampled = 2.0f * g2n > u_n;
    expert_idx[2 * n_ep] = t2.e1;
    expert_idx[2 * n_ep + 1] = t2.e2;
    weight[2 * n_ep] = g1n;          // provisional: zeroed later if the slot is lost
    weight[2 * n_ep + 1] = g2n;
    slot[2 * n_ep + 1] = sampled ? 0 : MOE_SLOT_NOT_SAMPLED;
    atomicAdd(&h1[t2.e1], 1);
    if (sampled) atomicAdd(&h2[t2.e2], 1);
  }
  // gate sums over the 32 tokens of the wavefront (butterfly over the lanes with the same half:
  // a fixed order), then over the two wavefronts of a chunk
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    float v = z[k];
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 8, 64);
    v += __shfl_xor(v, 32, 64);
    z[k] = v;
  }
  if ((lane & 47) == 0) {
#pragma unroll
    for (int k = 0; k < EPT; ++k) msw[wave * Epad + ebase + k] = z[k];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * Epad; i += 256) {
    const int c = i / Epad, e = i - c * Epad, ch = 2 * pr + c;
    if (ch < nch && e < E) {
      const size_t base = ((size_t)g * nch + ch) * E;
      msum[base + e] = msw[2 * c * Epad + e] + msw[(2 * c + 1) * Epad + e];
      hist1[base + e] = hh[c * 2 * Epad + e];
      hist2[base + e] = hh[c * 2 * Epad + Epad + e];
    }
  }
}

// Wide gates (64 < E <= 512): the NW wavefronts of a block share 128 tokens (staged
// through LDS, double buffered) and each owns ETW column tiles of 32 experts.  The
// packed weights go from L2 straight into the B operand, PB MFMA steps ahead of their use.
template <int ETW, int NW, int PB>
__global__ __launch_bounds__(64 * NW) void gate_mfma_cols_kernel(
    const bf16_t* __restrict__ x, const uint4* __restrict__ wgP, const float* __restrict__ u,
    int S, int M, int E, int nch,
    int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot, float* __restrict__ weight,
    float* __restrict__ gates_opt,
    int32_t* __restrict__ hist1, int32_t* __restrict__ hist2, float* __restrict__ msum) {
  constexpr int NT = 64 * NW, T = ETW * NW, Epad = 32 * T, pitch = Epad + 8;   // 8 mod 64: see the epilogue
  constexpr int AV = 1024 / NT;                        // 16-byte vectors of x per thread and block
  constexpr int kAPitch = 72;                          // 64 + 8 bf16: 16-byte pad
  constexpr int kABytes = 2 * 128 * kAPitch * 2;       // two stages
  constexpr int kZBytes = 64 * pitch * 4;              // logits of one chunk
  constexpr int kUnion = kABytes > kZBytes ? kABytes : kZBytes;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kUnion];
  __shared__ int hh[2 * Epad];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);
  float* zs = reinterpret_cast<float*>(smem);
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

  const int npair = (nch + 1) / 2;
  const int g = blockIdx.x / npair, pr = blockIdx.x % npair;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int KB = (M + 63) / 64;

  // cooperative x loads: 128 rows x 64 features = 1024 16-byte vectors per block of features;
  // rows past S are clamped (never used), features past M read the row start (zero weights)
  const int lrow = tid >> 3, lvec = tid & 7;           // rows lrow + (NT/8) i
  const bf16_t* xrow[AV];
#pragma unroll
  for (int i = 0; i < AV; ++i) {
    int s = pr * 128 + lrow + (NT / 8) * i;
    s = s < S ? s : S - 1;
    xrow[i] = x + ((size_t)g * S + s) * M;
  }
  f32x16_t acc[4][ETW];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int t = 0; t < ETW; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rt][t][i] = 0.f;

  // B operand of MFMA step ks (= 4 kb + j), column tile t, split sp: ring of four register
  // sets, slot ks & 3, filled PB steps ahead of its use
  const u32x4_t* bbase = reinterpret_cast<const u32x4_t*>(wgP) + (size_t)wave * ETW * 3 * 64 + lane;
  const int KS = 4 * KB;
  u32x4_t bq[4][ETW * 3];
#define MOE_GATE_LOAD_B(P, ks)                                                           \
  {                                                                                      \
    const int ksc_ = (ks) < KS ? (ks) : KS - 1;                                          \
    _Pragma("unroll") for (int q = 0; q < ETW * 3; ++q)                                  \
      bq[P][q] = bbase[((size_t)ksc_ * T * 3 + q) * 64];                                 \
  }
  // x: stage kb & 1 of LDS is multiplied while blocks kb+1 .. kb+3 sit in (or fly to)
  // register sets (kb+1)&3 .. (kb+3)&3 and block kb+4 is requested into set kb & 3:
  // a load has three iterations to land before it is written to LDS
  u32x4_t areg[4][AV];
#define MOE_GATE_LOAD_A(P, kb)                                                           \
  _Pragma("unroll") for (int i = 0; i < AV; ++i) {                                       \
    const int kbc_ = (kb) < KB ? (kb) : KB - 1;                                          \
    const int col_ = kbc_ * 64 + lvec * 8;                                               \
    areg[P][i] = *reinterpret_cast<const u32x4_t*>(xrow[i] + (col_ < M ? col_ : 0));     \
  }
#define MOE_GATE_STORE_A(P, buf)                                                         \
  _Pragma("unroll") for (int i = 0; i < AV; ++i)                                         \
    *reinterpret_cast<u32x4_t*>(As + (buf) * 128 * kAPitch +                             \
                                (lrow + (NT / 8) * i) * kAPitch + lvec * 8) = areg[P][i];
#define MOE_GATE_KBLOCK(kb, Q) /* Q = kb & 3 */                                          \
  {                                                                                      \
    MOE_GATE_LOAD_A(Q, (kb) + 4)                                                         \
    const bf16_t* as = As + ((Q) & 1) * 128 * kAPitch + r * kAPitch + 32 * h;            \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                      \
      MOE_GATE_LOAD_B((j + PB) & 3, (kb) * 4 + j + PB)                                   \
      u32x4_t af[4];                                                                     \
      _Pragma("unroll") for (int rt = 0; rt < 4; ++rt)                                   \
        af[rt] = *reinterpret_cast<const u32x4_t*>(as + rt * 32 * kAPitch + 8 * j);      \
      _Pragma("unroll") for (int t = 0; t < ETW; ++t)                                    \
        _Pragma("unroll") for (int rt = 0; rt < 4; ++rt) {                               \
          acc[rt][t] = MOE_GATE_MFMA(af[rt], bq[j][t * 3 + 2], acc[rt][t]);              \
          acc[rt][t] = MOE_GATE_MFMA(af[rt], bq[j][t * 3 + 1], acc[rt][t]);              \
          acc[rt][t] = MOE_GATE_MFMA(af[rt], bq[j][t * 3 + 0], acc[rt][t]);              \
        }                                                                                \
    }                                                                                    \
    MOE_GATE_STORE_A(((Q) + 1) & 3, ((Q) + 1) & 1) /* block kb+1 (a clamped copy at the end) */ \
    __syncthreads();                                                                     \
  }

  MOE_GATE_LOAD_A(0, 0)
  MOE_GATE_STORE_A(0, 0)
  MOE_GATE_LOAD_A(1, 1)
  MOE_GATE_LOAD_A(2, 2)
  MOE_GATE_LOAD_A(3, 3)
#pragma unroll
  for (int p = 0; p < PB; ++p) MOE_GATE_LOAD_B(p, p)
  __syncthreads();
  for (int kb = 0; kb < KB; kb += 4) {
    MOE_GATE_KBLOCK(kb, 0)
    if (kb + 1 < KB) MOE_GATE_KBLOCK(kb + 1, 1)
    if (kb + 2 < KB) MOE_GATE_KBLOCK(kb + 2, 2)
    if (kb + 3 < KB) MOE_GATE_KBLOCK(kb + 3, 3)
  }
#undef MOE_GATE_KBLOCK
#undef MOE_GATE_LOAD_A
#undef MOE_GATE_STORE_A
#undef MOE_GATE_LOAD_B
  // the A stages are dead from here on; the same LDS holds one chunk of logits at a time
#pragma unroll 1
  for (int c = 0; c < 2; ++c) {
    const int ch = pr * 2 + c;
    if (ch >= nch) break;                              // block-uniform
#pragma unroll
    for (int rr = 0; rr < 2; ++rr)
#pragma unroll
      for (int t = 0; t < ETW; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          zs[(rr * 32 + 8 * (i >> 2) + 4 * h + (i & 3)) * pitch + (wave * ETW + t) * 32 + r] =
              c == 0 ? acc[rr][t][i] : acc[2 + rr][t][i];
    __syncthreads();
    gate_chunk_epilogue<NT, Epad>(zs, pitch, g, ch, S, E, nch, u, expert_idx, slot, weight, gates_opt,
                            hist1, hist2, msum, hh, hh + Epad);
  }
}
// Wide gates, 64 < E <= 256: as gate_mfma_cols_kernel, but the x rows are fetched by four
// extra wavefronts that do nothing else.  Vector loads of one wavefront return in issue order,
// so in a wavefront that fetches both, every L2-resident weight fragment requested after an x
// block waits for that block's HBM latency; split by role, the multiplying wavefronts only wait
// for L2.  The loader wavefronts keep a ring of RD feature blocks in flight (global -> registers
// -> LDS stage); both roles pass the same barriers, one per 64-feature block.
// RT 32-token row tiles per block (4 or 8): with 256 tokens a weight fragment from L2 feeds 8 MFMA
// groups instead of 4, i.e. half the L2 traffic per token (one column tile per wavefront only:
// the accumulators of 8 x 2 tiles would fill the register file).
template <int ETW, int PB, int RB, int RT = 4>   // RB: ring of B register sets (power of two), PB < RB steps ahead
__global__ __launch_bounds__(512) void gate_mfma_cols_split_kernel(
    const bf16_t* __restrict__ x, const uint4* __restrict__ wgP, const float* __restrict__ u,
    int S, int M, int E, int nch,
    int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot, float* __restrict__ weight,
    float* __restrict__ gates_opt,
    int32_t* __restrict__ hist1, int32_t* __restrict__ hist2, float* __restrict__ msum) {
  constexpr int NW = 4, NT = 512, T = ETW * NW, Epad = 32 * T, pitch = Epad + 8;   // 8 mod 64: see the epilogue
  constexpr int ROWS = 32 * RT, CPB = RT / 2;          // tokens and chunks per block
  constexpr int AV = RT, RD = 32 / RT;                 // loader: 16-byte vectors per thread and block, ring depth
  constexpr int kAPitch = 72;                          // 64 + 8 bf16: 16-byte pad
  constexpr int kABytes = 2 * ROWS * kAPitch * 2;      // two stages
  constexpr int kZBytes = 64 * pitch * 4;              // logits of one chunk
  constexpr int kUnion = kABytes > kZBytes ? kABytes : kZBytes;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kUnion];
  __shared__ int hh[2 * Epad];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);
  float* zs = reinterpret_cast<float*>(smem);
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

  const int npair = (nch + CPB - 1) / CPB;
  const int g = blockIdx.x / npair, pr = blockIdx.x % npair;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int KB = (M + 63) / 64;

  f32x16_t acc[RT][ETW];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int t = 0; t < ETW; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rt][t][i] = 0.f;

  if (wave >= NW) {
    // ---- loader wavefronts: ROWS rows x 64 features = 8 ROWS 16-byte vectors per feature block;
    // rows past S are clamped (never used), features past M read the row start (zero weights)
    const int lt = tid - 64 * NW, lrow = lt >> 3, lvec = lt & 7;   // rows lrow + 32 i
    const bf16_t* xrow[AV];
#pragma unroll
    for (int i = 0; i < AV; ++i) {
      int s = pr * ROWS + lrow + 32 * i;
      s = s < S ? s : S - 1;
      xrow[i] = x + ((size_t)g * S + s) * M;
    }
    u32x4_t areg[RD][AV];
#define MOE_GATE_LOAD_A(P, kb)                                                           \
  _Pragma("unroll") for (int i = 0; i < AV; ++i) {                                       \
    const int kbc_ = (kb) < KB ? (kb) : KB - 1;                                          \
    const int col_ = kbc_ * 64 + lvec * 8;                                               \
    areg[P][i] = *reinterpret_cast<const u32x4_t*>(xrow[i] + (col_ < M ? col_ : 0));     \
  }
#define MOE_GATE_STORE_A(P, buf)                                                         \
  _Pragma("unroll") for (int i = 0; i < AV; ++i)                                         \
    *reinterpret_cast<u32x4_t*>(As + (buf) * ROWS * kAPitch + (lrow + 32 * i) * kAPitch + lvec * 8) = areg[P][i];
    MOE_GATE_LOAD_A(0, 0)
#pragma unroll
    for (int p = 1; p < RD; ++p) MOE_GATE_LOAD_A(p, p)
    MOE_GATE_STORE_A(0, 0)
    __syncthreads();
    for (int kb0 = 0; kb0 < KB; kb0 += RD) {
#pragma unroll
      for (int q = 0; q < RD; ++q) {
        if (kb0 + q < KB) {                            // block-uniform
          // block kb0+q is being multiplied from stage q&1: its ring slot is free again, and
          // block kb0+q+1 (a clamped copy at the end) goes into the other stage
          MOE_GATE_LOAD_A(q, kb0 + q + RD)
          MOE_GATE_STORE_A((q + 1) % RD, (q + 1) & 1)
          __syncthreads();
        }
      }
    }
#undef MOE_GATE_LOAD_A
#undef MOE_GATE_STORE_A
  } else {
    // ---- multiplying wavefronts: B operand of MFMA step ks (= 4 kb + j), column tile t, split
    // sp: ring of RB register sets, slot ks % RB, filled PB steps ahead of its use
    const u32x4_t* bbase = reinterpret_cast<const u32x4_t*>(wgP) + (size_t)wave * ETW * 3 * 64 + lane;
    const int KS = 4 * KB;
    u32x4_t bq[RB][ETW * 3];
#define MOE_GATE_LOAD_B(P, ks)                                                           \
  {                                                                                      \
    const int ksc_ = (ks) < KS ? (ks) : KS - 1;                                          \
    _Pragma("unroll") for (int q = 0; q < ETW * 3; ++q)                                  \
      bq[P][q] = bbase[((size_t)ksc_ * T * 3 + q) * 64];                                 \
  }
#pragma unroll
    for (int p = 0; p < PB; ++p) MOE_GATE_LOAD_B(p, p)
    __syncthreads();
    constexpr int KU = RB / 4;                          // feature blocks per trip: slots stay static
    for (int kb0 = 0; kb0 < KB; kb0 += KU) {
#pragma unroll
      for (int ku = 0; ku < KU; ++ku) {
        const int kb = kb0 + ku;
        if (kb < KB) {                                  // block-uniform
          const bf16_t* as = As + (kb & 1) * ROWS * kAPitch + r * kAPitch + 32 * h;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            MOE_GATE_LOAD_B((4 * ku + j + PB) % RB, kb * 4 + j + PB)
            u32x4_t af[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
              af[rt] = *reinterpret_cast<const u32x4_t*>(as + rt * 32 * kAPitch + 8 * j);
#pragma unroll
            for (int t = 0; t < ETW; ++t)
#pragma unroll
              for (int sp = 2; sp >= 0; --sp)           // smallest term first; RT independent MFMAs in a row
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                  acc[rt][t] = MOE_GATE_MFMA(af[rt], bq[(4 * ku + j) % RB][t * 3 + sp], acc[rt][t]);
          }
          __syncthreads();
        }
      }
    }
#undef MOE_GATE_LOAD_B
  }
  // the A stages are dead from here on; the same LDS holds one chunk of logits at a time
#pragma unroll
  for (int c = 0; c < CPB; ++c) {
    const int ch = pr * CPB + c;
    if (ch < nch) {                                    // block-uniform
      if (wave < NW) {
#pragma unroll
        for (int rr = 0; rr < 2; ++rr)
#pragma unroll
          for (int t = 0; t < ETW; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i)
              zs[(rr * 32 + 8 * (i >> 2) + 4 * h + (i & 3)) * pitch + (wave * ETW + t) * 32 + r] =
                  acc[2 * c + rr][t][i];
      }
      __syncthreads();
      gate_chunk_epilogue<NT, Epad>(zs, pitch, g, ch, S, E, nch, u, expert_idx, slot, weight, gates_opt,
                              hist1, hist2, msum, hh, hh + Epad);
    }
  }
}
#undef MOE_GATE_MFMA

// One block per (group, 32 experts); thread (e, k) owns expert e and the k-th of 8
// contiguous segments of the chunk axis.  hist1/hist2 are replaced by their exclusive
// prefix over chunks; hist2's prefix starts at c1 (second choices queue behind all first
// choices).  Two passes over the segment (sum, then prefix) with a tiny LDS scan between.
__global__ __launch_bounds__(256) void gate_scan_kernel(
    int S, int E, int C, int G, int nch,
    int32_t* __restrict__ hist1, int32_t* __restrict__ hist2, const float* __restrict__ msum,
    int32_t* __restrict__ c1, float* __restrict__ mean_gate, int32_t* __restrict__ fill,
    int32_t* __restrict__ src_token) {
  __shared__ int t1[8][32], t2[8][32];
  __shared__ float tm[8][32];
  const int etiles = (E + 31) / 32;
  const int g = blockIdx.x / etiles, e = (blockIdx.x % etiles) * 32 + (threadIdx.x & 31);
  const int k = threadIdx.x >> 5;
  const int seg = (nch + 7) / 8;
  const int ch0 = k * seg, ch1 = (ch0 + seg < nch) ? ch0 + seg : nch;
  const bool live = e < E;
  // the loads of a batch of UN chunks are independent (one memory latency per batch); a segment
  // that fits one batch stays in registers for the second pass
  constexpr int UN = 8;
  const bool single = seg <= UN;
  int a1[UN], a2[UN];
  int s1 = 0, s2 = 0;
  float ms = 0.f;
  if (live)
    for (int c0 = ch0; c0 < ch1; c0 += UN) {
      float am[UN];
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        const bool in = c0 + j < ch1;
        const size_t i = ((size_t)g * nch + (in ? c0 + j : ch0)) * E + e;
        a1[j] = in ? hist1[i] : 0;
        a2[j] = in ? hist2[i] : 0;
        am[j] = in ? msum[i] : 0.f;
      }
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        s1 += a1[j];
        s2 += a2[j];
        if (c0 + j < ch1) ms += am[j];                // chunk order, as a plain loop would add
      }
    }
  t1[k][threadIdx.x & 31] = s1;
  t2[k][threadIdx.x & 31] = s2;
  tm[k][threadIdx.x & 31] = ms;
  __syncthreads();
  if (!live) return;
  int base1 = 0, base2 = 0, tot1 = 0, tot2 = 0;
  float mtot = 0.f;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    const int a = t1[kk][threadIdx.x & 31], b = t2[kk][threadIdx.x & 31];
    if (kk < k) { base1 += a; base2 += b; }
    tot1 += a;
    tot2 += b;
    mtot += tm[kk][threadIdx.x & 31];
  }
  int run1 = base1, run2 = base2 + tot1;
  for (int c0 = ch0; c0 < ch1; c0 += UN) {
    if (!single) {
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        const bool in = c0 + j < ch1;
        const size_t i = ((size_t)g * nch + (in ? c0 + j : ch0)) * E + e;
        a1[j] = in ? hist1[i] : 0;
        a2[j] = in ? hist2[i] : 0;
      }
    }
#pragma unroll
    for (int j = 0; j < UN; ++j)
      if (c0 + j < ch1) {
        const size_t i = ((size_t)g * nch + c0 + j) * E + e;
        hist1[i] = run1; run1 += a1[j];
        hist2[i] = run2; run2 += a2[j];
      }
  }
  const long long tot = (long long)tot1 + tot2;
  const int f = tot < C ? (int)tot : C;
  if (k == 0) {
    c1[(size_t)g * E + e] = tot1;
    mean_gate[(size_t)g * E + e] = mtot / (float)S;
    fill[(size_t)g * E + e] = f;
  }
  int32_t* st = src_token + ((size_t)e * G + g) * C;
  for (int c = f + k; c < C; c += 8) st[c] = -1;
}

// One wavefront per chunk.  pk.packed_src != NULL: also builds the packed row layout of the
// expert GEMMs (row of a kept choice = kept rows of the same expert in earlier groups + slot).
__global__ __launch_bounds__(64) void gate_slots_kernel(
    int S, int E, int C, int G, int nch,
    const int32_t* __restrict__ base1, const int32_t* __restrict__ base2,
    const int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot,
    float* __restrict__ weight, int32_t* __restrict__ src_token,
    const int32_t* __restrict__ c1, const float* __restrict__ mean_gate, float* __restrict__ aux,
    uint32_t* __restrict__ zero_fill, int zero_words, const int32_t* __restrict__ fill, RowPacking pk) {
  const int g = blockIdx.x / nch, ch = blockIdx.x % nch;
  const int lane = threadIdx.x;
  const bool packing = pk.packed_src != nullptr;
  // optional: clear the all-zero activation row that stands in for empty expert slots when
  // the first expert GEMM gathers its rows from x
  if (blockIdx.x == 0)
    for (int i = lane; i < zero_words; i += 64) zero_fill[i] = 0u;
  if (ch == 0) {
    // l_aux[g] = (1/E) sum_e (c1/S) m_e, summed in a fixed order (lane-strided, then a tree)
    float part = 0.f;
    for (int e = lane; e < E; e += 64)
      part += ((float)c1[(size_t)g * E + e] / (float)S) * mean_gate[(size_t)g * E + e];
    part = wave_sum(part);
    if (lane == 0) aux[g] = part / (float)E;
  }
  // packed layout: row_base[:, e] = running sum of fill[:, e] over the groups, 64 experts per
  // block (coalesced rows of fill, G loads per lane)
  if (packing)
    for (int e = 64 * blockIdx.x + lane; e < E; e += 64 * gridDim.x) {   // no wave-level ops inside
      int run = 0;
      for (int gg = 0; gg < G; ++gg) {
        pk.row_base[(size_t)gg * E + e] = run;
        run += fill[(size_t)gg * E + e];
      }
      pk.kept[e] = run;
    }
  const int s = ch * kChunk + lane;
  const bool valid = s < S;
  const size_t n = (size_t)g * S + (valid ? s : 0);
  int e1 = -1, e2 = -1;      // -1: takes part in no ranking
  bool sampled = false;
  if (valid) {
    e1 = expert_idx[2 * n];
    sampled = slot[2 * n + 1] != MOE_SLOT_NOT_SAMPLED;
    if (sampled) e2 = expert_idx[2 * n + 1];
  }
  // packed layout: kept rows of the two experts in the groups before this one (loads that the
  // rank loop below hides)
  // Up to 128 experts: lane l sums the columns l and l + 64 of fill (coalesced) and the sums
  // meet in LDS after the rank loop; wider gates: every lane sums the columns of its own two
  // experts.
  __shared__ int rb_s[128];
  const bool rb_shared = E <= 128;
  int rb1 = 0, rb2 = 0;
  if (packing) {
    const int ca = rb_shared ? (lane < E ? lane : -1) : e1;
    const int cb = rb_shared ? (lane + 64 < E ? lane + 64 : -1) : e2;
    for (int gg = 0; gg < g; ++gg) {
      if (ca >= 0) rb1 += fill[(size_t)gg * E + ca];
      if (cb >= 0) rb2 += fill[(size_t)gg * E + cb];
    }
  }
  // stable rank among the earlier tokens of the chunk with the same expert: the lanes that agree
  // with this one in every bit of the expert index, one ballot per bit
  unsigned long long peers1 = __ballot(e1 >= 0), peers2 = __ballot(e2 >= 0);
  for (int bit = 0; (E - 1) >> bit; ++bit) {
    const bool b1 = (e1 >> bit) & 1, b2 = (e2 >> bit) & 1;
    const unsigned long long m1 = __ballot(b1), m2 = __ballot(b2);
    peers1 &= b1 ? m1 : ~m1;
    peers2 &= b2 ? m2 : ~m2;
  }
  const unsigned long long earlier = (1ull << lane) - 1;
  const int r1 = __popcll(peers1 & earlier), r2 = __popcll(peers2 & earlier);
  if (packing && rb_shared) {
    rb_s[lane] = rb1;
    rb_s[lane + 64] = rb2;
    __syncthreads();                                  // the block is this one wavefront
    rb1 = e1 >= 0 ? rb_s[e1] : 0;
    rb2 = e2 >= 0 ? rb_s[e2] : 0;
  }
  if (!valid) return;
  const size_t cb = ((size_t)g * nch + ch) * E;
  const int p1 = base1[cb + e1] + r1;
  const int s1 = p1 < C ? p1 : MOE_SLOT_OVERFLOW;
  int s2 = MOE_SLOT_NOT_SAMPLED;
  if (sampled) {
    const int p2 = base2[cb + e2] + r2;
    s2 = p2 < C ? p2 : MOE_SLOT_OVERFLOW;
  }
  slot[2 * n] = s1;
  slot[2 * n + 1] = s2;
  if (s1 < 0) weight[2 * n] = 0.f;
  if (s2 < 0) weight[2 * n + 1] = 0.f;
  if (s1 >= 0) src_token[((size_t)e1 * G + g) * C + s1] = s;
  if (s2 >= 0) src_token[((size_t)e2 * G + g) * C + s2] = s;
  if (packing) {
    const size_t R = (size_t)G * C;
    if (s1 >= 0) pk.packed_src[(size_t)e1 * R + rb1 + s1] = (int32_t)n;
    if (s2 >= 0) pk.packed_src[(size_t)e2 * R + rb2 + s2] = (int32_t)n;
  }
}

// The packed row layout from fill alone, for expert buffers in the [E,G,C,M] order of the staged
// entry points: row p of expert e comes from (and goes back to) row (e G + g) C + c of the buffer.
__global__ __launch_bounds__(64) void row_maps_from_fill_kernel(
    int E, int G, int C, const int32_t* __restrict__ fill, RowPacking pk,
    uint32_t* __restrict__ zero_fill, int zero_words) {
  const int lane = threadIdx.x;
  if (blockIdx.x == 0)
    for (int i = lane; i < zero_words; i += 64) zero_fill[i] = 0u;
  const size_t R = (size_t)G * C;
  const long long idx = (long long)blockIdx.x * 64 + lane;
  if (idx >= (long long)E * G * C) return;
  const int c = (int)(idx % C), g = (int)((idx / C) % G), e = (int)(idx / ((long long)C * G));
  int rb = 0;
  for (int gg = 0; gg < g; ++gg) rb += fill[(size_t)gg * E + e];
  if (c == 0) {
    pk.row_base[(size_t)g * E + e] = rb;
    if (g == G - 1) pk.kept[e] = rb + fill[(size_t)g * E + e];
  }
  if (c < fill[(size_t)g * E + e]) pk.packed_src[(size_t)e * R + rb + c] = (int32_t)idx;
}

template <typename T, bool PRE = false>
int launch_topk(const moe_config& c, int nch, const T* x, const float* wg, const float* u,
                int32_t* expert_idx, int32_t* slot, float* weight, float* gates_opt,
                int32_t* hist1, int32_t* hist2, float* msum, hipStream_t st,
                const float* zpre = nullptr, int cols = 0) {
  const size_t shm = ((PRE ? 0 : (size_t)4 * c.M) + (size_t)4 * c.E) * sizeof(float) +
                     (size_t)2 * c.E * sizeof(int);
  if (shm > 64 * 1024) return MOE_EUNSUPPORTED;   // the default dynamic LDS limit of a kernel
  const dim3 grid((unsigned)(c.G * nch)), block(256);
  const int epl = (c.E + 63) / 64;
#define MOE_GATE_CASE(N)                                                                        \
  hipLaunchKernelGGL((gate_topk_kernel<T, N, PRE>), grid, block, shm, st, x, wg, u, zpre, cols, \
                     c.S, c.M, c.E, nch, expert_idx, slot, weight, gates_opt, hist1, hist2, msum)
  if (epl <= 1) MOE_GATE_CASE(1);
  else if (epl <= 2) MOE_GATE_CASE(2);
  else if (epl <= 4) MOE_GATE_CASE(4);
  else if (epl <= 8) MOE_GATE_CASE(8);
  else if (epl <= 16) MOE_GATE_CASE(16);
  else if (epl <= 32) MOE_GATE_CASE(32);
  else return MOE_EUNSUPPORTED;  // more than 2048 experts
#undef MOE_GATE_CASE
  return check_launch();
}

}  // namespace

// Very wide gates (E > 512): wgk[3e+p, m] = term p of wg[m,e] (hi, mid, lo bf16 terms), rows
// past 3E zero: the K-contiguous B operand of a plain GEMM x . wgk^T whose fp32 result holds the
// three partial logits of every expert side by side.
namespace {
// K = reps * M: the row is repeated `reps` times along K (fp32 activations enter the product as
// three bf16 terms side by side, each of which meets every term of wg).
__global__ __launch_bounds__(256) void gate_pack_wide_kernel(
    const float* __restrict__ wg, bf16_t* __restrict__ wgk, int M, int E, int cols, int reps) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  const int K = reps * M;
  if (i >= (long long)cols * K) return;
  const int c = (int)(i / K), m = (int)(i % K) % M;
  bf16_t out = 0;
  if (c < 3 * E) {
    const float v = wg[(size_t)m * E + c / 3];
    const bf16_t hi = f32_to_bf16(v);
    const float r1 = v - bf16_to_f32(hi);
    const bf16_t mid = f32_to_bf16(r1);
    const bf16_t lo = f32_to_bf16(r1 - bf16_to_f32(mid));
    out = c % 3 == 0 ? hi : (c % 3 == 1 ? mid : lo);
  }
  wgk[i] = out;
}

// xk[n, a*M + m] = term a (hi, mid, lo) of the fp32 activation x[n,m]: x = hi + mid + lo exactly
__global__ __launch_bounds__(256) void gate_split_x_kernel(
    const float* __restrict__ x, bf16_t* __restrict__ xk, int M, long long tokens) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= tokens * M) return;
  const long long n = i / M;
  const int m = (int)(i % M);
  const float v = x[i];
  const bf16_t hi = f32_to_bf16(v);
  const float r1 = v - bf16_to_f32(hi);
  const bf16_t mid = f32_to_bf16(r1);
  bf16_t* d = xk + n * 3 * M + m;
  d[0] = hi;
  d[M] = mid;
  d[2 * (size_t)M] = f32_to_bf16(r1 - bf16_to_f32(mid));
}
}  // namespace

// Logits as one GEMM on the matrix cores, for bf16 gates wider than 512 experts and for fp32
// activations (x split into three bf16 terms, K = 3 M): needs the persistent GEMM's shapes (token
// count a multiple of 256, K of 32) and at most 2048 experts (registers of the epilogue kernel).
struct WideGeom { int cols, k; size_t z_bytes, w_bytes, x_bytes; };
static WideGeom wide_geom(const moe_config& c) {
  WideGeom w{};
  const long long tokens = (long long)c.G * c.S;
  const long long cols = ((long long)3 * c.E + 255) / 256 * 256;
  const long long k = c.act_dtype == MOE_F32 ? (long long)3 * c.M : c.M;
  if ((c.act_dtype == MOE_BF16 && c.E <= 512) || c.E > 2048 || tokens > 0x7fffffffLL ||
      k > 0x7fffffffLL || !gemm_bf16_f32out_ok((int)tokens, (int)cols, (int)k))
    return w;
  w.cols = (int)cols;
  w.k = (int)k;
  w.z_bytes = (size_t)tokens * cols * 4;
  w.w_bytes = (size_t)cols * k * 2;
  w.x_bytes = c.act_dtype == MOE_F32 ? (size_t)tokens * k * 2 : 0;
  return w;
}

// Geometry of the packed gate weights (bf16 MFMA path).
struct PackGeom { int T, KS; size_t bytes; };
static PackGeom pack_geom(const moe_config& c) {
  PackGeom p{};
  if (c.act_dtype != MOE_BF16 || c.E > 512) return p;   // bytes == 0: plain kernel
  const int epad = c.E <= 64 ? (c.E + 31) / 32 * 32 : c.E <= 128 ? 128 : c.E <= 256 ? 256 : 512;
  p.T = epad / 32;
  p.KS = (c.M + 63) / 64 * 4;
  p.bytes = (size_t)p.KS * p.T * 3 * 64 * 16;
  return p;
}

size_t gate_workspace_bytes(const moe_config& c) {
  const size_t nch = (size_t)(c.S + kChunk - 1) / kChunk;
  const WideGeom w = wide_geom(c);
  return 3 * align_up((size_t)c.G * nch * c.E * 4, 256) + align_up(pack_geom(c).bytes, 256) +
         align_up(w.w_bytes, 256) + align_up(w.z_bytes, 256) + align_up(w.x_bytes, 256);
}

// The gate weights in the form the logit kernels multiply: three bf16 terms per weight in the
// MFMA operand order (E <= 512, bf16 activations) or as the K-contiguous operand of the logit
// GEMM (wider gates, fp32 activations with GEMM-friendly shapes); 0 bytes when the gate reads
// wg as it is.
size_t gate_pack_bytes(const moe_config& c) {
  const PackGeom pg = pack_geom(c);
  return pg.bytes != 0 ? pg.bytes : wide_geom(c).w_bytes;
}

int launch_gate_pack(const moe_config& c, const float* wg, void* packed, hipStream_t st) {
  const WideGeom w = wide_geom(c);
  if (w.cols != 0) {
    const long long n = (long long)w.cols * w.k;
    hipLaunchKernelGGL(gate_pack_wide_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, wg,
                       static_cast<bf16_t*>(packed), c.M, c.E, w.cols, w.k / c.M);
    return check_launch();
  }
  const PackGeom pg = pack_geom(c);
  if (pg.bytes == 0) return MOE_OK;
  const int total = pg.KS * pg.T * 64;
  hipLaunchKernelGGL(gate_pack_wg_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, wg,
                     static_cast<uint4*>(packed), c.M, c.E, pg.T, total);
  return check_launch();
}

// partial logits [4][128][Epad + 4], per-wavefront gate sums [4][Epad], histograms [4][Epad]
constexpr size_t kGateRowsLds1 = (4 * 128 * 36 + 8 * 32) * 4, kGateRowsLds2 = (4 * 128 * 68 + 8 * 64) * 4;

int prepare_gate() {
  static LdsLimitOnce once1, once2;
  const int rc = ensure_lds_limit(once1, reinterpret_cast<const void*>(gate_mfma_rows_kernel<1>),
                                  (int)kGateRowsLds1);
  if (rc != MOE_OK) return rc;
  return ensure_lds_limit(once2, reinterpret_cast<const void*>(gate_mfma_rows_kernel<2>),
                          (int)kGateRowsLds2);
}

int launch_gate(const moe_config& c, const void* x, const float* wg, const float* u,
                int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
                int32_t* src_token, int32_t* c1, float* mean_gate, float* aux,
                float* gates_opt, void* ws, void* zero_row, const RowPacking* packing,
                const void* wg_prepacked, hipStream_t st) {
  const int nch = (c.S + kChunk - 1) / kChunk;
  const size_t seg = align_up((size_t)c.G * nch * c.E * 4, 256);
  int32_t* hist1 = reinterpret_cast<int32_t*>(ws);
  int32_t* hist2 = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + seg);
  float* msum = reinterpret_cast<float*>(static_cast<char*>(ws) + 2 * seg);
  // the packed weights: the caller's (packed once with launch_gate_pack) or this call's own
  char* const own = static_cast<char*>(ws) + 3 * seg;
  uint4* wgP = wg_prepacked != nullptr ? static_cast<uint4*>(const_cast<void*>(wg_prepacked))
                                        : reinterpret_cast<uint4*>(own);
  const PackGeom pg = pack_geom(c);
  int rc;
  if (wg_prepacked == nullptr && (rc = launch_gate_pack(c, wg, own, st)) != MOE_OK) return rc;
  if (wide_geom(c).cols != 0) {
    // pg.bytes == 0 here: the packed-operand region is empty; wgk, the logits and (fp32) the
    // split activations follow it
    const WideGeom w = wide_geom(c);
    const long long tokens = (long long)c.G * c.S;
    const bf16_t* wgk = reinterpret_cast<const bf16_t*>(wgP);
    char* after = own + align_up(w.w_bytes, 256);
    float* zpre = reinterpret_cast<float*>(after);
    bf16_t* xk = reinterpret_cast<bf16_t*>(after + align_up(w.z_bytes, 256));
    const void* a = x;
    if (c.act_dtype == MOE_F32) {
      hipLaunchKernelGGL(gate_split_x_kernel, dim3((unsigned)((tokens * c.M + 255) / 256)), dim3(256),
                         0, st, static_cast<const float*>(x), xk, c.M, tokens);
      if ((rc = check_launch()) != MOE_OK) return rc;
      a = xk;
    }
    rc = launch_gemm_bf16_f32out(false, a, wgk, zpre, 1, (int)tokens, w.cols, w.k, st);
    if (rc != MOE_OK) return rc;
    rc = c.act_dtype == MOE_F32
             ? launch_topk<float, true>(c, nch, static_cast<const float*>(x), wg, u, expert_idx, slot,
                                        weight, gates_opt, hist1, hist2, msum, st, zpre, w.cols)
             : launch_topk<bf16_t, true>(c, nch, static_cast<const bf16_t*>(x), wg, u, expert_idx,
                                         slot, weight, gates_opt, hist1, hist2, msum, st, zpre, w.cols);
  } else if (c.act_dtype == MOE_F32) {
    rc = launch_topk<float>(c, nch, static_cast<const float*>(x), wg, u, expert_idx, slot, weight,
                            gates_opt, hist1, hist2, msum, st);
  } else if (pg.bytes == 0) {
    rc = launch_topk<bf16_t>(c, nch, static_cast<const bf16_t*>(x), wg, u, expert_idx, slot,
                             weight, gates_opt, hist1, hist2, msum, st);
  } else {
    const dim3 grid((unsigned)(c.G * ((nch + 1) / 2))), block(256);
    const bf16_t* xb = static_cast<const bf16_t*>(x);
#define MOE_GATE_ARGS xb, wgP, u, c.S, c.M, c.E, nch, expert_idx, slot, weight, gates_opt, hist1, hist2, msum
    if (c.E <= 64) {
      const size_t lds1 = kGateRowsLds1, lds2 = kGateRowsLds2;
      if (prepare_gate() != MOE_OK) return MOE_EHIP;
      if (c.E <= 32) hipLaunchKernelGGL(gate_mfma_rows_kernel<1>, grid, block, lds1, st, MOE_GATE_ARGS);
      else hipLaunchKernelGGL(gate_mfma_rows_kernel<2>, grid, block, lds2, st, MOE_GATE_ARGS);
    }
    else if (c.E <= 128) {
      // 256-token blocks once they give every compute unit a block
      int cus = 0;
      if (compute_units(&cus) != MOE_OK) return MOE_EHIP;
      const long long blocks256 = (long long)c.G * ((nch + 3) / 4);
      if (blocks256 >= cus)
        hipLaunchKernelGGL((gate_mfma_cols_split_kernel<1, 6, 8, 8>), dim3((unsigned)blocks256), dim3(512), 0, st, MOE_GATE_ARGS);
      else
        hipLaunchKernelGGL((gate_mfma_cols_split_kernel<1, 6, 8>), grid, dim3(512), 0, st, MOE_GATE_ARGS);
    }
    else if (c.E <= 256) hipLaunchKernelGGL((gate_mfma_cols_split_kernel<2, 2, 4>), grid, dim3(512), 0, st, MOE_GATE_ARGS);
    else hipLaunchKernelGGL((gate_mfma_cols_kernel<2, 8, 2>), grid, dim3(512), 0, st, MOE_GATE_ARGS);
#undef MOE_GATE_ARGS
    rc = check_launch();
  }
  if (rc != MOE_OK) return rc;
  hipLaunchKernelGGL(gate_scan_kernel, dim3((unsigned)(c.G * ((c.E + 31) / 32))), dim3(256), 0, st,
                     c.S, c.E, c.C, c.G, nch, hist1, hist2, msum, c1, mean_gate, fill, src_token);
  if ((rc = check_launch()) != MOE_OK) return rc;
  hipLaunchKernelGGL(gate_slots_kernel, dim3((unsigned)(c.G * nch)), dim3(64), 0, st, c.S, c.E,
                     c.C, c.G, nch, hist1, hist2, expert_idx, slot, weight, src_token, c1,
                     mean_gate, aux, static_cast<uint32_t*>(zero_row),
                     zero_row != nullptr ? c.M / 2 : 0, fill,
                     packing != nullptr ? *packing : RowPacking{nullptr, nullptr, nullptr});
  return check_launch();
}

int launch_row_maps_from_fill(const moe_config& c, const int32_t* fill, const RowPacking& pk,
                              void* zero_row, hipStream_t st) {
  const long long slots = (long long)c.E * c.G * c.C;
  hipLaunchKernelGGL(row_maps_from_fill_kernel, dim3((unsigned)((slots + 63) / 64)), dim3(64), 0, st,
                     c.E, c.G, c.C, fill, pk, static_cast<uint32_t*>(zero_row),
                     zero_row != nullptr ? c.M / 2 : 0);
  return check_launch();
}

}  // namespace moe
