// Top2Gating (Algorithm 1 of the paper, for G independent groups) in three kernels:
//
//   gate_topk_kernel    per token: logits x.wg, softmax, top-2, renormalised gates,
//                       the random-routing decision; per 64-token chunk: histogram of
//                       first choices / sampled second choices and the gate sums
//   gate_scan_kernel    per group: exclusive scan of the chunk histograms over the
//                       chunks (the running counters c_E of Algorithm 1 at chunk
//                       boundaries), c1, mean gates m_E, l_aux, fill, empty slots
//   gate_slots_kernel   per chunk: stable rank of every token among the earlier
//                       tokens of its chunk with the same expert + the chunk base
//                       = position in the expert buffer; capacity test; combine
//                       weights; inverse map slot -> token
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
template <typename T, int EPL>
__global__ __launch_bounds__(256) void gate_topk_kernel(
    const T* __restrict__ x, const float* __restrict__ wg, const float* __restrict__ u,
    int S, int M, int E, int nch,
    int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot, float* __restrict__ weight,
    float* __restrict__ gates_opt,
    int32_t* __restrict__ hist1, int32_t* __restrict__ hist2, float* __restrict__ msum) {
  extern __shared__ unsigned char smem[];
  const int g = blockIdx.x / nch, ch = blockIdx.x % nch;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* xs = reinterpret_cast<float*>(smem) + (size_t)wave * M;  // this wave's token row
  float* msum_l = reinterpret_cast<float*>(smem) + (size_t)4 * M;  // [4][E]
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
    for (int m = lane; m < M; m += 64) xs[m] = Elt<T>::load(x + n * M + m);
    __syncthreads();
    if (!valid) continue;  // both barriers of the next iteration are still reached

    float z[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) z[j] = 0.f;
    for (int m = 0; m < M; ++m) {
      const float xv = xs[m];
      const float* wrow = wg + (size_t)m * E;
#pragma unroll
      for (int j = 0; j < EPL; ++j) {
        const int e = lane + 64 * j;
        if (e < E) z[j] = fmaf(xv, wrow[e], z[j]);
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

// One block per group.  hist1/hist2 are replaced by their exclusive prefix over
// chunks; hist2's prefix starts at c1 (second choices queue behind all first ones).
__global__ __launch_bounds__(256) void gate_scan_kernel(
    int S, int E, int C, int G, int nch,
    int32_t* __restrict__ hist1, int32_t* __restrict__ hist2, const float* __restrict__ msum,
    int32_t* __restrict__ c1, float* __restrict__ mean_gate, int32_t* __restrict__ fill,
    int32_t* __restrict__ src_token, float* __restrict__ aux) {
  __shared__ float red[256];
  const int g = blockIdx.x;
  float part = 0.f;
  for (int e = threadIdx.x; e < E; e += 256) {
    int run1 = 0, run2 = 0;
    float ms = 0.f;
    for (int ch = 0; ch < nch; ++ch) {
      const size_t i = ((size_t)g * nch + ch) * E + e;
      const int a = hist1[i]; hist1[i] = run1; run1 += a;
      const int b = hist2[i]; hist2[i] = run2; run2 += b;
      ms += msum[i];
    }
    for (int ch = 0; ch < nch; ++ch) hist2[((size_t)g * nch + ch) * E + e] += run1;
    const float mg = ms / (float)S;
    c1[(size_t)g * E + e] = run1;
    mean_gate[(size_t)g * E + e] = mg;
    const long long tot = (long long)run1 + run2;
    const int f = tot < C ? (int)tot : C;
    fill[(size_t)g * E + e] = f;
    int32_t* st = src_token + ((size_t)e * G + g) * C;
    for (int c = f; c < C; ++c) st[c] = -1;
    part += ((float)run1 / (float)S) * mg;
  }
  red[threadIdx.x] = part;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) aux[g] = red[0] / (float)E;
}

// One wavefront per chunk.
__global__ __launch_bounds__(64) void gate_slots_kernel(
    int S, int E, int C, int G, int nch,
    const int32_t* __restrict__ base1, const int32_t* __restrict__ base2,
    const int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot,
    float* __restrict__ weight, int32_t* __restrict__ src_token) {
  const int g = blockIdx.x / nch, ch = blockIdx.x % nch;
  const int lane = threadIdx.x;
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
  int r1 = 0, r2 = 0;
  for (int i = 0; i < kChunk - 1; ++i) {
    const int o1 = __shfl(e1, i, 64);
    const int o2 = __shfl(e2, i, 64);
    if (i < lane) {
      r1 += (o1 == e1);
      r2 += (o2 == e2);
    }
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
}

template <typename T>
int launch_topk(const moe_config& c, int nch, const T* x, const float* wg, const float* u,
                int32_t* expert_idx, int32_t* slot, float* weight, float* gates_opt,
                int32_t* hist1, int32_t* hist2, float* msum, hipStream_t st) {
  const size_t shm = ((size_t)4 * c.M + (size_t)4 * c.E) * sizeof(float) + (size_t)2 * c.E * sizeof(int);
  if (shm > 160 * 1024) return MOE_EUNSUPPORTED;
  const dim3 grid((unsigned)(c.G * nch)), block(256);
  const int epl = (c.E + 63) / 64;
#define MOE_GATE_CASE(N)                                                                        \
  hipLaunchKernelGGL((gate_topk_kernel<T, N>), grid, block, shm, st, x, wg, u, c.S, c.M, c.E,  \
                     nch, expert_idx, slot, weight, gates_opt, hist1, hist2, msum)
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

size_t gate_workspace_bytes(const moe_config& c) {
  const size_t nch = (size_t)(c.S + kChunk - 1) / kChunk;
  return 3 * align_up((size_t)c.G * nch * c.E * 4, 256);
}

int launch_gate(const moe_config& c, const void* x, const float* wg, const float* u,
                int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
                int32_t* src_token, int32_t* c1, float* mean_gate, float* aux,
                float* gates_opt, void* ws, hipStream_t st) {
  const int nch = (c.S + kChunk - 1) / kChunk;
  const size_t seg = align_up((size_t)c.G * nch * c.E * 4, 256);
  int32_t* hist1 = reinterpret_cast<int32_t*>(ws);
  int32_t* hist2 = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + seg);
  float* msum = reinterpret_cast<float*>(static_cast<char*>(ws) + 2 * seg);
  int rc;
  if (c.act_dtype == MOE_F32)
    rc = launch_topk<float>(c, nch, static_cast<const float*>(x), wg, u, expert_idx, slot, weight,
                            gates_opt, hist1, hist2, msum, st);
  else
    rc = launch_topk<bf16_t>(c, nch, static_cast<const bf16_t*>(x), wg, u, expert_idx, slot,
                             weight, gates_opt, hist1, hist2, msum, st);
  if (rc != MOE_OK) return rc;
  hipLaunchKernelGGL(gate_scan_kernel, dim3((unsigned)c.G), dim3(256), 0, st, c.S, c.E, c.C, c.G,
                     nch, hist1, hist2, msum, c1, mean_gate, fill, src_token, aux);
  if ((rc = check_launch()) != MOE_OK) return rc;
  hipLaunchKernelGGL(gate_slots_kernel, dim3((unsigned)(c.G * nch)), dim3(64), 0, st, c.S, c.E,
                     c.C, c.G, nch, hist1, hist2, expert_idx, slot, weight, src_token);
  return check_launch();
}

}  // namespace moe
