// Dispatch and combine of Algorithm 2, computed as row gathers instead of the
// one-hot einsums (the gather form is the one Section 3.2 sketches):
//
//   dispatch: buf[e,g,c,:] = x[g, src_token[e,g,c], :]       (zeros for empty slots)
//   combine : y[g,s,:]     = sum_k weight[g,s,k] * out[e_k, g, slot_k, :]
//
// Both are pure HBM traffic: one wavefront moves one row with 16-byte accesses.
#include "common.h"

namespace moe {
namespace {

constexpr int kRowsPerBlock = 4;  // one wavefront per row

// rows are M*sizeof(T) bytes, a multiple of 16
__global__ __launch_bounds__(256) void dispatch_kernel(
    const uint4* __restrict__ x, const int32_t* __restrict__ src_token, uint4* __restrict__ buf,
    int S, int G, int C, int vec_per_row, long long rows, const int32_t* __restrict__ kept) {
  const long long r = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int lane = threadIdx.x & 63;
  const int g = (int)((r / C) % G);
  // kept != NULL: packed rows (src_token holds token rows g*S + s for the first kept[e] rows of
  // expert e; zero rows up to the end of the last occupied 256-row tile, nothing beyond)
  int t = src_token[r];
  if (kept != nullptr) {
    const long long e = r / ((long long)G * C), p = r - e * G * C;
    const int ke = kept[e];
    if (p >= ((ke + 255) & ~255)) return;
    if (p >= ke) t = -1;
  }
  uint4* dst = buf + r * vec_per_row;
  if (t >= 0) {
    const uint4* src = x + (kept != nullptr ? (long long)t : (long long)g * S + t) * vec_per_row;
    for (int v = lane; v < vec_per_row; v += 64) dst[v] = src[v];
  } else {
    const uint4 zero = {0u, 0u, 0u, 0u};
    for (int v = lane; v < vec_per_row; v += 64) dst[v] = zero;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(
    const uint4* __restrict__ out, const int32_t* __restrict__ expert_idx,
    const int32_t* __restrict__ slot, const float* __restrict__ weight,
    const int32_t* __restrict__ row_base, uint4* __restrict__ y,
    int S, int G, int C, int E, int vec_per_row, long long tokens) {
  const long long n = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (n >= tokens) return;
  const int lane = threadIdx.x & 63;
  const int g = (int)(n / S);
  const int s0 = slot[2 * n], s1 = slot[2 * n + 1];
  const float w0 = weight[2 * n], w1 = weight[2 * n + 1];
  // row of a kept choice: (e G + g) C + slot in the [E,G,C,M] order, e G C + row_base[g,e] + slot
  // in the packed order
  const uint4 *r0 = nullptr, *r1 = nullptr;
  if (s0 >= 0) {
    const long long e = expert_idx[2 * n];
    const long long row = row_base != nullptr ? e * G * C + row_base[(long long)g * E + e] + s0
                                              : (e * G + g) * C + s0;
    r0 = out + row * vec_per_row;
  }
  if (s1 >= 0) {
    const long long e = expert_idx[2 * n + 1];
    const long long row = row_base != nullptr ? e * G * C + row_base[(long long)g * E + e] + s1
                                              : (e * G + g) * C + s1;
    r1 = out + row * vec_per_row;
  }
  uint4* dst = y + n * vec_per_row;
  constexpr int K = Vec16<T>::kElts;
  for (int v = lane; v < vec_per_row; v += 64) {
    float acc[K];
#pragma unroll
    for (int i = 0; i < K; ++i) acc[i] = 0.f;
    if (r0 != nullptr) {
      float f[K];
      Vec16<T>::unpack(r0[v], f);
#pragma unroll
      for (int i = 0; i < K; ++i) acc[i] = w0 * f[i];
    }
    if (r1 != nullptr) {
      float f[K];
      Vec16<T>::unpack(r1[v], f);
#pragma unroll
      for (int i = 0; i < K; ++i) acc[i] = fmaf(w1, f[i], acc[i]);
    }
    dst[v] = Vec16<T>::pack(acc);
  }
}

}  // namespace

int launch_dispatch(const moe_config& c, const void* x, const int32_t* src_token, void* buf,
                    const int32_t* kept, hipStream_t st) {
  const int elt = c.act_dtype == MOE_F32 ? 4 : 2;
  const int vec_per_row = c.M * elt / 16;
  const long long rows = (long long)c.E * c.G * c.C;
  const unsigned grid = (unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock);
  hipLaunchKernelGGL(dispatch_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint4*>(x),
                     src_token, static_cast<uint4*>(buf), c.S, c.G, c.C, vec_per_row, rows, kept);
  return check_launch();
}

int launch_combine(const moe_config& c, const void* out, const int32_t* expert_idx,
                   const int32_t* slot, const float* weight, const int32_t* row_base, void* y,
                   hipStream_t st) {
  const int elt = c.act_dtype == MOE_F32 ? 4 : 2;
  const int vec_per_row = c.M * elt / 16;
  const long long tokens = (long long)c.G * c.S;
  const unsigned grid = (unsigned)((tokens + kRowsPerBlock - 1) / kRowsPerBlock);
  if (c.act_dtype == MOE_F32)
    hipLaunchKernelGGL(combine_kernel<float>, dim3(grid), dim3(256), 0, st,
                       static_cast<const uint4*>(out), expert_idx, slot, weight, row_base,
                       static_cast<uint4*>(y), c.S, c.G, c.C, c.E, vec_per_row, tokens);
  else
    hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(grid), dim3(256), 0, st,
                       static_cast<const uint4*>(out), expert_idx, slot, weight, row_base,
                       static_cast<uint4*>(y), c.S, c.G, c.C, c.E, vec_per_row, tokens);
  return check_launch();
}

}  // namespace moe
