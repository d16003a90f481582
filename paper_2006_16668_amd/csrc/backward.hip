// Backward pass of the top-2 MoE layer: everything except the large expert GEMMs.
//
// The paper differentiates Algorithm 2 automatically and states only that the counts
// c_e of the auxiliary loss carry no gradient while the mean gates m_e do (Section 2.2,
// "Auxiliary loss").  Written out by the chain rule, with all discrete routing decisions
// of Algorithm 1 as constants:
//
//   combine_bwd   dout[e,g,c,:] = weight[g,s,k] * dy[g,s,:]          (Eq. 3 transposed)
//                 dweight[g,s,k] = <dy[g,s,:], out[e,g,c,:]>
//   gate_bwd      weight_1 = g1/(g1+g2), weight_2 = g2/(g1+g2)  (Algorithm 1) =>
//                 dgate[e1] = (dw1 - dw2) g2 / (g1+g2)^2,  dgate[e2] = (dw2 - dw1) g1 / (g1+g2)^2
//                 l_aux = (1/E) sum_e (c_e/S) m_e  =>  dgate[e] += daux[g] c_e / (E S^2)
//                 softmax: dz[e] = g[e] (dgate[e] - sum_e' g[e'] dgate[e'])
//   dwg           dwg[m,e] = sum_tokens x[t,m] dz[t,e]
//   dx            dx[g,s,:] = sum_k dbuf[e_k,g,c_k,:] + sum_e dz[g,s,e] wg[:,e]
//                 (dispatch transposed + the gate projection)
//
// plus a generic strided GEMM that serves the expert GEMMs of the backward pass for
// shapes and element types the MFMA kernels do not take.
#include "common.h"

namespace moe {
namespace {

constexpr int kRowsPerBlock = 4;  // one wavefront per row / token

template <typename T>
__global__ __launch_bounds__(256) void combine_bwd_kernel(
    const uint4* __restrict__ dy, const uint4* __restrict__ out,
    const int32_t* __restrict__ src_token, const int32_t* __restrict__ expert_idx,
    const float* __restrict__ weight, uint4* __restrict__ dout, float* __restrict__ dweight,
    int S, int G, int C, int vec_per_row, long long rows, const int32_t* __restrict__ kept) {
  const long long r = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int lane = threadIdx.x & 63;
  const int g = (int)((r / C) % G);
  const int e = (int)(r / ((long long)G * C));
  // kept != NULL: packed rows.  src_token then holds the token row g*S + s of packed row p of
  // expert e for p < kept[e]; the rows up to the end of the last occupied 256-row tile become
  // zero rows (they enter the weight gradients' sums), later rows are nobody's business.
  int t = src_token[r];
  if (kept != nullptr) {
    const long long p = r - (long long)e * G * C;
    const int ke = kept[e];
    if (p >= ((ke + 255) & ~255)) return;
    if (p >= ke) t = -1;
  }
  uint4* dst = dout + r * vec_per_row;
  if (t < 0) {
    const uint4 zero = {0u, 0u, 0u, 0u};
    for (int v = lane; v < vec_per_row; v += 64) dst[v] = zero;
    return;
  }
  const long long n = kept != nullptr ? (long long)t : (long long)g * S + t;
  const int k = expert_idx[2 * n] == e ? 0 : 1;        // the two experts of a token differ
  const float w = weight[2 * n + k];
  const uint4* dyr = dy + n * vec_per_row;
  const uint4* outr = out + r * vec_per_row;
  constexpr int K = Vec16<T>::kElts;
  float dot = 0.f;
  for (int v = lane; v < vec_per_row; v += 64) {
    float f[K], o[K];
    Vec16<T>::unpack(dyr[v], f);
    Vec16<T>::unpack(outr[v], o);
#pragma unroll
    for (int i = 0; i < K; ++i) {
      dot = fmaf(f[i], o[i], dot);
      f[i] *= w;
    }
    dst[v] = Vec16<T>::pack(f);
  }
  dot = wave_sum(dot);
  if (lane == 0) dweight[2 * n + k] = dot;
}

// one wavefront per token; dweight of a choice that is not kept is never read
__global__ __launch_bounds__(256) void gate_bwd_kernel(
    const float* __restrict__ gates, const int32_t* __restrict__ expert_idx,
    const int32_t* __restrict__ slot, const float* __restrict__ dweight,
    const int32_t* __restrict__ c1, const float* __restrict__ daux, float* __restrict__ dz,
    bf16_t* __restrict__ dzp, int cols, int S, int E, long long tokens) {
  const long long n = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (n >= tokens) return;
  const int lane = threadIdx.x & 63;
  const int g = (int)(n / S);
  const float* p = gates + n * E;
  const int e1 = expert_idx[2 * n], e2 = expert_idx[2 * n + 1];
  const float g1 = p[e1], g2 = p[e2];
  const float d1 = slot[2 * n] >= 0 ? dweight[2 * n] : 0.f;
  const float d2 = slot[2 * n + 1] >= 0 ? dweight[2 * n + 1] : 0.f;
  const float inv = 1.f / ((g1 + g2) * (g1 + g2));
  const float t1 = (d1 - d2) * g2 * inv, t2 = (d2 - d1) * g1 * inv;
  const float scale = daux[g] / ((float)E * (float)S * (float)S);
  const int32_t* cg = c1 + (long long)g * E;
  float dot = 0.f;
  for (int e = lane; e < E; e += 64) {
    const float dp = scale * (float)cg[e] + (e == e1 ? t1 : 0.f) + (e == e2 ? t2 : 0.f);
    dot = fmaf(p[e], dp, dot);
  }
  dot = wave_sum(dot);
  for (int e = lane; e < E; e += 64) {
    const float dp = scale * (float)cg[e] + (e == e1 ? t1 : 0.f) + (e == e2 ? t2 : 0.f);
    const float v = p[e] * (dp - dot);
    if (dz != nullptr) dz[n * E + e] = v;
    if (dzp != nullptr) {
      // v = hi + mid + lo exactly (three bf16 terms cover the 24 mantissa bits), stored side
      // by side so that a bf16 matrix product over these columns is an fp32-faithful one
      const bf16_t hi = f32_to_bf16(v);
      const float r1 = v - bf16_to_f32(hi);
      const bf16_t mid = f32_to_bf16(r1);
      const bf16_t lo = f32_to_bf16(r1 - bf16_to_f32(mid));
      bf16_t* d = dzp + n * cols + 3 * e;
      d[0] = hi; d[1] = mid; d[2] = lo;
    }
  }
  if (dzp != nullptr)
    for (int cidx = 3 * E + lane; cidx < cols; cidx += 64) dzp[n * cols + cidx] = 0;
}

// wgp[m, 3e+p] = bf16(wg[m,e]) for the three terms p of dz, zero in the padding columns
__global__ __launch_bounds__(256) void wg_pack_bwd_kernel(
    const float* __restrict__ wg, bf16_t* __restrict__ wgp, int M, int E, int cols) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)M * cols) return;
  const int m = (int)(i / cols), cidx = (int)(i % cols);
  wgp[i] = cidx < 3 * E ? f32_to_bf16(wg[(size_t)m * E + cidx / 3]) : (bf16_t)0;
}

// dx[n,:] = round( dxg[n,:] + dbuf row of the first kept choice + of the second ), bf16
__global__ __launch_bounds__(256) void dx_rows_kernel(
    const float4* __restrict__ dxg, const uint4* __restrict__ dbuf,
    const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ slot,
    uint4* __restrict__ dx, int S, int G, int C, int E, int vec_per_row, long long tokens,
    const int32_t* __restrict__ row_base) {
  const long long n = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (n >= tokens) return;
  const int lane = threadIdx.x & 63;
  const int g = (int)(n / S);
  const int s0 = slot[2 * n], s1 = slot[2 * n + 1];
  // row of a kept choice: (e G + g) C + slot, or e G C + row_base[g,e] + slot when packed
  const uint4 *r0 = nullptr, *r1 = nullptr;
  if (s0 >= 0) {
    const long long e = expert_idx[2 * n];
    r0 = dbuf + (row_base != nullptr ? e * G * C + row_base[(long long)g * E + e] + s0
                                     : (e * G + g) * C + s0) * vec_per_row;
  }
  if (s1 >= 0) {
    const long long e = expert_idx[2 * n + 1];
    r1 = dbuf + (row_base != nullptr ? e * G * C + row_base[(long long)g * E + e] + s1
                                     : (e * G + g) * C + s1) * vec_per_row;
  }
  for (int v = lane; v < vec_per_row; v += 64) {
    const float4 a = dxg[(n * vec_per_row + v) * 2], b = dxg[(n * vec_per_row + v) * 2 + 1];
    float acc[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    if (r0 != nullptr) {
      float f[8];
      Vec16<bf16_t>::unpack(r0[v], f);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += f[i];
    }
    if (r1 != nullptr) {
      float f[8];
      Vec16<bf16_t>::unpack(r1[v], f);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += f[i];
    }
    dx[n * vec_per_row + v] = Vec16<bf16_t>::pack(acc);
  }
}

// dwg[m,e] = sum_t x[t,m] dz[t,e]: partial sums over a range of tokens per block, then a
// reduction over the ranges in a fixed order (no atomics: the result is reproducible).
template <typename T>
__global__ __launch_bounds__(256) void dwg_partial_kernel(
    const T* __restrict__ x, const float* __restrict__ dz, float* __restrict__ partial,
    int M, int E, long long tokens, long long tokens_per_split) {
  __shared__ float xs[16][64];
  __shared__ float zs[16][64];
  const int m0 = blockIdx.x * 64, e0 = blockIdx.y * 64;
  const long long t_begin = (long long)blockIdx.z * tokens_per_split;
  const long long t_stop = t_begin + tokens_per_split < tokens ? t_begin + tokens_per_split : tokens;
  const int tid = threadIdx.x, tm = tid & 15, te = tid >> 4;
  const int lk = tid >> 4, lc = 4 * (tid & 15);
  float acc[4][4] = {};
  for (long long t0 = t_begin; t0 < t_stop; t0 += 16) {
    const long long t = t0 + lk;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + lc + i, e = e0 + lc + i;
      xs[lk][lc + i] = (t < t_stop && m < M) ? Elt<T>::load(x + t * M + m) : 0.f;
      zs[lk][lc + i] = (t < t_stop && e < E) ? dz[t * E + e] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = xs[k][4 * tm + i]; b[i] = zs[k][4 * te + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  float* dst = partial + (size_t)blockIdx.z * M * E;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + 4 * tm + i, e = e0 + 4 * te + j;
      if (m < M && e < E) dst[(size_t)m * E + e] = acc[i][j];
    }
}

// dwg[m,e] = sum over token ranges (in order) of the `terms` adjacent columns of e
__global__ __launch_bounds__(256) void dwg_reduce_kernel(
    const float* __restrict__ partial, float* __restrict__ dwg, int M, int E, int cols, int terms,
    int splits) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)M * E) return;
  const int m = (int)(i / E), e = (int)(i % E);
  float acc = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float* p = partial + ((size_t)s * M + m) * cols + (size_t)terms * e;
    float t = p[0];
    for (int k = 1; k < terms; ++k) t += p[k];
    acc += t;
  }
  dwg[i] = acc;
}

// dx tile of 64 tokens x 64 features: the gate projection dz . wg^T in fp32, then the
// gradient rows of the token's kept choices are added (first, then second choice) and the
// sum is rounded once.
template <typename T>
__global__ __launch_bounds__(256) void dx_kernel(
    const float* __restrict__ dz, const float* __restrict__ wg, const T* __restrict__ dbuf,
    const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ slot,
    T* __restrict__ dx, int S, int G, int C, int M, int E, long long tokens,
    const int32_t* __restrict__ row_base) {
  __shared__ float zs[16][65];
  __shared__ float ws[16][65];
  const long long n0 = (long long)blockIdx.x * 64;
  const int m0 = blockIdx.y * 64;
  const int tid = threadIdx.x, tt = tid & 15, tm = tid >> 4;
  const int lr = tid >> 2, lc = 4 * (tid & 3);
  float acc[4][4] = {};
  for (int e0 = 0; e0 < E; e0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = e0 + lc + i;
      const long long n = n0 + lr;
      const int m = m0 + lr;
      zs[lc + i][lr] = (n < tokens && e < E) ? dz[n * E + e] : 0.f;
      ws[lc + i][lr] = (m < M && e < E) ? wg[(size_t)m * E + e] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = zs[k][4 * tt + i]; b[i] = ws[k][4 * tm + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const long long n = n0 + 4 * tt + i;
    if (n >= tokens) continue;
    const int g = (int)(n / S);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int c = slot[2 * n + k];
      if (c < 0) continue;
      const size_t e = (size_t)expert_idx[2 * n + k];
      const T* row = dbuf + (row_base != nullptr ? e * G * C + row_base[(size_t)g * E + e] + c
                                                 : (e * G + g) * C + c) * M;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int m = m0 + 4 * tm + j;
        if (m < M) acc[i][j] += Elt<T>::load(row + m);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + 4 * tm + j;
      if (m < M) Elt<T>::store(dx + n * M + m, acc[i][j]);
    }
  }
}

// C[e,r,n] = epi( sum_k A[e*a_e + r*a_r + k*a_k] * B[e*b_e + k*b_k + n*b_n] ), C row-major
// [E,R,N]; fp32 accumulation; EPI 0: none, 1: relu, 2: zero where mask[e,r,n] <= 0.
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_strided_kernel(
    const T* __restrict__ A, long long a_e, long long a_r, long long a_k,
    const T* __restrict__ B, long long b_e, long long b_k, long long b_n,
    T* __restrict__ Cout, const T* __restrict__ mask, int R, int N, int K) {
  __shared__ float as[16][65];
  __shared__ float bs[16][65];
  const int n0 = blockIdx.x * 64, r0 = blockIdx.y * 64, e = blockIdx.z;
  const T* Ae = A + (size_t)e * a_e;
  const T* Be = B + (size_t)e * b_e;
  const int tid = threadIdx.x, tr = tid & 15, tn = tid >> 4;
  const int lr = tid >> 2, lc = 4 * (tid & 3);
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + lc + i;
      const int r = r0 + lr, n = n0 + lr;
      as[lc + i][lr] = (r < R && k < K) ? Elt<T>::load(Ae + (long long)r * a_r + (long long)k * a_k) : 0.f;
      bs[lc + i][lr] = (n < N && k < K) ? Elt<T>::load(Be + (long long)k * b_k + (long long)n * b_n) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = as[k][4 * tr + i]; b[i] = bs[k][4 * tn + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = r0 + 4 * tr + i, n = n0 + 4 * tn + j;
      if (r >= R || n >= N) continue;
      const size_t o = ((size_t)e * R + r) * N + n;
      float v = acc[i][j];
      if (EPI == 1) v = fmaxf(v, 0.f);
      if (EPI == 2) v = Elt<T>::load(mask + o) > 0.f ? v : 0.f;
      Elt<T>::store(Cout + o, v);
    }
}

template <typename T>
int gemm_strided(int epi, const void* A, long long a_e, long long a_r, long long a_k, const void* B,
                 long long b_e, long long b_k, long long b_n, void* Cout, const void* mask, int E,
                 int R, int N, int K, hipStream_t st) {
  if (E > 65535 || (R + 63) / 64 > 65535) return MOE_EUNSUPPORTED;
  const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((R + 63) / 64), (unsigned)E);
  auto a = static_cast<const T*>(A);
  auto b = static_cast<const T*>(B);
  auto c = static_cast<T*>(Cout);
  auto m = static_cast<const T*>(mask);
  if (epi == 0)
    hipLaunchKernelGGL((gemm_strided_kernel<T, 0>), grid, dim3(256), 0, st, a, a_e, a_r, a_k, b, b_e,
                       b_k, b_n, c, m, R, N, K);
  else if (epi == 1)
    hipLaunchKernelGGL((gemm_strided_kernel<T, 1>), grid, dim3(256), 0, st, a, a_e, a_r, a_k, b, b_e,
                       b_k, b_n, c, m, R, N, K);
  else
    hipLaunchKernelGGL((gemm_strided_kernel<T, 2>), grid, dim3(256), 0, st, a, a_e, a_r, a_k, b, b_e,
                       b_k, b_n, c, m, R, N, K);
  return check_launch();
}

}  // namespace

int launch_gemm_strided(const moe_config& c, int epi, const void* A, long long a_e, long long a_r,
                        long long a_k, const void* B, long long b_e, long long b_k, long long b_n,
                        void* Cout, const void* mask, int R, int N, int K, hipStream_t st) {
  if (c.act_dtype == MOE_F32 && R > 0 && N > 0 && K > 0 && a_e % 4 == 0 && b_e % 4 == 0 &&
      gemm_f32_mfma_ok(a_r, a_k, b_k, b_n, c.E, R, N, K))
    return launch_gemm_f32_mfma(epi, static_cast<const float*>(A), a_e, a_r, a_k,
                                static_cast<const float*>(B), b_e, b_k, b_n,
                                static_cast<float*>(Cout), static_cast<const float*>(mask), c.E, R,
                                N, K, st);
  return c.act_dtype == MOE_F32
             ? gemm_strided<float>(epi, A, a_e, a_r, a_k, B, b_e, b_k, b_n, Cout, mask, c.E, R, N, K, st)
             : gemm_strided<bf16_t>(epi, A, a_e, a_r, a_k, B, b_e, b_k, b_n, Cout, mask, c.E, R, N, K, st);
}

int launch_combine_bwd(const moe_config& c, const void* dy, const void* out,
                       const int32_t* src_token, const int32_t* expert_idx, const float* weight,
                       void* dout, float* dweight, const int32_t* kept, hipStream_t st) {
  const int elt = c.act_dtype == MOE_F32 ? 4 : 2;
  const int vec_per_row = c.M * elt / 16;
  const long long rows = (long long)c.E * c.G * c.C;
  const unsigned grid = (unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock);
  if (c.act_dtype == MOE_F32)
    hipLaunchKernelGGL(combine_bwd_kernel<float>, dim3(grid), dim3(256), 0, st,
                       static_cast<const uint4*>(dy), static_cast<const uint4*>(out), src_token,
                       expert_idx, weight, static_cast<uint4*>(dout), dweight, c.S, c.G, c.C,
                       vec_per_row, rows, kept);
  else
    hipLaunchKernelGGL(combine_bwd_kernel<bf16_t>, dim3(grid), dim3(256), 0, st,
                       static_cast<const uint4*>(dy), static_cast<const uint4*>(out), src_token,
                       expert_idx, weight, static_cast<uint4*>(dout), dweight, c.S, c.G, c.C,
                       vec_per_row, rows, kept);
  return check_launch();
}

GateBwdPlan gate_bwd_plan(const moe_config& c) {
  GateBwdPlan p{};
  const long long tokens = (long long)c.G * c.S;
  const long long cols = ((long long)3 * c.E + 255) / 256 * 256;
  p.mfma = c.act_dtype == MOE_BF16 && tokens % 256 == 0 && tokens <= 0x7fffffffLL &&
           cols <= 0x7fffffffLL && gemm_bf16_f32out_ok((int)tokens, c.M, (int)cols) &&
           gemm_bf16_f32out_ok(c.M, (int)cols, 128);
  if (p.mfma) {
    p.cols = (int)cols;
    // token ranges (a power of two of them, each a multiple of 32 tokens and at least 128)
    // so that there is about one 256x256 tile per compute unit
    const long long tiles = (long long)(c.M / 256) * (cols / 256);
    int s = 1;
    while ((long long)s * 2 * tiles <= 256 && (tokens / 32) % (s * 2) == 0 && tokens / (s * 2) >= 128)
      s *= 2;
    p.splits = s;
    p.dzp_bytes = (size_t)tokens * cols * 2;
    p.wgp_bytes = (size_t)c.M * cols * 2;
    p.dxg_bytes = (size_t)tokens * c.M * 4;
    p.partial_bytes = (size_t)s * c.M * cols * 4;
  } else {
    const long long s = (tokens + 511) / 512;
    p.splits = (int)(s < 1 ? 1 : (s > 128 ? 128 : s));
    p.dz_bytes = (size_t)tokens * c.E * 4;
    p.partial_bytes = (size_t)p.splits * c.M * c.E * 4;
  }
  return p;
}

int launch_gate_bwd(const moe_config& c, const void* x, const float* wg, const float* gates,
                    const int32_t* expert_idx, const int32_t* slot, const float* dweight,
                    const int32_t* c1, const float* daux, const GateBwdWs& w, float* dwg,
                    hipStream_t st) {
  const GateBwdPlan p = gate_bwd_plan(c);
  const long long tokens = (long long)c.G * c.S;
  const unsigned grid = (unsigned)((tokens + kRowsPerBlock - 1) / kRowsPerBlock);
  hipLaunchKernelGGL(gate_bwd_kernel, dim3(grid), dim3(256), 0, st, gates, expert_idx, slot,
                     dweight, c1, daux, p.mfma ? nullptr : w.dz, p.mfma ? w.dzp : nullptr, p.cols,
                     c.S, c.E, tokens);
  if (check_launch() != MOE_OK) return MOE_EHIP;
  const long long size = (long long)c.M * c.E;
  if (p.mfma) {
    // dwg = x^T . dz as one batched MFMA GEMM over the token ranges, the three bf16 terms of
    // dz side by side in the columns; the reduction adds ranges and terms in a fixed order
    const int rc = launch_gemm_bf16_f32out(true, x, w.dzp, w.partial, p.splits, c.M, p.cols,
                                           (int)(tokens / p.splits), st);
    if (rc != MOE_OK) return rc;
    hipLaunchKernelGGL(dwg_reduce_kernel, dim3((unsigned)((size + 255) / 256)), dim3(256), 0, st,
                       w.partial, dwg, c.M, c.E, p.cols, 3, p.splits);
    return check_launch();
  }
  long long tps = (tokens + p.splits - 1) / p.splits;
  tps = (tps + 15) / 16 * 16;
  const dim3 pgrid((unsigned)((c.M + 63) / 64), (unsigned)((c.E + 63) / 64), (unsigned)p.splits);
  if (c.act_dtype == MOE_F32)
    hipLaunchKernelGGL(dwg_partial_kernel<float>, pgrid, dim3(256), 0, st,
                       static_cast<const float*>(x), w.dz, w.partial, c.M, c.E, tokens, tps);
  else
    hipLaunchKernelGGL(dwg_partial_kernel<bf16_t>, pgrid, dim3(256), 0, st,
                       static_cast<const bf16_t*>(x), w.dz, w.partial, c.M, c.E, tokens, tps);
  if (check_launch() != MOE_OK) return MOE_EHIP;
  hipLaunchKernelGGL(dwg_reduce_kernel, dim3((unsigned)((size + 255) / 256)), dim3(256), 0, st,
                     w.partial, dwg, c.M, c.E, c.E, 1, p.splits);
  return check_launch();
}

int launch_dx(const moe_config& c, const float* wg, const void* dbuf, const int32_t* expert_idx,
              const int32_t* slot, const GateBwdWs& w, void* dx, const int32_t* row_base,
              hipStream_t st) {
  const GateBwdPlan p = gate_bwd_plan(c);
  const long long tokens = (long long)c.G * c.S;
  if (p.mfma) {
    // gate projection dz . wg^T on the matrix cores (fp32 result), then one pass that adds
    // the gradient rows of the kept choices and rounds once
    const long long n = (long long)c.M * p.cols;
    hipLaunchKernelGGL(wg_pack_bwd_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, wg,
                       w.wgp, c.M, c.E, p.cols);
    if (check_launch() != MOE_OK) return MOE_EHIP;
    const int rc = launch_gemm_bf16_f32out(false, w.dzp, w.wgp, w.dxg, 1, (int)tokens, c.M, p.cols, st);
    if (rc != MOE_OK) return rc;
    const unsigned grid = (unsigned)((tokens + kRowsPerBlock - 1) / kRowsPerBlock);
    hipLaunchKernelGGL(dx_rows_kernel, dim3(grid), dim3(256), 0, st,
                       reinterpret_cast<const float4*>(w.dxg), static_cast<const uint4*>(dbuf),
                       expert_idx, slot, static_cast<uint4*>(dx), c.S, c.G, c.C, c.E, c.M / 8, tokens,
                       row_base);
    return check_launch();
  }
  const dim3 grid((unsigned)((tokens + 63) / 64), (unsigned)((c.M + 63) / 64));
  if (grid.y > 65535) return MOE_EUNSUPPORTED;
  if (c.act_dtype == MOE_F32)
    hipLaunchKernelGGL(dx_kernel<float>, grid, dim3(256), 0, st, w.dz, wg,
                       static_cast<const float*>(dbuf), expert_idx, slot, static_cast<float*>(dx),
                       c.S, c.G, c.C, c.M, c.E, tokens, row_base);
  else
    hipLaunchKernelGGL(dx_kernel<bf16_t>, grid, dim3(256), 0, st, w.dz, wg,
                       static_cast<const bf16_t*>(dbuf), expert_idx, slot,
                       static_cast<bf16_t*>(dx), c.S, c.G, c.C, c.M, c.E, tokens, row_base);
  return check_launch();
}

}  // namespace moe
