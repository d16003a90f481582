// Backward pass of the encoder sub-layers around the MoE layer (Section 2.1 of the paper names
// the sub-layers; the paper trains them by automatic differentiation, the derivatives below are
// the chain rule written out).  The pieces that are not GEMMs:
//
//   layer norm     n = gamma * xhat + beta, xhat = (s - mean) * rstd:
//                  ds = rstd * (g - mean(g) - xhat * mean(g * xhat)),  g = gamma * dn
//                  dgamma = sum_rows dn * xhat,  dbeta = sum_rows dn      (two kernels)
//   attention core with p = softmax(q k^T / sqrt(d)), ctx = p v and D = rowsum(dctx * ctx):
//                  dv = p^T dctx,  ds = p * (dctx v^T - D) / sqrt(d),  dq = ds k,  dk = ds^T q
//                  The probabilities are recomputed from q, k and the row statistic
//                  lse = log sum_k exp(score) that the forward kernels store.
//
// The attention core has a plain form here (one wavefront per query row for dq, one per key row
// for dk and dv, any dtype and shape whose rows fit in LDS); the MFMA form lives in
// attention_bwd_mfma.hip.
#include <math.h>
#include "common.h"

namespace moe {
namespace {

// ---------------------------------------------------------------- layer normalisation
// One wavefront per row, a wavefront walks rows wave, wave + waves, ...; its column sums of
// dn * xhat and dn stay in registers; the four wavefronts of a block add theirs in LDS (fixed
// order) and the block leaves one partial row.
template <typename T, int VPL>
__global__ __launch_bounds__(256) void layer_norm_bwd_kernel(
    const uint4* __restrict__ s, const uint4* __restrict__ dn, const float* __restrict__ gamma,
    const uint4* dres, uint4* dx, float* __restrict__ partial, int M, int vec_per_row,
    long long rows, float eps) {
  const int lane = threadIdx.x & 63;
  const long long wave_id = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long waves = (long long)gridDim.x * 4;
  constexpr int K = Vec16<T>::kElts;
  float ag[VPL][K], ab[VPL][K], gam[VPL][K];
#pragma unroll
  for (int j = 0; j < VPL; ++j)
#pragma unroll
    for (int i = 0; i < K; ++i) {
      ag[j][i] = 0.f;
      ab[j][i] = 0.f;
      const int col = (lane + 64 * j) * K + i;
      gam[j][i] = col < M ? gamma[col] : 0.f;
    }
  const float inv_m = 1.0f / (float)M;
  for (long long row = wave_id; row < rows; row += waves) {
    float v[VPL][K], g[VPL][K];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int vi = lane + 64 * j;
#pragma unroll
      for (int i = 0; i < K; ++i) { v[j][i] = 0.f; g[j][i] = 0.f; }
      if (vi < vec_per_row) {
        Vec16<T>::unpack(s[row * vec_per_row + vi], v[j]);
        Vec16<T>::unpack(dn[row * vec_per_row + vi], g[j]);
#pragma unroll
        for (int i = 0; i < K; ++i) sum += v[j][i];
      }
    }
    const float mean = wave_sum(sum) * inv_m;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j)
      if (lane + 64 * j < vec_per_row)
#pragma unroll
        for (int i = 0; i < K; ++i) q += (v[j][i] - mean) * (v[j][i] - mean);
    const float rstd = 1.0f / sqrtf(wave_sum(q) * inv_m + eps);
    float sg = 0.f, sgx = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j)
      if (lane + 64 * j < vec_per_row)
#pragma unroll
        for (int i = 0; i < K; ++i) {
          const float xh = (v[j][i] - mean) * rstd;
          v[j][i] = xh;
          ag[j][i] += g[j][i] * xh;                 // g still holds dn
          ab[j][i] += g[j][i];
          g[j][i] *= gam[j][i];
          sg += g[j][i];
          sgx += g[j][i] * xh;
        }
    sg = wave_sum(sg) * inv_m;
    sgx = wave_sum(sgx) * inv_m;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int vi = lane + 64 * j;
      if (vi < vec_per_row) {
        float o[K];
#pragma unroll
        for (int i = 0; i < K; ++i) o[i] = rstd * (g[j][i] - sg - v[j][i] * sgx);
        if (dres != nullptr) {
          float r[K];
          Vec16<T>::unpack(dres[row * vec_per_row + vi], r);
#pragma unroll
          for (int i = 0; i < K; ++i) o[i] += r[i];
        }
        dx[row * vec_per_row + vi] = Vec16<T>::pack(o);
      }
    }
  }
  extern __shared__ float ln_bwd_smem[];              // [4 wavefronts][M], used twice
  float* mine = ln_bwd_smem + (size_t)(threadIdx.x >> 6) * M;
  float* pg = partial + (size_t)blockIdx.x * 2 * M;
#pragma unroll
  for (int which = 0; which < 2; ++which) {           // 0: dgamma sums, 1: dbeta sums
#pragma unroll
    for (int j = 0; j < VPL; ++j)
#pragma unroll
      for (int i = 0; i < K; ++i) {
        const int col = (lane + 64 * j) * K + i;
        if (col < M) mine[col] = which == 0 ? ag[j][i] : ab[j][i];
      }
    __syncthreads();
    for (int i = threadIdx.x; i < M; i += 256)
      pg[which * M + i] = ((ln_bwd_smem[i] + ln_bwd_smem[M + i]) + ln_bwd_smem[2 * M + i]) + ln_bwd_smem[3 * M + i];
    __syncthreads();
  }
}

// dgamma[m] = sum_p partial[p][0][m], dbeta[m] = sum_p partial[p][1][m]: a block owns 16 of the
// 2 M columns, its 16 groups of 16 threads each sum every 16th partial row, LDS adds the groups
// in a fixed order (bit-reproducible)
__global__ __launch_bounds__(256) void layer_norm_param_reduce_kernel(
    const float* __restrict__ partial, int parts, int M, float* __restrict__ dgamma,
    float* __restrict__ dbeta) {
  __shared__ float red[16][17];
  const int c = threadIdx.x & 15, pl = threadIdx.x >> 4;
  const int i = blockIdx.x * 16 + c;
  float acc = 0.f;
  if (i < 2 * M)
    for (int p = pl; p < parts; p += 16) acc += partial[(size_t)p * 2 * M + i];
  red[pl][c] = acc;
  __syncthreads();
  if (pl == 0 && i < 2 * M) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) t += red[k][c];
    if (i < M) dgamma[i] = t; else dbeta[i - M] = t;
  }
}

// ---------------------------------------------------------------- attention core, plain form
// dq: one wavefront per (sequence, head, query).  Also writes D = rowsum(dctx * ctx) of its row.
template <typename T>
__global__ __launch_bounds__(256) void attention_bwd_dq_rows_kernel(
    const T* __restrict__ qkv, const T* __restrict__ ctx, const T* __restrict__ dctx,
    const float* __restrict__ lse, T* __restrict__ dqkv, float* __restrict__ dvec, int L, int heads,
    int d, long long queries) {
  extern __shared__ float att_bwd_smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* sc = att_bwd_smem + (size_t)wave * (L + 2 * d);   // [L] ds of the row, [d] q, [d] dctx
  float* qs = sc + L;
  float* dos = qs + d;
  const long long id = (long long)blockIdx.x * 4 + wave;   // (b * heads + h) * L + l
  if (id >= queries) return;
  const int l = (int)(id % L);
  const long long bh = id / L;
  const int h = (int)(bh % heads);
  const long long b = bh / heads;
  const int A = heads * d;
  const size_t ld = (size_t)3 * A;
  const T* qrow = qkv + ((size_t)b * L + l) * ld + (size_t)h * d;
  const T* kbase = qkv + (size_t)b * L * ld + A + (size_t)h * d;
  const T* vbase = kbase + A;
  const size_t crow = ((size_t)b * L + l) * A + (size_t)h * d;
  float dd = 0.f;
  for (int i = lane; i < d; i += 64) {
    qs[i] = Elt<T>::load(qrow + i);
    const float g = Elt<T>::load(dctx + crow + i);
    dos[i] = g;
    dd += g * Elt<T>::load(ctx + crow + i);
  }
  dd = wave_sum(dd);
  if (lane == 0) dvec[id] = dd;
  __builtin_amdgcn_wave_barrier();
  const float scale = 1.0f / sqrtf((float)d);
  const float ls = lse[id];
  for (int k0 = 0; k0 < L; k0 += 64) {
    const int key = k0 + lane;
    if (key < L) {
      const T* kr = kbase + (size_t)key * ld;
      const T* vr = vbase + (size_t)key * ld;
      float dot = 0.f, dp = 0.f;
      for (int i = 0; i < d; ++i) {
        dot = fmaf(qs[i], Elt<T>::load(kr + i), dot);
        dp = fmaf(dos[i], Elt<T>::load(vr + i), dp);
      }
      const float p = expf(dot * scale - ls);
      sc[key] = p * (dp - dd) * scale;
    }
  }
  __builtin_amdgcn_wave_barrier();
  T* out = dqkv + ((size_t)b * L + l) * ld + (size_t)h * d;
  for (int i = lane; i < d; i += 64) {
    float acc = 0.f;
    for (int key = 0; key < L; ++key) acc = fmaf(sc[key], Elt<T>::load(kbase + (size_t)key * ld + i), acc);
    Elt<T>::store(out + i, acc);
  }
}

// dk, dv: one wavefront per (sequence, head, key); needs lse and D of every query of the head.
template <typename T>
__global__ __launch_bounds__(256) void attention_bwd_dkv_rows_kernel(
    const T* __restrict__ qkv, const T* __restrict__ dctx, const float* __restrict__ lse,
    const float* __restrict__ dvec, T* __restrict__ dqkv, int L, int heads, int d, long long keys) {
  extern __shared__ float att_bwd_smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* pp = att_bwd_smem + (size_t)wave * (2 * L + 2 * d);   // [L] p, [L] ds, [d] k, [d] v
  float* sd = pp + L;
  float* ks = sd + L;
  float* vs = ks + d;
  const long long id = (long long)blockIdx.x * 4 + wave;       // (b * heads + h) * L + key
  if (id >= keys) return;
  const int key = (int)(id % L);
  const long long bh = id / L;
  const int h = (int)(bh % heads);
  const long long b = bh / heads;
  const int A = heads * d;
  const size_t ld = (size_t)3 * A;
  const T* qbase = qkv + (size_t)b * L * ld + (size_t)h * d;
  const T* krow = qbase + (size_t)key * ld + A;
  const T* gbase = dctx + (size_t)b * L * A + (size_t)h * d;
  for (int i = lane; i < d; i += 64) {
    ks[i] = Elt<T>::load(krow + i);
    vs[i] = Elt<T>::load(krow + A + i);
  }
  __builtin_amdgcn_wave_barrier();
  const float scale = 1.0f / sqrtf((float)d);
  for (int q0 = 0; q0 < L; q0 += 64) {
    const int q = q0 + lane;
    if (q < L) {
      const T* qr = qbase + (size_t)q * ld;
      const T* gr = gbase + (size_t)q * A;
      float dot = 0.f, dp = 0.f;
      for (int i = 0; i < d; ++i) {
        dot = fmaf(Elt<T>::load(qr + i), ks[i], dot);
        dp = fmaf(Elt<T>::load(gr + i), vs[i], dp);
      }
      const float p = expf(dot * scale - lse[bh * L + q]);
      pp[q] = p;
      sd[q] = p * (dp - dvec[bh * L + q]) * scale;
    }
  }
  __builtin_amdgcn_wave_barrier();
  T* out = dqkv + ((size_t)b * L + key) * ld + A + (size_t)h * d;
  for (int i = lane; i < d; i += 64) {
    float dk = 0.f, dv = 0.f;
    for (int q = 0; q < L; ++q) {
      dk = fmaf(sd[q], Elt<T>::load(qbase + (size_t)q * ld + i), dk);
      dv = fmaf(pp[q], Elt<T>::load(gbase + (size_t)q * A + i), dv);
    }
    Elt<T>::store(out + i, dk);
    Elt<T>::store(out + A + i, dv);
  }
}

// out[i] = sum_s partial[s][i] (fixed order), rounded once to bf16; 8 elements per thread
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial,
                                                            int splits, long long elems,
                                                            uint4* __restrict__ out) {
  const long long v = (long long)blockIdx.x * 256 + threadIdx.x;
  if (v * 8 >= elems) return;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int sp = 0; sp < splits; ++sp) {
    const float4* p = reinterpret_cast<const float4*>(partial + (size_t)sp * elems + v * 8);
    const float4 a = p[0], b = p[1];
    acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
    acc[4] += b.x; acc[5] += b.y; acc[6] += b.z; acc[7] += b.w;
  }
  out[v] = Vec16<bf16_t>::pack(acc);
}

}  // namespace

// Weight gradient of a dense layer, dW [in,out] = X^T dY over `rows` tokens.  Its output has
// few 256 x 256 tiles (in/256 * out/256) but a very long K (the tokens), so the persistent GEMM
// alone would leave most compute units idle: the tokens are cut into `splits` ranges that run
// as a batch with fp32 results, and one pass adds the ranges in order and rounds once.
// The plan picks the number of ranges that fills the 256 compute units best.
int dense_wgrad_splits(int act_dtype, long long rows, int in, int out) {
  if (act_dtype != MOE_BF16 || in % 256 != 0 || out % 256 != 0) return 1;
  const long long tiles = (long long)(in / 256) * (out / 256);
  int best = 1;
  double best_fill = 0.0;
  for (int sp = 1; sp <= 16; sp *= 2) {
    if (rows % sp != 0 || (rows / sp) % 32 != 0 || rows / sp < 512) break;
    if (!gemm_bf16_f32out_ok(in, out, (int)(rows / sp))) continue;
    const long long t = tiles * sp;
    const double fill = (double)t / (double)((t + 255) / 256 * 256);
    if (fill > best_fill + 1e-9) { best_fill = fill; best = sp; }
  }
  return best;
}

size_t dense_wgrad_partial_bytes(int act_dtype, long long rows, int in, int out) {
  const int sp = dense_wgrad_splits(act_dtype, rows, in, out);
  return sp > 1 ? (size_t)sp * in * out * sizeof(float) : 0;
}

int launch_dense_wgrad(const moe_config& c, long long rows, int in, int out, const void* X,
                       const void* dY, void* dW, float* partial, hipStream_t st) {
  if (rows > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  const int sp = dense_wgrad_splits(c.act_dtype, rows, in, out);
  if (sp <= 1 || partial == nullptr) {
    moe_config g = c;
    g.E = 1; g.G = 1; g.C = (int)rows; g.M = in; g.H = out;
    return launch_expert_wgrad1(g, X, dY, dW, nullptr, st);
  }
  const int rc = launch_gemm_bf16_f32out(true, X, dY, partial, sp, in, out, (int)(rows / sp), st);
  if (rc != MOE_OK) return rc;
  const long long elems = (long long)in * out;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((elems / 8 + 255) / 256)), dim3(256), 0, st,
                     partial, sp, elems, static_cast<uint4*>(dW));
  return check_launch();
}

int layer_norm_bwd_parts(long long rows) {
  const long long blocks = (rows + 3) / 4;
  return (int)(blocks < 1024 ? blocks : 1024);
}

int launch_layer_norm_bwd(int act_dtype, const void* s, const void* dn, const float* gamma,
                          const void* dres, void* dx, float* partial, float* dgamma, float* dbeta,
                          long long rows, int M, hipStream_t st) {
  const int elt = act_dtype == MOE_F32 ? 4 : 2;
  const int vec_per_row = M * elt / 16;
  const int vpl = (vec_per_row + 63) / 64;
  const size_t lds = (size_t)4 * M * sizeof(float);
  if (vpl > 8 || lds > 64 * 1024) return MOE_EUNSUPPORTED;
  const int parts = layer_norm_bwd_parts(rows);
  const unsigned grid = (unsigned)parts;
  const float eps = 1e-6f;
#define MOE_LNB_CASE(T, V)                                                                    \
  hipLaunchKernelGGL((layer_norm_bwd_kernel<T, V>), dim3(grid), dim3(256), lds, st,           \
                     static_cast<const uint4*>(s), static_cast<const uint4*>(dn), gamma,      \
                     static_cast<const uint4*>(dres), static_cast<uint4*>(dx), partial, M,    \
                     vec_per_row, rows, eps)
  if (act_dtype == MOE_F32) {
    if (vpl <= 1) MOE_LNB_CASE(float, 1); else if (vpl <= 2) MOE_LNB_CASE(float, 2);
    else if (vpl <= 4) MOE_LNB_CASE(float, 4); else MOE_LNB_CASE(float, 8);
  } else {
    if (vpl <= 1) MOE_LNB_CASE(bf16_t, 1); else if (vpl <= 2) MOE_LNB_CASE(bf16_t, 2);
    else if (vpl <= 4) MOE_LNB_CASE(bf16_t, 4); else MOE_LNB_CASE(bf16_t, 8);
  }
#undef MOE_LNB_CASE
  int rc = check_launch();
  if (rc != MOE_OK) return rc;
  hipLaunchKernelGGL(layer_norm_param_reduce_kernel, dim3((unsigned)((2 * M + 15) / 16)), dim3(256),
                     0, st, partial, parts, M, dgamma, dbeta);
  return check_launch();
}

// dqkv [B*L, 3*heads*d] from qkv, ctx, dctx [B*L, heads*d], lse [B*heads*L]; dvec [B*heads*L] scratch
int launch_attention_core_bwd(int act_dtype, const void* qkv, const void* ctx, const void* dctx,
                              const float* lse, void* dqkv, float* dvec, long long B, int L,
                              int heads, int d, hipStream_t st) {
  if (attention_bwd_mfma_ok(act_dtype, L, d))
    return launch_attention_bwd_mfma(qkv, ctx, dctx, lse, dqkv, dvec, B, L, heads, d, st);
  const long long rows = B * heads * L;
  const size_t lds = (size_t)4 * (2 * L + 2 * d) * sizeof(float);
  if (lds > 64 * 1024 || (rows + 3) / 4 > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  const size_t lds_q = (size_t)4 * (L + 2 * d) * sizeof(float);
  const unsigned grid = (unsigned)((rows + 3) / 4);
  if (act_dtype == MOE_F32) {
    hipLaunchKernelGGL(attention_bwd_dq_rows_kernel<float>, dim3(grid), dim3(256), lds_q, st,
                       static_cast<const float*>(qkv), static_cast<const float*>(ctx),
                       static_cast<const float*>(dctx), lse, static_cast<float*>(dqkv), dvec, L,
                       heads, d, rows);
    hipLaunchKernelGGL(attention_bwd_dkv_rows_kernel<float>, dim3(grid), dim3(256), lds, st,
                       static_cast<const float*>(qkv), static_cast<const float*>(dctx), lse, dvec,
                       static_cast<float*>(dqkv), L, heads, d, rows);
  } else {
    hipLaunchKernelGGL(attention_bwd_dq_rows_kernel<bf16_t>, dim3(grid), dim3(256), lds_q, st,
                       static_cast<const bf16_t*>(qkv), static_cast<const bf16_t*>(ctx),
                       static_cast<const bf16_t*>(dctx), lse, static_cast<bf16_t*>(dqkv), dvec, L,
                       heads, d, rows);
    hipLaunchKernelGGL(attention_bwd_dkv_rows_kernel<bf16_t>, dim3(grid), dim3(256), lds, st,
                       static_cast<const bf16_t*>(qkv), static_cast<const bf16_t*>(dctx), lse, dvec,
                       static_cast<bf16_t*>(dqkv), L, heads, d, rows);
  }
  return check_launch();
}

}  // namespace moe
