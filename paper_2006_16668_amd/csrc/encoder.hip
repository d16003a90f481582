// The Transformer encoder sub-layers around the MoE layer (Section 2.1 of the paper: a
// self-attention layer and a position-wise feed-forward layer per encoder layer, with
// residual connections and layer normalisation; every other feed-forward layer is the MoE
// layer).  This file holds the pieces that are not GEMMs:
//
//   add_layer_norm   s = x (+ delta);  n = gamma * (s - mean) / sqrt(var + eps) + beta
//   attention core   ctx[b,l,h,:] = softmax_l'( q[b,l,h,:] . k[b,l',h,:] / sqrt(d) ) v[b,l',h,:]
//                    on the output of the fused Q|K|V projection, qkv [tokens, 3*heads*d]
//
// The attention core has two forms: a flash-style MFMA kernel (bf16, d = 64 or 128, L a
// multiple of 128) and a plain one-wavefront-per-query kernel for everything else.
#include <math.h>
#include "common.h"

namespace moe {
namespace {

// ---------------------------------------------------------------- layer normalisation
// one wavefront per row; the row lives in registers between the two passes
template <typename T, int VPL>   // VPL: 16-byte vectors per lane (row <= 64 * VPL vectors)
__global__ __launch_bounds__(256) void add_layer_norm_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ delta, const float* __restrict__ gamma,
    const float* __restrict__ beta, uint4* __restrict__ sum_out, uint4* __restrict__ norm_out,
    int M, int vec_per_row, long long rows, float eps) {
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  constexpr int K = Vec16<T>::kElts;
  float v[VPL][K];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int vi = lane + 64 * j;
#pragma unroll
    for (int i = 0; i < K; ++i) v[j][i] = 0.f;
    if (vi < vec_per_row) {
      Vec16<T>::unpack(x[row * vec_per_row + vi], v[j]);
      if (delta != nullptr) {
        float d[K];
        Vec16<T>::unpack(delta[row * vec_per_row + vi], d);
#pragma unroll
        for (int i = 0; i < K; ++i) v[j][i] += d[i];
        const uint4 packed = Vec16<T>::pack(v[j]);
        sum_out[row * vec_per_row + vi] = packed;
        Vec16<T>::unpack(packed, v[j]);               // normalise the stored (rounded) sum
      }
#pragma unroll
      for (int i = 0; i < K; ++i) s += v[j][i];
    }
  }
  const float mean = wave_sum(s) / (float)M;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j)
    if (lane + 64 * j < vec_per_row)
#pragma unroll
      for (int i = 0; i < K; ++i) q += (v[j][i] - mean) * (v[j][i] - mean);
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)M + eps);
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int vi = lane + 64 * j;
    if (vi < vec_per_row) {
      float o[K];
#pragma unroll
      for (int i = 0; i < K; ++i)
        o[i] = gamma[vi * K + i] * ((v[j][i] - mean) * rstd) + beta[vi * K + i];
      norm_out[row * vec_per_row + vi] = Vec16<T>::pack(o);
    }
  }
}

// y = a + b, 16 bytes per thread
template <typename T>
__global__ __launch_bounds__(256) void add_rows_kernel(const uint4* __restrict__ a,
                                                       const uint4* __restrict__ b,
                                                       uint4* __restrict__ y, long long vecs) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= vecs) return;
  constexpr int K = Vec16<T>::kElts;
  float fa[K], fb[K];
  Vec16<T>::unpack(a[i], fa);
  Vec16<T>::unpack(b[i], fb);
#pragma unroll
  for (int k = 0; k < K; ++k) fa[k] += fb[k];
  y[i] = Vec16<T>::pack(fa);
}

// ---------------------------------------------------------------- attention, plain form
// One wavefront per (sequence, head, query).  Scores of the whole row sit in LDS.
template <typename T>
__global__ __launch_bounds__(256) void attention_rows_kernel(
    const T* __restrict__ qkv, T* __restrict__ ctx, float* __restrict__ lse, int L, int heads, int d,
    long long queries) {
  extern __shared__ float att_smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* sc = att_smem + (size_t)wave * (L + d);        // [L] scores, then [d] the query row
  float* qs = sc + L;
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
  for (int i = lane; i < d; i += 64) qs[i] = Elt<T>::load(qrow + i);
  __builtin_amdgcn_wave_barrier();
  const float scale = 1.0f / sqrtf((float)d);
  float mx = -INFINITY;
  for (int k0 = 0; k0 < L; k0 += 64) {
    const int key = k0 + lane;
    if (key < L) {
      const T* kr = kbase + (size_t)key * ld;
      float dot = 0.f;
      for (int i = 0; i < d; ++i) dot = fmaf(qs[i], Elt<T>::load(kr + i), dot);
      dot *= scale;
      sc[key] = dot;
      mx = fmaxf(mx, dot);
    }
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int key = lane; key < L; key += 64) {
    const float p = expf(sc[key] - mx);
    sc[key] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if (lse != nullptr && lane == 0) lse[id] = mx + logf(sum);   // log sum_k exp(score), for the backward pass
  __builtin_amdgcn_wave_barrier();
  const float inv = 1.0f / sum;
  T* out = ctx + ((size_t)b * L + l) * A + (size_t)h * d;
  for (int i = lane; i < d; i += 64) {
    float acc = 0.f;
    for (int key = 0; key < L; ++key) acc = fmaf(sc[key], Elt<T>::load(vbase + (size_t)key * ld + i), acc);
    Elt<T>::store(out + i, acc * inv);
  }
}

// ---------------------------------------------------------------- attention, MFMA form
// Block = 128 queries of one (sequence, head); wavefront w owns queries 32 w .. 32 w + 31.
// Everything is computed transposed so that a lane owns ONE query column:
//   S^T = K . Q^T  (keys x queries): MFMA A operand = 32 keys x 16 d, B operand = Q^T, both
//         read as 16 contiguous bytes of a qkv row.  In the result a lane holds, per 32-key
//         tile, the 16 scores of its query for the keys 8 (i/4) + 4 (lane/32) + i%4.
//   online softmax over the keys: in-lane over those scores plus one exchange with the
//         partner lane (lane ^ 32), running maximum m and sum l per query.
//   O^T += V^T . P^T (d x queries): P^T is the B operand straight from the score registers
//         (acc values 8 s .. 8 s + 7 of a tile are the 8 keys of MFMA step s); V^T is the A
//         operand, fetched with the transposing LDS read from the V block staged as
//         [keys][d] with the key rows stored in the matching order (bits 2 and 3 of the key
//         index swapped inside each 32-key tile).
// The K and V blocks (64 keys x D each) are staged through LDS once per block and step, double
// buffered, the next block waiting in registers while the current one is multiplied.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <int D>
__global__ __launch_bounds__(256, 2) void attention_mfma_kernel(
    const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx, float* __restrict__ lse, int L,
    int heads) {
  constexpr int KS = D / 16;                 // MFMA steps over d for the scores
  constexpr int DT = D / 32;                 // 32-row tiles of O^T
  // Row pitches of the staged blocks, chosen for the 64 LDS banks: the 16-byte K reads of 16
  // consecutive rows must start 4 banks apart (pitch = 4 words mod 64), the transposing 8-byte V
  // reads of a half-wavefront touch 4 rows x 16 words (pitch = 16 words mod 64).
  constexpr int kKPitch = D * 2 + 16, kVPitch = D * 2 + 64;
  constexpr int kKTile = 64 * kKPitch;       // one staged K block of 64 keys (the V block follows it)
  constexpr int kStage = kKTile + 64 * kVPitch;
  __shared__ __attribute__((aligned(16))) unsigned char kvs[2][kStage];      // stage: K block, V block
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hf = lane >> 5;
  const int qblocks = L / 128;
  // Consecutive workgroups go to different XCDs (8, each with its own L2): give every XCD a
  // contiguous range of work items, so the query blocks of one (sequence, head), which read
  // the same K and V rows, run under one L2.
  unsigned work = blockIdx.x;
  const unsigned per_xcd = gridDim.x / 8;
  if (work < per_xcd * 8) work = (work % 8) * per_xcd + work / 8;
  const int qb = work % qblocks;
  const long long bh = work / qblocks;
  const int h = (int)(bh % heads);
  const long long b = bh / heads;
  const int A = heads * D;
  const size_t ld = (size_t)3 * A;
  const bf16_t* base = qkv + (size_t)b * L * ld + (size_t)h * D;
  const bf16_t* kbase = base + A;
  const bf16_t* vbase = base + 2 * A;

  // Q^T fragments of this wavefront's 32 queries: lane (r, hf) holds d = 16 s + 8 hf .. + 7
  const bf16_t* qrow = base + (size_t)(qb * 128 + wave * 32 + r) * ld;
  u32x4_t qf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const u32x4_t*>(qrow + 16 * s + 8 * hf);

  f32x16_t o[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[t][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;       // running maximum (in log2 units) and sum
  const float sl2 = 1.4426950408889634f / sqrtf((float)D);

  // cooperative staging of a block of 64 keys: K rows as they are, V rows in the order the
  // P^T operand needs (bits 2 and 3 of the key index swapped); 64 * D / 8 16-byte vectors each.
  // The block after the current one waits in registers while the current one is multiplied.
  constexpr int VV = 64 * D / 8 / 256;       // vectors per thread and operand
  constexpr int VPR = D / 8;                 // vectors per row
  u32x4_t kreg[VV], vreg[VV];
#define MOE_ATT_LOAD_KV(kb)                                                                   \
  _Pragma("unroll") for (int i = 0; i < VV; ++i) {                                            \
    const int f = tid + 256 * i, key = f / VPR, c = f % VPR;                                  \
    kreg[i] = *reinterpret_cast<const u32x4_t*>(kbase + (size_t)((kb) * 64 + key) * ld + 8 * c); \
    vreg[i] = *reinterpret_cast<const u32x4_t*>(vbase + (size_t)((kb) * 64 + key) * ld + 8 * c); \
  }
#define MOE_ATT_STORE_KV(stage)                                                               \
  _Pragma("unroll") for (int i = 0; i < VV; ++i) {                                            \
    const int f = tid + 256 * i, key = f / VPR, c = f % VPR;                                  \
    const int pos = (key & ~12) | ((key & 4) << 1) | ((key & 8) >> 1); /* swap bits 2, 3 */   \
    *reinterpret_cast<u32x4_t*>(&kvs[stage][key * kKPitch + 16 * c]) = kreg[i];               \
    *reinterpret_cast<u32x4_t*>(&kvs[stage][kKTile + pos * kVPitch + 16 * c]) = vreg[i];      \
  }
  const int nkb = L / 64;
  MOE_ATT_LOAD_KV(0)
  MOE_ATT_STORE_KV(0)
  __syncthreads();

  typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
  typedef u32x4_t __attribute__((address_space(3))) * lds_u4_ptr;
  typedef unsigned char __attribute__((address_space(3))) * lds_ptr;
  const uint32_t kvs0 = (uint32_t)(uintptr_t)((lds_ptr)&kvs[0][0]);
  const int p16 = lane & 15, bb = lane >> 4;
  const int krow0 = 8 * (bb >> 1) + (p16 >> 2);          // staged key row inside a 16-row step
  for (int kb = 0; kb < nkb; ++kb) {
    if (kb + 1 < nkb) MOE_ATT_LOAD_KV(kb + 1)
    const uint32_t kst = kvs0 + (kb & 1) * kStage, vst = kst + kKTile;
    // ---- scores S^T for 64 keys: two 32-key tiles; lane (r, hf) reads 16 bytes of key row r
    f32x16_t sacc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[t][i] = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const u32x4_t kf = *(lds_u4_ptr)(uintptr_t)(kst + (32 * t + r) * kKPitch + 32 * s + 16 * hf);
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf),
                                                          __builtin_bit_cast(bf16x8_t, qf[s]),
                                                          sacc[t], 0, 0, 0);
      }
    }
    // ---- online softmax for this lane's query (partner lane ^ 32 holds the other keys)
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[t][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sl2;        // sl2 > 0: scaling commutes with max
    const float m_new = fmaxf(m_run, mx);
    float psum = 0.f;
    u32x4_t pf[2][2];                                    // P^T fragments: tile t, MFMA step s
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float p[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) { p[i] = __builtin_amdgcn_exp2f(fmaf(sacc[t][i], sl2, -m_new)); psum += p[i]; }
#pragma unroll
      for (int s = 0; s < 2; ++s)
        pf[t][s] = u32x4_t{pack_bf16x2(p[8 * s], p[8 * s + 1]), pack_bf16x2(p[8 * s + 2], p[8 * s + 3]),
                           pack_bf16x2(p[8 * s + 4], p[8 * s + 5]), pack_bf16x2(p[8 * s + 6], p[8 * s + 7])};
    }
    psum += __shfl_xor(psum, 32, 64);
    // the running maximum rarely moves after the first blocks: rescale only when some query
    // of the wavefront needs it (alpha == 1 exactly otherwise)
    if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first block (m_run = -inf)
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[t][i] *= alpha;
    }
    l_run += psum;
    m_run = m_new;
    // ---- O^T += V^T . P^T: MFMA step (t, s) covers staged key rows 32 t + 16 s .. + 15
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          // lane needs V^T[d = 32 dt + lane%32][8 consecutive staged keys of its half]:
          // 16-lane block bb reads rows krow0 (+4), columns 32 dt + 16 (bb&1) + 4 (p16&3) .. +3
          const int col = 32 * dt + 16 * (bb & 1) + 4 * (p16 & 3);
          const uint32_t pv = vst + (32 * t + 16 * s + krow0) * kVPitch + 2 * col;
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)pv);
          const s16x4_t hi =
              __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(pv + 4 * kVPitch));
          const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8_t, pf[t][s]),
                                                          o[dt], 0, 0, 0);
        }
    // the other stage was last read one iteration ago, before the previous barrier
    if (kb + 1 < nkb) MOE_ATT_STORE_KV((kb + 1) & 1)
    __syncthreads();
  }
#undef MOE_ATT_LOAD_KV
#undef MOE_ATT_STORE_KV
  // o[dt][i]: d = 32 dt + 8 (i/4) + 4 hf + i%4 of query r: four consecutive d per 8-byte store
  const float inv = 1.0f / l_run;
  // row statistic for the backward pass: log sum_k exp(score) in natural-log units
  if (lse != nullptr && hf == 0)
    lse[(size_t)bh * L + qb * 128 + wave * 32 + r] = (m_run + log2f(l_run)) * 0.6931471805599453f;
  bf16_t* orow = ctx + ((size_t)b * L + qb * 128 + wave * 32 + r) * A + (size_t)h * D;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
      const u32x2_t w = {pack_bf16x2(o[dt][4 * q4] * inv, o[dt][4 * q4 + 1] * inv),
                         pack_bf16x2(o[dt][4 * q4 + 2] * inv, o[dt][4 * q4 + 3] * inv)};
      *reinterpret_cast<u32x2_t*>(orow + 32 * dt + 8 * q4 + 4 * hf) = w;
    }
}

}  // namespace

int launch_add_layer_norm(int act_dtype, const void* x, const void* delta, const float* gamma,
                          const float* beta, void* sum_out, void* norm_out, long long rows, int M,
                          hipStream_t st) {
  const int elt = act_dtype == MOE_F32 ? 4 : 2;
  const int vec_per_row = M * elt / 16;
  const int vpl = (vec_per_row + 63) / 64;
  if (vpl > 8) return MOE_EUNSUPPORTED;        // rows of more than 8192 bytes per lane set
  const unsigned grid = (unsigned)((rows + 3) / 4);
  const float eps = 1e-6f;
#define MOE_LN_CASE(T, V)                                                                     \
  hipLaunchKernelGGL((add_layer_norm_kernel<T, V>), dim3(grid), dim3(256), 0, st,             \
                     static_cast<const uint4*>(x), static_cast<const uint4*>(delta), gamma,   \
                     beta, static_cast<uint4*>(sum_out), static_cast<uint4*>(norm_out), M,    \
                     vec_per_row, rows, eps)
  if (act_dtype == MOE_F32) {
    if (vpl <= 1) MOE_LN_CASE(float, 1); else if (vpl <= 2) MOE_LN_CASE(float, 2);
    else if (vpl <= 4) MOE_LN_CASE(float, 4); else MOE_LN_CASE(float, 8);
  } else {
    if (vpl <= 1) MOE_LN_CASE(bf16_t, 1); else if (vpl <= 2) MOE_LN_CASE(bf16_t, 2);
    else if (vpl <= 4) MOE_LN_CASE(bf16_t, 4); else MOE_LN_CASE(bf16_t, 8);
  }
#undef MOE_LN_CASE
  return check_launch();
}

int launch_add_rows(int act_dtype, const void* a, const void* b, void* y, long long elems,
                    hipStream_t st) {
  const int elt = act_dtype == MOE_F32 ? 4 : 2;
  const long long vecs = elems * elt / 16;
  const unsigned grid = (unsigned)((vecs + 255) / 256);
  if (act_dtype == MOE_F32)
    hipLaunchKernelGGL(add_rows_kernel<float>, dim3(grid), dim3(256), 0, st,
                       static_cast<const uint4*>(a), static_cast<const uint4*>(b),
                       static_cast<uint4*>(y), vecs);
  else
    hipLaunchKernelGGL(add_rows_kernel<bf16_t>, dim3(grid), dim3(256), 0, st,
                       static_cast<const uint4*>(a), static_cast<const uint4*>(b),
                       static_cast<uint4*>(y), vecs);
  return check_launch();
}

// ctx [B*L, heads*d] from qkv [B*L, 3*heads*d]
int launch_attention_core(int act_dtype, const void* qkv, void* ctx, float* lse, long long B, int L,
                          int heads, int d, hipStream_t st) {
  if (act_dtype == MOE_BF16 && (d == 64 || d == 128) && L % 128 == 0) {
    const long long blocks = B * heads * (L / 128);
    if (blocks > 0x7fffffffLL) return MOE_EUNSUPPORTED;
    if (d == 64)
      hipLaunchKernelGGL(attention_mfma_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, st,
                         static_cast<const bf16_t*>(qkv), static_cast<bf16_t*>(ctx), lse, L, heads);
    else
      hipLaunchKernelGGL(attention_mfma_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, st,
                         static_cast<const bf16_t*>(qkv), static_cast<bf16_t*>(ctx), lse, L, heads);
    return check_launch();
  }
  const size_t shm = (size_t)4 * (L + d) * sizeof(float);
  if (shm > 64 * 1024) return MOE_EUNSUPPORTED;          // sequences of more than ~4000 tokens
  const long long queries = B * heads * L;
  const long long blocks = (queries + 3) / 4;
  if (blocks > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  if (act_dtype == MOE_F32)
    hipLaunchKernelGGL(attention_rows_kernel<float>, dim3((unsigned)blocks), dim3(256), shm, st,
                       static_cast<const float*>(qkv), static_cast<float*>(ctx), lse, L, heads, d, queries);
  else
    hipLaunchKernelGGL(attention_rows_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), shm, st,
                       static_cast<const bf16_t*>(qkv), static_cast<bf16_t*>(ctx), lse, L, heads, d, queries);
  return check_launch();
}

}  // namespace moe
