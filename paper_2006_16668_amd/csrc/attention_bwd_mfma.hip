// Backward of the scaled dot-product attention core on the matrix cores (bf16, d = 64 or 128,
// L a multiple of 128).  Section 2.1 of the paper names the self-attention sub-layer; the
// derivative is the chain rule of ctx = softmax(q k^T / sqrt(d)) v, with the probabilities
// recomputed from q, k and the stored row statistic lse = log sum_k exp(score):
//
//   p = exp(score - lse),  D = rowsum(dctx * ctx),  dv = p^T dctx,
//   ds = p * (dctx v^T - D) / sqrt(d),  dq = ds k,  dk = ds^T q
//
// Two kernels in the transposed arrangement of the forward kernel (a lane owns one column):
//
//   dq kernel   block = 128 queries of one (sequence, head), wavefront = 32 queries, two blocks
//               per CU with one LDS stage each (one block multiplies while the other stages the
//               next keys; 10-14 % faster than one block with two stages), loop over blocks of
//               64 keys:  S^T = K Q^T and dP^T = V dO^T (keys x queries; K, V rows from
//               LDS, Q^T and dO^T fragments in registers), dS^T in registers becomes the B operand
//               of dQ^T += K^T dS^T (K^T by the transposing LDS read).  Also writes D.
//   dkv kernel  block = 128 keys, wavefront = 32 keys, loop over blocks of 64 queries:
//               S = Q K^T and dP = dO V^T (queries x keys; Q, dO rows from LDS, K^T and V^T
//               fragments in registers), P and dS in registers become the B operands of
//               dV^T += dO^T P and dK^T += Q^T dS.
//
// MFMA register layout (v_mfma_f32_32x32x16_bf16): lane (r = lane % 32, hf = lane / 32) supplies
// row r of the first operand and column r of the second, k = 8 hf .. 8 hf + 7 of the step; it
// receives C[8 (i/4) + 4 hf + i%4][r] in value i.  Values 8 s .. 8 s + 7 of a result tile are
// therefore exactly the 8 k-values that lane owes the next product's step s, for the rows
// 16 s + 8 (j/4) + 4 hf + j%4: the operand read with the transposing LDS load is staged with
// bits 2 and 3 of its row index swapped, which puts those rows at 16 s + 8 hf + j.
#include <math.h>
#include "common.h"

namespace moe {
namespace {


typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
typedef u32x4_t __attribute__((address_space(3))) * lds_u4_ptr;
typedef f32x4_t __attribute__((address_space(3))) * lds_f4_ptr;
typedef unsigned char __attribute__((address_space(3))) * lds_ptr;

// Row pitches of staged 64-row blocks (64 LDS banks): 16-byte row reads of 16 consecutive rows
// start 4 banks apart; the transposing 8-byte reads of a half-wavefront touch 4 rows x 16 words.
template <int D> struct AttBwdGeom {
  static constexpr int kRowPitch = D * 2 + 16, kTrPitch = D * 2 + 64;
  static constexpr int kRowBlock = 64 * kRowPitch, kTrBlock = 64 * kTrPitch;
};

#define MOE_MFMA(a, b, c)                                                                      \
  __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),                      \
                                          __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0)

__device__ __forceinline__ u32x4_t pack8(const float* v) {
  return u32x4_t{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                 pack_bf16x2(v[6], v[7])};
}
// Consecutive workgroups go to different XCDs (8, each with its own L2).  This gives every XCD
// a contiguous range of work items instead, so the blocks of one (sequence, head), which read
// the same K / V (or Q / dO) rows, run under one L2.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned block, unsigned blocks) {
  const unsigned per_xcd = blocks / 8;
  return block < per_xcd * 8 ? (block % 8) * per_xcd + block / 8 : block;
}
__device__ __forceinline__ int swap_bits_2_3(int row) {
  return (row & ~12) | ((row & 4) << 1) | ((row & 8) >> 1);
}
// first operand fragment [32 d-rows x 16 staged rows] of a block staged [rows][d] with the
// transposing pitch: lane needs (d = 32 dt + lane%32, 8 consecutive staged rows of its half)
template <int PITCH>
__device__ __forceinline__ bf16x8_t read_transposed(uint32_t block, int row16, int dt, int lane) {
  const int p16 = lane & 15, bb = lane >> 4;
  const int krow0 = 8 * (bb >> 1) + (p16 >> 2);
  const int col = 32 * dt + 16 * (bb & 1) + 4 * (p16 & 3);
  const uint32_t pv = block + (row16 + krow0) * PITCH + 2 * col;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)pv);
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(pv + 4 * PITCH));
  return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// ---------------------------------------------------------------- dq (and D)
template <int D>
__global__ __launch_bounds__(256, 2) void attention_bwd_dq_mfma_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ ctx, const bf16_t* __restrict__ dctx,
    const float* __restrict__ lse, bf16_t* __restrict__ dqkv, float* __restrict__ dvec, int L,
    int heads) {
  using GM = AttBwdGeom<D>;
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int kVRows = GM::kRowBlock, kKPerm = 2 * GM::kRowBlock;   // stage: K rows, V rows, K permuted
  constexpr int kStage = 2 * GM::kRowBlock + GM::kTrBlock;
  extern __shared__ __attribute__((aligned(16))) unsigned char att_bwd_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hf = lane >> 5;
  const int qblocks = L / 128;
  const unsigned work = xcd_contiguous(blockIdx.x, gridDim.x);
  const int qb = work % qblocks;
  const long long bh = work / qblocks;
  const int h = (int)(bh % heads);
  const long long b = bh / heads;
  const int A = heads * D;
  const size_t ld = (size_t)3 * A;
  const bf16_t* base = qkv + (size_t)b * L * ld + (size_t)h * D;
  const bf16_t* kbase = base + A;
  const bf16_t* vbase = base + 2 * A;
  const int q = qb * 128 + wave * 32 + r;

  // Q^T and dO^T fragments of this wavefront's queries, D of the lane's query
  const bf16_t* qrow = base + (size_t)q * ld;
  const size_t crow = ((size_t)b * L + q) * A + (size_t)h * D;
  u32x4_t qf[KS], dof[KS];
  float dd = 0.f;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    qf[s] = *reinterpret_cast<const u32x4_t*>(qrow + 16 * s + 8 * hf);
    dof[s] = *reinterpret_cast<const u32x4_t*>(dctx + crow + 16 * s + 8 * hf);
    const u32x4_t of = *reinterpret_cast<const u32x4_t*>(ctx + crow + 16 * s + 8 * hf);
    float g[8], o[8];
    Vec16<bf16_t>::unpack(uint4{dof[s][0], dof[s][1], dof[s][2], dof[s][3]}, g);
    Vec16<bf16_t>::unpack(uint4{of[0], of[1], of[2], of[3]}, o);
#pragma unroll
    for (int i = 0; i < 8; ++i) dd = fmaf(g[i], o[i], dd);
  }
  dd += __shfl_xor(dd, 32, 64);
  if (hf == 0) dvec[(size_t)bh * L + q] = dd;
  const float lse2 = lse[(size_t)bh * L + q] * 1.4426950408889634f;
  const float scale = 1.0f / sqrtf((float)D);
  const float sl2 = 1.4426950408889634f * scale;

  f32x16_t dq[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) dq[t][i] = 0.f;

  constexpr int VV = 64 * D / 8 / 256, VPR = D / 8;
  u32x4_t kreg[VV], vreg[VV];
#define MOE_ATTB_LOAD(kb)                                                                     \
  _Pragma("unroll") for (int i = 0; i < VV; ++i) {                                            \
    const int f = tid + 256 * i, key = f / VPR, c = f % VPR;                                  \
    kreg[i] = *reinterpret_cast<const u32x4_t*>(kbase + (size_t)((kb) * 64 + key) * ld + 8 * c); \
    vreg[i] = *reinterpret_cast<const u32x4_t*>(vbase + (size_t)((kb) * 64 + key) * ld + 8 * c); \
  }
#define MOE_ATTB_STORE(stage)                                                                 \
  _Pragma("unroll") for (int i = 0; i < VV; ++i) {                                            \
    const int f = tid + 256 * i, key = f / VPR, c = f % VPR;                                  \
    unsigned char* sb = att_bwd_lds + (stage) * kStage;                                       \
    *reinterpret_cast<u32x4_t*>(sb + key * GM::kRowPitch + 16 * c) = kreg[i];                 \
    *reinterpret_cast<u32x4_t*>(sb + kVRows + key * GM::kRowPitch + 16 * c) = vreg[i];        \
    *reinterpret_cast<u32x4_t*>(sb + kKPerm + swap_bits_2_3(key) * GM::kTrPitch + 16 * c) = kreg[i]; \
  }
  const int nkb = L / 64;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_ptr)att_bwd_lds);
  for (int kb = 0; kb < nkb; ++kb) {
    // one LDS stage, two blocks per CU: the other block multiplies while this one stages
    MOE_ATTB_LOAD(kb)
    __syncthreads();                         // the previous key block has been read by everyone
    MOE_ATTB_STORE(0)
    __syncthreads();
    const uint32_t kst = lds0, vst = kst + kVRows, kpst = kst + kKPerm;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16_t sacc, dpacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const uint32_t off = (32 * t + r) * GM::kRowPitch + 32 * s + 16 * hf;
        const u32x4_t kf = *(lds_u4_ptr)(uintptr_t)(kst + off);
        const u32x4_t vf = *(lds_u4_ptr)(uintptr_t)(vst + off);
        sacc = MOE_MFMA(kf, qf[s], sacc);
        dpacc = MOE_MFMA(vf, dof[s], dpacc);
      }
      float ds[16];
#pragma unroll
      for (int i = 0; i < 16; ++i)
        ds[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], sl2, -lse2)) * (dpacc[i] - dd);
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const u32x4_t dsf = pack8(ds + 8 * s);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              read_transposed<GM::kTrPitch>(kpst, 32 * t + 16 * s, dt, lane),
              __builtin_bit_cast(bf16x8_t, dsf), dq[dt], 0, 0, 0);
      }
    }
  }
#undef MOE_ATTB_LOAD
#undef MOE_ATTB_STORE
  // dq[dt][i]: d = 32 dt + 8 (i/4) + 4 hf + i%4 of query r
  bf16_t* orow = dqkv + ((size_t)b * L + q) * ld + (size_t)h * D;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const u32x2_t w = {pack_bf16x2(dq[dt][4 * q4] * scale, dq[dt][4 * q4 + 1] * scale),
                         pack_bf16x2(dq[dt][4 * q4 + 2] * scale, dq[dt][4 * q4 + 3] * scale)};
      *reinterpret_cast<u32x2_t*>(orow + 32 * dt + 8 * q4 + 4 * hf) = w;
    }
}

// ---------------------------------------------------------------- dk, dv
template <int D>
__global__ __launch_bounds__(256, 1) void attention_bwd_dkv_mfma_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx, const float* __restrict__ lse,
    const float* __restrict__ dvec, bf16_t* __restrict__ dqkv, int L, int heads) {
  using GM = AttBwdGeom<D>;
  constexpr int KS = D / 16, DT = D / 32;
  // stage: Q rows, dO rows, Q permuted, dO permuted, then 64 lse (log2 units) and 64 D
  constexpr int kGRows = GM::kRowBlock, kQPerm = 2 * GM::kRowBlock, kGPerm = kQPerm + GM::kTrBlock;
  constexpr int kStats = kGPerm + GM::kTrBlock;
  constexpr int kStage = kStats + 512;
  extern __shared__ __attribute__((aligned(16))) unsigned char att_bwd_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hf = lane >> 5;
  const int kblocks = L / 128;
  const unsigned work = xcd_contiguous(blockIdx.x, gridDim.x);
  const int kblk = work % kblocks;
  const long long bh = work / kblocks;
  const int h = (int)(bh % heads);
  const long long b = bh / heads;
  const int A = heads * D;
  const size_t ld = (size_t)3 * A;
  const bf16_t* qbase = qkv + (size_t)b * L * ld + (size_t)h * D;
  const bf16_t* gbase = dctx + (size_t)b * L * A + (size_t)h * D;
  const float* lse_h = lse + (size_t)bh * L;
  const float* dvec_h = dvec + (size_t)bh * L;
  const int key = kblk * 128 + wave * 32 + r;

  // K and V fragments of this wavefront's keys: lane (r, hf) holds d = 16 s + 8 hf .. + 7
  const bf16_t* krow = qbase + (size_t)key * ld + A;
  u32x4_t kf[KS], vf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    kf[s] = *reinterpret_cast<const u32x4_t*>(krow + 16 * s + 8 * hf);
    vf[s] = *reinterpret_cast<const u32x4_t*>(krow + A + 16 * s + 8 * hf);
  }
  const float scale = 1.0f / sqrtf((float)D);
  const float sl2 = 1.4426950408889634f * scale;

  f32x16_t dk[DT], dv[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dk[t][i] = 0.f; dv[t][i] = 0.f; }

  constexpr int VV = 64 * D / 8 / 256, VPR = D / 8;
  u32x4_t qreg[VV], greg[VV];
  float st_reg = 0.f;                        // threads 0..63: lse, 64..127: D of query tid % 64
#define MOE_ATTB_LOAD(qb)                                                                     \
  {                                                                                           \
    _Pragma("unroll") for (int i = 0; i < VV; ++i) {                                          \
      const int f = tid + 256 * i, row = f / VPR, c = f % VPR;                                \
      qreg[i] = *reinterpret_cast<const u32x4_t*>(qbase + (size_t)((qb) * 64 + row) * ld + 8 * c); \
      greg[i] = *reinterpret_cast<const u32x4_t*>(gbase + (size_t)((qb) * 64 + row) * A + 8 * c); \
    }                                                                                         \
    if (tid < 64) st_reg = lse_h[(qb) * 64 + tid] * 1.4426950408889634f;                      \
    else if (tid < 128) st_reg = dvec_h[(qb) * 64 + tid - 64];                                \
  }
#define MOE_ATTB_STORE(stage)                                                                 \
  {                                                                                           \
    unsigned char* sb = att_bwd_lds + (stage) * kStage;                                       \
    _Pragma("unroll") for (int i = 0; i < VV; ++i) {                                          \
      const int f = tid + 256 * i, row = f / VPR, c = f % VPR;                                \
      const int pos = swap_bits_2_3(row);                                                     \
      *reinterpret_cast<u32x4_t*>(sb + row * GM::kRowPitch + 16 * c) = qreg[i];               \
      *reinterpret_cast<u32x4_t*>(sb + kGRows + row * GM::kRowPitch + 16 * c) = greg[i];      \
      *reinterpret_cast<u32x4_t*>(sb + kQPerm + pos * GM::kTrPitch + 16 * c) = qreg[i];       \
      *reinterpret_cast<u32x4_t*>(sb + kGPerm + pos * GM::kTrPitch + 16 * c) = greg[i];       \
    }                                                                                         \
    if (tid < 128) *reinterpret_cast<float*>(sb + kStats + 4 * tid) = st_reg;                 \
  }
  const int nqb = L / 64;
  MOE_ATTB_LOAD(0)
  MOE_ATTB_STORE(0)
  __syncthreads();
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_ptr)att_bwd_lds);
  for (int qb = 0; qb < nqb; ++qb) {
    if (qb + 1 < nqb) MOE_ATTB_LOAD(qb + 1)
    const uint32_t qst = lds0 + (qb & 1) * kStage, gst = qst + kGRows;
    const uint32_t qpst = qst + kQPerm, gpst = qst + kGPerm, sst = qst + kStats;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16_t sacc, dpacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const uint32_t off = (32 * t + r) * GM::kRowPitch + 32 * s + 16 * hf;
        const u32x4_t qf = *(lds_u4_ptr)(uintptr_t)(qst + off);
        const u32x4_t gf = *(lds_u4_ptr)(uintptr_t)(gst + off);
        sacc = MOE_MFMA(qf, kf[s], sacc);         // S[query][key]
        dpacc = MOE_MFMA(gf, vf[s], dpacc);       // dP[query][key]
      }
      // value i belongs to query 32 t + 8 (i/4) + 4 hf + i%4: four consecutive queries per i/4
      float p[16], ds[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int q0 = 32 * t + 8 * g4 + 4 * hf;
        const f32x4_t l4 = *(lds_f4_ptr)(uintptr_t)(sst + 4 * q0);
        const f32x4_t d4 = *(lds_f4_ptr)(uintptr_t)(sst + 256 + 4 * q0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int i = 4 * g4 + j;
          p[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], sl2, -l4[j]));
          ds[i] = p[i] * (dpacc[i] - d4[j]);
        }
      }
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const u32x4_t pf = pack8(p + 8 * s), dsf = pack8(ds + 8 * s);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              read_transposed<GM::kTrPitch>(gpst, 32 * t + 16 * s, dt, lane),
              __builtin_bit_cast(bf16x8_t, pf), dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              read_transposed<GM::kTrPitch>(qpst, 32 * t + 16 * s, dt, lane),
              __builtin_bit_cast(bf16x8_t, dsf), dk[dt], 0, 0, 0);
        }
      }
    }
    if (qb + 1 < nqb) MOE_ATTB_STORE((qb + 1) & 1)
    __syncthreads();
  }
#undef MOE_ATTB_LOAD
#undef MOE_ATTB_STORE
  // dk[dt][i], dv[dt][i]: d = 32 dt + 8 (i/4) + 4 hf + i%4 of key r
  bf16_t* orow = dqkv + ((size_t)b * L + key) * ld + A + (size_t)h * D;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const u32x2_t wk = {pack_bf16x2(dk[dt][4 * q4] * scale, dk[dt][4 * q4 + 1] * scale),
                          pack_bf16x2(dk[dt][4 * q4 + 2] * scale, dk[dt][4 * q4 + 3] * scale)};
      const u32x2_t wv = {pack_bf16x2(dv[dt][4 * q4], dv[dt][4 * q4 + 1]),
                          pack_bf16x2(dv[dt][4 * q4 + 2], dv[dt][4 * q4 + 3])};
      *reinterpret_cast<u32x2_t*>(orow + 32 * dt + 8 * q4 + 4 * hf) = wk;
      *reinterpret_cast<u32x2_t*>(orow + A + 32 * dt + 8 * q4 + 4 * hf) = wv;
    }
}

template <int D>
int prepare_bwd() {
  using GM = AttBwdGeom<D>;
  constexpr int kLdsQ = 2 * GM::kRowBlock + GM::kTrBlock;      // one stage
  constexpr int kLdsKV = 2 * (2 * GM::kRowBlock + 2 * GM::kTrBlock + 512);
  static_assert(kLdsKV <= 160 * 1024, "two stages must fit the 160 KB of LDS");
  static LdsLimitOnce once_q, once_kv;
  const int rc = ensure_lds_limit(once_q, reinterpret_cast<const void*>(attention_bwd_dq_mfma_kernel<D>), kLdsQ);
  if (rc != MOE_OK) return rc;
  return ensure_lds_limit(once_kv, reinterpret_cast<const void*>(attention_bwd_dkv_mfma_kernel<D>), kLdsKV);
}

template <int D>
int launch_bwd(const bf16_t* qkv, const bf16_t* ctx, const bf16_t* dctx, const float* lse,
               bf16_t* dqkv, float* dvec, long long B, int L, int heads, hipStream_t st) {
  using GM = AttBwdGeom<D>;
  constexpr int kLdsQ = 2 * GM::kRowBlock + GM::kTrBlock;      // one stage
  constexpr int kLdsKV = 2 * (2 * GM::kRowBlock + 2 * GM::kTrBlock + 512);
  auto kq = attention_bwd_dq_mfma_kernel<D>;
  auto kkv = attention_bwd_dkv_mfma_kernel<D>;
  if (prepare_bwd<D>() != MOE_OK) return MOE_EHIP;
  const long long blocks = B * heads * (L / 128);
  if (blocks > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  hipLaunchKernelGGL(kq, dim3((unsigned)blocks), dim3(256), kLdsQ, st, qkv, ctx, dctx, lse, dqkv, dvec,
                     L, heads);
  hipLaunchKernelGGL(kkv, dim3((unsigned)blocks), dim3(256), kLdsKV, st, qkv, dctx, lse, dvec, dqkv, L,
                     heads);
  return check_launch();
}

}  // namespace

bool attention_bwd_mfma_ok(int act_dtype, int L, int d) {
  return act_dtype == MOE_BF16 && (d == 64 || d == 128) && L % 128 == 0;
}

int prepare_attention_bwd() {
  const int rc = prepare_bwd<64>();
  return rc != MOE_OK ? rc : prepare_bwd<128>();
}

int launch_attention_bwd_mfma(const void* qkv, const void* ctx, const void* dctx, const float* lse,
                              void* dqkv, float* dvec, long long B, int L, int heads, int d,
                              hipStream_t st) {
  if (!attention_bwd_mfma_ok(MOE_BF16, L, d)) return MOE_EUNSUPPORTED;
  auto q = static_cast<const bf16_t*>(qkv);
  auto c = static_cast<const bf16_t*>(ctx);
  auto g = static_cast<const bf16_t*>(dctx);
  auto o = static_cast<bf16_t*>(dqkv);
  return d == 64 ? launch_bwd<64>(q, c, g, lse, o, dvec, B, L, heads, st)
                 : launch_bwd<128>(q, c, g, lse, o, dvec, B, L, heads, st);
}

}  // namespace moe
