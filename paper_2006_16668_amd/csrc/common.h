// Shared device helpers for the gfx950 MoE kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "../../include/moe_gfx950.h"

namespace moe {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int kWave = 64;
constexpr int kChunk = 64;  // tokens per routing chunk (one wavefront)

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(((uint32_t)v) << 16);
}
// round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// two fp32 -> packed bf16 with the hardware conversion (v_cvt_pk_bf16_f32, round to nearest even)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// max(v, 0) on two packed bf16 in one op: a negative bf16 is a negative 16-bit integer
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t v) {
  typedef short s16x2_t __attribute__((ext_vector_type(2)));
  const s16x2_t zero = {0, 0};
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2_t, v), zero));
}

template <typename T> struct Elt;
template <> struct Elt<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elt<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 16 bytes of a row as floats and back (one rounding on the way back)
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int kElts = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return uint4{__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                 __float_as_uint(f[3])};
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int kElts = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return uint4{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                 pack_bf16x2(f[6], f[7])};
  }
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Packed row layout of the expert GEMMs (Section 2.2, "Expert capacity": a buffer position holds
// a token or nothing, and FFN_e(0) = 0, so positions that hold nothing need not be multiplied).
// The kept rows of expert e (kept_e = sum over g of fill[g,e]), in (group, slot) order, occupy
// rows 0 .. kept_e - 1 of its block of R = G*C rows; only the ceil(kept_e / 256) row tiles that
// hold them are multiplied.  The GEMM kernels derive the tile counts from kept.
struct RowPacking {
  int32_t* row_base;     // [G,E]  kept rows of expert e in the groups before g
  int32_t* kept;         // [E]    kept_e
  int32_t* packed_src;   // [E,R]  source row of packed row p < kept_e (a row index into the A
                         //        operand's matrix); entries from kept_e on are not written
};
inline size_t row_packing_bytes(const moe_config& c) {      // the three arrays, each 256-aligned
  const size_t rows = (size_t)c.E * c.G * c.C;
  return align_up((size_t)c.G * c.E * 4, 256) + align_up((size_t)c.E * 4, 256) + align_up(rows * 4, 256);
}
inline RowPacking carve_row_packing(const moe_config& c, void* base) {
  const size_t rows = (size_t)c.E * c.G * c.C;
  char* p = static_cast<char*>(base);
  RowPacking pk;
  pk.row_base = reinterpret_cast<int32_t*>(p);
  p += align_up((size_t)c.G * c.E * 4, 256);
  pk.kept = reinterpret_cast<int32_t*>(p);
  p += align_up((size_t)c.E * 4, 256);
  pk.packed_src = reinterpret_cast<int32_t*>(p);
  (void)rows;
  return pk;
}

// host-side launchers (each returns a moe_status)
// zero_row: NULL, or M bf16 elements that the gate also clears (see launch_expert_gemm1_gather)
// packing: NULL, or the arrays of the packed row layout that the gate also fills (packed_src
// then holds token rows g*S + s of x)
int launch_gate(const moe_config& c, const void* x, const float* wg, const float* u,
                int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
                int32_t* src_token, int32_t* c1, float* mean_gate, float* aux,
                float* gates_opt, void* ws, void* zero_row, const RowPacking* packing,
                const void* wg_prepacked, hipStream_t st);
// wg in the form the logit kernels multiply (gate_pack_bytes may be 0: nothing to pack);
// wg_prepacked of launch_gate: NULL, or the result of launch_gate_pack for the same config and wg
size_t gate_pack_bytes(const moe_config& c);
int launch_gate_pack(const moe_config& c, const float* wg, void* packed, hipStream_t st);
// the packed row layout from fill alone, sources = rows of an [E,G,C,M] buffer; clears zero_row
int launch_row_maps_from_fill(const moe_config& c, const int32_t* fill, const RowPacking& pk,
                              void* zero_row, hipStream_t st);
size_t gate_workspace_bytes(const moe_config& c);
// kept: NULL, or the packed layout's row counts (src_token is then its packed_src)
int launch_dispatch(const moe_config& c, const void* x, const int32_t* src_token, void* buf,
                    const int32_t* kept, hipStream_t st);
// row_base: NULL (out is [E,G,C,M]) or the [G,E] offsets of the packed row layout
int launch_combine(const moe_config& c, const void* out, const int32_t* expert_idx,
                   const int32_t* slot, const float* weight, const int32_t* row_base, void* y,
                   hipStream_t st);
// h = relu(buf . wi) and out = h . wo, one grouped GEMM launch each
int launch_expert_gemm1(const moe_config& c, const void* buf, const void* wi, void* h,
                        hipStream_t st);
int launch_expert_gemm2(const moe_config& c, const void* h, const void* wo, void* out,
                        hipStream_t st);
// h = relu(dispatch(x) . wi) without materialising the dispatched buffer: the GEMM's copies
// gather the rows of x through src_token (zero_row: M zeros of the activation type).
bool expert_gemm1_can_gather(const moe_config& c);
// signbits: NULL, or expert_signbits_bytes(c) bytes that receive one bit per element of h
// (set where h > 0) in the GEMM kernel's private tile order, for launch_expert_dgrad2
int launch_expert_gemm1_gather(const moe_config& c, const void* x, const int32_t* src_token,
                               const void* zero_row, const void* wi, void* h, void* signbits,
                               hipStream_t st);
// both GEMMs over the packed row layout (bf16 layers the persistent kernel takes, M >= 128)
bool expert_ffn_can_pack(const moe_config& c);
int launch_expert_ffn_packed(const moe_config& c, const void* a, const RowPacking& pk,
                             const void* zero_row, const void* wi, const void* wo, void* h,
                             void* out, bool scatter_out, void* signbits, hipStream_t st,
                             void* event_between);
inline size_t expert_signbits_bytes(const moe_config& c) {
  return (size_t)c.E * c.G * c.C * c.H / 8;
}

// backward pass (backward.hip); epi of the strided GEMM: 0 none, 1 relu, 2 zero where mask <= 0
int launch_combine_bwd(const moe_config& c, const void* dy, const void* out,
                       const int32_t* src_token, const int32_t* expert_idx, const float* weight,
                       void* dout, float* dweight, const int32_t* kept, hipStream_t st);
// Gate gradients: on bf16 layers whose token count and M are multiples of 256 the two
// projections (dwg = x^T dz, dz . wg^T) run on the matrix cores; otherwise fp32 FMA kernels.
struct GateBwdPlan {
  bool mfma;
  int cols;     // mfma: columns of the 3-term bf16 copy of dz, 3E rounded up to 256
  int splits;   // token ranges of the dwg partial sums
  size_t dz_bytes, dzp_bytes, wgp_bytes, dxg_bytes, partial_bytes;
};
GateBwdPlan gate_bwd_plan(const moe_config& c);
struct GateBwdWs {
  float* dz;        // [N,E] fp32 (FMA path)
  bf16_t* dzp;      // [N,cols] bf16 terms of dz (MFMA path)
  bf16_t* wgp;      // [M,cols] bf16 wg repeated per term (MFMA path)
  float* dxg;       // [N,M] fp32 gate part of dx (MFMA path)
  float* partial;   // [splits,M,E or cols] fp32
};
int launch_gate_bwd(const moe_config& c, const void* x, const float* wg, const float* gates,
                    const int32_t* expert_idx, const int32_t* slot, const float* dweight,
                    const int32_t* c1, const float* daux, const GateBwdWs& w, float* dwg,
                    hipStream_t st);
int launch_dx(const moe_config& c, const float* wg, const void* dbuf, const int32_t* expert_idx,
              const int32_t* slot, const GateBwdWs& w, void* dx, const int32_t* row_base,
              hipStream_t st);
int launch_gemm_strided(const moe_config& c, int epi, const void* A, long long a_e, long long a_r,
                        long long a_k, const void* B, long long b_e, long long b_k, long long b_n,
                        void* Cout, const void* mask, int R, int N, int K, hipStream_t st);
// expert GEMMs of the backward pass (expert_gemm.hip), per expert with rows = G*C:
//   dgrad2: dh   = (dout . wo^T) masked by h > 0     [rows,M] x [H,M]^T -> [rows,H]
//           (signbits as written by launch_expert_gemm1_gather when that path ran, else NULL)
//   wgrad2: dwo  = h^T . dout                        [rows,H]^T x [rows,M] -> [H,M]
//   dgrad1: dbuf = dh . wi^T                         [rows,H] x [M,H]^T -> [rows,M]
//   wgrad1: dwi  = buf^T . dh                        [rows,M]^T x [rows,H] -> [M,H]
// kept: NULL, or the row counts of the packed layout (then rows are packed rows: the data
// gradients walk the occupied row tiles only and the weight gradients sum over them only)
int launch_expert_dgrad2(const moe_config& c, const void* dout, const void* wo, const void* h,
                         const void* signbits, void* dh, const int32_t* kept, hipStream_t st);
int launch_expert_wgrad2(const moe_config& c, const void* h, const void* dout, void* dwo,
                         const int32_t* kept, hipStream_t st);
int launch_expert_dgrad1(const moe_config& c, const void* dh, const void* wi, void* dbuf,
                         const int32_t* kept, hipStream_t st);
int launch_expert_wgrad1(const moe_config& c, const void* buf, const void* dh, void* dwi,
                         const int32_t* kept, hipStream_t st);

// batched bf16 MFMA GEMM with an fp32 result (expert_gemm.hip): transposed_a ? C = A^T.B with
// A [batch,K,R], B [batch,K,N] : C = A.B^T with A [batch,R,K], B [batch,N,K]; C [batch,R,N]
bool gemm_bf16_f32out_ok(int R, int N, int K);
int launch_gemm_bf16_f32out(bool transposed_a, const void* A, const void* B, float* Cout,
                            int batch, int R, int N, int K, hipStream_t st);

// fp32 GEMM on the matrix cores (gemm_f32.hip), strides as in launch_gemm_strided; every operand
// needs one unit stride and 16-byte alignment along it (gemm_f32_mfma_ok says whether it fits)
bool gemm_f32_mfma_ok(long long a_r, long long a_k, long long b_k, long long b_n, int E, int R, int N,
                      int K);
int launch_gemm_f32_mfma(int epi, const float* A, long long a_e, long long a_r, long long a_k,
                         const float* B, long long b_e, long long b_k, long long b_n, float* Cout,
                         const float* mask, int E, int R, int N, int K, hipStream_t st);

// Transformer encoder sub-layers around the MoE layer (encoder.hip)
int launch_add_layer_norm(int act_dtype, const void* x, const void* delta, const float* gamma,
                          const float* beta, void* sum_out, void* norm_out, long long rows, int M,
                          hipStream_t st);
int launch_add_rows(int act_dtype, const void* a, const void* b, void* y, long long elems,
                    hipStream_t st);
// lse: NULL, or [B*heads*L] fp32 that receives log sum_k exp(score) per query row (training)
int launch_attention_core(int act_dtype, const void* qkv, void* ctx, float* lse, long long B, int L,
                          int heads, int d, hipStream_t st);

// backward of the encoder sub-layers (encoder_bwd.hip)
//   ds = dres (may be NULL) + d LN(s) / d s applied to dn; dgamma, dbeta [M]; partial:
//   layer_norm_bwd_parts(rows) * 2 * M floats of scratch.  dx may alias dres.
int layer_norm_bwd_parts(long long rows);
int launch_layer_norm_bwd(int act_dtype, const void* s, const void* dn, const float* gamma,
                          const void* dres, void* dx, float* partial, float* dgamma, float* dbeta,
                          long long rows, int M, hipStream_t st);
//   dqkv [B*L, 3*heads*d] from qkv, ctx, dctx [B*L, heads*d] and lse; dvec: [B*heads*L] scratch
// dW [in,out] = X^T dY over rows tokens (X [rows,in], dY [rows,out]); partial: scratch of
// dense_wgrad_partial_bytes() for the token ranges of the split (may be NULL: no split)
int dense_wgrad_splits(int act_dtype, long long rows, int in, int out);
size_t dense_wgrad_partial_bytes(int act_dtype, long long rows, int in, int out);
int launch_dense_wgrad(const moe_config& c, long long rows, int in, int out, const void* X,
                       const void* dY, void* dW, float* partial, hipStream_t st);
// MFMA form (attention_bwd_mfma.hip): bf16, d = 64 or 128, L % 128 == 0
bool attention_bwd_mfma_ok(int act_dtype, int L, int d);
int launch_attention_bwd_mfma(const void* qkv, const void* ctx, const void* dctx, const float* lse,
                              void* dqkv, float* dvec, long long B, int L, int heads, int d,
                              hipStream_t st);
int launch_attention_core_bwd(int act_dtype, const void* qkv, const void* ctx, const void* dctx,
                              const float* lse, void* dqkv, float* dvec, long long B, int L,
                              int heads, int d, hipStream_t st);

inline int check_launch() { return hipPeekAtLastError() == hipSuccess ? MOE_OK : MOE_EHIP; }

// A kernel that uses more than 64 KB of dynamic LDS needs its limit raised once per device
// before its first launch.  Every launcher of such a kernel calls ensure_lds_limit (cheap after
// the first time, safe from several host threads: the flag is atomic and setting the attribute
// twice is harmless); the prepare_* functions do the same for every such kernel of a source
// file up front, so that the first real call has nothing left to set up.
constexpr int kMaxDevices = 64;   // devices one process can address
struct LdsLimitOnce { std::atomic<int> done[kMaxDevices]; };
inline int ensure_lds_limit(LdsLimitOnce& once, const void* kernel, int bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_EHIP;
  if (once.done[dev].load(std::memory_order_acquire) != 0) return MOE_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return MOE_EHIP;
  once.done[dev].store(1, std::memory_order_release);
  return MOE_OK;
}
int compute_units(int* cus);      // of the current device (cached per device)
int prepare_expert_gemm();        // expert_gemm.hip
int prepare_gate();               // gate.hip
int prepare_attention_bwd();      // attention_bwd_mfma.hip

}  // namespace moe
