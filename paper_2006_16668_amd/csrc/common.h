// Shared device helpers for the gfx950 MoE kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/moe_gfx950.h"

namespace moe {

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

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// host-side launchers (each returns a moe_status)
// zero_row: NULL, or M bf16 elements that the gate also clears (see launch_expert_gemm1_gather)
int launch_gate(const moe_config& c, const void* x, const float* wg, const float* u,
                int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
                int32_t* src_token, int32_t* c1, float* mean_gate, float* aux,
                float* gates_opt, void* ws, void* zero_row, hipStream_t st);
size_t gate_workspace_bytes(const moe_config& c);
int launch_dispatch(const moe_config& c, const void* x, const int32_t* src_token, void* buf,
                    hipStream_t st);
int launch_combine(const moe_config& c, const void* out, const int32_t* expert_idx,
                   const int32_t* slot, const float* weight, void* y, hipStream_t st);
// h = relu(buf . wi) and out = h . wo, one grouped GEMM launch each
int launch_expert_gemm1(const moe_config& c, const void* buf, const void* wi, void* h,
                        hipStream_t st);
int launch_expert_gemm2(const moe_config& c, const void* h, const void* wo, void* out,
                        hipStream_t st);
// h = relu(dispatch(x) . wi) without materialising the dispatched buffer: the GEMM's copies
// gather the rows of x through src_token (zero_row: M zeros of the activation type).
bool expert_gemm1_can_gather(const moe_config& c);
int launch_expert_gemm1_gather(const moe_config& c, const void* x, const int32_t* src_token,
                               const void* zero_row, const void* wi, void* h, hipStream_t st);

inline int check_launch() { return hipPeekAtLastError() == hipSuccess ? MOE_OK : MOE_EHIP; }

}  // namespace moe
