// fp32 expert GEMMs on the matrix cores (v_mfma_f32_32x32x2_f32: full fp32 products, fp32
// accumulation).  The paper trained its experts in fp32 (Section 4, "Model Details"); bf16 is
// this library's fast path, this kernel is the fp32 one for all six expert GEMMs of the forward
// and backward pass and the dense layers around them.
//
//   C[e,r,n] = epi( sum_k A[e*a_e + r*a_r + k*a_k] * B[e*b_e + k*b_k + n*b_n] ),  C row-major
//
// Each operand must have one unit stride (K-contiguous or row-contiguous); the kernel reads it
// with 16-byte loads along that direction and stages it K-major in LDS ([k][row], padded), so
// that the MFMA operands (lane l: row l % 32, k = l / 32) are conflict-free 4-byte reads.
// Block = 128 x 128 tile, 4 wavefronts of 64 x 64 (2 x 2 MFMA tiles), 16-wide K steps, double
// buffered through registers.  Dimensions along a unit stride must be multiples of 4.
#include "common.h"

namespace moe {
namespace {

typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kT = 128, kBK = 16, kPitch = kT + 4;

// one operand tile: 128 rows x 16 k; thread t fetches two 16-byte vectors
struct TileRegs { f32x4_t v[2]; };

// UNIT_K: the operand is K-contiguous (thread: row t/2, k 8 (t%2) .. +7)
//         else row-contiguous          (thread: k t/16, rows 8 (t%16) .. +7)
template <bool UNIT_K>
__device__ __forceinline__ void load_tile(TileRegs& r, const float* __restrict__ base,
                                          long long s_row, long long s_k, int row0, int k0,
                                          int rows, int K, int tid) {
  const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
  if (UNIT_K) {
    const int row = row0 + (tid >> 1), k = k0 + 8 * (tid & 1);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const bool ok = row < rows && k + 4 * i < K;          // K % 4 == 0: no straddling
      const float* p = base + (long long)(ok ? row : 0) * s_row + (ok ? k + 4 * i : 0);
      const f32x4_t v = *reinterpret_cast<const f32x4_t*>(p);
      r.v[i] = ok ? v : zero;
    }
  } else {
    const int k = k0 + (tid >> 4), row = row0 + 8 * (tid & 15);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const bool ok = k < K && row + 4 * i < rows;          // rows % 4 == 0
      const float* p = base + (long long)(ok ? k : 0) * s_k + (ok ? row + 4 * i : 0);
      const f32x4_t v = *reinterpret_cast<const f32x4_t*>(p);
      r.v[i] = ok ? v : zero;
    }
  }
}

template <bool UNIT_K>
__device__ __forceinline__ void store_tile(const TileRegs& r, float* s, int tid) {   // s: [16][kPitch]
  if (UNIT_K) {
    const int row = tid >> 1, k = 8 * (tid & 1);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) s[(k + 4 * i + j) * kPitch + row] = r.v[i][j];
  } else {
    const int k = tid >> 4, row = 8 * (tid & 15);
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<f32x4_t*>(&s[k * kPitch + row + 4 * i]) = r.v[i];
  }
}

// EPI 0: plain, 1: relu, 2: zero where mask[e,r,n] <= 0
template <int EPI, bool A_UNIT_K, bool B_UNIT_K>
__global__ __launch_bounds__(256) void gemm_f32_mfma_kernel(
    const float* __restrict__ A, long long a_e, long long a_r, long long a_k,
    const float* __restrict__ B, long long b_e, long long b_k, long long b_n,
    float* __restrict__ Cout, const float* __restrict__ mask, int R, int N, int K, int tiles_r,
    int tiles_n) {
  __shared__ __attribute__((aligned(16))) float As[2][kBK * kPitch];
  __shared__ __attribute__((aligned(16))) float Bs[2][kBK * kPitch];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // Consecutive workgroups go to different XCDs (8, each with its own L2).  Give every XCD a
  // contiguous range of tiles, row tiles fastest, so that the tiles that share a panel of B
  // run next to each other under one L2.
  unsigned t = blockIdx.x;
  const unsigned per_xcd = gridDim.x / 8;
  if (t < per_xcd * 8) t = (t % 8) * per_xcd + t / 8;
  const unsigned per_e = (unsigned)tiles_r * tiles_n;
  const int e = t / per_e;
  t -= e * per_e;
  const int r0 = (int)(t % tiles_r) * kT, n0 = (int)(t / tiles_r) * kT;
  const float* Ae = A + (size_t)e * a_e;
  const float* Be = B + (size_t)e * b_e;
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
  const int l32 = lane & 31, hf = lane >> 5;

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  TileRegs ra, rb;
  load_tile<A_UNIT_K>(ra, Ae, a_r, a_k, r0, 0, R, K, tid);
  load_tile<B_UNIT_K>(rb, Be, b_n, b_k, n0, 0, N, K, tid);
  store_tile<A_UNIT_K>(ra, As[0], tid);
  store_tile<B_UNIT_K>(rb, Bs[0], tid);
  __syncthreads();
  const int steps = (K + kBK - 1) / kBK;
  for (int s = 0; s < steps; ++s) {
    const int cur = s & 1;
    if (s + 1 < steps) {
      load_tile<A_UNIT_K>(ra, Ae, a_r, a_k, r0, (s + 1) * kBK, R, K, tid);
      load_tile<B_UNIT_K>(rb, Be, b_n, b_k, n0, (s + 1) * kBK, N, K, tid);
    }
#pragma unroll
    for (int kk = 0; kk < kBK / 2; ++kk) {
      float a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = As[cur][(2 * kk + hf) * kPitch + wm0 + 32 * i + l32];
        b[i] = Bs[cur][(2 * kk + hf) * kPitch + wn0 + 32 * i + l32];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (s + 1 < steps) {
      store_tile<A_UNIT_K>(ra, As[cur ^ 1], tid);        // last read two barriers ago
      store_tile<B_UNIT_K>(rb, Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }
  // acc[i][j][v]: row 32 i + 8 (v/4) + 4 hf + v%4, column 32 j + lane%32 of the wavefront tile
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = r0 + wm0 + 32 * i + 8 * (v >> 2) + 4 * hf + (v & 3);
        const int n = n0 + wn0 + 32 * j + l32;
        if (r >= R || n >= N) continue;
        const size_t o = ((size_t)e * R + r) * N + n;
        float x = acc[i][j][v];
        if (EPI == 1) x = fmaxf(x, 0.f);
        if (EPI == 2) x = mask[o] > 0.f ? x : 0.f;
        Cout[o] = x;
      }
}

template <bool A_UNIT_K, bool B_UNIT_K>
int launch_layout(int epi, const float* A, long long a_e, long long a_r, long long a_k,
                  const float* B, long long b_e, long long b_k, long long b_n, float* Cout,
                  const float* mask, int E, int R, int N, int K, hipStream_t st) {
  const int tiles_r = (R + kT - 1) / kT, tiles_n = (N + kT - 1) / kT;
  const dim3 grid((unsigned)((long long)E * tiles_r * tiles_n));
#define MOE_F32_CASE(EP)                                                                       \
  hipLaunchKernelGGL((gemm_f32_mfma_kernel<EP, A_UNIT_K, B_UNIT_K>), grid, dim3(256), 0, st, A, \
                     a_e, a_r, a_k, B, b_e, b_k, b_n, Cout, mask, R, N, K, tiles_r, tiles_n)
  if (epi == 0) MOE_F32_CASE(0);
  else if (epi == 1) MOE_F32_CASE(1);
  else MOE_F32_CASE(2);
#undef MOE_F32_CASE
  return check_launch();
}

}  // namespace

// true when the fp32 MFMA kernel takes these strides and sizes
bool gemm_f32_mfma_ok(long long a_r, long long a_k, long long b_k, long long b_n, int E, int R, int N,
                      int K) {
  if (E < 1 || R < 1 || N < 1 || K < 1) return false;
  if ((long long)E * ((R + kT - 1) / kT) * ((N + kT - 1) / kT) > 0x7fffffffLL) return false;
  const bool a_unit_k = a_k == 1, b_unit_k = b_k == 1;
  if (!a_unit_k && a_r != 1) return false;
  if (!b_unit_k && b_n != 1) return false;
  // 16-byte loads: the dimension along the unit stride and the other stride are multiples of 4
  if (a_unit_k ? (K % 4 != 0 || a_r % 4 != 0) : (R % 4 != 0 || a_k % 4 != 0)) return false;
  if (b_unit_k ? (K % 4 != 0 || b_n % 4 != 0) : (N % 4 != 0 || b_k % 4 != 0)) return false;
  return true;
}

int launch_gemm_f32_mfma(int epi, const float* A, long long a_e, long long a_r, long long a_k,
                         const float* B, long long b_e, long long b_k, long long b_n, float* Cout,
                         const float* mask, int E, int R, int N, int K, hipStream_t st) {
  if (!gemm_f32_mfma_ok(a_r, a_k, b_k, b_n, E, R, N, K) || a_e % 4 != 0 || b_e % 4 != 0)
    return MOE_EUNSUPPORTED;
  const bool ak = a_k == 1, bk = b_k == 1;
  if (ak && bk) return launch_layout<true, true>(epi, A, a_e, a_r, a_k, B, b_e, b_k, b_n, Cout, mask, E, R, N, K, st);
  if (ak) return launch_layout<true, false>(epi, A, a_e, a_r, a_k, B, b_e, b_k, b_n, Cout, mask, E, R, N, K, st);
  if (bk) return launch_layout<false, true>(epi, A, a_e, a_r, a_k, B, b_e, b_k, b_n, Cout, mask, E, R, N, K, st);
  return launch_layout<false, false>(epi, A, a_e, a_r, a_k, B, b_e, b_k, b_n, Cout, mask, E, R, N, K, st);
}

}  // namespace moe
