// Expert networks (Eq. 2 of the paper; Algorithm 2: EGCM,EMH->EGCH, relu,
// EGCH,EHM->EGCM) as two grouped GEMMs over the experts:
//
//   h[e]   = relu(buf[e] . wi[e])     [R, M] x [M, H],  R = G*C rows per expert
//   out[e] = h[e] . wo[e]             [R, H] x [H, M]
//
// bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulation.  A tiles (row-major,
// K contiguous) sit in LDS as [m][k] and are read with 16-byte loads; the weight
// tiles are [k][n] in memory (N contiguous), stay that way in LDS and are read
// with ds_read_b64_tr_b16, which hands every lane the 4 consecutive k of its
// column that the MFMA B operand wants.  Global -> register -> LDS double
// buffering, one barrier per K step.  Blocks are renumbered so that each XCD
// (own L2) walks a contiguous range of tiles with the row tile varying fastest:
// neighbours share one weight panel.
//
// fp32 path: plain LDS-tiled FMA kernel (small reference-precision configs).
#include "common.h"

namespace moe {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;

__device__ __forceinline__ int xcd_remap(int bid, int nblk) {
  const int q = nblk / kXcds, r = nblk % kXcds;
  const int xcd = bid % kXcds, idx = bid / kXcds;
  return xcd * q + (xcd < r ? xcd : r) + idx;
}

template <int BM, int BN, int BK>
struct GemmSmem {
  static constexpr int kAPitch = BK + 8;    // bf16 elements; 16 B pad: conflict-free b128 reads
  static constexpr int kBPitch = BN + 16;   // 32 B pad: 4 consecutive k rows hit distinct banks
  static constexpr int kAElems = BM * kAPitch;
  static constexpr int kBElems = BK * kBPitch;
  static constexpr size_t kBytes = (size_t)2 * (kAElems + kBElems) * sizeof(bf16_t);
};

template <int BM, int BN, int BK, int WM, int WN, bool RELU>
__global__ __launch_bounds__(256) void expert_gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, bf16_t* __restrict__ Cout,
    int R, int N, int K, int tiles_m, int tiles_n, int nblk) {
  using SM = GemmSmem<BM, BN, BK>;
  constexpr int WTM = BM / WM, WTN = BN / WN;      // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;      // 32x32 MFMA tiles per wave
  constexpr int AV = BM * BK / 8 / 256;            // 16-byte vectors per thread
  constexpr int BV = BK * BN / 8 / 256;
  static_assert(WM * WN == 4, "four wavefronts per block");
  static_assert(AV >= 1 && BV >= 1, "tile too small for 256 threads");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);            // [2][BM][kAPitch]
  bf16_t* Bs = As + 2 * SM::kAElems;                           // [2][BK][kBPitch]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int logical = xcd_remap(blockIdx.x, nblk);
  const int per_e = tiles_m * tiles_n;
  const int e = logical / per_e;
  const int t = logical - e * per_e;
  const int m0 = (t % tiles_m) * BM, n0 = (t / tiles_m) * BN;
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  const bf16_t* Ae = A + (size_t)e * R * K;
  const bf16_t* Be = B + (size_t)e * K * N;
  bf16_t* Ce = Cout + (size_t)e * R * N;

  uint4 areg[AV], breg[BV];
  bf16_t* const as_w = As + (tid / (BK / 8)) * SM::kAPitch + (tid % (BK / 8)) * 8;
  bf16_t* const bs_w = Bs + (tid / (BN / 8)) * SM::kBPitch + (tid % (BN / 8)) * 8;

#define MOE_LOAD_TILES(k0)                                                                   \
  {                                                                                          \
    _Pragma("unroll") for (int i = 0; i < AV; ++i) {                                         \
      int gr = m0 + i * (256 / (BK / 8)) + tid / (BK / 8);                                   \
      gr = gr < R ? gr : R - 1; /* clamp: extra rows are never stored */                     \
      const int gk = (k0) + (tid % (BK / 8)) * 8;                                            \
      areg[i] = gk < K ? *reinterpret_cast<const uint4*>(Ae + (size_t)gr * K + gk)           \
                       : uint4{0u, 0u, 0u, 0u};                                              \
    }                                                                                        \
    _Pragma("unroll") for (int i = 0; i < BV; ++i) {                                         \
      const int gk = (k0) + i * (256 / (BN / 8)) + tid / (BN / 8);                           \
      const int gn = n0 + (tid % (BN / 8)) * 8;                                              \
      breg[i] = (gk < K && gn < N) ? *reinterpret_cast<const uint4*>(Be + (size_t)gk * N + gn) \
                                   : uint4{0u, 0u, 0u, 0u};                                  \
    }                                                                                        \
  }
#define MOE_STORE_TILES(buf)                                                                 \
  {                                                                                          \
    _Pragma("unroll") for (int i = 0; i < AV; ++i)                                           \
      *reinterpret_cast<uint4*>(as_w + (buf) * SM::kAElems +                                 \
                                i * (256 / (BK / 8)) * SM::kAPitch) = areg[i];               \
    _Pragma("unroll") for (int i = 0; i < BV; ++i)                                           \
      *reinterpret_cast<uint4*>(bs_w + (buf) * SM::kBElems +                                 \
                                i * (256 / (BN / 8)) * SM::kBPitch) = breg[i];               \
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // per-lane LDS offsets (elements)
  const int a_off = (wm0 + (lane & 31)) * SM::kAPitch + 8 * (lane >> 5);
  const int b_off = (8 * (lane >> 5) + ((lane & 15) >> 2)) * SM::kBPitch + wn0 +
                    16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  const int KT = (K + BK - 1) / BK;
  MOE_LOAD_TILES(0)
  MOE_STORE_TILES(0)
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) MOE_LOAD_TILES((kt + 1) * BK)
    const bf16_t* as = As + cur * SM::kAElems + a_off;
    const bf16_t* bs = Bs + cur * SM::kBElems + b_off;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8_t af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8_t*>(as + i * 32 * SM::kAPitch + kk * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
        const bf16_t* p = bs + kk * 16 * SM::kBPitch + j * 32;
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * SM::kBPitch));
        bfr[j] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) MOE_STORE_TILES(cur ^ 1)
    __syncthreads();
  }

  // epilogue: acc[i][j][r] is C[row][col] with
  //   row = 32 i + 8 (r/4) + 4 (lane/32) + r%4,  col = 32 j + lane%32
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn0 + 32 * j + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        float v = acc[i][j][r];
        if (RELU) v = fmaxf(v, 0.f);
        if (row < R && col < N) Ce[(size_t)row * N + col] = f32_to_bf16(v);
      }
    }
#undef MOE_LOAD_TILES
#undef MOE_STORE_TILES
}

template <int BM, int BN, int BK, int WM, int WN, bool RELU>
int launch_bf16(const bf16_t* A, const bf16_t* B, bf16_t* Cout, int E, int R, int N, int K,
                hipStream_t st) {
  using SM = GemmSmem<BM, BN, BK>;
  auto kern = expert_gemm_bf16_kernel<BM, BN, BK, WM, WN, RELU>;
  static bool attr_set = false;   // idempotent: a repeated call sets the same value
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)SM::kBytes) != hipSuccess)
      return MOE_EHIP;
    attr_set = true;
  }
  const int tiles_m = (R + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const long long nblk = (long long)E * tiles_m * tiles_n;
  if (nblk > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), SM::kBytes, st, A, B, Cout, R, N, K,
                     tiles_m, tiles_n, (int)nblk);
  return check_launch();
}

template <bool RELU>
int gemm_bf16(const bf16_t* A, const bf16_t* B, bf16_t* Cout, int E, int R, int N, int K,
              hipStream_t st) {
  if (R > 128 && N >= 256) return launch_bf16<256, 256, 64, 2, 2, RELU>(A, B, Cout, E, R, N, K, st);
  return launch_bf16<128, 128, 64, 2, 2, RELU>(A, B, Cout, E, R, N, K, st);
}

// ---------------------------------------------------------------- fp32 path
template <bool RELU>
__global__ __launch_bounds__(256) void expert_gemm_f32_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ Cout,
    int R, int N, int K, int tiles_m, int tiles_n) {
  constexpr int T = 64, BK = 16;
  __shared__ float As[BK][T + 1];
  __shared__ float Bs[BK][T + 1];
  const int per_e = tiles_m * tiles_n;
  const int e = blockIdx.x / per_e, t = blockIdx.x % per_e;
  const int m0 = (t % tiles_m) * T, n0 = (t / tiles_m) * T;
  const float* Ae = A + (size_t)e * R * K;
  const float* Be = B + (size_t)e * K * N;
  float* Ce = Cout + (size_t)e * R * N;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = threadIdx.x; i < T * BK; i += 256) {
      const int r = i / BK, k = i % BK;
      As[k][r] = (m0 + r < R && k0 + k < K) ? Ae[(size_t)(m0 + r) * K + k0 + k] : 0.f;
      const int kb = i / T, c = i % T;
      Bs[kb][c] = (k0 + kb < K && n0 + c < N) ? Be[(size_t)(k0 + kb) * N + n0 + c] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
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
      const int r = m0 + ty * 4 + i, c = n0 + tx * 4 + j;
      if (r < R && c < N) Ce[(size_t)r * N + c] = RELU ? fmaxf(acc[i][j], 0.f) : acc[i][j];
    }
}

template <bool RELU>
int gemm_f32(const float* A, const float* B, float* Cout, int E, int R, int N, int K,
             hipStream_t st) {
  const int tiles_m = (R + 63) / 64, tiles_n = (N + 63) / 64;
  const long long nblk = (long long)E * tiles_m * tiles_n;
  if (nblk > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  hipLaunchKernelGGL(expert_gemm_f32_kernel<RELU>, dim3((unsigned)nblk), dim3(256), 0, st, A, B,
                     Cout, R, N, K, tiles_m, tiles_n);
  return check_launch();
}

}  // namespace

static int rows_per_expert(const moe_config& c, int* R) {
  const long long rows = (long long)c.G * c.C;
  if (rows > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  *R = (int)rows;
  return MOE_OK;
}

int launch_expert_gemm1(const moe_config& c, const void* buf, const void* wi, void* h,
                        hipStream_t st) {
  int R;
  const int rc = rows_per_expert(c, &R);
  if (rc != MOE_OK) return rc;
  if (c.act_dtype == MOE_F32)
    return gemm_f32<true>(static_cast<const float*>(buf), static_cast<const float*>(wi),
                          static_cast<float*>(h), c.E, R, c.H, c.M, st);
  return gemm_bf16<true>(static_cast<const bf16_t*>(buf), static_cast<const bf16_t*>(wi),
                         static_cast<bf16_t*>(h), c.E, R, c.H, c.M, st);
}

int launch_expert_gemm2(const moe_config& c, const void* h, const void* wo, void* out,
                        hipStream_t st) {
  int R;
  const int rc = rows_per_expert(c, &R);
  if (rc != MOE_OK) return rc;
  if (c.act_dtype == MOE_F32)
    return gemm_f32<false>(static_cast<const float*>(h), static_cast<const float*>(wo),
                           static_cast<float*>(out), c.E, R, c.M, c.H, st);
  return gemm_bf16<false>(static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(wo),
                          static_cast<bf16_t*>(out), c.E, R, c.M, c.H, st);
}

}  // namespace moe
