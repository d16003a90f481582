// Expert networks (Eq. 2 of the paper; Algorithm 2: EGCM,EMH->EGCH, relu,
// EGCH,EHM->EGCM) as two grouped GEMMs over the experts, and the four GEMMs of
// their backward pass:
//
//   h[e]   = relu(buf[e] . wi[e])     [R, M] x [M, H],  R = G*C rows per expert
//   out[e] = h[e] . wo[e]             [R, H] x [H, M]
//
// bf16, v_mfma_f32_32x32x16_bf16 with fp32 accumulation, in two kernels:
//
//   expert_gemm_bf16_dma_kernel   shapes made of whole 256x256 tiles with K % 32 == 0
//     (every benchmarked layer): persistent, one block per CU walks its share of the
//     tiles as one stream of K steps; operands travel global -> LDS without passing
//     the registers; either operand in either layout; gathered rows, packed rows,
//     scattered result rows and a per-expert k range as template options.
//   expert_gemm_bf16_kernel       every other shape: one block per tile, operands
//     staged global -> registers -> LDS (double buffered, one barrier per K step),
//     clamped addresses and select masks at the ragged edges.
//
// In both, activation tiles (K contiguous) sit in LDS as [m][k] and are read with
// 16-byte loads; weight tiles are [k][n] in memory (N contiguous), stay that way in
// LDS and are read with ds_read_b64_tr_b16, which hands every lane the 4 consecutive
// k of its column that the MFMA operand wants.  Blocks of one XCD (own L2) take
// neighbouring tiles so that they share operand panels.
//
// fp32 layers run the fp32 MFMA kernel of gemm_f32.hip.
#include "common.h"

namespace moe {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // native 16-byte vector
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kXcds = 8;

__device__ __forceinline__ int xcd_remap(int bid, int nblk) {
  const int q = nblk / kXcds, r = nblk % kXcds;
  const int xcd = bid % kXcds, idx = bid / kXcds;
  return xcd * q + (xcd < r ? xcd : r) + idx;
}

// LDS staging of one operand tile of ROWS output rows (or columns) x BK.  "K-contiguous"
// (KC): the operand is stored [rows][K]; staged as [ROWS][BK + 8] (16 B pad: conflict-free
// 16-byte reads).  "row-of-k" (MNC): stored [K][rows]; staged as [BK][ROWS + 16] (32 B pad:
// 4 consecutive k rows hit distinct banks) and read with the transposing LDS load.
template <int ROWS, int BK, bool MNC>
struct OperandSmem {
  static constexpr int kPitch = MNC ? ROWS + 16 : BK + 8;
  static constexpr int kElems = MNC ? BK * kPitch : ROWS * kPitch;
  static constexpr int kVecs = ROWS * BK / 8 / 256;             // 16-byte vectors per thread
  static constexpr int kVecsPerLine = MNC ? ROWS / 8 : BK / 8;  // along the contiguous dimension
  static constexpr int kLinesPerPass = 256 / kVecsPerLine;
};

template <int BM, int BN, int BK, bool A_MNC, bool B_KC>
struct GemmSmem {
  using SA = OperandSmem<BM, BK, A_MNC>;
  using SB = OperandSmem<BN, BK, !B_KC>;
  static constexpr size_t kBytes = (size_t)2 * (SA::kElems + SB::kElems) * sizeof(bf16_t);
};

// One block per 256x256 or 128x128 tile of C, any shape (clamped addresses and select masks at
// the ragged edges; EXACT drops them), either operand in either layout (the same three products
// as the persistent kernel below):
//   C = A . B      A KC [R,K], B MNC [K,N]      C = A . B^T    A KC, B KC [N,K]
//   C = A^T . B    A MNC [K,R], B MNC [K,N]
// EPI: 0 plain, 1 relu, 2 zero every element whose `mask` element (same index as C) is <= 0.
// Contiguous dimensions are multiples of 8 elements (16-byte loads are whole or masked whole).
template <int BM, int BN, int BK, int WM, int WN, int EPI, bool A_MNC, bool B_KC, bool EXACT>
__global__ __launch_bounds__(256) void expert_gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, bf16_t* __restrict__ Cout,
    const bf16_t* __restrict__ mask, int R, int N, int K, int tiles_m, int tiles_n, int nblk) {
  using SM = GemmSmem<BM, BN, BK, A_MNC, B_KC>;
  using SA = typename SM::SA;
  using SB = typename SM::SB;
  constexpr int WTM = BM / WM, WTN = BN / WN;      // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;      // 32x32 MFMA tiles per wave
  static_assert(WM * WN == 4, "four wavefronts per block");
  static_assert(SA::kVecs >= 1 && SB::kVecs >= 1, "tile too small for 256 threads");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);            // two stages
  bf16_t* Bs = As + 2 * SA::kElems;                            // two stages

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int logical = xcd_remap(blockIdx.x, nblk);
  const int per_e = tiles_m * tiles_n;
  const int e = logical / per_e;
  const int t = logical - e * per_e;
  const int m0 = (t % tiles_m) * BM, n0 = (t / tiles_m) * BN;
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  const bf16_t* Ae = A + (size_t)e * R * K;
  const bf16_t* Be = B + (size_t)e * K * N;
  const size_t c_e = (size_t)e * R * N;

  // One 16-byte vector of an operand tile: `line` counts rows of the operand's memory layout
  // (output rows / columns for KC, k for MNC), `vec` the position along the contiguous
  // dimension.  Out-of-range pieces are read from a clamped address and replaced by zeros;
  // surplus output rows of a KC operand are clamped only (their results are never stored).
  typedef u32x4_t vec_t;
#define MOE_LOAD_OPERAND(REGS, SX, MNC, BASE, EXTENT, ORIGIN, k0)                              \
  _Pragma("unroll") for (int i = 0; i < SX::kVecs; ++i) {                                    \
    const int line_ = tid / SX::kVecsPerLine + i * SX::kLinesPerPass;                        \
    const int vec_ = (tid % SX::kVecsPerLine) * 8;                                           \
    if (MNC) {                                                                               \
      int gk = (k0) + line_, gx = (ORIGIN) + vec_;                                           \
      const bool ok = EXACT || (gk < K && gx < (EXTENT));                                    \
      if (!EXACT) { gk = gk < K ? gk : K - 1; gx = gx < (EXTENT) ? gx : (EXTENT) - 8; }     \
      const vec_t v = *reinterpret_cast<const vec_t*>((BASE) + (size_t)gk * (EXTENT) + gx);  \
      REGS[i] = ok ? v : vec_t{0u, 0u, 0u, 0u};                                              \
    } else {                                                                                 \
      int gx = (ORIGIN) + line_, gk = (k0) + vec_;                                           \
      const bool ok = EXACT || gk < K;                                                       \
      if (!EXACT) { gx = gx < (EXTENT) ? gx : (EXTENT) - 1; gk = gk < K ? gk : K - 8; }     \
      const vec_t v = *reinterpret_cast<const vec_t*>((BASE) + (size_t)gx * K + gk);         \
      REGS[i] = ok ? v : vec_t{0u, 0u, 0u, 0u};                                              \
    }                                                                                        \
  }
#define MOE_STORE_OPERAND(REGS, SX, XS, buf)                                                    \
  _Pragma("unroll") for (int i = 0; i < SX::kVecs; ++i) {                                    \
    const int line_ = tid / SX::kVecsPerLine + i * SX::kLinesPerPass;                        \
    const int vec_ = (tid % SX::kVecsPerLine) * 8;                                           \
    *reinterpret_cast<vec_t*>(XS + (buf) * SX::kElems + line_ * SX::kPitch + vec_) = REGS[i]; \
  }
  vec_t areg[SA::kVecs], breg[SB::kVecs];          // staging registers of the tile in flight
#define MOE_LOAD_TILES(k0)                                                                   \
  MOE_LOAD_OPERAND(areg, SA, A_MNC, Ae, R, m0, k0)                                           \
  MOE_LOAD_OPERAND(breg, SB, !B_KC, Be, N, n0, k0)
#define MOE_STORE_TILES(buf)                                                                 \
  MOE_STORE_OPERAND(areg, SA, As, buf)                                                       \
  MOE_STORE_OPERAND(breg, SB, Bs, buf)

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // MFMA operands of one 16-wide k step: each lane gets the 8 consecutive k of one output row
  // (A) / column (B).  KC: one 16-byte read; MNC: two transposing 8-byte reads.
  typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
  const int kc_off_a = (wm0 + (lane & 31)) * SA::kPitch + 8 * (lane >> 5);
  const int kc_off_b = (wn0 + (lane & 31)) * SB::kPitch + 8 * (lane >> 5);
  const int mnc_line = 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int mnc_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  struct Frags { bf16x8_t a[TM]; bf16x8_t b[TN]; };
#define MOE_READ_OPERAND(DST, CNT, SX, MNC, XS, KC_OFF, W0, buf, kk)                           \
  _Pragma("unroll") for (int i = 0; i < CNT; ++i) {                                          \
    if (MNC) {                                                                               \
      const bf16_t* p_ = XS + (buf) * SX::kElems + ((kk) * 16 + mnc_line) * SX::kPitch + (W0) + mnc_col + i * 32; \
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p_);         \
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p_ + 4 * SX::kPitch)); \
      DST[i] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7)); \
    } else {                                                                                 \
      DST[i] = *reinterpret_cast<const bf16x8_t*>(XS + (buf) * SX::kElems + (KC_OFF) + (kk) * 16 + i * 32 * SX::kPitch); \
    }                                                                                        \
  }
#define MOE_READ_FRAGS(F, buf, kk)                                                           \
  MOE_READ_OPERAND((F).a, TM, SA, A_MNC, As, kc_off_a, wm0, buf, kk)                         \
  MOE_READ_OPERAND((F).b, TN, SB, !B_KC, Bs, kc_off_b, wn0, buf, kk)
  // The B fragment goes in as the first MFMA operand: the 32x32 result is then
  // the transposed tile, i.e. a lane owns 4 consecutive columns of one row of C.
#define MOE_MFMA_STEP(F)                                                                     \
  _Pragma("unroll") for (int i = 0; i < TM; ++i)                                             \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                           \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16((F).b[j], (F).a[i], acc[i][j], 0, 0, 0);

  const int KT = (K + BK - 1) / BK;
  constexpr int KK = BK / 16;
  Frags fr[2];
  // Pipeline: tile kt is consumed from LDS stage kt&1 while tile kt+1 travels
  // through the staging registers (loaded right after the barrier, written to the
  // other LDS stage during the last k step).
  MOE_LOAD_TILES(0)
  MOE_STORE_TILES(0)
  __syncthreads();
  if (KT > 1) { MOE_LOAD_TILES(BK) }
  MOE_READ_FRAGS(fr[0], 0, 0)
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + 1 < KK) { MOE_READ_FRAGS(fr[(kk + 1) & 1], cur, kk + 1) }
      if (kk + 1 == KK && kt + 1 < KT) { MOE_STORE_TILES(cur ^ 1) }
      MOE_MFMA_STEP(fr[kk & 1])
    }
    __syncthreads();
    if (kt + 2 < KT) { MOE_LOAD_TILES((kt + 2) * BK) }
    if (kt + 1 < KT) { MOE_READ_FRAGS(fr[0], cur ^ 1, 0) }
  }

  // epilogue: acc[i][j][r] = C[row][col .. col+3 for r%4 = 0..3] with
  //   row = 32 i + lane%32,  col = 32 j + 8 (r/4) + 4 (lane/32)
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wm0 + 32 * i + (lane & 31);
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = n0 + wn0 + 32 * j + 8 * q + 4 * (lane >> 5);
        if (!(EXACT || (row < R && col < N))) continue;   // N % 8 == 0: the 4 columns are in or out together
        const size_t o = c_e + (size_t)row * N + col;
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v[r] = acc[i][j][4 * q + r];
          if (EPI == 1) v[r] = fmaxf(v[r], 0.f);
        }
        if (EPI == 2) {
          const uint2 mk = *reinterpret_cast<const uint2*>(mask + o);
          // a bf16 is positive iff its bits, read as a 16-bit integer, are positive
          if ((int16_t)(mk.x & 0xffffu) <= 0) v[0] = 0.f;
          if ((int16_t)(mk.x >> 16) <= 0) v[1] = 0.f;
          if ((int16_t)(mk.y & 0xffffu) <= 0) v[2] = 0.f;
          if ((int16_t)(mk.y >> 16) <= 0) v[3] = 0.f;
        }
        *reinterpret_cast<uint2*>(Cout + o) = uint2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
      }
  }
#undef MOE_READ_OPERAND
#undef MOE_READ_FRAGS
#undef MOE_MFMA_STEP
#undef MOE_LOAD_OPERAND
#undef MOE_STORE_OPERAND
#undef MOE_LOAD_TILES
#undef MOE_STORE_TILES
}

// ----------------------------------------------------------------------------
// Exact 256x256 tiles: a persistent kernel (one block per CU) that walks its share
// of the tiles as ONE stream of 32-wide K steps.
//
// Global -> LDS copies bypass the registers (global_load_lds_dwordx4), ST stages of
// 32 KB, the copy of step g+ST-1 is started during step g, also across a tile
// boundary: the next tile's first stages land while the current tile is finished
// and stored, so neither the fill of the pipeline nor the drain of the stores is
// paid per tile.
//
// One wavefront copy instruction fills 1 KB of LDS (lane l -> bytes 16 l ..), which
// fixes the LDS layout to unpadded rows; bank conflicts are avoided by permuting
// which 16-byte chunk of a row a lane fetches:
//   A stage [256 rows][4 chunks of 8 k]:  chunk c of row r sits at position c ^ ((r>>2)&3)
//   B stage [32 k][32 chunks of 8 n]:     chunk c of row k sits at position c ^ (4 (k&3))
// (64 banks of 4 bytes: a 16-lane group of a 16-byte read, or a 32-lane group of an
// 8-byte transposing read, then touches every bank exactly once)
//
// Step g: fetch the fragments of the second k half, multiply the first half; wait
// for the own copies of step g+1 and barrier (step g+1 is now visible to all, the
// stage of step g-1 is free); then, spread between the four MFMA rows of the second
// half, start the copies of step g+ST-1 and fetch the first fragments of step g+1.
// ----------------------------------------------------------------------------
template <int ST>
struct DmaSmem {
  static constexpr int kAStage = 256 * 32 * 2, kBStage = 32 * 256 * 2;
  static constexpr int kStage = kAStage + kBStage;
  static constexpr size_t kBytes = (size_t)ST * kStage;
};

#define MOE_DMA16(LDS_U32, VOFF_U32, SBASE)                                         \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"     \
               :: "s"(LDS_U32), "v"(VOFF_U32), "s"(SBASE) : "memory")

// GATHER: the A rows are not a dense [E,R,K] buffer but rows of x picked by the dispatch
// indices (A = x [G,S,K]; row r of expert e is x[r / C, src_token[e,r], :], a zero row when
// the slot is empty), i.e. the dispatch of Algorithm 2 folded into the first GEMM's copies.
//
// Operand layouts.  "K-contiguous" (KC): the operand is stored [rows][K] (row = its index in
// the output) and staged as [256 rows][4 chunks]; "row-of-k" (MNC): stored [K][rows] and
// staged as [32 k][32 chunks], read with the transposing LDS load.  Either operand can have
// either layout; both fragment kinds hand a lane the 8 consecutive k of its row:
//   forward       C = A . B        A KC  [R,K],  B MNC [K,N]
//   data gradient C = A . B^T      A KC  [R,K],  B KC  [N,K]      (A_MNC = false, B_KC = true)
//   weight grad.  C = A^T . B      A MNC [K,R],  B MNC [K,N]      (A_MNC = true,  B_KC = false)
// EPI: 0 plain, 1 relu, 2 zero every element whose `mask` element (same [E,R,N] index as C)
// is zero -- the derivative of relu taken from the stored activations, 3 plain with an fp32
// result (Cout points to floats), 4 relu that also records which results are non-zero, one
// bit per element in `signbits`, 5 zero every element whose recorded bit is clear.
// The bit record is private to this kernel: 8 KB per 256x256 tile (tile index
// (e * tiles_m + row tile) * tiles_n + column tile), inside a tile 2 KB per wavefront laid
// out as [2][64 lanes][16 bytes] = the 32 bytes a lane meets in its own store phase (4 row
// groups x 8 stores, one byte each: bit b = column 8 c + b of that store).  Writer and reader
// are the same tiling of the same [E,R,N] matrix, so no lane ever needs another lane's bits.
// The reader fetches a tile's 8 KB into spare LDS with two register-bypassing copies issued
// in the tile's first K step; the waits of the next two steps cover them.
// GATHER 2: the indices are absolute rows of the matrix A ([rows, K], row p of expert e comes
// from row src_token[e * R + p], -1 = zero row): the packed row layout (RowPacking).
// PACKED: expert e has only its first ceil(kept[e] / 256) row tiles multiplied (kept[e] = its
// occupied rows): every block copies kept to LDS and forms the running tile counts there when it
// starts; the tiles of all experts are numbered consecutively in expert order, and since a
// block's tile numbers only grow it finds a tile's expert by stepping a cursor forward.  Rows
// from kept[e] to the end of the last tile are multiplied as zero rows.  SCATTER (with PACKED):
// the rows of C go to the absolute rows src_token[e * R + p] of Cout ([rows, N]), -1 = not stored.
// DYNK: the sum over k of expert e stops at 256 ceil(kept[e] / 256) instead of K (the weight
// gradients, whose k runs over an expert's packed rows); an expert with no rows gets zeros.
template <int ST, int EPI, int GATHER, bool A_MNC, bool B_KC, bool PACKED, bool SCATTER, bool DYNK>
__global__ __launch_bounds__(256) void expert_gemm_bf16_dma_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, bf16_t* __restrict__ Cout,
    int R, int N, int K, int tiles_m, int tiles_n, int ntiles_static,
    const int32_t* __restrict__ src_token, const bf16_t* __restrict__ zero_row, int S,
    uint32_t c_magic, int c_shift, const bf16_t* __restrict__ mask,
    unsigned char* __restrict__ signbits, const int32_t* __restrict__ kept, int E) {
  static_assert(!(GATHER && A_MNC), "the gather form addresses whole rows of a K-contiguous A");
  static_assert(!SCATTER || (PACKED && EPI == 0), "scattered rows: plain bf16 result of a packed launch");
  static_assert(!(DYNK && (PACKED || GATHER)), "a shortened k range comes with the full list of output tiles");
  constexpr bool RELU = EPI == 1 || EPI == 4;
  using SM = DmaSmem<ST>;
  constexpr int BM = 256, BN = 256, BK = 32, TM = 4, TN = 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  typedef unsigned char __attribute__((address_space(3))) * lds_ptr;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_ptr)smem_raw);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 128;
  const int per_e = tiles_m * tiles_n;
  const int KT = K / BK;
  // Tile t of an expert -> (row tile, column tile): bands of kBand row tiles, inside a band
  // row tile fastest, then column tile.  The ~32 tiles an XCD works on at a time then span
  // about 8 row tiles x 4 column tiles, the split that shares the most operand panels in that
  // XCD's L2 (a tall output, as in the weight gradients, would otherwise re-read its A panel
  // once per column tile).
  constexpr int kBand = 8;   // bands of 2 or 4 row tiles measured the same on the forward shapes
  // PACKED: kept_s[e] = occupied rows of expert e, rts_s[e] = occupied row tiles of the experts
  // before e (rts_s[E] = all of them), behind the stages and the token / bit areas in LDS
  int* const kept_s = reinterpret_cast<int*>(smem_raw + SM::kBytes + (GATHER ? 1024 : 0) + (EPI == 5 ? 8192 : 0));
  int* const rts_s = kept_s + E;
  if (PACKED || DYNK) {
    for (int e = tid; e < E; e += 256) kept_s[e] = kept[e];
    __syncthreads();
  }
  if (PACKED) {
    if (wave == 0) {
      // lane l scans experts [l per, (l+1) per); the lanes' sums meet in a wavefront scan
      const int per = (E + 63) / 64, b0 = lane * per;
      int sum = 0;
      for (int j = 0; j < per; ++j)
        if (b0 + j < E) sum += (kept_s[b0 + j] + 255) >> 8;
      int incl = sum;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      int run = incl - sum;
      for (int j = 0; j < per; ++j)
        if (b0 + j < E) {
          rts_s[b0 + j] = run;
          run += (kept_s[b0 + j] + 255) >> 8;
        }
      if (lane == 63) rts_s[E] = incl;
    }
    __syncthreads();
  }
  const int ntiles = PACKED ? __builtin_amdgcn_readfirstlane(rts_s[E]) * tiles_n : ntiles_static;
  // PACKED: expert of the tile located last and its range of row tiles [rs, re) in the global
  // numbering; one cursor for the copies (producer side), one for the epilogues
  struct TileCursor { int e, rs, re; };
  TileCursor pcur{-1, 0, 0}, ccur{-1, 0, 0};
#define MOE_DMA_TILE(T_, CUR_, e_, rt_, ct_)                                                 \
  int e_, rt_, ct_;                                                                          \
  {                                                                                          \
    int t_, tm_;                                                                             \
    if (PACKED) {                                                                            \
      /* ends at the latest with e = E - 1: T_ < ntiles = rts_s[E] * tiles_n */              \
      while ((T_) >= CUR_.re * tiles_n && CUR_.e + 1 < E) {                                  \
        ++CUR_.e;                                                                            \
        CUR_.rs = CUR_.re;                                                                   \
        CUR_.re = __builtin_amdgcn_readfirstlane(rts_s[CUR_.e + 1]);                         \
      }                                                                                      \
      e_ = CUR_.e;                                                                           \
      t_ = (T_) - CUR_.rs * tiles_n;                                                         \
      tm_ = CUR_.re - CUR_.rs;                                                               \
    } else {                                                                                 \
      e_ = (T_) / per_e;                                                                     \
      t_ = (T_) - e_ * per_e;                                                                \
      tm_ = tiles_m;                                                                         \
    }                                                                                        \
    const int band_ = t_ / (kBand * tiles_n), rem_ = t_ - band_ * kBand * tiles_n;           \
    const int left_ = tm_ - band_ * kBand, rows_ = left_ < kBand ? left_ : kBand;            \
    ct_ = rem_ / rows_;                                                                      \
    rt_ = band_ * kBand + (rem_ - ct_ * rows_);                                              \
  }

  // This block's tiles: XCD x = blockIdx % 8 owns a contiguous range of tiles; its
  // blocks take them round-robin, so at any time they work on neighbouring tiles
  // (row tile fastest: neighbours share a weight panel in that XCD's L2).
  const int nb = gridDim.x;
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int xq = ntiles / kXcds, xr = ntiles % kXcds;
  const int t_begin = xcd * xq + (xcd < xr ? xcd : xr);
  const int t_end = t_begin + xq + (xcd < xr ? 1 : 0);
  const int stride = (nb - xcd + kXcds - 1) / kXcds;           // blocks on this XCD
  const int first = t_begin + slot;
  if (first >= t_end) return;                                  // block-uniform
  // K steps of a tile of expert e_
#define MOE_DMA_STEPS(e_) (DYNK ? ((kept_s[e_] + 255) >> 8) * (256 / BK) : KT)

  // per-lane source byte offsets of the 4 + 4 copy instructions of this wavefront
  uint32_t a_voff[4], b_voff[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = 16 * (wave * 4 + q) + (lane >> 2);
    const int ca = (lane & 3) ^ ((row >> 2) & 3);
    const int krow = 2 * (wave * 4 + q) + (lane >> 5);
    const int cb = (lane & 31) ^ (4 * (krow & 3));
    a_voff[q] = A_MNC ? (uint32_t)((krow * R + 8 * cb) * 2) : (uint32_t)((row * K + 8 * ca) * 2);
    b_voff[q] = B_KC ? (uint32_t)((row * K + 8 * ca) * 2) : (uint32_t)((krow * N + 8 * cb) * 2);
  }

  // producer cursor: the next step to copy (tile p_tile, k step p_kt) and its sources
  // (p_steps: steps of that tile; p_more: such a step exists; p_g: steps started so far)
  int p_tile = first, p_kt = 0, p_stage = 0, p_g = 0, p_steps = KT, p_more = 1;
  const bf16_t* p_a;
  const bf16_t* p_b;
  // GATHER: per-lane source addresses of the 4 row copies.  The 64 dispatch indices of this
  // wavefront's rows of a tile are copied to LDS (one more register-bypassing copy, issued
  // 4 steps before the tile's first step, so the regular waits of the steps in between
  // cover it) and read from there when the producer moves on to that tile.
  uint64_t a_addr[4];
  const uint32_t lds_tok = lds0 + (uint32_t)SM::kBytes + wave * 256;
  const uint32_t lds_bits = lds0 + (uint32_t)SM::kBytes + wave * 2048;   // EPI 5 (never with GATHER)
  typedef int __attribute__((address_space(3))) * lds_int_ptr;
#define MOE_DMA_TOKENS(TILE)                                                                 \
  {                                                                                          \
    MOE_DMA_TILE(TILE, pcur, e_, rt_, ct_)                                                   \
    (void)ct_;                                                                               \
    const uint64_t ta_ = (uint64_t)(uintptr_t)(                                              \
        src_token + (size_t)e_ * R + (size_t)rt_ * BM + 64 * wave + lane);                   \
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"            \
                 :: "s"(lds_tok), "v"(ta_) : "memory");                                      \
  }
#define MOE_DMA_GATHER_ROWS(e_, m0_)                                                         \
  {                                                                                          \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                          \
      const int rl_ = 16 * q + (lane >> 2);                                                  \
      const int tok_ = *(lds_int_ptr)(uintptr_t)(lds_tok + 4 * rl_);                         \
      const int row_ = 64 * wave + rl_;                                                      \
      const int ca_ = (lane & 3) ^ ((row_ >> 2) & 3);                                        \
      const bf16_t* src_;                                                                    \
      if (GATHER == 2) {                                                                     \
        src_ = (m0_) + row_ < kept_s[e_] && tok_ >= 0 ? A + (size_t)tok_ * K : zero_row;     \
      } else {                                                                               \
        const uint32_t n_ = (uint32_t)((m0_) + row_);                                        \
        const uint32_t g_ = c_magic ? __umulhi(n_, c_magic) >> c_shift : n_; /* n_ / C */    \
        src_ = tok_ >= 0 ? A + ((size_t)g_ * S + tok_) * K : zero_row;                       \
      }                                                                                      \
      a_addr[q] = (uint64_t)(uintptr_t)(src_ + 8 * ca_);                                     \
    }                                                                                        \
  }
#define MOE_DMA16_ADDR(LDS_U32, ADDR_U64)                                                    \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"            \
               :: "s"(LDS_U32), "v"(ADDR_U64) : "memory")
#define MOE_DMA_COPY_A(LDS_U32, q)                                                           \
  if (GATHER) { MOE_DMA16_ADDR(LDS_U32, a_addr[q]); } else { MOE_DMA16(LDS_U32, a_voff[q], p_a); }
#define MOE_DMA_SET_SOURCES()                                                                \
  {                                                                                          \
    if (DYNK) {                                 /* pass over tiles without a single k step */ \
      while (p_tile < t_end && MOE_DMA_STEPS(p_tile / per_e) == 0) p_tile += stride;         \
    }                                                                                        \
    p_more = __builtin_amdgcn_readfirstlane(p_tile < t_end);                                 \
    if (p_more) {                                                                            \
      MOE_DMA_TILE(p_tile, pcur, e_, rt_, ct_)                                               \
      p_steps = __builtin_amdgcn_readfirstlane(MOE_DMA_STEPS(e_));                           \
      if (GATHER) MOE_DMA_GATHER_ROWS(e_, rt_ * BM)                                          \
      else if (A_MNC) p_a = A + (size_t)e_ * K * R + (size_t)rt_ * BM;                       \
      else p_a = A + ((size_t)e_ * R + (size_t)rt_ * BM) * K;                                \
      if (B_KC) p_b = B + ((size_t)e_ * N + (size_t)ct_ * BN) * K;                           \
      else p_b = B + (size_t)e_ * K * N + (size_t)ct_ * BN;                                  \
    }                                                                                        \
  }
#define MOE_DMA_ADVANCE()                                                                    \
  {                                                                                          \
    ++p_g;                                                                                   \
    p_stage = p_stage + 1 == ST ? 0 : p_stage + 1;                                           \
    if (GATHER) {                                                                            \
      _Pragma("unroll") for (int q = 0; q < 4; ++q) a_addr[q] += BK * 2;                     \
      if (p_kt == KT - 4 && p_tile + stride < t_end) MOE_DMA_TOKENS(p_tile + stride)         \
    } else p_a += A_MNC ? (size_t)BK * R : (size_t)BK;                                       \
    p_b += B_KC ? (size_t)BK : (size_t)BK * N;                                               \
    if (++p_kt == p_steps) { p_kt = 0; p_tile += stride; MOE_DMA_SET_SOURCES() }             \
  }
  if (GATHER) {
    MOE_DMA_TOKENS(first)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  MOE_DMA_SET_SOURCES()

  // fragment read offsets (bytes inside a stage); w0 = the wavefront's first row of the operand
  //   KC operand: row w0 + 32 i + lane%32, chunk 2 kk + lane/32 at its permuted position
  //   MNC operand (transposing read): 16-lane block b = lane/16 covers k rows
  //   8 (b/2) + (lane%16)/4 (+4), rows w0 + 32 j + 16 (b%2) + 4 (lane%4) .. +3; chunk = row / 8
  const int ar = lane & 31;
  const int p16 = lane & 15, bb = lane >> 4;
  const int bk = 8 * (bb >> 1) + (p16 >> 2);                   // k row inside a 16-wide step
  const int bsw = 4 * (bk & 3);                                // permutation of that row
  uint32_t a_rd[4], b_rd[4];                                   // KC: [kk], MNC: [sub-tile]
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int kc_chunk = (2 * (j & 1) + (lane >> 5)) ^ ((ar >> 2) & 3);
    const int ca = (wm0 >> 3) + 4 * j + 2 * (bb & 1) + ((p16 & 3) >> 1);
    const int cb = (wn0 >> 3) + 4 * j + 2 * (bb & 1) + ((p16 & 3) >> 1);
    a_rd[j] = A_MNC ? (uint32_t)(bk * 512 + ((ca ^ bsw) * 16) + (p16 & 1) * 8)
                    : (uint32_t)((wm0 + ar) * 64 + kc_chunk * 16);
    b_rd[j] = B_KC ? (uint32_t)(SM::kAStage + (wn0 + ar) * 64 + kc_chunk * 16)
                   : (uint32_t)(SM::kAStage + bk * 512 + ((cb ^ bsw) * 16) + (p16 & 1) * 8);
  }
  typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
  typedef bf16x8_t __attribute__((address_space(3))) * lds_bf16x8_ptr;
  struct Frags { bf16x8_t a[TM]; bf16x8_t b[TN]; };
#define MOE_DMA_READ_KC(DST, STAGE, RD, kk, i)                                               \
  DST = *(lds_bf16x8_ptr)(uintptr_t)(lds0 + (STAGE) * SM::kStage + RD[kk] + (i) * 32 * 64);
#define MOE_DMA_READ_MNC(DST, STAGE, RD, kk, j)                                              \
  {                                                                                          \
    const uint32_t pb_ = lds0 + (STAGE) * SM::kStage + RD[j] + (kk) * 16 * 512;              \
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)pb_); \
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(                              \
        (lds_s16x4_ptr)(uintptr_t)(pb_ + 4 * 512));                                          \
    DST = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7)); \
  }
#define MOE_DMA_READ_A(F, STAGE, kk, i)                                                      \
  { if (A_MNC) MOE_DMA_READ_MNC((F).a[i], STAGE, a_rd, kk, i) else { MOE_DMA_READ_KC((F).a[i], STAGE, a_rd, kk, i) } }
#define MOE_DMA_READ_B(F, STAGE, kk, j)                                                      \
  { if (B_KC) { MOE_DMA_READ_KC((F).b[j], STAGE, b_rd, kk, j) } else MOE_DMA_READ_MNC((F).b[j], STAGE, b_rd, kk, j) }
  // The weight fragment goes in as the first MFMA operand: the 32x32 result is then
  // the transposed tile, i.e. a lane owns 4 consecutive columns of one row of C.
#define MOE_DMA_MFMA_ROW(F, i)                                                               \
  _Pragma("unroll") for (int j = 0; j < TN; ++j)                                             \
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16((F).b[j], (F).a[i], acc[i][j], 0, 0, 0);

  Frags fr[2];
  // start the first ST-1 steps (as many as there are), wait for step 0
  for (int tl = 0; tl < ST - 1 && p_more; ++tl) {
    const uint32_t la_ = lds0 + p_stage * SM::kStage + wave * 4096;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      MOE_DMA_COPY_A(la_ + q * 1024, q)
      MOE_DMA16(la_ + SM::kAStage + q * 1024, b_voff[q], p_b);
    }
    MOE_DMA_ADVANCE()
  }
  if (p_g >= 3) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else if (p_g == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) { MOE_DMA_READ_A(fr[0], 0, 0, i) MOE_DMA_READ_B(fr[0], 0, 0, i) }

  int stage = 0, g = 0;                                        // consumer cursor
  // The fragment reads are unconditional (the very last step fetches fragments nobody
  // multiplies, from a valid stage): a conditional read would make every later wait
  // for LDS data wait for all outstanding reads instead of the older ones only.
  for (int c_tile = first; c_tile < t_end; c_tile += stride) {
    MOE_DMA_TILE(c_tile, ccur, e, rt, ct)
    const int c_steps = __builtin_amdgcn_readfirstlane(MOE_DMA_STEPS(e));
    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int kt = 0; kt < c_steps; ++kt, ++g) {
      // (a fragment row's reads go out right before the MFMA row of the other k half: pinned,
      // it measures 0.6-0.8 % faster than leaving the order to the compiler)
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        MOE_DMA_READ_A(fr[1], stage, 1, i) MOE_DMA_READ_B(fr[1], stage, 1, i)
        MOE_DMA_MFMA_ROW(fr[0], i)
        __builtin_amdgcn_sched_barrier(0);
      }
      // The own copies of step g+1 must have landed; younger steps (8 copies each) may
      // still fly.  p_g steps have been started.  Copies land in the order they were issued,
      // but stores complete in no fixed order relative to them: "at most n operations
      // outstanding" therefore still proves that all but the n youngest copies have landed,
      // it just may wait for stores as well.  An epilogue first awaits every copy issued so
      // far (steps up to g+3) and only then issues its stores, so the first two steps of the
      // following tile need no wait at all and the stores drain behind their MFMAs.
      // (The counts pass through an empty asm so that the optimiser cannot peel or
      // duplicate the loop body around these conditions: copies of the body would shuffle
      // the 256 accumulator registers between them.)
      // the step to await is g+1, or the last one when the producer has started them all
      int younger = p_g - 1 - (p_more || g + 1 < p_g ? g + 1 : p_g - 1);
      if (kt < 2 && c_tile != first) younger = 3;              // landed before the last epilogue
      younger = __builtin_amdgcn_readfirstlane(younger);
      asm volatile("" : "+s"(younger));
      if (younger <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      else if (younger == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else if (younger == 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      __syncthreads();
      if (EPI == 5 && kt == 0) {
        const unsigned char* src5 = signbits + ((size_t)(e * tiles_m + rt) * tiles_n + ct) * 8192 +
                                    wave * 2048 + lane * 16;
        MOE_DMA16_ADDR(lds_bits, (uint64_t)(uintptr_t)src5);
        MOE_DMA16_ADDR(lds_bits + 1024, (uint64_t)(uintptr_t)(src5 + 1024));
      }
      const int nstage = stage + 1 == ST ? 0 : stage + 1;      // stage of step g+1
      int more = p_more;                                       // p_stage: stage of step g-1, free now
      asm volatile("" : "+s"(more));
      const uint32_t la_ = lds0 + p_stage * SM::kStage + wave * 4096;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (more) {
          MOE_DMA_COPY_A(la_ + q * 1024, q)
          MOE_DMA16(la_ + SM::kAStage + q * 1024, b_voff[q], p_b);
        }
        MOE_DMA_READ_A(fr[0], nstage, 0, q)
        MOE_DMA_READ_B(fr[0], nstage, 0, q)
        MOE_DMA_MFMA_ROW(fr[1], q)
        __builtin_amdgcn_sched_barrier(0);
      }
      if (more) MOE_DMA_ADVANCE()
      stage = nstage;
    }

    // Tile finished: acc[i][j][4 q + r] = C[32 i + r32][32 j + 8 q + 4 h + r], r32 = lane%32,
    // h = lane/32.  The stage of the step just consumed is free until the next step's
    // barrier, so each wavefront turns its tile through 8 KB of it, 32 rows at a time, into
    // full-row 16-byte stores.  Staging layout: [32 rows][16 chunks of 16 bytes], chunk c of
    // row r at position c ^ (r & 15), its two 8-byte halves swapped when r >= 16 (then the
    // 32 lanes of a half-wave write 256 distinct bytes: no bank conflict).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // every copy issued so far
    const int m0 = rt * BM, n0 = ct * BN;
    const size_t c_off = ((size_t)e * R + m0 + wm0) * N + n0 + wn0;
    bf16_t* Ce = Cout + c_off;
    const uint32_t st_base = lds0 + (stage == 0 ? ST - 1 : stage - 1) * SM::kStage + wave * 8192;
    const int r32 = lane & 31, hh = lane >> 5;
    const uint32_t st_wr = st_base + r32 * 256 + 8 * (hh ^ (r32 >> 4));
    typedef u32x2_t __attribute__((address_space(3))) * lds_u2_ptr;
    typedef u32x4_t __attribute__((address_space(3))) * lds_u4_ptr;
    if (EPI == 3) {
      // fp32 result: Cout is a float array; each lane stores its 4 consecutive columns
      float* Cf = reinterpret_cast<float*>(Cout) + c_off;
      typedef float f32x4_t __attribute__((ext_vector_type(4)));
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            *reinterpret_cast<f32x4_t*>(Cf + (size_t)(32 * i + r32) * N + 32 * j + 8 * q + 4 * hh) =
                f32x4_t{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                        acc[i][j][4 * q + 3]};
        __builtin_amdgcn_sched_barrier(0);
      }
      continue;
    }
    u32x4_t bits[2] = {u32x4_t{0u, 0u, 0u, 0u}, u32x4_t{0u, 0u, 0u, 0u}};
    if (EPI == 5) {
      bits[0] = *(lds_u4_ptr)(uintptr_t)(lds_bits + lane * 16);
      bits[1] = *(lds_u4_ptr)(uintptr_t)(lds_bits + 1024 + lane * 16);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      int drow[8];                                             // SCATTER: destination rows
      if (SCATTER) {
#pragma unroll
        for (int ps = 0; ps < 8; ++ps) {
          const int pr = m0 + wm0 + 32 * i + 4 * ps + (lane >> 4);
          drow[ps] = pr < kept_s[e] ? src_token[(size_t)e * R + pr] : -1;
        }
      }
      u32x4_t mk[8];
      if (EPI == 2) {
#pragma unroll
        for (int ps = 0; ps < 8; ++ps)
          mk[ps] = *reinterpret_cast<const u32x4_t*>(
              mask + c_off + (size_t)(32 * i + 4 * ps + (lane >> 4)) * N + 8 * (lane & 15));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint32_t lo = pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
          uint32_t hi = pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
          if (RELU) { lo = relu_bf16x2(lo); hi = relu_bf16x2(hi); }
          *(lds_u2_ptr)(uintptr_t)(st_wr + (((4 * j + q) ^ (r32 & 15)) * 16)) = u32x2_t{lo, hi};
        }
#pragma unroll
      for (int ps = 0; ps < 8; ++ps) {
        const int rr = 4 * ps + (lane >> 4), c = lane & 15;
        u32x4_t d = *(lds_u4_ptr)(uintptr_t)(st_base + rr * 256 + ((c ^ (rr & 15)) * 16));
        if (ps >= 4) d = u32x4_t{d[2], d[3], d[0], d[1]};      // rows 16..31: halves were swapped
        if (EPI == 2) {
#pragma unroll
          for (int w = 0; w < 4; ++w)
            d[w] &= ((mk[ps][w] & 0xffffu) ? 0xffffu : 0u) | ((mk[ps][w] >> 16) ? 0xffff0000u : 0u);
        }
        if (EPI == 4) {
          uint32_t byte = 0;
#pragma unroll
          for (int w = 0; w < 4; ++w)
            byte |= ((d[w] & 0xffffu) ? 1u : 0u) << (2 * w) | ((d[w] >> 16) ? 2u : 0u) << (2 * w);
          bits[i >> 1][2 * (i & 1) + (ps >> 2)] |= byte << (8 * (ps & 3));
        }
        if (EPI == 5) {
          const uint32_t byte = bits[i >> 1][2 * (i & 1) + (ps >> 2)] >> (8 * (ps & 3));
#pragma unroll
          for (int w = 0; w < 4; ++w)
            d[w] &= ((byte >> (2 * w)) & 1u ? 0xffffu : 0u) | ((byte >> (2 * w + 1)) & 1u ? 0xffff0000u : 0u);
        }
        if (SCATTER) {
          if (drow[ps] >= 0)
            *reinterpret_cast<u32x4_t*>(Cout + (size_t)drow[ps] * N + n0 + wn0 + 8 * c) = d;
        } else {
          *reinterpret_cast<u32x4_t*>(Ce + (size_t)(32 * i + rr) * N + 8 * c) = d;
        }
      }
      __builtin_amdgcn_sched_barrier(0);   // one row group at a time: small register need
    }
    if (EPI == 4) {
      unsigned char* dst4 = signbits + ((size_t)(e * tiles_m + rt) * tiles_n + ct) * 8192 +
                            wave * 2048 + lane * 16;
      *reinterpret_cast<u32x4_t*>(dst4) = bits[0];
      *reinterpret_cast<u32x4_t*>(dst4 + 1024) = bits[1];
    }
  }
#undef MOE_DMA_SET_SOURCES
#undef MOE_DMA_STEPS
#undef MOE_DMA_TILE
#undef MOE_DMA_GATHER_ROWS
#undef MOE_DMA_TOKENS
#undef MOE_DMA16_ADDR
#undef MOE_DMA_COPY_A
#undef MOE_DMA_ADVANCE
#undef MOE_DMA_READ_A
#undef MOE_DMA_READ_KC
#undef MOE_DMA_READ_MNC
#undef MOE_DMA_READ_B
#undef MOE_DMA_MFMA_ROW
}

// LDS limit of one instantiation of the persistent kernel on the current device (all of the
// 160 KB when the size depends on the number of experts)
template <int ST, int EPI, int GATHER, bool A_MNC = false, bool B_KC = false, bool PACKED = false,
          bool SCATTER = false, bool DYNK = false>
int prepare_dma() {
  static LdsLimitOnce once;
  constexpr int kFixed = (int)DmaSmem<ST>::kBytes + (GATHER ? 1024 : 0) + (EPI == 5 ? 8192 : 0);
  return ensure_lds_limit(
      once, reinterpret_cast<const void*>(
                expert_gemm_bf16_dma_kernel<ST, EPI, GATHER, A_MNC, B_KC, PACKED, SCATTER, DYNK>),
      PACKED || DYNK ? 160 * 1024 : kFixed);
}

template <int ST, int EPI, int GATHER, bool A_MNC = false, bool B_KC = false, bool PACKED = false,
          bool SCATTER = false, bool DYNK = false>
int launch_bf16_dma(const bf16_t* A, const bf16_t* B, bf16_t* Cout, int E, int R, int N, int K,
                    const int32_t* src_token, const bf16_t* zero_row, int S, int C, hipStream_t st,
                    const bf16_t* mask = nullptr, unsigned char* signbits = nullptr,
                    const int32_t* kept = nullptr) {
  using SM = DmaSmem<ST>;
  static_assert(!(GATHER && EPI == 5), "the two users of the spare LDS exclude each other");
  // PACKED / DYNK: 2 E + 1 more integers of LDS (row counts and running tile counts of the experts)
  const size_t kLds = SM::kBytes + (GATHER ? 4 * 64 * sizeof(int32_t) : 0) + (EPI == 5 ? 8192 : 0) +
                      (PACKED || DYNK ? align_up(((size_t)2 * E + 1) * sizeof(int32_t), 16) : 0);
  if (kLds > 160 * 1024) return MOE_EUNSUPPORTED;
  // n / C for n < 2^31 as (n * c_magic) >> (32 + c_shift), c_magic = ceil(2^(31+l) / C) with
  // l = ceil(log2 C); C == 1 is flagged by c_magic == 0
  uint32_t c_magic = 0;
  int c_shift = 0;
  if (GATHER == 1 && C > 1) {
    int l = 0;
    while ((1LL << l) < C) ++l;
    c_magic = (uint32_t)((((unsigned long long)1 << (31 + l)) + C - 1) / C);
    c_shift = l - 1;
  }
  if ((PACKED || DYNK) && kept == nullptr) return MOE_EINVAL;
  auto kern = expert_gemm_bf16_dma_kernel<ST, EPI, GATHER, A_MNC, B_KC, PACKED, SCATTER, DYNK>;
  int cus = 0;
  if (prepare_dma<ST, EPI, GATHER, A_MNC, B_KC, PACKED, SCATTER, DYNK>() != MOE_OK ||
      compute_units(&cus) != MOE_OK)
    return MOE_EHIP;
  const int tiles_m = R / 256, tiles_n = N / 256;
  const long long ntiles = (long long)E * tiles_m * tiles_n;
  if (ntiles > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  const unsigned grid = (unsigned)(ntiles < cus ? ntiles : cus);   // one block per CU (LDS-bound)
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), kLds, st, A, B, Cout, R, N, K, tiles_m,
                     tiles_n, (int)ntiles, src_token, zero_row, S, c_magic, c_shift, mask, signbits,
                     kept, E);
  return check_launch();
}

// shapes the persistent 256x256 kernel takes (its per-lane byte offsets are 32-bit)
inline bool dma_shape_ok(int R, int N, int K) {
  const long long big = R > N ? (R > K ? R : K) : (N > K ? N : K);
  return R % 256 == 0 && N % 256 == 0 && K % 32 == 0 && 256 * big * 2 < (1LL << 31);
}

template <int BM, int BN, int BK, int EPI, bool A_MNC, bool B_KC, bool EXACT>
int prepare_tiled() {
  static LdsLimitOnce once;
  return ensure_lds_limit(
      once,
      reinterpret_cast<const void*>(expert_gemm_bf16_kernel<BM, BN, BK, 2, 2, EPI, A_MNC, B_KC, EXACT>),
      (int)GemmSmem<BM, BN, BK, A_MNC, B_KC>::kBytes);
}

template <int BM, int BN, int BK, int EPI, bool A_MNC, bool B_KC, bool EXACT>
int launch_bf16_kernel(const bf16_t* A, const bf16_t* B, bf16_t* Cout, const bf16_t* mask, int E,
                       int R, int N, int K, hipStream_t st) {
  using SM = GemmSmem<BM, BN, BK, A_MNC, B_KC>;
  auto kern = expert_gemm_bf16_kernel<BM, BN, BK, 2, 2, EPI, A_MNC, B_KC, EXACT>;
  if (prepare_tiled<BM, BN, BK, EPI, A_MNC, B_KC, EXACT>() != MOE_OK) return MOE_EHIP;
  const int tiles_m = (R + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const long long nblk = (long long)E * tiles_m * tiles_n;
  if (nblk > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), SM::kBytes, st, A, B, Cout, mask, R, N, K,
                     tiles_m, tiles_n, (int)nblk);
  return check_launch();
}

// C [E,R,N] for any R, N, K with N % 8 == 0 and the operands' contiguous dimensions % 8 == 0
// (K for a K-contiguous operand, R / N for a row-of-k one): 256x256 tiles when the output is
// large enough, else 128x128.
template <int EPI, bool A_MNC, bool B_KC>
int gemm_bf16_tiled(const bf16_t* A, const bf16_t* B, bf16_t* Cout, const bf16_t* mask, int E, int R,
                    int N, int K, hipStream_t st) {
  if (R > 128 && N >= 256) {
    if (R % 256 == 0 && N % 256 == 0 && K % 64 == 0)
      return launch_bf16_kernel<256, 256, 64, EPI, A_MNC, B_KC, true>(A, B, Cout, mask, E, R, N, K, st);
    return launch_bf16_kernel<256, 256, 64, EPI, A_MNC, B_KC, false>(A, B, Cout, mask, E, R, N, K, st);
  }
  if (R % 128 == 0 && N % 128 == 0 && K % 64 == 0)
    return launch_bf16_kernel<128, 128, 64, EPI, A_MNC, B_KC, true>(A, B, Cout, mask, E, R, N, K, st);
  return launch_bf16_kernel<128, 128, 64, EPI, A_MNC, B_KC, false>(A, B, Cout, mask, E, R, N, K, st);
}

template <bool RELU>
int gemm_bf16(const bf16_t* A, const bf16_t* B, bf16_t* Cout, int E, int R, int N, int K,
              hipStream_t st) {
  if (dma_shape_ok(R, N, K))
    return launch_bf16_dma<4, RELU ? 1 : 0, 0>(A, B, Cout, E, R, N, K, nullptr, nullptr, 0, 0,
                                                   st);
  return gemm_bf16_tiled<RELU ? 1 : 0, false, false>(A, B, Cout, nullptr, E, R, N, K, st);
}

// ---------------------------------------------------------------- fp32 path
// fp32 layers multiply on the matrix cores in full fp32 (gemm_f32.hip); M and H are multiples
// of 8, so every operand meets that kernel's 16-byte rule.
template <bool RELU>
int gemm_f32(const float* A, const float* B, float* Cout, int E, int R, int N, int K,
             hipStream_t st) {
  const long long ae = (long long)R * K, be = (long long)K * N;
  if (ae % 4 != 0 || be % 4 != 0 || !gemm_f32_mfma_ok(K, 1, N, 1, E, R, N, K))
    return MOE_EUNSUPPORTED;
  return launch_gemm_f32_mfma(RELU ? 1 : 0, A, ae, K, 1, B, be, N, 1, Cout, nullptr, E, R, N, K, st);
}

}  // namespace

int compute_units(int* cus) {
  static std::atomic<int> cus_of[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_EHIP;
  int n = cus_of[dev].load(std::memory_order_acquire);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
      return MOE_EHIP;
    cus_of[dev].store(n, std::memory_order_release);
  }
  *cus = n;
  return MOE_OK;
}

// Every instantiation the launchers of this file use (a kernel missing from this list is
// still set up by its launcher's first call).
int prepare_expert_gemm() {
  const int rcs[] = {
      // forward
      prepare_dma<4, 1, 0>(), prepare_dma<4, 0, 0>(), prepare_dma<4, 1, 1>(), prepare_dma<4, 4, 1>(),
      prepare_dma<4, 1, 2, false, false, true>(), prepare_dma<4, 4, 2, false, false, true>(),
      prepare_dma<4, 0, 0, false, false, true, false>(), prepare_dma<4, 0, 0, false, false, true, true>(),
      // fp32 results (gate logits and gate gradients)
      prepare_dma<4, 3, 0, true, false>(), prepare_dma<4, 3, 0, false, true>(),
      // backward
      prepare_dma<4, 5, 0, false, true>(), prepare_dma<4, 2, 0, false, true>(),
      prepare_dma<4, 0, 0, true, false>(), prepare_dma<4, 0, 0, false, true>(),
      prepare_dma<4, 5, 0, false, true, true>(), prepare_dma<4, 0, 0, false, true, true>(),
      prepare_dma<4, 0, 0, true, false, false, false, true>(),
      // ragged shapes: forward (relu / plain), data gradients (plain / masked), weight gradients
#define MOE_TILED_BOTH(EPI, AM, BK_)                                                              \
      prepare_tiled<256, 256, 64, EPI, AM, BK_, true>(), prepare_tiled<256, 256, 64, EPI, AM, BK_, false>(), \
      prepare_tiled<128, 128, 64, EPI, AM, BK_, true>(), prepare_tiled<128, 128, 64, EPI, AM, BK_, false>()
      MOE_TILED_BOTH(1, false, false), MOE_TILED_BOTH(0, false, false), MOE_TILED_BOTH(0, false, true),
      MOE_TILED_BOTH(2, false, true), MOE_TILED_BOTH(0, true, false)};
#undef MOE_TILED_BOTH
  int cus = 0;
  if (compute_units(&cus) != MOE_OK) return MOE_EHIP;
  for (int rc : rcs)
    if (rc != MOE_OK) return rc;
  return MOE_OK;
}

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

// Batched bf16 GEMM with an fp32 result for the gate gradients (A, B, C as in the kernel's
// layout table; batch plays the role of the expert index).
bool gemm_bf16_f32out_ok(int R, int N, int K) { return dma_shape_ok(R, N, K); }

int launch_gemm_bf16_f32out(bool transposed_a, const void* A, const void* B, float* Cout,
                            int batch, int R, int N, int K, hipStream_t st) {
  if (!dma_shape_ok(R, N, K)) return MOE_EUNSUPPORTED;
  auto a = static_cast<const bf16_t*>(A);
  auto b = static_cast<const bf16_t*>(B);
  auto c = reinterpret_cast<bf16_t*>(Cout);
  // transposed_a: C = A^T . B with A [K,R], B [K,N];  else C = A . B^T with A [R,K], B [N,K]
  return transposed_a
             ? launch_bf16_dma<4, 3, 0, true, false>(a, b, c, batch, R, N, K, nullptr, nullptr, 0, 0, st)
             : launch_bf16_dma<4, 3, 0, false, true>(a, b, c, batch, R, N, K, nullptr, nullptr, 0, 0, st);
}

bool expert_gemm1_can_gather(const moe_config& c) {
  const long long rows = (long long)c.G * c.C;
  // the kernel fetches a tile's dispatch indices 4 K-steps (of 32) ahead of its first copy
  return c.act_dtype == MOE_BF16 && rows <= 0x7fffffffLL && c.M >= 128 &&
         dma_shape_ok((int)rows, c.H, c.M);
}

int launch_expert_gemm1_gather(const moe_config& c, const void* x, const int32_t* src_token,
                               const void* zero_row, const void* wi, void* h, void* signbits,
                               hipStream_t st) {
  if (!expert_gemm1_can_gather(c)) return MOE_EUNSUPPORTED;
  if (signbits != nullptr)
    return launch_bf16_dma<4, 4, 1>(static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(wi),
                                       static_cast<bf16_t*>(h), c.E, c.G * c.C, c.H, c.M, src_token,
                                       static_cast<const bf16_t*>(zero_row), c.S, c.C, st, nullptr,
                                       static_cast<unsigned char*>(signbits));
  return launch_bf16_dma<4, 1, 1>(static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(wi),
                                        static_cast<bf16_t*>(h), c.E, c.G * c.C, c.H, c.M, src_token,
                                        static_cast<const bf16_t*>(zero_row), c.S, c.C, st);
}

// Packed row layout: both GEMMs walk the list of occupied row tiles.  The first gathers its rows
// through pk.packed_src (absolute rows of `a`: token rows of x, or rows of an [E,G,C,M] buffer),
// h and (scatter_out == false) out hold packed rows; scatter_out sends the rows of out back to
// the absolute rows pk.packed_src names.
int launch_expert_ffn_packed(const moe_config& c, const void* a, const RowPacking& pk,
                             const void* zero_row, const void* wi, const void* wo, void* h,
                             void* out, bool scatter_out, void* signbits, hipStream_t st,
                             void* event_between) {
  if (!expert_ffn_can_pack(c)) return MOE_EUNSUPPORTED;
  const int R = c.G * c.C;
  int rc = signbits != nullptr
               ? launch_bf16_dma<4, 4, 2, false, false, true>(
                     static_cast<const bf16_t*>(a), static_cast<const bf16_t*>(wi),
                     static_cast<bf16_t*>(h), c.E, R, c.H, c.M, pk.packed_src,
                     static_cast<const bf16_t*>(zero_row), c.S, c.C, st, nullptr,
                     static_cast<unsigned char*>(signbits), pk.kept)
               : launch_bf16_dma<4, 1, 2, false, false, true>(
                     static_cast<const bf16_t*>(a), static_cast<const bf16_t*>(wi),
                     static_cast<bf16_t*>(h), c.E, R, c.H, c.M, pk.packed_src,
                     static_cast<const bf16_t*>(zero_row), c.S, c.C, st, nullptr, nullptr, pk.kept);
  if (rc != MOE_OK) return rc;
  if (event_between != nullptr &&
      hipEventRecord(static_cast<hipEvent_t>(event_between), st) != hipSuccess)
    return MOE_EHIP;
  if (scatter_out)
    return launch_bf16_dma<4, 0, 0, false, false, true, true>(
        static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(wo), static_cast<bf16_t*>(out), c.E,
        R, c.M, c.H, pk.packed_src, nullptr, 0, 0, st, nullptr, nullptr, pk.kept);
  return launch_bf16_dma<4, 0, 0, false, false, true, false>(
      static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(wo), static_cast<bf16_t*>(out), c.E, R,
      c.M, c.H, nullptr, nullptr, 0, 0, st, nullptr, nullptr, pk.kept);
}

bool expert_ffn_can_pack(const moe_config& c) {
  // E: the kernels keep 2 E + 1 integers in the LDS left over by the stages
  return expert_gemm1_can_gather(c) && dma_shape_ok(c.G * c.C, c.M, c.H) && c.E <= 2048;
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

// ---- backward pass: A K-contiguous x B K-contiguous (dgrad), A and B row(k)-major (wgrad) ----
int launch_expert_dgrad2(const moe_config& c, const void* dout, const void* wo, const void* h,
                         const void* signbits, void* dh, const int32_t* kept, hipStream_t st) {
  const long long R = (long long)c.G * c.C;
  if (kept != nullptr) {
    if (signbits == nullptr || !expert_ffn_can_pack(c)) return MOE_EINVAL;
    return launch_bf16_dma<4, 5, 0, false, true, true>(
        static_cast<const bf16_t*>(dout), static_cast<const bf16_t*>(wo), static_cast<bf16_t*>(dh),
        c.E, (int)R, c.H, c.M, nullptr, nullptr, 0, 0, st, nullptr,
        const_cast<unsigned char*>(static_cast<const unsigned char*>(signbits)), kept);
  }
  // the forward pass recorded the sign bits exactly when its first GEMM gathered (K >= 128)
  if (signbits != nullptr && expert_gemm1_can_gather(c))
    return launch_bf16_dma<4, 5, 0, false, true>(
        static_cast<const bf16_t*>(dout), static_cast<const bf16_t*>(wo), static_cast<bf16_t*>(dh),
        c.E, (int)R, c.H, c.M, nullptr, nullptr, 0, 0, st, nullptr,
        const_cast<unsigned char*>(static_cast<const unsigned char*>(signbits)));
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL && dma_shape_ok((int)R, c.H, c.M))
    return launch_bf16_dma<4, 2, 0, false, true>(
        static_cast<const bf16_t*>(dout), static_cast<const bf16_t*>(wo), static_cast<bf16_t*>(dh),
        c.E, (int)R, c.H, c.M, nullptr, nullptr, 0, 0, st, static_cast<const bf16_t*>(h));
  // other bf16 shapes: the tiled MFMA kernel, A . B^T with the mask epilogue
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL)
    return gemm_bf16_tiled<2, false, true>(static_cast<const bf16_t*>(dout), static_cast<const bf16_t*>(wo),
                                           static_cast<bf16_t*>(dh), static_cast<const bf16_t*>(h), c.E,
                                           (int)R, c.H, c.M, st);
  return launch_gemm_strided(c, 2, dout, R * c.M, c.M, 1, wo, (long long)c.H * c.M, 1, c.M, dh, h,
                             (int)R, c.H, c.M, st);
}

int launch_expert_wgrad2(const moe_config& c, const void* h, const void* dout, void* dwo,
                         const int32_t* kept, hipStream_t st) {
  const long long R = (long long)c.G * c.C;
  if (kept != nullptr) {
    if (!expert_ffn_can_pack(c)) return MOE_EINVAL;
    return launch_bf16_dma<4, 0, 0, true, false, false, false, true>(
        static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(dout), static_cast<bf16_t*>(dwo),
        c.E, c.H, c.M, (int)R, nullptr, nullptr, 0, 0, st, nullptr, nullptr, kept);
  }
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL && dma_shape_ok(c.H, c.M, (int)R))
    return launch_bf16_dma<4, 0, 0, true, false>(
        static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(dout), static_cast<bf16_t*>(dwo),
        c.E, c.H, c.M, (int)R, nullptr, nullptr, 0, 0, st);
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL)       // A^T . B on the tiled MFMA kernel
    return gemm_bf16_tiled<0, true, false>(static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(dout),
                                           static_cast<bf16_t*>(dwo), nullptr, c.E, c.H, c.M, (int)R, st);
  return launch_gemm_strided(c, 0, h, R * c.H, 1, c.H, dout, R * c.M, c.M, 1, dwo, nullptr, c.H,
                             c.M, (int)R, st);
}

int launch_expert_dgrad1(const moe_config& c, const void* dh, const void* wi, void* dbuf,
                         const int32_t* kept, hipStream_t st) {
  const long long R = (long long)c.G * c.C;
  if (kept != nullptr) {
    if (!expert_ffn_can_pack(c)) return MOE_EINVAL;
    return launch_bf16_dma<4, 0, 0, false, true, true>(
        static_cast<const bf16_t*>(dh), static_cast<const bf16_t*>(wi), static_cast<bf16_t*>(dbuf),
        c.E, (int)R, c.M, c.H, nullptr, nullptr, 0, 0, st, nullptr, nullptr, kept);
  }
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL && dma_shape_ok((int)R, c.M, c.H))
    return launch_bf16_dma<4, 0, 0, false, true>(
        static_cast<const bf16_t*>(dh), static_cast<const bf16_t*>(wi), static_cast<bf16_t*>(dbuf),
        c.E, (int)R, c.M, c.H, nullptr, nullptr, 0, 0, st);
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL)       // A . B^T on the tiled MFMA kernel
    return gemm_bf16_tiled<0, false, true>(static_cast<const bf16_t*>(dh), static_cast<const bf16_t*>(wi),
                                           static_cast<bf16_t*>(dbuf), nullptr, c.E, (int)R, c.M, c.H, st);
  return launch_gemm_strided(c, 0, dh, R * c.H, c.H, 1, wi, (long long)c.M * c.H, 1, c.H, dbuf,
                             nullptr, (int)R, c.M, c.H, st);
}

int launch_expert_wgrad1(const moe_config& c, const void* buf, const void* dh, void* dwi,
                         const int32_t* kept, hipStream_t st) {
  const long long R = (long long)c.G * c.C;
  if (kept != nullptr) {
    if (!expert_ffn_can_pack(c)) return MOE_EINVAL;
    return launch_bf16_dma<4, 0, 0, true, false, false, false, true>(
        static_cast<const bf16_t*>(buf), static_cast<const bf16_t*>(dh), static_cast<bf16_t*>(dwi),
        c.E, c.M, c.H, (int)R, nullptr, nullptr, 0, 0, st, nullptr, nullptr, kept);
  }
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL && dma_shape_ok(c.M, c.H, (int)R))
    return launch_bf16_dma<4, 0, 0, true, false>(
        static_cast<const bf16_t*>(buf), static_cast<const bf16_t*>(dh), static_cast<bf16_t*>(dwi),
        c.E, c.M, c.H, (int)R, nullptr, nullptr, 0, 0, st);
  if (c.act_dtype == MOE_BF16 && R <= 0x7fffffffLL)       // A^T . B on the tiled MFMA kernel
    return gemm_bf16_tiled<0, true, false>(static_cast<const bf16_t*>(buf), static_cast<const bf16_t*>(dh),
                                           static_cast<bf16_t*>(dwi), nullptr, c.E, c.M, c.H, (int)R, st);
  return launch_gemm_strided(c, 0, buf, R * c.M, 1, c.M, dh, R * c.H, c.H, 1, dwi, nullptr, c.M,
                             c.H, (int)R, st);
}

}  // namespace moe
