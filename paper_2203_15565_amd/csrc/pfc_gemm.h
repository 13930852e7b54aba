// MFMA tile engine for the three GEMMs of the PFC step (gfx950).
//
// All three products are brought to the "NT" form  C[m][n] = sum_k A[m][k] * B[n][k]  with both
// operands row-major and k contiguous, so that every lane's MFMA fragment is one 16-byte load:
//   logits    C[j][i] = <Wn_j, Xn_i>                 A = Wn  [kp x D],  B = Xn  [Bp x D]
//   dweight   C[j][d] = sum_i ET[j][i] * XsT[d][i]   A = ET  [kp x Bp], B = XsT [D x Bp]
//   dfeatures C[i][d] = sum_j E[i][j]  * WnT[d][j]   A = E   [Bp x kp], B = WnT [D x kp]
// Operands are padded with zeros to whole tiles by their producers: no bounds checks here.
//
// A workgroup of WM x WN wavefronts (64 lanes each) owns a BM x BN tile of C.  K is walked in
// slabs of 128 bytes per row (64 bf16 / 32 fp32); a slab of A and B is staged in LDS (double
// buffered, rows padded by 16 bytes so that a 16-byte fragment read by 16 consecutive rows
// touches every bank once) and consumed with v_mfma_f32_32x32x16_bf16 (bf16) or
// v_mfma_f32_32x32x2_f32 (fp32).
//
// Fragment convention (both operands alike, which is all that a dot product needs): within a
// 32-byte group g of a row, lanes 0..31 take bytes [0,16) and lanes 32..63 bytes [16,32).
// For bf16 that is 8 consecutive k per lane = one 32x32x16 MFMA; for fp32 it is 4 consecutive k
// per lane = four 32x32x2 MFMAs, the t-th of which pairs element t of every lane.
//
// Accumulator layout of a 32x32 block (16 floats per lane): register r of lane l holds
//   row = (r / 4) * 8 + (l / 32) * 4 + (r % 4),  col = l % 32.
#pragma once

#include "pfc_common.h"

namespace pfc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSlabBytes = 128;            // bytes of K per row per slab
constexpr int kLdsRow = kSlabBytes + 16;   // padded LDS row stride

template <typename T, int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
  using elem = T;
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int BK = kSlabBytes / (int)sizeof(T);   // elements of K per slab
  static constexpr int THREADS = WM * WN * 64;
  static constexpr int WTM = BM / WM, WTN = BN / WN;       // tile of one wavefront
  static constexpr int TM = WTM / 32, TN = WTN / 32;       // 32x32 blocks per wavefront
  static constexpr int A_BYTES = BM * kLdsRow, B_BYTES = BN * kLdsRow;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int A_CHUNKS = BM * 8 / THREADS;        // 16-byte chunks per thread per slab
  static constexpr int B_CHUNKS = BN * 8 / THREADS;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be whole 32x32 blocks");
  static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "slab must divide evenly");
};

template <typename T>
__device__ __forceinline__ void mfma_group(const u32x4& a, const u32x4& b, f32x16& c);

template <>
__device__ __forceinline__ void mfma_group<__bf16>(const u32x4& a, const u32x4& b, f32x16& c) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                              __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mfma_group<float>(const u32x4& a, const u32x4& b, f32x16& c) {
  // whole-vector casts: a bit_cast applied to a single vector element reads element 0
  const f32x4 af = __builtin_bit_cast(f32x4, a);
  const f32x4 bf = __builtin_bit_cast(f32x4, b);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[0], bf[0], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[1], bf[1], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[2], bf[2], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[3], bf[3], c, 0, 0, 0);
}

// Accumulate acc += A_tile * B_tile^T over `nslabs` slabs of K.
//   A: first row of this workgroup's BM rows, at the first k of its range; lda in elements.
//   B: likewise for its BN rows.
//   smem: Cfg::LDS_BYTES bytes, 16-byte aligned.
template <class Cfg>
__device__ __forceinline__ void gemm_tile_nt(const typename Cfg::elem* __restrict__ A, int64_t lda,
                                             const typename Cfg::elem* __restrict__ B, int64_t ldb,
                                             int nslabs, char* smem,
                                             f32x16 (&acc)[Cfg::TM][Cfg::TN]) {
  using T = typename Cfg::elem;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
  const int half = lane >> 5, l32 = lane & 31;

  // global -> LDS staging: thread handles chunk (tid % 8) of rows (tid / 8) + i * THREADS/8
  const int ld_row = tid >> 3, ld_chunk = tid & 7;
  constexpr int ROWS_PER_PASS = Cfg::THREADS / 8;
  const char* gA = reinterpret_cast<const char*>(A) + (int64_t)ld_row * lda * (int64_t)sizeof(T) +
                   ld_chunk * 16;
  const char* gB = reinterpret_cast<const char*>(B) + (int64_t)ld_row * ldb * (int64_t)sizeof(T) +
                   ld_chunk * 16;
  const int64_t strideA = (int64_t)ROWS_PER_PASS * lda * (int64_t)sizeof(T);
  const int64_t strideB = (int64_t)ROWS_PER_PASS * ldb * (int64_t)sizeof(T);
  const int st_off = ld_row * kLdsRow + ld_chunk * 16;

  u32x4 ra[Cfg::A_CHUNKS], rb[Cfg::B_CHUNKS];

#pragma unroll
  for (int i = 0; i < Cfg::A_CHUNKS; ++i)
    ra[i] = *reinterpret_cast<const u32x4*>(gA + i * strideA);
#pragma unroll
  for (int i = 0; i < Cfg::B_CHUNKS; ++i)
    rb[i] = *reinterpret_cast<const u32x4*>(gB + i * strideB);
#pragma unroll
  for (int i = 0; i < Cfg::A_CHUNKS; ++i)
    *reinterpret_cast<u32x4*>(smem + st_off + i * ROWS_PER_PASS * kLdsRow) = ra[i];
#pragma unroll
  for (int i = 0; i < Cfg::B_CHUNKS; ++i)
    *reinterpret_cast<u32x4*>(smem + Cfg::A_BYTES + st_off + i * ROWS_PER_PASS * kLdsRow) = rb[i];
  __syncthreads();

  const int fa_off = (wm * Cfg::WTM + l32) * kLdsRow + half * 16;
  const int fb_off = Cfg::A_BYTES + (wn * Cfg::WTN + l32) * kLdsRow + half * 16;

  for (int s = 0; s < nslabs; ++s) {
    const char* cur = smem + (s & 1) * Cfg::STAGE_BYTES;
    char* nxt = smem + ((s + 1) & 1) * Cfg::STAGE_BYTES;
    const bool more = (s + 1 < nslabs);
    if (more) {
      const int64_t koff = (int64_t)(s + 1) * kSlabBytes;
#pragma unroll
      for (int i = 0; i < Cfg::A_CHUNKS; ++i)
        ra[i] = *reinterpret_cast<const u32x4*>(gA + koff + i * strideA);
#pragma unroll
      for (int i = 0; i < Cfg::B_CHUNKS; ++i)
        rb[i] = *reinterpret_cast<const u32x4*>(gB + koff + i * strideB);
    }
#pragma unroll
    for (int g = 0; g < kSlabBytes / 32; ++g) {
      u32x4 fa[Cfg::TM], fb[Cfg::TN];
#pragma unroll
      for (int bm = 0; bm < Cfg::TM; ++bm)
        fa[bm] = *reinterpret_cast<const u32x4*>(cur + fa_off + bm * 32 * kLdsRow + g * 32);
#pragma unroll
      for (int bn = 0; bn < Cfg::TN; ++bn)
        fb[bn] = *reinterpret_cast<const u32x4*>(cur + fb_off + bn * 32 * kLdsRow + g * 32);
#pragma unroll
      for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
        for (int bn = 0; bn < Cfg::TN; ++bn) mfma_group<T>(fa[bm], fb[bn], acc[bm][bn]);
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < Cfg::A_CHUNKS; ++i)
        *reinterpret_cast<u32x4*>(nxt + st_off + i * ROWS_PER_PASS * kLdsRow) = ra[i];
#pragma unroll
      for (int i = 0; i < Cfg::B_CHUNKS; ++i)
        *reinterpret_cast<u32x4*>(nxt + Cfg::A_BYTES + st_off + i * ROWS_PER_PASS * kLdsRow) = rb[i];
    }
    __syncthreads();
  }
}

// Row / column of accumulator register r of block (bm, bn) inside the workgroup tile.
template <class Cfg>
__device__ __forceinline__ int acc_row(int bm, int r) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  return (wave / Cfg::WN) * Cfg::WTM + bm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
}
template <class Cfg>
__device__ __forceinline__ int acc_col(int bn) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  return (wave % Cfg::WN) * Cfg::WTN + bn * 32 + (lane & 31);
}

// XCD-aware order of workgroups: consecutive workgroup ids are dealt round-robin to the 8 XCDs
// (each with its own L2), so the `inner` workgroups that share an operand tile are given ids
// that land on one XCD.  Returns false for the padding ids of a rounded-up grid.
__device__ __forceinline__ bool xcd_tile(int wg, int inner, int outer, int& o, int& i) {
  const int xcd = wg & 7, local = wg >> 3;
  o = (local / inner) * 8 + xcd;
  i = local % inner;
  return o < outer;
}
inline int xcd_grid(int inner, int outer) { return (int)round_up(outer, 8) * inner; }

}  // namespace pfc
