// MFMA tile engine for the three GEMMs of the PFC step (gfx950).
//
//   logits    C[j][i] = sum_d Wn[j][d] * Xn[i][d]        A = Wn  (k contiguous), B = Xn (k contiguous)
//   dweight   C[j][d] = sum_i E[i][j]  * Xs[i][d]        A = E   (k-major),      B = Xs (k-major)
//   dfeatures C[i][d] = sum_j E[i][j]  * Wn[j][d]        A = E   (k contiguous), B = Wn (k-major)
//
// Every matrix stays in its one natural row-major layout in HBM; an operand whose reduction
// index is its ROW index ("k-major") is staged in LDS as it is and transposed on the way into
// the MFMA registers by the LDS transpose read of gfx950 (ds_read_b64_tr_b16), so no transposed
// copy of E, Wn or Xs is ever written.  Operands are padded with zeros to whole tiles by their
// producers: the main loop has no bounds checks.
//
// A workgroup of WM x WN wavefronts (64 lanes each) owns a BM x BN tile of C.  K is walked in
// slabs of BK = 64 (bf16) or 32 (fp32) reduction steps, double buffered in LDS; slab s+1 waits in
// the second LDS stage and the global loads of slab s+2 are in flight in registers while slab s
// is multiplied.
//
// LDS layouts of one operand slab (R = BM or BN rows of the operand tile):
//   k contiguous: R rows of 128 bytes, row stride 144: a 16-byte fragment read by 16 consecutive
//                 rows touches every bank once.
//   k-major:      BK rows of R*sizeof(T) bytes, row stride + 64: the four k-rows that one
//                 transpose read gathers fall into different banks.
//
// Fragment convention (the same for A and B, which is all a dot product needs): a group of 16
// (bf16) or 8 (fp32) reduction steps is split between the lane halves, lanes 0..31 taking the
// first half and lanes 32..63 the second; for bf16 that is one v_mfma_f32_32x32x16_bf16 per
// group, for fp32 four v_mfma_f32_32x32x2_f32, the t-th of which pairs element t of every lane.
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
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));


// Geometry of one operand slab in LDS.
// SLAB: bytes of K per operand row per slab (128, or 64 for tiles whose wide operand would not fit).
template <typename T, int R, bool KMAJOR, int SLAB>
struct OperandLds {
  static constexpr int SLAB_BYTES = SLAB;
  static constexpr int BK = SLAB / (int)sizeof(T);
  static constexpr int ROWS = KMAJOR ? BK : R;                                   // LDS rows
  static constexpr int ROW_BYTES = KMAJOR ? R * (int)sizeof(T) : SLAB;     // payload
  static constexpr int STRIDE = ROW_BYTES + (KMAJOR ? 64 : 16);                  // padded
  static constexpr int BYTES = ROWS * STRIDE;
  static constexpr int CHUNKS_PER_ROW = ROW_BYTES / 16;
  static constexpr int CHUNKS = ROWS * CHUNKS_PER_ROW;                           // 16-byte chunks
};

template <typename T, int BM_, int BN_, int WM_, int WN_, bool AKM, bool BKM, int SLAB = 128>
struct TileCfg {
  using elem = T;
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr bool A_KMAJOR = AKM, B_KMAJOR = BKM;
  static constexpr int BK = SLAB / (int)sizeof(T);   // reduction steps per slab
  static constexpr int GROUPS = SLAB / 32;           // reduction groups (fragment reads) per slab
  static constexpr int THREADS = WM * WN * 64;
  static constexpr int WTM = BM / WM, WTN = BN / WN;       // tile of one wavefront
  static constexpr int TM = WTM / 32, TN = WTN / 32;       // 32x32 blocks per wavefront
  using LA = OperandLds<T, BM, AKM, SLAB>;
  using LB = OperandLds<T, BN, BKM, SLAB>;
  static constexpr int A_BYTES = LA::BYTES, B_BYTES = LB::BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int A_CHUNKS = LA::CHUNKS / THREADS;    // 16-byte chunks per thread per slab
  static constexpr int B_CHUNKS = LB::CHUNKS / THREADS;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be whole 32x32 blocks");
  static_assert(LA::CHUNKS % THREADS == 0 && LB::CHUNKS % THREADS == 0, "slab must divide evenly");
  static_assert(THREADS % LA::CHUNKS_PER_ROW == 0 && THREADS % LB::CHUNKS_PER_ROW == 0,
                "a staging pass must cover whole LDS rows");
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

// Global -> register -> LDS staging of one operand slab.  Thread t owns chunk (t % CPR) of LDS
// rows (t / CPR) + p * (THREADS / CPR), p = 0 .. NCH-1.  Addresses are a wave-uniform 64-bit
// base (tile, slab, pass) plus one 32-bit per-thread offset, which lets the loads use the
// scalar-base addressing form and keeps address registers out of the vector register budget.
template <typename T, class L, int THREADS, int NCH, bool KMAJOR>
struct Stager {
  const char* base;   // wave-uniform: first byte of the operand tile at the first k of the range
  uint32_t toff;      // this thread's byte offset from the pass base
  int64_t pass;       // global byte step between passes (uniform)
  int64_t slab;       // global byte step between slabs (uniform)
  int lds;            // this thread's first LDS byte offset inside the operand region
  static constexpr int RPP = THREADS / L::CHUNKS_PER_ROW;   // LDS rows per pass

  // tile: element (row 0 of the operand tile, first k of the range); ld in elements.
  __device__ __forceinline__ void init(const T* tile, int64_t ld) {
    const int t = threadIdx.x;
    const int row = t / L::CHUNKS_PER_ROW, ch = t % L::CHUNKS_PER_ROW;
    // k contiguous: LDS row = tile row, advancing a slab moves 128 bytes along the row.
    // k-major:      LDS row = reduction step, advancing a slab moves BK rows down.
    base = reinterpret_cast<const char*>(tile);
    toff = (uint32_t)((int64_t)row * ld * (int64_t)sizeof(T) + ch * 16);
    pass = (int64_t)RPP * ld * (int64_t)sizeof(T);
    slab = KMAJOR ? (int64_t)L::BK * ld * (int64_t)sizeof(T) : (int64_t)L::SLAB_BYTES;
    lds = row * L::STRIDE + ch * 16;
  }
  // The chunks of one slab live in ONE vector value (not an array), so they are registers by
  // construction whatever the control flow around the loads.
  typedef uint32_t Regs __attribute__((ext_vector_type(NCH * 4)));
  __device__ __forceinline__ Regs load(int s) const {
    const char* sb = base + (int64_t)s * slab;
    Regs r;
#pragma unroll
    for (int p = 0; p < NCH; ++p) {
      const u32x4 t = *reinterpret_cast<const u32x4*>(sb + p * pass + toff);
      r[4 * p + 0] = t[0]; r[4 * p + 1] = t[1]; r[4 * p + 2] = t[2]; r[4 * p + 3] = t[3];
    }
    return r;
  }
  // chunk p of slab s alone (lets the caller spread the loads of a slab between its MFMAs)
  __device__ __forceinline__ void load_chunk(int s, int p, Regs& r) const {
    const u32x4 t = *reinterpret_cast<const u32x4*>(base + (int64_t)s * slab + p * pass + toff);
    r[4 * p + 0] = t[0]; r[4 * p + 1] = t[1]; r[4 * p + 2] = t[2]; r[4 * p + 3] = t[3];
  }
  __device__ __forceinline__ void store(char* region, const Regs& r) const {
#pragma unroll
    for (int p = 0; p < NCH; ++p) {
      u32x4 t;
      t[0] = r[4 * p + 0]; t[1] = r[4 * p + 1]; t[2] = r[4 * p + 2]; t[3] = r[4 * p + 3];
      *reinterpret_cast<u32x4*>(region + lds + p * RPP * L::STRIDE) = t;
    }
  }
};

// One 16-byte MFMA fragment of 32 tile rows starting at row `r0`, reduction group `g`
// (16 steps for bf16, 8 for fp32), from an operand slab in LDS.
template <typename T, class L, bool KMAJOR>
__device__ __forceinline__ u32x4 read_frag(const char* region, int r0, int g) {
  const int lane = threadIdx.x & 63;
  if constexpr (!KMAJOR) {
    return *reinterpret_cast<const u32x4*>(region + (r0 + (lane & 31)) * L::STRIDE + g * 32 +
                                           (lane >> 5) * 16);
  } else if constexpr (sizeof(T) == 2) {
    // ds_read_b64_tr_b16: inside each group of 16 lanes, lane s addresses the 4 consecutive tile
    // rows r0' + 4*(s%4).. of reduction step k0 + s/4, and lane i receives tile row r0' + i for
    // the 4 steps k0..k0+3.  Lane groups: (rows 0..15 | 16..31) x (first | second half of the group).
    const int grp = lane >> 4, s = lane & 15;
    const int k0 = g * 16 + (grp >> 1) * 8 + (s >> 2);
    const int col = r0 + (grp & 1) * 16 + (s & 3) * 4;
    const char* p = region + k0 * L::STRIDE + col * 2;
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * L::STRIDE));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    u32x4 r;
    r[0] = l2[0]; r[1] = l2[1]; r[2] = h2[0]; r[3] = h2[1];
    return r;
  } else {
    // fp32: four scalar reads, reduction steps g*8 + half*4 + 0..3 of tile row r0 + lane%32
    const char* p = region + (g * 8 + (lane >> 5) * 4) * L::STRIDE + (r0 + (lane & 31)) * 4;
    u32x4 r;
    r[0] = *reinterpret_cast<const uint32_t*>(p);
    r[1] = *reinterpret_cast<const uint32_t*>(p + L::STRIDE);
    r[2] = *reinterpret_cast<const uint32_t*>(p + 2 * L::STRIDE);
    r[3] = *reinterpret_cast<const uint32_t*>(p + 3 * L::STRIDE);
    return r;
  }
}

// The MFMA fragments of one reduction group for a whole wavefront tile.
template <class Cfg>
struct Frags {
  u32x4 a[Cfg::TM];
  u32x4 b[Cfg::TN];
};

template <class Cfg>
__device__ __forceinline__ void read_group(const char* stage, int g, int wm, int wn,
                                           Frags<Cfg>& f) {
  using T = typename Cfg::elem;
#pragma unroll
  for (int bm = 0; bm < Cfg::TM; ++bm)
    f.a[bm] = read_frag<T, typename Cfg::LA, Cfg::A_KMAJOR>(stage, wm * Cfg::WTM + bm * 32, g);
#pragma unroll
  for (int bn = 0; bn < Cfg::TN; ++bn)
    f.b[bn] = read_frag<T, typename Cfg::LB, Cfg::B_KMAJOR>(stage + Cfg::A_BYTES,
                                                            wn * Cfg::WTN + bn * 32, g);
}

template <class Cfg>
__device__ __forceinline__ void mma_group(const Frags<Cfg>& f, f32x16 (&acc)[Cfg::TM][Cfg::TN]) {
  using T = typename Cfg::elem;
#pragma unroll
  for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) mfma_group<T>(f.a[bm], f.b[bn], acc[bm][bn]);
}

// Accumulate acc += A_tile * B_tile^T over `nslabs` slabs of K.
//   A: element (first of this workgroup's BM tile rows, first reduction step of its range)
//   B: likewise for its BN tile rows;  lda / ldb in elements.
//   smem: Cfg::LDS_BYTES bytes, 16-byte aligned.  Ends with a barrier (smem may be reused).
// Software pipeline (two LDS stages, one register set, global loads two slabs ahead):
//   * at the top of iteration s the registers hold slab s+1, loaded during iteration s-1, so it
//     has had a whole iteration to arrive; it goes to the idle LDS stage at once, and the barrier
//     at the end of the iteration publishes it;
//   * the loads of slab s+2 then refill the registers, issued one at a time between the MFMAs of
//     the first groups: a wavefront that issues a whole slab in one burst queues up at the
//     memory pipe (measured: up to 1400 cycles) with its MFMAs stuck behind the loads;
//   * inside a slab the fragments of group g+1 are read from LDS while group g is multiplied;
//   * the last group of a slab is multiplied AFTER the barrier, behind the first fragment reads
//     of the next slab, so the LDS latency at the slab boundary is covered as well.
// Slab numbers past the end are clamped to the last slab: such loads and LDS stores are
// redundant but in bounds, and keep the loop body free of branches.
template <class Cfg>
__device__ __forceinline__ void gemm_tile(const typename Cfg::elem* __restrict__ A, int64_t lda,
                                          const typename Cfg::elem* __restrict__ B, int64_t ldb,
                                          int nslabs, char* smem,
                                          f32x16 (&acc)[Cfg::TM][Cfg::TN]) {
  using T = typename Cfg::elem;
  using LA = typename Cfg::LA;
  using LB = typename Cfg::LB;
  const int wave = threadIdx.x >> 6;
  const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;

  typedef Stager<T, LA, Cfg::THREADS, Cfg::A_CHUNKS, Cfg::A_KMAJOR> SA;
  typedef Stager<T, LB, Cfg::THREADS, Cfg::B_CHUNKS, Cfg::B_KMAJOR> SB;
  SA sa;
  SB sb;
  sa.init(A, lda);
  sb.init(B, ldb);
  char* st0 = smem;
  char* st1 = smem + Cfg::STAGE_BYTES;
  const int last = nslabs - 1;
  constexpr int NA = Cfg::A_CHUNKS, NL = Cfg::A_CHUNKS + Cfg::B_CHUNKS;
  constexpr int MM = Cfg::TM * Cfg::TN;            // MFMAs per group
  constexpr int HEAD = Cfg::GROUPS - 1;            // groups multiplied before the barrier
  // the loads of a slab are placed in front of the MFMAs of the first one or two groups (of all
  // groups before the barrier if two do not have an MFMA for each load)
  constexpr int SPAN = (NL <= 2 * MM ? (HEAD < 2 ? HEAD : 2) : HEAD) * MM;
  static_assert(HEAD >= 1 && NL <= SPAN, "one load per MFMA slot at most");

  // prologue: slabs 0 and 1 are requested back to back; slab 0 goes to stage 0
  typename SA::Regs a0 = {};
  typename SB::Regs b0 = {};
  {
    typename SA::Regs af = sa.load(0);
    typename SB::Regs bf = sb.load(0);
    a0 = sa.load(last < 1 ? last : 1);
    b0 = sb.load(last < 1 ? last : 1);
    sa.store(st0, af);
    sb.store(st0 + Cfg::A_BYTES, bf);
  }
  __syncthreads();
  Frags<Cfg> fc;
  read_group<Cfg>(st0, 0, wm, wn, fc);
  for (int s = 0; s < nslabs; ++s) {
    char* cur = (s & 1) ? st1 : st0;
    char* nxt = (s & 1) ? st0 : st1;
    const int s2 = s + 2 < last ? s + 2 : last;
    sa.store(nxt, a0);
    sb.store(nxt + Cfg::A_BYTES, b0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < HEAD; ++g) {
      Frags<Cfg> fn;
      read_group<Cfg>(cur, g + 1, wm, wn, fn);
      __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs they do not feed
#pragma unroll
      for (int q = 0; q < MM; ++q) {
#pragma unroll
        for (int c = 0; c < NL; ++c) {     // chunk c is requested in front of MFMA c*SPAN/NL
          if (c * SPAN / NL == g * MM + q) {
            if (c < NA) sa.load_chunk(s2, c, a0);
            else sb.load_chunk(s2, c - NA, b0);
          }
        }
        mfma_group<T>(fc.a[q / Cfg::TN], fc.b[q % Cfg::TN], acc[q / Cfg::TN][q % Cfg::TN]);
      }
      __builtin_amdgcn_sched_barrier(0);
      fc = fn;
    }
    __syncthreads();
    Frags<Cfg> fn;
    read_group<Cfg>(nxt, 0, wm, wn, fn);
    __builtin_amdgcn_sched_barrier(0);
    mma_group<Cfg>(fc, acc);
    __builtin_amdgcn_sched_barrier(0);
    fc = fn;
  }
  __syncthreads();
}

template <class Cfg>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[Cfg::TM][Cfg::TN]) {
#pragma unroll
  for (int a = 0; a < Cfg::TM; ++a)
#pragma unroll
    for (int b = 0; b < Cfg::TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
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
// that land on one XCD.  This is done for the outer indices that form whole groups of 8; the
// remaining outer % 8 (all of them when outer < 8) are laid out plainly, inner index fastest, so
// that their workgroups spread over all XCDs instead of filling outer % 8 of them.  The grid is
// exactly inner * outer workgroups; returns false for ids beyond it.
__device__ __forceinline__ bool xcd_tile(int wg, int inner, int outer, int& o, int& i) {
  const int full = outer & ~7;
  if (wg < full * inner) {
    const int xcd = wg & 7, local = wg >> 3;
    o = (local / inner) * 8 + xcd;
    i = local % inner;
  } else {
    const int t = wg - full * inner;
    o = full + t / inner;
    i = t % inner;
  }
  return o < outer;
}
inline int xcd_grid(int inner, int outer) { return inner * outer; }

}  // namespace pfc
