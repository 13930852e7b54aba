// pfc_forward_backward: margin-softmax loss over the sampled centers and its gradients
// (arXiv 2203.15565: Eq. 1 restricted to the sampled set S as in Eq. 4; Eq. 2 / Eq. 4 for the
// feature gradient, the bracket of Eq. 3 for the center gradient).
//
// Pipeline (one stream, no host synchronisation):
//   normalize_x        Xn = x/|x|                                   (HBM bound, tiny)
//   gather_normalize_w Wn = W[idx]/|W[idx]|                         (HBM bound)
//   gemm_logits        c = Wn Xn^T, margin, e = exp(s c) -> E and per-tile row sums (MFMA)
//   row_combine        l_i, lse_i, per-row loss, s/(B l_i), label-column coefficient,
//                      Xs = (s/(B l_i)) xn_i
//   gemm_dweight       dWn = E^T Xs  (off-label part)                (MFMA)
//   dweight_label      adds the label-column term to the rows of positive classes (fp32)
//   gemm_dfeatures     partial sums of E Wn over slices of S         (MFMA, split over S)
//   dfeatures_final    reduce slices, scale, label term, project through x -> x/|x|; mean loss
//
// Cosines lie in [-1,1]: up to s = 64, exp(s c) lies in [e^-64, e^64] and a row sum over at most
// 2^31 classes stays below 3.4e38, so exp needs no running maximum and one fixed reference (zero)
// serves every tile, p_ij = E_ij / l_i with l_i known only after the GEMM.  Above s = 64 one more
// pass of the logit GEMM (gemm_rowmax, row_ref) finds each sample's largest logit first and the
// softmax runs relative to it.
// The label column is kept out of E (stored as zero) and handled in fp32 on the side, where
// (p - 1) and the margin derivative are formed without bf16 rounding.
#include <limits.h>
#include <math.h>

#include <type_traits>

#include "pfc_common.h"
#include "pfc_gemm.h"

// Phase clocks for tuning, compiled in only with -DPFC_PHASES (never in the shipped library):
// thread 0 of every workgroup of the selected kernel stores the constant-rate clock at up to 8
// points.  Kernel tags: 1 logits, 2 dweight, 3 dweight+update.
#ifdef PFC_PHASES
__device__ unsigned long long pfc_phase_buf[32768 * 8];
__device__ int pfc_phase_sel;
#define PFC_PHASE(tag, slot)                                                               \
  do {                                                                                     \
    if (threadIdx.x == 0 && blockIdx.x < 32768 && pfc_phase_sel == (tag))                  \
      pfc_phase_buf[blockIdx.x * 8 + (slot)] = __builtin_amdgcn_s_memrealtime();               \
  } while (0)
extern "C" int pfc_debug_phases(unsigned long long* host_out, int n) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(pfc_phase_buf), (size_t)n * 8);
}
extern "C" int pfc_debug_select(int tag) {
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(pfc_phase_buf)) != hipSuccess) return -1;
  if (hipMemset(p, 0, sizeof(unsigned long long) * 32768 * 8) != hipSuccess) return -2;
  return (int)hipMemcpyToSymbol(HIP_SYMBOL(pfc_phase_sel), &tag, sizeof(int));
}
#else
#define PFC_PHASE(tag, slot)
#endif

namespace pfc {

namespace {

constexpr float kEpsNorm = 1e-12f;
constexpr float kEpsSin2 = 1e-12f;

// ---------------------------------------------------------------------------------------------
// normalize_x: one wavefront per (padded) feature row.
//
// Row length: the caller's arrays (X, W, v, dX, dWn) have rows of D floats, D a multiple of 64.
// The library's own GEMM operands (Xn, Xs, Wn and the dfeatures partial sums) have rows of
// Dp = 256 * NC >= D elements, the columns from D on being zero, so that the GEMMs only ever
// see whole 256-column tiles; kernels that touch the caller's rows skip the columns from D on.
// ---------------------------------------------------------------------------------------------
template <typename T, int NC>
__global__ void normalize_x_kernel(const float* __restrict__ X, int B, int Bp, int D,
                                   const int32_t* __restrict__ yl, int64_t k, T* __restrict__ Xn,
                                   float* __restrict__ rnormX, float* __restrict__ clabel,
                                   int32_t* __restrict__ err_flag) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= Bp) return;
  constexpr int nchunk = NC;   // float4 chunks per lane
  constexpr int Dp = 256 * NC;
  float4 v[NC];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < nchunk; ++c) {
    const int d = c * 256 + lane * 4;
    v[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < B && d < D) v[c] = *reinterpret_cast<const float4*>(X + (int64_t)i * D + d);
    ss += v[c].x * v[c].x + v[c].y * v[c].y + v[c].z * v[c].z + v[c].w * v[c].w;
  }
  ss = wave_sum(ss);
  const float rn = (i < B) ? 1.f / fmaxf(sqrtf(ss), kEpsNorm) : 0.f;
#pragma unroll
  for (int c = 0; c < nchunk; ++c) {
    T* dst = Xn + (int64_t)i * Dp + c * 256 + lane * 4;   // rn == 0 for padded rows
    dst[0] = from_float<T>(v[c].x * rn);
    dst[1] = from_float<T>(v[c].y * rn);
    dst[2] = from_float<T>(v[c].z * rn);
    dst[3] = from_float<T>(v[c].w * rn);
  }
  if (lane == 0) {
    rnormX[i] = rn;
    clabel[i] = 0.f;
    if (i < B) {
      const int32_t y = yl[i];
      if (y < 0 || (int64_t)y >= k) atomicOr(err_flag, 2);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// gather_normalize_w: one wavefront per group of NB consecutive sampled rows, all NB row reads
// (2 KB each at D = 512, ascending row ids) in flight before the first is reduced.
// Rows k..kp-1 of Wn are written as zeros.
// ---------------------------------------------------------------------------------------------
template <typename T, int NC>
__global__ void gather_normalize_w_kernel(const float* __restrict__ W, int64_t N,
                                          const int32_t* __restrict__ idx, int64_t k, int64_t kp,
                                          int D, T* __restrict__ Wn, float* __restrict__ rnormW,
                                          int32_t* __restrict__ head, int nwin,
                                          int32_t* __restrict__ err_flag) {
  constexpr int NB = 4;
  constexpr int Dp = 256 * NC;
  const int lane = threadIdx.x & 63;
  const int64_t jb = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * NB;
  if (jb >= kp) return;
  float4 v[NB][NC];
  bool ok[NB];
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    const int64_t j = jb + u;
    ok[u] = false;
    if (j < k) {
      const int64_t row = idx[j];
      ok[u] = (row >= 0 && row < N);
      if (!ok[u] && lane == 0) atomicOr(err_flag, 4);
      if (ok[u]) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          // streamed once: a nontemporal load keeps these rows from displacing what the GEMMs
          // that follow want in the L2 (measured: 0.145 -> 0.121 ms at the headline workload)
          const int d = c * 256 + lane * 4;
          v[u][c] = make_float4(0.f, 0.f, 0.f, 0.f);
          if (d < D) {
            const f32x4 t =
                __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(W + row * D + d));
            v[u][c] = make_float4(t[0], t[1], t[2], t[3]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    const int64_t j = jb + u;
    if (j >= kp) break;
    float ss = 0.f;
    if (ok[u]) {
#pragma unroll
      for (int c = 0; c < NC; ++c)
        ss += v[u][c].x * v[u][c].x + v[u][c].y * v[u][c].y + v[u][c].z * v[u][c].z +
              v[u][c].w * v[u][c].w;
    }
    ss = wave_sum(ss);
    const float rn = ok[u] ? 1.f / fmaxf(sqrtf(ss), kEpsNorm) : 0.f;
    if (lane == 0) {
      rnormW[j] = rn;
      head[j] = 0x7fffffff;   // first sample carrying this class: filled in by row_combine
    }
    // likewise the first sample of every window of kLabelWindow samples (large batches only)
    if (lane < nwin) head[(int64_t)(1 + lane) * kp + j] = 0x7fffffff;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      T o[4];
      if (ok[u]) {
        o[0] = from_float<T>(v[u][c].x * rn);
        o[1] = from_float<T>(v[u][c].y * rn);
        o[2] = from_float<T>(v[u][c].z * rn);
        o[3] = from_float<T>(v[u][c].w * rn);
      } else {
        o[0] = o[1] = o[2] = o[3] = from_float<T>(0.f);
      }
      T* g = Wn + j * Dp + c * 256 + lane * 4;
      if constexpr (sizeof(T) == 2) {
        uint2 pk;
        __builtin_memcpy(&pk, o, 8);
        *reinterpret_cast<uint2*>(g) = pk;
      } else {
        float4 f4;
        f4.x = (float)o[0]; f4.y = (float)o[1]; f4.z = (float)o[2]; f4.w = (float)o[3];
        *reinterpret_cast<float4*>(g) = f4;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// gemm_logits: tile of c[j][i] (rows = sampled classes, columns = samples), fused epilogue:
// clamp, margin on the label entry, e = exp(s*c), per-tile column sums, and E[i][j] = e (label
// entry and padding stored as zero).  A lane holds one sample i and runs of 4 consecutive
// classes j, so the sums over j are in-lane; the bf16 tile is transposed through LDS so that E
// is written in whole 512-byte rows.
//
// The element-wise part exists in four versions.  GUARDED: the wavefront's part of the tile holds
// a label entry or padding (few wavefronts do); the plain version costs 5 VALU instructions per
// entry.  EXTRAS: the options are on -- negatives whose cosine exceeds `tau` are left out of the
// softmax (the PFC* filter, Sec. 3.3 / Fig. 4 caption) and the largest non-label cosine of every
// sample is tracked (for AMNCS, Sec. 3.3).
// ---------------------------------------------------------------------------------------------
struct LossParams {
  float s, s_log2e;
  float m, cos_m, sin_m;
  int32_t cosface;   // 0: label logit s*cos(theta+m); 1: s*(cos(theta) - m)
  float tau;         // filter threshold (entries with cosine > tau are dropped); >= 1: off
  int32_t extras;    // filter, column maxima and/or a per-sample reference requested
  const float* rowref;   // [Bp] largest logit of every sample, or null: exp(z - rowref_i) instead
                         // of exp(z) (scales above 64, where exp(z) could leave the fp32 range)
};

__device__ __forceinline__ float label_logit(const LossParams& lp, float c) {
  if (lp.cosface) return lp.s * (c - lp.m);
  return lp.s * (c * lp.cos_m - sqrtf(fmaxf(1.f - c * c, 0.f)) * lp.sin_m);
}

template <class Cfg, bool GUARDED, bool EXTRAS>
__device__ __forceinline__ void logits_epilogue_columns(
    const f32x16 (&acc)[Cfg::TM][Cfg::TN], int64_t j0, int i0, int B, int klim, int64_t kp,
    const int (&ylane)[Cfg::TN], const LossParams& lp, char* smem, int SX,
    typename Cfg::elem* __restrict__ E, float* __restrict__ clabel, float (&colsum)[Cfg::TN],
    float (&colmax)[Cfg::TN]) {
  using T = typename Cfg::elem;
  constexpr bool kStage = (sizeof(T) == 2);
#pragma unroll
  for (int bn = 0; bn < Cfg::TN; ++bn) {
    const int il = acc_col<Cfg>(bn);
    const int i = i0 + il;
    const bool vi = i < B;
    const int yloc = ylane[bn];
    float sum = 0.f, clab = 0.f, cmax = -2.f;
    float ref = 0.f;
    if constexpr (EXTRAS) ref = lp.rowref ? lp.rowref[i] : 0.f;   // i < Bp: padded entries are 0
    const float ref2 = ref * 1.44269504088896340736f;
#pragma unroll
    for (int bm = 0; bm < Cfg::TM; ++bm) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        T pack[4];
        const int jl = acc_row<Cfg>(bm, g4 * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float c = __builtin_amdgcn_fmed3f(acc[bm][bn][g4 * 4 + e], -1.f, 1.f);
          // exp(s*c), |s*c*log2(e)| <= 93 without a reference; exp(s*c - ref) <= 1 with one
          float ev = EXTRAS ? __builtin_amdgcn_exp2f(fmaf(c, lp.s_log2e, -ref2))
                            : __builtin_amdgcn_exp2f(c * lp.s_log2e);
          if constexpr (GUARDED) {
            const bool lab = (jl + e == yloc);
            const bool neg = vi && jl + e < klim && !lab;      // a real, non-label entry
            ev = neg ? ev : 0.f;
            clab = lab ? c : clab;
            if constexpr (EXTRAS) {
              cmax = neg ? fmaxf(cmax, c) : cmax;
              ev = (c > lp.tau) ? 0.f : ev;
            }
          } else if constexpr (EXTRAS) {
            cmax = fmaxf(cmax, c);
            ev = (c > lp.tau) ? 0.f : ev;
          }
          sum += ev;
          pack[e] = from_float<T>(ev);
        }
        if constexpr (kStage) {
          uint2 pk;
          __builtin_memcpy(&pk, pack, 8);
          *reinterpret_cast<uint2*>(smem + il * SX + jl * 2) = pk;
        } else {
          uint4 pk;
          __builtin_memcpy(&pk, pack, 16);
          *reinterpret_cast<uint4*>(E + (int64_t)i * kp + j0 + jl) = pk;
        }
      }
    }
    if constexpr (GUARDED) {
      if (yloc >= 0) {   // this lane holds sample i's label entry: it was left out of `sum`
        clabel[i] = clab;
        sum += __expf(label_logit(lp, clab) - ref);
      }
    }
    sum += __shfl_xor(sum, 32, 64);
    colsum[bn] = sum;
    if constexpr (EXTRAS) colmax[bn] = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
  }
}

template <class Cfg, bool EXTRAS>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_logits_kernel(
    const typename Cfg::elem* __restrict__ Wn, const typename Cfg::elem* __restrict__ Xn, int D,
    int64_t k, int B, int Bp, int64_t kp, const int32_t* __restrict__ yl, LossParams lp,
    typename Cfg::elem* __restrict__ E, float* __restrict__ rowpart,
    float* __restrict__ rowmaxpart, float* __restrict__ clabel, int tiles_j, int tiles_i,
    int ahead) {
  using T = typename Cfg::elem;
  extern __shared__ __align__(16) char smem[];
  int tj, ti;
  if (!xcd_tile(blockIdx.x, tiles_i, tiles_j, tj, ti)) return;
  const int64_t j0 = (int64_t)tj * Cfg::BM;
  const int i0 = ti * Cfg::BN;

  f32x16 acc[Cfg::TM][Cfg::TN];
  zero_acc<Cfg>(acc);
  PFC_PHASE(1, 0);
  gemm_tile<Cfg>(Wn + j0 * D, D, Xn + (int64_t)i0 * D, D, D / Cfg::BK, smem, acc);
  PFC_PHASE(1, 1);
  // Pull the Wn block of the class tile that the workgroups `ahead` ids later will multiply (same
  // XCD, about one round later) into this XCD's L2: the tiles_i workgroups of a class tile touch
  // a part of the rows each, one 4-byte load per 128-byte line.  The values are only kept alive
  // until the end of the kernel, never used.
  uint32_t touched = 0;
  {
    int ntj, nti;
    const int nb = (int)blockIdx.x + ahead;
    if (nb < (int)gridDim.x && (int)(threadIdx.x >> 1) < Cfg::BM &&
        xcd_tile(nb, tiles_i, tiles_j, ntj, nti)) {
      const int row_bytes = D * (int)sizeof(T);
      const int off = ((nti * 256) % row_bytes) + (threadIdx.x & 1) * 128;
      const char* p = reinterpret_cast<const char*>(Wn + (int64_t)ntj * Cfg::BM * D) +
                      (int64_t)(threadIdx.x >> 1) * row_bytes + off;
      touched = *reinterpret_cast<const uint32_t*>(p);
    }
    __builtin_amdgcn_sched_barrier(0);
  }

  constexpr bool kStage = (sizeof(T) == 2);          // bf16: transpose the tile through LDS
  constexpr int SX = Cfg::BM * 2 + 8;                // staging row (one sample) stride in bytes
  constexpr int RED_OFF = Cfg::BN * SX;              // cross-wave reduction scratch behind it
  static_assert(RED_OFF + 2 * Cfg::WM * Cfg::BN * 4 <= Cfg::LDS_BYTES, "epilogue LDS");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t krem = k - j0;
  const int klim = krem < (int64_t)Cfg::BM ? (int)krem : Cfg::BM;   // valid classes in this tile

  // ylane[bn]: tile row of sample i's label entry if THIS lane holds it, else -1.  A lane holds
  // the rows  wm*WTM + bm*32 + (r/4)*8 + half*4 + r%4.
  int ylane[Cfg::TN];
  bool any_label = false;
#pragma unroll
  for (int bn = 0; bn < Cfg::TN; ++bn) {
    const int i = i0 + acc_col<Cfg>(bn);
    ylane[bn] = -1;
    if (i < B) {
      const int64_t y = (int64_t)yl[i] - j0;
      if (y >= 0 && y < (int64_t)klim) {
        const int rel = (int)y - (wave / Cfg::WN) * Cfg::WTM;
        if (rel >= 0 && rel < Cfg::WTM && ((rel >> 2) & 1) == (lane >> 5)) ylane[bn] = (int)y;
      }
    }
    any_label = any_label || (ylane[bn] >= 0);
  }
  const bool guarded = __any(any_label) || klim < Cfg::BM || i0 + Cfg::BN > B;   // wave-uniform

  float colsum[Cfg::TN], colmax[Cfg::TN];
#pragma unroll
  for (int bn = 0; bn < Cfg::TN; ++bn) colmax[bn] = -2.f;
  if (guarded)
    logits_epilogue_columns<Cfg, true, EXTRAS>(acc, j0, i0, B, klim, kp, ylane, lp, smem, SX, E,
                                               clabel, colsum, colmax);
  else
    logits_epilogue_columns<Cfg, false, EXTRAS>(acc, j0, i0, B, klim, kp, ylane, lp, smem, SX, E,
                                                clabel, colsum, colmax);

  PFC_PHASE(1, 2);
  // cross-wave reduction over the WM wavefronts that share a column (fixed order)
  float* red = reinterpret_cast<float*>(smem + RED_OFF);   // [WM][BN] sums, then [WM][BN] maxima
  if (lane < 32) {
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) {
      const int o = (wave / Cfg::WN) * Cfg::BN + (wave % Cfg::WN) * Cfg::WTN + bn * 32 + lane;
      red[o] = colsum[bn];
      red[Cfg::WM * Cfg::BN + o] = colmax[bn];
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < Cfg::BN; t += Cfg::THREADS) {
    float v = 0.f, mx = -2.f;
#pragma unroll
    for (int w = 0; w < Cfg::WM; ++w) {
      v += red[w * Cfg::BN + t];
      mx = fmaxf(mx, red[Cfg::WM * Cfg::BN + w * Cfg::BN + t]);
    }
    rowpart[(int64_t)(i0 + t) * tiles_j + tj] = v;
    if constexpr (EXTRAS) rowmaxpart[(int64_t)(i0 + t) * tiles_j + tj] = mx;
  }
  if constexpr (kStage) {
    // whole rows of the tile (BM * 2 bytes, 8 per lane) leave in one piece
    constexpr int LPR = Cfg::BM / 4;        // lanes per tile row
    constexpr int RPW = 64 / LPR;           // tile rows per wavefront instruction
    static_assert(LPR <= 64 && 64 % LPR == 0, "row write-out: 4 classes per lane");
    const int sub = lane / LPR, l = lane % LPR;
    for (int row = wave * RPW + sub; row < Cfg::BN; row += (Cfg::THREADS / 64) * RPW) {
      const uint2 v = *reinterpret_cast<const uint2*>(smem + row * SX + l * 8);
      // E is far larger than the L2 and next read by another kernel: store it nontemporally
      // (measured: 0.320 -> 0.302 ms for this kernel at the headline workload)
      __builtin_nontemporal_store(__builtin_bit_cast(u32x2, v),
                                  reinterpret_cast<u32x2*>(E + (int64_t)(i0 + row) * kp + j0 + l * 4));
    }
  }
  PFC_PHASE(1, 3);
  asm volatile("" ::"v"(touched));
}

// ---------------------------------------------------------------------------------------------
// gemm_rowmax (scales above 64 only): the logits GEMM once more, in front of gemm_logits, with an
// epilogue that keeps nothing but the largest logit of every sample in every tile (label entry
// with its margin); row_ref reduces the tiles.  The softmax then runs relative to that maximum,
// as an online softmax would, and works for any scale; at s <= 64 a zero reference is exact as
// well and this pass is skipped.
// ---------------------------------------------------------------------------------------------
template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_rowmax_kernel(
    const typename Cfg::elem* __restrict__ Wn, const typename Cfg::elem* __restrict__ Xn, int D,
    int64_t k, int B, const int32_t* __restrict__ yl, LossParams lp,
    float* __restrict__ rowmaxpart, int tiles_j, int tiles_i) {
  extern __shared__ __align__(16) char smem[];
  int tj, ti;
  if (!xcd_tile(blockIdx.x, tiles_i, tiles_j, tj, ti)) return;
  const int64_t j0 = (int64_t)tj * Cfg::BM;
  const int i0 = ti * Cfg::BN;
  f32x16 acc[Cfg::TM][Cfg::TN];
  zero_acc<Cfg>(acc);
  gemm_tile<Cfg>(Wn + j0 * D, D, Xn + (int64_t)i0 * D, D, D / Cfg::BK, smem, acc);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t krem = k - j0;
  const int klim = krem < (int64_t)Cfg::BM ? (int)krem : Cfg::BM;
  float* red = reinterpret_cast<float*>(smem);   // [WM][BN]
#pragma unroll
  for (int bn = 0; bn < Cfg::TN; ++bn) {
    const int i = i0 + acc_col<Cfg>(bn);
    const int yloc = i < B ? (int)((int64_t)yl[i] - j0) : -1;   // tile row of the label entry
    float zmax = -3.0e38f;
#pragma unroll
    for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int jl = acc_row<Cfg>(bm, r);
        const float c = __builtin_amdgcn_fmed3f(acc[bm][bn][r], -1.f, 1.f);
        const bool lab = jl == yloc;
        const float z = lab ? label_logit(lp, c) : lp.s * c;
        // entries the filter leaves out of the softmax do not count (the label is never filtered)
        const bool in = i < B && jl < klim && (lab || !(c > lp.tau));
        zmax = in ? fmaxf(zmax, z) : zmax;
      }
    zmax = fmaxf(zmax, __shfl_xor(zmax, 32, 64));
    if (lane < 32)
      red[(wave / Cfg::WN) * Cfg::BN + (wave % Cfg::WN) * Cfg::WTN + bn * 32 + lane] = zmax;
  }
  __syncthreads();
  for (int t = threadIdx.x; t < Cfg::BN; t += Cfg::THREADS) {
    float mx = -3.0e38f;
#pragma unroll
    for (int w = 0; w < Cfg::WM; ++w) mx = fmaxf(mx, red[w * Cfg::BN + t]);
    rowmaxpart[(int64_t)(i0 + t) * tiles_j + tj] = mx;
  }
}

// rowref[i] = max over the tiles of sample i (0 for padded samples); one wavefront per sample.
__global__ void row_ref_kernel(const float* __restrict__ rowmaxpart, int tiles_j, int B, int Bp,
                               float* __restrict__ rowref) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= Bp) return;
  float mx = -3.0e38f;
  if (i < B)
    for (int t = lane; t < tiles_j; t += 64) mx = fmaxf(mx, rowmaxpart[(int64_t)i * tiles_j + t]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if (lane == 0) rowref[i] = i < B ? mx : 0.f;
}

// ---------------------------------------------------------------------------------------------
// row_combine: one wavefront per (padded) sample.  l_i = sum of the per-tile partial sums (lane
// strided, then a fixed shuffle tree: the same order on every run), the per-row scalars, and the
// row of Xs = (s/(B l_i)) * x_i/|x_i| that feeds the dweight GEMM (zero for padded rows).
// ---------------------------------------------------------------------------------------------
template <typename T, int NC>
__global__ void row_combine_kernel(const float* __restrict__ rowpart, int tiles_j, int B, int Bp,
                                   int D, const float* __restrict__ X,
                                   const float* __restrict__ rnormX,
                                   const float* __restrict__ clabel, LossParams lp,
                                   const float* __restrict__ rowmaxpart,
                                   float* __restrict__ rowscale, float* __restrict__ dlabel,
                                   float* __restrict__ lossrow, float* __restrict__ rowmax,
                                   const int32_t* __restrict__ yl, int64_t k, int64_t kp,
                                   int32_t* __restrict__ head, int nwin, T* __restrict__ Xs) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= Bp) return;
  float scale = 0.f;
  if (i < B) {
    float l = 0.f;
    for (int t = lane; t < tiles_j; t += 64) l += rowpart[(int64_t)i * tiles_j + t];
    l = wave_sum(l);
    scale = (lp.s / (float)B) / l;   // B * l could leave the fp32 range, s/B never does
    float mx = -2.f;
    if (lp.extras) {
      for (int t = lane; t < tiles_j; t += 64) mx = fmaxf(mx, rowmaxpart[(int64_t)i * tiles_j + t]);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    }
    if (lane == 0) {
      const float c = clabel[i];
      const float sin2 = 1.f - c * c;
      const float zlab = label_logit(lp, c);
      const float ref = lp.rowref ? lp.rowref[i] : 0.f;   // l is the sum of exp(z - ref)
      const float p = __expf(zlab - ref) / l;
      // d(label logit)/d cos / s: sin(theta+m)/sin(theta) for the angular margin, 1 for the cosine one
      const float rho = lp.cosface ? 1.f : lp.cos_m + c * lp.sin_m / sqrtf(fmaxf(sin2, kEpsSin2));
      lossrow[i] = (logf(l) + ref) - zlab;
      rowscale[i] = scale;
      dlabel[i] = (lp.s / (float)B) * (p - 1.f) * rho;
      rowmax[i] = mx;
      const int32_t y = yl[i];
      if (y >= 0 && (int64_t)y < k) {   // integer atomics: order-independent
        // A frequent class would bring thousands of atomics onto one word: look first (past the
        // L1, which may hold an old value; a value read too high only costs the atomic)
        int32_t* h = &head[y];
        if (__hip_atomic_load(h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > i) atomicMin(h, i);
        if (nwin) {
          h = &head[(int64_t)(1 + i / kLabelWindow) * kp + y];
          if (__hip_atomic_load(h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > i) atomicMin(h, i);
        }
      }
    }
  } else if (lane == 0) {
    lossrow[i] = 0.f;
    rowscale[i] = 0.f;
    dlabel[i] = 0.f;
    rowmax[i] = 0.f;
  }
  const float f = (i < B) ? rnormX[i] * scale : 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int d = c * 256 + lane * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < B && d < D) v = *reinterpret_cast<const float4*>(X + (int64_t)i * D + d);
    T o[4] = {from_float<T>(v.x * f), from_float<T>(v.y * f), from_float<T>(v.z * f),
              from_float<T>(v.w * f)};
    if constexpr (sizeof(T) == 2) {
      uint2 pk;
      __builtin_memcpy(&pk, o, 8);
      *reinterpret_cast<uint2*>(Xs + (int64_t)i * (256 * NC) + d) = pk;
    } else {
      uint4 pk;
      __builtin_memcpy(&pk, o, 16);
      *reinterpret_cast<uint4*>(Xs + (int64_t)i * (256 * NC) + d) = pk;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// gemm_dweight: dWn[j][d] = sum_i E[i][j] * Xs[i][d] (both operands k-major); rows j < k are
// written.  When k is small and the batch large (the regime without extra negatives, Sec. 3.3)
// there are too few tiles to fill the GPU: SPLIT cuts the batch (the reduction) into slices that
// write partial tiles, summed in fixed order by dweight_reduce.  Xs has rows of Dp elements; the
// partial tiles too; dWn (the caller's) has rows of D floats, columns from D on are not stored.
// ---------------------------------------------------------------------------------------------
template <class Cfg, bool SPLIT>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_dweight_kernel(
    const typename Cfg::elem* __restrict__ E, const typename Cfg::elem* __restrict__ Xs, int D,
    int Dp, int64_t k, int64_t kp, int Bp, float* __restrict__ out, int tiles_j, int tiles_d,
    int slabs_per, int splits) {
  extern __shared__ __align__(16) char smem[];
  int tj, td, sp = 0, ns = Bp / Cfg::BK;
  if constexpr (SPLIT) {
    int tile;
    if (!xcd_tile(blockIdx.x, tiles_j * tiles_d, splits, sp, tile)) return;
    tj = tile / tiles_d;
    td = tile % tiles_d;
    ns -= sp * slabs_per;
    if (ns > slabs_per) ns = slabs_per;
  } else {
    if (!xcd_tile(blockIdx.x, tiles_d, tiles_j, tj, td)) return;
  }
  const int64_t j0 = (int64_t)tj * Cfg::BM;
  const int d0 = td * Cfg::BN;
  const int64_t i0 = (int64_t)sp * slabs_per * Cfg::BK;   // first sample of this slice
  f32x16 acc[Cfg::TM][Cfg::TN];
  zero_acc<Cfg>(acc);
  PFC_PHASE(2, 0);
  gemm_tile<Cfg>(E + i0 * kp + j0, kp, Xs + i0 * Dp + d0, Dp, ns, smem, acc);
  PFC_PHASE(2, 1);
  float* dst = SPLIT ? out + (int64_t)sp * kp * Dp : out;
  const int ld = SPLIT ? Dp : D;
  auto store_tile = [&](auto guarded) {
    bool col_in[Cfg::TN];
#pragma unroll
    for (int bn = 0; bn < Cfg::TN; ++bn) col_in[bn] = !guarded.value || d0 + acc_col<Cfg>(bn) < D;
#pragma unroll
    for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t j = j0 + acc_row<Cfg>(bm, r);
        if (SPLIT || j < k) {
#pragma unroll
          for (int bn = 0; bn < Cfg::TN; ++bn)
            if (col_in[bn]) dst[j * ld + d0 + acc_col<Cfg>(bn)] = acc[bm][bn][r];
        }
      }
  };
  // only the last column tile of a D that is no multiple of the tile width needs the guard
  if (SPLIT || d0 + Cfg::BN <= D)
    store_tile(std::false_type{});
  else
    store_tile(std::true_type{});
  PFC_PHASE(2, 2);
}

// dW[j][d] = sum over slices of part[slice][j][d], in slice order (rows of Dp floats in `part`, of
// D floats in dW).
__global__ void dweight_reduce_kernel(const float* __restrict__ part, int splits, int64_t k,
                                      int64_t kp, int D, int Dp, float* __restrict__ dW) {
  const int64_t e4 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e4 >= k * D / 4) return;
  const int64_t j = e4 / (D / 4);
  const int d = (int)(e4 - j * (D / 4)) * 4;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sp = 0; sp < splits; ++sp) {
    const float4 t =
        *reinterpret_cast<const float4*>(part + ((int64_t)sp * kp + j) * Dp + d);
    a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
  }
  *reinterpret_cast<float4*>(dW + e4 * 4) = a;
}

// dweight_label: dWn[y] += sum over samples i with label y of dlabel_i * xn_i.
// Block i does the whole sum for its class if i is the first sample carrying that label
// (head[y] == i, found with an integer atomicMin by row_combine).  The
// matching samples are listed in ascending order; thread group g (one float4 column per thread)
// sums the matches whose ordinal is congruent to g, and the groups are combined in fixed order,
// so the result does not depend on timing.
// LABEL_COMPACT (fused step): the sum is not added to dWn[y] but written to row i of a B x D side
// buffer, i being that first sample; the fused GEMM picks it up through head[].
// LABEL_WINDOW (batches of more than kLabelWindow samples; Sec. 3.3 enlarges the batch to 8K and
// 16K): with long-tailed labels one class can own a fifth of the batch, and one workgroup cannot
// read thousands of feature rows quickly (a compute unit draws a small share of the memory
// bandwidth).  The batch is cut into windows of kLabelWindow samples; block i sums the samples of
// its class inside its own window if it is the first of them there (`head` then points at that
// window's heads), and writes the partial sum to row i of the side buffer; dweight_label_combine
// adds a class's window sums in window order.
constexpr int kLabelThreads = 1024;
static_assert(kLabelWindow == kLabelThreads, "a window is scanned in one pass of the workgroup");
enum LabelMode { LABEL_ADD, LABEL_COMPACT, LABEL_WINDOW };
template <LabelMode MODE>
__global__ __launch_bounds__(kLabelThreads) void dweight_label_kernel(
    const float* __restrict__ X, int B, int D, const int32_t* __restrict__ yl, int64_t k,
    const int32_t* __restrict__ head, int64_t kp, const float* __restrict__ rnormX,
    const float* __restrict__ dlabel, float* __restrict__ dW) {
  __shared__ int s_list[kLabelThreads];
  __shared__ float s_coef[kLabelThreads];   // dlabel_p / |x_p| of the listed samples
  __shared__ int s_wcnt[kLabelThreads / 64];
  __shared__ float4 s_part[kLabelThreads];
  const int i = blockIdx.x, t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int32_t y = yl[i];
  if (y < 0 || (int64_t)y >= k) return;
  int p_end = B;
  if constexpr (MODE == LABEL_WINDOW) {
    const int w = i / kLabelWindow;
    head += (int64_t)(1 + w) * kp;   // the heads of this window
    p_end = min(B, (w + 1) * kLabelWindow);
  }
  if (head[y] != i) return;   // an earlier sample carries this label and does the sum
  const int cols = D >> 2;                 // float4 columns: 64 .. 256
  const int G = kLabelThreads / cols;      // thread groups
  const int col = t % cols, g = t / cols;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  int ordinal0 = 0;                        // matches seen in earlier chunks
  for (int p0 = i; p0 < p_end; p0 += kLabelThreads) {
    const int p = p0 + t;
    const bool hit = (p < p_end) && (yl[p] == y);
    const unsigned long long bal = __ballot(hit);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) s_wcnt[wave] = __popcll(bal);
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < kLabelThreads / 64; ++w) {
      const int c = s_wcnt[w];
      if (w < wave) base += c;
      total += c;
    }
    if (hit) {
      s_list[base + before] = p;
      s_coef[base + before] = dlabel[p] * rnormX[p];
    }
    __syncthreads();
    // group g takes list entries whose global ordinal is congruent to g modulo G; eight row
    // loads are in flight at a time, the additions stay in list order
    int e = (g - ordinal0 % G + G) % G;
    constexpr int UN = 8;
    for (; e + (UN - 1) * G < total; e += UN * G) {
      float4 x[UN];
      float a[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int q = s_list[e + u * G];
        a[u] = s_coef[e + u * G];
        x[u] = *reinterpret_cast<const float4*>(X + (int64_t)q * D + col * 4);
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        acc.x += a[u] * x[u].x; acc.y += a[u] * x[u].y; acc.z += a[u] * x[u].z; acc.w += a[u] * x[u].w;
      }
    }
    for (; e < total; e += G) {
      const int q = s_list[e];
      const float4 x = *reinterpret_cast<const float4*>(X + (int64_t)q * D + col * 4);
      const float a = s_coef[e];
      acc.x += a * x.x; acc.y += a * x.y; acc.z += a * x.z; acc.w += a * x.w;
    }
    ordinal0 += total;
    __syncthreads();
  }
  s_part[t] = acc;
  __syncthreads();
  if (g == 0) {
    float4 r = s_part[col];
    for (int gg = 1; gg < G; ++gg) {
      const float4 o = s_part[gg * cols + col];
      r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w;
    }
    if constexpr (MODE != LABEL_ADD) {
      *reinterpret_cast<float4*>(dW + (int64_t)i * D + col * 4) = r;
    } else {
      float4* dst = reinterpret_cast<float4*>(dW + (int64_t)y * D + col * 4);
      float4 cur = *dst;
      cur.x += r.x; cur.y += r.y; cur.z += r.z; cur.w += r.w;
      *dst = cur;
    }
  }
}

// dweight_label_combine (after dweight_label<LABEL_WINDOW>): block i, if sample i is the first of
// its class in the whole batch, adds the class's window sums (rows of `part` named by the window
// heads) in window order; the total goes to row i of `part` (COMPACT, fused step) or is added to
// dWn[y].  One float4 column per thread.
template <bool COMPACT>
__global__ void dweight_label_combine_kernel(int B, int D, const int32_t* __restrict__ yl,
                                             int64_t k, const int32_t* __restrict__ head,
                                             int64_t kp, int nwin, float* __restrict__ part,
                                             float* __restrict__ dW) {
  const int i = blockIdx.x, col = threadIdx.x;
  const int32_t y = yl[i];
  if (y < 0 || (int64_t)y >= k) return;
  if (head[y] != i || col >= (D >> 2)) return;
  float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int w = i / kLabelWindow; w < nwin; ++w) {
    const int32_t h = head[(int64_t)(1 + w) * kp + y];
    if (h == 0x7fffffff) continue;
    const float4 o = *reinterpret_cast<const float4*>(part + (int64_t)h * D + col * 4);
    r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w;
  }
  if constexpr (COMPACT) {
    *reinterpret_cast<float4*>(part + (int64_t)i * D + col * 4) = r;
  } else {
    float4* dst = reinterpret_cast<float4*>(dW + (int64_t)y * D + col * 4);
    float4 cur = *dst;
    cur.x += r.x; cur.y += r.y; cur.z += r.z; cur.w += r.w;
    *dst = cur;
  }
}

// ---------------------------------------------------------------------------------------------
// gemm_dweight_update (fused step): the dweight GEMM on tiles that span all D columns, followed
// in the same workgroup by the SGD-momentum update of the tile's rows (Eq. 3; text after Eq. 4),
// so dWn is never written to memory: dWn_j = GEMM row + label part, g = (dWn - <dWn,wn> wn)/|w|,
// v <- mu v + g, W <- W - lr v, with the arithmetic of update_kernel in the same order.
// The accumulators go through LDS one half of the tile at a time (the rows of the wavefronts
// with the same wm); then every wavefront takes whole rows, 16 bytes per lane and column chunk,
// RB rows in flight.
// ---------------------------------------------------------------------------------------------
template <class Cfg>
struct FusedUpdateLds {
  static constexpr int HR = Cfg::WTM;               // rows per half
  static constexpr int SROW = Cfg::BN + 4;          // floats per staged row (+4: the two rows a
                                                    // store instruction touches fall 16 banks apart)
  static constexpr int BYTES = HR * SROW * 4;
  static constexpr int LDS = BYTES > Cfg::LDS_BYTES ? BYTES : Cfg::LDS_BYTES;
};

template <class Cfg>
__device__ __forceinline__ void fused_update_tile(
    int64_t j0, char* smem, const typename Cfg::elem* __restrict__ E,
    const typename Cfg::elem* __restrict__ Xs, int64_t k, int64_t kp, int Bp,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ head,
    const float* __restrict__ lab, float* spare, float* __restrict__ W, float* __restrict__ V,
    int64_t N, float lr, float mu, int32_t* __restrict__ err_flag) {
  using FL = FusedUpdateLds<Cfg>;
  constexpr int D = Cfg::BN, NC = D / 256, HR = FL::HR, SROW = FL::SROW;
  constexpr int WAVES = Cfg::THREADS / 64, RPW = HR / WAVES;   // rows per wavefront and half
  constexpr int ROWS = Cfg::WM * RPW;                           // rows per wavefront and tile
  constexpr int WIN = 3;                                        // rows of W, v and label part in flight
  static_assert(D % 256 == 0 && HR % WAVES == 0 && ROWS <= 64 && WIN <= ROWS, "fused update geometry");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Two spare rows of D floats: the first holds zeros (never written) and is what a center that
  // is nobody's label reads instead of a label part, and what a padding row of the last tile
  // reads instead of W and v; the second takes the stores of the padding rows and is never read.
  // Every row thus issues the same loads and stores in the same order with no branch in between,
  // which is what lets the wait for row n's operands leave the younger requests of rows
  // n+1 .. n+WIN in flight.
  const float* zero_row = spare;
  float* trash_row = spare + D;

  // Row n of this wavefront (n = h*RPW + q) is tile row h*HR + q*WAVES + wave: neighbouring
  // wavefronts take neighbouring rows.  Lane n fetches its class id and label head now, so that
  // the epilogue starts its row loads without a dependent index load in front.
  int32_t idxv = -1, headv = INT_MAX;
  if (lane < ROWS) {
    const int64_t j = j0 + (lane / RPW) * HR + (lane % RPW) * WAVES + wave;
    if (j < k) {
      idxv = idx[j];
      headv = head[j];
      if (idxv < 0 || (int64_t)idxv >= N) {
        atomicOr(err_flag, 8);
        idxv = -1;
      }
    }
  }

  f32x16 acc[Cfg::TM][Cfg::TN];
  zero_acc<Cfg>(acc);
  PFC_PHASE(3, 0);
  gemm_tile<Cfg>(E + j0, kp, Xs, D, Bp / Cfg::BK, smem, acc);
  PFC_PHASE(3, 1);

  // A window of WIN rows of W, v and the label part is kept in flight: the loads of row n+WIN
  // are issued as soon as row n has been used, across the two halves.  (Native vector types:
  // arrays of them stay in registers.)
  f32x4 w[WIN][NC], v[WIN][NC], lb[WIN][NC];
  auto request = [&](int n) {
    const int64_t row = __builtin_amdgcn_readlane(idxv, n);   // wave-uniform
    const int hd = __builtin_amdgcn_readlane(headv, n);
    const float* wsrc = row >= 0 ? W + row * D : zero_row;    // scalar selects, no branch
    const float* vsrc = row >= 0 ? V + row * D : zero_row;
    const float* lsrc = hd != INT_MAX ? lab + (int64_t)hd * D : zero_row;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      w[n % WIN][c] = *reinterpret_cast<const f32x4*>(wsrc + c * 256 + lane * 4);
      v[n % WIN][c] = *reinterpret_cast<const f32x4*>(vsrc + c * 256 + lane * 4);
      lb[n % WIN][c] = *reinterpret_cast<const f32x4*>(lsrc + c * 256 + lane * 4);
    }
  };
#pragma unroll
  for (int n = 0; n < WIN; ++n) request(n);

  float* stage = reinterpret_cast<float*>(smem);
  const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
#pragma unroll
  for (int h = 0; h < Cfg::WM; ++h) {
    if (wm == h) {
#pragma unroll
      for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = bm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
#pragma unroll
          for (int bn = 0; bn < Cfg::TN; ++bn)
            stage[row * SROW + wn * Cfg::WTN + bn * 32 + (lane & 31)] = acc[bm][bn][r];
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < RPW; ++q) {
      const int n = h * RPW + q;
      const int64_t row = __builtin_amdgcn_readlane(idxv, n);
      const int r = q * WAVES + wave;
      float* wdst = row >= 0 ? W + row * D : trash_row;
      float* vdst = row >= 0 ? V + row * D : trash_row;
      f32x4 g[NC];
      float ww = 0.f, gw = 0.f;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int d = c * 256 + lane * 4;
        // GEMM row + label part (zeros unless this center is the label of a sample)
        g[c] = *reinterpret_cast<const f32x4*>(stage + r * SROW + d) + lb[n % WIN][c];
        const f32x4 wc = w[n % WIN][c];
        ww += wc[0] * wc[0] + wc[1] * wc[1] + wc[2] * wc[2] + wc[3] * wc[3];
        gw += g[c][0] * wc[0] + g[c][1] * wc[1] + g[c][2] * wc[2] + g[c][3] * wc[3];
      }
      ww = wave_sum(ww);
      gw = wave_sum(gw);
      const float rn = 1.f / fmaxf(sqrtf(ww), 1e-12f);
      const float t = gw * rn * rn;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int d = c * 256 + lane * 4;
        const f32x4 wc = w[n % WIN][c], vc = v[n % WIN][c];
        f32x4 vn, wq;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          vn[e] = mu * vc[e] + (g[c][e] - t * wc[e]) * rn;
          wq[e] = wc[e] - lr * vn[e];
        }
        // not read again before the next step's gather: nontemporal, so that the rows do not
        // sit dirty in the L2 while the next kernels run
        __builtin_nontemporal_store(vn, reinterpret_cast<f32x4*>(vdst + d));
        __builtin_nontemporal_store(wq, reinterpret_cast<f32x4*>(wdst + d));
      }
      if (n + WIN < ROWS) request(n + WIN);
    }
    __syncthreads();   // the next half overwrites the staged rows
    PFC_PHASE(3, 2 + h);
  }
}

// The first n_big workgroups take tiles of CfgB::BM rows; the rows left over when those no longer
// fill a whole round of workgroups on the GPU go to the following workgroups in tiles of
// CfgS::BM rows, so that the last, partly filled round is short.
template <class CfgB, class CfgS>
__global__ __launch_bounds__(CfgB::THREADS) void gemm_dweight_update_kernel(
    const typename CfgB::elem* __restrict__ E, const typename CfgB::elem* __restrict__ Xs,
    int64_t k, int64_t kp, int Bp, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ head, const float* __restrict__ lab, float* spare,
    float* __restrict__ W, float* __restrict__ V, int64_t N, float lr, float mu,
    int32_t* __restrict__ err_flag, int n_big) {
  static_assert(CfgB::THREADS == CfgS::THREADS && CfgB::BN == CfgS::BN, "one launch shape");
  extern __shared__ __align__(16) char smem[];
  const int b = blockIdx.x;
  if (b < n_big)
    fused_update_tile<CfgB>((int64_t)b * CfgB::BM, smem, E, Xs, k, kp, Bp, idx, head, lab, spare,
                            W, V, N, lr, mu, err_flag);
  else
    fused_update_tile<CfgS>((int64_t)n_big * CfgB::BM + (int64_t)(b - n_big) * CfgS::BM, smem, E,
                            Xs, k, kp, Bp, idx, head, lab, spare, W, V, N, lr, mu, err_flag);
}

// ---------------------------------------------------------------------------------------------
// gemm_dfeatures: slice `sp` of S: part[sp][i][d] = sum_{j in slice} E[i][j] * Wn[j][d]
// (A = E with k contiguous, B = Wn k-major).
// ---------------------------------------------------------------------------------------------
template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_dfeatures_kernel(
    const typename Cfg::elem* __restrict__ E, const typename Cfg::elem* __restrict__ Wn, int D,
    int Bp, int64_t kp, int slabs_total, int slabs_per, int splits, float* __restrict__ part,
    int tiles_i, int tiles_d) {
  extern __shared__ __align__(16) char smem[];
  int sp, tile;
  if (!xcd_tile(blockIdx.x, tiles_i * tiles_d, splits, sp, tile)) return;
  const int ti = tile / tiles_d, td = tile % tiles_d;
  const int i0 = ti * Cfg::BM, d0 = td * Cfg::BN;
  const int slab0 = sp * slabs_per;
  int ns = slabs_total - slab0;
  if (ns > slabs_per) ns = slabs_per;
  f32x16 acc[Cfg::TM][Cfg::TN];
  zero_acc<Cfg>(acc);
  const int64_t koff = (int64_t)slab0 * Cfg::BK;
  gemm_tile<Cfg>(E + (int64_t)i0 * kp + koff, kp, Wn + koff * D + d0, D, ns, smem, acc);
  float* out = part + (int64_t)sp * Bp * D;
#pragma unroll
  for (int bm = 0; bm < Cfg::TM; ++bm)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = i0 + acc_row<Cfg>(bm, r);
#pragma unroll
      for (int bn = 0; bn < Cfg::TN; ++bn)
        out[(int64_t)i * D + d0 + acc_col<Cfg>(bn)] = acc[bm][bn][r];
    }
}

// dfeatures_final: one wavefront per sample.
//   g  = (s/(B l_i)) * sum_slices part + dlabel_i * wn_{y_i}        (dL/d xn_i)
//   dx = (g - <g, xn_i> xn_i) / |x_i|
template <int NC>
__global__ void dfeatures_final_kernel(const float* __restrict__ part, int splits, int B, int Bp,
                                       int D, const float* __restrict__ X,
                                       const float* __restrict__ W, int64_t N,
                                       const int32_t* __restrict__ idx,
                                       const int32_t* __restrict__ yl, int64_t k,
                                       const float* __restrict__ rnormX,
                                       const float* __restrict__ rnormW,
                                       const float* __restrict__ rowscale,
                                       const float* __restrict__ dlabel, float* __restrict__ dX,
                                       const float* __restrict__ lossrow,
                                       float* __restrict__ loss_out,
                                       const float* __restrict__ clabel,
                                       const float* __restrict__ rowmax,
                                       float* __restrict__ stats_out) {
  const int lane = threadIdx.x & 63;
  if (blockIdx.x == gridDim.x - 1) {
    // the extra last block: mean loss (and, on request, mean label cosine = APCS and mean largest
    // non-label cosine = AMNCS), each summed in a fixed order (strided partials, then a tree)
    __shared__ float sm[256];
    const int nq = stats_out ? 3 : 1;
    for (int q = 0; q < nq; ++q) {
      const float* src = q == 0 ? lossrow : q == 1 ? clabel : rowmax;
      float v = 0.f;
      for (int r = threadIdx.x; r < B; r += 256) v += src[r];
      sm[threadIdx.x] = v;
      __syncthreads();
      for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
        __syncthreads();
      }
      if (threadIdx.x == 0) (q == 0 ? loss_out : stats_out + (q - 1))[0] = sm[0] / (float)B;
      __syncthreads();
    }
    return;
  }
  // One workgroup per sample.  The four wavefronts share the slices of S (wavefront w takes
  // slices w, w+4, ...: several independent loads in flight each); their partial rows are added
  // in wavefront order by wavefront 0, which then finishes the row: the same order on every run.
  const int i = blockIdx.x;
  const int wave = threadIdx.x >> 6;
  constexpr int nchunk = NC;
  constexpr int Dp = 256 * NC;   // row length of the partial sums
  __shared__ float4 s_part[3][NC][64];
  float4 sum[NC];
#pragma unroll
  for (int c = 0; c < nchunk; ++c) sum[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sp = wave; sp < splits; sp += 4) {
#pragma unroll
    for (int c = 0; c < nchunk; ++c) {
      const float4 t = *reinterpret_cast<const float4*>(part + ((int64_t)sp * Bp + i) * Dp +
                                                        c * 256 + lane * 4);
      sum[c].x += t.x; sum[c].y += t.y; sum[c].z += t.z; sum[c].w += t.w;
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int c = 0; c < nchunk; ++c) s_part[wave - 1][c][lane] = sum[c];
  }
  __syncthreads();
  if (wave > 0) return;
#pragma unroll
  for (int c = 0; c < nchunk; ++c) {
#pragma unroll
    for (int w = 0; w < 3; ++w) {
      const float4 t = s_part[w][c][lane];
      sum[c].x += t.x; sum[c].y += t.y; sum[c].z += t.z; sum[c].w += t.w;
    }
  }
  const float rs = rowscale[i], rnx = rnormX[i], dl = dlabel[i];
  const int32_t y = yl[i];
  int64_t wrow = -1;
  float rnw = 0.f;
  if (y >= 0 && (int64_t)y < k) {
    wrow = idx[y];
    rnw = rnormW[y];
    if (wrow < 0 || wrow >= N) wrow = -1;
  }
  float4 g[NC], xn[NC];
  float u = 0.f;
#pragma unroll
  for (int c = 0; c < nchunk; ++c) {
    const int d = c * 256 + lane * 4;
    float4 a = sum[c];
    a.x *= rs; a.y *= rs; a.z *= rs; a.w *= rs;
    if (wrow >= 0 && d < D) {
      const float4 w = *reinterpret_cast<const float4*>(W + wrow * D + d);
      const float f = dl * rnw;
      a.x += f * w.x; a.y += f * w.y; a.z += f * w.z; a.w += f * w.w;
    }
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);   // partial sums and x are zero from column D on
    if (d < D) x = *reinterpret_cast<const float4*>(X + (int64_t)i * D + d);
    x.x *= rnx; x.y *= rnx; x.z *= rnx; x.w *= rnx;
    g[c] = a;
    xn[c] = x;
    u += a.x * x.x + a.y * x.y + a.z * x.z + a.w * x.w;
  }
  u = wave_sum(u);
#pragma unroll
  for (int c = 0; c < nchunk; ++c) {
    float4 o;
    o.x = (g[c].x - u * xn[c].x) * rnx;
    o.y = (g[c].y - u * xn[c].y) * rnx;
    o.z = (g[c].z - u * xn[c].z) * rnx;
    o.w = (g[c].w - u * xn[c].w) * rnx;
    if (c * 256 + lane * 4 < D)
      *reinterpret_cast<float4*>(dX + (int64_t)i * D + c * 256 + lane * 4) = o;
  }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
// Number of batch slices of the dweight GEMM (1: none): slices only when the tiles alone leave
// most CUs idle, limited by the room in the split buffer and by a minimum slice length.
template <class CfgW>
int dweight_slices(const pfc_ctx* c, int tiles, int Bp, int64_t kp) {
  const int slabs_total = Bp / CfgW::BK;
  int want = c->num_cu / tiles;
  const int64_t room = (int64_t)kMaxSplits * Bp / kp;
  if (want > room) want = (int)room;
  if (want > slabs_total / 8) want = slabs_total / 8;   // a slice must stay long enough to pay
                                                        // for its own partial tile
  return want < 1 ? 1 : want;
}

template <typename T, int NC>
int run(pfc_ctx* c, const float* X, const float* W, const int32_t* idx, int64_t k,
        const int32_t* yl, int32_t B, const LossParams& lp, float* loss_out, float* dX_out,
        float* dW_out, float* stats_out, const UpdateArgs* upd) {
  using CfgF = TileCfg<T, 256, 256, 2, 4, false, false>;   // logits: 256 classes x 256 samples
  using CfgW = TileCfg<T, 256, 256, 2, 4, true, true>;     // dweight: 256 classes x 256 of D
  // fused dweight + update: 128 classes x all 512 columns, half-size slabs so that the wide
  // operand fits; this one-kernel form exists for D == 512 only
  using CfgU = TileCfg<T, 128, 512, 2, 4, true, true, 64>;
  using CfgUS = TileCfg<T, 64, 512, 1, 8, true, true, 128>;   // its tiles for the last round
  using CfgX = TileCfg<T, 256, 256, 2, 4, false, true>;    // dfeatures: 256 samples x 256 of D
  // small problems (fewer big tiles than compute units): 128 x 128 tiles, four times
  // as many workgroups, two of them resident per compute unit (74 KB of LDS each)
  using CfgFs = TileCfg<T, 128, 128, 2, 4, false, false>;
  using CfgWs = TileCfg<T, 128, 128, 2, 4, true, true>;
  constexpr int kFusedLds = FusedUpdateLds<CfgU>::LDS > FusedUpdateLds<CfgUS>::LDS
                                ? FusedUpdateLds<CfgU>::LDS : FusedUpdateLds<CfgUS>::LDS;
  static_assert(kFusedLds <= 160 * 1024, "LDS of one compute unit");
  const int D = c->D;
  constexpr int Dp = 256 * NC;   // row length of the library's own GEMM operands
  const int Bp = (int)round_up(B, kPadB);
  const int64_t kp = round_up(k, kPadK);
  T* Xn = (T*)c->Xn; T* Xs = (T*)c->Xs; T* Wn = (T*)c->Wn; T* E = (T*)c->E;
  // windows of the label part (0: the batch fits one window, or the context has no room for them)
  const int nwin = (B > kLabelWindow && c->label_windows) ? (B + kLabelWindow - 1) / kLabelWindow : 0;

  auto norm_kernel = normalize_x_kernel<T, NC>;
  PFC_LAUNCH(c, KID_NORM_X, norm_kernel, dim3((Bp + 3) / 4), dim3(256), 0, X, B, Bp, D,
             yl, k, Xn, c->rnormX, c->clabel, c->err_flag);

  auto gather_kernel = gather_normalize_w_kernel<T, NC>;
  PFC_LAUNCH(c, KID_GATHER_W, gather_kernel, dim3((unsigned)((kp / 4 + 3) / 4)), dim3(256), 0, W,
             c->N, idx, k, kp, D, Wn, c->rnormW, c->head, nwin, c->err_flag);

  // raise the dynamic LDS limit of this context's kernels once (a context has one precision and
  // one D, hence one instantiation of run)
  if (!c->lds_attr_set) {
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_logits_kernel<CfgF, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgF::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_logits_kernel<CfgF, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgF::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_rowmax_kernel<CfgF>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgF::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_dweight_kernel<CfgW, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgW::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_dweight_kernel<CfgW, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgW::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_logits_kernel<CfgFs, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgFs::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_logits_kernel<CfgFs, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgFs::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_rowmax_kernel<CfgFs>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgFs::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_dweight_kernel<CfgWs, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgWs::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_dweight_kernel<CfgWs, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgWs::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)gemm_dfeatures_kernel<CfgX>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, CfgX::LDS_BYTES));
    PFC_HIP(hipFuncSetAttribute((const void*)(gemm_dweight_update_kernel<CfgU, CfgUS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLds));
    c->lds_attr_set = 1;
  }
  auto launch_logits = [&](auto cfg) -> int {
    using Cfg = decltype(cfg);
    const int tiles_j = (int)(kp / Cfg::BM), tiles_i = Bp / Cfg::BN;
    if (lp.rowref) {   // scale above 64: the largest logit of every sample first
      PFC_LAUNCH(c, KID_GEMM_ROWMAX, gemm_rowmax_kernel<Cfg>, dim3(xcd_grid(tiles_i, tiles_j)),
                 dim3(Cfg::THREADS), Cfg::LDS_BYTES, Wn, Xn, Dp, k, B, yl, lp, c->rowmaxpart,
                 tiles_j, tiles_i);
      PFC_LAUNCH(c, KID_ROW_REF, row_ref_kernel, dim3((Bp + 3) / 4), dim3(256), 0, c->rowmaxpart,
                 tiles_j, B, Bp, c->rowref);
    }
    // the options (filter, column maxima, reference) have a kernel of their own: the plain one
    // stays lean
    auto logits_kernel = lp.extras ? gemm_logits_kernel<Cfg, true> : gemm_logits_kernel<Cfg, false>;
    PFC_LAUNCH(c, KID_GEMM_LOGITS, logits_kernel, dim3(xcd_grid(tiles_i, tiles_j)),
               dim3(Cfg::THREADS), Cfg::LDS_BYTES, Wn, Xn, Dp, k, B, Bp, kp, yl, lp, E, c->rowpart,
               c->rowmaxpart, c->clabel, tiles_j, tiles_i, c->num_cu / 8 * 8);
    auto combine_kernel = row_combine_kernel<T, NC>;
    PFC_LAUNCH(c, KID_ROW_COMBINE, combine_kernel, dim3((Bp + 3) / 4), dim3(256), 0, c->rowpart,
               tiles_j, B, Bp, D, X, c->rnormX, c->clabel, lp, c->rowmaxpart, c->rowscale,
               c->dlabel, c->lossrow, c->rowmax, yl, k, kp, c->head, nwin, Xs);
    return PFC_OK;
  };
  {
    const bool small = (kp / CfgF::BM) * (Bp / CfgF::BN) < (int64_t)c->num_cu;
    const int rc = small ? launch_logits(CfgFs{}) : launch_logits(CfgF{});
    if (rc != PFC_OK) return rc;
  }
  // label part of dWn: added to dW_out, or (compact) left in the side buffer for the fused kernel
  auto launch_label = [&](bool compact) -> int {
    if (nwin) {
      PFC_LAUNCH(c, KID_DW_LABEL, dweight_label_kernel<LABEL_WINDOW>, dim3(B), dim3(kLabelThreads),
                 0, X, B, D, yl, k, c->head, kp, c->rnormX, c->dlabel, c->dlab);
      if (compact) {
        PFC_LAUNCH(c, KID_DW_LABEL_SUM, dweight_label_combine_kernel<true>, dim3(B), dim3(256), 0,
                   B, D, yl, k, c->head, kp, nwin, c->dlab, dW_out);
      } else {
        PFC_LAUNCH(c, KID_DW_LABEL_SUM, dweight_label_combine_kernel<false>, dim3(B), dim3(256), 0,
                   B, D, yl, k, c->head, kp, nwin, c->dlab, dW_out);
      }
    } else if (compact) {
      PFC_LAUNCH(c, KID_DW_LABEL, dweight_label_kernel<LABEL_COMPACT>, dim3(B), dim3(kLabelThreads),
                 0, X, B, D, yl, k, c->head, kp, c->rnormX, c->dlabel, c->dlab);
    } else {
      PFC_LAUNCH(c, KID_DW_LABEL, dweight_label_kernel<LABEL_ADD>, dim3(B), dim3(kLabelThreads), 0,
                 X, B, D, yl, k, c->head, kp, c->rnormX, c->dlabel, dW_out);
    }
    return PFC_OK;
  };
  // dweight (+ label part) into dW_out
  auto launch_dweight_cfg = [&](auto cfg) -> int {
    using Cfg = decltype(cfg);
    const int tiles_j = (int)(kp / Cfg::BM), tiles_d = Dp / Cfg::BN;
    const int slabs_total = Bp / Cfg::BK;
    // slices of the batch when the tiles alone leave most CUs idle; the partial tiles borrow the
    // dfeatures split buffer, which is not in use at that point
    const int want = dweight_slices<Cfg>(c, tiles_j * tiles_d, Bp, kp);
    if (want >= 2) {
      const int slabs_per = (slabs_total + want - 1) / want;
      const int nsp = (slabs_total + slabs_per - 1) / slabs_per;
      PFC_LAUNCH(c, KID_GEMM_DW, (gemm_dweight_kernel<Cfg, true>),
                 dim3(xcd_grid(tiles_j * tiles_d, nsp)), dim3(Cfg::THREADS), Cfg::LDS_BYTES, E, Xs,
                 D, Dp, k, kp, Bp, c->dXpart, tiles_j, tiles_d, slabs_per, nsp);
      PFC_LAUNCH(c, KID_DW_REDUCE, dweight_reduce_kernel,
                 dim3((unsigned)((k * D / 4 + 255) / 256)), dim3(256), 0, c->dXpart, nsp, k, kp, D,
                 Dp, dW_out);
    } else {
      PFC_LAUNCH(c, KID_GEMM_DW, (gemm_dweight_kernel<Cfg, false>),
                 dim3(xcd_grid(tiles_d, tiles_j)), dim3(Cfg::THREADS), Cfg::LDS_BYTES, E, Xs, D,
                 Dp, k, kp, Bp, dW_out, tiles_j, tiles_d, slabs_total, 1);
    }
    return launch_label(false);
  };
  auto launch_dweight = [&]() -> int {
    // small tiles only when the big ones, sliced over the batch as far as that goes, still leave
    // more than half of the compute units idle (a long batch is better cut into slices of big
    // tiles: half the LDS traffic per flop)
    const int64_t tiles_big = (kp / CfgW::BM) * (Dp / CfgW::BN);
    const bool small =
        tiles_big * dweight_slices<CfgW>(c, (int)tiles_big, Bp, kp) * 2 < (int64_t)c->num_cu;
    return small ? launch_dweight_cfg(CfgWs{}) : launch_dweight_cfg(CfgW{});
  };
  // dfeatures GEMM (split over S) + final reduction, projection, loss
  auto launch_dfeatures = [&]() -> int {
    const int tiles_i = Bp / CfgX::BM, tiles_d = Dp / CfgX::BN;
    const int slabs_total = (int)(kp / CfgX::BK);
    int want = c->num_cu / (tiles_i * tiles_d);   // one workgroup per compute unit
    if (want < 1) want = 1;
    if (want > kMaxSplits) want = kMaxSplits;
    if (want > slabs_total) want = slabs_total;
    const int slabs_per = (slabs_total + want - 1) / want;
    const int splits = (slabs_total + slabs_per - 1) / slabs_per;
    PFC_LAUNCH(c, KID_GEMM_DX, gemm_dfeatures_kernel<CfgX>,
               dim3(xcd_grid(tiles_i * tiles_d, splits)), dim3(CfgX::THREADS), CfgX::LDS_BYTES, E,
               Wn, Dp, Bp, kp, slabs_total, slabs_per, splits, c->dXpart, tiles_i, tiles_d);
    PFC_LAUNCH(c, KID_DX_FINAL, dfeatures_final_kernel<NC>, dim3(B + 1), dim3(256), 0,
               c->dXpart, splits, B, Bp, D, X, W, c->N, idx, yl, k, c->rnormX, c->rnormW,
               c->rowscale, c->dlabel, dX_out, c->lossrow, loss_out, c->clabel, c->rowmax,
               stats_out);
    return PFC_OK;
  };

  if (!upd) {
    int rc = launch_dweight();
    if (rc != PFC_OK) return rc;
    return launch_dfeatures();
  }
  // Fused step.  dfeatures goes first: its final kernel reads the label rows of W, which the
  // update is about to change.
  int rc = launch_dfeatures();
  if (rc != PFC_OK) return rc;
  // one kernel only if D fits its tile and there is at least one tile per CU
  const bool one_kernel = D == CfgU::BN && kp / CfgU::BM >= c->num_cu;
  if (!one_kernel) {   // dWn through memory (dW_out is the context's own buffer here)
    rc = launch_dweight();
    if (rc != PFC_OK) return rc;
    return update_impl(c, upd->W, upd->v, idx, k, dW_out, upd->lr, upd->mu);
  }
  rc = launch_label(true);
  if (rc != PFC_OK) return rc;
  {
    const int tiles_big = (int)(kp / CfgU::BM);
    const int n_big = tiles_big / c->num_cu * c->num_cu;          // whole rounds
    const int n_small = (tiles_big - n_big) * (CfgU::BM / CfgUS::BM);
    PFC_LAUNCH(c, KID_GEMM_DW_UPDATE, (gemm_dweight_update_kernel<CfgU, CfgUS>),
               dim3((unsigned)(n_big + n_small)), dim3(CfgU::THREADS), kFusedLds, E, Xs, k, kp, Bp,
               idx, c->head, c->dlab, c->spare, upd->W, upd->v, c->N, upd->lr, upd->mu, c->err_flag,
               n_big);
  }
  return PFC_OK;
}

}  // namespace

int forward_backward_impl(pfc_ctx* c, const float* X, const float* W, const int32_t* idx,
                          int64_t k, const int32_t* yl, int32_t B, float s, float m,
                          int32_t margin_type, float filter_threshold, float* loss_out,
                          float* dX_out, float* dW_out, float* stats_out,
                          const UpdateArgs* upd) {
  LossParams lp;
  lp.s = s;
  lp.s_log2e = s * 1.44269504088896340736f;
  lp.m = m;
  lp.cos_m = cosf(m);
  lp.sin_m = sinf(m);
  lp.cosface = margin_type == PFC_MARGIN_COSFACE ? 1 : 0;
  lp.tau = filter_threshold;
  // cosines lie in [-1, 1]: up to s = 64 exp(s*cos) and its row sums stay inside the fp32 (and
  // bf16) range without a reference; above, the softmax runs relative to each sample's maximum
  lp.rowref = s > 64.f ? c->rowref : nullptr;
  lp.extras = (filter_threshold < 1.f || stats_out != nullptr || lp.rowref) ? 1 : 0;
#define PFC_RUN(T, NC) \
  return run<T, NC>(c, X, W, idx, k, yl, B, lp, loss_out, dX_out, dW_out, stats_out, upd)
  const int nc = (c->D + 255) / 256;
  if (c->precision == PFC_PRECISION_BF16) {
    switch (nc) {
      case 1: PFC_RUN(__bf16, 1);
      case 2: PFC_RUN(__bf16, 2);
      case 3: PFC_RUN(__bf16, 3);
      case 4: PFC_RUN(__bf16, 4);
    }
  } else {
    switch (nc) {
      case 1: PFC_RUN(float, 1);
      case 2: PFC_RUN(float, 2);
      case 3: PFC_RUN(float, 3);
      case 4: PFC_RUN(float, 4);
    }
  }
#undef PFC_RUN
  return PFC_EINVAL;
}

}  // namespace pfc
