// Shared host/device declarations of libpfc.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pfc.h"

namespace pfc {

// ---------------------------------------------------------------------------------------------
// Padded problem geometry.  Every scratch operand of the three GEMMs is padded with zeros to a
// whole number of tiles, so the GEMM main loops need no bounds checks.
// ---------------------------------------------------------------------------------------------
constexpr int kPadB = 256;   // batch rows are padded to a multiple of this
constexpr int kPadK = 256;   // sampled rows are padded to a multiple of this
constexpr int kMaxSplits = 64;
constexpr int kLabelWindow = 1024;     // samples per window of the label part of dWn
constexpr int kMaxLabelWindows = 64;   // one lane of a wavefront initialises one window's head

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Kernel ids for the optional per-kernel timing.
enum KernelId {
  KID_SAMPLE_HIST0 = 0,
  KID_SAMPLE_HIST1,
  KID_SAMPLE_HIST2,
  KID_SAMPLE_COUNT,
  KID_SAMPLE_WRITE,
  KID_SAMPLE_REMAP,
  KID_NORM_X,
  KID_GATHER_W,
  KID_GEMM_ROWMAX,
  KID_ROW_REF,
  KID_GEMM_LOGITS,
  KID_ROW_COMBINE,
  KID_GEMM_DW,
  KID_DW_REDUCE,
  KID_DW_LABEL,
  KID_DW_LABEL_SUM,
  KID_GEMM_DX,
  KID_DX_FINAL,
  KID_UPDATE,
  KID_GEMM_DW_UPDATE,
  KID_COUNT
};

// State of the radix select, kept in device memory between the sampler's kernels.
struct SelState {
  uint32_t U;          // number of distinct labels (positives); cleared again once consumed
  uint32_t k;          // |S| = max(U, ceil(r*N))
  uint32_t none;       // 1: no negative is taken at all (k == U)
  uint32_t total;      // number of ids written (must equal k)
  uint32_t need[3];    // after radix pass P: negatives still to be taken inside the chosen bin
  uint32_t prefix[3];  // after radix pass P: threshold bits fixed so far (in place, low bits zero)
  uint32_t pad[2];
};

}  // namespace pfc

struct pfc_ctx {
  int64_t N;
  int32_t D;
  int32_t B_max;
  double r_max;
  int32_t precision;
  hipStream_t stream;

  int64_t k_cap;    // pfc_num_sampled(N, B_max, r_max)
  int64_t kp_cap;   // padded
  int32_t Bp_cap;   // padded
  size_t esize;     // bytes per GEMM operand element (4 or 2)

  // sampler scratch
  uint32_t* pos_bits;     // ceil(N/32) words (+ slack): bit j set <=> class j is in the batch
  uint32_t* hist;         // 3 x 4096 bins (radix passes of 8, 12 and 12 bits)
  pfc::SelState* sel;
  uint32_t* blk_cnt;      // 2 x nblk: per block (#sure, #equal-to-threshold)
  int32_t nblk_cap;
  int32_t* err_flag;      // device: nonzero once a bad label / index was seen
  uint32_t* host_pin;     // pinned host words for read-backs

  // forward/backward scratch (T = float or bf16 according to precision)
  void* Xn;        // [Bp x Dp]  normalised features (Dp = D rounded up to 256, zero columns)
  void* Xs;        // [Bp x Dp]  (s/(B*l_i)) * xn_i
  float* rnormX;   // [Bp]
  void* Wn;        // [kp x Dp]  normalised sampled centers
  float* rnormW;   // [kp]
  int32_t* head;   // [(1 + label_windows) x kp] first sample of the batch that carries class
                   // idx[j], else INT_MAX; then the same for every window of kLabelWindow samples
                   // (kp = k rounded up to 256 in the call at hand)
  int32_t label_windows;   // windows the head buffer has room for (0: none, batch in one piece)
  void* E;         // [Bp x kp]  exp(z), label column zeroed
  float* rowpart;  // [Bp x tiles_j] partial row sums of exp(z)
  float* rowmaxpart;  // [Bp x tiles_j] partial row maxima of the non-label cosines (options)
  float* rowmax;   // [Bp]
  float* rowref;   // [Bp] largest logit of every sample (scales above 64 only)
  float* clabel;   // [Bp] cosine of the label column
  float* rowscale; // [Bp] s/(B*l_i)
  float* dlabel;   // [Bp] (s/B)(p_iy - 1) rho_i
  float* lossrow;  // [Bp]
  float* dXpart;   // [splits x Bp x Dp]
  float* dlab;     // [Bp x D] label-column part of dWn, one row per first sample of a class (fused step)
  float* dWtmp;    // [k_cap x D] dWn of the fused step whenever its one-kernel form does not apply
  float* spare;    // [2 x D] a row of zeros (never written) and a row that only takes the stores of
                   // padding rows (fused step)

  // timing
  int32_t num_cu;   // compute units of the device
  int32_t lds_attr_set;   // the dynamic LDS limit of the GEMM kernels has been raised
  int32_t timing;
  hipEvent_t ev0[pfc::KID_COUNT];
  hipEvent_t ev1[pfc::KID_COUNT];
  uint8_t ev_used[pfc::KID_COUNT];
};

namespace pfc {

void set_hip_error(hipError_t e, const char* what);

#define PFC_HIP(expr)                                   \
  do {                                                  \
    hipError_t e__ = (expr);                            \
    if (e__ != hipSuccess) {                            \
      ::pfc::set_hip_error(e__, #expr);                 \
      return PFC_EHIP;                                  \
    }                                                   \
  } while (0)

// Launch helper: optional event pair around the kernel for the timing hooks.
struct TimedLaunch {
  pfc_ctx* c;
  int id;
  TimedLaunch(pfc_ctx* ctx, int kid) : c(ctx), id(kid) {
    if (c->timing) (void)hipEventRecord(c->ev0[id], c->stream);
  }
  ~TimedLaunch() {
    if (c->timing) {
      (void)hipEventRecord(c->ev1[id], c->stream);
      c->ev_used[id] = 1;
    }
  }
};

#define PFC_LAUNCH(ctx, kid, kernel, grid, block, shmem, ...)                          \
  do {                                                                                 \
    ::pfc::TimedLaunch tl__(ctx, kid);                                                 \
    hipLaunchKernelGGL(kernel, grid, block, shmem, (ctx)->stream, __VA_ARGS__);        \
  } while (0);                                                                         \
  PFC_HIP(hipGetLastError())

// Present when forward/backward is to end in the update of the sampled rows (the fused step).
struct UpdateArgs {
  float* W;   // [N x D] in/out
  float* v;   // [N x D] in/out
  float lr, mu;
};

// entry points implemented per translation unit (called by the extern "C" layer)
int sample_impl(pfc_ctx* ctx, const int64_t* labels, int32_t B, double r, uint64_t seed,
                uint64_t step, uint32_t score_mask, int32_t* idx_out, int32_t* yl_out,
                int64_t* k_out);
int forward_backward_impl(pfc_ctx* ctx, const float* X, const float* W, const int32_t* idx,
                          int64_t k, const int32_t* yl, int32_t B, float s, float m,
                          int32_t margin_type, float filter_threshold, float* loss_out,
                          float* dX_out, float* dW_out, float* stats_out, const UpdateArgs* upd);
int update_impl(pfc_ctx* ctx, float* W, float* v, const int32_t* idx, int64_t k,
                const float* dW, float lr, float mu);

// ---------------------------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------------------------
#if defined(__HIPCC__)
// Sum over the 64 lanes of a wavefront, the same bits in every lane.  Inside each row of 16
// lanes the exchange runs through the cross-lane modifiers of the vector ALU (xor 1, xor 2, mirror
// of 8, mirror of 16: every lane of a row adds the same pairs, and a + b == b + a, so the row's 16
// lanes end with one value); the four row sums are then read out lane by lane and added in a
// fixed order.  No LDS round trip (a shuffle-based butterfly costs six of them in a chain).
template <int CTRL>
__device__ __forceinline__ float dpp_xadd(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true);
  return v + __builtin_bit_cast(float, moved);
}
__device__ __forceinline__ float wave_sum(float v) {
  v = dpp_xadd<0xB1>(v);    // quad_perm [1,0,3,2]
  v = dpp_xadd<0x4E>(v);    // quad_perm [2,3,0,1]
  v = dpp_xadd<0x141>(v);   // row_half_mirror
  v = dpp_xadd<0x140>(v);   // row_mirror
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}

template <typename T>
__device__ __forceinline__ T from_float(float x);
template <>
__device__ __forceinline__ float from_float<float>(float x) { return x; }
template <>
__device__ __forceinline__ __bf16 from_float<__bf16>(float x) { return (__bf16)x; }  // RNE
#endif

}  // namespace pfc
