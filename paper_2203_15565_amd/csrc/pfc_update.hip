// pfc_update: SGD with momentum on the sampled rows only (arXiv 2203.15565, Eq. 3; text after
// Eq. 4: only the sampled centers are updated in an iteration; all others are kept as they are).
//
// One wavefront per sampled row.  The row of W is needed for the update anyway, so the Jacobian
// of w -> w/|w| is applied here from registers:  g = (dWn - <dWn, wn> wn)/|w|.  HBM bound:
// 3 row reads (dWn, W, v) and 2 row writes (W, v) of D floats; rows outside idx are never
// addressed, so they stay bit-identical.
#include "pfc_common.h"
#include "pfc_gemm.h"

namespace pfc {

namespace {

// The gradient is read once and the new rows are not read again before the next step, so both go
// through nontemporal accesses (measured at the headline workload: 0.403 -> 0.384 ms; more rows
// per wavefront or other block sizes change nothing).
template <int NC>
__global__ void update_kernel(float* __restrict__ W, float* __restrict__ V, int64_t N,
                              const int32_t* __restrict__ idx, int64_t k,
                              const float* __restrict__ dWn, int D, float lr, float mu,
                              int32_t* __restrict__ err_flag) {
  const int lane = threadIdx.x & 63;
  const int64_t j = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (j >= k) return;
  const int64_t row = idx[j];
  if (row < 0 || row >= N) {
    if (lane == 0) atomicOr(err_flag, 8);
    return;
  }
  f32x4 w[NC], g[NC], v[NC];
  float ww = 0.f, gw = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {   // 256 * (NC - 1) < D <= 256 * NC, D a multiple of 64
    const int d = c * 256 + lane * 4;
    w[c] = g[c] = v[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (d < D) {
      w[c] = *reinterpret_cast<const f32x4*>(W + row * D + d);
      g[c] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(dWn + j * D + d));
      v[c] = *reinterpret_cast<const f32x4*>(V + row * D + d);
    }
    ww += w[c][0] * w[c][0] + w[c][1] * w[c][1] + w[c][2] * w[c][2] + w[c][3] * w[c][3];
    gw += g[c][0] * w[c][0] + g[c][1] * w[c][1] + g[c][2] * w[c][2] + g[c][3] * w[c][3];
  }
  ww = wave_sum(ww);
  gw = wave_sum(gw);
  const float rn = 1.f / fmaxf(sqrtf(ww), 1e-12f);
  const float t = gw * rn * rn;   // <dWn, wn> / |w|  (multiplies the raw row w)
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int d = c * 256 + lane * 4;
    f32x4 vn, wq;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vn[e] = mu * v[c][e] + (g[c][e] - t * w[c][e]) * rn;
      wq[e] = w[c][e] - lr * vn[e];
    }
    if (d < D) {
      __builtin_nontemporal_store(vn, reinterpret_cast<f32x4*>(V + row * D + d));
      __builtin_nontemporal_store(wq, reinterpret_cast<f32x4*>(W + row * D + d));
    }
  }
}

}  // namespace

int update_impl(pfc_ctx* c, float* W, float* v, const int32_t* idx, int64_t k, const float* dW,
                float lr, float mu) {
  const int rows_per_block = 4;   // one wavefront per row
  const unsigned grid = (unsigned)((k + rows_per_block - 1) / rows_per_block);
  switch ((c->D + 255) / 256) {
#define PFC_UPD(NC)                                                                              \
  case NC: {                                                                                     \
    PFC_LAUNCH(c, KID_UPDATE, update_kernel<NC>, dim3(grid), dim3(rows_per_block * 64), 0, W, v, \
               c->N, idx, k, dW, c->D, lr, mu, c->err_flag);                                     \
    return PFC_OK;                                                                               \
  }
    PFC_UPD(1)
    PFC_UPD(2)
    PFC_UPD(3)
    PFC_UPD(4)
#undef PFC_UPD
  }
  return PFC_EINVAL;
}

}  // namespace pfc
