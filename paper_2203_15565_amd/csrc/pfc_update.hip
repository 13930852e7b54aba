// pfc_update: SGD with momentum on the sampled rows only (arXiv 2203.15565, Eq. 3; text after
// Eq. 4: only the sampled centers are updated in an iteration; all others are kept as they are).
//
// One wavefront per sampled row.  The row of W is needed for the update anyway, so the Jacobian
// of w -> w/|w| is applied here from registers:  g = (dWn - <dWn, wn> wn)/|w|.  HBM bound:
// 3 row reads (dWn, W, v) and 2 row writes (W, v) of D floats; rows outside idx are never
// addressed, so they stay bit-identical.
#include "pfc_common.h"

namespace pfc {

namespace {

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
  constexpr int nchunk = NC;   // D = 256 * NC
  float4 w[NC], g[NC], v[NC];
  float ww = 0.f, gw = 0.f;
#pragma unroll
  for (int c = 0; c < nchunk; ++c) {
    const int d = c * 256 + lane * 4;
    w[c] = *reinterpret_cast<const float4*>(W + row * D + d);
    g[c] = *reinterpret_cast<const float4*>(dWn + j * D + d);
    v[c] = *reinterpret_cast<const float4*>(V + row * D + d);
    ww += w[c].x * w[c].x + w[c].y * w[c].y + w[c].z * w[c].z + w[c].w * w[c].w;
    gw += g[c].x * w[c].x + g[c].y * w[c].y + g[c].z * w[c].z + g[c].w * w[c].w;
  }
  ww = wave_sum(ww);
  gw = wave_sum(gw);
  const float rn = 1.f / fmaxf(sqrtf(ww), 1e-12f);
  const float t = gw * rn * rn;   // <dWn, wn> / |w|  (multiplies the raw row w)
#pragma unroll
  for (int c = 0; c < nchunk; ++c) {
    const int d = c * 256 + lane * 4;
    float4 vn, wn;
    vn.x = mu * v[c].x + (g[c].x - t * w[c].x) * rn;
    vn.y = mu * v[c].y + (g[c].y - t * w[c].y) * rn;
    vn.z = mu * v[c].z + (g[c].z - t * w[c].z) * rn;
    vn.w = mu * v[c].w + (g[c].w - t * w[c].w) * rn;
    wn.x = w[c].x - lr * vn.x;
    wn.y = w[c].y - lr * vn.y;
    wn.z = w[c].z - lr * vn.z;
    wn.w = w[c].w - lr * vn.w;
    *reinterpret_cast<float4*>(V + row * D + d) = vn;
    *reinterpret_cast<float4*>(W + row * D + d) = wn;
  }
}

}  // namespace

int update_impl(pfc_ctx* c, float* W, float* v, const int32_t* idx, int64_t k, const float* dW,
                float lr, float mu) {
  const int rows_per_block = 4;
  const unsigned grid = (unsigned)((k + rows_per_block - 1) / rows_per_block);
  switch (c->D / 256) {
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
