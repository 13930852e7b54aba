// Context management, argument checks and the extern "C" layer of libpfc.so.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "pfc_common.h"

namespace pfc {

static thread_local char g_hip_err[512] = "";

void set_hip_error(hipError_t e, const char* what) {
  snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what, hipGetErrorString(e));
}

static const char* const kKernelNames[KID_COUNT] = {
    "sample_hist0", "sample_hist1", "sample_hist2", "sample_count",
    "sample_write",  "sample_remap", "normalize_x",  "gather_normalize_w", "gemm_rowmax",
    "row_ref", "gemm_logits",
    "row_combine",   "gemm_dweight", "dweight_reduce", "dweight_label", "dweight_label_combine",
    "gemm_dfeatures", "dfeatures_final", "update", "gemm_dweight_update"};

static int64_t ceil_rN(int64_t N, double r) { return (int64_t)ceil(r * (double)N); }

}  // namespace pfc

using namespace pfc;

extern "C" {

int64_t pfc_num_sampled(int64_t N, int32_t B, double r) {
  if (N < 1 || N >= (int64_t)1 << 31 || B < 1 || !(r > 0.0) || !(r <= 1.0)) return -1;
  int64_t c = ceil_rN(N, r);
  if (c > N) c = N;
  int64_t b = B < N ? B : N;
  return c > b ? c : b;
}

const char* pfc_strerror(int code) {
  switch (code) {
    case PFC_OK: return "ok";
    case PFC_EINVAL: return "invalid argument";
    case PFC_ELABEL: return "label or index out of range on the device";
    case PFC_EHIP: return "HIP runtime error";
    case PFC_ENOMEM: return "device memory allocation failed";
    default: return "unknown error code";
  }
}

const char* pfc_last_hip_error(void) { return g_hip_err; }

static int dev_alloc(void** p, size_t bytes) {
  *p = nullptr;
  hipError_t e = hipMalloc(p, bytes ? bytes : 16);
  if (e != hipSuccess) {
    set_hip_error(e, "hipMalloc");
    (void)hipGetLastError();
    return PFC_ENOMEM;
  }
  return PFC_OK;
}

int pfc_destroy(pfc_ctx* c) {
  if (!c) return PFC_EINVAL;
  (void)hipStreamSynchronize(c->stream);
  void* bufs[] = {c->pos_bits, c->hist, c->sel, c->blk_cnt, c->err_flag, c->Xn,
                  c->Xs, c->rnormX, c->Wn, c->rnormW, c->head, c->E, c->rowpart, c->rowmaxpart, c->rowmax,
                  c->rowref,
                  c->clabel, c->rowscale, c->dlabel, c->lossrow, c->dXpart, c->dlab, c->dWtmp,
                  c->spare};
  for (void* b : bufs)
    if (b) (void)hipFree(b);
  if (c->host_pin) (void)hipHostFree(c->host_pin);
  for (int i = 0; i < KID_COUNT; ++i) {
    if (c->ev0[i]) (void)hipEventDestroy(c->ev0[i]);
    if (c->ev1[i]) (void)hipEventDestroy(c->ev1[i]);
  }
  delete c;
  return PFC_OK;
}

int pfc_create(pfc_ctx** out, int64_t N, int32_t D, int32_t B_max, double r_max,
               int32_t precision, void* hip_stream) {
  if (!out) return PFC_EINVAL;
  *out = nullptr;
  if (N < 1 || N >= (int64_t)1 << 31) return PFC_EINVAL;
  if (D < 64 || D > 1024 || D % 64 != 0) return PFC_EINVAL;
  if (B_max < 1 || B_max > (1 << 20)) return PFC_EINVAL;
  if (!(r_max > 0.0) || !(r_max <= 1.0)) return PFC_EINVAL;
  if (precision != PFC_PRECISION_FP32 && precision != PFC_PRECISION_BF16) return PFC_EINVAL;

  pfc_ctx* c = new (std::nothrow) pfc_ctx;
  if (!c) return PFC_ENOMEM;
  memset(c, 0, sizeof(*c));
  c->N = N;
  c->D = D;
  c->B_max = B_max;
  c->r_max = r_max;
  c->precision = precision;
  c->stream = (hipStream_t)hip_stream;
  {
    int dev = 0, ncu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        ncu < 1)
      ncu = 256;
    c->num_cu = ncu;
  }
  c->k_cap = pfc_num_sampled(N, B_max, r_max);
  c->kp_cap = round_up(c->k_cap, kPadK);
  c->Bp_cap = (int32_t)round_up(B_max, kPadB);
  c->esize = precision == PFC_PRECISION_BF16 ? 2 : 4;
  // the GEMM staging code addresses up to 64 rows of E (row length kp elements) through one
  // 32-bit byte offset per thread
  if ((uint64_t)c->kp_cap * 64u * c->esize >= ((uint64_t)1 << 32)) {
    delete c;
    return PFC_EINVAL;
  }

  const size_t es = c->esize;
  const size_t Bp = (size_t)c->Bp_cap, kp = (size_t)c->kp_cap, Dz = (size_t)D;
  const size_t Dpz = (size_t)round_up(D, 256);   // row length of the GEMM operands
  c->nblk_cap = (int32_t)((N + 2047) / 2048);
  int rc = PFC_OK;
#define ALLOC(field, bytes)                                  \
  if (rc == PFC_OK) rc = dev_alloc((void**)&c->field, (bytes))
  ALLOC(pos_bits, ((size_t)(N + 31) / 32 + 64) * 4);
  ALLOC(hist, 3 * 4096 * 4);
  ALLOC(sel, sizeof(SelState));
  ALLOC(blk_cnt, (size_t)c->nblk_cap * 2 * 4);
  ALLOC(err_flag, 16);
  ALLOC(Xn, Bp * Dpz * es);
  ALLOC(Xs, Bp * Dpz * es);
  ALLOC(rnormX, Bp * 4);
  ALLOC(Wn, kp * Dpz * es);
  ALLOC(rnormW, kp * 4);
  {
    // window heads of the label part: for batches above one window, when the table stays small
    const int64_t nw = (B_max + kLabelWindow - 1) / kLabelWindow;
    c->label_windows =
        (nw >= 2 && nw <= kMaxLabelWindows && nw * (int64_t)kp <= ((int64_t)1 << 26)) ? (int32_t)nw : 0;
  }
  ALLOC(head, (size_t)(1 + c->label_windows) * kp * 4);
  ALLOC(E, Bp * kp * es);
  ALLOC(rowpart, (kp / kPadK) * 2 * Bp * 4);
  ALLOC(rowmaxpart, (kp / kPadK) * 2 * Bp * 4);
  ALLOC(rowmax, Bp * 4);
  ALLOC(rowref, Bp * 4);
  ALLOC(clabel, Bp * 4);
  ALLOC(rowscale, Bp * 4);
  ALLOC(dlabel, Bp * 4);
  ALLOC(lossrow, Bp * 4);
  ALLOC(dXpart, (size_t)kMaxSplits * Bp * Dpz * 4);
  ALLOC(dlab, Bp * Dz * 4);
  ALLOC(dWtmp, (size_t)c->k_cap * Dz * 4);
  ALLOC(spare, 2 * Dz * 4);
#undef ALLOC
  if (rc == PFC_OK) {
    hipError_t e = hipHostMalloc((void**)&c->host_pin, 64, hipHostMallocDefault);
    if (e != hipSuccess) {
      set_hip_error(e, "hipHostMalloc");
      rc = PFC_ENOMEM;
    }
  }
  // the sampler keeps its scratch all zero between calls (every last reader clears its piece)
  if (rc == PFC_OK) {
    hipError_t e = hipMemsetAsync(c->pos_bits, 0, ((size_t)(N + 31) / 32 + 64) * 4, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->hist, 0, 3 * 4096 * 4, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->sel, 0, sizeof(SelState), c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->spare, 0, 2 * Dz * 4, c->stream);
    if (e != hipSuccess) {
      set_hip_error(e, "hipMemsetAsync(sampler scratch)");
      rc = PFC_EHIP;
    }
  }
  if (rc == PFC_OK) {
    hipError_t e = hipMemsetAsync(c->err_flag, 0, 16, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
      set_hip_error(e, "hipMemsetAsync(err_flag)");
      rc = PFC_EHIP;
    }
  }
  if (rc != PFC_OK) {
    pfc_destroy(c);
    return rc;
  }
  *out = c;
  return PFC_OK;
}

int pfc_check(pfc_ctx* c) {
  if (!c) return PFC_EINVAL;
  PFC_HIP(hipMemcpyAsync(c->host_pin + 8, c->err_flag, 4, hipMemcpyDeviceToHost, c->stream));
  PFC_HIP(hipStreamSynchronize(c->stream));
  if (c->host_pin[8] != 0) {
    PFC_HIP(hipMemsetAsync(c->err_flag, 0, 4, c->stream));
    PFC_HIP(hipStreamSynchronize(c->stream));
    return PFC_ELABEL;
  }
  return PFC_OK;
}

int pfc_set_timing(pfc_ctx* c, int32_t enabled) {
  if (!c) return PFC_EINVAL;
  if (enabled && !c->ev0[0]) {
    for (int i = 0; i < KID_COUNT; ++i) {
      PFC_HIP(hipEventCreate(&c->ev0[i]));
      PFC_HIP(hipEventCreate(&c->ev1[i]));
    }
  }
  c->timing = enabled ? 1 : 0;
  memset(c->ev_used, 0, sizeof(c->ev_used));
  return PFC_OK;
}

int pfc_get_timing(pfc_ctx* c, const char** names_out, float* ms_out, int32_t cap) {
  if (!c || !names_out || !ms_out || cap < 0) return PFC_EINVAL;
  PFC_HIP(hipStreamSynchronize(c->stream));
  int n = 0;
  for (int i = 0; i < KID_COUNT && n < cap; ++i) {
    if (!c->ev_used[i]) continue;
    float ms = 0.f;
    PFC_HIP(hipEventElapsedTime(&ms, c->ev0[i], c->ev1[i]));
    names_out[n] = kKernelNames[i];
    ms_out[n] = ms;
    ++n;
  }
  return n;
}

int pfc_sample_masked(pfc_ctx* c, const int64_t* labels, int32_t B, double r, uint64_t seed,
                      uint64_t step, uint32_t score_mask, int32_t* idx_out, int32_t* yl_out,
                      int64_t* k_out) {
  if (!c || !labels || !idx_out || !yl_out || !k_out) return PFC_EINVAL;
  if (B < 1 || B > c->B_max) return PFC_EINVAL;
  if (!(r > 0.0) || !(r <= 1.0) || r > c->r_max) return PFC_EINVAL;
  return sample_impl(c, labels, B, r, seed, step, score_mask, idx_out, yl_out, k_out);
}

int pfc_sample(pfc_ctx* c, const int64_t* labels, int32_t B, double r, uint64_t seed,
               uint64_t step, int32_t* idx_out, int32_t* yl_out, int64_t* k_out) {
  return pfc_sample_masked(c, labels, B, r, seed, step, 0xFFFFFFFFu, idx_out, yl_out, k_out);
}

int pfc_forward_backward_ex(pfc_ctx* c, const float* X, const float* W, const int32_t* idx,
                            int64_t k, const int32_t* yl, int32_t B, float s, float m,
                            int32_t margin_type, float filter_threshold, float* loss_out,
                            float* dX_out, float* dW_out, float* stats_out) {
  if (!c || !X || !W || !idx || !yl || !loss_out || !dX_out || !dW_out) return PFC_EINVAL;
  if (B < 1 || B > c->B_max) return PFC_EINVAL;
  if (k < 1 || k > c->k_cap || k > c->N) return PFC_EINVAL;
  if (!(s > 0.f) || !(s <= 65536.f)) return PFC_EINVAL;
  if (margin_type != PFC_MARGIN_ARCFACE && margin_type != PFC_MARGIN_COSFACE) return PFC_EINVAL;
  if (!(m >= 0.f) || !(m < 3.14159265f)) return PFC_EINVAL;
  if (!(filter_threshold == filter_threshold) || filter_threshold < -1.f) return PFC_EINVAL;
  return forward_backward_impl(c, X, W, idx, k, yl, B, s, m, margin_type, filter_threshold,
                               loss_out, dX_out, dW_out, stats_out, nullptr);
}

int pfc_forward_backward_update(pfc_ctx* c, const float* X, float* W, float* v,
                                const int32_t* idx, int64_t k, const int32_t* yl, int32_t B,
                                float s, float m, int32_t margin_type, float filter_threshold,
                                float lr, float mu, float* loss_out, float* dX_out,
                                float* stats_out) {
  if (!c || !X || !W || !v || !idx || !yl || !loss_out || !dX_out) return PFC_EINVAL;
  if (B < 1 || B > c->B_max) return PFC_EINVAL;
  if (k < 1 || k > c->k_cap || k > c->N) return PFC_EINVAL;
  if (!(s > 0.f) || !(s <= 65536.f)) return PFC_EINVAL;
  if (margin_type != PFC_MARGIN_ARCFACE && margin_type != PFC_MARGIN_COSFACE) return PFC_EINVAL;
  if (!(m >= 0.f) || !(m < 3.14159265f)) return PFC_EINVAL;
  if (!(filter_threshold == filter_threshold) || filter_threshold < -1.f) return PFC_EINVAL;
  if (!(lr == lr) || !(mu == mu)) return PFC_EINVAL;
  UpdateArgs upd{W, v, lr, mu};
  return forward_backward_impl(c, X, W, idx, k, yl, B, s, m, margin_type, filter_threshold,
                               loss_out, dX_out, c->dWtmp, stats_out, &upd);
}

int pfc_forward_backward(pfc_ctx* c, const float* X, const float* W, const int32_t* idx,
                         int64_t k, const int32_t* yl, int32_t B, float s, float m,
                         float* loss_out, float* dX_out, float* dW_out) {
  return pfc_forward_backward_ex(c, X, W, idx, k, yl, B, s, m, PFC_MARGIN_ARCFACE, 2.f, loss_out,
                                 dX_out, dW_out, nullptr);
}

int pfc_update(pfc_ctx* c, float* W, float* v, const int32_t* idx, int64_t k, const float* dW,
               float lr, float mu) {
  if (!c || !W || !v || !idx || !dW) return PFC_EINVAL;
  if (k < 1 || k > c->N) return PFC_EINVAL;
  if (!(lr == lr) || !(mu == mu)) return PFC_EINVAL;
  return update_impl(c, W, v, idx, k, dW, lr, mu);
}

}  // extern "C"
