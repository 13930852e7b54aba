// Calibration probes for benchmarks (libpfc_probe.so, not part of libpfc.so): what this GPU
// sustains on a plain stream copy and on a bare MFMA issue loop, measured with HIP events on the
// given stream.  They are reported next to the nominal peaks (8 TB/s HBM3E, 2.5 PFLOP/s dense
// bf16) so that a roofline fraction can be read against both.
#include "pfc_common.h"
#include "pfc_gemm.h"
#include "pfc_probe.h"

namespace pfc {
// this library has no context: errors are only reported through the return code
void set_hip_error(hipError_t, const char*) {}
}  // namespace pfc

namespace pfc {
namespace {

__global__ void probe_copy_kernel(const float4* __restrict__ a, float4* __restrict__ b, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) b[i] = a[i];
}

// Each wavefront: 8 independent 32x32 accumulators, `iters` rounds of 8 bf16 MFMAs on operands
// with pseudo-random bit patterns in [-1, 1) (data toggling matters for the sustained clock).
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* __restrict__ sink) {
  const uint32_t t = blockIdx.x * 256u + threadIdx.x;
  u32x4 a, b;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    uint32_t h = (t * 4u + e) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    // two bf16 values with exponent 0x7E/0x7D (|x| in [0.25, 1)) and random sign / mantissa
    const uint32_t lo = (h & 0x80FFu) | 0x3E80u, hi = ((h >> 16) & 0x80FFu) | 0x3F00u;
    a[e] = lo | (hi << 16);
    b[e] = hi | (lo << 16);
  }
  f32x16 acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 8; ++q) mfma_group<__bf16>(a, b, acc[q]);
    // flip mantissa bits every round: operand toggling is what a real GEMM presents to the
    // MFMA pipe, and the sustained clock depends on it
    const uint32_t flip = ((uint32_t)it * 0x9E3779B9u) & 0x007F007Fu;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      a[e] ^= flip;
      b[e] ^= (flip >> 1) & 0x007F007Fu;
    }
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < 8; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[q][r];
  if (s == 12345.678f) sink[0] = s;   // never true: keeps the loop alive
}

}  // namespace
}  // namespace pfc

using namespace pfc;

extern "C" {

int pfc_probe_stream_copy(void* hip_stream, const void* src, void* dst, int64_t bytes,
                          int32_t reps, double* gbs_out) {
  if (!src || !dst || !gbs_out || bytes < 16 || bytes % 16 != 0 || reps < 1) return PFC_EINVAL;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  PFC_HIP(hipEventCreate(&e0));
  PFC_HIP(hipEventCreate(&e1));
  const size_t n = (size_t)bytes / 16;
  hipLaunchKernelGGL(probe_copy_kernel, dim3(65536), dim3(256), 0, stream, (const float4*)src,
                     (float4*)dst, n);
  PFC_HIP(hipEventRecord(e0, stream));
  for (int i = 0; i < reps; ++i)
    hipLaunchKernelGGL(probe_copy_kernel, dim3(65536), dim3(256), 0, stream, (const float4*)src,
                       (float4*)dst, n);
  PFC_HIP(hipEventRecord(e1, stream));
  PFC_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  PFC_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *gbs_out = 2.0 * (double)bytes * reps / ((double)ms * 1e-3) / 1e9;   // read + write
  return PFC_OK;
}

int pfc_probe_mfma_bf16(void* hip_stream, float* sink, int32_t reps, double* tflops_out) {
  if (!sink || !tflops_out || reps < 1) return PFC_EINVAL;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  PFC_HIP(hipEventCreate(&e0));
  PFC_HIP(hipEventCreate(&e1));
  const int iters = 2048, blocks = 2048;   // 8 wavefronts per CU at a time, 8192 in total
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(256), 0, stream, iters, sink);
  PFC_HIP(hipEventRecord(e0, stream));
  for (int i = 0; i < reps; ++i)
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(256), 0, stream, iters, sink);
  PFC_HIP(hipEventRecord(e1, stream));
  PFC_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  PFC_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  const double flops = (double)blocks * 4.0 * iters * 8.0 * 32768.0 * reps;   // 2*32*32*16 per MFMA
  *tflops_out = flops / ((double)ms * 1e-3) / 1e12;
  return PFC_OK;
}

}  // extern "C"
