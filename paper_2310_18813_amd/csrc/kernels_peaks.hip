// Two microkernels that measure what this part delivers, for roofline fractions against measured as well as
// nominal peaks: a pure 16-byte-load stream over a caller's buffer, and back-to-back issue of the one MFMA
// instruction the GEMM kernels use.
#include "spec_internal.h"
#include "mfma_tiles.h"

namespace spec {

constexpr int STREAM_DEPTH = 8;  // loads in flight per wave

// Every workgroup walks its own contiguous share of the buffer, wave w taking the 1 KB pieces w, w + 8, ...
__global__ __launch_bounds__(512) void k_peak_stream(const u32x4_v *__restrict__ p, long pieces_per_wg) {
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const u32x4_v *base = p + (size_t)blockIdx.x * pieces_per_wg * 64 + lane;
  const long n = pieces_per_wg / 8;  // pieces per wave, a multiple of STREAM_DEPTH (host)
  u32x4_v acc = (u32x4_v){0u, 0u, 0u, 0u};
  for (long i0 = 0; i0 < n; i0 += STREAM_DEPTH) {
    u32x4_v r[STREAM_DEPTH];
#pragma unroll
    for (int d = 0; d < STREAM_DEPTH; ++d) r[d] = __builtin_nontemporal_load(base + (size_t)(w + 8 * (i0 + d)) * 64);
#pragma unroll
    for (int d = 0; d < STREAM_DEPTH; ++d) acc ^= r[d];
  }
  asm volatile("" ::"v"(acc[0]), "v"(acc[1]), "v"(acc[2]), "v"(acc[3]));  // keeps the loads alive; nothing is written
}

// Eight independent accumulator chains per wave, four waves per workgroup (one per SIMD).  The instruction
// is written out so that the compiler cannot reshape the loop; nothing reads an accumulator before the
// waits after the loop.
__global__ __launch_bounds__(256) void k_peak_mfma(int n) {
  f32x4_v acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = (f32x4_v){0.f, 0.f, 0.f, 0.f};
  f16x8_v a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(float)(threadIdx.x & 3); b[i] = (_Float16)1.0f; }
  for (int it = 0; it < n; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0];
  asm volatile("" ::"v"(s));  // keeps the chains alive; nothing is written
}

}  // namespace spec

using namespace spec;

extern "C" int spec_measure_peaks(void *hip_stream, void *d_buf, size_t bytes, double *h_hbm_gbs, double *h_mfma_tflops) {
  if (!d_buf || !h_hbm_gbs || !h_mfma_tflops) return SPEC_ERR_INVALID_ARG;
  if (((uintptr_t)d_buf & 15) != 0) return SPEC_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  int dev = 0, n_cu = 256;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
    n_cu = prop.multiProcessorCount;
  // the stream: as many 1 KB pieces per workgroup as fit, a multiple of 8 waves x STREAM_DEPTH
  const long unit = 8 * STREAM_DEPTH;
  const long pieces_per_wg = (long)(bytes / 1024 / n_cu) / unit * unit;
  if (pieces_per_wg < unit) return SPEC_ERR_CAPACITY;  // the buffer needs at least 64 KB per CU
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return SPEC_ERR_HIP;
  float ms = 0.f;
  int rc = SPEC_OK;
  double best_gbs = 0.0, best_tf = 0.0;
  for (int rep = 0; rep < 3 && rc == SPEC_OK; ++rep) {
    (void)hipEventRecord(e0, st);
    hipLaunchKernelGGL(k_peak_stream, dim3(n_cu), dim3(512), 0, st, (const u32x4_v *)d_buf, pieces_per_wg);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = SPEC_ERR_HIP; break; }
    if (rep > 0) best_gbs = std::max(best_gbs, (double)n_cu * pieces_per_wg * 1024.0 / (ms * 1e-3) / 1e9);
    const int iters = 20000, wgs = n_cu * 2;
    (void)hipEventRecord(e0, st);
    hipLaunchKernelGGL(k_peak_mfma, dim3(wgs), dim3(256), 0, st, iters);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = SPEC_ERR_HIP; break; }
    if (rep > 0) best_tf = std::max(best_tf, (double)wgs * 4 * 8.0 * iters * 16384.0 / (ms * 1e-3) / 1e12);
  }
  if (hipGetLastError() != hipSuccess) rc = SPEC_ERR_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *h_hbm_gbs = best_gbs;
  *h_mfma_tflops = best_tf;
  return rc;
}
