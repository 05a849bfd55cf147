// Measured ceilings of the machine the library runs on, for the roofline fractions a benchmark
// reports next to the published peaks: the rate of a loop of nothing but bf16 MFMAs, and the
// bandwidth of a plain device-to-device copy kernel.
#include "rf2_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Four independent accumulator chains per wavefront, four wavefronts per workgroup.
__global__ void __launch_bounds__(256) mfma_loop_kernel(float* sink, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)1.0f; b[e] = (__bf16)0.5f; }
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  const float s = c0[0] + c1[1] + c2[2] + c3[3];
  if (s == 12345.f) sink[0] = s;   // never true: keeps the loop alive
}

__global__ void __launch_bounds__(256) copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" int rf2_measure_peaks(double* mfma_bf16_tflops, double* copy_gbps, void* stream) {
  if (!mfma_bf16_tflops && !copy_gbps) return RF2_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  int dev = 0, n_cu = 0;
  RF2_HIP(hipGetDevice(&dev));
  RF2_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  hipEvent_t e0, e1;
  RF2_HIP(hipEventCreate(&e0));
  RF2_HIP(hipEventCreate(&e1));
  int rc = RF2_OK;
  float ms = 0.f;
  unsigned char* buf = nullptr;
  const size_t bytes = (size_t)1 << 30;                 // source and destination: 1 GiB each
  auto fail = [&](hipError_t e) { rc = (e == hipErrorOutOfMemory) ? RF2_ERR_ALLOC : rf2_note_hip_error(e); };
  do {
    hipError_t e = hipMalloc((void**)&buf, 2 * bytes);
    if (e != hipSuccess) { fail(e); break; }
    if (mfma_bf16_tflops) {
      const int iters = 20000, wgs = 2 * n_cu;
      mfma_loop_kernel<<<wgs, 256, 0, st>>>((float*)buf, 100);
      if ((e = hipEventRecord(e0, st)) != hipSuccess) { fail(e); break; }
      mfma_loop_kernel<<<wgs, 256, 0, st>>>((float*)buf, iters);
      if ((e = hipEventRecord(e1, st)) != hipSuccess) { fail(e); break; }
      if ((e = hipEventSynchronize(e1)) != hipSuccess) { fail(e); break; }
      if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) { fail(e); break; }
      const double flop = (double)wgs * 4 /*wavefronts*/ * iters * 4 /*MFMAs*/ * 2.0 * 32 * 32 * 16;
      *mfma_bf16_tflops = flop / (ms * 1e-3) / 1e12;
    }
    if (copy_gbps) {
      if ((e = hipMemsetAsync(buf, 1, 2 * bytes, st)) != hipSuccess) { fail(e); break; }
      const size_t n = bytes / 16;
      const int wgs = (int)(n / 256), reps = 5;        // one 16-byte element per lane: the fastest shape on this chip
      copy_kernel<<<wgs, 256, 0, st>>>((const uint4*)buf, (uint4*)(buf + bytes), n);
      if ((e = hipEventRecord(e0, st)) != hipSuccess) { fail(e); break; }
      for (int r = 0; r < reps; ++r) copy_kernel<<<wgs, 256, 0, st>>>((const uint4*)buf, (uint4*)(buf + bytes), n);
      if ((e = hipEventRecord(e1, st)) != hipSuccess) { fail(e); break; }
      if ((e = hipEventSynchronize(e1)) != hipSuccess) { fail(e); break; }
      if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) { fail(e); break; }
      *copy_gbps = 2.0 * bytes * reps / (ms * 1e-3) / 1e9;
    }
    if ((e = hipGetLastError()) != hipSuccess) fail(e);
  } while (false);
  if (buf) (void)hipFree(buf);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}
