// Measured ceilings of the machine the library runs on, for the roofline fractions a benchmark
// reports next to the published peaks: the rate of a loop of nothing but bf16 MFMAs, and the
// bandwidth of a plain device-to-device copy kernel.
#include "rf2_internal.h"

#include <mutex>

// Per-workgroup table of rf2_probe_xcd_mapping_static: 32 KiB on every GPU the library runs on, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress: the
// array's address on a device is looked up once per device (scratch_on_current_device) and it is
// that pointer which kernels and copies receive.
static __device__ __align__(256) int32_t scratch[RF2_XCD_PROBE_MAX_WORKGROUPS];

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

// The same loop on operands that differ from lane to lane and from register to register (pseudo-random
// bf16 values in (-2, 2)): the matrix cores draw far more power on such data than on constants, and what
// the chip sustains under its power limit is this rate, not the one of the loop above.
__global__ void __launch_bounds__(256) mfma_random_loop_kernel(float* sink, int iters) {
  uint32_t seed = threadIdx.x * 7919u + blockIdx.x * 104729u + 1u;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      seed = seed * 1664525u + 1013904223u;
      a[i][e] = (__bf16)(((int)(seed >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
      seed = seed * 1664525u + 1013904223u;
      b[i][e] = (__bf16)(((int)(seed >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
    }
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[2], c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3], b[3], c3, 0, 0, 0);
    if ((it & 63) == 63) {   // keep the accumulators in range
#pragma unroll
      for (int i = 0; i < 16; ++i) { c0[i] *= 1e-3f; c1[i] *= 1e-3f; c2[i] *= 1e-3f; c3[i] *= 1e-3f; }
    }
  }
  const float s = c0[0] + c1[1] + c2[2] + c3[3];
  if (s == 12345.f) sink[0] = s;   // never true: keeps the loop alive
}

// Workgroup g of a one-dimensional grid records the number of the XCD (accelerator die) it runs on.
__global__ void __launch_bounds__(256) xcd_of_workgroup_kernel(int32_t* out) {
  const int xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));   // hardware register XCC_ID, bits 3:0
  float x = (float)threadIdx.x;
  for (int i = 0; i < 2000; ++i) x = x * 1.0001f + 0.5f;    // stay resident for a while, so that the grid spreads out
  if (threadIdx.x == 0) out[blockIdx.x] = xcc + (x == 12345.f ? 1 : 0);
}

__global__ void __launch_bounds__(256) fill_kernel(int32_t* p, int n, int32_t value) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = value;
}

// One workgroup: result[0] = entries g < n of the table that equal entry g % 8, provided the first
// eight entries are eight different valid XCD numbers (0 otherwise); result[1] = entry 0.
__global__ void __launch_bounds__(256) xcd_agreement_kernel(const int32_t* __restrict__ table, int n,
                                                            int32_t* __restrict__ result) {
  __shared__ int count;
  if (threadIdx.x == 0) count = 0;
  __syncthreads();
  bool distinct = true;
  for (int a = 0; a < 8; ++a) {
    distinct = distinct && table[a] >= 0;
    for (int b = a + 1; b < 8; ++b) distinct = distinct && table[a] != table[b];
  }
  int mine = 0;
  for (int g = threadIdx.x; g < n; g += 256) mine += (distinct && table[g] == table[g & 7]);
  atomicAdd(&count, mine);
  __syncthreads();
  if (threadIdx.x == 0) {
    result[0] = count;
    result[1] = table[0];
  }
}

// Address of `scratch` on the device that is current, looked up on the first call made on that device.
std::mutex g_scratch_mutex;
constexpr int MAX_DEVICES = 64;
int32_t* g_scratch_ptr[MAX_DEVICES] = {};

int scratch_on_current_device(int32_t** out) {
  int dev = -1;
  RF2_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return RF2_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    RF2_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return rf2_note_hip_error(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  *out = g_scratch_ptr[dev];
  return RF2_OK;
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

extern "C" int rf2_measure_sustained_mfma(double seconds, double* mfma_bf16_tflops, void* stream) {
  if (!mfma_bf16_tflops || !(seconds > 0.0) || seconds > 30.0) return RF2_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  int dev = 0, n_cu = 0;
  RF2_HIP(hipGetDevice(&dev));
  RF2_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  float* sink = nullptr;
  hipEvent_t e0, e1;
  RF2_HIP(hipMalloc((void**)&sink, 256));
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipFree(sink); return rf2_note_hip_error(e); }
  const int iters = 20000, wgs = 2 * n_cu;
  const double flop_per_launch = (double)wgs * 4 /*wavefronts*/ * iters * 4 /*MFMAs*/ * 2.0 * 32 * 32 * 16;
  double total_ms = 0.0, timed_ms = 0.0;
  long launches = 0;
  // the first third of the time only warms up (the clock settles at the power limit), the rest is timed
  while (e == hipSuccess && total_ms < seconds * 1e3) {
    float ms = 0.f;
    e = hipEventRecord(e0, st);
    for (int r = 0; r < 4 && e == hipSuccess; ++r) {
      mfma_random_loop_kernel<<<wgs, 256, 0, st>>>(sink, iters);
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (total_ms >= seconds * 1e3 / 3.0) { timed_ms += ms; launches += 4; }
    total_ms += ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  if (e != hipSuccess) return rf2_note_hip_error(e);
  *mfma_bf16_tflops = launches ? flop_per_launch * (double)launches / (timed_ms * 1e-3) / 1e12 : 0.0;
  return RF2_OK;
}

extern "C" int rf2_probe_xcd_mapping(int32_t* n_agree, int32_t* n_workgroups, int32_t* first_xcd, void* stream) {
  if (!n_agree || !n_workgroups) return RF2_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const int n = 8192;
  int32_t* d = nullptr;
  RF2_HIP(hipMalloc((void**)&d, n * sizeof(int32_t)));
  std::vector<int32_t> h((size_t)n, -1);
  xcd_of_workgroup_kernel<<<n, 256, 0, st>>>(d);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(h.data(), d, n * sizeof(int32_t), hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  (void)hipFree(d);
  if (e != hipSuccess) return rf2_note_hip_error(e);
  // the first eight workgroups define where each residue class g % 8 lives; the classes must sit on
  // eight different XCDs and every later workgroup on the XCD of its class
  bool distinct = true;
  for (int a = 0; a < 8; ++a)
    for (int b = a + 1; b < 8; ++b) distinct = distinct && h[(size_t)a] != h[(size_t)b];
  int agree = 0;
  for (int g = 0; g < n; ++g) agree += (distinct && h[(size_t)g] == h[(size_t)(g & 7)]);
  *n_agree = agree;
  *n_workgroups = n;
  if (first_xcd) *first_xcd = h[0];
  return RF2_OK;
}

extern "C" int rf2_probe_xcd_mapping_static(int32_t n_launch, int32_t* result, void* stream) {
  if (!result || n_launch < 8) return RF2_ERR_INVALID_ARG;
  if (n_launch > RF2_XCD_PROBE_MAX_WORKGROUPS) return RF2_ERR_TOO_LARGE;
  hipStream_t st = (hipStream_t)stream;
  int32_t* table = nullptr;
  if (const int rc = scratch_on_current_device(&table)) return rc;
  // the table keeps the previous call's entries: mark the ones this call reads, so that a workgroup
  // that failed to report is counted as a disagreement and not as the last call's answer
  fill_kernel<<<(n_launch + 255) / 256, 256, 0, st>>>(table, n_launch, -1);
  RF2_LAUNCH_CHECK();
  xcd_of_workgroup_kernel<<<n_launch, 256, 0, st>>>(table);
  RF2_LAUNCH_CHECK();
  xcd_agreement_kernel<<<1, 256, 0, st>>>(table, n_launch, result);
  RF2_LAUNCH_CHECK();
  return RF2_OK;
}
