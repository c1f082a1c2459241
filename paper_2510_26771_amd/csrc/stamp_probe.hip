// Measurement aid: the rate the matrix pipeline of this GPU sustains on the operand VALUES of this
// layer with no memory traffic at all.  A register-only loop of independent MFMAs over pseudo-random
// 4-bit codes in the operand format of the chosen engine, on every CU, timed with events.  The clock
// of the chip under such a load depends on the data (random operands draw more power than constant
// ones), so this rate, not the data-sheet peak, is what a GEMM on these values can approach.
#include "stamp_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// code in [-7, 7] from 4 random bits (the value -8 is folded onto 0)
__device__ __forceinline__ int code_of(uint32_t r) { const int c = (int)(r & 15u) - 8; return c == -8 ? 0 : c; }

__global__ __launch_bounds__(256) void k_rate_int8(int iters, float* sink) {
  v16i acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0;
  v4i a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t wa = 0, wb = 0;
    const uint32_t ra = mix(threadIdx.x * 8u + i + 1u), rb = mix(threadIdx.x * 8u + i + 0x9000u);
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // codes * 16 as int8, the integer engine's operand format
      wa |= ((uint32_t)(code_of(ra >> (4 * j)) * 16) & 0xFFu) << (8 * j);
      wb |= ((uint32_t)(code_of(rb >> (4 * j)) * 16) & 0xFFu) << (8 * j);
    }
    a[i] = (int)wa;
    b[i] = (int)wb;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 0x7fffffff) sink[0] = (float)s;
}

__global__ __launch_bounds__(256) void k_rate_fp6(int iters, float* sink) {
  v16f acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  v8i a, b;
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    // five sign-magnitude 6-bit fields and two more random bits per register: close enough to a packed
    // stream of E2M3 numbers code / 8 for the purpose of this measurement
    uint32_t wa = 0, wb = 0;
    const uint32_t ra = mix(threadIdx.x * 8u + i + 1u), rb = mix(threadIdx.x * 8u + i + 0x9000u);
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      const int ca = code_of(ra >> (4 * j)), cb = code_of(rb >> (4 * j));
      wa |= (uint32_t)((ca < 0 ? 32 - ca : ca)) << (6 * j);
      wb |= (uint32_t)((cb < 0 ? 32 - cb : cb)) << (6 * j);
    }
    a[i] = (int)(wa | (ra & 0xC0000000u));
    b[i] = (int)(wb | (rb & 0xC0000000u));
  }
  a[6] = a[7] = b[6] = b[7] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 2, 2, 0, 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 1.2345e30f) sink[0] = s;
}

}  // namespace

extern "C" stamp_status_t stamp_debug_mfma_rate(int32_t engine, double* tera_ops_per_s) {
  if (tera_ops_per_s == nullptr) return STAMP_ERR_NULL;
  if (engine != STAMP_GEMM_INT8 && engine != STAMP_GEMM_FP6) return STAMP_ERR_UNSUPPORTED;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return STAMP_ERR_DEVICE;
  float* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&sink), sizeof(float)) != hipSuccess) { (void)hipGetLastError(); return STAMP_ERR_ALLOC; }
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
  const int blocks = 2 * cus, iters = 20000;  // two workgroups of four waves per CU = two waves per SIMD
  const double ops_per_mfma = engine == STAMP_GEMM_FP6 ? 2.0 * 32 * 32 * 64 : 2.0 * 32 * 32 * 32;
  double best = 0.0;
  for (int rep = 0; ok && rep < 4; ++rep) {  // the first repetition warms up
    ok = hipEventRecord(e0, nullptr) == hipSuccess;
    if (engine == STAMP_GEMM_FP6) hipLaunchKernelGGL(k_rate_fp6, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
    else hipLaunchKernelGGL(k_rate_int8, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, nullptr) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
    float ms = 0.0f;
    ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    if (ok && rep > 0 && ms > 0.0f) {
      const double rate = (double)blocks * 4 * iters * 8 * ops_per_mfma / (ms * 1e-3) / 1e12;
      if (rate > best) best = rate;
    }
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  if (!ok) return STAMP_ERR_DEVICE;
  *tera_ops_per_s = best;
  return STAMP_OK;
}
