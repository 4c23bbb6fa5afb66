// Measured ceilings of the box the roofline fractions are quoted against: a streaming
// copy (HBM) and a register-resident bf16 MFMA loop (matrix cores).  Not on the hot path.
#include "common.h"
#include "device_utils.h"

namespace adwin {

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                   int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    store16(dst + i, src[i]);
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_loop_kernel(float* out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int k = 0; k < 8; ++k) { a[k] = (__bf16)(float)(threadIdx.x & 3); b[k] = (__bf16)1.0f; }
  f32x16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) s += acc[j][0];
  if (s == 12345.678f) out[0] = s;   // keeps the loop alive, practically never taken
}

// The same loop with pseudo-random operands (random sign and mantissa, exponents within a
// band of 8): the matrix cores then toggle as they do on real data, and the clock the
// power limit allows is lower than with constant operands.  Every 64 iterations the signs
// of A flip so that the accumulators stay bounded.
__global__ __launch_bounds__(256) void mfma_loop_random_kernel(float* out, int iters) {
  uint32_t st = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
  auto rnd16 = [&]() {
    st = st * 1664525u + 1013904223u;
    const uint32_t r = st >> 8;
    return ((r & 1u) << 15) | ((120u + ((r >> 8) & 7u)) << 7) | ((r >> 1) & 0x7fu);
  };
  uint4 wa[4], wb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    wa[i].x = rnd16() | (rnd16() << 16); wa[i].y = rnd16() | (rnd16() << 16);
    wa[i].z = rnd16() | (rnd16() << 16); wa[i].w = rnd16() | (rnd16() << 16);
    wb[i].x = rnd16() | (rnd16() << 16); wb[i].y = rnd16() | (rnd16() << 16);
    wb[i].z = rnd16() | (rnd16() << 16); wb[i].w = rnd16() | (rnd16() << 16);
  }
  f32x16 acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wa[j >> 2]),
                                                       __builtin_bit_cast(bf16x8, wb[j & 3]), acc[j], 0, 0, 0);
    if ((it & 63) == 63) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        wa[i].x ^= 0x80008000u; wa[i].y ^= 0x80008000u; wa[i].z ^= 0x80008000u; wa[i].w ^= 0x80008000u;
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 16; ++j) s += acc[j][0];
  if (s == 12345.678f) out[0] = s;
}

}  // namespace adwin

using namespace adwin;

// Copies `bytes` (multiple of 16) from src to dst, `reps` times, and returns the average
// milliseconds per copy in *ms (host).  Synchronises.
extern "C" int adwin_opd_ceiling_copy(const void* src, void* dst, size_t bytes, int reps,
                                      void* hip_stream, float* ms) {
  if (!src || !dst || !ms) return ADWIN_E_NULL;
  if ((bytes & 15) || reps < 1 || (((uintptr_t)src | (uintptr_t)dst) & 15)) return ADWIN_E_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t a, b;
  ADWIN_HIP_TRY(hipEventCreate(&a));
  ADWIN_HIP_TRY(hipEventCreate(&b));
  const int64_t n = (int64_t)(bytes / 16);
  copy_kernel<<<256 * 16, 256, 0, st>>>((const uint4*)src, (uint4*)dst, n);   // warm-up
  ADWIN_HIP_TRY(hipEventRecord(a, st));
  for (int r = 0; r < reps; ++r) copy_kernel<<<256 * 16, 256, 0, st>>>((const uint4*)src, (uint4*)dst, n);
  ADWIN_HIP_TRY(hipEventRecord(b, st));
  ADWIN_HIP_TRY(hipEventSynchronize(b));
  float t = 0.f;
  ADWIN_HIP_TRY(hipEventElapsedTime(&t, a, b));
  *ms = t / reps;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return ADWIN_OK;
}

// Runs a register-resident v_mfma_f32_32x32x16_bf16 loop on every CU and returns the
// achieved dense bf16 TFLOP/s in *tflops (host).  `scratch` is 4 bytes of device memory.
extern "C" int adwin_opd_ceiling_mfma(void* scratch, int iters, void* hip_stream, float* tflops) {
  if (!scratch || !tflops) return ADWIN_E_NULL;
  if (iters < 1) return ADWIN_E_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t a, b;
  ADWIN_HIP_TRY(hipEventCreate(&a));
  ADWIN_HIP_TRY(hipEventCreate(&b));
  const int blocks = 256 * 2;
  mfma_loop_kernel<<<blocks, 256, 0, st>>>((float*)scratch, 16);
  ADWIN_HIP_TRY(hipEventRecord(a, st));
  mfma_loop_kernel<<<blocks, 256, 0, st>>>((float*)scratch, iters);
  ADWIN_HIP_TRY(hipEventRecord(b, st));
  ADWIN_HIP_TRY(hipEventSynchronize(b));
  float t = 0.f;
  ADWIN_HIP_TRY(hipEventElapsedTime(&t, a, b));
  const double flops = (double)blocks * 4.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
  *tflops = (float)(flops / (t * 1e-3) / 1e12);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return ADWIN_OK;
}

// As adwin_opd_ceiling_mfma, with pseudo-random operands: the rate the matrix cores sustain
// on data that toggles like real inputs.
extern "C" int adwin_opd_ceiling_mfma_random(void* scratch, int iters, void* hip_stream,
                                             float* tflops) {
  if (!scratch || !tflops) return ADWIN_E_NULL;
  if (iters < 1) return ADWIN_E_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t a, b;
  ADWIN_HIP_TRY(hipEventCreate(&a));
  ADWIN_HIP_TRY(hipEventCreate(&b));
  const int blocks = 256;
  mfma_loop_random_kernel<<<blocks, 256, 0, st>>>((float*)scratch, 16);
  ADWIN_HIP_TRY(hipEventRecord(a, st));
  mfma_loop_random_kernel<<<blocks, 256, 0, st>>>((float*)scratch, iters);
  ADWIN_HIP_TRY(hipEventRecord(b, st));
  ADWIN_HIP_TRY(hipEventSynchronize(b));
  float t = 0.f;
  ADWIN_HIP_TRY(hipEventElapsedTime(&t, a, b));
  const double flops = (double)blocks * 4.0 * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
  *tflops = (float)(flops / (t * 1e-3) / 1e12);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return ADWIN_OK;
}
