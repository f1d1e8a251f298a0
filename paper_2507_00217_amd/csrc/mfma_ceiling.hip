// Measurement aid, not part of the stage's path: the rate this GPU sustains on nothing but back-to-back
// v_mfma_f32_16x16x32_bf16, the GEMM's instruction (two wavefronts per SIMD, eight independent accumulator chains each, operands in registers,
// no memory or LDS traffic), and the shader clock it holds meanwhile.  With constant operands the clock stays at its
// nominal value and the rate is the published peak; with random operands the clock settles much lower (the matrix
// cores' power depends on how many bits toggle), and that lower rate -- not the published one -- is what a kernel
// working on real data can approach.  bench.py reports both next to the roofline figure.
#include "common.h"
#include "../../include/stage.h"
#include "../../include/stage_kernels.h"

namespace stg {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int CEIL_THREADS = 512, CEIL_MFMA_PER_ITER = 32;

__global__ __launch_bounds__(CEIL_THREADS) void mfma_ceiling_kernel(float* out, unsigned long long* clocks, int iters, int random_operands) {
  f32x4 acc[8];
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) acc[i][e] = 0.f;
  bf16x8 a[4], b[4];
  unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;       // a small LCG per lane
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 8; ++e) {
      h = h * 1664525u + 1013904223u;
      const float x = random_operands ? ((int)(h >> 8) - (1 << 23)) * (1.f / (1 << 23)) : 1.f;    // uniform in [-1, 1)
      h = h * 1664525u + 1013904223u;
      const float y = random_operands ? ((int)(h >> 8) - (1 << 23)) * (1.f / (1 << 23)) : 1.f;
      a[i][e] = (bf16)x;
      b[i][e] = (bf16)y;
    }
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < CEIL_MFMA_PER_ITER / 8; ++r)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(i + r) & 3], b[i & 3], acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) s += acc[i][e];
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  out[(size_t)blockIdx.x * CEIL_THREADS + threadIdx.x] = s;
  // the youngest wavefront of a SIMD gets the matrix core last, so its span is the workgroup's
  if (blockIdx.x == 0 && threadIdx.x == CEIL_THREADS - 64) { clocks[0] = c1 - c0; clocks[1] = r1 - r0; }
}

}  // namespace
}  // namespace stg

extern "C" int stage_probe_mfma_ceiling(int random_operands, int iters, void* scratch_dev, size_t scratch_bytes, double* tflops,
                                        double* shader_mhz, void* hip_stream) {
  using namespace stg;
  if (iters < 1 || iters > (1 << 22) || !tflops || !shader_mhz || !scratch_dev || ((uintptr_t)scratch_dev & 15)) return STAGE_E_INVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return STAGE_E_HIP;
  // scratch: two clock counts, then one float per thread (so that the compiler cannot drop the MFMAs)
  if (scratch_bytes < 16 + (size_t)cus * CEIL_THREADS * sizeof(float)) return STAGE_E_INVAL;
  unsigned long long* clocks = (unsigned long long*)scratch_dev;
  float* out = (float*)((char*)scratch_dev + 16);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = STAGE_E_HIP;
  float ms = 0.f;
  unsigned long long h[2] = {0, 0};
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto done;
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(cus), dim3(CEIL_THREADS), 0, s, out, clocks, iters / 8 + 1, random_operands);   // warm-up
  if (hipEventRecord(e0, s) != hipSuccess) goto done;
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(cus), dim3(CEIL_THREADS), 0, s, out, clocks, iters, random_operands);
  if (hipGetLastError() != hipSuccess || hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) goto done;
  if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f) goto done;
  if (hipMemcpy(h, clocks, sizeof h, hipMemcpyDeviceToHost) != hipSuccess || h[1] == 0) goto done;
  *tflops = (double)cus * (CEIL_THREADS / 64) * CEIL_MFMA_PER_ITER * (double)iters * (2.0 * 16 * 16 * 32) / (ms * 1e-3) / 1e12;
  *shader_mhz = (double)h[0] / ((double)h[1] / 100.0);       // the reference counter runs at 100 MHz
  rc = STAGE_OK;
done:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  return rc;
}
