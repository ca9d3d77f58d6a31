// Measurement aid: what the matrix pipe alone sustains on this device.  A register-only loop of
// bf16 MFMA 32x32x16 on pseudo-random operands (no LDS, no memory traffic), at one or two
// wavefronts per SIMD.  On a power-limited part this is the practical ceiling a GEMM can be held
// against, next to the published peak.  Used by bench.py only.
#include "common.h"

namespace mixlora {

__global__ __launch_bounds__(256) void mfma_probe_kernel(float *__restrict__ sink, int iters) {
  constexpr int NACC = 8;
  f32x16_t acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[i][e] = 0.f;
  bf16x8_t a, b;
#pragma unroll
  for (int e = 0; e < 8; e++) {
    unsigned h = (threadIdx.x * 8 + e) * 2654435761u + blockIdx.x * 40503u;
    h ^= h >> 13;
    h *= 2246822519u;
    h ^= h >> 16;
    a[e] = (bf16_t)(0.001f * (float)((int)(h & 0xffff) - 32768));
    b[e] = (bf16_t)(0.001f * (float)((int)(h >> 16) - 32768));
  }
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < NACC; i++)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(i & 1 ? a : b, i & 2 ? b : a, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) s += acc[i][e];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace mixlora

extern "C" int mixlora_mfma_probe(void *sink, size_t sink_bytes, int32_t waves_per_simd,
                                  int32_t iters, double *tflops, void *stream) {
  using namespace mixlora;
  if (!sink || !tflops) return MIXLORA_E_NULL;
  if (waves_per_simd < 1 || waves_per_simd > 2 || iters < 1 || iters > (1 << 20)) return MIXLORA_E_SHAPE;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return MIXLORA_E_HIP;
  const int blocks = cus * waves_per_simd;   // 4 waves per workgroup, 4 SIMDs per CU
  if (sink_bytes < (size_t)blocks * 256 * sizeof(float)) return MIXLORA_E_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return MIXLORA_E_HIP;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return MIXLORA_E_HIP; }
  int rc = MIXLORA_OK;
  float ms = 0.f;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, (float *)sink, iters);   // warm-up
  if (hipEventRecord(e0, st) != hipSuccess) rc = MIXLORA_E_HIP;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, (float *)sink, iters);
  if (hipGetLastError() != hipSuccess || hipEventRecord(e1, st) != hipSuccess ||
      hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
    rc = MIXLORA_E_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == MIXLORA_OK) *tflops = (double)blocks * 4.0 * iters * 8.0 * 32768.0 / (ms * 1e-3) / 1e12;
  return rc;
}
