// Matrix-core ceiling probe: a loop of bf16 MFMAs (16x16x32, the product the matrix-core GEMM is built
// from) with nothing else going on: one wave per SIMD, an 8 x 8 block of accumulators per wave, operands
// held in registers, every MFMA written out so that no loop arithmetic sits between them.  Fed with zeros
// or with operands drawn roughly from N(0, 1).  MI355X runs under a power limit, so the sustained MFMA
// rate depends on how many operand bits toggle; kernels that multiply N(0,1)-like data cannot reach what
// the same loop reaches on zeros.  bench.py reports both figures next to the datasheet peak.
#include <hip/hip_runtime.h>

#include "../../include/runlora.h"
#include "gemm_engine.hpp"

namespace rl {

__global__ __launch_bounds__(256) void mfma_probe_kernel(float* out, int iters, int random_data) {
  i32x4 a[8], b[8];
  unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  auto next16 = [&]() -> unsigned {  // a bf16 close to N(0, 1): twelve uniforms summed, minus six
    float s = -6.f;
    for (int k = 0; k < 12; ++k) {
      h ^= h << 13; h ^= h >> 17; h ^= h << 5;
      s += (float)(h >> 8) * (1.0f / 16777216.0f);
    }
    return random_data ? (__builtin_bit_cast(unsigned, s) >> 16) : 0u;
  };
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) a[i][e] = (int)(next16() | (next16() << 16));
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) b[i][e] = (int)(next16() | (next16() << 16));
  f32x4 acc[8][8];
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 8; ++j)
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 64; ++q)  // one operand held for eight products, the other changing: the GEMM's order
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[q >> 3][q & 7]) : "v"(a[q >> 3]), "v"(b[q & 7]));
  }
  asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");  // the last MFMAs finish before their results are read
  float s = 0.f;
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 8; ++j)
      for (int v = 0; v < 4; ++v) s += acc[i][j][v];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace rl

extern "C" int runlora_probe_mfma(void* scratch, size_t scratch_bytes, int random_data, void* stream,
                                  double* tflops) {
  if (!scratch || !tflops) return RL_ERR_NULL;
  const int blocks = 256, threads = 256, iters = 4000, reps = 5;
  if (scratch_bytes < (size_t)blocks * threads * sizeof(float)) return RL_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return RL_ERR_HIP;
  float* out = static_cast<float*>(scratch);
  hipLaunchKernelGGL(rl::mfma_probe_kernel, dim3(blocks), dim3(threads), 0, st, out, iters, random_data);
  hipError_t e = hipEventRecord(e0, st);
  for (int r = 0; r < reps; ++r)
    hipLaunchKernelGGL(rl::mfma_probe_kernel, dim3(blocks), dim3(threads), 0, st, out, iters, random_data);
  if (e == hipSuccess) e = hipEventRecord(e1, st);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess || ms <= 0.f) return RL_ERR_HIP;
  const double flops = (double)blocks * (threads / 64) * iters * 64.0 * 2.0 * 16 * 16 * 32 * reps;
  *tflops = flops / (ms * 1e-3) / 1e12;
  return RL_OK;
}
