// Matrix-core ceiling probe: a loop of independent bf16 MFMAs with nothing else going on, fed with
// zeros or with random operands.  MI355X runs under a power limit, so the sustained MFMA rate
// depends on how many operand bits toggle; kernels that multiply N(0,1)-like data cannot reach what
// the same loop reaches on zeros.  bench.py reports both figures next to the datasheet peak.
#include <hip/hip_runtime.h>

#include "../../include/runlora.h"
#include "gemm_engine.hpp"

namespace rl {

__global__ __launch_bounds__(512) void mfma_probe_kernel(float* out, int iters, int random_data) {
  constexpr int NA = 4, NB = 2;
  i32x4 a[NA], b[NB];
  unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  auto next16 = [&]() -> unsigned {  // a bf16 with random sign, exponent in [2^-2, 2^1], random mantissa
    h ^= h << 13; h ^= h >> 17; h ^= h << 5;
    const unsigned sign = (h >> 3) & 0x8000u, expo = (125u + ((h >> 9) & 3u)) << 7, man = (h >> 20) & 0x7Fu;
    return random_data ? (sign | expo | man) : 0u;
  };
  for (int i = 0; i < NA; ++i)
    for (int e = 0; e < 4; ++e) a[i][e] = (int)(next16() | (next16() << 16));
  for (int i = 0; i < NB; ++i)
    for (int e = 0; e < 4; ++e) b[i][e] = (int)(next16() | (next16() << 16));
  f32x16 acc[NA][NB];
  for (int i = 0; i < NA; ++i)
    for (int j = 0; j < NB; ++j)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                            __builtin_bit_cast(bf16x8, b[j]), acc[i][j], 0, 0, 0);
    if (random_data) {  // keep the operands changing, as a K loop does
#pragma unroll
      for (int i = 0; i < NA; ++i) a[i][it & 3] ^= 0x00400040;
    }
  }
  float s = 0.f;
  for (int i = 0; i < NA; ++i)
    for (int j = 0; j < NB; ++j)
      for (int v = 0; v < 16; ++v) s += acc[i][j][v];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace rl

extern "C" int runlora_probe_mfma(void* scratch, size_t scratch_bytes, int random_data, void* stream,
                                  double* tflops) {
  if (!scratch || !tflops) return RL_ERR_NULL;
  const int blocks = 256, threads = 512, iters = 3000, reps = 5;
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
  const double flops = (double)blocks * (threads / 64) * iters * 8.0 * 2.0 * 32 * 32 * 16 * reps;
  *tflops = flops / (ms * 1e-3) / 1e12;
  return RL_OK;
}
