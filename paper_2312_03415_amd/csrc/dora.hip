// Small kernels of the DoRA layer (see dora.hpp).  Only the dm pass moves real data (it reads dY and Y once,
// 2 n o e bytes, HBM-bound); the others touch o or r x o elements.
#include "dora.hpp"

#include "gemm.hpp"

namespace rl {
namespace {

constexpr int kThreads = 256;

template <typename T>
__global__ __launch_bounds__(kThreads) void dora_norm_finish_kernel(const float* __restrict__ partial, int rows,
                                                                    const T* __restrict__ m, float* __restrict__ c,
                                                                    float* __restrict__ g, int O) {
  const int j = blockIdx.x * kThreads + threadIdx.x;
  if (j >= O) return;
  float sum = 0.f;
  for (int y = 0; y < rows; ++y) sum += partial[(int64_t)y * O + j];
  const float cj = sqrtf(sum);
  c[j] = cj;
  g[j] = (float)m[j] / cj;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void dora_g_kernel(const T* __restrict__ m, const float* __restrict__ c,
                                                          float* __restrict__ g, int O) {
  const int j = blockIdx.x * kThreads + threadIdx.x;
  if (j < O) g[j] = (float)m[j] / c[j];
}

template <typename T>
__global__ __launch_bounds__(kThreads) void dora_colscale_kernel(const T* in, int64_t ldi, const float* __restrict__ g, T* out,
                                                                 int64_t ldo, int R, int O) {
  const int j = blockIdx.x * kThreads + threadIdx.x;
  const int k = blockIdx.y;
  if (j >= O || k >= R) return;
  out[(int64_t)k * ldo + j] = (T)((float)in[(int64_t)k * ldi + j] * g[j]);
}

// A workgroup owns 128 columns and a slice of rows.  Thread (rr, cg) = (tid / 16, tid % 16) reads 16 bytes
// (8 columns) of dY and of Y from the rows rr, rr + 16, ... of the slice (a wave instruction covers four whole
// 256-byte row segments) and keeps 8 running sums; the 16 threads of a column group are then added in the
// order of rr through LDS.  Requires o % 8 == 0 and 16-byte aligned rows.
template <typename T>
__global__ __launch_bounds__(kThreads) void dora_dm_partial_kernel(const T* __restrict__ dY, int64_t lddy,
                                                                   const T* __restrict__ Y, int64_t ldy,
                                                                   const T* __restrict__ bias, float* __restrict__ partial,
                                                                   int n, int O, int rows_per_slice) {
  __shared__ float part[16][128];
  using V4 = __attribute__((__vector_size__(4 * sizeof(int)))) int;
  const int rr = threadIdx.x >> 4, cg = threadIdx.x & 15;
  const int j0 = blockIdx.x * 128 + cg * 8;
  const bool col_ok = j0 < O;
  float acc[8], bj[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    acc[e] = 0.f;
    bj[e] = (bias != nullptr && col_ok) ? (float)bias[j0 + e] : 0.f;
  }
  const int t0 = blockIdx.y * rows_per_slice;
  int t1 = t0 + rows_per_slice;
  if (t1 > n) t1 = n;
  if (col_ok) {
#pragma unroll 4
    for (int t = t0 + rr; t < t1; t += 16) {
      const V4 a = *reinterpret_cast<const V4*>(dY + (int64_t)t * lddy + j0);
      const V4 y = *reinterpret_cast<const V4*>(Y + (int64_t)t * ldy + j0);
      const T* a8 = reinterpret_cast<const T*>(&a);
      const T* y8 = reinterpret_cast<const T*>(&y);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += (float)a8[e] * ((float)y8[e] - bj[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rr][cg * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < 128) {
    const int j = blockIdx.x * 128 + threadIdx.x;
    float sum = part[0][threadIdx.x];
#pragma unroll
    for (int q = 1; q < 16; ++q) sum += part[q][threadIdx.x];
    if (j < O) partial[(int64_t)blockIdx.y * O + j] = sum;
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void dora_dm_finish_kernel(const float* __restrict__ partial, int rows,
                                                                  const T* __restrict__ m, T* __restrict__ dm, int O) {
  const int j = blockIdx.x * kThreads + threadIdx.x;
  if (j >= O) return;
  float sum = 0.f;
  for (int y = 0; y < rows; ++y) sum += partial[(int64_t)y * O + j];
  dm[j] = (T)(sum / (float)m[j]);
}

int rows_per_slice(int64_t n, int64_t o) {
  const int64_t gx = (o + 127) / 128;
  int64_t slices = 1024 / gx;  // about four workgroups per compute unit
  if (slices < 1) slices = 1;
  int64_t rows = (n + slices - 1) / slices;
  rows = (rows + 15) / 16 * 16;
  if (rows < 64) rows = 64;
  return (int)rows;
}

template <typename T>
hipError_t dm_t(const void* dY, int64_t lddy, const void* Y, int64_t ldy, const void* bias, const void* m, float* partial,
                void* dm, int64_t n, int64_t o, hipStream_t s) {
  const int rows = rows_per_slice(n, o), slices = dora_dm_slices(n, o);
  hipLaunchKernelGGL(dora_dm_partial_kernel<T>, dim3((unsigned)((o + 127) / 128), (unsigned)slices), dim3(kThreads), 0, s,
                     static_cast<const T*>(dY), lddy, static_cast<const T*>(Y), ldy, static_cast<const T*>(bias), partial,
                     (int)n, (int)o, rows);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(dora_dm_finish_kernel<T>, dim3((unsigned)((o + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, partial,
                     slices, static_cast<const T*>(m), static_cast<T*>(dm), (int)o);
  return hipGetLastError();
}

template <typename T>
hipError_t colscale_t(const void* in, int64_t ldi, const float* g, void* out, int64_t ldo, int64_t R, int64_t O, hipStream_t s) {
  if (R > 65535) return hipErrorInvalidValue;  // r <= 128 here
  hipLaunchKernelGGL(dora_colscale_kernel<T>, dim3((unsigned)((O + kThreads - 1) / kThreads), (unsigned)R), dim3(kThreads), 0, s,
                     static_cast<const T*>(in), ldi, g, static_cast<T*>(out), ldo, (int)R, (int)O);
  return hipGetLastError();
}

}  // namespace

int dora_dm_slices(int64_t n, int64_t o) {
  const int rows = rows_per_slice(n, o);
  return (int)((n + rows - 1) / rows);
}

hipError_t dora_norm_finish_run(int dtype, const float* partial, int rows, const void* m, float* c, float* g, int64_t O,
                                hipStream_t stream) {
  const dim3 grid((unsigned)((O + kThreads - 1) / kThreads));
  if (dtype == DT_F16)
    hipLaunchKernelGGL(dora_norm_finish_kernel<_Float16>, grid, dim3(kThreads), 0, stream, partial, rows,
                       static_cast<const _Float16*>(m), c, g, (int)O);
  else if (dtype == DT_BF16)
    hipLaunchKernelGGL(dora_norm_finish_kernel<__bf16>, grid, dim3(kThreads), 0, stream, partial, rows,
                       static_cast<const __bf16*>(m), c, g, (int)O);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t dora_g_run(int dtype, const void* m, const float* c, float* g, int64_t O, hipStream_t stream) {
  const dim3 grid((unsigned)((O + kThreads - 1) / kThreads));
  if (dtype == DT_F16)
    hipLaunchKernelGGL(dora_g_kernel<_Float16>, grid, dim3(kThreads), 0, stream, static_cast<const _Float16*>(m), c, g, (int)O);
  else if (dtype == DT_BF16)
    hipLaunchKernelGGL(dora_g_kernel<__bf16>, grid, dim3(kThreads), 0, stream, static_cast<const __bf16*>(m), c, g, (int)O);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t dora_colscale_run(int dtype, const void* in, int64_t ldi, const float* g, void* out, int64_t ldo, int64_t R,
                             int64_t O, hipStream_t stream) {
  if (dtype == DT_F16) return colscale_t<_Float16>(in, ldi, g, out, ldo, R, O, stream);
  if (dtype == DT_BF16) return colscale_t<__bf16>(in, ldi, g, out, ldo, R, O, stream);
  return hipErrorInvalidValue;
}

hipError_t dora_dm_run(int dtype, const void* dY, int64_t lddy, const void* Y, int64_t ldy, const void* bias, const void* m,
                       float* partial, void* dm, int64_t n, int64_t o, hipStream_t stream) {
  if (dtype == DT_F16) return dm_t<_Float16>(dY, lddy, Y, ldy, bias, m, partial, dm, n, o, stream);
  if (dtype == DT_BF16) return dm_t<__bf16>(dY, lddy, Y, ldy, bias, m, partial, dm, n, o, stream);
  return hipErrorInvalidValue;
}

}  // namespace rl
