// Element-wise kernels of the VeRA layer (see vera.hpp): the scaled factor B~ = diag(d) B diag(b) and the
// reduction of dB~ into the gradients of d and b.  Bound by nothing that matters: r x o elements.
#include "vera.hpp"

#include "gemm.hpp"

namespace rl {
namespace {

constexpr int kThreads = 256;

template <typename T>
__global__ __launch_bounds__(kThreads) void vera_scale_kernel(const T* __restrict__ B, int64_t ldb, const T* __restrict__ d,
                                                              const T* __restrict__ b, T* __restrict__ Bt, int64_t ldt,
                                                              int R, int O) {
  const int j = blockIdx.x * kThreads + threadIdx.x;
  const int k = blockIdx.y;
  if (j >= O || k >= R) return;
  const float v = (float)d[k] * (float)B[(int64_t)k * ldb + j] * (float)b[j];
  Bt[(int64_t)k * ldt + j] = (T)v;
}

// a workgroup owns 32 columns; thread (c, g) sums the rows k = g, g + 8, g + 16, ... of column c in that
// order, then the eight partial sums of a column are added in the order of g
template <typename T>
__global__ __launch_bounds__(kThreads) void vera_db_kernel(const T* __restrict__ G, int64_t ldg, const T* __restrict__ B,
                                                           int64_t ldb, const T* __restrict__ d, T* __restrict__ db, int R, int O) {
  __shared__ float part[8][32];
  const int c = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int j = blockIdx.x * 32 + c;
  float acc = 0.f;
  if (j < O) {
#pragma unroll 4
    for (int k = g; k < R; k += 8) acc += (float)G[(int64_t)k * ldg + j] * ((float)d[k] * (float)B[(int64_t)k * ldb + j]);
  }
  part[g][c] = acc;
  __syncthreads();
  if (g == 0 && j < O) {
    float sum = part[0][c];
#pragma unroll
    for (int q = 1; q < 8; ++q) sum += part[q][c];
    db[j] = (T)sum;
  }
}

// one workgroup per row k: every thread sums its columns j = tid, tid + 256, ... in order, then a
// fixed binary tree over the 256 partial sums
template <typename T>
__global__ __launch_bounds__(kThreads) void vera_dd_kernel(const T* __restrict__ G, int64_t ldg, const T* __restrict__ B,
                                                           int64_t ldb, const T* __restrict__ b, T* __restrict__ dd, int R, int O) {
  __shared__ float part[kThreads];
  const int k = blockIdx.x;
  float acc = 0.f;
  for (int j = threadIdx.x; j < O; j += kThreads)
    acc += (float)G[(int64_t)k * ldg + j] * ((float)B[(int64_t)k * ldb + j] * (float)b[j]);
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) dd[k] = (T)part[0];
}

template <typename T>
hipError_t scale_t(const void* B, int64_t ldb, const void* d, const void* b, void* Bt, int64_t ldt, int64_t R, int64_t O,
                   hipStream_t s) {
  // gridDim.y is limited to 65535: walk the rows in slabs
  for (int64_t k0 = 0; k0 < R; k0 += 65535) {
    const int rows = (int)((R - k0) < 65535 ? (R - k0) : 65535);
    dim3 grid((unsigned)((O + kThreads - 1) / kThreads), (unsigned)rows);
    hipLaunchKernelGGL(vera_scale_kernel<T>, grid, dim3(kThreads), 0, s, static_cast<const T*>(B) + k0 * ldb, ldb,
                       static_cast<const T*>(d) + k0, static_cast<const T*>(b), static_cast<T*>(Bt) + k0 * ldt, ldt, rows, (int)O);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <typename T>
hipError_t grad_t(const void* G, int64_t ldg, const void* B, int64_t ldb, const void* d, const void* b, void* dd, void* db,
                  int64_t R, int64_t O, hipStream_t s) {
  if (db) {
    hipLaunchKernelGGL(vera_db_kernel<T>, dim3((unsigned)((O + 31) / 32)), dim3(kThreads), 0, s,
                       static_cast<const T*>(G), ldg, static_cast<const T*>(B), ldb, static_cast<const T*>(d),
                       static_cast<T*>(db), (int)R, (int)O);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (dd) {
    hipLaunchKernelGGL(vera_dd_kernel<T>, dim3((unsigned)R), dim3(kThreads), 0, s, static_cast<const T*>(G), ldg,
                       static_cast<const T*>(B), ldb, static_cast<const T*>(b), static_cast<T*>(dd), (int)R, (int)O);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

hipError_t vera_scale_run(int dtype, const void* B, int64_t ldb, const void* d, const void* b, void* Bt, int64_t ldt,
                          int64_t R, int64_t O, hipStream_t stream) {
  switch (dtype) {
    case DT_F32: return scale_t<float>(B, ldb, d, b, Bt, ldt, R, O, stream);
    case DT_F16: return scale_t<_Float16>(B, ldb, d, b, Bt, ldt, R, O, stream);
    default: return scale_t<__bf16>(B, ldb, d, b, Bt, ldt, R, O, stream);
  }
}

hipError_t vera_grad_run(int dtype, const void* G, int64_t ldg, const void* B, int64_t ldb, const void* d,
                         const void* b, void* dd, void* db, int64_t R, int64_t O, hipStream_t stream) {
  switch (dtype) {
    case DT_F32: return grad_t<float>(G, ldg, B, ldb, d, b, dd, db, R, O, stream);
    case DT_F16: return grad_t<_Float16>(G, ldg, B, ldb, d, b, dd, db, R, O, stream);
    default: return grad_t<__bf16>(G, ldg, B, ldb, d, b, dd, db, R, O, stream);
  }
}

}  // namespace rl
