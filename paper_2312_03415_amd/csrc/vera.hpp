// VeRA on top of the LoRA computation graphs (the conclusion of arxiv 2312.03415 names VeRA among the
// adapters the method carries over to): frozen A [i,r], B [r,o], trainable vectors d [r], b [o],
//     Y = XW + s ((XA) diag(d)) B diag(b)  =  XW + s (XA) B~,      B~ = diag(d) B diag(b).
// So every forward / backward graph of the LoRA layer serves unchanged on (A, B~); what the LoRA backward
// returns as dB~ = s (XA)^T dY holds both vector gradients,
//     dd[k] = sum_j dB~[k,j] B[k,j] b[j],        db[j] = sum_k dB~[k,j] d[k] B[k,j],
// and dA is not needed.  Two element-wise kernels over the r x o factor (a few hundred KB) are all that
// is added; both reduce in a fixed order.  Internal to the library.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace rl {

// Bt[k,j] = d[k] * B[k,j] * b[j], product in fp32, rounded once
hipError_t vera_scale_run(int dtype, const void* B, int64_t ldb, const void* d, const void* b, void* Bt, int64_t ldt,
                          int64_t R, int64_t O, hipStream_t stream);
// dd / db (either may be null) from G = dB~ as above; fp32 sums, rounded once
hipError_t vera_grad_run(int dtype, const void* G, int64_t ldg, const void* B, int64_t ldb, const void* d,
                         const void* b, void* dd, void* db, int64_t R, int64_t O, hipStream_t stream);

}  // namespace rl
