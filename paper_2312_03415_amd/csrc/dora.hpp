// DoRA on top of the merged-weight computation graphs (the conclusion of arxiv 2312.03415 names DoRA among the
// adapters the method carries over to): with V = W + s A B, c[j] = ||V[:, j]||, trainable magnitudes m [o],
//     Y = X (V diag(g)) + 1 bias^T,   g = m / c,   c a constant of the backward pass (the published method
// detaches it).  With c fixed the layer is the LoRA layer on (W diag(g), A, B diag(g)), and in forward2 and in
// backward 4 / 5 / 7 / 8 the frozen weight enters only through M = W + s A B, which the merge kernel forms with
// W's columns scaled on the way: W diag(g) is never written.  What DoRA adds per step:
//   - one more pass of the merge kernel over W that stores nothing and sums (W + s A B)^2 per column
//     (merge.hpp, sq_partial), finished here into c and g;
//   - B~ = B diag(g) and dB = dB~ diag(g): r x o elements each;
//   - dm[j] = sum_t dY[t,j] (Y[t,j] - bias[j]) / m[j]: one pass over dY and the forward's output.
// All sums are fp32 in a fixed order.  Internal to the library; 16-bit types only.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace rl {

// c[j] = sqrt(sum over the `rows` rows of partial[.][j]), g[j] = m[j] / c[j]
hipError_t dora_norm_finish_run(int dtype, const float* partial, int rows, const void* m, float* c, float* g, int64_t O,
                                hipStream_t stream);
// g[j] = m[j] / c[j]
hipError_t dora_g_run(int dtype, const void* m, const float* c, float* g, int64_t O, hipStream_t stream);
// out[k,j] = in[k,j] * g[j], product in fp32, rounded once (in == out allowed)
hipError_t dora_colscale_run(int dtype, const void* in, int64_t ldi, const float* g, void* out, int64_t ldo, int64_t R,
                             int64_t O, hipStream_t stream);
// row slices of the dm pass (rows of `partial`, o floats each)
int dora_dm_slices(int64_t n, int64_t o);
// dm[j] = (sum_t dY[t,j] (Y[t,j] - bias[j])) / m[j]; bias may be null; partial: dora_dm_slices(n, o) * o floats
hipError_t dora_dm_run(int dtype, const void* dY, int64_t lddy, const void* Y, int64_t ldy, const void* bias, const void* m,
                       float* partial, void* dm, int64_t n, int64_t o, hipStream_t stream);

}  // namespace rl
