/*
 * runlora.h - C ABI of the MI355X (gfx950) LoRA-linear library.
 *
 * One layer of RunLoRA (arxiv 2312.03415, Section 2):
 *     forward   Y  = X W + (X A) B                      (Eq. 1; W frozen)
 *     backward  dA = X^T dY B^T,  dB = A^T X^T dY,
 *               dX = dY W^T + dY B^T A^T                (Eq. 3; no dW)
 * in each of the algebraically equivalent computation graphs the paper lists, plus the selector
 * that picks a (forward, backward) pair per shape.
 *
 * Beyond the paper's layer (which has neither): an optional LoRA scale s and an optional frozen
 * bias b of the base layer, Y = X W + 1 b^T + s (X A) B; the gradients of Eq. 3 then carry the
 * factor s on their adapter terms (dA = s X^T dY B^T, dB = s A^T X^T dY, dX = dY W^T + s dY B^T A^T)
 * and b, being frozen like W, has none.  LoRA dropout on the adapter's input is available too (the
 * paper's experiments run with dropout 0): Y = X W + 1 b^T + s/(1-p) ((X o m) A) B with a keep-mask m that
 * forward and backward regenerate from a seed.  See rl_opts_t.
 *
 * Notation (Table 1 caption): n = b*s tokens, i = d_in, o = d_out, r = LoRA rank.
 * All tensors are dense row-major DEVICE buffers described by rl_tensor_t:
 *     X [n,i]  W [i,o]  A [i,r]  B [r,o]  Y,dY [n,o]  dX [n,i]  dA [i,r]  dB [r,o]
 * (W is d_in x d_out because the paper writes Y = XW).
 *
 * Conventions shared by every entry point
 *   - Pointers inside rl_tensor_t / rl_saved_t / rl_opts_t.workspace are device pointers; the
 *     structs themselves and all int* outputs are host memory.
 *   - The caller owns every buffer.  The library allocates no device memory, frees nothing and
 *     keeps no pointer after a call returns, except those it writes into *saved.
 *   - Work is enqueued on opts->stream (a hipStream_t; NULL = the default stream) and the call
 *     returns without synchronising.  Buffers must stay alive until the stream has drained.
 *   - Outputs are overwritten, never accumulated into.
 *   - Return value: RL_OK (0) or a negative rl_status_t.  All argument checks happen before the
 *     first HIP call, so they behave the same on a host without a GPU.  No exception crosses
 *     the boundary.
 *   - Element types: RL_F32, RL_F16, RL_BF16 for every tensor of a call (one type per call).
 *     RL_INT4_G64 is allowed for W only (see rl_tensor_t), with RL_F16 / RL_BF16 activations: W is
 *     dequantised inside the GEMMs that read it (q * scale, rounded to the activation type) and
 *     never written out densely.  The graphs that need W + AB as a matrix (RL_FWD2, RL_BWD4,
 *     RL_BWD5, RL_BWD7, RL_BWD8) return RL_ERR_UNSUPPORTED for an int4 W.  Accumulation is fp32
 *     throughout; each result is rounded once (nearest even) to the storage type.
 *   - Alignment: data pointers 16-byte aligned; ld (elements between rows) >= cols and a
 *     multiple of 8 (16-bit types) or 4 (fp32); i, o and r multiples of 8 (16-bit) or 4 (fp32);
 *     n is arbitrary (>= 1).  Anything else returns RL_ERR_ALIGN / RL_ERR_SHAPE.
 */
#ifndef RUNLORA_H
#define RUNLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RL_F32 = 0,
  RL_F16 = 1,
  RL_BF16 = 2,
  RL_INT4_G64 = 3 /* frozen W only: symmetric int4, one fp16 scale per 64 rows (d_in) per column */
} rl_dtype_t;

typedef enum {
  RL_OK = 0,
  RL_ERR_NULL = -1,           /* a required pointer is NULL                                   */
  RL_ERR_SHAPE = -2,          /* dimensions of the tensors do not fit together, or are < 1    */
  RL_ERR_DTYPE = -3,          /* unknown dtype, or tensors of one call differ in dtype        */
  RL_ERR_VARIANT = -4,        /* unknown variant id                                           */
  RL_ERR_SAVED_MISMATCH = -5, /* *saved does not come from a forward this backward can use    */
  RL_ERR_ALIGN = -6,          /* pointer / ld / dimension alignment rule violated             */
  RL_ERR_ALIAS = -7,          /* an output buffer overlaps an input buffer                    */
  RL_ERR_WORKSPACE = -8,      /* workspace missing or smaller than runlora_workspace_bytes()  */
                              /* (runlora_last_hip_error() names the size needed)             */
  RL_ERR_UNSUPPORTED = -9,    /* legal request this build does not implement (e.g. merged-W   */
                              /* graphs on an int4 W)                                         */
  RL_ERR_HIP = -10            /* a HIP launch failed; runlora_last_hip_error() has the text   */
} rl_status_t;

/*
 * Forward computation graphs (Section 2, "major forward variants", and the default chain that
 * Section 2 contrasts them with).
 */
typedef enum {
  RL_FWD_DEFAULT = 0, /* T = XA kept for the backward; Y = XW; Y += T B.  One kernel per product. */
  RL_FWD1 = 1,        /* Y = (XW) + ((XA)B): T = XA, then one GEMM over the concatenated          */
                      /* contraction [X|T] [W;B]; T is scratch, not kept.                         */
  RL_FWD2 = 2,        /* Y = X (W + AB): M = W + AB, then Y = X M  (Eq. 2).                       */
  RL_FWD3 = 3         /* RL_FWD1's graph in ONE kernel: every workgroup of the GEMM forms its rows */
                      /* of T = XA next to X W (X is read once, T never reaches memory), rounds    */
                      /* them and contracts them with B as a last K tile.  r <= 32, dense W, no    */
                      /* dropout; otherwise the call runs as RL_FWD1.  No workspace when it applies.*/
} rl_fwd_variant_t;

/*
 * Backward computation graphs.  1..5 are Algorithms 1-5 of Section 2 (backward1..backward5); 6..8
 * are items 6-8 of the section's list of the eight bracketings of Eq. 3, which the paper leaves out
 * because Table 1 never ranks them first (the selector never returns them either).
 * Where a graph ends with dX = dY W^T + Z1 A^T the two products run as one GEMM over the
 * concatenated contraction [dY|Z1] [W^T;A^T].
 */
typedef enum {
  RL_BWD_DEFAULT = 0, /* autograd's backward of the default chain; needs T from RL_FWD_DEFAULT:  */
                      /* Z1 = dY B^T; dB = T^T dY; dA = X^T Z1; dX = dY W^T; dX += Z1 A^T.        */
  RL_BWD1 = 1,
  RL_BWD2 = 2,
  RL_BWD3 = 3,
  RL_BWD4 = 4,
  RL_BWD5 = 5,
  RL_BWD6 = 6, /* dA = (X^T dY) B^T;  dB = (A^T X^T) dY;  dX = dY W^T + (dY B^T) A^T */
  RL_BWD7 = 7, /* dA = (X^T dY) B^T;  dB = (A^T X^T) dY;  dX = dY (W^T + B^T A^T)    */
  RL_BWD8 = 8  /* dA = X^T (dY B^T);  dB = A^T (X^T dY);  dX = dY (W^T + B^T A^T)    */
} rl_bwd_variant_t;

/*
 * A dense row-major matrix in device memory.
 *   data   device pointer to element (0,0); for RL_INT4_G64: packed nibbles, two per byte, element
 *          (k,j) in byte (k*ld + j)/2, low nibble for even j, value = nibble - 8 in [-7,7]
 *          (ld a multiple of 8, data and scales 16-byte aligned)
 *   rows, cols, ld   in elements; ld = distance between consecutive rows
 *   dtype  rl_dtype_t
 *   scales RL_INT4_G64 only: device pointer to fp16 scales [ceil(rows/64), cols], row-major, dense
 *   group  RL_INT4_G64 only: must be 64
 */
typedef struct {
  void* data;
  int64_t rows, cols, ld;
  int32_t dtype;
  void* scales;
  int32_t group;
} rl_tensor_t;

/*
 * What a forward leaves for its backward (Section 2: RunLoRA forwards keep X but not XA).
 * Zero the struct, set the fields named below if wanted, and pass it to runlora_forward, which
 * fills the rest; runlora_backward reads it.  X is borrowed: the caller keeps the buffer alive and
 * unchanged until the backward has run.
 *   T  caller-provided [n,r] buffer (ldt elements per row, same dtype as X).  Set T/ldt BEFORE
 *      calling runlora_forward(RL_FWD_DEFAULT, ...), which fills it with s XA (required).  Optional
 *      for RL_FWD1 (and RL_FWD3, which then runs as RL_FWD1): s XA is written there instead of into
 *      the workspace and left for the backward, and RL_BWD1 / 5 / 6 / 7 read it instead of forming
 *      X A again (one pass over X saved, n*r elements held meanwhile: the memory Section 2 says the
 *      RunLoRA forwards do not spend, r/i of X).  A T left by RL_FWD_DEFAULT serves them as well.
 *      NULL: nothing is kept.  RL_FWD2 ignores it and sets it to NULL.
 *   M  optional caller-provided [i,o] buffer (ldm elements per row, same dtype as X).  Set M/ldm
 *      BEFORE calling runlora_forward(RL_FWD2, ...): W + s AB is then formed there instead of in
 *      the workspace and left for the backward, and RL_BWD4 / 5 / 7 / 8 read it instead of forming
 *      it again (one pass over W saved, i*o elements held meanwhile).  Valid only while W, A and B
 *      are what the forward saw.  NULL: nothing is kept.  Other forward variants set it to NULL.
 *   scale  the forward's LoRA scale (rl_opts_t.scale), applied again by the backward.
 * runlora_saved_bytes() tells how many bytes a forward keeps besides X.
 */
typedef struct {
  int32_t fwd_variant, dtype;
  int64_t n, i, o, r;
  const void* X;
  int64_t ldx;
  void* T;
  int64_t ldt;
  void* M;
  int64_t ldm;
  float scale;
  uint32_t dropout_thr, dropout_seed; /* the forward's dropout (rl_opts_t), 0 = none */
} rl_saved_t;

/*
 * Per-call options (zero the struct first).  workspace is device scratch of at least
 * runlora_workspace_bytes() bytes for the variant and shape of the call, 256-byte aligned; its
 * contents are undefined afterwards.  Two calls that share a workspace must be ordered on one
 * stream.
 *   scale  runlora_forward only: the LoRA scale s of Y = XW + s (XA) B (alpha / r in common use);
 *          0 means 1, the paper's layer.  The forward records it in *saved and the backward takes
 *          it from there.  It is applied in fp32 where a rank-r factor or W + s AB is formed
 *          (s XA, s dY B^T, s Z2 B^T, s A^T Z2), before that factor is rounded to the storage type.
 *   bias   runlora_forward only: device pointer to the base layer's frozen bias, o elements of
 *          the activation dtype, 16-byte aligned, added in fp32 by the GEMM that writes Y; NULL =
 *          no bias.  Ignored by runlora_backward and runlora_gemm (rl_gemm_t has its own).
 *   dropout_p, dropout_seed   runlora_forward only: LoRA dropout on the adapter's input, 0 = none.
 *          p is rounded to thr/256, thr = round(256 p) in [1, 255]; element (t, c) of X is kept iff
 *          byte (c & 3) of H(t * (i/4) + (c >> 2)) is >= thr, where H(x) = mix(x ^ mix(seed ^ 0x9E3779B9))
 *          and mix(x): x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16 (mod 2^32);
 *          kept elements are scaled by 256/(256-thr).  The forward records thr and seed in *saved and
 *          the backward regenerates the mask from them.  With dropout only RL_FWD_DEFAULT / RL_FWD1 and
 *          RL_BWD_DEFAULT / RL_BWD1 exist (the others merge AB into W or form X^T dY; they return
 *          RL_ERR_UNSUPPORTED), r must be <= 128 and n * ld(X) < 2^30 (the masked products run on the streaming kernel).
 */
typedef struct {
  void* stream;
  void* workspace;
  size_t workspace_bytes;
  float scale;
  const void* bias;
  float dropout_p;
  uint32_t dropout_seed;
} rl_opts_t;

/*
 * Forward pass in computation graph `variant` (rl_fwd_variant_t): Y = XW + (XA)B  (Eq. 1).
 * X, W, A, B are inputs (device), Y is overwritten, *saved (host struct) is filled.
 * opts may be NULL only if the variant needs no workspace and the default stream is meant.
 */
int runlora_forward(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                    const rl_tensor_t* B, rl_tensor_t* Y, rl_saved_t* saved, const rl_opts_t* opts);

/*
 * Backward pass in computation graph `variant` (rl_bwd_variant_t): the gradients of Eq. 3.
 * dY [n,o] and *saved (from the forward) are inputs together with W, A, B; dX, dA, dB are
 * overwritten.  Any of dX / dA / dB may be NULL: that gradient is skipped.
 * RL_BWD_DEFAULT requires saved->fwd_variant == RL_FWD_DEFAULT (it reads saved->T).
 */
int runlora_backward(int variant, const rl_tensor_t* dY, const rl_saved_t* saved,
                     const rl_tensor_t* W, const rl_tensor_t* A, const rl_tensor_t* B,
                     rl_tensor_t* dX, rl_tensor_t* dA, rl_tensor_t* dB, const rl_opts_t* opts);

/*
 * runlora_forward for callers that can neither allocate device memory nor hand over a workspace (code under HIP
 * graph capture, serving loops and harnesses that forbid hipMalloc): same arguments, same kernels, same results
 * bit for bit, but the variant's scratch (T = XA of RL_FWD1, W + AB of RL_FWD2, fp32 partials of a split
 * contraction) lives in a fixed array of RL_STATIC_SCRATCH_BYTES inside the library's device image instead of
 * opts->workspace, which is ignored.  The call allocates and frees nothing on the device.
 *   - A call whose variant and shape need more scratch than the array holds returns RL_ERR_WORKSPACE before
 *     anything is enqueued (runlora_workspace_bytes(variant, -1, ...) tells the need; runlora_last_hip_error()
 *     has both figures as text).
 *   - Every GPU the library runs on holds its own copy of the array until the process ends; the copy used is
 *     that of the calling thread's current device.
 *   - All calls on one GPU share that GPU's array, and it keeps the last call's contents (no call relies on
 *     them: every scratch element is written before it is read).  Calls that may overlap on one GPU (different
 *     streams, or several host threads) race on it: order them on one stream.
 */
#define RL_STATIC_SCRATCH_BYTES (16u << 20)
int runlora_forward_static(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                           const rl_tensor_t* B, rl_tensor_t* Y, rl_saved_t* saved, const rl_opts_t* opts);

/*
 * VeRA on the same computation graphs.  The paper's conclusion names VeRA among the LoRA variants its
 * method extends to and gives no formulas; the layer here is the published one in this header's
 * orientation: A [i,r] and B [r,o] frozen (random, shared between layers), trainable vectors d [r], b [o],
 *     Y  = X W + 1 bias^T + s ((X A) diag(d)) B diag(b)
 *     dX = dY W^T + s ((dY diag(b) B^T) diag(d)) A^T
 *     dd[k] = s sum_t (XA)[t,k] (dY diag(b) B^T)[t,k],      db[j] = s sum_t dY[t,j] ((XA) diag(d) B)[t,j].
 * It runs as the LoRA layer on (A, B~), B~ = diag(d) B diag(b) (r*o elements formed in the workspace, rounded
 * to the storage type like every rank-r factor): `variant` is any rl_fwd_variant_t / rl_bwd_variant_t, *saved
 * is the same record (a forward of one family may not be followed by a backward of the other), rl_opts_t
 * means the same (scale, bias, dropout, stream), and the vector gradients are reductions of the LoRA
 * graph's dB~ = s (XA)^T dY:  dd[k] = sum_j dB~[k,j] B[k,j] b[j],  db[j] = sum_k dB~[k,j] d[k] B[k,j]
 * (fp32 sums in a fixed order, rounded once).  No gradient is formed for A.
 *   d, b     device pointers, r and o elements of the activation dtype, 16-byte aligned
 *   dd, db   device pointers (same sizes, dtype, alignment), overwritten; either may be NULL (skipped),
 *            as may dX
 *   workspace  required: runlora_vera_workspace_bytes(fwd, bwd, ...) bytes (fwd or bwd < 0: that side only)
 * A kept W + s A B~ (rl_saved_t.M) is valid only while d and b are what the forward saw.
 */
int runlora_vera_forward(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                         const rl_tensor_t* B, const void* d, const void* b, rl_tensor_t* Y, rl_saved_t* saved,
                         const rl_opts_t* opts);
int runlora_vera_backward(int variant, const rl_tensor_t* dY, const rl_saved_t* saved, const rl_tensor_t* W,
                          const rl_tensor_t* A, const rl_tensor_t* B, const void* d, const void* b,
                          rl_tensor_t* dX, void* dd, void* db, const rl_opts_t* opts);
size_t runlora_vera_workspace_bytes(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype);

/*
 * DoRA on the merged-weight computation graphs.  The paper's conclusion names DoRA among the LoRA variants its
 * method extends to and gives no formulas; the layer here is the published one in this header's orientation
 * (output feature j = column j), with the column norm a constant of the backward pass as published:
 *     V = W + s A B,   c[j] = ||V[:, j]||_2,   g = m / c,   Y = X (V diag(g)) + 1 bias^T,    m [o] trainable
 *     dX = (dY diag(g)) V^T,   dA = s X^T ((dY diag(g)) B^T),   dB = s (X A)^T (dY diag(g)),
 *     dm[j] = sum_t dY[t,j] (X V)[t,j] / c[j]  =  sum_t dY[t,j] (Y[t,j] - bias[j]) / m[j].
 * With c fixed this is the LoRA layer on (W diag(g), A, B diag(g)).  W diag(g) is never formed: only the graphs
 * in which W enters through W + s A B alone exist (variant = RL_FWD2; RL_BWD4 / 5 / 7 / 8; anything else returns
 * RL_ERR_UNSUPPORTED), and there the kernel that forms W + s A B scales W's columns on the way.  16-bit dtypes,
 * r <= 128, no LoRA dropout (otherwise RL_ERR_UNSUPPORTED).  *saved and rl_opts_t mean what they mean for
 * runlora_forward / runlora_backward (scale, bias, stream; rl_saved_t.M keeps (W + s A B) diag(g), valid while
 * W, A, B and m are what the forward saw); a forward of one family may not be followed by a backward of another.
 *   m        device pointer, o elements of the activation dtype, 16-byte aligned; no element may be 0 if dm
 *            is asked for (dm divides by it; DoRA initialises m to the column norms of W)
 *   c        device pointer, o floats (fp32 whatever the dtype), 16-byte aligned: written by the forward (the
 *            column norms, fp32 sums of the unrounded W + s A B in a fixed order), read by the backward.  A
 *            zero column of W + s A B gives c = 0 and a non-finite g, as the definition does.
 *   Y        runlora_dora_backward: the forward's output [n,o], unchanged, required only for dm; the bias the
 *            forward added is taken from opts->bias of the backward call (NULL = none)
 *   dX, dA, dB, dm   overwritten; any may be NULL (skipped); dm has o elements of the activation dtype
 *   workspace  required: runlora_dora_workspace_bytes(fwd, bwd, ...) bytes (fwd or bwd < 0: that side only)
 */
int runlora_dora_forward(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                         const rl_tensor_t* B, const void* m, rl_tensor_t* Y, rl_saved_t* saved, float* c,
                         const rl_opts_t* opts);
int runlora_dora_backward(int variant, const rl_tensor_t* dY, const rl_saved_t* saved, const rl_tensor_t* W,
                          const rl_tensor_t* A, const rl_tensor_t* B, const void* m, const float* c,
                          const rl_tensor_t* Y, rl_tensor_t* dX, rl_tensor_t* dA, rl_tensor_t* dB, void* dm,
                          const rl_opts_t* opts);
size_t runlora_dora_workspace_bytes(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype);

/*
 * Choose the (forward, backward) pair of computation graphs for one layer shape, by estimated time
 * or by operation count (the selection step named in the abstract).  Pure host function,
 * thread-safe, no HIP call.  Uses the time model unless the environment variable
 * RUNLORA_CRITERION=flops asks for the Table 1 FLOP criterion.  dtype is the activation dtype;
 * pass RL_INT4_G64 to restrict the choice to the graphs an int4 W supports.
 * Debugging overrides: RUNLORA_FORCE_FWD=<rl_fwd_variant_t id> and RUNLORA_FORCE_BWD=<rl_bwd_variant_t
 * id> in the environment pin that side of the pair.  The other side stays the selector's, except that
 * it is moved to keep the pair legal (a forced default backward takes the default forward with it; a
 * forced non-default forward turns a selected default backward into RL_BWD1).  RL_ERR_VARIANT if a
 * value is not an id or both are forced to an illegal pair, RL_ERR_UNSUPPORTED if a forced graph does
 * not exist for an int4 W.  runlora_select_by ignores them.
 */
int runlora_select(int64_t n_tokens, int64_t d_in, int64_t d_out, int64_t r, int dtype,
                   int* fwd_variant, int* bwd_variant);

/* Same, with the criterion explicit: 0 = Table 1 FLOPs (ties -> lower id), 1 = time model,
 * 2 = time model for a caller that lets forward2 keep W + AB for the backward (rl_saved_t.M):
 * pairs of forward2 with backward4 / 5 are then priced without the second W + AB pass;
 * 3 = time model for a caller that lets forward1 keep T = XA (rl_saved_t.T): forward1 with
 * backward1 / 5 is then priced without the second X A pass. */
int runlora_select_by(int criterion, int64_t n_tokens, int64_t d_in, int64_t d_out, int64_t r,
                      int dtype, int* fwd_variant, int* bwd_variant);

/*
 * Table 1 closed forms.  is_bwd = 0: variant 1,2 = forward1,2 (0 = default chain = forward1's
 * products).  is_bwd = 1: variant 1..8 = backward1..8 (0 = default chain = backward1 minus the
 * XA recompute).  Returns -1 for an unknown variant.
 */
int64_t runlora_flops(int is_bwd, int variant, int64_t n, int64_t i, int64_t o, int64_t r);

/* Modelled time in microseconds of one variant on MI355X (what criterion 1 minimises);
 * negative for an unknown variant. */
double runlora_model_time_us(int is_bwd, int variant, int64_t n, int64_t i, int64_t o, int64_t r,
                             int dtype);

/*
 * Bytes a forward variant keeps for its backward besides X itself: n*r elements for the default
 * chain's T = XA, nothing for forward1 / forward2 (the memory saving of Section 2), plus what the
 * caller asks to be kept (keep_merged is a bit set): bit 0, i*o elements if forward2 keeps W + AB
 * (rl_saved_t.M); bit 1, n*r elements if forward1 / forward 3 keeps T = XA (rl_saved_t.T).
 * 0 for an unknown variant.
 */
size_t runlora_saved_bytes(int fwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype, int keep_merged);

/* Scratch bytes needed by a forward variant (bwd < 0), a backward variant (fwd < 0), or the
 * larger of the two, for a dense W of the layer dtype and tensors with dense rows (ld = columns).
 * Which kernel a rank-r product runs on depends on its operands' extents in memory, so a call on
 * tensors with padded rows whose extent reaches 2 GiB may need more: it then returns
 * RL_ERR_WORKSPACE and runlora_last_hip_error() names the size.  0 for an unknown variant or dtype. */
size_t runlora_workspace_bytes(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r,
                               int dtype);
/* Same with W's dtype explicit: w_dtype = dtype (dense) or RL_INT4_G64. */
size_t runlora_workspace_bytes_w(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r,
                                 int dtype, int w_dtype);

/*
 * The building block every step above is made of, exposed for tests, tuning and calibration of
 * the selector's time model:  C[M,N] = op(A)[M,K] op(B)[K,N] (+ op(A2)[M,K2] op(B2)[K2,N]) (+ D)
 * on the matrix cores with fp32 accumulation.
 *   a_strided  0: A (and A2) stored [M,K] row-major;  1: stored [K,M]   (X^T dY style)
 *   b_kcontig  0: B (and B2) stored [K,N] row-major;  1: stored [N,K]   (dY W^T style)
 *              (a_strided = 1 with b_kcontig = 1 is not provided)
 *   K2 = 0     no second segment.   D = NULL: no addend (D may alias C).
 *   tile_cfg   -1 = library heuristic; 0..5 = 256x256, 128x128, 128x32, 128x64, 32x128, 64x128
 *              output tile per workgroup in the generic engine; 6 / 7 = the matrix-core kernels for
 *              the large contractions (256x256 tile, 4 wavefronts, operands straight from global
 *              memory to LDS by LDS-DMA loads, epilogue staged through LDS so that whole row segments
 *              are stored; 16-bit types, fp32 falls back to 0; a call whose M and N are multiples of
 *              256 and that has no addend, bias or alpha runs a build with a shorter epilogue, same
 *              results): 6 = K tile 32, LDS ring of 3 stages, 32x32x16 products (also the route of an
 *              int4 W); 7 = K tile 64, 2 LDS stages, 16x16x32 products (what the heuristic picks for
 *              dense operands); 8 = the
 *              streaming kernel for rank-r products (N <= 128, no second segment, no addend:
 *              4 wavefronts per 32 output rows split the contraction)
 *   trans_out  1 = store C transposed, as [N,M] with ldc >= M (streaming kernel only); else 0
 *   splits     0 = heuristic, n > 0 = split the contraction n ways (fp32 partials in the
 *              workspace, summed in a fixed order)
 *   alpha      C = alpha * (the products) + D + bias; 0 means 1
 *   bias       NULL, or a row vector of N elements added to every row (16-byte aligned; not with
 *              the streaming kernel)
 * Same dtype / alignment rules as the layer calls (M arbitrary when A is [M,K]; every other
 * dimension a multiple of 8, or 4 for fp32).  Workspace: runlora_gemm_workspace_bytes().
 */
typedef struct {
  int32_t dtype, a_strided, b_kcontig, tile_cfg, splits;
  int64_t M, N, K, K2;
  const void *A, *B, *A2, *B2, *D;
  void* C;
  int64_t lda, ldb, lda2, ldb2, ldc, ldd;
  int32_t trans_out;
  float alpha;
  const void* bias;
} rl_gemm_t;
int runlora_gemm(const rl_gemm_t* g, const rl_opts_t* opts);
size_t runlora_gemm_workspace_bytes(const rl_gemm_t* g);

/*
 * Per-kernel timing, for measurement runs (the bench's roofline figures, calibration of the time
 * model).  While enabled, every layer call made from this thread records a pair of HIP events
 * around each step it enqueues (at most max_steps per collect; further steps go untimed).
 * runlora_profile_collect waits for the recorded events, writes one rl_step_time_t per step in
 * launch order (up to cap), forgets them, and returns how many it wrote (or a negative status).
 * `what` points to a static string naming the product in the paper's notation; flops = 2*M*N*K of
 * that product; bytes = one read of each operand plus the output (and addend) in the storage
 * dtype.  us is the time between the two events around the step (all of its kernels plus a few microseconds of
 * event handling).  After runlora_profile_kernel_times(1) (per thread, off by default) every kernel the step
 * launches (its main kernel, the launch for cut-off tile columns if the plan has one, the reduce pass behind a
 * split contraction) gets a pair of events bound to its own dispatch: kernel_us is the sum of those kernels'
 * durations (what a kernel trace reports for them, added up), main_us the first (main) kernel's alone, kernels
 * how many were timed; us then also holds the handling of those events.  Otherwise kernel_us = main_us = us
 * and kernels = 0.
 * tile_cfg names the kernel that ran the step: 0..7 as in rl_gemm_t, 8 / 9 / 10 = the streaming kernel with up to
 * 32 / 64 / 128 output columns, 11 = the W + alpha A B kernel (also the default chain's rank-r updates).
 * Events are host objects created at enable and destroyed at disable; no device memory.
 */
typedef struct {
  const char* what;
  double us;
  double flops, bytes;
  int64_t M, N, K;
  int32_t tile_cfg, splits, a_strided, b_kcontig;
  double kernel_us;
  double main_us;
  int32_t kernels;
} rl_step_time_t;
int runlora_profile_enable(int max_steps);
int runlora_profile_kernel_times(int on);
int runlora_profile_collect(rl_step_time_t* out, int cap);
int runlora_profile_disable(void);

/*
 * Measure what the matrix cores sustain on this GPU with nothing else running: back-to-back bf16
 * MFMAs (16x16x32, the matrix-core GEMM's product; one wave per SIMD, operands held in registers)
 * on zeros (random_data = 0) or on operands drawn roughly from N(0, 1) (random_data = 1).
 * The chip is power-limited, so the two differ; the second is the ceiling for N(0,1)-like data.
 * scratch: device buffer of at least 512 KiB (overwritten).  Synchronises the stream.  Result in
 * TFLOP/s through *tflops (host).  For measurement reports only.
 */
int runlora_probe_mfma(void* scratch, size_t scratch_bytes, int random_data, void* stream, double* tflops);

const char* runlora_strerror(int code);
const char* runlora_last_hip_error(void); /* text of the last RL_ERR_HIP (and the byte counts of the last RL_ERR_WORKSPACE) on this thread */
int runlora_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RUNLORA_H */
