/*
 * tesseract.h -- C ABI of the MI355X (gfx950) library for the per-processor
 * compute of a linear layer partitioned over a Tesseract [q, q, d] grid.
 *
 * Problem statement (Section 3.1 and Alg. 3 of the Tesseract paper): the
 * p = d*q*q processors form a [q, q, d] grid, 1 <= d <= q.  A[a,b] is cut
 * into q*d block rows and q block columns, B[b,c] into q x q blocks that every
 * depth layer holds, C[a,c] like A.  Processor (i,j,k) owns block row
 * h = i + k*q.  With m = a/(q*d), kb = b/q, n = c/q the blocks are [m,kb],
 * [kb,n] and [m,n].  At step t = 0..q-1 the processor receives A_{i,t,k} by a
 * broadcast along its grid row and B_{t,j} by a broadcast along its grid
 * column and accumulates their product.  This library does the accumulation
 * of all q steps in one kernel launch: the panels that the broadcasts would
 * deliver are passed as q device pointers per operand.
 *
 * Conventions common to every entry point
 *  - `*_panels` are HOST arrays of q DEVICE pointers.  The pointers are copied
 *    into the kernel arguments at the call; the array may be freed afterwards.
 *  - All matrices are row-major.  Leading dimensions (ld*) are in ELEMENTS and
 *    are shared by the q panels of one operand, so a panel may be a packed
 *    receive buffer (ld = row length) or a view into a larger matrix.
 *  - Ownership: the caller owns every buffer, including the workspace.  The
 *    library allocates nothing, keeps no state between calls (apart from having
 *    set a launch attribute of its kernels once per device) and never
 *    synchronises; calls that share a workspace must be ordered (same stream); kernels are enqueued on `hip_stream` (a hipStream_t cast to
 *    void*, NULL = the default stream) of the current device.
 *  - Errors: a status code is returned, nothing is thrown or aborted.  All
 *    argument checks happen before the first HIP call, so they work on a
 *    host without a GPU; on a non-OK status no output has been touched.
 *  - Inputs must not alias outputs.  q <= TESS_MAX_Q.
 *  - in_dtype TESS_BF16 computes bf16 x bf16 products on the matrix cores with
 *    fp32 accumulation over all q steps; TESS_F32 uses fp32 fused multiply-add.
 *    Down-casts to bf16 round to nearest, ties to even.
 *  - Results are deterministic run to run (no floating-point atomics).
 */
#ifndef TESSERACT_H_
#define TESSERACT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TESS_MAX_Q 16

typedef enum {
    TESS_OK = 0,
    TESS_ERR_NULL = 1,        /* a required pointer (descriptor, panel, output) is NULL      */
    TESS_ERR_GRID = 2,        /* q<1, d<1, d>q, q>TESS_MAX_Q or a coordinate outside the grid */
    TESS_ERR_SHAPE = 3,       /* a%(q*d), b%q or c%q non-zero, a size < 1, or ld < row length */
    TESS_ERR_ALIGN = 4,       /* bf16 matrix-core plan, but a panel pointer is not 16-byte
                                 aligned or a leading dimension is no multiple of 8          */
    TESS_ERR_UNSUPPORTED = 5, /* dtype / activation / flag combination not implemented        */
    TESS_ERR_WORKSPACE = 6,   /* workspace NULL or smaller than tess_linear_workspace_bytes   */
    TESS_ERR_HIP = 7          /* a HIP runtime call (kernel launch) failed                    */
} tess_status;

typedef enum { TESS_F32 = 0, TESS_BF16 = 1 } tess_dtype;

/* Activation of the fused epilogue.  The paper's MLP has "an activation" between
 * its two linear layers without naming it; GELU in its exact (erf) and tanh
 * forms are offered. */
typedef enum { TESS_ACT_NONE = 0, TESS_ACT_GELU_ERF = 1, TESS_ACT_GELU_TANH = 2 } tess_act;

typedef enum { TESS_OP_FWD = 0, TESS_OP_BWD_DX = 1, TESS_OP_BWD_DW = 2,
               TESS_OP_BWD_DX_STEP = 3, TESS_OP_BWD_DW_STEP = 4 } tess_op;

/* The problem as the paper states it: the grid, this processor's coordinates and
 * the GLOBAL matrix sizes (Alg. 3 inputs). */
typedef struct {
    int32_t q, d;      /* grid [q, q, d], 1 <= d <= q                      */
    int32_t i, j, k;   /* this processor: 0 <= i,j < q, 0 <= k < d         */
    int64_t a, b, c;   /* A[a,b] (activations), B[b,c] (weights), C[a,c]   */
    int32_t in_dtype;  /* tess_dtype of every input block (and of bias)    */
    int32_t out_dtype; /* tess_dtype of c_out / preact_out / dx_out / dw_out
                          (dw_out is fp32 regardless when accumulate != 0) */
} tess_desc;

/* Forward (Alg. 3 inner loop, then the bias add of Section 3.2.2 and the MLP
 * activation):   C_{i,j,k} = act( sum_{t<q} A_{i,t,k} * B_{t,j} + bias_j ).
 *   a_panels[t] : device, [m, kb], leading dimension lda   (block A_{i,t,k})
 *   b_panels[t] : device, [kb, n], leading dimension ldb   (block B_{t,j})
 *   bias        : device, [n] in in_dtype (slice j of the bias), or NULL
 *   c_out       : device, [m, n], ldc, out_dtype
 *   preact_out  : device, [m, n], ldc, out_dtype, or NULL: receives the sum plus
 *                 bias before the activation (what a GELU backward needs); asking for it
 *                 does not change c_out
 *   TESS_ACT_GELU_ERF is evaluated in fp32 with the library erf when c_out is fp32 and,
 *   when c_out is bf16, with a branch-free erfc form whose absolute error (< 5e-7) is far
 *   below a bf16 step: the two are different roundings of the same function, and a bf16
 *   result is not always the rounding of the fp32 result.
 *   workspace   : device scratch of >= tess_linear_workspace_bytes(desc, TESS_OP_FWD)
 *                 bytes, 256-byte aligned; may be NULL when that size is 0.        */
tess_status tess_linear_fwd(const tess_desc* desc,
                            const void* const* a_panels, int64_t lda,
                            const void* const* b_panels, int64_t ldb,
                            const void* bias, int act,
                            void* c_out, int64_t ldc, void* preact_out,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Input gradient (A' = C' B^T of the SUMMA gradient equation, Section 2.2; the
 * C = A B^T procedure of Section 3.1), computed on the owner of the block:
 *   dX_{i,j,k} = sum_{t<q} dY_{i,t,k} * (W_{j,t})^T.
 *   dy_panels[t] : device, [m, n],  lddy   (block dY_{i,t,k})
 *   w_panels[t]  : device, [kb, n], ldw    (block row j, block column t of W)
 *   dx_out       : device, [m, kb], lddx, out_dtype                               */
tess_status tess_linear_bwd_dx(const tess_desc* desc,
                               const void* const* dy_panels, int64_t lddy,
                               const void* const* w_panels, int64_t ldw,
                               void* dx_out, int64_t lddx,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Weight gradient of depth layer k (B' = A^T C', Section 2.2; the C = A^T B
 * procedure of Section 3.1):
 *   dW^(k)_{i,j} = sum_{t<q} (X_{t,i,k})^T * dY_{t,j,k}.
 *   x_panels[t]  : device, [m, kb], ldx    (block row t + k*q, block column i of X)
 *   dy_panels[t] : device, [m, n],  lddy   (block row t + k*q, block column j of dY)
 *   dw_out       : device, [kb, n], lddw
 *   accumulate   : 0 -> dw_out (out_dtype) is overwritten.
 *                  1 -> dw_out is fp32 and the result is ADDED to it: d calls with
 *                  k = 0..d-1 into one buffer form the sum over the depth layers
 *                  that Section 3.1 obtains with an all-reduce.                   */
tess_status tess_linear_bwd_dw(const tess_desc* desc,
                               const void* const* x_panels, int64_t ldx,
                               const void* const* dy_panels, int64_t lddy,
                               void* dw_out, int64_t lddw, int accumulate,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* tess_linear_bwd_dw for callers that cannot allocate or hand over device memory at the
 * call: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments and results as tess_linear_bwd_dw without the workspace: the
 * K-split partial sums go to a scratch array that is part of the library's code object
 * (tess_noalloc_scratch_bytes() = 80 MiB per device, held until the process ends).  The
 * call allocates nothing; its first use on a device looks the array's address up.
 *   - A launch plan that needs more scratch than that returns TESS_ERR_WORKSPACE (check
 *     with tess_linear_workspace_bytes(desc, TESS_OP_BWD_DW)); nothing is enqueued then.
 *   - Every call on a device shares that device's array: calls that may overlap on one
 *     device (different streams, different threads) race on it and must be ordered by
 *     the caller.  Nothing in it has to start at zero (every partial tile is written
 *     before it is read), so the last call's contents do no harm.                     */
tess_status tess_linear_bwd_dw_noalloc(const tess_desc* desc,
                                       const void* const* x_panels, int64_t ldx,
                                       const void* const* dy_panels, int64_t lddy,
                                       void* dw_out, int64_t lddw, int accumulate,
                                       void* hip_stream);
size_t tess_noalloc_scratch_bytes(void);

/* Input gradient through the activation that produced this layer's input (the MLP's
 * middle activation, Section 2.4): the same sum as tess_linear_bwd_dx, multiplied
 * element by element by the derivative of `act` at the saved pre-activation,
 *   dZ_{i,j,k} = ( sum_{t<q} dY_{i,t,k} * (W_{j,t})^T ) .* act'(Z_{i,j,k}).
 *   preact : device, [m, kb], ldz, in in_dtype: what the previous layer's
 *            tess_linear_fwd wrote to preact_out (its sum plus bias).
 *   act    : TESS_ACT_NONE makes this call identical to tess_linear_bwd_dx.
 *   dz_out : device, [m, kb], lddz, out_dtype.  Must not alias preact.           */
tess_status tess_linear_bwd_dx_act(const tess_desc* desc,
                                   const void* const* dy_panels, int64_t lddy,
                                   const void* const* w_panels, int64_t ldw,
                                   const void* preact, int64_t ldz, int act,
                                   void* dz_out, int64_t lddz,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* Weight gradient as tess_linear_bwd_dw, plus the bias gradient of the same depth
 * layer from the dY panels the call already streams (Section 3.2, bias-add: the
 * gradients of block column j are reduced along the column to grid row 0; the q
 * panels dY_{t,j,k} are exactly that column's blocks):
 *   db^(k)_j[s] = sum_{t<q} sum_{r<m} dY_{t,j,k}[r, s].
 *   dbias_out : device, [n], always fp32; overwritten when accumulate == 0, added
 *               to when accumulate == 1 (the depth sum, like dw_out).              */
tess_status tess_linear_bwd_dw_bias(const tess_desc* desc,
                                    const void* const* x_panels, int64_t ldx,
                                    const void* const* dy_panels, int64_t lddy,
                                    void* dw_out, int64_t lddw, void* dbias_out, int accumulate,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* The backward as Section 3.1 words it (C = A B^T and C = A^T B procedures): one step's
 * partial product on the processor that holds the dY block, to be REDUCED by the caller
 * to the block's owner (the reduction itself, a collective, is not part of this library;
 * `accumulate` lets one GPU play all members of the reduce group into one buffer).
 * Summed over the group, the partials equal tess_linear_bwd_dx / tess_linear_bwd_dw.
 *
 * Step t of the input gradient on processor (i,j,k):
 *   P[m, kb] (+)= dY_{i,j,k} [m,n] * (W_{t,j})^T [n,kb],  reduced over j to owner (i,t,k).
 * Step t of the weight gradient on processor (i,j,k):
 *   P[kb, n] (+)= (X_{i,t,k})^T [kb,m] * dY_{i,j,k} [m,n], reduced over i to owner (t,j,k).
 *   dy_block : device [m, n], lddy;  w_block : device [kb, n], ldw;  x_block : device [m, kb], ldx
 *   partial_out : device, fp32 whatever out_dtype says; overwritten (accumulate 0) or added to (1). */
tess_status tess_linear_bwd_dx_step(const tess_desc* desc, const void* dy_block, int64_t lddy,
                                    const void* w_block, int64_t ldw,
                                    void* partial_out, int64_t ldp, int accumulate,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);
tess_status tess_linear_bwd_dw_step(const tess_desc* desc, const void* x_block, int64_t ldx,
                                    const void* dy_block, int64_t lddy,
                                    void* partial_out, int64_t ldp, int accumulate,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Layer normalisation of a hidden dimension spread over the q processors of a grid row
 * (Section 3.2, "Other procedure": every processor computes the sums of X and X^2 of its
 * block, the sums are all-reduced along the row, then E[X] = S1/n, Var[X] = S2/n - E[X]^2).
 * The all-reduce is the caller's; `accumulate` adds a further block's sums so that one GPU
 * can play the whole row.
 *   x        : device, [m, w] in `dtype` (a tess_dtype), ldx
 *   sums_out : device, [m, 2] fp32 packed: sum, sum of squares                      */
tess_status tess_layernorm_row_sums(const void* x, int64_t m, int64_t w, int64_t ldx, int dtype,
                                    void* sums_out, int accumulate, void* hip_stream);
/* xhat = (x - S1/n) / sqrt(S2/n - (S1/n)^2 + eps) with the REDUCED sums of the whole row,
 * n_total the full hidden size.  xhat_out: device, [m, w] in `dtype`, ldo; may equal x. */
tess_status tess_layernorm_normalize(const void* x, int64_t m, int64_t w, int64_t ldx, int dtype,
                                     const void* sums, int64_t n_total, float eps,
                                     void* xhat_out, int64_t ldo, void* hip_stream);

/* Backward of the same normalisation (the X' equation of Section 3.2, "Other procedure"):
 * with g = dJ/dxhat,  X' = (g - (xhat * sum(xhat g) + sum(g)) / n) / sqrt(Var[X] + eps).
 * The two row sums are local partial sums that the caller reduces along the grid row
 * (`accumulate` adds a further block's sums).
 *   xhat, g  : device, [m, w] in `dtype`, ldx / ldg
 *   sums_out : device, [m, 2] fp32: sum(xhat * g), sum(g)                              */
tess_status tess_layernorm_bwd_row_sums(const void* xhat, int64_t ldx, const void* g, int64_t ldg,
                                        int64_t m, int64_t w, int dtype, void* sums_out,
                                        int accumulate, void* hip_stream);
/* X' of one block from the REDUCED backward sums and the REDUCED forward sums (which give
 * Var[X]); dx_out: device, [m, w] in `dtype`, ldo; may equal g.                         */
tess_status tess_layernorm_bwd_apply(const void* xhat, int64_t ldx, const void* g, int64_t ldg,
                                     int64_t m, int64_t w, int dtype, const void* sums_bwd,
                                     const void* sums_fwd, int64_t n_total, float eps,
                                     void* dx_out, int64_t ldo, void* hip_stream);

/* Bytes of device scratch that the call `op` (a tess_op) needs for this
 * descriptor on the current device (0 when none).  TESS_OP_BWD_DX also covers
 * tess_linear_bwd_dx_act and TESS_OP_BWD_DW covers tess_linear_bwd_dw_bias; the *_STEP
 * codes are the single-step partial products.  Pure host arithmetic. */
size_t tess_linear_workspace_bytes(const tess_desc* desc, int op);

/* Launch shape that the call `op` would use for this descriptor: output macro tile and
 * number of K splits (1 = the whole q-step sum stays in one workgroup's registers; > 1 =
 * that many equal parts of the K range, whose partial sums go through the workspace and are
 * added in ascending K order by a reduction kernel that applies the epilogue).  tile 0 x 0
 * means the plain
 * fp32 kernel: fp32 inputs, or a bf16 block whose contiguous extents are no multiple of 8.
 * Pure host arithmetic.  A call whose plan uses the matrix cores needs 16-byte aligned
 * panel pointers and leading dimensions that are multiples of 8 elements, and returns
 * TESS_ERR_ALIGN otherwise (it never drops to the plain kernel silently); a panel of 4 GiB
 * or more returns TESS_ERR_UNSUPPORTED. */
tess_status tess_linear_plan(const tess_desc* desc, int op, int32_t* tile_m, int32_t* tile_n,
                             int32_t* k_splits);

/* Validates a descriptor alone (grid rules and divisibility). */
tess_status tess_desc_check(const tess_desc* desc);

/* Block shape of this descriptor: m = a/(q*d), kb = b/q, n = c/q. */
tess_status tess_block_shape(const tess_desc* desc, int64_t* m, int64_t* kb, int64_t* n);

/* Static, NUL-terminated name of a status code. */
const char* tess_status_string(int status);

/* Library version, "major.minor". */
const char* tess_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TESSERACT_H_ */
