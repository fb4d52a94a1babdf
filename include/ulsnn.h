/*
 * ulsnn -- single-precision GEMM and the one-hidden-layer MLP gradient built on it, for AMD MI355X (gfx950).
 *
 * The two operations are the hot path of the training method of "92c/MFlops/s, Ultra-Large-Scale
 * Neural-Network Training on a PIII Cluster": a Level-3 BLAS SGEMM (section 3) and the error gradient of a
 * one-hidden-layer network computed as a series of matrix products (section 4.2), summed over the training
 * patterns (section 4.3).
 *
 * Conventions shared by every entry point
 *   - All matrix and vector pointers are DEVICE pointers owned by the caller.  The library borrows them until
 *     the work it queued on the stream has run.  Nothing is copied to or from the host.
 *   - Matrices are ROW-major.  A leading dimension (lda, ldb, ldc) is the distance, in elements, between the
 *     starts of consecutive rows (the "stride" of section 3.4); it may exceed the row length.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only queue work:
 *     they return before it has run, and work of one call is ordered on that stream.
 *   - Every function returns a ulsnn_status.  Arguments are checked on the host BEFORE any HIP call; a call
 *     that returns ULSNN_ERR_NULL..ULSNN_ERR_UNSUPPORTED has queued nothing and touched no memory.
 *     ULSNN_ERR_HIP reports a failed launch (hipGetLastError after the launch).
 *   - No entry point allocates or frees device memory.  Scratch space comes from the caller (workspace).
 *   - Input operands must not overlap outputs.
 */
#ifndef ULSNN_H
#define ULSNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ulsnn_status {
    ULSNN_OK = 0,
    ULSNN_ERR_NULL = 1,        /* a required pointer is NULL                                   */
    ULSNN_ERR_TRANS = 2,       /* transa / transb is not one of N n T t C c                    */
    ULSNN_ERR_DIM = 3,         /* a negative size, or a network dimension < 1                  */
    ULSNN_ERR_LD = 4,          /* a leading dimension smaller than the stored row length       */
    ULSNN_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned (256 B) or smaller than required  */
    ULSNN_ERR_UNSUPPORTED = 6, /* a documented option this build does not implement            */
    ULSNN_ERR_HIP = 7          /* the HIP runtime refused a launch                             */
} ulsnn_status;

/*
 * SGEMM:  C = alpha * op(A) * op(B) + beta * C        (section 3.1; Level-3 BLAS SGEMM interface, row-major)
 *
 *   op(X) = X for trans 'N'/'n', X^T for 'T'/'t' ('C'/'c' is accepted and means 'T').
 *   op(A) is m x k, op(B) is k x n, C is m x n.  As stored, A is m x k ('N') or k x m ('T'), B is k x n ('N')
 *   or n x k ('T').  lda >= max(1, stored row length of A), likewise ldb; ldc >= max(1, n).
 *   Counts 2*m*n*k floating-point operations.
 *
 *   Reference-BLAS rules: m == 0 or n == 0 returns ULSNN_OK and touches nothing; k == 0 or alpha == 0 gives
 *   C = beta*C; with beta == 0, C is written WITHOUT being read (NaN or Inf already in C do not propagate).
 *   Only the m x n entries of C are written; padding columns (n .. ldc-1) are left as they are.
 *   Products are accumulated in fp32 on the matrix cores; the order of summation is unspecified.
 *   A, B read-only; pointers need only 4-byte alignment.  A or B NULL is an error unless that operand is
 *   never read (m, n == 0, or k == 0, or alpha == 0).
 *   lda and ldb may not exceed ULSNN_MAX_LD (the kernels keep 32-bit element offsets inside a tile of up to 256
 *   rows): a larger one returns ULSNN_ERR_UNSUPPORTED.  ldc has no such limit.
 */
#define ULSNN_MAX_LD (1 << 24)
int ulsnn_sgemm(char transa, char transb, int m, int n, int k, float alpha, const float *A, int lda,
                const float *B, int ldb, float beta, float *C, int ldc, void *hip_stream);

/*
 * The same operation with scratch memory for a deterministic k split (section 3.1's product; a product with few
 * tiles of C and a long k cannot fill 256 compute units otherwise).  The library's planner chooses tile shape and
 * number of k slices (at most what `workspace` holds partial products for: slices * m * n * 4 bytes; with less than
 * 2 * m * n * 4 bytes the call is ulsnn_sgemm); partial products are added in slice order, so the same call gives
 * the same bits.  workspace: device memory, 256-byte aligned (ULSNN_ERR_WORKSPACE otherwise), contents undefined on
 * return; may be NULL with workspace_bytes == 0.  Everything else as ulsnn_sgemm.
 */
int ulsnn_sgemm_ws(char transa, char transb, int m, int n, int k, float alpha, const float *A, int lda,
                   const float *B, int ldb, float beta, float *C, int ldc, void *workspace, size_t workspace_bytes,
                   void *hip_stream);

/*
 * Description of the network and of one gradient call (everything the 8-argument call below cannot carry).
 *
 *   Network (section 4.1, with the weight matrices stored transposed with respect to the paper's W_ih, W_ho):
 *     W1 is n_in x n_hid, W2 is n_hid x n_out, both dense row-major.
 *   b1[n_hid], b2[n_out]: optional biases.  The paper's network has none (section 5.1 counts
 *     400*480 + 480*3203 parameters): pass NULL for both.  If given, db1/db2 receive their gradients
 *     (b1, b2, db1, db2 are all NULL or all non-NULL).
 *   accumulate: 0 -> dW1, dW2, db1, db2 and loss are overwritten;
 *               1 -> the call ADDS to them (gradient and error are additive over patterns, section 4.3;
 *                    this is how an epoch is summed over chunks of patterns).
 *   operand_dtype: 0 = fp32 storage of W1, W2, X (the paper's precision; section 4.2 reports 32 bits to be enough).
 *                  1 = bf16 storage (section 4.2 notes that 16 bits can suffice for small nets): W1, W2 and X point
 *                      at bf16 values (upper 16 bits of an IEEE float, row-major, dense); H, the logits, dO and dA1
 *                      are bf16 as well (round to nearest even; dO is formed from the rounded logits inside the
 *                      products that use it) and multiplied on the bf16 matrix instructions; every
 *                      product accumulates in fp32; the softmax statistics (row maximum, sum of exponentials, the
 *                      label's logit) and with them the loss are taken from the fp32 accumulators of the output
 *                      layer before its logits are rounded; dW1, dW2, db1, db2 (and b1, b2) stay fp32.
 *                      Fastest when n_in and n_hid are multiples of 8 (16-byte rows); other sizes are correct but
 *                      use an element-wise fetch for the operands whose rows are not 16-byte aligned (W1 and W2
 *                      are re-laid out internally, X is not).  Any other value: ULSNN_ERR_UNSUPPORTED.
 *   n_in, n_hid and n_out may not exceed ULSNN_MAX_LD (ULSNN_ERR_UNSUPPORTED).
 *   workspace: device scratch of at least ulsnn_mlp_grad_workspace_bytes(desc, batch) bytes, 256-byte aligned.
 *     Its contents on entry do not matter and are undefined on return.  Two calls that may run concurrently
 *     (different streams) need different workspaces.
 */
typedef struct ulsnn_mlp_desc {
    int n_in, n_hid, n_out;
    const float *b1, *b2;
    float *db1, *db2;
    int accumulate;
    int operand_dtype;
    void *workspace;
    size_t workspace_bytes;
    void *hip_stream;
} ulsnn_mlp_desc;

/* Bytes of workspace ulsnn_mlp_grad needs for this network and batch (0 if desc is NULL or invalid).
 * Host-only computation; non-decreasing in batch and constant above an internal slab size. */
size_t ulsnn_mlp_grad_workspace_bytes(const ulsnn_mlp_desc *desc, int batch);

/*
 * Loss and gradient of the one-hidden-layer MLP over `batch` patterns (section 4.2):
 *
 *     H   = tanh(X W1 + 1 b1^T)                         hidden activations        [batch x n_hid]
 *     Z   = H W2 + 1 b2^T                               output pre-activations    [batch x n_out]
 *     P   = row softmax of Z;   loss = sum_r -ln P[r][labels[r]]
 *     dO  = P - onehot(labels)                          output delta (the role of the paper's Y_Delta)
 *     dW2 = H^T dO,  db2 = 1^T dO                       (the paper's grad_ho, transposed layout)
 *     dA1 = (dO W2^T) ** (1 - H ** H)                   hidden delta (the paper's H_Delta; ** elementwise)
 *     dW1 = X^T dA1, db1 = 1^T dA1                      (the paper's grad_ih, transposed layout)
 *
 *   Loss and gradients are sums over the patterns, not means.  The paper's own output stage (tanh outputs,
 *   squared error against a dense target matrix) is replaced by softmax / cross-entropy against integer labels.
 *   Counts batch * (4 n_in n_hid + 6 n_hid n_out) floating-point operations (section 6.2).
 *
 *   W1, W2, X [batch x n_in, dense row-major]: const device fp32 (bf16 if desc->operand_dtype == 1).
 *   labels[batch]: device int32; a label
 *   outside [0, n_out) marks a pattern that is ignored (zero delta, nothing added to the loss).
 *   dW1 [n_in x n_hid], dW2 [n_hid x n_out]: device fp32, dense.  loss: ONE device float.
 *   batch == 0 is valid: with accumulate == 0 the outputs are zeroed, with accumulate == 1 nothing changes.
 *   Large batches are processed in slabs of patterns internally; results are deterministic (no atomics):
 *   the same call on the same data gives the same bits.
 */
int ulsnn_mlp_grad(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                   const int32_t *labels, int batch, float *dW1, float *dW2, float *loss);

/*
 * ulsnn_mlp_grad for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same operation, kernels, results and error
 * rules as ulsnn_mlp_grad, but the scratch is a static device array inside the library of
 * ULSNN_STATIC_SCRATCH_BYTES bytes (held on every GPU the library runs on until the process ends); desc->workspace
 * and desc->workspace_bytes are ignored.  A network / batch whose ulsnn_mlp_grad_workspace_bytes exceeds that size
 * returns ULSNN_ERR_WORKSPACE and queues nothing.  The call allocates and frees nothing.  The array's address on the
 * current device is looked up on the first call on that device (or by ulsnn_static_scratch_init, which callers
 * that capture the call in a graph should run once, outside the capture, with the device current).  All calls on
 * one GPU share the one array: calls that may overlap on a GPU (different streams or host threads) race; order them.
 */
#define ULSNN_STATIC_SCRATCH_BYTES (64u << 20)
size_t ulsnn_static_scratch_bytes(void);
int ulsnn_static_scratch_init(void);
int ulsnn_mlp_grad_static(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                          const int32_t *labels, int batch, float *dW1, float *dW2, float *loss);

/*
 * Debug helper for the label rule above: *count (ONE device int64) = number of labels[0..batch) outside
 * [0, n_out), i.e. of patterns ulsnn_mlp_grad would ignore.  Asynchronous on hip_stream.  batch == 0 gives 0.
 */
int ulsnn_check_labels(const int32_t *labels, int64_t batch, int n_out, int64_t *count, void *hip_stream);

/*
 * Error-only evaluation (forward pass and loss, no gradient): what a line search calls between gradients.
 * Same network, operands, labels, workspace, accumulate and error rules as ulsnn_mlp_grad; only `loss` is
 * written ((+)= with accumulate).  db1 / db2 of the descriptor are ignored.
 * Counts 2 * batch * (n_in + n_out) * n_hid floating-point operations (section 6.2).
 */
int ulsnn_mlp_loss(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                   const int32_t *labels, int batch, float *loss);

/*
 * The paper's own output stage (sections 4.1, 4.2): tanh outputs and a summed squared error against a dense
 * target matrix T [batch x n_out, dense row-major, device fp32]:
 *
 *     Y = tanh(H W2 + 1 b2^T)                       eq. (nn)
 *     E = sum_r sum_c (Y[r][c] - T[r][c])^2         eq. (error): no 1/2, no 1/n; written to `loss`
 *     dZ = 2 (Y - T) ** (1 - Y ** Y),  dW2 = H^T dZ,  dA1 = (dZ W2^T) ** (1 - H ** H),  dW1 = X^T dA1
 *
 * dW1 and dW2 are the TRUE derivatives of E.  In the paper's notation (Y_Delta = (1 - Y**Y)**(T - Y),
 * grad_ho = Y_Delta^T * H, grad_ih = H_Delta^T * X, W_ho = W2^T, W_ih = W1^T): dW2 = -2 grad_ho^T and
 * dW1 = -2 grad_ih^T; the paper's "gradient" is an ascent direction of -E/2.
 * Operands fp32 or bf16 (desc->operand_dtype as for ulsnn_mlp_grad; T is fp32 in both cases; with bf16 operands the
 * output stage runs inside the output layer's epilogue: E is summed from the fp32 outputs, dZ is stored as bf16).
 * Everything else as ulsnn_mlp_grad.  ulsnn_mlp_mse is the error-only form (E alone).
 */
int ulsnn_mlp_grad_mse(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X, const float *T,
                       int batch, float *dW1, float *dW2, float *loss);
int ulsnn_mlp_mse(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X, const float *T,
                  int batch, float *loss);

/*
 * Gradient over a whole training set held in device memory, taken `chunk` patterns at a time and summed
 * (section 4.3: additive over patterns; section 6.2: each processor steps through its patterns a fixed
 * number at a time).  Equivalent to ulsnn_mlp_grad on patterns [0, chunk), then with accumulate = 1 on
 * [chunk, 2 chunk), ... ; desc->accumulate applies to the first chunk.  The workspace must satisfy
 * ulsnn_mlp_grad_workspace_bytes(desc, min(chunk, n_patterns)).  chunk < 1 is ULSNN_ERR_DIM.
 * n_patterns is 64-bit: X may hold more than 2^31 elements.
 */
int ulsnn_mlp_grad_epoch(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                         const int32_t *labels, int64_t n_patterns, int chunk, float *dW1, float *dW2,
                         float *loss);

/*
 * Diagnostic form of ulsnn_mlp_grad for measurement: the same work on the same kernels, with a HIP event
 * recorded on the stream at each stage boundary.  The call WAITS for the stream to finish and writes the
 * elapsed milliseconds of the ULSNN_MLP_STAGES stages to the HOST array stage_ms:
 *   0 hidden layer (H)            1 output layer (Z)        2 softmax, cross-entropy, output delta, loss sum
 *   3 backward products: hidden delta dA1 = dO W2^T and dW2 = H^T dO (one paired launch when both are k-split)
 *   4 their split-k reductions    5 dW1 = X^T dA1 product   6 its split-k reduction      7 bias gradients
 * (section 4.2 names the products; stages 4 and 6 are empty without a k split, 7 without biases).  Only batches that fit one
 * internal pass are accepted (1 <= batch <= 65536), otherwise ULSNN_ERR_UNSUPPORTED.  Creates and destroys
 * HIP events; allocates no device memory.
 */
#define ULSNN_MLP_STAGES 8
int ulsnn_mlp_grad_timed(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                         const int32_t *labels, int batch, float *dW1, float *dW2, float *loss,
                         float *stage_ms);

/*
 * Host-only diagnostic: writes to buf (NUL-terminated, truncated to buf_bytes) one line per matrix product of
 * the gradient (section 4.2) with the tile shape, tile grid, k split and modelled time this build would use
 * for `batch` patterns: for the first internal pass if the batch is processed in several, followed, when the last
 * pass is shorter, by a line "tail_rows=R" and the five lines of that pass.  The first line also
 * says whether the call would take the two-launch path for small networks instead (small_network_path=1: nets up
 * to 128-64-64 at up to 4096 patterns, softmax form, fp32).  Launches nothing.
 */
int ulsnn_mlp_grad_describe_plan(const ulsnn_mlp_desc *desc, int batch, char *buf, size_t buf_bytes);

/*
 * Optimiser step (section 4.2, last paragraph).  The paper names the ingredients -- the plain step
 * W := W - alpha grad E, the Polak-Ribiere conjugate-gradient direction, a line search built from an exponential
 * step-size scheme, a quadratic interpolation and a bracketing test on the SIGN of grad E . direction estimated
 * from few patterns -- without printing an algorithm; the functions below fix one.  All vectors are dense fp32
 * device arrays of n elements; scalar results are device floats unless stated; sums are taken in double in a
 * fixed order (deterministic).  `workspace` of the three vector calls: device memory, 256-byte aligned, at
 * least ULSNN_VEC_WORKSPACE_BYTES (else ULSNN_ERR_WORKSPACE).  Asynchronous on hip_stream.
 */
#define ULSNN_VEC_WORKSPACE_BYTES 16640

/* *result = sum_i x[i]*y[i]. */
int ulsnn_dot(int64_t n, const float *x, const float *y, float *result, void *workspace, size_t workspace_bytes,
              void *hip_stream);

/* y += alpha*x (alpha = -step, x = grad E gives the plain gradient step). */
int ulsnn_axpy(int64_t n, float alpha, const float *x, float *y, void *hip_stream);

/*
 * Polak-Ribiere direction: beta = g_new.(g_new - g_old) / g_old.g_old (0 if the denominator is 0), then
 * d := -g_new + beta*d in place.  g_old == NULL starts (or restarts) the sequence: d := -g_new, beta = 0 and d is
 * not read.  `beta`, if not NULL, receives the coefficient (device float).
 */
int ulsnn_cg_direction(int64_t n, const float *g_new, const float *g_old, float *d, float *beta, void *workspace,
                       size_t workspace_bytes, void *hip_stream);

/*
 * Line search along (d1, d2) for the softmax / cross-entropy network without biases, fp32 (biases or bf16
 * operands: ULSNN_ERR_UNSUPPORTED).  E0 = E(W) on all `batch` patterns.  Steps alpha_k = alpha0 * 2^k,
 * k = 0..max_doublings (<= 60): the first k at which grad E_sub(W + alpha_k d) . d >= 0, the gradient taken on the
 * first min(bracket_batch, batch) patterns only, closes the bracket [lo, hi] = [alpha_(k-1) or 0, alpha_k]; if none
 * does, the last two steps are the bracket.  E is evaluated (all patterns) at lo (E0 if lo = 0), (lo + hi)/2 and
 * hi; if the parabola through these is convex, also at its vertex clamped to the bracket.  The step with the
 * smallest E among those evaluated is applied: W := W + alpha d in place (W unchanged if that step is 0).
 * `result` is HOST memory.  The host reads device scalars only where it must decide what to launch next: it
 * synchronises hip_stream once per group of bracketing steps (groups of 2, 4, 8, 8, ... steps; all steps of a group
 * are evaluated, also those after
 * the one that closes the bracket: spare gradients on the small subset instead of a round trip each) and once at the
 * end; the vertex of the parabola, the comparison of the errors and the weight update use steps computed on the
 * device (when the parabola is not convex the midpoint is evaluated a second time in the vertex's place).  The
 * evaluation counts in `result` are the algorithm's own (what a sequential search would have evaluated).
 * desc->workspace must hold ulsnn_mlp_line_search_workspace_bytes(desc, batch) bytes (the gradient
 * workspace for `batch` patterns plus two weight-sized and two gradient-sized arrays); desc->accumulate is ignored.
 */
typedef struct {
    float alpha;               /* step applied */
    float loss;                /* E at that step */
    float loss0;               /* E before the step */
    float bracket_lo, bracket_hi;
    int error_evaluations;     /* forward-only passes over all patterns */
    int gradient_evaluations;  /* gradients on the bracketing subset */
} ulsnn_line_search_result;
size_t ulsnn_mlp_line_search_workspace_bytes(const ulsnn_mlp_desc *desc, int batch);
int ulsnn_mlp_line_search(const ulsnn_mlp_desc *desc, float *W1, float *W2, const float *d1, const float *d2,
                          const float *X, const int32_t *labels, int batch, int bracket_batch, float alpha0,
                          int max_doublings, ulsnn_line_search_result *result);

/*
 * The same operation as ulsnn_sgemm (section 3.1) with the blocking chosen by the caller instead of the built-in
 * planner (for autotuning, and for tests that must reach every tile shape): `tile_shape` is one of
 * ULSNN_TILE_*, `k_splits` >= 1 the number of slices the k range is cut into (slices are rounded up to the k
 * step of the tile shape, 16 or 64, so fewer may remain).  With more than one slice the partial products go to `workspace` (device
 * memory, 256-byte aligned, at least k_splits*m*n*4 bytes; else ULSNN_ERR_WORKSPACE) and are added in slice
 * order, so results are deterministic.  Argument rules, layout, ownership and error behaviour otherwise as
 * for ulsnn_sgemm.
 */
#define ULSNN_TILE_256x128 0   /* 8 wavefronts */
#define ULSNN_TILE_128x128_W8 1 /* 8 wavefronts */
#define ULSNN_TILE_128x128 2   /* 4 wavefronts */
#define ULSNN_TILE_128x64 3
#define ULSNN_TILE_64x128 4
#define ULSNN_TILE_64x64 5
#define ULSNN_TILE_64x64_K64 6 /* k step 64, 8 wavefronts: two groups of four each take half of every step; for
                                  launches too small to fill the chip */
#define ULSNN_TILE_160x128 7   /* 5 accumulator blocks per wavefront: no padding when a dimension is 480 */
#define ULSNN_TILE_64x64_K32 8 /* k step 32, 8 wavefronts in two groups as above */
#define ULSNN_TILE_COUNT 9
int ulsnn_sgemm_planned(int tile_shape, int k_splits, char transa, char transb, int m, int n, int k, float alpha,
                        const float *A, int lda, const float *B, int ldb, float beta, float *C, int ldc,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Host-only diagnostic: the tile shape, tile grid and modelled time ulsnn_sgemm would use for this product
 * (section 3.1's operation), one line in the format of the lines above.  Launches nothing.
 */
int ulsnn_sgemm_describe_plan(char transa, char transb, int m, int n, int k, char *buf, size_t buf_bytes);
/* The same for ulsnn_sgemm_ws with a workspace of `workspace_bytes` bytes (splits > 1: k is cut and reduced). */
int ulsnn_sgemm_ws_describe_plan(char transa, char transb, int m, int n, int k, size_t workspace_bytes, char *buf,
                                 size_t buf_bytes);

/*
 * Measurement aids (what a roofline fraction "at the measured clock" needs; the paper times wall clock, section 3.4).
 * ulsnn_device_info: compute units, maximum shader clock and rate of the constant wall clock of the current device
 * (kHz); any pointer may be NULL.  ULSNN_ERR_HIP without a device.
 * ulsnn_clock_probe: queues ONE wavefront on hip_stream that reads the shader cycle counter and the wall clock for
 * about window_ms milliseconds (0 < window_ms <= 1000; it ends by itself after a bounded number of readings) and
 * writes cycles_and_ticks[0] = shader cycles, [1] = wall-clock ticks elapsed (device memory, two 64-bit values).
 * Queued on a second stream beside a workload, cycles / ticks * wall clock rate is the shader clock under that load.
 */
int ulsnn_device_info(int *compute_units, int *max_shader_clock_khz, int *wall_clock_khz);
int ulsnn_clock_probe(double window_ms, unsigned long long *cycles_and_ticks, void *hip_stream);

/* Counting conventions (host-only): 2mnk (section 3.1) and batch*(4 n_in n_hid + 6 n_hid n_out) (section 6.2). */
double ulsnn_sgemm_flops(int m, int n, int k);
double ulsnn_mlp_grad_flops(int n_in, int n_hid, int n_out, int64_t batch);
/* 2 * batch * (n_in + n_out) * n_hid for one evaluation of the error alone (section 6.2). */
double ulsnn_mlp_loss_flops(int n_in, int n_hid, int n_out, int64_t batch);

/* Human-readable name of a status code (static storage; never NULL). */
const char *ulsnn_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int ulsnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ULSNN_H */
