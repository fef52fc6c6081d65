/*
 * rmm.h -- C ABI of the randomized-matrix-multiplication (RMM) linear layer for
 * AMD MI355X (gfx950).
 *
 * The layer is the one of "Memory-Efficient Backpropagation through Large Linear
 * Layers" (arXiv 2201.13195), Section 2.1 and Algorithm 1: the forward pass
 * returns Y = X W^T (+ 1 b^T) and keeps only X_proj = S^T X (k x d_in) plus a
 * 16-byte PRNG state instead of X (N x d_in); the backward pass returns the exact
 * dX = dY W and the unbiased estimate dW = (S^T dY)^T X_proj, with the N x k
 * sketch S re-made from the state (it never exists in memory).
 *
 * Conventions shared by every entry point
 *   - Matrix arguments are DEVICE pointers to dense, row-major, contiguous
 *     arrays whose base address is 16-byte aligned.  The caller allocates and
 *     owns all of them; the library never allocates, frees or keeps a pointer.
 *   - `ws` is caller-provided device scratch of at least
 *     rmm_workspace_bytes(...) bytes (16-byte aligned); its contents are
 *     undefined on entry and on return.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     work is enqueued on it and the call returns without waiting.
 *   - Output buffers are overwritten; the one entry point that adds to what its
 *     outputs hold is rmm_backward_accumulate.
 *   - Return value: RMM_OK or a negative rmm_status_t.  Nothing is printed, no
 *     exception crosses the boundary, the process is never aborted.  Arguments,
 *     sizes and the workspace are checked before anything is launched, so
 *     RMM_ERR_INVALID_ARG, RMM_ERR_UNSUPPORTED, RMM_ERR_WORKSPACE and
 *     RMM_ERR_SCRATCH_LIMIT mean that no kernel ran.  RMM_ERR_LAUNCH (the HIP
 *     runtime refused a launch) can come after earlier kernels of the same call
 *     were enqueued; the outputs are then undefined.
 *   - The library holds no mutable global state and calls are re-entrant; the one exception is
 *     rmm_sketch_static, whose scratch array is shared by all calls on a GPU (see there).
 *   - dtype RMM_DTYPE_BF16: inputs, Y, dX, X_proj, dW are bfloat16 (round to
 *     nearest even from fp32 accumulators); bias / dbias are bfloat16 too and,
 *     like every other pointer, 16-byte aligned (a misaligned one is
 *     RMM_ERR_INVALID_ARG).
 *     dtype RMM_DTYPE_F32: everything is fp32.
 *
 * The sketch.  state = (seed, offset).  Entry (i, j) of S (token i, sketch
 * column j) is P[i][j] / sqrt(k), with P a pure function of (state, i, j) built
 * on Philox-4x32-10 with key (seed mod 2^32, seed div 2^32):
 *   Gaussian   (Eq. 5): call counter (i div 8, j, offset mod 2^32, offset div 2^32)
 *              gives words r0..r3; w = r[(i mod 8) div 2];
 *              u1 = ((w div 2^16) + 1/2) / 2^16, u2 = (w mod 2^16) / 2^16;
 *              P = sqrt(-2 ln u1) * (cos(2 pi u2) if i even, sin(2 pi u2) if i odd).
 *   Rademacher (Section 3.5): call counter (i div 128, j, offset lo, offset hi);
 *              t = i mod 128; bit = (r[t div 32] >> (t mod 32)) & 1; P = 1 - 2 bit.
 *   SORS       (subsampled orthonormal matrix with random signs: Section 2.1 names the family,
 *              Section 3.5 and the future-work paragraph its O(B N log B) product; the paper gives
 *              no construction, this one is the subsampled randomized Walsh-Hadamard transform):
 *              n_pad = smallest power of two >= n;
 *              sigma_i = the Rademacher entry of token i for the column number 0xFFFFFFFF;
 *              r_j = word (j mod 4) of call counter (j div 4, 0xFFFFFFFE, offset lo, offset hi)
 *              AND (n_pad - 1);   P = sigma_i * (-1)^popcount(i AND r_j).
 *              So S^T A = sqrt(n_pad / k) * R H D [A; 0]: D = diag(sigma), H the orthonormal
 *              Walsh-Hadamard matrix in Sylvester order, R the selection of rows r_0 .. r_{k-1}
 *              (uniform, independent, with replacement), and E[S S^T] = I.  bf16 with d a multiple
 *              of 8 and n <= 32768 runs the fast transform (one pass over A); other cases apply the
 *              same S entry by entry (correct, O(n k d)).  rmm_variance_stats has no closed form
 *              for this kind (RMM_ERR_UNSUPPORTED).
 * Entries of the Gaussian and Rademacher kinds do not depend on n or k (SORS entries depend on n
 * through n_pad), so a forward and a backward call that pass
 * the same state, n, k and kind see the same S (Algorithm 1, "rematerialize S").
 * The caller must use a fresh offset for every forward call so that sketches of
 * different layers and steps are independent of each other and of dY
 * (Section 2.1, the independence requirement below Eq. 4).
 */
#ifndef RMM_H_
#define RMM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RMM_OK = 0,
    RMM_ERR_INVALID_ARG = -1, /* NULL required pointer, non-positive size, unknown enum, misaligned pointer */
    RMM_ERR_UNSUPPORTED = -2, /* sizes beyond the documented limits */
    RMM_ERR_WORKSPACE = -3,   /* ws is NULL or ws_bytes is below rmm_workspace_bytes() */
    RMM_ERR_LAUNCH = -4,      /* the HIP runtime refused a launch */
    RMM_ERR_SCRATCH_LIMIT = -5 /* rmm_sketch_static only: the shape needs more than RMM_STATIC_SCRATCH_BYTES */
} rmm_status_t;

typedef enum { RMM_DTYPE_F32 = 0, RMM_DTYPE_BF16 = 1 } rmm_dtype_t;
typedef enum { RMM_SKETCH_GAUSSIAN = 0, RMM_SKETCH_RADEMACHER = 1, RMM_SKETCH_SORS = 2 } rmm_sketch_kind_t;
typedef enum { RMM_OP_FORWARD = 0, RMM_OP_BACKWARD = 1, RMM_OP_SKETCH = 2, RMM_OP_VARIANCE = 3 } rmm_op_t;

/* The "PRNG state" saved between forward and backward (Algorithm 1): 16 bytes. */
typedef struct {
    uint64_t seed;
    uint64_t offset;
} rmm_rng_state_t;

/* Shape of one layer call.  n = tokens (rows of X; the paper's B), k = sketch
 * size (the paper's B_proj).  Limits: 1 <= n, d_in, d_out, k < 2^31 and every
 * matrix below 2^40 elements; k > n is accepted (Section 2.1 only asks for
 * E[S S^T] = I). */
typedef struct {
    int64_t n, d_in, d_out, k;
    int32_t dtype; /* rmm_dtype_t */
    int32_t kind;  /* rmm_sketch_kind_t */
} rmm_layer_desc_t;

/* Scratch bytes the given operation needs for this shape.  For RMM_OP_SKETCH
 * only n, k, dtype, kind and d_in (= the operand's column count d) are read.
 * Returns 0 for an invalid descriptor. */
size_t rmm_workspace_bytes(const rmm_layer_desc_t *desc, int op);

/* Static, NUL-terminated description of a status code. */
const char *rmm_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int rmm_version(void);

/* Randomized-matmul primitive (Eq. 4, second line): A_proj[k x d] = S^T A[n x d].
 * A: device, read only.  A_proj: device, written.  Output dtype = dtype. */
int rmm_sketch(int64_t n, int64_t d, int64_t k, int dtype, int kind, rmm_rng_state_t state,
               const void *A, void *A_proj, void *ws, size_t ws_bytes, void *stream);

/* rmm_sketch for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for bit) and
 * errors as rmm_sketch, but the scratch the kernels need (fp32 partial sums of the token slices) is
 * a fixed array of RMM_STATIC_SCRATCH_BYTES inside the library's device code, one copy per GPU,
 * held until the process ends.  A shape whose rmm_workspace_bytes(desc, RMM_OP_SKETCH) exceeds that
 * size is refused with RMM_ERR_SCRATCH_LIMIT before anything is launched.  The call allocates and
 * frees nothing (its first use on a device looks the array's address up once).  All calls on one
 * GPU share the array: two calls that may run at the same time on one GPU (different streams, or
 * different host threads) race and must be serialised by the caller; calls on one stream are
 * ordered.  The array keeps the last call's contents; every call overwrites what it later reads,
 * nothing needs to start at zero. */
#define RMM_STATIC_SCRATCH_BYTES (32u << 20)
int rmm_sketch_static(int64_t n, int64_t d, int64_t k, int dtype, int kind, rmm_rng_state_t state,
                      const void *A, void *A_proj, void *stream);

/* Algorithm 1, Forward: Y[n x d_out] = X[n x d_in] W[d_out x d_in]^T (+ bias[d_out] on
 * every row if bias != NULL; Eq. 1), X_proj[k x d_in] = S^T X.  After the call the
 * caller may drop X and keeps X_proj and `state` for the backward call: the saved
 * bytes are k*d_in*sizeof(dtype) + 16 instead of n*d_in*sizeof(dtype) (Section 2.4.1).
 * X_proj may be NULL when no backward pass will follow (inference): the sketch is then
 * skipped, k and state are ignored beyond validation, and no workspace is needed. */
int rmm_forward(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *X, const void *W,
                const void *bias, void *Y, void *X_proj, void *ws, size_t ws_bytes, void *stream);

/* Algorithm 1, Backward, with the state given to the forward call:
 * dX[n x d_in] = dY[n x d_out] W (Eq. 2), dW[d_out x d_in] = (S^T dY)^T X_proj,
 * and, if dbias != NULL, dbias[d_out] = dY^T 1 (Eq. 3).  dX may be NULL to skip
 * the input gradient (first layer of a network). */
int rmm_backward(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *dY, const void *W,
                 const void *X_proj, void *dX, void *dW, void *dbias, void *ws, size_t ws_bytes,
                 void *stream);

/* rmm_backward for gradient accumulation over micro-batches: dW (and dbias, if given) must
 * hold valid values on entry and receive old value + this call's estimate (Algorithm 1,
 * Backward, applied to a sum of losses; the sum is formed in fp32 and rounded once to the
 * output dtype).  dX is overwritten as in rmm_backward.  Same arguments and errors. */
int rmm_backward_accumulate(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *dY, const void *W,
                            const void *X_proj, void *dX, void *dW, void *dbias, void *ws, size_t ws_bytes,
                            void *stream);

/* Variance monitors of Section 2.3 for one layer call, from X[n x d_in] and dY[n x d_out]
 * (device, read only; Y of the lemmas is dY).  out: 8 doubles on the device, 8-byte aligned:
 *   out[0] = |X|_F^2            out[1] = |dY|_F^2
 *   out[2] = sum_k |x_k|^2 |y_k|^2 over the token rows        out[3] = |X^T dY|_F^2
 *   out[4] = D^2_SGD = n/(n-1) out[2] - out[3]/(n-1)           (Lemma 2.1; 0 for n = 1)
 *   out[5] = D^2_RMM for sketch size desc->k and kind desc->kind: (out[0] out[1] + out[3]) / k
 *            for Gaussian S, less 2 out[2] / k for Rademacher S (Lemma 2.2 with the sign that
 *            the fourth moment of the sketch entries gives to the |X^T dY|^2 term)
 *   out[6] = alpha = out[3] / (out[0] out[1])                  (Theorem 2.3)
 *   out[7] = (out[0] out[1] - out[3]) / k                      (Lemma 2.2 as printed)
 * Sums are taken in fixed order (bit-reproducible).  Workspace: rmm_workspace_bytes(desc,
 * RMM_OP_VARIANCE), never zero. */
int rmm_variance_stats(const rmm_layer_desc_t *desc, const void *X, const void *dY, double *out, void *ws,
                       size_t ws_bytes, void *stream);

/* Stages of the two passes, for the profiled variants below. */
typedef enum {
    RMM_STAGE_NONE = -1,
    RMM_STAGE_FWD_Y = 0,      /* Y = X W^T (+ bias)          */
    RMM_STAGE_FWD_XPROJ = 1,  /* X_proj = S^T X              */
    RMM_STAGE_BWD_DX = 2,     /* dX = dY W                   */
    RMM_STAGE_BWD_G = 3,      /* G = S^T dY (into workspace) */
    RMM_STAGE_BWD_DW = 4,     /* dW = G^T X_proj             */
    RMM_STAGE_BWD_DBIAS = 5,  /* dbias = dY^T 1              */
    /* The product kernel of a sketch stage alone, without the kernel that sums
     * the token-slice partial results (identical to the stage when the library
     * uses a single slice). */
    RMM_STAGE_FWD_XPROJ_PRODUCT = 6,
    RMM_STAGE_BWD_G_PRODUCT = 7,
    /* Where the library issues the two independent products of a pass (Y with X_proj, dX with G)
     * as ONE kernel launch, so that each takes the compute units the other leaves idle: that
     * kernel alone.  Asking for one of the stages 0-3, 6 or 7 makes the call launch the two
     * products one after the other instead (same results, bit for bit), so that each can be timed;
     * a call that launches them separately anyway records nothing for these two. */
    RMM_STAGE_FWD_PAIR = 8,
    RMM_STAGE_BWD_PAIR = 9
} rmm_stage_t;

/* Measurement hooks: identical to rmm_forward / rmm_backward, and in addition
 * record the hipEvent_t `ev_begin` on `stream` right before the kernels of
 * `stage` and `ev_end` right after them, so a caller can time one stage inside
 * a full pass.  Events are created and owned by the caller.  A stage that does
 * not run in this call (wrong pass, dX or dbias skipped) records nothing. */
int rmm_forward_profiled(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *X, const void *W,
                         const void *bias, void *Y, void *X_proj, void *ws, size_t ws_bytes, void *stream,
                         int stage, void *ev_begin, void *ev_end);
int rmm_backward_profiled(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *dY, const void *W,
                          const void *X_proj, void *dX, void *dW, void *dbias, void *ws, size_t ws_bytes,
                          void *stream, int stage, void *ev_begin, void *ev_end);

/* rmm_sketch with an event pair recorded around its product kernel alone (the
 * kernel that reads A), as RMM_STAGE_FWD_XPROJ_PRODUCT does inside a forward
 * pass.  Either event may be NULL, which records nothing. */
int rmm_sketch_profiled(int64_t n, int64_t d, int64_t k, int dtype, int kind, rmm_rng_state_t state,
                        const void *A, void *A_proj, void *ws, size_t ws_bytes, void *stream,
                        void *ev_begin, void *ev_end);

/* Whether an unprofiled rmm_forward (op = RMM_OP_FORWARD) / rmm_backward with dX (RMM_OP_BACKWARD)
 * of this shape issues its two independent products as one paired launch (RMM_STAGE_FWD_PAIR /
 * RMM_STAGE_BWD_PAIR): 1 or 0; 0 for an invalid descriptor. */
int rmm_uses_paired_launch(const rmm_layer_desc_t *desc, int op);

/* Ceilings of the chip as a kernel sees them, for reporting measured fractions beside the
 * published peaks (the caller times the launch with events).
 * rmm_probe_mfma: `work_groups` work-groups of four waves, each wave issuing 16 * iters
 *   independent 32x32x16 bf16 MFMAs from registers: work_groups * 4 * 16 * iters * 32768 flop.
 * rmm_probe_read: streams `bytes` bytes (rounded down to 16) from `src` (device, 16-byte aligned)
 *   once with 16-byte loads, split evenly over `work_groups` work-groups.
 * `sink` is a device buffer of at least 1 KiB that keeps the work alive; it is practically never
 * written. */
int rmm_probe_mfma(int work_groups, int iters, void *sink, void *stream);
int rmm_probe_read(const void *src, size_t bytes, int work_groups, void *sink, void *stream);

/* Test hooks for the bit-exactness requirement on the generator.
 *
 * rmm_debug_philox: out[4*t .. 4*t+3] (device, uint32) = Philox-4x32-10 of counter
 * (c0 + t, c1, offset lo, offset hi) under the key of state.seed, t = 0..ncalls-1
 * (c0 + t wraps modulo 2^32).
 *
 * rmm_debug_sketch_tile: P_out[r*cols + c] (device, fp32) = P[i0 + r][j0 + c], the
 * UNSCALED sketch entry exactly as the fp32 kernels generate it, for 0 <= r < rows,
 * 0 <= c < cols.  For Rademacher the values are exactly +1 / -1. */
int rmm_debug_philox(rmm_rng_state_t state, uint32_t c0, uint32_t c1, int64_t ncalls, uint32_t *out,
                     void *stream);
int rmm_debug_sketch_tile(int kind, rmm_rng_state_t state, int64_t i0, int64_t j0, int64_t rows,
                          int64_t cols, float *P_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RMM_H_ */
