/*
 * dion.h — C ABI of the MI355X (gfx950) Dion optimizer-step library (libdion.so).
 *
 * The library computes one step of the Dion optimizer for one matrix parameter, or for a
 * batch of them, following the paper's Algorithm 1 (outer step) with the unsharded update
 * rule and its PowerIter1 sub-routine (Section 3), the error-feedback equation of
 * Section 3.1, and Cholesky-QR orthonormalisation (Section 3.2, Appendix A):
 *
 *     B     = M + G                        (never stored in fp32; see "How M + G reaches the products" below)
 *     Z     = B Q                          (m x r)
 *     P     = Orthonormalize(Z)            (thin-QR factor, by CholeskyQR2)
 *     R     = B^T P                        (n x r)
 *     M_new = B - (1 - mu) P R^T           (error feedback; the paper's beta = 1 - mu)
 *     Q_new = ColNorm(R)                   (each column divided by (its 2-norm + 1e-8))
 *     X_new = X - eta sqrt(m/n) P Q_new^T  (m = "out" rows, n = "in" columns)
 *
 * Names: the paper's V, P, U, W, beta are Q, Z, P, R, 1 - mu here.
 *
 * How M + G reaches the products.  The fused update adds M + G in fp32 in its epilogue.  The two products Z and R
 * take it as an operand: in DION_MATH_F32, and in DION_MATH_BF16 for shapes whose outputs cannot fill the GPU with
 * 256 x 256 tiles, the sum is formed in registers on the way into the matrix cores; for the large shapes of
 * DION_MATH_BF16 (m, n multiples of 256, r a multiple of 256, at least 128 output tiles of 256 x 256 per group of
 * equal shapes) one pass first stores bf16(M + G) in the workspace, once and row-major (2 bytes per element), and
 * both products read that copy (the product with (M + G)^T transposes it on the way from LDS into the registers).
 *
 * Conventions
 *   - All matrices are row-major and contiguous: X, G, M have leading dimension n, Q has r.
 *   - X, M, Q are fp32 and updated in place; G is read only (fp32 or bf16, see DION_G_*).
 *   - Every pointer named *_dev / X / G / M / Q is DEVICE memory owned by the caller and must
 *     be 16-byte aligned; pointer arrays and shape arrays are HOST memory, read during the call.
 *   - X, G, M, Q and the workspace must not overlap one another.
 *   - Calls enqueue work on the given HIP stream (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without waiting; only dion_last_status and
 *     dion_stage_times synchronise.  For very large matrices (the stated rule: where a copy pass over M and G hides
 *     behind the first product of the step for longer than the parts it is cut into cost) a step also enqueues on
 *     a second stream that the state created at dion_init_state (non-blocking, default priority) and orders the two
 *     with events; all of that work has been waited for on the given stream before the step's later stages, so the
 *     caller sees one stream, and a stream capture of the given stream captures both.
 *   - Return value: 0 on success, < 0 for a usage or runtime error found on the host (then
 *     nothing was launched by that call and no state was touched).  Numerical trouble is
 *     found on the device and reported later by dion_last_status.
 *   - No function throws.  The only process-wide data are per-device caches of "this kernel may use more than
 *     64 KB of LDS" (set once per device and kernel).  One dion_state_t must not be used from two threads at once,
 *     and steps sharing a state must run on one stream.
 *   - Ranks of 256 and more (up to 128 matrices per group of equal shapes) are factored by single-launch kernels
 *     whose workgroups wait for one another and therefore must all be resident at once: one per compute unit,
 *     sized from the device's compute-unit count read at dion_init_state.  Steps of two states that run
 *     concurrently on two streams, or any other kernels that occupy compute units for long, can keep them from
 *     becoming resident; the waits then give up after dion_set_wait_limit polls and the matrix is reported as
 *     DION_WAIT_TIMEOUT (state untouched; dion_retry_breakdowns repeats it without those kernels).  Run steps of
 *     different states one after another on one stream, or make the later one wait on an event of the earlier.
 *   - Precondition 1 <= r <= min(m, n).
 */
#ifndef DION_H
#define DION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DION_OK = 0,
  DION_EINVAL = -1,      /* null/misaligned pointer, m|n|r <= 0, r > min(m,n), mu outside [0,1], non-finite mu/eta,
                            shapes that were not declared to dion_init_state */
  DION_EWORKSPACE = -2,  /* workspace too small */
  DION_ELAUNCH = -3,     /* a HIP runtime call failed */
  DION_ENOMEM = -4,      /* host allocation failed */
  DION_NUM_BREAKDOWN = 1, /* Cholesky met a non-positive or non-finite pivot: Z is rank deficient or too ill
                             conditioned for Cholesky-QR (Appendix A); X, M, Q of that matrix were left untouched */
  DION_WAIT_TIMEOUT = 2   /* a bounded wait between the workgroups of a single-launch factorisation or inverse gave
                             up (the GPU could not keep the whole launch resident); says nothing about the matrix;
                             X, M, Q of that matrix were left untouched */
};

enum { DION_G_F32 = 0, DION_G_BF16 = 1 };       /* storage type of the gradient G */
enum { DION_MATH_F32 = 0, DION_MATH_BF16 = 1 }; /* operand type of the four large products (Z, R and the two
                                                   rank-r updates); accumulation and all state are fp32 in both
                                                   modes.  Orthonormalisation: DION_MATH_F32 runs CholeskyQR2 on
                                                   the fp32 matrix pipe (||P^T P - I||_max <= 1e-5).  DION_MATH_BF16
                                                   runs its Gram matrix and triangular multiply as three bf16
                                                   products of split operands (x = hi + lo, about 16 mantissa
                                                   bits), the r x r factorisation and inverse in fp32, and cuts the
                                                   second pass short: when the first pass' result P1 has
                                                   ||P1^T P1 - I||_F <= 1e-3 it is taken as P (both consumers of P
                                                   round it to bf16 anyway), so the usual step is one Cholesky-QR
                                                   pass plus that check; ||P^T P - I||_max <= 1e-3 is what this
                                                   mode guarantees */

typedef struct dion_state dion_state_t; /* opaque host object: declared shapes, flags, carved workspace */

/* Bytes of device workspace needed for `count` matrices of shapes (m[i], n[i], r[i]).
 * m, n, r: host arrays of length count.  Writes *bytes_out. */
int dion_workspace_bytes(int count, const int64_t* m, const int64_t* n, const int64_t* r,
                         int g_dtype, int math, size_t* bytes_out);

/* Creates the optimizer state for `count` matrices (Algorithm 1: the state of a matrix is its
 * momentum M and right factor Q) and initialises it on the device:
 *   M[i] <- 0;   Q[i] <- ColNorm(Q[i]) if q_is_filled, else ColNorm of an n x r draw of N(0,1)
 *   (Philox-4x32-10 keyed by `seed`, stream = i, Box-Muller).
 * workspace_dev: device buffer of at least dion_workspace_bytes(...) bytes, 256-byte aligned,
 * owned by the caller and kept alive until dion_destroy_state.  M_dev / Q_dev: host arrays of
 * `count` device pointers.  *st receives the new state (release with dion_destroy_state). */
int dion_init_state(dion_state_t** st, int count, const int64_t* m, const int64_t* n, const int64_t* r,
                    int g_dtype, int math, void* workspace_dev, size_t workspace_bytes,
                    void* const* M_dev, void* const* Q_dev, int q_is_filled, uint64_t seed,
                    void* hip_stream);

/* As dion_init_state, with the form of the power iteration chosen per matrix (Section 4.3, "Other variants":
 * it can run on M or on M^T).  form: host array of `count` DION_FORM_* values, or NULL for all standard.
 *   DION_FORM_STANDARD    the factor Q is n x r; Z = B Q (m x r) is orthonormalised     (as described above)
 *   DION_FORM_TRANSPOSED  the factor is m x r (call it Vt; it lives in the Q argument of every call):
 *                           Z' = B^T Vt (n x r);  P' = Orthonormalize(Z');  R' = B P' (m x r)
 *                           M_new = B - (1 - mu) R' P'^T;  Vt_new = ColNorm(R');
 *                           X_new = X - eta sqrt(m/n) Vt_new P'^T
 *                         the same rule applied to X^T, with the parameter's own scale factor sqrt(m/n) kept;
 *                         the orthonormalisation then acts on n x r, which is the cheaper side when n < m.
 * dion_step / dion_step_batched / dion_retry_breakdowns follow the form declared here; dion_step looks a
 * matrix up by its shape and takes the first declared entry of that shape.  The Lazy-Dion calls accept the
 * standard form only. */
enum { DION_FORM_STANDARD = 0, DION_FORM_TRANSPOSED = 1 };
int dion_init_state_ex(dion_state_t** st, int count, const int64_t* m, const int64_t* n, const int64_t* r,
                       const int* form, int g_dtype, int math, void* workspace_dev, size_t workspace_bytes,
                       void* const* M_dev, void* const* Q_dev, int q_is_filled, uint64_t seed,
                       void* hip_stream);

/* One Dion step for one matrix (Algorithm 1 with the unsharded update rule).  The shape
 * (m, n, r) must be one declared to dion_init_state.  mu in [0,1] (the paper's 1 - beta),
 * eta = learning rate. */
int dion_step(dion_state_t* st, void* X, const void* G, void* M, void* Q,
              int64_t m, int64_t n, int64_t r, float mu, float eta, void* hip_stream);

/* One Dion step for `count` matrices (the paper's batch axis over same-shaped matrices,
 * Section 4.1): matrices of equal shape are processed together by grouped kernel launches.
 * X, G, M, Q: host arrays of device pointers; m, n, r: host arrays; matrix i must have the
 * shape declared as entry i of dion_init_state.  count = 0 is a no-op. */
int dion_step_batched(dion_state_t* st, int count, void* const* X, const void* const* G,
                      void* const* M, void* const* Q, const int64_t* m, const int64_t* n,
                      const int64_t* r, float mu, float eta, void* hip_stream);

/* Lazy-Dion (Section 5.1, "Faster Dion with Lazy Orthonormalization", the Lazy-Dion update rule and its
 * SymPowerIter1): the state is M and a right factor V (n x r, in the buffer the other calls name Q) that is
 * only refreshed on the steps the caller chooses (the paper: every k-th step):
 *     B = M + G
 *     refresh != 0:  V <- Orthonormalize(B^T (B V))      (thin-QR factor, by Cholesky-QR on n x r)
 *     W = B V;   M <- B - (1 - mu) W V^T;   X <- X - eta sqrt(m/n) ColNorm(W) V^T
 * Without a refresh the step has no orthonormalisation at all (three products and a column normalisation).
 * The update assumes V has orthonormal columns, so the first step after dion_init_state must refresh.
 * A breakdown of the refresh is reported as for dion_step and leaves X, M, V untouched.  Arguments and
 * conventions as for dion_step / dion_step_batched; the same state object serves both kinds of step. */
int dion_lazy_step(dion_state_t* st, void* X, const void* G, void* M, void* V,
                   int64_t m, int64_t n, int64_t r, float mu, float eta, int refresh, void* hip_stream);
int dion_lazy_step_batched(dion_state_t* st, int count, void* const* X, const void* const* G,
                           void* const* M, void* const* V, const int64_t* m, const int64_t* n,
                           const int64_t* r, float mu, float eta, int refresh, void* hip_stream);

/* Double Dion (Section 5.2 and the Double Dion algorithm; here without sharding, so that the data-parallel
 * synchronisation of its first stage has nothing to do): two chained Dion steps per matrix,
 *     stage 1 (rank r1):  B1 = M1 + G;  U1, W1 = PowerIter1(B1, V1);  M1 <- B1 - (1 - mu1) U1 W1^T;  V1 <- ColNorm(W1)
 *     stage 2 (rank r2):  B2 = M2 + U1 W1^T;  U2, W2 = PowerIter1(B2, V2);  M2 <- B2 - (1 - mu2) U2 W2^T;
 *                         V2 <- ColNorm(W2);   X <- X - eta sqrt(m/n) U2 V2^T
 * st1 / st2: states created for the shapes (m, n, r1) / (m, n, r2) in this order, standard form, on separate
 * workspaces; st1 with the storage type of G, st2 with DION_G_F32.  D: host array of `count` device buffers of
 * m x n floats (caller-owned scratch) that receive the sketch U1 W1^T between the stages.
 * Stage 2 has no failure branch (the algorithm's Orthonormalize is a QR, which cannot fail): while M2, a sum of
 * rank-r1 sketches, has rank below r2 (from M2 = 0: the first r2/r1 steps) the columns of B2 V2 that depend on the
 * columns before them (pivot of the Gram matrix' factorisation at most 1e-3 of that column's squared norm) get zero
 * columns in U2 and W2, add nothing to M2 and X, and keep their columns of V2; the remaining columns are the QR factor
 * of the independent ones, so X moves on every step by the rank that is there.  A matrix whose stage 1 breaks down
 * (rank-deficient B1 V1, as in dion_step) is skipped in stage 2 as well, so its X, M1, V1, M2, V2 all stay untouched.
 * dion_last_status(st2) reports breakdowns of stage 1 and non-finite input of stage 2 (dion_last_status(st1) those
 * of stage 1).  Other conventions as for dion_step_batched; both states must be used on the same stream. */
int dion_double_step(dion_state_t* st1, dion_state_t* st2, int count, void* const* X, const void* const* G,
                     void* const* M1, void* const* V1, void* const* M2, void* const* V2, void* const* D,
                     const int64_t* m, const int64_t* n, const int64_t* r1, const int64_t* r2,
                     float mu1, float mu2, float eta, void* hip_stream);

/* For callers that cannot allocate device memory and cannot let a library do it: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  One Dion step for one matrix in the standard form, as
 * dion_step computes it, on a workspace that is part of the library: a static device array of
 * DION_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends.  There is no state
 * object: the caller owns the optimizer state M (m x n, zero before the first step) and Q (n x r, columns of unit
 * norm before the first step) and passes it to every call, with the storage type of G and the operand mode that
 * dion_init_state would have been given.  status_dev: device pointer (4-byte aligned, or NULL) that receives the
 * matrix' status word once the step has run on the stream: 0, DION_NUM_BREAKDOWN or DION_WAIT_TIMEOUT.
 * The call enqueues kernels on hip_stream and nothing else: no hipMalloc, hipFree, memset, copy or host wait.
 * The first call on a device does the one-time set-up of that device (looks up the array's address, gives the
 * large-tile kernels leave to use more than 64 KB of LDS) and should be made outside a capture.
 * Errors: DION_EINVAL as for dion_step; DION_EWORKSPACE when dion_workspace_bytes of the shape exceeds
 * DION_STATIC_SCRATCH_BYTES (1024 x 1024 at r = 256 still fits; nothing is launched then).
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (two streams, two
 * threads) race; calls on one stream, or ordered by events, are fine.  Not thread-safe per device. */
#define DION_STATIC_SCRATCH_BYTES (32u << 20)
int dion_step_static(void* X, const void* G, void* M, void* Q, int64_t m, int64_t n, int64_t r, int g_dtype, int math,
                     float mu, float eta, int* status_dev, void* hip_stream);

/* Waits for the stream of the last step and reports its status: *first_bad_index is the lowest matrix index
 * whose step did not complete (-1 if none), *status_out what happened to that matrix (DION_OK,
 * DION_NUM_BREAKDOWN or DION_WAIT_TIMEOUT).  Either pointer may be NULL. */
int dion_last_status(dion_state_t* st, int* status_out, int* first_bad_index);

/* Orthonormalisation variant used by later steps (Section 3.2 and Appendix A: Cholesky-QR is the fast
 * choice, with a fallback for the rare inputs it cannot handle).
 *   DION_ORTH_CHOLQR2          Cholesky-QR applied twice (default); reports DION_NUM_BREAKDOWN when B Q is
 *                              rank deficient or its condition number exceeds a few thousand.
 *   DION_ORTH_SHIFTED_CHOLQR3  a shifted Cholesky-QR pass in front of the two (about 1.5x the orthonormalisation
 *                              cost): does not break down for condition numbers up to about 1e5; an exactly rank
 *                              deficient B Q is still reported.  Since a breakdown leaves X, M, Q untouched, a
 *                              caller can switch to this mode and repeat the step.
 *   DION_ORTH_CHOLQR2_FALLBACK the default passes, and behind them, in the same step and without the host taking
 *                              part, the fallback: the matrices whose factorisation broke down (decided on the
 *                              device) are orthonormalised again from the untouched B Q by shifted CholeskyQR3 in
 *                              fp32 arithmetic, in either arithmetic mode; for all other matrices those launches
 *                              return at once (about 20 of them per shape group: measured 0.03-0.08 ms per step).  The step
 *                              then completes with DION_OK for condition numbers up to about 1e5;
 *                              DION_NUM_BREAKDOWN is left for B Q that is rank deficient outright.  Applies to
 *                              dion_step, dion_step_batched and the first stage of dion_double_step for matrices of
 *                              the standard form; the transposed form and the Lazy-Dion refresh have no third
 *                              buffer for it and behave as with DION_ORTH_CHOLQR2. */
enum { DION_ORTH_CHOLQR2 = 0, DION_ORTH_SHIFTED_CHOLQR3 = 1, DION_ORTH_CHOLQR2_FALLBACK = 2 };
int dion_set_orth_mode(dion_state_t* st, int mode);

/* Fallback for matrices whose last step did not complete (Appendix A: when Cholesky-QR fails the step falls
 * back to a more robust orthonormalisation).  Waits for the last step, reads the per-matrix status words and
 * repeats the step for exactly the matrices concerned (their X, M, Q were left untouched, so this completes the
 * step; matrices that succeeded are not stepped again): with DION_ORTH_SHIFTED_CHOLQR3 after a
 * DION_NUM_BREAKDOWN; in the state's own mode but with one launch per panel, i.e. without the kernels that
 * wait, after a DION_WAIT_TIMEOUT.
 * Arguments as for the dion_step_batched call being completed, G unchanged since then.  *retried_out (may be
 * NULL) receives the number of matrices repeated.  The state's orthonormalisation mode is left as it was;
 * dion_last_status afterwards reports the outcome of the repeated steps. */
int dion_retry_breakdowns(dion_state_t* st, int count, void* const* X, const void* const* G, void* const* M,
                          void* const* Q, const int64_t* m, const int64_t* n, const int64_t* r, float mu, float eta,
                          void* hip_stream, int* retried_out);

/* Bound on the waits inside the single-launch Cholesky kernel and the single-launch triangular inverse that
 * follows it, which factor and invert up to 128 matrices of rank 256 and more with workgroups that wait for one
 * another's results (Appendix A names the factorisation; how it is scheduled is this library's business).  A
 * workgroup that has polled `polls` times without success gives up, all others follow, the kernel ends, and the
 * matrix is reported as DION_WAIT_TIMEOUT with X, M, Q untouched; a later step is not affected.  The default (about a million polls, on the order of a second) is only ever reached when
 * the GPU cannot keep all workgroups of the kernel resident; 0 makes every wait fail, for tests of this path. */
int dion_set_wait_limit(dion_state_t* st, unsigned polls);

/* How the r x r factorisation of Cholesky-QR (Appendix A) would be scheduled for `batch` matrices of rank r on a
 * GPU with `compute_units` compute units: *workgroups_out workgroups per matrix in one launch, all of which
 * (workgroups x batch, never more than compute_units) have to be resident at once, or 0 for one launch per
 * 64-column panel with no waits between workgroups.  Host only: touches no GPU. */
int dion_cholesky_grid(int compute_units, int batch, int64_t r, int* workgroups_out);

/* Stage timing.  With enable != 0 every later step brackets its stages with HIP events on
 * the step's stream.  dion_stage_times waits for the last step and writes, for stage s <
 * DION_STAGE_COUNT, the summed duration in milliseconds of that stage over the last call. */
enum {
  DION_STAGE_K1_BQ = 0,     /* Z = (M+G) Q          (Lazy-Dion: W = (M+G) V) */
  DION_STAGE_ORTH = 1,      /* CholeskyQR2          (Lazy-Dion: the whole refresh, 0 without one) */
  DION_STAGE_K2_BTP = 2,    /* R = (M+G)^T P        (Lazy-Dion: 0) */
  DION_STAGE_COLNORM = 3,   /* column norms of R and Q_new = R diag(d) */
  DION_STAGE_K5_UPDATE = 4, /* fused M and X update */
  DION_STAGE_COUNT = 5
};
int dion_set_stage_timing(dion_state_t* st, int enable);
int dion_stage_times(dion_state_t* st, float* ms_out /* [DION_STAGE_COUNT] */);

/* Measured ceilings of the GPU the calling thread has current, for quoting achieved rates against (the hot path's
 * bounds are the bf16 matrix pipe for the products at r >= 1024 and HBM for the fused update at smaller r; see the
 * step-time analysis around Figure 1 of the paper for the same split on its hardware):
 *   *mfma_tflops  an issue-only loop of the bf16 matrix instruction the products use (no memory traffic),
 *   *stream_gbps  a streaming pass with the traffic of the fused update: per element it reads fp32, bf16, fp32
 *                 and writes fp32, fp32 (18 bytes), with 16-byte accesses.
 * scratch_dev: device memory, 256-byte aligned, owned by the caller and overwritten; at least 10 MiB, and the
 * streaming pass covers scratch_bytes / 10 elements rounded down to a multiple of 2^20 (at most 2^26 of them), so
 * give it more than the 256 MB Infinity Cache holds (1 GiB is what bench.py uses).  The call enqueues on hip_stream and waits for the result (host outputs).
 * Errors: DION_EINVAL (null or misaligned arguments), DION_EWORKSPACE (scratch too small), DION_ELAUNCH. */
int dion_measure_ceilings(void* scratch_dev, size_t scratch_bytes, double* mfma_tflops, double* stream_gbps,
                          void* hip_stream);

/* Test access to the intermediates of matrix `index` left in the workspace by the last step:
 * which = 0: Z (m x r; after a Lazy-Dion step: W), 1: P (m x r), 2: R (n x r), 3: column norms s (r),
 * 4: status word (int32), 5: the output of the first Cholesky-QR pass, 6 / 7 / 8: Gram matrix, its Cholesky
 * factor and that factor's inverse of the last pass (rp x rp, rp = r rounded up to 64), 9: 1 / (s + eps),
 * 10: int32 per column (rp of them), 1 where stage 2 of the last Double Dion step found the column dependent.
 * Writes the device pointer and the leading dimension (elements). */
int dion_debug_buffer(dion_state_t* st, int index, int which, void** ptr_out, int64_t* ld_out);

int dion_destroy_state(dion_state_t* st);

const char* dion_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DION_H */
