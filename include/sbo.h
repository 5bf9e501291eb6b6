/*
 * libsbo -- one Single Block Orthogonal (SBO) dictionary-learning iteration on
 * one MI355X (gfx950): sparse coding, grouping, block accumulation and the
 * batched SVD update Q_j = U V^T.
 *
 * Problem (Section 1, eq. (1)-(3)): signals Y in R^{p x m}, sparsity s0, a
 * dictionary D = [Q_1 ... Q_K] of K orthonormal p x p blocks, Q_j^T Q_j = I.
 *
 * Conventions for every call
 *   - Every array pointer is a DEVICE pointer owned by the caller.  The library
 *     never frees or reallocates caller memory.  It owns only the workspace it
 *     allocates in sbo_create and frees in sbo_destroy.
 *   - Y    [m][p]     float : signal-major (row i = y_i; same bytes as a
 *                             column-major p x m matrix with ld = p).  Read only.
 *   - D    [K][p][p]  float : atom-major, D[j][k][:] = atom k of Q_j (same bytes
 *                             as column-major Q_j).
 *   - blk  [m]        int32 : block chosen for each signal, 0..K-1.
 *   - supp [m][s0]    int32 : kept atom indices inside that block, ASCENDING.
 *   - coef [m][s0]    float : coef[i][t] pairs with supp[i][t].
 *   - err  [m]        float : ||y_i - Q_blk x_i||^2 (squared residual).
 *   - All per-signal outputs are in the ORIGINAL signal order.
 *   - Work is enqueued on the HIP stream given to sbo_create; calls return
 *     without synchronising the host (exceptions, each stated at its declaration:
 *     sbo_stage_ms, sbo_svd_sweeps, sbo_learn).  Calls on one context must not overlap.
 *   - Return value: 0 on success, a negative SBO_E* code otherwise.  On error no
 *     output is defined; no exception crosses this boundary.
 *   - Supported shapes: p in {16, 32, 64, 256}, 1 <= s0 <= min(p, 16), 1 <= K <= 1024,
 *     1 <= m <= m_max < 2^31 / max(p, s0).
 *   - Signals or atoms holding NaN give unspecified results.  The atoms in one signal's
 *     supp row must be distinct; block or atom ids outside their range are ignored.
 */
#ifndef SBO_H
#define SBO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SBO_OK       0
#define SBO_EINVAL  (-1)  /* bad or unsupported shape, NULL pointer, m > m_max */
#define SBO_ENOMEM  (-2)  /* workspace allocation failed */
#define SBO_EHIP    (-3)  /* a HIP call failed; text via sbo_strerror */
#define SBO_ELIMIT  (-4)  /* a size beyond a stated fixed limit; text via sbo_strerror */

typedef struct sbo_ctx sbo_ctx;   /* opaque: shapes, stream, device workspace */

/* Stages timed by sbo_stage_ms, in this order. */
enum {
    SBO_STAGE_ENERGY = 0,  /* projection onto all K blocks + top-s0 energy + block argmax */
    SBO_STAGE_GROUP  = 1,  /* counting-sort bucketing of signals by block */
    SBO_STAGE_SELECT = 2,  /* support/coefficients/error in the winning block */
    SBO_STAGE_ACCUM  = 3,  /* P_j = Y_j X_j^T */
    SBO_STAGE_SVD    = 4,  /* Q_j = U V^T of each P_j (Algorithm 1, steps 6-7) */
    SBO_N_STAGES     = 5
};

/* Create a context for fixed (p, K, s0) and at most m_max signals per call.
 * hip_stream: a hipStream_t (NULL = the default stream).  Allocates the device
 * workspace (sbo_workspace_bytes).  *out is set only on success. */
int sbo_create(sbo_ctx** out, int p, int K, int s0, int64_t m_max, void* hip_stream);

/* Free the workspace and the context.  Synchronises the stream first. */
int sbo_destroy(sbo_ctx* c);

/* Device bytes sbo_create will allocate for these shapes; 0 if unsupported. */
size_t sbo_workspace_bytes(int p, int K, int s0, int64_t m_max);

/* Sparse coding of every signal with a single block (Section 2, eq. (4);
 * Section 3.1; Algorithm 2 step 4).  For each signal and each block j:
 * c = Q_j^T y, keep the s0 entries of largest magnitude (ties: lower atom index),
 * E_j = sum of kept c^2; blk = argmax_j E_j (ties: lowest j).
 * in : Y[m][p], D[K][p][p]          out: blk[m], supp[m][s0], coef[m][s0], err[m]
 * The K*p x m projection is never written to memory. */
int sbo_code(sbo_ctx* c, const float* Y, int64_t m, const float* D,
             int32_t* blk, int32_t* supp, float* coef, float* err);

/* Grouping of the signals by chosen block (Section 3.3, grouping before the
 * training step): counts[K], offsets[K+1] (exclusive prefix sums) and perm[m],
 * the signal ids listed block by block, original order inside a block (stable).
 * in : blk[m]                        out: counts[K], offsets[K+1], perm[m]
 * Any output pointer may be NULL (that output is then not copied out). */
int sbo_group(sbo_ctx* c, const int32_t* blk, int64_t m,
              int32_t* counts, int32_t* offsets, int32_t* perm);

/* sbo_group for callers that cannot allocate device memory or hold a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as
 * sbo_group (same kernels); takes no context and calls no allocating routine: its scratch
 * (per-chunk histograms and bases, 1 MiB) is a static device array that every GPU the
 * library runs on holds until the process ends.
 * Limits: 1 <= K <= SBO_GROUP_STATIC_MAX_K, 1 <= m <= SBO_GROUP_STATIC_MAX_M; beyond them
 * SBO_ELIMIT is returned and nothing is enqueued.  counts, offsets and perm are all required.
 * Work is enqueued on hip_stream (NULL = the default stream) of the current device.  All
 * calls on one GPU share the one scratch array: calls that overlap on a GPU (different
 * streams, different threads) race; serialise them.  Nothing in the scratch needs clearing
 * between calls (every entry read is written first by the same call). */
#define SBO_GROUP_STATIC_MAX_K 128
#define SBO_GROUP_STATIC_MAX_M 1048576
int sbo_group_static(const int32_t* blk, int64_t m, int K, int32_t* counts, int32_t* offsets,
                     int32_t* perm, void* hip_stream);

/* Block accumulation P_j = Y_j X_j^T for every block (Algorithm 1, step 5),
 * atom-major: M[j][k][:] = sum over the block's signals of x_i[k] * y_i.
 * Summation order is fixed: results are bitwise repeatable.  Blocks without
 * signals give M[j] = 0.
 * in : Y, blk, supp, coef            out: M[K][p][p] */
int sbo_accumulate(sbo_ctx* c, const float* Y, int64_t m, const int32_t* blk,
                   const int32_t* supp, const float* coef, float* M);

/* Orthogonal factor of each M_j (Algorithm 1, steps 6-7): with M_j = U S V^T,
 * Q_j = U V^T written to D[j] (atom-major, same convention as M).  U V^T is the
 * orthogonal polar factor of M_j; it is computed by the Newton-Schulz iteration on the
 * matrix cores where that converges (condition numbers up to about 3000) and by a
 * one-sided Jacobi SVD otherwise (or always: sbo_set_option).  A block with counts[j] == 0 is left untouched
 * (counts may be NULL = all blocks updated).  Rank-deficient M_j: the null directions
 * are completed to an orthonormal basis (any completion is a valid U V^T).
 * in : M[K][p][p], counts[K] or NULL in/out: D[K][p][p] */
int sbo_polar(sbo_ctx* c, const float* M, const int32_t* counts, float* D);

/* Train every orthobase over its own signals, one round (Algorithm 2 step 5 with
 * R = 1; Algorithm 1 steps 5-7): grouping, accumulation, SVD, Q_j = U V^T, in
 * place in D.  counts (device, [K]) may be NULL. */
int sbo_update(sbo_ctx* c, const float* Y, int64_t m, const int32_t* blk,
               const int32_t* supp, const float* coef, float* D, int32_t* counts);

/* R rounds of single-orthobase training per block with the block assignment frozen
 * (Algorithm 1 with R rounds, as used by Algorithm 2 step 5): for every block j over the
 * signals with blk == j, repeat R times { x = Q_j^T y hard-thresholded to its s0 largest
 * magnitudes; P_j = Y_j X_j^T; Q_j = U V^T }.  D is updated in place R times; supp, coef
 * and err receive the codes of the LAST round (i.e. with respect to D before the last
 * update).  R = 1 with blk from sbo_code equals sbo_code's code followed by sbo_update.
 * in : Y, blk[m], R >= 1     in/out: D     out: supp[m][s0], coef[m][s0], err[m] */
int sbo_train_rounds(sbo_ctx* c, const float* Y, int64_t m, const int32_t* blk, float* D, int R,
                     int32_t* supp, float* coef, float* err);

/* n_iter x (sbo_code; sbo_update) (Algorithm 2, steps 4-5).  blk/supp/coef/err
 * hold the LAST coding pass (i.e. with respect to D before the last update).
 * sqerr_per_iter: device double[n_iter] or NULL; entry t = sum_i err_i of coding
 * pass t (RMSE = sqrt(sqerr / (p m)), Section 4). */
int sbo_iterate(sbo_ctx* c, const float* Y, int64_t m, float* D, int n_iter,
                int32_t* blk, int32_t* supp, float* coef, float* err,
                double* sqerr_per_iter);

/* Total squared representation error sum_i err[i] (numerator of the RMSE of Section 4;
 * the stopping rule of Algorithm 2 compares it, or the number of orthobases, with a
 * target on the host).  Fixed-order sum in double precision.
 * in : err[m] (device)      out: out (device double[1]) */
int sbo_sqerr(sbo_ctx* c, const float* err, int64_t m, double* out);

/* The W worst represented signals (Algorithm 2, step 3, first half): the W largest
 * err[i]; among equal values the lower signal index is taken first.  ids (device,
 * int32[W]) receives the chosen signal indices in ascending order.  1 <= W <= m, else
 * SBO_EINVAL.  NaN entries are ordered by their bit pattern (unspecified position). */
int sbo_worst(sbo_ctx* c, const float* err, int64_t m, int64_t W, int32_t* ids);

/* Starting orthobase for a set of signals (eq. (5)): Y_sub = U S V^T, Q_0 = U, computed as
 * the eigenvectors of the set's Gram matrix sum_i y_i y_i^T.
 * in : Y[m][p], ids[n] (device, signal indices; values outside [0, m) are clamped into it),
 *      1 <= n <= m
 * out: Q[p][p] atom-major, atom k = left singular vector of the k-th largest singular value
 *      (sign not determined; directions of vanishing singular values are an arbitrary
 *      orthonormal completion); sv[p] (device, may be NULL) = the singular values, descending.
 * Uses the context's workspace (K may be anything; the set is treated as one block). */
int sbo_init_base(sbo_ctx* c, const float* Y, int64_t m, const int32_t* ids, int64_t n,
                  float* Q, float* sv);

/* A new orthobase trained on a set of signals (Algorithm 2, steps 1 and 3): unless
 * have_q0 != 0 start from sbo_init_base, then R rounds of Algorithm 1 on the set
 * { x = Q^T y hard-thresholded to s0 entries; P = Y_sub X^T; Q = U V^T }.
 * in : Y, ids[n] (as for sbo_init_base), R >= 0      in/out: Q[p][p] (input only if have_q0)
 * out: rows ids[.] of supp[m][s0], coef[m][s0], err[m] receive the codes of the set's signals
 *      in the last round (other rows are not touched; not written when R == 0);
 *      sqerr_per_round (device double[R], may be NULL): total squared error of each round's codes. */
int sbo_new_base(sbo_ctx* c, const float* Y, int64_t m, const int32_t* ids, int64_t n, int R,
                 int have_q0, float* Q, int32_t* supp, float* coef, float* err,
                 double* sqerr_per_round);

/* Number of orthobases in use by the calls that follow: 1 <= K <= the K given to
 * sbo_create (which sized the workspace).  A dictionary that grows (Algorithm 2, step 3)
 * is handled by creating the context for the largest K and raising the count here. */
int sbo_set_blocks(sbo_ctx* c, int K);

/* Algorithm 2 as a whole.
 *   Initialisation: K0 orthobases, base j trained by sbo_new_base (eq. (5) start + R rounds)
 *   on the P0 signals init_ids[j][0..P0) (device int32 [K0][P0]; the random choice of those
 *   signals is the caller's); then every signal is represented (sbo_code).
 *   Iterations, while fewer than K_max orthobases exist and the RMSE is above target_rmse:
 *   a new orthobase is trained on the W worst represented signals (sbo_worst, sbo_new_base)
 *   and appended; every signal is represented; every orthobase is trained over its own
 *   signals for R rounds (sbo_train_rounds); the stopping rule is evaluated on the host.
 *   The error used by the stopping rule and by the next worst-W set is that of the codes of
 *   the last training round.
 * in : Y[m][p]; 1 <= K0 <= K_max <= K of sbo_create; 1 <= P0, W <= m; R >= 1
 * out: D (device, room for K_max orthobases, the first *K_final are valid);
 *      blk/supp/coef/err (device): the last representation and the codes of the last round;
 *      K_final, n_hist (HOST ints); rmse_hist (HOST double[K_max - K0 + 1]): entry 0 after the
 *      initial representation, then one per iteration, *n_hist entries.
 * Synchronises the stream once per iteration (the stopping rule reads the error). */
int sbo_learn(sbo_ctx* c, const float* Y, int64_t m, float* D, const int32_t* init_ids, int K0,
              int64_t P0, int R, int64_t W, int K_max, double target_rmse, int32_t* blk,
              int32_t* supp, float* coef, float* err, int* K_final, double* rmse_hist, int* n_hist);

/* Work of the most recent SVD stage of this context, per orthobase: a positive value is
 * the number of Jacobi sweeps, a negative one minus the number of Newton-Schulz steps, 0 an
 * orthobase that kept its basis.  sweeps: HOST int32[K].  Synchronises the stream. */
int sbo_svd_sweeps(sbo_ctx* c, int32_t* sweeps);

/* Options of a context (sbo_set_option). */
enum {
    SBO_OPT_SVD_METHOD   = 0,  /* how Q_j = U V^T is computed: SBO_SVD_AUTO or SBO_SVD_JACOBI */
    SBO_OPT_CODING_ARITH = 1   /* how the projection Q_j^T y onto all K orthobases is multiplied out:
                                  SBO_ARITH_F32, SBO_ARITH_BF16X3, SBO_ARITH_BF16X3_SCREEN or SBO_ARITH_F16X2 */
};
enum {
    SBO_SVD_AUTO   = 0,  /* default: Newton-Schulz polar factor on the matrix cores, the one-sided
                            Jacobi SVD for the orthobases it flags (rank-deficient P_j) */
    SBO_SVD_JACOBI = 1   /* the one-sided Jacobi SVD (one workgroup per orthobase) for every orthobase */
};

enum {
    SBO_ARITH_F32    = 0,  /* the fp32 matrix instruction (v_mfma_f32_32x32x2_f32) */
    SBO_ARITH_BF16X3 = 1,  /* every fp32 operand entry written as the exact sum of three bf16 numbers;
                              the six partial products that matter at fp32 accuracy run on the bf16
                              matrix cores with fp32 accumulation (same fp32 inputs and outputs, rounding
                              at the fp32 level: the dropped partial products are below 2^-24 of |a||b|) */
    SBO_ARITH_F16X2 = 3,   /* default: the choice of the orthobase (eq. (4)) on the fp16 matrix cores: every signal
                              scaled by a power of two, signal and dictionary entries each written as
                              hi + lo in fp16 (22 significand bits), three partial products with fp32
                              accumulation: per-term error 3 * 2^-22 |a||b|, below the p * 2^-24 sum |a||b|
                              an fp32 dot product of p terms guarantees; half the matrix work of
                              SBO_ARITH_BF16X3.  Supports and coefficients still come from the six bf16
                              products.  Dictionary entries
                              must be below 8 in magnitude (orthonormal atoms: at most 1); a signal whose
                              largest magnitude is below 2^-63 is coded as a zero signal (its energies
                              underflow in fp32 under any arithmetic). */
    SBO_ARITH_BF16X3_SCREEN = 2  /* as SBO_ARITH_BF16X3, but the choice of the orthobase (eq. (4))
                              first runs with the three largest partial products only, for all signals; that
                              decides every signal whose two best kept energies are further apart than twice
                              the error bound of the shortened product, 2 (2 sqrt(s0) c + s0 c^2) ||y||^2 with
                              c = 3.01 * 2^-16 + 2e-6, and only the remaining signals get the six products
                              over all orthobases.  The chosen orthobases are those of SBO_ARITH_BF16X3;
                              supports and coefficients always come from the six products.  Used for
                              p <= 64 when the signals fill the chip; otherwise as SBO_ARITH_BF16X3.
                              Pays when the orthobases are well separated (few undecided signals); with
                              near-random orthobases it is about as fast as SBO_ARITH_BF16X3. */
};

/* Set an option for every later call on this context (Algorithm 1 steps 6-7 leave the SVD
 * routine open; both choices give the same Q_j up to rounding).  Unknown option or value:
 * SBO_EINVAL, nothing changed. */
int sbo_set_option(sbo_ctx* c, int option, int value);

/* Per-stage timing with HIP events on the context's stream.  enable = 1 makes every
 * later call record events around each stage it runs; enable = 2 only around the energy
 * kernel (an event pair costs a few microseconds on the stream, which shows in a step of
 * under a millisecond); 0 switches timing off. */
int sbo_set_timing(sbo_ctx* c, int enable);

/* Synchronises the stream and writes, for the most recent timed call,
 * milliseconds per stage into ms[SBO_N_STAGES] (HOST pointer); stages that call
 * did not run read 0.  For sbo_iterate the times are summed over iterations. */
int sbo_stage_ms(sbo_ctx* c, float* ms);

/* Text for a return code; for SBO_EHIP the text of the last HIP error seen by
 * this thread.  Never NULL; the pointer stays valid until the next call. */
const char* sbo_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SBO_H */
