/*
 * same_lda.h - C ABI of the MI355X (gfx950) SAME Gibbs LDA sweep library.
 *
 * The library runs the per-nonzero hot path of SAME (State Augmentation for
 * Marginal Estimation) Gibbs parameter estimation for Latent Dirichlet Allocation
 * (Zhao, Jiang, Canny, arXiv 1409.5402) on one GPU:
 *
 *   for every nonzero (d, w, c) of the sparse words x documents count matrix
 *     weights   w_k = theta[d][k] * phi[w][k]                (Algorithm 3, normaliser and lambda)
 *     draw      the m copies of each of the c tokens as ONE multinomial count vector
 *               totalling m*c (Section 4, "coordinate-factored" multinomial form)
 *     scatter   the counts into new document-topic and word-topic matrices
 *   then add the priors, normalise phi over words and blend (Algorithm 3, last steps; Eq. 6).
 *
 * Conventions
 *   - Every function returns SAME_LDA_OK (0) or a negative SAME_LDA_E* code; the text of the
 *     last failure is available from same_lda_last_error().  No exception crosses the boundary.
 *   - "host" / "device" on a pointer says where the memory must live.  Device pointers are plain
 *     HIP device allocations of the current device (for example the data_ptr of a torch tensor).
 *   - Matrices are dense row-major: theta and n_dk are [D][K], phi and n_wk are [V][K]
 *     (word-major, so the K values of one word are contiguous).
 *   - All device state is allocated in same_lda_init / same_lda_set_batch; same_lda_sweep
 *     allocates nothing (the paper's matrix-caching rule, Section 5.3).
 *   - The input matrix is borrowed for the duration of the call only: the library keeps its own
 *     device-side work list and never modifies the caller's arrays.
 *   - Work is enqueued on the HIP stream given at init; calls are asynchronous unless stated.
 *   - One handle must not be used from two threads at once.
 */
#ifndef SAME_LDA_H
#define SAME_LDA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAME_LDA_OK       0
#define SAME_LDA_EINVAL  (-1)  /* null pointer, bad shape, K < 1, m < 1, alpha <= 0, beta <= 0, bad selector */
#define SAME_LDA_ECSC    (-2)  /* malformed matrix: column pointers not ascending, word id out of range,
                                  count not a positive integer, m * count too large, or m times the tokens
                                  of one document or word beyond the 32-bit count matrices                  */
#define SAME_LDA_ENOMEM  (-3)  /* host or device allocation failed                                         */
#define SAME_LDA_EHIP    (-4)  /* HIP runtime error (text in same_lda_last_error)                          */

typedef struct same_lda same_lda_t;   /* opaque; owns all device state */

/* Sparse words x documents matrix in compressed-column form: column d is document d
 * (the D_t of Algorithm 3).  All three arrays live on the host (on_device = 0) or all on the
 * device (on_device = 1).                                                                     */
typedef struct {
    int32_t        D;        /* number of documents (columns), >= 0                           */
    int32_t        V;        /* vocabulary size (rows), >= 1                                  */
    int64_t        nnz;      /* number of stored entries, == colptr[D], < 2^31                */
    const int32_t* colptr;   /* [D+1] ascending, colptr[0] == 0                               */
    const int32_t* rowidx;   /* [nnz] word id in [0, V)                                       */
    const float*   val;      /* [nnz] token counts: integer-valued, >= 1, stored as float     */
    int32_t        on_device;
} same_lda_csc;

/* Selectors for same_lda_get / same_lda_set. */
#define SAME_LDA_THETA 0   /* float    [D][K]  theta = n_dk/m + alpha (unnormalised)             */
#define SAME_LDA_PHI   1   /* float    [V][K]  phi, each topic normalised over words             */
#define SAME_LDA_NDK   2   /* uint32_t [D][K]  document-topic counts of the last pass            */
#define SAME_LDA_NWK   3   /* uint32_t [V][K]  word-topic counts of the last pass                */
#define SAME_LDA_NK    4   /* uint64_t [K]     topic totals of the last pass                     */

/* Create a handle for matrix X and run the random initialisation (Algorithm 2, step 1):
 * one pass with uniform topic weights and m0 copies per token, followed by the parameter update.
 *   K                number of topics, 1 <= K <= 2048
 *   alpha, beta      Dirichlet priors of Eq. 6, > 0
 *   seed             key of the counter-based random stream
 *   m0               copies per token of the initial pass, >= 1
 *   tokens_per_draw  the c tokens of a nonzero are drawn in groups of at most this many
 *                    (each group is one multinomial of m * group-size copies), >= 1
 *   hip_stream       hipStream_t to run on (NULL = the default stream)
 * Synchronises with the stream before returning.  On failure *out is NULL.                     */
int same_lda_init(same_lda_t** out, const same_lda_csc* X, int32_t K, float alpha, float beta,
                  uint64_t seed, int32_t m0, int32_t tokens_per_draw, void* hip_stream);

/* One SAME sweep over the resident matrix (Algorithm 3, one iteration): zero the count
 * matrices, draw and scatter for every nonzero with m_t copies per token, then
 * theta = n_dk/m_t + alpha, phi_hat = (n_wk/m_t + beta) / (n_k/m_t + V*beta),
 * phi = (1-rho_t)*phi + rho_t*phi_hat (rho_t = 1 replaces phi).  Asynchronous.
 *   m_t    >= 1, m_t * (largest group size) < 2^24, and m_t * (tokens of any one document or word) < 2^32
 *          (the count matrices are 32-bit; the error text names the document or word)
 *   rho_t  in (0, 1]                                                                           */
int same_lda_sweep(same_lda_t* h, int32_t m_t, float rho_t);

/* The same sweep in the Poisson form of the factored draw (Section 4, second part; the sampling
 * line of Algorithm 3 as printed): the count of topic k for a group of g tokens is an independent
 * Poisson variable with rate m_t * g * w_k / mu, so the copies of a token no longer total exactly
 * m_t * c, and m_t may be any positive real (the real-valued schedules of Section 6.1.3 apply as
 * they are).  The update divides by the same real m_t.  Takes the next pass index of the training
 * stream like same_lda_sweep; the two forms may alternate on one handle.  Asynchronous.
 *   m_t    > 0, and m_t * (largest group size) < 2^22
 *   rho_t  in (0, 1]                                                                           */
int same_lda_sweep_poisson(same_lda_t* h, float m_t, float rho_t);

/* A sweep whose parameter step is sampled instead of collapsed (Algorithm 2, third step; Section
 * 3.1: given the m copies the parameters follow the product of the single-copy conditionals, for
 * LDA a Dirichlet again): the draws and counts are those of same_lda_sweep; then
 *   theta_d ~ Dirichlet(n_dk' + m_t*alpha), kept unnormalised with mean n_dk'/m_t + alpha,
 *   phi_k   ~ Dirichlet over words (n_wk' + m_t*beta),
 * whose means are the update of Eq. 6 and whose spread shrinks as m_t grows.  The Gamma variables
 * come from the handle's seed on streams of their own (Marsaglia-Tsang on Philox blocks, one per
 * attempt), so the result is a function of (seed, pass index, counts).  Takes the next pass index
 * like same_lda_sweep; the sweep forms may alternate on one handle.  Allocates nothing (its
 * (V/64 + 1) * K doubles of scratch belong to the handle from same_lda_init on).  Asynchronous.
 *   m_t    >= 1, and m_t * (largest group size) < 2^24                                         */
int same_lda_sweep_sampled(same_lda_t* h, int32_t m_t);

/* Per-word log-likelihood of held-out documents (Section 6.1.1): theta of the held-out
 * documents is fitted with phi frozen (a uniform-weight pass, then foldin_sweeps passes with
 * m_eval copies, on a separate random stream), then
 * ll = sum_i c_i * log( sum_k theta_dk phi_wk / sum_k theta_dk ) / sum_i c_i.
 * Allocates temporary device memory, synchronises, writes *ll_per_word (host).                 */
int same_lda_loglik(same_lda_t* h, const same_lda_csc* Xtest, int32_t foldin_sweeps,
                    int32_t m_eval, double* ll_per_word);

/* Release the handle and all its device memory (NULL is allowed). */
void same_lda_free(same_lda_t* h);

/* Replace the resident matrix by a new minibatch with the same vocabulary (Section 5.2):
 * phi is kept; theta of the new documents is initialised by one uniform-weight pass with
 * m_init copies per token.  Reallocates per-document state; synchronises.                      */
int same_lda_set_batch(same_lda_t* h, const same_lda_csc* X, int32_t m_init);

/* The same in two steps, for streams of minibatches (Section 5.2: the data as a stream of
 * minibatches; one sweep per minibatch): same_lda_stage_batch copies the next minibatch, builds
 * its work list and draws the initial pass of its documents on a second stream of the library,
 * while sweeps already enqueued on the handle's stream keep running; same_lda_commit_batch then
 * makes it the resident matrix.  Call order for overlap: same_lda_sweep (asynchronous), then
 * same_lda_stage_batch for the next minibatch, then same_lda_commit_batch.
 *   sweeps_ahead  number of same_lda_sweep / _sweep_poisson calls that will still be made before the
 *                 commit (0 in the order above).  The initial pass takes the pass index it would
 *                 have had in same_lda_set_batch at that point; if the count turns out different,
 *                 the commit draws the initial pass again, so results never depend on it.
 * A device matrix must be complete when stage_batch is called (it is read on another stream than the
 * handle's); a host matrix should be in pinned memory for the copy to overlap.  stage_batch returns when the
 * staged minibatch is complete (it waits for the device once, to release temporaries); a second
 * stage_batch replaces a staged minibatch that was not committed.                               */
int same_lda_stage_batch(same_lda_t* h, const same_lda_csc* X, int32_t m_init, int32_t sweeps_ahead);
int same_lda_commit_batch(same_lda_t* h);

/* Copy a state matrix out of / into the handle.  bytes must equal the matrix size.
 * same_lda_set accepts SAME_LDA_THETA and SAME_LDA_PHI only.  Both synchronise.                */
int same_lda_get(same_lda_t* h, int32_t which, void* dst, size_t bytes, int32_t dst_on_device);
int same_lda_set(same_lda_t* h, int32_t which, const void* src, size_t bytes, int32_t src_on_device);

/* Index of the next pass of the training stream (0 was the initialisation), and a setter so that
 * a run restored with same_lda_set continues bit-identically.                                   */
int same_lda_get_pass(const same_lda_t* h, int32_t* pass_index);
int same_lda_set_pass(same_lda_t* h, int32_t pass_index);

/* Number of draw tasks (groups of tokens) of the resident matrix: task ids are
 * 0 .. count-1 in storage order, ceil(c / tokens_per_draw) consecutive ids per nonzero.        */
int same_lda_task_count(const same_lda_t* h, int64_t* count);

/* Test hook: count vectors that the NEXT same_lda_sweep(h, m_t, .) will draw for the listed
 * tasks, computed by the same device code on the current theta and phi; state is not changed.
 *   task_ids    host, [n]
 *   counts_out  host, [n][K] uint32                                                            */
int same_lda_debug_draw(same_lda_t* h, int32_t m_t, const int64_t* task_ids, int32_t n,
                        uint32_t* counts_out);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): the same hook as same_lda_debug_draw, same arguments and same result, but it
 * calls no hipMalloc / hipFree: the staged task ids, the count rows and the draw kernel's segment counter live
 * in a device array that is part of the library (about 4.2 MB on every GPU the library runs on, held until the
 * process ends).  At most 4096 tasks and 2^20 counts (n * K) per call; more is refused with SAME_LDA_EINVAL.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two handles, two threads)
 * race; the array keeps the last call's contents and the call clears what it needs.  Synchronises.         */
int same_lda_debug_draw_noalloc(same_lda_t* h, int32_t m_t, const int64_t* task_ids, int32_t n,
                                uint32_t* counts_out);
/* The same hook as same_lda_debug_draw for the NEXT same_lda_sweep_poisson(h, m_t, .).           */
int same_lda_debug_draw_poisson(same_lda_t* h, float m_t, const int64_t* task_ids, int32_t n,
                                uint32_t* counts_out);

/* Test hook for the scatter of Algorithm 3's two accumulation lines.  A task records its (topic, count) pairs in a
 * slot of 15 and continues in 64-byte chunks taken from a pool in device memory that the handle allocates with its
 * matrix (at most eight chunks per slot and a quarter of the free memory); counts that find the pool used up are
 * added straight to the word rows.  Results never depend on the pool's size.  This call lowers the number of chunks a
 * sweep may use (0: none; negative: all that were allocated) so that tests reach the fallback at small sizes.
 *   chunks_in_use  host, optional out: chunks the sweeps may use after the call                      */
int same_lda_debug_chunk_limit(same_lda_t* h, int64_t max_chunks, int64_t* chunks_in_use);

/* The normaliser of Algorithm 3 as an operation of its own (Section 5.3, SDDMM: a product of two
 * dense matrices evaluated at the nonzeros of a sparse one): mu[i] = sum_k theta[d][k] * phi[w][k]
 * for every nonzero i = (d, w) of the resident matrix, in its storage order, from the current
 * theta and phi.  Accumulated in binary32 in a fixed tree order (not the running sum of the draw:
 * the two agree to rounding).  State is not changed.
 *   mu_out         [nnz] float, device (asynchronous) or host (synchronises)
 *   out_on_device  1 if mu_out is a device pointer
 * When kernel timing is enabled the launch is recorded like a draw launch.                       */
int same_lda_sddmm(same_lda_t* h, float* mu_out, int32_t out_on_device);

/* A second consumer of the normaliser (Section 5.3 names it as the bottleneck the sampler shares with online
 * variational Bayes LDA): the E-step of that method on the resident matrix.  The paper does not print the method;
 * the update is the published one (Hoffman, Blei and Bach, 2010):
 *     a_dk = exp(psi(gamma_dk) - psi(sum_k gamma_dk)),  b_wk = exp(psi(lambda_wk) - psi(sum_w lambda_wk)),
 *     mu_i = sum_k a_dk b_wk for nonzero i = (d, w, c),  gamma'_dk = alpha + a_dk sum_{i in d} (c_i / mu_i) b_wk.
 * psi and exp in double, sums over topics and nonzeros in binary32; the handle's theta and phi are not used or
 * changed.  All pointers are DEVICE pointers owned by the caller; both calls are asynchronous on the handle's
 * stream and allocate nothing.  Entries of lambda and gamma must be positive (not checked: others give NaN).
 * gamma' is unchanged when a word's row of b is multiplied by a constant, and exp of E[log beta] leaves the range
 * of binary32 for small lambda (psi(0.01) = -100.6): a row of b is therefore stored divided by its largest entry
 * and the logarithm of that entry is kept beside it.
 *
 * same_lda_vb_exp_elog_beta:
 *   lambda     [V][K] float, word-major like phi (a topic is a column, normalised over the V words)
 *   b_out      [V][K] float: exp(E[log beta_kw] - shift_w), the largest entry of every row is 1
 *   shift_out  [V] float: shift_w = max_k E[log beta_kw]
 * same_lda_vb_estep: `iters` iterations gamma -> gamma' for every document of the resident matrix.
 *   b, shift    from same_lda_vb_exp_elog_beta (shift may be null: log_mu_out then lacks the word's shift)
 *   alpha       the documents' Dirichlet prior of this method (positive; the handle's own alpha is not used)
 *   gamma       [D][K] float, in: the start (e.g. all ones), out: the result; iters = 0 leaves it as it is
 *   log_mu_out  [nnz] float or null: log mu_i of the last iteration, in storage order
 * When kernel timing is enabled the E-step launch is recorded like a draw launch.                     */
int same_lda_vb_exp_elog_beta(same_lda_t* h, const float* lambda, float* b_out, float* shift_out);
int same_lda_vb_estep(same_lda_t* h, const float* b, const float* shift, float alpha, int32_t iters, float* gamma,
                      float* log_mu_out);

/* Kernel timing.  When enabled, HIP events bracket the draw-and-scatter kernel of every sweep on
 * the handle's stream.  same_lda_get_timing synchronises, returns the summed duration (ms) and
 * the number of launches since the last call, and resets both.                                  */
int same_lda_set_timing(same_lda_t* h, int32_t enabled);
int same_lda_get_timing(same_lda_t* h, double* draw_ms_total, int64_t* launches);

/* Device self-test of building blocks that the parity tests exercise only indirectly (no handle
 * needed; runs on the current device's default stream and synchronises):
 *   - the Philox4x32-10 block function against the three published known-answer vectors
 *     (Salmon et al., SC'11);
 *   - the integer reciprocal used in the pmf walk against the correctly rounded 1/x for EVERY
 *     integer x in [1, 2^24);
 *   - the exclusive sum and the stable radix sort that build the work list, on a seeded million
 *     items, against the host's sum and the (key, position) order.
 * *failures (host) receives the number of mismatches; 0 means all hold.                         */
int same_lda_selftest(int64_t* failures);

/* Wait for everything enqueued on the handle's stream. */
int same_lda_synchronize(same_lda_t* h);

/* Text of the last failure of this handle (of the last failed same_lda_init when h is NULL).
 * The pointer stays valid until the next failing call.                                          */
const char* same_lda_last_error(const same_lda_t* h);

#ifdef __cplusplus
}
#endif
#endif /* SAME_LDA_H */
