/*
 * CPU oracle for the SAME Gibbs LDA sweep (test infrastructure, not product code).
 *
 * A plain, slow, single-file C implementation of what one SAME sweep computes,
 * written from the paper's text: Section 4 (the m tied copies of a latent
 * variable form one multinomial count vector), Section 5.1 / Eq. 6-7 (the LDA
 * update and its count statistics) and Algorithm 3 (zero the accumulators,
 * normaliser, draw, accumulate, add priors, normalise over words, blend).
 * It shares no code with the GPU library.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may use it.
 *
 * Everything that decides an integer is done in IEEE binary32 with one rounding
 * per operation (compile with -ffp-contract=off, no fast-math), so that a second
 * implementation following the same steps obtains the same integers.
 *
 * Parts the paper does not fix (build decisions; "parity unpinned" by the paper,
 * pinned only in distribution): how the multinomial count vector is drawn (here:
 * topic by topic from the top, each step placing the highest remaining copy and
 * the copies that share its topic), the binomial sampler, the random number
 * generator and its keying, the summation order, the grouping of a nonzero's
 * tokens into draws, the initialisation and the held-out fold-in.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 * as 1, 2, 3", SC'11): ten rounds; each round multiplies counter words 0 and 2
 * by two fixed constants, mixes the high halves with words 1 and 3 and the key,
 * and the key is advanced by the Weyl constants between rounds.               */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* A random word becomes a uniform in (0,1): its top 23 bits j give (2j+1)/2^24,
 * an odd multiple of 2^-24, exactly representable and never 0 or 1.           */
float oracle_uniform_from_word(uint32_t x)
{
    return (float)(2u * (x >> 9) + 1u) * 5.9604644775390625e-8f; /* 2^-24 */
}

/* Stream layouts.  One draw task (see oracle_pass) has a 40-bit id tau; the key
 * is the 64-bit seed; "pass" carries the pass index in its low 28 bits and a
 * stream domain (0 training, 1 held-out fold-in) above.
 *
 * Multinomial form (oracle_draw): the draw proceeds in steps 0, 1, 2, ... (one per
 * topic that receives copies).  Step s takes two uniforms from the block with
 * counter (tau_lo, tau_hi, s/2, pass): slot 0, word 2*(s mod 2), places the highest
 * remaining copy; slot 1, word 2*(s mod 2)+1, decides the first piece of the
 * step's binomial.  Slot j >= 2 (piece j-1 of that binomial) is word ((j-2) mod 4)
 * of the block (tau_lo, tau_hi | ((j-2)/4) << 8, 2^31 | s, pass).               */
static float chain_uniform(uint64_t seed, uint64_t tau, uint32_t step, uint32_t slot, uint32_t pass)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4], out[4];
    ctr[0] = (uint32_t)tau;
    ctr[1] = (uint32_t)(tau >> 32) & 0xFFu;
    ctr[3] = pass;
    if (slot < 2u) {
        ctr[2] = step >> 1;
        oracle_philox4x32_10(ctr, key, out);
        return oracle_uniform_from_word(out[2u * (step & 1u) + slot]);
    }
    ctr[1] |= ((slot - 2u) >> 2) << 8;
    ctr[2] = 0x80000000u | step;
    oracle_philox4x32_10(ctr, key, out);
    return oracle_uniform_from_word(out[(slot - 2u) & 3u]);
}

float oracle_chain_uniform(uint64_t seed, uint64_t tau, uint32_t step, uint32_t slot, uint32_t pass)
{
    return chain_uniform(seed, tau, step, slot, pass);
}

/* Poisson form (oracle_draw_poisson): the uniform that decides topic k's first
 * piece is word (k mod 4) of the block with counter (tau_lo, tau_hi, k/4, pass).
 * Piece j >= 1 of topic k uses word ((j-1) mod 4) of the block
 * (tau_lo, tau_hi | ((j-1)/4) << 8, 2^31 | k, pass).                            */
static float stream_uniform(uint64_t seed, uint64_t tau, uint32_t k, uint32_t piece, uint32_t pass)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4], out[4];
    ctr[0] = (uint32_t)tau;
    ctr[1] = (uint32_t)(tau >> 32) & 0xFFu;
    ctr[3] = pass;
    if (piece == 0) {
        ctr[2] = k >> 2;
        oracle_philox4x32_10(ctr, key, out);
        return oracle_uniform_from_word(out[k & 3u]);
    }
    ctr[1] |= ((piece - 1u) >> 2) << 8;
    ctr[2] = 0x80000000u | k;
    oracle_philox4x32_10(ctr, key, out);
    return oracle_uniform_from_word(out[(piece - 1u) & 3u]);
}

float oracle_stream_uniform(uint64_t seed, uint64_t tau, uint32_t k, uint32_t piece, uint32_t pass)
{
    return stream_uniform(seed, tau, k, piece, pass);
}

/* ------------------------------------------------------------------------- */
/* exp(-y) for 0 <= y <= 48 from + - * only, so that a second implementation
 * obtains the same bits: t = y*log2(e), n = trunc(t), f = t-n in [0,1),
 * g = f - 1/2, 2^-(g+1/2) by the degree-7 Taylor polynomial of
 * 2^-1/2 * exp(-g ln 2) in Horner form (every product and sum rounded once),
 * scaled by 2^-n.  Relative error below 3e-6, below 2e-7 for y <= 2 (tests).   */
float oracle_expneg(float y)
{
    static const float c[8] = {
        0.7071067811865476f,       /* 2^-1/2                      */
        -0.4901290717342736f,      /* 2^-1/2 * (-ln2)             */
        0.16986579209153746f,      /* 2^-1/2 * (ln2)^2 / 2        */
        -0.039247331620610344f,    /* 2^-1/2 * (-ln2)^3 / 6       */
        0.006801044314331813f,     /* 2^-1/2 * (ln2)^4 / 24       */
        -0.0009428249382684684f,   /* 2^-1/2 * (-ln2)^5 / 120     */
        0.00010891940795373223f,   /* 2^-1/2 * (ln2)^6 / 720      */
        -1.0785311504483996e-05f   /* 2^-1/2 * (-ln2)^7 / 5040    */
    };
    float t = y * 1.4426950408889634f;
    int n = (int)t;
    float f = t - (float)n;
    float g = f - 0.5f;
    float p = c[7];
    for (int i = 6; i >= 0; --i) {
        p = p * g;
        p = p + c[i];
    }
    return ldexpf(p, -n);
}

/* log x for a positive normal x: x = 2^e * f with f in [sqrt(1/2), sqrt(2)),
 * log f = 2 atanh(s), s = (f-1)/(f+1), by the odd series up to s^11.         */
float oracle_flog(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, sizeof bits);
    int32_t e = (int32_t)(bits >> 23) - 127;
    uint32_t fb = (bits & 0x007FFFFFu) | 0x3F800000u;
    float f;
    memcpy(&f, &fb, sizeof f);
    if (f > 1.41421354f) { f = f * 0.5f; e += 1; }
    float num = f - 1.0f, den = f + 1.0f;
    float s = num / den;
    float z = s * s;
    float p = 0.0909090936f;
    p = p * z; p = p + 0.111111112f;
    p = p * z; p = p + 0.142857149f;
    p = p * z; p = p + 0.2f;
    p = p * z; p = p + 0.333333343f;
    p = p * z; p = p + 1.0f;
    float lf = 2.0f * s;
    lf = lf * p;
    float le = (float)e * 0.693147182f;
    return le + lf;
}

/* -log(1 - x) for 0 < x <= 1/2 without ever rounding 1 - x (which would lose x
 * below 2^-24): log((1+t)/(1-t)) = 2 atanh(t) with t = x / (2 - x), by the odd
 * series through t^17 in Horner form.  Relative error below 3e-7 (tests).      */
float oracle_log1m(float x)
{
    float den = 2.0f - x;
    float t = x / den;
    float z = t * t;
    float p = 0.0588235296f;                 /* 1/17 */
    p = p * z; p = p + 0.0666666701f;        /* 1/15 */
    p = p * z; p = p + 0.0769230798f;        /* 1/13 */
    p = p * z; p = p + 0.0909090936f;        /* 1/11 */
    p = p * z; p = p + 0.111111112f;         /* 1/9  */
    p = p * z; p = p + 0.142857149f;         /* 1/7  */
    p = p * z; p = p + 0.2f;
    p = p * z; p = p + 0.333333343f;
    p = p * z; p = p + 1.0f;
    float two_t = 2.0f * t;
    return two_t * p;
}

/* Binomial(n, qq) for one piece by inversion: walk the pmf upward from 0,
 * pm(x) = pm(x-1) * r * (n-x+1) / x with r = qq/(1-qq), until the cdf reaches
 * u.  The walk also ends when the pmf has fallen below the resolution of the
 * running cdf (the tail is numerically exhausted).                            */
uint32_t oracle_binom_walk(uint32_t n, float pm0, float r, float u)
{
    uint32_t x = 0;
    float pm = pm0, cdf = pm0;
    while (u > cdf && x < n) {
        x += 1;
        float inv_x = 1.0f / (float)x;
        pm = pm * r;
        pm = pm * (float)(n - x + 1u);
        pm = pm * inv_x;
        float next = cdf + pm;
        if (next == cdf) break;
        cdf = next;
    }
    return x;
}

/* n ~ Binomial(R, q), the binomial of step `step` of task tau.  The smaller of q
 * and 1-q is sampled (the result is complemented for q > 1/2).  One piece of R
 * trials serves when R*qq <= 32; otherwise R is cut into pieces of floor(32/qq)
 * trials and a shorter last one, each with its own uniform, so that the
 * probability of zero successes never underflows.  That probability, (1-qq)^n,
 * is exp(-n * (-log(1-qq))) with the two functions above: forming 1-qq first
 * would round qq to a multiple of 2^-24 and the pmf would no longer sum to one
 * (for millions of trials the missing mass exceeds the law's own).            */
uint32_t oracle_binom(uint32_t R, float q, uint64_t seed, uint64_t tau, uint32_t step, uint32_t pass)
{
    if (R == 0 || !(q > 0.0f)) return 0;
    if (q >= 1.0f) return R;
    int flip = q > 0.5f;
    float qq = flip ? 1.0f - q : q;
    float s = 1.0f - qq;
    float r = qq / s;
    float lq = oracle_log1m(qq);
    int single = ((float)R * qq) <= 32.0f;
    uint32_t L = single ? R : (uint32_t)(32.0f / qq);
    uint32_t rem = R, piece = 0, total = 0;
    while (rem > 0) {
        uint32_t n = rem < L ? rem : L;
        float pm0 = oracle_expneg((float)n * lq);
        float u = chain_uniform(seed, tau, step, 1u + piece, pass);
        total += oracle_binom_walk(n, pm0, r, u);
        rem -= n;
        piece += 1;
    }
    return flip ? R - total : total;
}

/* Running sums of the weights in two levels.  The K topics are taken in blocks
 * of T = 4*ceil(K/128) consecutive topics (at most 32 blocks; T = 8 at K = 256).
 * Inside a block the weights are added left to right starting from zero
 * (r_0 = w_0, r_j = r_{j-1} + w_j); the sums S of whole blocks are added left to
 * right (S = 0 before the first block); P[k] = S + r.  P is non-decreasing, the
 * last P of a block is the S of the next, and the return value P[K-1] is the
 * normaliser mu of Algorithm 3.                                                */
int32_t oracle_block_len(int32_t K)
{
    return 4 * ((K + 127) / 128);
}

float oracle_prefix(int32_t K, const float* w, float* P)
{
    int32_t T = oracle_block_len(K);
    float S = 0.0f;
    for (int32_t b0 = 0; b0 < K; b0 += T) {
        float r = 0.0f;
        int32_t b1 = b0 + T < K ? b0 + T : K;
        for (int32_t k = b0; k < b1; ++k) {
            r = r + w[k];
            P[k] = S + r;
        }
        S = S + r;
    }
    return S;
}

/* Position of the highest of R copies spread uniformly over (0, U): the largest of
 * R independent uniforms has distribution function (y/U)^R, so y = U * u^(1/R)
 * for one uniform u; u^(1/R) = exp(log(u)/R) with the logarithm and exponential
 * above.  One copy needs neither.                                              */
float oracle_top_position(float U, uint32_t R, float u)
{
    float y;
    if (R == 1u) {
        y = U * u;
    } else {
        float a = -oracle_flog(u);
        float z = a / (float)R;
        float e = oracle_expneg(z);
        if (e > 1.0f) e = 1.0f;
        y = U * e;
    }
    if (!(y > 0.0f)) y = U;
    return y;
}

/* The factored draw (Section 4): the N = m*g copies of a latent topic variable
 * with conditional weights w[0..K) are one Multinomial(N, w/sum w) count
 * vector.  Picture every copy as a point uniform on (0, mu), topic k owning the
 * interval (P[k-1], P[k]].  The draw walks down from the top, one step per topic
 * that receives copies.  With R copies left, all of them below U:
 *   - the highest copy sits at y = oracle_top_position(U, R, u); its topic is the
 *     first k with P[k] >= y;
 *   - given y, the other R-1 copies are uniform on (0, y), so each of them falls
 *     into the same topic, i.e. above P[k-1], with probability q = (y - P[k-1]) / y:
 *     that topic receives 1 + Binomial(R-1, q) copies;
 *   - the copies left are all below P[k-1], the next step's U.
 * Returns mu.  scratch holds K floats.                                         */
float oracle_draw(int32_t K, const float* w, uint32_t N, uint64_t seed, uint64_t tau,
                  uint32_t pass, uint32_t* counts, float* scratch)
{
    float* P = scratch;
    float mu = oracle_prefix(K, w, P);
    for (int32_t k = 0; k < K; ++k) counts[k] = 0;
    uint32_t R = N, step = 0;
    float U = mu;
    int32_t top = K;                    /* the copies left belong to topics below top */
    while (R > 0) {
        if (!(U > 0.0f)) { counts[top - 1] += R; break; }       /* no weight left: a degenerate input */
        float u = chain_uniform(seed, tau, step, 0, pass);
        float y = oracle_top_position(U, R, u);
        int32_t k = 0;
        while (k < top - 1 && !(P[k] >= y)) ++k;                 /* P[top-1] == U >= y */
        float prev = k > 0 ? P[k - 1] : 0.0f;
        uint32_t n = 1;
        if (R > 1u) {
            float width = y - prev;
            float q = width / y;
            n += oracle_binom(R - 1u, q, seed, tau, step, pass);
        }
        counts[k] += n;
        R -= n;
        U = prev;
        top = k;
        step += 1;
        if (top == 0 && R > 0) { counts[0] += R; break; }       /* k = 0 gives q = 1: nothing can be left */
    }
    return mu;
}

/* ------------------------------------------------------------------------- */
/* Poisson form of the factored draw (Section 4, second part; Algorithm 3, the
 * sampling line): the count of topic k among the copies of a latent variable is
 * an independent Poisson variable with rate (number of copies) * P(topic k).
 * The number of copies may be any positive real.  exp(-rate) is oracle_expneg.  */

/* Poisson(rate) for one piece by inversion: walk the pmf upward from 0,
 * pm(x) = pm(x-1) * rate / x, until the cdf reaches u or the pmf has fallen
 * below the resolution of the running cdf.                                   */
uint32_t oracle_poisson_walk(float rate, float pm0, float u)
{
    uint32_t x = 0;
    float pm = pm0, cdf = pm0;
    while (u > cdf) {
        x += 1;
        float inv_x = 1.0f / (float)x;
        pm = pm * rate;
        pm = pm * inv_x;
        float next = cdf + pm;
        if (next == cdf) break;
        cdf = next;
    }
    return x;
}

/* z ~ Poisson(lambda) for topic k of task tau.  A rate above 32 is cut into
 * J = trunc(lambda/32) + 1 equal pieces (a sum of independent Poisson variables
 * is Poisson with the summed rate), so that exp(-rate) never underflows; each
 * piece has its own uniform (same stream layout as the binomial pieces).      */
uint32_t oracle_poisson(float lambda, uint64_t seed, uint64_t tau, uint32_t k, uint32_t pass)
{
    if (!(lambda > 0.0f)) return 0;
    uint32_t J = 1;
    float rate = lambda;
    if (lambda > 32.0f) {
        J = (uint32_t)(lambda / 32.0f) + 1u;
        rate = lambda / (float)J;
    }
    float pm0 = oracle_expneg(rate);
    uint32_t total = 0;
    for (uint32_t piece = 0; piece < J; ++piece) {
        float u = stream_uniform(seed, tau, k, piece, pass);
        total += oracle_poisson_walk(rate, pm0, u);
    }
    return total;
}

/* All topics of one task: with Nf copies (a positive real) and weights w,
 * counts[k] ~ Poisson(Nf * w_k / mu), mu = w_0 + ... + w_{K-1} accumulated left
 * to right (the same normaliser as in oracle_draw).  Returns mu.              */
float oracle_draw_poisson(int32_t K, const float* w, float Nf, uint64_t seed, uint64_t tau,
                          uint32_t pass, uint32_t* counts)
{
    float mu = w[0];
    for (int32_t k = 1; k < K; ++k) mu = mu + w[k];
    for (int32_t k = 0; k < K; ++k) {
        counts[k] = 0;
        if (!(w[k] > 0.0f)) continue;
        float scaled = Nf * w[k];
        float lambda = scaled / mu;
        counts[k] = oracle_poisson(lambda, seed, tau, (uint32_t)k, pass);
    }
    return mu;
}

/* ------------------------------------------------------------------------- */
/* Draw tasks.  A nonzero (d, w, c) stands for c tokens with identical
 * conditionals; its tokens are drawn in groups of at most G: task j of the
 * nonzero covers g = min(G, c - j*G) tokens and draws Multinomial(m*g, p).
 * Task ids number the tasks of all nonzeros consecutively in storage order.   */
static uint32_t tasks_of(float c, int32_t G)
{
    uint32_t ci = (uint32_t)c;
    return (ci + (uint32_t)G - 1u) / (uint32_t)G;
}

int64_t oracle_task_count(int64_t nnz, const float* val, int32_t G)
{
    int64_t n = 0;
    for (int64_t i = 0; i < nnz; ++i) n += tasks_of(val[i], G);
    return n;
}

/* task_base[i] = id of the first task of nonzero i (task_base has nnz+1 entries). */
void oracle_task_base(int64_t nnz, const float* val, int32_t G, int64_t* task_base)
{
    int64_t n = 0;
    for (int64_t i = 0; i < nnz; ++i) { task_base[i] = n; n += tasks_of(val[i], G); }
    task_base[nnz] = n;
}

static void fill_weights(int32_t K, const float* theta_d, const float* phi_w, float* w)
{
    if (theta_d == NULL) { for (int32_t k = 0; k < K; ++k) w[k] = 1.0f; return; }
    for (int32_t k = 0; k < K; ++k) w[k] = theta_d[k] * phi_w[k];
}

/* One pass over all nonzeros of a CSC matrix whose columns are documents
 * (Algorithm 3, the loop over document-word pairs): for every task form the
 * weights theta[d][k]*phi[w][k] (all ones when theta == NULL: the random
 * initialisation), draw the count vector and add it to ndk[d][.] and, unless
 * nwk == NULL, to nwk[w][.].  mu (may be NULL) receives the normaliser of each
 * nonzero.  theta is [D][K], phi is [V][K] (word-major), counts are u32.      */
void oracle_pass(int32_t D, int32_t V, const int32_t* colptr, const int32_t* rowidx,
                 const float* val, int32_t K, int32_t G, uint32_t m, uint64_t seed,
                 uint32_t pass, const float* theta, const float* phi,
                 uint32_t* ndk, uint32_t* nwk, float* mu)
{
    (void)V;
    int64_t nnz = colptr[D];
    int64_t* base = (int64_t*)malloc((size_t)(nnz + 1) * sizeof(int64_t));
    oracle_task_base(nnz, val, G, base);
#pragma omp parallel
    {
        float* w = (float*)malloc((size_t)K * sizeof(float));
        float* scratch = (float*)malloc((size_t)K * sizeof(float));
        uint32_t* cnt = (uint32_t*)malloc((size_t)K * sizeof(uint32_t));
#pragma omp for schedule(dynamic, 64)
        for (int32_t d = 0; d < D; ++d) {
            for (int64_t i = colptr[d]; i < colptr[d + 1]; ++i) {
                int32_t word = rowidx[i];
                uint32_t c = (uint32_t)val[i];
                fill_weights(K, theta ? theta + (size_t)d * K : NULL,
                             phi ? phi + (size_t)word * K : NULL, w);
                uint32_t ntask = tasks_of(val[i], G);
                for (uint32_t j = 0; j < ntask; ++j) {
                    uint32_t g = c - j * (uint32_t)G;
                    if (g > (uint32_t)G) g = (uint32_t)G;
                    float S = oracle_draw(K, w, m * g, seed, (uint64_t)(base[i] + j), pass, cnt, scratch);
                    if (mu && j == 0) mu[i] = S;
                    for (int32_t k = 0; k < K; ++k) {
                        if (cnt[k] == 0) continue;
                        ndk[(size_t)d * K + k] += cnt[k];   /* document d belongs to this thread */
                        if (nwk) {
#pragma omp atomic
                            nwk[(size_t)word * K + k] += cnt[k];
                        }
                    }
                }
            }
        }
        free(w); free(scratch); free(cnt);
    }
    free(base);
}

/* Count vectors of selected tasks (for sampled parity checks at large sizes).
 * out is [n][K].  task_ids must be valid ids of this matrix.                  */
void oracle_draw_tasks(int32_t D, const int32_t* colptr, const int32_t* rowidx, const float* val,
                       int32_t K, int32_t G, uint32_t m, uint64_t seed, uint32_t pass,
                       const float* theta, const float* phi,
                       int64_t n, const int64_t* task_ids, uint32_t* out)
{
    int64_t nnz = colptr[D];
    int64_t* base = (int64_t*)malloc((size_t)(nnz + 1) * sizeof(int64_t));
    oracle_task_base(nnz, val, G, base);
    float* w = (float*)malloc((size_t)K * sizeof(float));
    float* scratch = (float*)malloc((size_t)K * sizeof(float));
    for (int64_t t = 0; t < n; ++t) {
        int64_t tau = task_ids[t];
        int64_t lo = 0, hi = nnz;            /* last nonzero whose base <= tau */
        while (hi - lo > 1) { int64_t mid = (lo + hi) / 2; if (base[mid] <= tau) lo = mid; else hi = mid; }
        int64_t i = lo;
        int32_t dl = 0, dh = D;              /* document holding nonzero i */
        while (dh - dl > 1) { int32_t mid = (dl + dh) / 2; if (colptr[mid] <= i) dl = mid; else dh = mid; }
        int32_t d = dl;
        uint32_t j = (uint32_t)(tau - base[i]);
        uint32_t c = (uint32_t)val[i];
        uint32_t g = c - j * (uint32_t)G;
        if (g > (uint32_t)G) g = (uint32_t)G;
        fill_weights(K, theta ? theta + (size_t)d * K : NULL,
                     phi ? phi + (size_t)rowidx[i] * K : NULL, w);
        oracle_draw(K, w, m * g, seed, (uint64_t)tau, pass, out + (size_t)t * K, scratch);
    }
    free(w); free(scratch); free(base);
}

/* The same pass in the Poisson form: m is a positive real, a task of g tokens
 * has Nf = m*g copies (one rounded product).                                  */
void oracle_pass_poisson(int32_t D, int32_t V, const int32_t* colptr, const int32_t* rowidx,
                         const float* val, int32_t K, int32_t G, float m, uint64_t seed,
                         uint32_t pass, const float* theta, const float* phi,
                         uint32_t* ndk, uint32_t* nwk)
{
    (void)V;
    int64_t nnz = colptr[D];
    int64_t* base = (int64_t*)malloc((size_t)(nnz + 1) * sizeof(int64_t));
    oracle_task_base(nnz, val, G, base);
#pragma omp parallel
    {
        float* w = (float*)malloc((size_t)K * sizeof(float));
        uint32_t* cnt = (uint32_t*)malloc((size_t)K * sizeof(uint32_t));
#pragma omp for schedule(dynamic, 64)
        for (int32_t d = 0; d < D; ++d) {
            for (int64_t i = colptr[d]; i < colptr[d + 1]; ++i) {
                int32_t word = rowidx[i];
                uint32_t c = (uint32_t)val[i];
                fill_weights(K, theta + (size_t)d * K, phi + (size_t)word * K, w);
                uint32_t ntask = tasks_of(val[i], G);
                for (uint32_t j = 0; j < ntask; ++j) {
                    uint32_t g = c - j * (uint32_t)G;
                    if (g > (uint32_t)G) g = (uint32_t)G;
                    float Nf = m * (float)g;
                    oracle_draw_poisson(K, w, Nf, seed, (uint64_t)(base[i] + j), pass, cnt);
                    for (int32_t k = 0; k < K; ++k) {
                        if (cnt[k] == 0) continue;
                        ndk[(size_t)d * K + k] += cnt[k];   /* document d belongs to this thread */
                        if (nwk) {
#pragma omp atomic
                            nwk[(size_t)word * K + k] += cnt[k];
                        }
                    }
                }
            }
        }
        free(w); free(cnt);
    }
    free(base);
}

void oracle_draw_tasks_poisson(int32_t D, const int32_t* colptr, const int32_t* rowidx, const float* val,
                               int32_t K, int32_t G, float m, uint64_t seed, uint32_t pass,
                               const float* theta, const float* phi,
                               int64_t n, const int64_t* task_ids, uint32_t* out)
{
    int64_t nnz = colptr[D];
    int64_t* base = (int64_t*)malloc((size_t)(nnz + 1) * sizeof(int64_t));
    oracle_task_base(nnz, val, G, base);
    float* w = (float*)malloc((size_t)K * sizeof(float));
    for (int64_t t = 0; t < n; ++t) {
        int64_t tau = task_ids[t];
        int64_t lo = 0, hi = nnz;            /* last nonzero whose base <= tau */
        while (hi - lo > 1) { int64_t mid = (lo + hi) / 2; if (base[mid] <= tau) lo = mid; else hi = mid; }
        int64_t i = lo;
        int32_t dl = 0, dh = D;              /* document holding nonzero i */
        while (dh - dl > 1) { int32_t mid = (dl + dh) / 2; if (colptr[mid] <= i) dl = mid; else dh = mid; }
        int32_t d = dl;
        uint32_t j = (uint32_t)(tau - base[i]);
        uint32_t c = (uint32_t)val[i];
        uint32_t g = c - j * (uint32_t)G;
        if (g > (uint32_t)G) g = (uint32_t)G;
        fill_weights(K, theta + (size_t)d * K, phi + (size_t)rowidx[i] * K, w);
        oracle_draw_poisson(K, w, m * (float)g, seed, (uint64_t)tau, pass, out + (size_t)t * K);
    }
    free(w); free(base);
}

/* ------------------------------------------------------------------------- */
/* The normaliser of Algorithm 3 as an operation of its own (Section 5.3: a sampled
 * dense-dense matrix product): mu[i] = sum_k theta[d][k] * phi[w][k] for every
 * nonzero i = (d, w) of the matrix, evaluated in double.                        */
void oracle_sddmm(int32_t D, const int32_t* colptr, const int32_t* rowidx, int32_t K,
                  const float* theta, const float* phi, double* mu)
{
    for (int32_t d = 0; d < D; ++d) {
        for (int64_t i = colptr[d]; i < colptr[d + 1]; ++i) {
            const float* t = theta + (size_t)d * K;
            const float* p = phi + (size_t)rowidx[i] * K;
            double acc = 0.0;
            for (int32_t k = 0; k < K; ++k) acc += (double)t[k] * (double)p[k];
            mu[i] = acc;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Parameter update (Eq. 6 and Algorithm 3's last three steps).  Counts hold all
 * m copies, so they are divided by m; theta keeps its prior and stays
 * unnormalised (its per-document normaliser cancels in the draw); phi gets its
 * prior and is normalised over words per topic (the c_k../m + W*beta term of
 * Eq. 6), then blended into the running model with weight rho.                */
void oracle_theta_update_real(int32_t D, int32_t K, const uint32_t* ndk, float mf, float alpha, float* theta)
{
    for (size_t e = 0; e < (size_t)D * K; ++e) {
        float avg = (float)ndk[e] / mf;
        theta[e] = avg + alpha;
    }
}

void oracle_phi_update_real(int32_t V, int32_t K, const uint32_t* nwk, float mf, float beta, float rho, float* phi)
{
    float vbeta = (float)V * beta;
    float one_minus_rho = 1.0f - rho;
    for (int32_t k = 0; k < K; ++k) {
        uint64_t nk = 0;
        for (int32_t w = 0; w < V; ++w) nk += nwk[(size_t)w * K + k];
        float avg_k = (float)nk / mf;
        float den = avg_k + vbeta;
        for (int32_t w = 0; w < V; ++w) {
            float avg = (float)nwk[(size_t)w * K + k] / mf;
            float num = avg + beta;
            float hat = num / den;
            if (rho == 1.0f) {
                phi[(size_t)w * K + k] = hat;
            } else {
                float keep = one_minus_rho * phi[(size_t)w * K + k];
                float add = rho * hat;
                phi[(size_t)w * K + k] = keep + add;
            }
        }
    }
}

/* The multinomial form counts exactly m copies per token: m is an integer there. */
void oracle_theta_update(int32_t D, int32_t K, const uint32_t* ndk, uint32_t m, float alpha, float* theta)
{
    oracle_theta_update_real(D, K, ndk, (float)m, alpha, theta);
}

void oracle_phi_update(int32_t V, int32_t K, const uint32_t* nwk, uint32_t m, float beta, float rho, float* phi)
{
    oracle_phi_update_real(V, K, nwk, (float)m, beta, rho, phi);
}

/* ------------------------------------------------------------------------- */
/* The sampled parameter step (Algorithm 2, third step; Section 3.1: the
 * conditional of the parameters given the m copies is the product of the m
 * single-copy conditionals, for LDA a Dirichlet again).  Taken here as
 *   theta_d ~ Dirichlet(n_dk + m*alpha),   phi_k ~ Dirichlet over words (n_wk + m*beta),
 * whose means are exactly the collapsed update of Eq. 6 and whose spread
 * shrinks as m grows.  A Dirichlet vector is a vector of independent
 * Gamma(shape, 1) variables divided by their sum.  theta is left unnormalised
 * as in the collapsed update (its Gamma variables are divided by m, so that its
 * mean is n_dk/m + alpha); phi is normalised over words per topic.
 *
 * Gamma variables: Marsaglia and Tsang, "A simple method for generating gamma
 * variables" (ACM TOMS 26, 2000): with d = a - 1/3 and c = 1/sqrt(9d), draw a
 * standard normal z, set v = (1 + c z)^3, accept d*v when v > 0 and
 * log u < z^2/2 + d (1 - v + log v) (first tried without logarithms:
 * u < 1 - 0.0331 z^4); a shape below one uses Gamma(a+1) * u'^(1/a).  The normal
 * comes from two uniforms (Box and Muller).  Attempt j of element (row, k) takes
 * the Philox block with counter (row, k, j, pass word); its words give the two
 * uniforms of the normal, the acceptance uniform and the uniform of the
 * small-shape factor.  After 64 refused attempts (probability below 1e-80) the
 * shape itself is returned.
 *
 * Logarithm, cosine and exponential are evaluated from + - * / only, one
 * rounding each, so that a second implementation takes the same decisions.   */

/* cos(2 pi u) for u in (0,1): the quarter turn and the angle inside it, then the
 * Taylor polynomial of sine or cosine on [0, pi/2).                           */
float oracle_cos2pi(float u)
{
    float t = u * 4.0f;
    int32_t quarter = (int32_t)t;
    float frac = t - (float)quarter;
    float x = frac * 1.57079637f;
    float x2 = x * x;
    float sn = 1.60590444e-10f;
    sn = sn * x2; sn = sn + -2.50521079e-08f;
    sn = sn * x2; sn = sn + 2.75573188e-06f;
    sn = sn * x2; sn = sn + -0.000198412701f;
    sn = sn * x2; sn = sn + 0.00833333377f;
    sn = sn * x2; sn = sn + -0.166666672f;
    sn = sn * x2; sn = sn + 1.0f;
    sn = sn * x;
    float cs = -1.14707454e-11f;
    cs = cs * x2; cs = cs + 2.08767570e-09f;
    cs = cs * x2; cs = cs + -2.75573188e-07f;
    cs = cs * x2; cs = cs + 2.48015876e-05f;
    cs = cs * x2; cs = cs + -0.00138888892f;
    cs = cs * x2; cs = cs + 0.0416666679f;
    cs = cs * x2; cs = cs + -0.5f;
    cs = cs * x2; cs = cs + 1.0f;
    switch (quarter & 3) {
        case 0:  return cs;
        case 1:  return -sn;
        case 2:  return -cs;
        default: return sn;
    }
}

/* Standard normal from two uniforms in (0,1). */
float oracle_normal(float u1, float u2)
{
    float l = oracle_flog(u1);
    float r2 = -2.0f * l;
    float r = sqrtf(r2);
    return r * oracle_cos2pi(u2);
}

float oracle_gamma(float a, uint64_t seed, uint32_t row, uint32_t k, uint32_t pass)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    int small = a < 1.0f;
    float a1 = small ? a + 1.0f : a;
    float d = a1 - 0.333333343f;
    float nine_d = 9.0f * d;
    float c = 1.0f / sqrtf(nine_d);
    float g = a1;
    uint32_t out[4] = { 0, 0, 0, 0 };
    for (uint32_t attempt = 0; attempt < 64u; ++attempt) {
        uint32_t ctr[4] = { row, k, attempt, pass };
        oracle_philox4x32_10(ctr, key, out);
        float z = oracle_normal(oracle_uniform_from_word(out[0]), oracle_uniform_from_word(out[1]));
        float u = oracle_uniform_from_word(out[2]);
        float cz = c * z;
        float t = 1.0f + cz;
        if (!(t > 0.0f)) continue;
        float v = t * t;
        v = v * t;
        float z2 = z * z;
        float z4 = z2 * z2;
        float squeeze = 0.0331f * z4;
        squeeze = 1.0f - squeeze;
        int accept = u < squeeze;
        if (!accept) {
            float lhs = oracle_flog(u);
            float half = 0.5f * z2;
            float one_minus_v = 1.0f - v;
            float inner = one_minus_v + oracle_flog(v);
            float rhs = d * inner;
            rhs = half + rhs;
            accept = lhs < rhs;
        }
        if (accept) { g = d * v; break; }
    }
    if (small) {
        float l = oracle_flog(oracle_uniform_from_word(out[3]));
        float y = -l;
        y = y / a;
        if (y > 200.0f) y = 200.0f;
        g = g * oracle_expneg(y);
    }
    if (g < 1e-30f) g = 1e-30f;
    return g;
}

void oracle_theta_sample(int32_t D, int32_t K, const uint32_t* ndk, float mf, float alpha,
                         uint64_t seed, uint32_t pass, float* theta)
{
    float prior = mf * alpha;
#pragma omp parallel for schedule(static)
    for (int32_t d = 0; d < D; ++d)
        for (int32_t k = 0; k < K; ++k) {
            float a = (float)ndk[(size_t)d * K + k] + prior;
            float g = oracle_gamma(a, seed, (uint32_t)d, (uint32_t)k, pass);
            theta[(size_t)d * K + k] = g / mf;
        }
}

void oracle_phi_sample(int32_t V, int32_t K, const uint32_t* nwk, float mf, float beta,
                       uint64_t seed, uint32_t pass, float* phi)
{
    float prior = mf * beta;
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < K; ++k) {
        double total = 0.0;
        for (int32_t w = 0; w < V; ++w) {
            float a = (float)nwk[(size_t)w * K + k] + prior;
            float g = oracle_gamma(a, seed, (uint32_t)w, (uint32_t)k, pass);
            phi[(size_t)w * K + k] = g;
            total += (double)g;
        }
        float den = (float)total;
        for (int32_t w = 0; w < V; ++w) phi[(size_t)w * K + k] = phi[(size_t)w * K + k] / den;
    }
}

/* Per-word log-likelihood of a matrix under (theta, phi) (Section 6.1.1):
 * sum_i c_i * log( sum_k theta_dk phi_wk / sum_k theta_dk ) / sum_i c_i.
 * phi is already normalised over words.  The inner sum is the fp32 normaliser
 * of the draw; logs and the outer sum are in double.                          */
double oracle_loglik_eval(int32_t D, const int32_t* colptr, const int32_t* rowidx, const float* val,
                          int32_t K, const float* theta, const float* phi)
{
    double total = 0.0, tokens = 0.0;
    for (int32_t d = 0; d < D; ++d) {
        double tsum = 0.0;
        for (int32_t k = 0; k < K; ++k) tsum += (double)theta[(size_t)d * K + k];
        double log_tsum = log(tsum);
        for (int64_t i = colptr[d]; i < colptr[d + 1]; ++i) {
            const float* ph = phi + (size_t)rowidx[i] * K;
            const float* th = theta + (size_t)d * K;
            float S = th[0] * ph[0];
            for (int32_t k = 1; k < K; ++k) { float wk = th[k] * ph[k]; S = S + wk; }
            total += (double)val[i] * (log((double)S) - log_tsum);
            tokens += (double)val[i];
        }
    }
    return tokens > 0.0 ? total / tokens : 0.0;
}
