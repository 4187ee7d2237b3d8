// E-step of online variational Bayes LDA on the normaliser of Algorithm 3 (Section 5.3: the product of two
// dense matrices at the nonzeros of a sparse one is the bottleneck the sampler shares with online variational
// Bayes LDA).  The paper does not print that method; the update below is the published one (Hoffman, Blei and
// Bach, 2010), restated:
//     a_dk = exp(psi(gamma_dk) - psi(sum_k gamma_dk)),   b_wk = exp(psi(lambda_wk) - psi(sum_w lambda_wk)),
//     mu_i = sum_k a_dk b_wk  for nonzero i = (d, w, c),   gamma'_dk = alpha + a_dk sum_{i in d} (c_i / mu_i) b_wk.
// psi and exp are evaluated in double (they are a few per row element and iteration), mu in binary32 with fused
// multiply-adds, the sums over a document's nonzeros and gamma itself in double.  gamma' does not change when a word's row of b is
// multiplied by a constant (mu_i takes the same factor): rows of b are stored divided by their largest entry,
// with the logarithm of that entry beside them, and the normaliser is returned as log mu.
#pragma once
#include "update_kernels.h"

namespace same {

// psi(x) for x > 0: the recurrence psi(x) = psi(x + 1) - 1/x up to x >= 6, then the asymptotic series
// ln x - 1/(2x) - sum_n B_2n / (2n x^2n) through x^-14 (below 1e-12 there).
__device__ __forceinline__ double digamma_d(double x)
{
    double r = 0.0;
    while (x < 6.0) { r -= 1.0 / x; x += 1.0; }
    const double f = 1.0 / (x * x);
    const double t = f * (1.0 / 12.0 - f * (1.0 / 120.0 - f * (1.0 / 252.0 - f * (1.0 / 240.0 - f * (1.0 / 132.0
                     - f * (691.0 / 32760.0 - f * (1.0 / 12.0)))))));
    return r + log(x) - 0.5 / x - t;
}

constexpr int kVbRows = 64;             // rows of lambda per workgroup of the column sums

// partial[blk][k] = sum of lambda[w][k] over the workgroup's rows, in row order, in double
__global__ __launch_bounds__(256) void vb_colsum_kernel(const float* __restrict__ lam, int V, int K,
                                                        double* __restrict__ partial)
{
    const int w0 = blockIdx.x * kVbRows;
    const int w1 = w0 + kVbRows < V ? w0 + kVbRows : V;
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
        double s = 0.0;
        for (int w = w0; w < w1; ++w) s += (double)lam[(size_t)w * K + k];
        partial[(size_t)blockIdx.x * K + k] = s;
    }
}

// psi_total[k] = psi(sum_w lambda[w][k]): the block sums are added in block order (results repeat from run to run)
__global__ void vb_colpsi_kernel(const double* __restrict__ partial, int blocks, int K, double* __restrict__ psi_total)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    double s = 0.0;
    for (int b = 0; b < blocks; ++b) s += partial[(size_t)b * K + k];
    psi_total[k] = digamma_d(s);
}

// One wave per word: e_k = psi(lambda[w][k]) - psi_total[k] (= E[log beta_kw]); shift[w] = max_k e_k;
// b[w][k] = exp(e_k - shift[w]).  The largest entry of a row is 1: a word's row never underflows as a whole,
// whatever the size of its lambda (psi(0.01) is -100.6, and exp of that is not a binary32 number).
__global__ __launch_bounds__(256) void vb_exp_elog_beta_kernel(const float* __restrict__ lam, int V, int K,
                                                               const double* __restrict__ psi_total,
                                                               float* __restrict__ b, float* __restrict__ shift)
{
    const int lane = threadIdx.x & 63;
    const int w = (int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    if (w >= V) return;                                            // the whole wave
    const float* __restrict__ row = lam + (size_t)w * K;
    double top = -1.0e300;
    for (int k = lane; k < K; k += 64) {
        const double e = digamma_d((double)row[k]) - psi_total[k];
        top = e > top ? e : top;
    }
    for (int o = 32; o > 0; o >>= 1) {
        const double other = __shfl_xor(top, o);
        top = other > top ? other : top;
    }
    for (int k = lane; k < K; k += 64)
        b[(size_t)w * K + k] = (float)exp(digamma_d((double)row[k]) - psi_total[k] - top);
    if (lane == 0) shift[w] = (float)top;
}

// One wave per document, lanes across topics (lane l owns topics 256 c + 4 l .. + 3 of chunk c: a row of b is read
// with 16-byte loads, 1 KB per instruction), K a multiple of 4 and at most 256 CH.  The document's gamma, a and the
// sums over its nonzeros stay in registers over all iterations; two nonzeros are in flight at a time (up to 256
// topics: four, and the next four behind them).
template <int CH>
__global__ __launch_bounds__(256) void vb_estep_kernel(const int32_t* __restrict__ colptr, const int32_t* __restrict__ rowidx,
                                                       const float* __restrict__ val, int32_t D, int K,
                                                       const float* __restrict__ b, const float* __restrict__ shift,
                                                       float alpha, int iters, float* __restrict__ gamma,
                                                       float* __restrict__ log_mu_out)
{
    const int lane = threadIdx.x & 63;
    const int32_t d = (int32_t)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    if (d >= D) return;                                            // the whole wave
    const int64_t lo = colptr[d], hi = colptr[d + 1];
    float* __restrict__ grow = gamma + (size_t)d * K;
    // gamma and the sums over the document's nonzeros are kept in double from one iteration to the next: the
    // iteration converges slowly along some directions, and binary32 rounding fed back ten times shows at 1e-5
    double g[CH][4], acc[CH][4];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int k = 256 * c + 4 * lane;
        const float4 v = k < K ? *reinterpret_cast<const float4*>(grow + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        g[c][0] = v.x; g[c][1] = v.y; g[c][2] = v.z; g[c][3] = v.w;
    }
    for (int it = 0; it < iters; ++it) {
        double s = 0.0;
#pragma unroll
        for (int c = 0; c < CH; ++c) s += (g[c][0] + g[c][1]) + (g[c][2] + g[c][3]);
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        const double ps = digamma_d(s);
        float4 a[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const bool in = 256 * c + 4 * lane < K;
            a[c].x = in ? (float)exp(digamma_d(g[c][0]) - ps) : 0.f;
            a[c].y = in ? (float)exp(digamma_d(g[c][1]) - ps) : 0.f;
            a[c].z = in ? (float)exp(digamma_d(g[c][2]) - ps) : 0.f;
            a[c].w = in ? (float)exp(digamma_d(g[c][3]) - ps) : 0.f;
            acc[c][0] = 0.0; acc[c][1] = 0.0; acc[c][2] = 0.0; acc[c][3] = 0.0;
        }
        if constexpr (CH == 1) {
            // Up to 256 topics: kR nonzeros per round, and the rows of the next round are loaded while this round is
            // worked off (their word ids were loaded a round earlier still).  Every round issues the same loads,
            // past the document's end with the index of its last nonzero and a count of zero, so that the number of
            // loads in flight behind the ones a round waits for is fixed and the wait lets them fly.
            constexpr int kR = 2;                                  // nonzeros per round (even; four cost 171 registers and half the waves)
            const int k = 4 * lane;
            const bool in = k < K;
            const int64_t last = hi - 1;
            auto ids = [&](int64_t i0, int32_t (&wv)[kR], float (&cv)[kR]) {
#pragma unroll
                for (int j = 0; j < kR; ++j) {
                    const int64_t i = i0 + j;
                    const int64_t ic = i < hi ? i : last;
                    wv[j] = rowidx[ic];
                    cv[j] = i < hi ? val[ic] : 0.f;
                }
            };
            auto rows = [&](const int32_t (&wv)[kR], float4 (&bv)[kR]) {
#pragma unroll
                for (int j = 0; j < kR; ++j)
                    bv[j] = in ? *reinterpret_cast<const float4*>(b + (size_t)wv[j] * K + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            };
            if (lo < hi) {
                int32_t w[kR], nw[kR];
                float cnt[kR], ncnt[kR];
                float4 bv[kR], nbv[kR];
                ids(lo, w, cnt);
                ids(lo + kR, nw, ncnt);
                rows(w, bv);
                for (int64_t i = lo; i < hi; i += kR) {
                    int32_t nnw[kR];
                    float nncnt[kR];
                    rows(nw, nbv);
                    ids(i + 2 * kR, nnw, nncnt);
                    __builtin_amdgcn_sched_barrier(0);             // the next round's loads first, then this round's work
                    float m[kR];
                    double r[kR];
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
                        float sj = 0.f;
                        sj = __builtin_fmaf(a[0].x, bv[j].x, sj); sj = __builtin_fmaf(a[0].y, bv[j].y, sj);
                        sj = __builtin_fmaf(a[0].z, bv[j].z, sj); sj = __builtin_fmaf(a[0].w, bv[j].w, sj);
                        m[j] = wave_sum(sj);
                        r[j] = cnt[j] > 0.f ? (double)cnt[j] / (double)m[j] : 0.0;
                    }
#pragma unroll
                    for (int j = 0; j < kR; j += 2) {               // pairs of nonzeros, as in the loop for more topics
                        acc[0][0] = __builtin_fma(r[j], (double)bv[j].x, __builtin_fma(r[j + 1], (double)bv[j + 1].x, acc[0][0]));
                        acc[0][1] = __builtin_fma(r[j], (double)bv[j].y, __builtin_fma(r[j + 1], (double)bv[j + 1].y, acc[0][1]));
                        acc[0][2] = __builtin_fma(r[j], (double)bv[j].z, __builtin_fma(r[j + 1], (double)bv[j + 1].z, acc[0][2]));
                        acc[0][3] = __builtin_fma(r[j], (double)bv[j].w, __builtin_fma(r[j + 1], (double)bv[j + 1].w, acc[0][3]));
                    }
                    if (log_mu_out != nullptr && it == iters - 1 && lane == 0) {
#pragma unroll
                        for (int j = 0; j < kR; ++j)
                            if (i + j < hi) log_mu_out[i + j] = logf(m[j]) + (shift ? shift[w[j]] : 0.f);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < kR; ++j) { bv[j] = nbv[j]; w[j] = nw[j]; cnt[j] = ncnt[j]; nw[j] = nnw[j]; ncnt[j] = nncnt[j]; }
                }
            }
        } else
        for (int64_t i = lo; i < hi; i += 2) {
            const bool two = i + 1 < hi;
            const int32_t w0 = rowidx[i], w1 = two ? rowidx[i + 1] : w0;
            const float c0 = val[i], c1 = two ? val[i + 1] : 0.f;
            const float* __restrict__ p0 = b + (size_t)w0 * K;
            const float* __restrict__ p1 = b + (size_t)w1 * K;
            float4 b0[CH], b1[CH];
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int k = 256 * c + 4 * lane;
                b0[c] = k < K ? *reinterpret_cast<const float4*>(p0 + k) : make_float4(0.f, 0.f, 0.f, 0.f);
                b1[c] = k < K ? *reinterpret_cast<const float4*>(p1 + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                s0 = __builtin_fmaf(a[c].x, b0[c].x, s0); s0 = __builtin_fmaf(a[c].y, b0[c].y, s0);
                s0 = __builtin_fmaf(a[c].z, b0[c].z, s0); s0 = __builtin_fmaf(a[c].w, b0[c].w, s0);
                s1 = __builtin_fmaf(a[c].x, b1[c].x, s1); s1 = __builtin_fmaf(a[c].y, b1[c].y, s1);
                s1 = __builtin_fmaf(a[c].z, b1[c].z, s1); s1 = __builtin_fmaf(a[c].w, b1[c].w, s1);
            }
            const float m0 = wave_sum(s0), m1 = wave_sum(s1);
            const double r0 = (double)c0 / (double)m0, r1 = two ? (double)c1 / (double)m1 : 0.0;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                acc[c][0] = __builtin_fma(r0, (double)b0[c].x, __builtin_fma(r1, (double)b1[c].x, acc[c][0]));
                acc[c][1] = __builtin_fma(r0, (double)b0[c].y, __builtin_fma(r1, (double)b1[c].y, acc[c][1]));
                acc[c][2] = __builtin_fma(r0, (double)b0[c].z, __builtin_fma(r1, (double)b1[c].z, acc[c][2]));
                acc[c][3] = __builtin_fma(r0, (double)b0[c].w, __builtin_fma(r1, (double)b1[c].w, acc[c][3]));
            }
            if (log_mu_out != nullptr && it == iters - 1 && lane == 0) {
                log_mu_out[i] = logf(m0) + (shift ? shift[w0] : 0.f);
                if (two) log_mu_out[i + 1] = logf(m1) + (shift ? shift[w1] : 0.f);
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            if (256 * c + 4 * lane < K) {                          // topics past K stay zero: they are part of the row sum
                g[c][0] = __builtin_fma((double)a[c].x, acc[c][0], (double)alpha);
                g[c][1] = __builtin_fma((double)a[c].y, acc[c][1], (double)alpha);
                g[c][2] = __builtin_fma((double)a[c].z, acc[c][2], (double)alpha);
                g[c][3] = __builtin_fma((double)a[c].w, acc[c][3], (double)alpha);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int k = 256 * c + 4 * lane;
        if (k < K) *reinterpret_cast<float4*>(grow + k) = make_float4((float)g[c][0], (float)g[c][1], (float)g[c][2], (float)g[c][3]);
    }
}

// Any K (not a multiple of 4): the same steps with the document's vectors in LDS (gamma and the sums in double, a in
// binary32: 20 K bytes per wave).
__global__ __launch_bounds__(256) void vb_estep_any_kernel(const int32_t* __restrict__ colptr, const int32_t* __restrict__ rowidx,
                                                           const float* __restrict__ val, int32_t D, int K,
                                                           const float* __restrict__ b, const float* __restrict__ shift,
                                                           float alpha, int iters, float* __restrict__ gamma,
                                                           float* __restrict__ log_mu_out)
{
    extern __shared__ double vb_lds[];                             // [waves][g: K doubles][acc: K doubles][a: K floats, padded]
    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const int32_t d = (int32_t)(blockIdx.x * (blockDim.x >> 6) + wv);
    if (d >= D) return;
    const int per_wave = 2 * K + (K + 1) / 2;                      // doubles
    double* g = vb_lds + (size_t)wv * per_wave;
    double* acc = g + K;
    float* a = reinterpret_cast<float*>(acc + K);
    const int64_t lo = colptr[d], hi = colptr[d + 1];
    float* __restrict__ grow = gamma + (size_t)d * K;
    for (int k = lane; k < K; k += 64) g[k] = (double)grow[k];
    for (int it = 0; it < iters; ++it) {
        double s = 0.0;
        for (int k = lane; k < K; k += 64) s += g[k];
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        const double ps = digamma_d(s);
        for (int k = lane; k < K; k += 64) { a[k] = (float)exp(digamma_d(g[k]) - ps); acc[k] = 0.0; }
        for (int64_t i = lo; i < hi; ++i) {
            const float* __restrict__ p = b + (size_t)rowidx[i] * K;
            float s0 = 0.f;
            for (int k = lane; k < K; k += 64) s0 = __builtin_fmaf(a[k], p[k], s0);
            const float m0 = wave_sum(s0);
            const double r0 = (double)val[i] / (double)m0;
            for (int k = lane; k < K; k += 64) acc[k] = __builtin_fma(r0, (double)p[k], acc[k]);
            if (log_mu_out != nullptr && it == iters - 1 && lane == 0)
                log_mu_out[i] = logf(m0) + (shift ? shift[rowidx[i]] : 0.f);
        }
        for (int k = lane; k < K; k += 64) g[k] = __builtin_fma((double)a[k], acc[k], (double)alpha);
    }
    for (int k = lane; k < K; k += 64) grow[k] = (float)g[k];
}

}  // namespace same
