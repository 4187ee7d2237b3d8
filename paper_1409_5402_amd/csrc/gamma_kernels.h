// The sampled parameter step (Algorithm 2, third step; Section 3.1) for gfx950: theta and phi drawn
// from their Dirichlet conditionals given the counts of the m copies,
//   theta_d ~ Dirichlet(n_dk + m*alpha),   phi_k ~ Dirichlet over words (n_wk + m*beta),
// as independent Gamma(shape, 1) variables (theta: divided by m and left unnormalised, mean
// n_dk/m + alpha as in the collapsed update; phi: divided by their sum over words).
//
// Gamma variables after Marsaglia and Tsang (ACM TOMS 26, 2000): d = a - 1/3, c = 1/sqrt(9d),
// z standard normal, v = (1 + c z)^3, accept d*v when v > 0 and log u < z^2/2 + d(1 - v + log v),
// tried first as u < 1 - 0.0331 z^4; a shape below one takes Gamma(a+1) * u'^(1/a).  The normal is
// sqrt(-2 log u1) cos(2 pi u2).  Attempt j of element (row, k) uses the Philox block with counter
// (row, k, j, pass word): words 0 and 1 make the normal, word 2 the acceptance uniform, word 3 the
// uniform of the small-shape factor.  After 64 refused attempts the shape itself is the result.
// Logarithm, cosine and exponential are fixed sequences of + - * / in binary32, one rounding each,
// so that every acceptance is decided the same way by any implementation of these steps.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rng_binom.h"

namespace same {

// cos(2 pi u), u in (0,1): quarter turn, then the Taylor polynomial of sine or cosine on [0, pi/2).
__device__ __forceinline__ float cos2pi(float u)
{
    const float t = u * 4.0f;
    const int quarter = (int)t;
    const float x = (t - (float)quarter) * 1.57079637f;
    const float x2 = x * x;
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
    const int q = quarter & 3;
    return q == 0 ? cs : q == 1 ? -sn : q == 2 ? -cs : sn;
}

// Gamma(a, 1) for element (row, k) of the stream with the given pass word.
__device__ __forceinline__ float gamma_variable(float a, uint32_t seed_lo, uint32_t seed_hi, uint32_t row,
                                                uint32_t k, uint32_t pass)
{
    const bool small = a < 1.0f;
    const float a1 = small ? a + 1.0f : a;
    const float d = a1 - 0.333333343f;
    const float c = 1.0f / sqrtf(9.0f * d);
    float g = a1;
    uint32_t x[4] = {0u, 0u, 0u, 0u};
    for (uint32_t attempt = 0; attempt < 64u; ++attempt) {
        philox4x32_10(row, k, attempt, pass, seed_lo, seed_hi, x);
        const float l1 = flog(uniform_from_word(x[0]));
        const float r = sqrtf(-2.0f * l1);
        const float z = r * cos2pi(uniform_from_word(x[1]));
        const float u = uniform_from_word(x[2]);
        const float t = 1.0f + c * z;
        if (!(t > 0.0f)) continue;
        float v = t * t;
        v = v * t;
        const float z2 = z * z;
        const float z4 = z2 * z2;
        bool accept = u < 1.0f - 0.0331f * z4;
        if (!accept) {
            const float lhs = flog(u);
            const float inner = (1.0f - v) + flog(v);
            const float rhs = 0.5f * z2 + d * inner;
            accept = lhs < rhs;
        }
        if (accept) { g = d * v; break; }
    }
    if (small) {
        float y = -flog(uniform_from_word(x[3]));
        y = y / a;
        if (y > 200.0f) y = 200.0f;
        g = g * expneg(y);
    }
    return g < 1e-30f ? 1e-30f : g;
}

// theta[d][k] = Gamma(n_dk + m*alpha) / m
__global__ void gamma_theta_kernel(const uint32_t* __restrict__ ndk, float* __restrict__ theta, size_t n, int K,
                                   float mf, float prior, uint32_t seed_lo, uint32_t seed_hi, uint32_t pass)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t d = (uint32_t)(i / (size_t)K), k = (uint32_t)(i % (size_t)K);
        const float a = (float)ndk[i] + prior;
        theta[i] = gamma_variable(a, seed_lo, seed_hi, d, k, pass) / mf;
    }
}

// phi[w][k] = Gamma(n_wk + m*beta), and the sum of each topic over this block's rows (double, row order)
__global__ void gamma_phi_kernel(const uint32_t* __restrict__ nwk, float* __restrict__ phi, int V, int K,
                                 float prior, uint32_t seed_lo, uint32_t seed_hi, uint32_t pass,
                                 int rows_per_block, double* __restrict__ partial)
{
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(V, r0 + rows_per_block);
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
        double acc = 0.0;
        for (int r = r0; r < r1; ++r) {
            const size_t i = (size_t)r * K + k;
            const float g = gamma_variable((float)nwk[i] + prior, seed_lo, seed_hi, (uint32_t)r, (uint32_t)k, pass);
            phi[i] = g;
            acc += (double)g;
        }
        partial[(size_t)blockIdx.x * K + k] = acc;
    }
}

// total[k] = sum of the block sums in block order (double), rounded to binary32
__global__ void gamma_phi_totals_kernel(const double* __restrict__ partial, int blocks, int K, float* __restrict__ total)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    double acc = 0.0;
    for (int b = 0; b < blocks; ++b) acc += partial[(size_t)b * K + k];
    total[k] = (float)acc;
}

__global__ void gamma_phi_normalise_kernel(float* __restrict__ phi, size_t n, int K, const float* __restrict__ total)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        phi[i] = phi[i] / total[i % (size_t)K];
}

}  // namespace same
