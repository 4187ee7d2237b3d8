// Device-side random stream and binomial sampler of the SAME LDA draw (gfx950).
//
// Every floating-point step here is a single IEEE binary32 operation with one rounding
// (the file is compiled with -ffp-contract=off); the integer results therefore depend only
// on the inputs and the seed, never on the launch shape or on thread timing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace same {

// Philox4x32-10 (Salmon et al., SC'11): ten multiply-and-mix rounds over a 128-bit counter
// with a 64-bit key advanced by the two Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Top 23 bits j of a random word -> (2j+1) * 2^-24: an exactly representable uniform in (0,1).
__device__ __forceinline__ float uniform_from_word(uint32_t x)
{
    return (float)(2u * (x >> 9) + 1u) * 5.9604644775390625e-8f;
}

// Keys of one draw task: the seed is the Philox key; the counter is
// (task id low, task id high byte [| piece block << 8], topic field, pass word).
struct StreamKey {
    uint32_t seed_lo, seed_hi;
    uint32_t tau_lo, tau_hi;   // tau_hi < 256
    uint32_t pass;
};

// Block holding the first-piece uniforms of topics 4*quad .. 4*quad+3.
__device__ __forceinline__ void primary_block(const StreamKey& s, uint32_t quad, uint32_t (&out)[4])
{
    philox4x32_10(s.tau_lo, s.tau_hi, quad, s.pass, s.seed_lo, s.seed_hi, out);
}

// Block holding the uniforms of pieces 4*pb+1 .. 4*pb+4 of topic k.
__device__ __forceinline__ void piece_block(const StreamKey& s, uint32_t k, uint32_t pb, uint32_t (&out)[4])
{
    philox4x32_10(s.tau_lo, s.tau_hi | (pb << 8), 0x80000000u | k, s.pass, s.seed_lo, s.seed_hi, out);
}

// s^n by binary square-and-multiply, least significant bit first.
__device__ __forceinline__ float ipow(float s, uint32_t n)
{
    float result = 1.0f, base = s;
    uint32_t e = n;
    while (e > 0) {
        if (e & 1u) result = result * base;
        e >>= 1;
        if (e > 0) base = base * base;
    }
    return result;
}

// One binomial piece by inversion: walk the pmf upward from 0 until the cdf reaches u,
// the piece is exhausted, or the pmf has fallen below the resolution of the running cdf.
__device__ __forceinline__ uint32_t binom_walk(uint32_t n, float pm0, float r, float u)
{
    uint32_t x = 0;
    float pm = pm0, cdf = pm0;
    while (u > cdf && x < n) {
        x += 1;
        const float inv_x = 1.0f / (float)x;
        pm = pm * r;
        pm = pm * (float)(n - x + 1u);
        pm = pm * inv_x;
        const float next = cdf + pm;
        if (next == cdf) break;
        cdf = next;
    }
    return x;
}

// n ~ Binomial(R, q) for topic k.  The rarer outcome (probability qq <= 1/2) is sampled and the
// result complemented when q > 1/2; R is cut into pieces of at most floor(32/qq) trials so the
// starting pmf (1-qq)^piece never underflows.  u0 is the uniform of the first piece; later
// pieces fetch theirs from the task's piece stream.
__device__ __forceinline__ uint32_t binom(uint32_t R, float q, float u0, const StreamKey& s, uint32_t k)
{
    if (R == 0 || !(q > 0.0f)) return 0;
    if (q >= 1.0f) return R;
    const bool flip = q > 0.5f;
    const float qq = flip ? 1.0f - q : q;
    const float sc = 1.0f - qq;
    const float r = qq / sc;
    const float Lf = 32.0f / qq;
    const uint32_t L = (Lf >= (float)R) ? R : (uint32_t)Lf;
    const float pmL = ipow(sc, L);
    uint32_t rem = R, piece = 0, total = 0;
    uint32_t xb[4] = {0u, 0u, 0u, 0u};
    while (rem > 0) {
        const uint32_t n = rem < L ? rem : L;
        const float pm0 = (n == L) ? pmL : ipow(sc, n);
        float u = u0;
        if (piece > 0) {
            const uint32_t j = piece - 1u;
            if ((j & 3u) == 0u) piece_block(s, k, j >> 2, xb);
            const uint32_t word = (j & 3u) == 0u ? xb[0] : (j & 3u) == 1u ? xb[1] : (j & 3u) == 2u ? xb[2] : xb[3];
            u = uniform_from_word(word);
        }
        total += binom_walk(n, pm0, r, u);
        rem -= n;
        piece += 1;
    }
    return flip ? R - total : total;
}

}  // namespace same
