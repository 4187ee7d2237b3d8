// Device-side random stream and elementary functions of the SAME LDA draw (gfx950).
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

// The same block with the first two rounds split by what their inputs depend on.  Of the four
// products of those rounds, two depend only on the task (its id, the pass, the seed): PrimaryPre holds
// them, computed once per task.  The other two depend on the quad and, through one exclusive-or, on
// the high byte of the task id: where that byte is the same for the whole wave (it is zero for every
// launch whose task ids fit 32 bits) they are scalar work.  Eight general rounds follow.
struct PrimaryPre { uint32_t c2a, c3a, hi1, lo1; };

__device__ __forceinline__ PrimaryPre primary_pre(const StreamKey& s)
{
    PrimaryPre r;
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)s.tau_lo;     // round 1, counter word 0
    r.c3a = (uint32_t)p0;
    r.c2a = (uint32_t)(p0 >> 32) ^ s.pass ^ s.seed_hi;                  // counter word 2 after round 1
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)r.c2a;        // round 2, counter word 2
    r.hi1 = (uint32_t)(p1 >> 32);
    r.lo1 = (uint32_t)p1;
    return r;
}

__device__ __forceinline__ void primary_block(const StreamKey& s, const PrimaryPre& pre, uint32_t quad,
                                              uint32_t (&out)[4])
{
    uint32_t k0 = s.seed_lo, k1 = s.seed_hi;
    // round 1
    const uint64_t q1 = (uint64_t)0xCD9E8D57u * (uint64_t)quad;
    uint32_t c0 = (uint32_t)(q1 >> 32) ^ s.tau_hi ^ k0;
    uint32_t c1 = (uint32_t)q1;
    uint32_t c3 = pre.c3a;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    // round 2
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    c0 = pre.hi1 ^ c1 ^ k0;
    uint32_t c2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = pre.lo1;
    c3 = (uint32_t)p0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
#pragma unroll
    for (int round = 2; round < 10; ++round) {
        const uint64_t a0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t a1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(a1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(a0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)a1;
        c3 = (uint32_t)a0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Block holding the uniforms of pieces 4*pb+1 .. 4*pb+4 of topic k.
__device__ __forceinline__ void piece_block(const StreamKey& s, uint32_t k, uint32_t pb, uint32_t (&out)[4])
{
    philox4x32_10(s.tau_lo, s.tau_hi | (pb << 8), 0x80000000u | k, s.pass, s.seed_lo, s.seed_hi, out);
}

// 1/x for an integer-valued x in [1, 2^24): the hardware reciprocal followed by one Newton step
// equals the correctly rounded quotient for every such x (checked exhaustively by the library's
// self-test), at a third of the cost of a full division.
__device__ __forceinline__ float inv_int(float x)
{
    const float y = __builtin_amdgcn_rcpf(x);
    const float e = __builtin_fmaf(-x, y, 1.0f);
    return __builtin_fmaf(y, e, y);
}

// log x, x a positive normal number: x = 2^e f, f in [sqrt(1/2), sqrt(2)); log f = 2 atanh((f-1)/(f+1))
// by the odd series through the eleventh power.
__device__ __forceinline__ float flog(float x)
{
    const uint32_t bits = __float_as_uint(x);
    int e = (int)(bits >> 23) - 127;
    float f = __uint_as_float((bits & 0x007FFFFFu) | 0x3F800000u);
    if (f > 1.41421354f) { f = f * 0.5f; e += 1; }
    const float s = (f - 1.0f) / (f + 1.0f);
    const float z = s * s;
    float p = 0.0909090936f;
    p = p * z; p = p + 0.111111112f;
    p = p * z; p = p + 0.142857149f;
    p = p * z; p = p + 0.2f;
    p = p * z; p = p + 0.333333343f;
    p = p * z; p = p + 1.0f;
    float lf = 2.0f * s;
    lf = lf * p;
    const float le = (float)e * 0.693147182f;
    return le + lf;
}

// -log(1 - x) for 0 < x <= 1/2 without rounding 1 - x (which would lose x below 2^-24):
// 2 atanh(t) with t = x / (2 - x), by the odd series through the seventeenth power.
__device__ __forceinline__ float log1m(float x)
{
    const float t = x / (2.0f - x);
    const float z = t * t;
    float p = 0.0588235296f;
    p = p * z; p = p + 0.0666666701f;
    p = p * z; p = p + 0.0769230798f;
    p = p * z; p = p + 0.0909090936f;
    p = p * z; p = p + 0.111111112f;
    p = p * z; p = p + 0.142857149f;
    p = p * z; p = p + 0.2f;
    p = p * z; p = p + 0.333333343f;
    p = p * z; p = p + 1.0f;
    const float two_t = 2.0f * t;
    return two_t * p;
}

// exp(-y) for 0 <= y <= 48 from + - * only: t = y*log2(e), n = trunc(t),
// f = t-n in [0,1), g = f - 1/2, 2^-(g+1/2) by the degree-7 Taylor polynomial of
// 2^-1/2 * exp(-g ln 2) in Horner form, every product and sum rounded once, scaled by 2^-n.
__device__ __forceinline__ float expneg(float y)
{
    const float t = y * 1.4426950408889634f;
    const int n = (int)t;
    const float f = t - (float)n;
    const float g = f - 0.5f;
    float p = -1.0785311504483996e-05f;
    p = p * g; p = p + 0.00010891940795373223f;
    p = p * g; p = p + -0.0009428249382684684f;
    p = p * g; p = p + 0.006801044314331813f;
    p = p * g; p = p + -0.039247331620610344f;
    p = p * g; p = p + 0.16986579209153746f;
    p = p * g; p = p + -0.4901290717342736f;
    p = p * g; p = p + 0.7071067811865476f;
    return ldexpf(p, -n);
}

}  // namespace same
