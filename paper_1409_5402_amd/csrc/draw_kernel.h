// Draw-and-scatter kernel of the SAME LDA sweep (Algorithm 3, the loop over document-word
// pairs; Section 4, multinomial form of the factored draw) for gfx950.
//
// Mapping: one wave per workgroup, one lane per draw task (a group of tokens of one nonzero).
// A lane walks the K topics of its task twice.
//   pass 1  accumulates the running sums P_k = w_0 + ... + w_k left to right
//           (w_k = theta[d][k] * phi[w][k]), checkpoints P at every 16th topic in LDS and finds
//           the heaviest topic;
//   pass 2  revisits the 16-topic blocks from the last to the first, rebuilds P_k inside the
//           block from its checkpoint, generates the topics' uniforms (one Philox block per 4
//           topics) and tests every topic: a topic whose uniform already proves that its
//           conditional binomial is 0 for ANY remaining count up to the current bound is
//           dropped; the others are queued in LDS in chain order (descending k).
// The heaviest topic of the task is never drawn (it keeps the remainder); for a topic below it the
// undecided weight is P_k plus the heaviest weight.  The queue is drained by a per-lane state
// machine that runs the chain n_k ~ Bin(R, w_k / M_k), R -= n_k with the exact division and the
// exact inversion sampler: every trip of the drain loop lets each lane either fetch its next
// queued topic (re-testing it against the now exact remaining count) or advance its pmf walk by a
// few steps, so lanes with long walks do not hold up lanes with many short ones.  A binomial that
// the sampler cuts into several pieces (independent, one uniform each) is handed to the whole wave,
// one piece per lane.
//
// The drop test is conservative and never changes a result.  For a single-piece binomial with
// R <= Rb trials and success probability q <= 1/2 the sampler returns 0 iff u <= (1-q)^R
// evaluated in binary32 by square-and-multiply; that value is >= 1 - Rb*(q + 2^-22)
// (Bernoulli's inequality plus at most 2R roundings of relative size 2^-24 and the rounding of
// 1-q).  The test checks q <= 0.499 (so the sampler does not take its complement branch) and
// u + Rb*(q*(1+1e-4) + 1e-6) <= 1 - 1e-4, evaluated without a division (see ZeroTest), which
// implies the former (and Rb*q < 1 implies a single piece).  A topic of zero weight passes it.
#pragma once
#include "rng_binom.h"

namespace same {

#ifndef SAME_QCAP
#define SAME_QCAP 12
#endif
#ifndef SAME_WALK_STEPS
#define SAME_WALK_STEPS 4
#endif
constexpr int kWave = 64;               // lanes per workgroup (one wave)
constexpr int kBlk = 16;                // topics per checkpoint block
constexpr int kQCap = SAME_QCAP;        // queued topics per lane between drains (drain when > kQCap - 4)
constexpr int kWalkSteps = SAME_WALK_STEPS;   // pmf steps per trip of the drain loop

struct DrawArgs {
    int64_t         n;          // tasks in this launch
    const int32_t*  t_doc;      // [n_tasks] document of the task
    const int32_t*  t_word;     // [n_tasks] word of the task
    const uint32_t* t_g;        // [n_tasks] tokens in the task's group
    const int32_t*  order;      // [n_tasks] task id handled at each launch position
    uint32_t*       cost;       // [n_tasks] out: drain trips this task was busy for (null: not recorded)
    const int64_t*  ids;        // debug launches: task ids to draw instead (else null)
    const float*    theta;      // [D][K]   (unused when weights are uniform)
    const float*    phi;        // [V][K]
    uint32_t*       ndk;        // [D][K]   (debug launches: [n][K] output rows)
    uint32_t*       nwk;        // [V][K] or null
    int32_t         K;
    uint32_t        m;
    uint32_t        seed_lo, seed_hi, pass;
#ifdef SAME_STATS
    unsigned long long* stats;  // profiling builds only: event counters
#endif
};

#ifdef SAME_STATS
#define SAME_COUNT(a, i, v) do { if ((a).stats) atomicAdd((a).stats + (i), (unsigned long long)(v)); } while (0)
#else
#define SAME_COUNT(a, i, v) do { } while (0)
#endif

template <bool UNIFORM>
__device__ __forceinline__ float weight(const float* __restrict__ th, const float* __restrict__ ph, int k)
{
    if (UNIFORM) return 1.0f;
    return th[k] * ph[k];
}

// Sixteen phi values of one block, loaded ahead of their use (K % 16 == 0 only).
struct PhiBlock { float4 v[kBlk / 4]; };

template <bool UNIFORM, bool VEC>
__device__ __forceinline__ PhiBlock load_phi(const float* __restrict__ ph, int b)
{
    PhiBlock r;
    if (!UNIFORM && VEC) {
#pragma unroll
        for (int v = 0; v < kBlk / 4; ++v) r.v[v] = *reinterpret_cast<const float4*>(ph + b * kBlk + 4 * v);
    }
    return r;
}

// The 16 weights of block b (zero beyond K).
template <bool UNIFORM, bool VEC>
__device__ __forceinline__ void block_weights(const float* __restrict__ th, const float* __restrict__ ph,
                                              const PhiBlock& pre, int b, int K, float (&wv)[kBlk])
{
    const int k0 = b * kBlk;
    if (UNIFORM) {
#pragma unroll
        for (int j = 0; j < kBlk; ++j) wv[j] = (k0 + j < K) ? 1.0f : 0.0f;
        return;
    }
    if (VEC) {
#pragma unroll
        for (int v = 0; v < kBlk / 4; ++v) {
            const float4 t = *reinterpret_cast<const float4*>(th + k0 + 4 * v);
            const float4 c = pre.v[v];
            wv[4 * v + 0] = t.x * c.x;
            wv[4 * v + 1] = t.y * c.y;
            wv[4 * v + 2] = t.z * c.z;
            wv[4 * v + 3] = t.w * c.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kBlk; ++j) wv[j] = (k0 + j < K) ? th[k0 + j] * ph[k0 + j] : 0.0f;
    }
}

// The drop test without a division: for q = w/M it checks q <= 0.499 and
// u + Rf*(q*(1+1e-4) + 1e-6) <= 1 - 1e-4, both multiplied through by M > 0
// (the margins cover the few roundings of this evaluation).  ZeroTest holds the two terms that
// depend only on the bound Rf; x is the raw random word of the topic (u = (2*(x>>9)+1)/2^24).
struct ZeroTest {
    float A, Bp;
    __device__ __forceinline__ explicit ZeroTest(float Rf)
        : A(Rf * 1.0001f), Bp((0.9999f - Rf * 1.0e-6f) - 5.9604644775390625e-8f) {}
    // true when Bin(R', w/M) is certainly 0 for every R' <= Rf (see the header comment)
    __device__ __forceinline__ bool surely_zero(float wk, float Mk, uint32_t x) const
    {
        const float d = __builtin_fmaf((float)(x >> 9), -1.1920928955078125e-7f, Bp);   // (1-1e-4) - Rf*1e-6 - u
        return (wk <= 0.499f * Mk) && (A * wk <= d * Mk);
    }
};

// 1/x for an integer-valued x in [1, 2^24): the hardware reciprocal followed by one Newton step
// equals the correctly rounded quotient for every such x (checked exhaustively by the library's
// self-test), at a third of the cost of a full division.
__device__ __forceinline__ float inv_int(float x)
{
    const float y = __builtin_amdgcn_rcpf(x);
    const float e = __builtin_fmaf(-x, y, 1.0f);
    return __builtin_fmaf(y, e, y);
}

template <bool UNIFORM, bool VEC, bool DEBUG>
__global__ __launch_bounds__(kWave) void draw_kernel(DrawArgs a)
{
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int K = a.K;
    const int nblk = (K + kBlk - 1) / kBlk;
    const int qw = K <= 512 ? 3 : 4;                               // words per queue entry
    float*    chk = reinterpret_cast<float*>(lds);                 // [nblk][64]
    uint32_t* que = lds + (size_t)nblk * kWave;                    // [kQCap][qw][64]

    // lanes past the end take the last task with zero copies: all loads stay valid, nothing is emitted
    const int64_t slot = (int64_t)blockIdx.x * kWave + lane;
    const bool live = slot < a.n;
    const int64_t row = live ? slot : a.n - 1;
    const int64_t tau = DEBUG ? a.ids[row] : (int64_t)a.order[row];
    const int32_t d = a.t_doc[tau];
    const int32_t w = a.t_word[tau];
    const uint32_t N = live ? a.m * a.t_g[tau] : 0u;
    const float* __restrict__ th = UNIFORM ? nullptr : a.theta + (size_t)d * K;
    const float* __restrict__ ph = UNIFORM ? nullptr : a.phi + (size_t)w * K;
    uint32_t* __restrict__ out_d = DEBUG ? a.ndk + (size_t)row * K : a.ndk + (size_t)d * K;
    uint32_t* __restrict__ out_w = (DEBUG || a.nwk == nullptr) ? nullptr : a.nwk + (size_t)w * K;

    StreamKey key;
    key.seed_lo = a.seed_lo; key.seed_hi = a.seed_hi;
    key.tau_lo = (uint32_t)tau; key.tau_hi = (uint32_t)((uint64_t)tau >> 32) & 0xFFu;
    key.pass = a.pass;

    // ---- pass 1: running sum, checkpoint before every block; heaviest topic (highest index among ties)
    float wmax = -1.0f;
    int kstar = 0;
    {
        float P = 0.0f;
        PhiBlock cur = load_phi<UNIFORM, VEC>(ph, 0);
        for (int b = 0; b < nblk; ++b) {
            PhiBlock nxt = cur;
            if (b + 1 < nblk) nxt = load_phi<UNIFORM, VEC>(ph, b + 1);
            chk[b * kWave + lane] = P;
            float wv[kBlk];
            block_weights<UNIFORM, VEC>(th, ph, cur, b, K, wv);
#pragma unroll
            for (int j = 0; j < kBlk; ++j) {
                P = P + wv[j];
                const int k = b * kBlk + j;
                if ((VEC || k < K) && wv[j] >= wmax) { wmax = wv[j]; kstar = k; }
            }
            cur = nxt;
        }
    }

    uint32_t R = N;
    int cnt = 0;
    uint32_t busy = 0;      // drain trips in which this lane still had work: its cost for the next ordering

    auto emit = [&](int k, uint32_t n) {
        atomicAdd(out_d + k, n);
        if (out_w) atomicAdd(out_w + k, n);
    };

    // ---- the conditional-binomial chain over the queued topics (descending k), as a state machine
    auto drain = [&]() {
        int e = 0;
        int st = 0;   // 0: fetch the next queued topic, 1: walking a single piece, 2: queue exhausted,
                      // 3: holds a binomial of several pieces for the whole wave to work on
        // state of the binomial in flight
        uint32_t bR = 0, L = 0, xw = 0;
        float sc = 0.f, r = 0.f, pm = 0.f, cdf = 0.f, u = 0.f;
        bool flip = false, stalled = false;
        int kk = 0;
        if (lane == 0) SAME_COUNT(a, 0, 1);                      // drains
        SAME_COUNT(a, 1, cnt);                                     // queued topics
        for (;;) {
            if (lane == 0) SAME_COUNT(a, 2, 1);                  // drain loop trips
            busy += (st != 2) ? 1u : 0u;
            if (st == 0) {
                bool found = false;
                float wq = 0.f, Mq = 1.f;
                while (e < cnt && R > 0) {
                    wq = __uint_as_float(que[(e * qw + 0) * kWave + lane]);
                    Mq = __uint_as_float(que[(e * qw + 1) * kWave + lane]);
                    const uint32_t xk = que[(e * qw + 2) * kWave + lane];
                    kk = qw == 3 ? (int)(xk & 511u) : (int)que[(e * qw + 3) * kWave + lane];
                    u = uniform_from_word(xk);
                    ++e;
                    if (!ZeroTest((float)R).surely_zero(wq, Mq, xk)) { found = true; break; }
                }
                if (!found) {
                    st = 2;
                } else {
                    const float q = wq / Mq;
                    if (q >= 1.0f) {
                        emit(kk, R);
                        R = 0;
                    } else if (q > 0.0f) {
                        flip = q > 0.5f;
                        const float qq = flip ? 1.0f - q : q;
                        sc = 1.0f - qq;
                        r = qq / sc;
                        bR = R;
                        SAME_COUNT(a, 3, 1);                       // binomials set up
                        if (((float)R * qq) <= 32.0f) {            // one piece of R trials
                            L = R;
                            const float pm0 = ipow(sc, R);
                            xw = 0; pm = pm0; cdf = pm0; stalled = false;
                            st = 1;
                        } else {                                   // pieces of L trials: shared by the wave
                            L = (uint32_t)(32.0f / qq);
                            st = 3;
                            SAME_COUNT(a, 6, 1);                   // binomials in several pieces
                        }
                    }
                }
            }
            if (!__any(st != 2)) break;

            // Binomials cut into pieces: the pieces are independent (own uniform each), so the 64
            // lanes take one piece each; the owner lane receives the total.
            for (uint64_t pend = __ballot(st == 3); pend != 0; pend &= pend - 1) {
                const int src = __ffsll((unsigned long long)pend) - 1;
                const uint32_t cR = __shfl(bR, src), cL = __shfl(L, src);
                const float csc = __shfl(sc, src), cr = __shfl(r, src), cu0 = __shfl(u, src);
                const uint32_t ck = (uint32_t)__shfl(kk, src);
                StreamKey ckey = key;
                ckey.tau_lo = __shfl(key.tau_lo, src);
                ckey.tau_hi = __shfl(key.tau_hi, src);
                const uint32_t npieces = (cR + cL - 1u) / cL;
                const float cpmL = ipow(csc, cL);
                uint32_t part = 0;
                for (uint32_t base = 0; base < npieces; base += kWave) {
                    const uint32_t jp = base + (uint32_t)lane;
                    if (jp < npieces) {
                        const uint32_t nj = (jp == npieces - 1u) ? cR - jp * cL : cL;
                        float pmj = (nj == cL) ? cpmL : ipow(csc, nj);
                        float uj = cu0;
                        if (jp > 0) {
                            uint32_t xb[4];
                            piece_block(ckey, ck, (jp - 1u) >> 2, xb);
                            const uint32_t sel = (jp - 1u) & 3u;
                            uj = uniform_from_word(sel == 0u ? xb[0] : sel == 1u ? xb[1] : sel == 2u ? xb[2] : xb[3]);
                        }
                        uint32_t xj = 0;
                        float cdfj = pmj;
                        while (uj > cdfj && xj < nj) {
                            xj += 1;
                            pmj = pmj * cr;
                            pmj = pmj * (float)(nj - xj + 1u);
                            pmj = pmj * inv_int((float)xj);
                            const float next = cdfj + pmj;
                            if (next == cdfj) break;
                            cdfj = next;
                        }
                        part += xj;
                    }
                }
#pragma unroll
                for (int off = kWave / 2; off > 0; off >>= 1) part += __shfl_xor(part, off);
                if (lane == src) {
                    const uint32_t nk = flip ? bR - part : part;
                    if (nk > 0) { emit(kk, nk); SAME_COUNT(a, 5, 1); }
                    R -= nk;
                    st = 0;
                }
            }

            if (__any(st == 1)) {
                const bool walking = st == 1;
#pragma unroll
                for (int i = 0; i < kWalkSteps; ++i) {
                    const bool go = walking && !stalled && u > cdf && xw < L;
                    const uint32_t xn = xw + 1u;
                    float pmn = pm * r;
                    pmn = pmn * (float)(L - xn + 1u);
                    pmn = pmn * inv_int((float)xn);
                    const float next = cdf + pmn;
                    const bool still = next == cdf;
                    if (go) SAME_COUNT(a, 4, 1);                   // walk steps
                    xw = go ? xn : xw;
                    pm = go ? pmn : pm;
                    cdf = (go && !still) ? next : cdf;
                    stalled = stalled || (go && still);
                }
                if (walking && (stalled || !(u > cdf && xw < L))) {   // the piece is finished
                    const uint32_t nk = flip ? bR - xw : xw;
                    if (nk > 0) { emit(kk, nk); SAME_COUNT(a, 5, 1); }   // nonzero counts
                    R -= nk;
                    st = 0;
                }
            }
        }
        cnt = 0;
    };

    // ---- pass 2: blocks from last to first
    {
        PhiBlock cur = load_phi<UNIFORM, VEC>(ph, nblk - 1);
        for (int b = nblk - 1; b >= 0; --b) {
            if (!__any(R > 0)) break;
            PhiBlock nxt = cur;
            if (b > 0) nxt = load_phi<UNIFORM, VEC>(ph, b - 1);
            float wv[kBlk], Pv[kBlk];
            block_weights<UNIFORM, VEC>(th, ph, cur, b, K, wv);
            cur = nxt;
            {
                float P = chk[b * kWave + lane];
#pragma unroll
                for (int j = 0; j < kBlk; ++j) { P = P + wv[j]; Pv[j] = P; }
            }
            ZeroTest zt((float)R);   // R bounds the remaining count until the next drain
#pragma unroll
            for (int g = kBlk / 4 - 1; g >= 0; --g) {
                uint32_t x[4];
                primary_block(key, (uint32_t)(b * (kBlk / 4) + g), x);
#pragma unroll
                for (int j = 3; j >= 0; --j) {
                    const int k = b * kBlk + g * 4 + j;
                    const float wk = wv[g * 4 + j];
                    const float Mk = Pv[g * 4 + j] + (k < kstar ? wmax : 0.0f);   // weight not yet decided at k
                    const bool cand = (k != kstar) && !zt.surely_zero(wk, Mk, x[j]);   // a zero weight passes the test
                    if (cand) {
                        que[(cnt * qw + 0) * kWave + lane] = __float_as_uint(wk);
                        que[(cnt * qw + 1) * kWave + lane] = __float_as_uint(Mk);
                        if (qw == 3) {
                            que[(cnt * qw + 2) * kWave + lane] = (x[j] & ~511u) | (uint32_t)k;   // the uniform uses the top 23 bits
                        } else {
                            que[(cnt * qw + 2) * kWave + lane] = x[j];
                            que[(cnt * qw + 3) * kWave + lane] = (uint32_t)k;
                        }
                        cnt += 1;
                    }
                }
                if (__any(cnt > kQCap - 4)) { drain(); zt = ZeroTest((float)R); }
            }
        }
    }
    drain();
    if (R > 0) emit(kstar, R);
    if (!DEBUG && live && a.cost) a.cost[tau] = busy;
}

inline size_t draw_lds_bytes(int K)
{
    const int nblk = (K + kBlk - 1) / kBlk;
    const int qw = K <= 512 ? 3 : 4;
    return 4u * (size_t)kWave * (size_t)(nblk + qw * kQCap);
}

}  // namespace same
