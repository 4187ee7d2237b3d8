// Draw-and-scatter kernel of the SAME LDA sweep (Algorithm 3, the loop over document-word
// pairs; Section 4, multinomial form of the factored draw) for gfx950.
//
// Mapping: one wave per workgroup, one lane per draw task (a group of tokens of one nonzero).
// A lane walks the K topics of its task twice.
//   pass 1  accumulates the running sums P_k = w_0 + ... + w_k left to right
//           (w_k = theta[d][k] * phi[w][k]) and checkpoints P at every 16th topic in LDS;
//   pass 2  revisits the 16-topic blocks from the last to the first, rebuilds P_k inside the
//           block from its checkpoint, generates the topics' uniforms (one Philox block per 4
//           topics) and tests every topic: a topic whose uniform already proves that its
//           conditional binomial is 0 for ANY remaining count up to the current bound is
//           dropped; the others are queued in LDS in chain order (descending k).
// The heaviest topic of the task is never drawn (it keeps the remainder); for a topic below it the
// undecided weight is P_k plus the heaviest weight.  The queue is drained by a per-lane state
// machine that runs the chain n_k ~ Bin(R, w_k / M_k), R -= n_k with the exact division and the
// exact inversion sampler:
// every trip of the drain loop lets each lane either fetch its next queued topic (re-testing it
// against the now exact remaining count) or advance its pmf walk by up to four steps, so lanes
// with long walks do not hold up lanes with many short ones.
//
// The drop test is conservative and never changes a result.  For a single-piece binomial with
// R <= Rb trials and success probability q <= 1/2 the sampler returns 0 iff u <= (1-q)^R
// evaluated in binary32 by square-and-multiply; that value is >= 1 - Rb*(q + 2^-22)
// (Bernoulli's inequality plus at most 2R roundings of relative size 2^-24 and the rounding of
// 1-q).  The test uses an approximate quotient q~ (hardware reciprocal, relative error
// < 2^-21) and checks q~ <= 0.499 (so the sampler does not take its complement branch) and
// u + Rb*(q~*(1+1e-5) + 1e-6) <= 1 - 1e-5, which implies the former (and Rb*q < 1 implies a
// single piece).
#pragma once
#include "rng_binom.h"

namespace same {

constexpr int kWave = 64;   // lanes per workgroup (one wave)
constexpr int kBlk = 16;    // topics per checkpoint block
constexpr int kQCap = 12;   // queued candidates per lane between drains (drain when > kQCap - 4)
constexpr int kInvTab = 256;

struct DrawArgs {
    int64_t         n;          // tasks in this launch
    const int32_t*  t_doc;      // [n_tasks] document of the task
    const int32_t*  t_word;     // [n_tasks] word of the task
    const uint32_t* t_g;        // [n_tasks] tokens in the task's group
    const int32_t*  order;      // [n_tasks] task id handled at each launch position
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

// The 16 weights of block b (zero beyond K).
template <bool UNIFORM, bool VEC>
__device__ __forceinline__ void block_weights(const float* __restrict__ th, const float* __restrict__ ph,
                                              int b, int K, float (&wv)[kBlk])
{
    const int k0 = b * kBlk;
    if (UNIFORM) {
#pragma unroll
        for (int j = 0; j < kBlk; ++j) wv[j] = (k0 + j < K) ? 1.0f : 0.0f;
        return;
    }
    if (VEC) {   // K % 16 == 0: four aligned 16-byte loads per operand
#pragma unroll
        for (int v = 0; v < kBlk / 4; ++v) {
            const float4 a = *reinterpret_cast<const float4*>(th + k0 + 4 * v);
            const float4 c = *reinterpret_cast<const float4*>(ph + k0 + 4 * v);
            wv[4 * v + 0] = a.x * c.x;
            wv[4 * v + 1] = a.y * c.y;
            wv[4 * v + 2] = a.z * c.z;
            wv[4 * v + 3] = a.w * c.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kBlk; ++j) wv[j] = (k0 + j < K) ? th[k0 + j] * ph[k0 + j] : 0.0f;
    }
}

// true when Bin(R', q) is certainly 0 for every R' <= Rf (see the header comment)
__device__ __forceinline__ bool surely_zero(float wk, float Pk, float u, float Rf)
{
    const float qa = wk * __builtin_amdgcn_rcpf(Pk);
    const float tt = Rf * (qa * 1.00001f + 1.0e-6f);
    return (qa <= 0.499f) && ((u + tt) <= 0.99999f);
}

template <bool UNIFORM, bool VEC, bool DEBUG>
__global__ __launch_bounds__(kWave) void draw_kernel(DrawArgs a)
{
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int K = a.K;
    const int nblk = (K + kBlk - 1) / kBlk;
    float*    inv_tab = reinterpret_cast<float*>(lds);             // [kInvTab]  1/x, correctly rounded
    float*    chk = inv_tab + kInvTab;                             // [nblk][64]
    uint32_t* que = lds + kInvTab + (size_t)nblk * kWave;          // [kQCap][4][64]

    for (int i = lane; i < kInvTab; i += kWave) inv_tab[i] = 1.0f / (float)i;
    __syncthreads();

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
        for (int b = 0; b < nblk; ++b) {
            chk[b * kWave + lane] = P;
            float wv[kBlk];
            block_weights<UNIFORM, VEC>(th, ph, b, K, wv);
#pragma unroll
            for (int j = 0; j < kBlk; ++j) {
                P = P + wv[j];
                const int k = b * kBlk + j;
                if ((VEC || k < K) && wv[j] >= wmax) { wmax = wv[j]; kstar = k; }
            }
        }
    }

    uint32_t R = N;
    int cnt = 0;
#ifdef SAME_STATS
    uint32_t st_wave_trips = 0, st_lane_trips = 0;
#endif

#ifdef SAME_NO_ATOMICS   // timing experiments only: results are wrong
    uint32_t sink = 0;
    auto emit = [&](int k, uint32_t n) { sink += n * (uint32_t)(k + 1); };
#else
    auto emit = [&](int k, uint32_t n) {
        atomicAdd(out_d + k, n);
        if (out_w) atomicAdd(out_w + k, n);
    };
#endif

    // ---- the conditional-binomial chain over the queued topics (descending k), as a state machine
    auto drain = [&]() {
        int e = 0;
        int st = 0;                    // 0: fetch the next queued topic, 1: walking a piece, 2: queue exhausted
        // state of the binomial in flight
        uint32_t bR = 0, rem = 0, L = 0, piece = 0, total = 0, n = 0, xw = 0;
        float sc = 0.f, r = 0.f, pmL = 0.f, pm = 0.f, cdf = 0.f, u = 0.f;
        bool flip = false, stalled = false;
        int kk = 0;
        uint32_t xb[4] = {0u, 0u, 0u, 0u};
        if (lane == 0) SAME_COUNT(a, 0, 1);                      // drains
        SAME_COUNT(a, 1, cnt);                                     // queued topics
        for (;;) {
            if (lane == 0) SAME_COUNT(a, 2, 1);                  // drain loop trips
#ifdef SAME_STATS
            st_wave_trips += 1; if (st != 2) st_lane_trips += 1;
#endif
            if (st == 0) {
                bool found = false;
                float wq = 0.f, Pq = 1.f;
                while (e < cnt && R > 0) {
                    wq = __uint_as_float(que[(e * 4 + 0) * kWave + lane]);
                    Pq = __uint_as_float(que[(e * 4 + 1) * kWave + lane]);
                    u = uniform_from_word(que[(e * 4 + 2) * kWave + lane]);
                    kk = (int)que[(e * 4 + 3) * kWave + lane];
                    ++e;
                    if (!surely_zero(wq, Pq, u, (float)R)) { found = true; break; }
                }
                if (!found) {
                    st = 2;
                } else {
                    const float q = wq / Pq;
                    if (q >= 1.0f) {
                        emit(kk, R);
                        R = 0;
                    } else if (q > 0.0f) {
                        flip = q > 0.5f;
                        const float qq = flip ? 1.0f - q : q;
                        sc = 1.0f - qq;
                        r = qq / sc;
                        const bool single = ((float)R * qq) <= 32.0f;
                        L = single ? R : (uint32_t)(32.0f / qq);
                        pmL = ipow(sc, L);
                        bR = R; rem = R; piece = 0; total = 0;
                        n = L;                      // L <= R: the first piece is a full one
                        xw = 0; pm = pmL; cdf = pmL; stalled = false;
                        st = 1;
                        SAME_COUNT(a, 3, 1);                       // binomials set up
                        if (!single) SAME_COUNT(a, 6, 1);          // ... of which in several pieces
                    }
                }
            }
            if (!__any(st != 2)) break;
            if (st == 1) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (!stalled && u > cdf && xw < n) {
                        SAME_COUNT(a, 4, 1);                       // walk steps
                        if (L < bR) SAME_COUNT(a, 7, 1);           // ... of which inside multi-piece binomials
                        xw += 1;
                        const float inv_x = xw < (uint32_t)kInvTab ? inv_tab[xw] : 1.0f / (float)xw;
                        pm = pm * r;
                        pm = pm * (float)(n - xw + 1u);
                        pm = pm * inv_x;
                        const float next = cdf + pm;
                        if (next == cdf) stalled = true; else cdf = next;
                    }
                }
                if (stalled || !(u > cdf && xw < n)) {          // this piece is finished
                    total += xw;
                    rem -= n;
                    if (rem > 0) {                               // next piece of the same binomial
                        piece += 1;
                        n = rem < L ? rem : L;
                        const float pm0 = (n == L) ? pmL : ipow(sc, n);
                        const uint32_t j = piece - 1u;
                        if ((j & 3u) == 0u) piece_block(key, (uint32_t)kk, j >> 2, xb);
                        const uint32_t word = (j & 3u) == 0u ? xb[0] : (j & 3u) == 1u ? xb[1] : (j & 3u) == 2u ? xb[2] : xb[3];
                        u = uniform_from_word(word);
                        xw = 0; pm = pm0; cdf = pm0; stalled = false;
                    } else {
                        const uint32_t nk = flip ? bR - total : total;
                        if (nk > 0) { emit(kk, nk); SAME_COUNT(a, 5, 1); }   // nonzero counts
                        R -= nk;
                        st = 0;
                    }
                }
            }
        }
        cnt = 0;
    };

    // ---- pass 2: blocks from last to first
    for (int b = nblk - 1; b >= 0; --b) {
        if (!__any(R > 0)) break;
        float wv[kBlk], Pv[kBlk];
        block_weights<UNIFORM, VEC>(th, ph, b, K, wv);
        {
            float P = chk[b * kWave + lane];
#pragma unroll
            for (int j = 0; j < kBlk; ++j) { P = P + wv[j]; Pv[j] = P; }
        }
        float Rb = (float)R;   // bound on the remaining count until the next drain
#pragma unroll
        for (int g = kBlk / 4 - 1; g >= 0; --g) {
            uint32_t x[4];
            primary_block(key, (uint32_t)(b * (kBlk / 4) + g), x);
#pragma unroll
            for (int j = 3; j >= 0; --j) {
                const int k = b * kBlk + g * 4 + j;
                const float wk = wv[g * 4 + j];
                const float Pk = Pv[g * 4 + j] + (k < kstar ? wmax : 0.0f);   // weight not yet decided at k
                const bool cand = (k != kstar) && (wk > 0.0f) && !surely_zero(wk, Pk, uniform_from_word(x[j]), Rb);
                if (cand) {
                    que[(cnt * 4 + 0) * kWave + lane] = __float_as_uint(wk);
                    que[(cnt * 4 + 1) * kWave + lane] = __float_as_uint(Pk);
                    que[(cnt * 4 + 2) * kWave + lane] = x[j];
                    que[(cnt * 4 + 3) * kWave + lane] = (uint32_t)k;
                    cnt += 1;
                }
            }
            if (__any(cnt > kQCap - 4)) { drain(); Rb = (float)R; }
        }
    }
    drain();
    if (R > 0) emit(kstar, R);
#ifdef SAME_NO_ATOMICS
    if (sink == 0xFFFFFFFFu) atomicAdd(out_d, sink);
#endif
#ifdef SAME_STATS
    if (lane == 0) SAME_COUNT(a, 8 + (32 - __clz(st_wave_trips)), 1);      // histogram of trips per wave (log2)
    if (live) SAME_COUNT(a, 24 + (32 - __clz(st_lane_trips)), 1);          // histogram of busy trips per lane
#endif
}

inline size_t draw_lds_bytes(int K)
{
    const int nblk = (K + kBlk - 1) / kBlk;
    return 4u * (size_t)(kInvTab + kWave * (nblk + 4 * kQCap));
}

}  // namespace same
