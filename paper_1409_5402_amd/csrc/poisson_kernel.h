// Draw-and-scatter kernel of the SAME LDA sweep in the Poisson form (Section 4, second part; the
// sampling line of Algorithm 3 as printed) for gfx950: topic k of a task with Nf = mf * g copies gets
// an independent Poisson(Nf * w_k / mu) count, mu = the running sum of all weights.
//
// Mapping: one wave per workgroup, one lane per draw task.  A lane walks the K topics of its task twice.
//   pass 1  accumulates the running sums P_k = w_0 + ... + w_k left to right
//           (w_k = theta[d][k] * phi[w][k]) up to mu;
//   pass 2  revisits the 16-topic blocks from the last to the first, generates the topics' uniforms
//           (one Philox block per 4 topics) and tests every topic: a topic whose uniform already
//           proves that its count is 0 is dropped; the others are queued in LDS.
// The queue is drained by a per-lane state machine: every trip of the drain loop lets each lane either
// fetch its next queued topic and start its draw, or advance its pmf walk by a few steps, so lanes
// with long walks do not hold up lanes with many short ones.  A rate above 32 is cut into equal
// pieces (independent, one uniform each) that are handed to the whole wave, one piece per lane.
//
// The drop test is conservative and never changes a result.  A Poisson variable of rate
// lambda <= Nf * q (q = w/mu) drawn by inversion is 0 iff u <= exp(-lambda) as the sampler evaluates
// it; that value is >= 1 - Nf*(q + 2^-22).  The test checks q <= 0.499 and
// u + Nf*(q*(1+1e-4) + 1e-6) <= 1 - 1e-4, evaluated without a division (see ZeroTest), which
// implies the former.  A topic of zero weight passes it.
#pragma once
#include "scatter.h"

namespace same {

#ifndef SAME_QCAP
#define SAME_QCAP 8
#endif
constexpr int kBlk = 16;                // topics per block of the Poisson kernel's second pass
constexpr int kQCap = SAME_QCAP;        // queued topics per lane between drains (drain when > kQCap - 4)

// The sixteen theta and phi values of one block, loaded ahead of their use (K % 16 == 0 only).
struct PhiBlock { float4 v[kBlk / 4]; float4 t[kBlk / 4]; };

template <bool VEC>
__device__ __forceinline__ PhiBlock load_phi(const float* __restrict__ th, const float* __restrict__ ph, int b)
{
    PhiBlock r;
    if (VEC) {
#pragma unroll
        for (int v = 0; v < kBlk / 4; ++v) {
            r.v[v] = *reinterpret_cast<const float4*>(ph + b * kBlk + 4 * v);
            r.t[v] = *reinterpret_cast<const float4*>(th + b * kBlk + 4 * v);
        }
    }
    return r;
}

// The 16 weights of block b (zero beyond K).
template <bool VEC>
__device__ __forceinline__ void block_weights(const float* __restrict__ th, const float* __restrict__ ph,
                                              const PhiBlock& pre, int b, int K, float (&wv)[kBlk])
{
    const int k0 = b * kBlk;
    if (VEC) {
#pragma unroll
        for (int v = 0; v < kBlk / 4; ++v) {
            const float4 t = pre.t[v];
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
// (the margins cover the few roundings of this evaluation), in one comparison A*w <= d*M:
//   d = (1-1e-4) - Rf*1e-6 - u', with u' = x * 2^-32 rounded, never below u - 2^-24 (x is the raw
//       random word of the topic, u = (2*(x>>9)+1)/2^24; the 2^-24 is taken off in Bp);
//   A = max(Rf*(1+1e-4), 2.0041): since d < 1, A*w <= d*M also gives w/M < 1/2.0041 < 0.499.
// ZeroTest holds the two terms that depend only on the bound Rf.
struct ZeroTest {
    float A, Bp;
    __device__ __forceinline__ explicit ZeroTest(float Rf)
        : A(fmaxf(Rf * 1.0001f, 2.0041f)), Bp((0.9999f - Rf * 1.0e-6f) - 5.9604644775390625e-8f) {}
    // true when the count of a topic of weight wk is certainly 0 for every number of copies <= Rf
    __device__ __forceinline__ bool surely_zero(float wk, float Mk, uint32_t x) const
    {
        const float d = __builtin_fmaf((float)x, -2.3283064365386963e-10f, Bp);
        return A * wk <= d * Mk;
    }
};

template <bool VEC, bool DEBUG, int KC = 0>   // KC: the number of topics where it is known at compile time
__global__ __launch_bounds__(kWave) void poisson_draw_kernel(DrawArgs a)
{
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int K = KC > 0 ? KC : a.K;
    const int nblk = (K + kBlk - 1) / kBlk;
    constexpr int qw = 3;                                          // words per queue entry
    uint32_t* que = lds;                                           // [kQCap][qw][64], a ring per lane
    uint32_t* acc = lds + (size_t)(qw * kQCap) * kWave;            // [64] piece totals by owner lane
    uint32_t* stage = acc + kWave + threadIdx.x;                   // [3][64] pairs on their way to the pair list
    static_assert(kQCap <= 16, "two bits per ring slot in one register");
    uint32_t khi = 0;       // bits 9 and 10 of the topic queued in each ring slot (the entry holds the low nine)

    // lanes past the end take the last task with zero copies: all loads stay valid, nothing is emitted
    const int64_t slot = (int64_t)blockIdx.x * kWave + lane;
    const bool live = slot < a.n;
    const int64_t row = live ? slot : a.n - 1;
    // order holds non-negative 32-bit ids: the high byte of tau is then a constant zero for the whole launch
    const int64_t tau = DEBUG ? a.ids[row] : (int64_t)(uint32_t)a.order[row];
    const int32_t d = a.t_doc[tau];
    const int32_t w = a.t_word[tau];
    const float Nf = live ? a.mf * (float)a.t_g[tau] : 0.0f;
    const float* __restrict__ th = a.theta + (size_t)d * K;
    const float* __restrict__ ph = a.phi + (size_t)w * K;
    Scatter sc = make_scatter<DEBUG>(a, row, tau, d, w);
    acc[lane] = 0u;

    StreamKey key;
    key.seed_lo = a.seed_lo; key.seed_hi = a.seed_hi;
    key.tau_lo = (uint32_t)tau; key.tau_hi = (uint32_t)((uint64_t)tau >> 32) & 0xFFu;
    key.pass = a.pass;
    const PrimaryPre pre = primary_pre(key);

    // ---- pass 1: the normaliser mu (left-to-right running sum)
    float mu = 0.0f;
    {
        float P = 0.0f;
        PhiBlock cur = load_phi<VEC>(th, ph, 0);
        for (int b = 0; b < nblk; ++b) {
            PhiBlock nxt = cur;
            if (b + 1 < nblk) nxt = load_phi<VEC>(th, ph, b + 1);
            float wv[kBlk];
            block_weights<VEC>(th, ph, cur, b, K, wv);
#pragma unroll
            for (int j = 0; j < kBlk; ++j) P = P + wv[j];
            cur = nxt;
        }
        mu = P;
    }

    // ---- the draws of the queued topics, a per-lane state machine that lives across the whole scan
    int qh = 0, cnt = 0;    // ring queue: position of the oldest entry, entries queued
    int st = 0;             // 0: between draws, 1: walking a single piece,
                            // 3: holds a variable of several pieces, waiting for the wave to share it
    uint32_t np = 0, xw = 0;
    float r = 0.f, pm = 0.f, cdf = 0.f, u = 0.f;
    bool stalled = false;
    int kk = 0;
    uint32_t busy = 0;      // trips in which this lane had work: its cost for the next ordering

    // Variables cut into pieces.  The pieces are independent (own uniform each): those of all the
    // lanes in state 3 are numbered consecutively and dealt out over the 64 lanes; every owner
    // receives the total of its pieces through an LDS counter.
    auto pool = [&](uint64_t pend) {
        const uint32_t mine = (st == 3) ? np : 0u;
        uint32_t total = 0;
        for (uint64_t p = pend; p != 0; p &= p - 1) total += __shfl(mine, __ffsll((unsigned long long)p) - 1);
        if (lane == 0) { SAME_COUNT(a, 6, 1); SAME_COUNT(a, 7, total); }
        for (uint32_t base = 0; base < total; base += kWave) {
            const uint32_t p = base + (uint32_t)lane;
            int owner = lane;
            uint32_t first = 0, off = 0;
            for (uint64_t q = pend; q != 0; q &= q - 1) {        // the last owner whose first piece is <= p
                const int src = __ffsll((unsigned long long)q) - 1;
                if (p >= off) { owner = src; first = off; }
                off += __shfl(mine, src);
            }
            const float opm = __shfl(pm, owner), orr = __shfl(r, owner), ou = __shfl(u, owner);
            const uint32_t ok = (uint32_t)__shfl(kk, owner);
            StreamKey okey = key;
            okey.tau_lo = __shfl(key.tau_lo, owner);
            okey.tau_hi = __shfl(key.tau_hi, owner);
            if (p < total) {
                const uint32_t jp = p - first;
                float pmj = opm;                                   // the owner's exp(-rate)
                float uj = ou;
                if (jp > 0) {
                    uint32_t xb[4];
                    piece_block(okey, ok, (jp - 1u) >> 2, xb);
                    const uint32_t sel = (jp - 1u) & 3u;
                    uj = uniform_from_word(sel == 0u ? xb[0] : sel == 1u ? xb[1] : sel == 2u ? xb[2] : xb[3]);
                }
                uint32_t xj = 0;
                float cdfj = pmj;
                while (uj > cdfj) {
                    xj += 1;
                    pmj = pmj * orr;
                    pmj = pmj * inv_int((float)xj);
                    const float next = cdfj + pmj;
                    if (next == cdfj) break;
                    cdfj = next;
                }
                if (xj > 0) atomicAdd(acc + owner, xj);
            }
        }
        __syncthreads();
        if (st == 3) {
            const uint32_t nk = acc[lane];
            acc[lane] = 0u;
            if (nk > 0) { sc.emit(a, kk, nk, stage); SAME_COUNT(a, 5, 1); }
            st = 0;
        }
        __syncthreads();
    };

    // One trip of the machine for the whole wave: lanes in state 0 take their next queued topic,
    // shared variables are worked off when enough of them wait or nothing else is in flight,
    // walking lanes advance by kWalkSteps pmf steps.
    auto trip = [&]() {
        if (lane == 0) SAME_COUNT(a, 2, 1);
        busy += (st != 0 || cnt > 0) ? 1u : 0u;
        if (st == 0 && cnt > 0) {
            const float wq = __uint_as_float(que[(qh * qw + 0) * kWave + lane]);
            const float Mq = __uint_as_float(que[(qh * qw + 1) * kWave + lane]);
            const uint32_t xk = que[(qh * qw + 2) * kWave + lane];
            kk = (int)((xk & 511u) | (((khi >> (2 * qh)) & 3u) << 9));
            u = uniform_from_word(xk);
            qh = (qh + 1 == kQCap) ? 0 : qh + 1;
            --cnt;
            const float scaled = Nf * wq;
            const float lam = scaled / Mq;
            if (lam > 0.0f) {
                if (lam <= kPieceMean) {                           // one piece
                    r = lam;
                    const float pm0 = expneg(lam);
                    xw = 0; pm = pm0; cdf = pm0; stalled = false;
                    st = 1;
                } else {                                           // equal pieces: shared by the wave
                    np = (uint32_t)(lam / kPieceMean) + 1u;
                    r = lam / (float)np;
                    pm = expneg(r);
                    st = 3;
                }
            }
        }
        {
            const uint64_t pend = __ballot(st == 3);
            if (pend != 0 && (__popcll((unsigned long long)pend) >= kPoolMin || !__any(st == 1))) pool(pend);
        }
        if (__any(st == 1)) {
            const bool walking = st == 1;
#pragma unroll
            for (int i = 0; i < kWalkSteps; ++i) {
                const bool go = walking && !stalled && u > cdf;
                const uint32_t xn = xw + 1u;
                float pmn = pm * r;
                pmn = pmn * inv_int((float)xn);
                const float next = cdf + pmn;
                const bool still = next == cdf;
                if (go) SAME_COUNT(a, 4, 1);                       // walk steps
                xw = go ? xn : xw;
                pm = go ? pmn : pm;
                cdf = (go && !still) ? next : cdf;
                stalled = stalled || (go && still);
            }
            if (walking && (stalled || !(u > cdf))) {              // the piece is finished
                if (xw > 0) { sc.emit(a, kk, xw, stage); SAME_COUNT(a, 5, 1); }
                st = 0;
            }
        }
    };

    // ---- pass 2: blocks from last to first
    {
        PhiBlock cur = load_phi<VEC>(th, ph, nblk - 1);
        const ZeroTest zt(Nf);
        for (int b = nblk - 1; b >= 0; --b) {
            if (!__any(Nf > 0.0f)) break;
            PhiBlock nxt = cur;
            if (b > 0) nxt = load_phi<VEC>(th, ph, b - 1);
            float wv[kBlk];
            block_weights<VEC>(th, ph, cur, b, K, wv);
            cur = nxt;
#pragma unroll
            for (int g = kBlk / 4 - 1; g >= 0; --g) {
                uint32_t x[4];
                primary_block(key, pre, (uint32_t)(b * (kBlk / 4) + g), x);
#pragma unroll
                for (int j = 3; j >= 0; --j) {
                    const int k = b * kBlk + g * 4 + j;
                    const float wk = wv[g * 4 + j];
                    // a zero weight passes the test
                    const bool cand = (VEC || k < K) && Nf > 0.0f && !zt.surely_zero(wk, mu, x[j]);
                    if (cand) {
                        int e = qh + cnt;
                        e = e >= kQCap ? e - kQCap : e;
                        que[(e * qw + 0) * kWave + lane] = __float_as_uint(wk);
                        que[(e * qw + 1) * kWave + lane] = __float_as_uint(mu);
                        que[(e * qw + 2) * kWave + lane] = (x[j] & ~511u) | ((uint32_t)k & 511u);   // the uniform uses the top 23 bits
                        khi = (khi & ~(3u << (2 * e))) | (((uint32_t)k >> 9) << (2 * e));
                        cnt += 1;
                        SAME_COUNT(a, 1, 1);                       // queued topics
                    }
                }
                // trips are run only while some lane could not take the next four topics
                while (__any(cnt > kQCap - 4)) trip();
            }
        }
    }
    while (__any(st != 0 || cnt > 0)) trip();
    sc.close(a, live, stage);
    // The ordering key for the next pass: a running mean (weight 1/4 on this pass) predicts a task's next
    // cost a little better than this pass's cost alone.
    if (!DEBUG && live && a.cost) a.cost[tau] = (3u * a.cost[tau] + busy + 2u) >> 2;
}

inline size_t poisson_lds_bytes() { return 4u * (size_t)kWave * (size_t)(3 * kQCap + 4); }

}  // namespace same
