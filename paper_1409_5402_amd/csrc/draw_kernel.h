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
#define SAME_QCAP 8
#endif
#ifndef SAME_WALK_STEPS
#define SAME_WALK_STEPS 8
#endif
constexpr int kWave = 64;               // lanes per workgroup (one wave)
constexpr int kBlk = 16;                // topics per checkpoint block
constexpr int kQCap = SAME_QCAP;        // queued topics per lane between drains (drain when > kQCap - 4)
constexpr int kPairWords = 16;          // words of a pair-list slot: a count and up to 15 (topic, count) pairs
constexpr int kPairShift = 11;          // a pair is topic | count << 11 (topics < 2048, counts < 2^21)
constexpr int kWalkSteps = SAME_WALK_STEPS;   // pmf steps per trip of the chain machine
#ifndef SAME_POOL_MIN
#define SAME_POOL_MIN 8
#endif
constexpr float kPieceMean = 32.0f;     // a binomial whose mean exceeds this is cut into pieces of about this mean
constexpr int kPoolMin = SAME_POOL_MIN;       // waiting multi-piece binomials that trigger a shared pass

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
    uint32_t*       pairs;      // [n_slots][kPairWords] pair list in word order, or null (update nwk directly)
    const int32_t*  t_slot;     // [n_tasks] slot of each task in the pair list, -1 for a task without one
    int32_t         K;
    uint32_t        m;          // copies per token (multinomial form)
    float           mf;         // copies per token (Poisson form: any positive real)
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

// The sixteen theta and phi values of one block, loaded ahead of their use (K % 16 == 0 only).
struct PhiBlock { float4 v[kBlk / 4]; float4 t[kBlk / 4]; };

template <bool UNIFORM, bool VEC>
__device__ __forceinline__ PhiBlock load_phi(const float* __restrict__ th, const float* __restrict__ ph, int b)
{
    PhiBlock r;
    if (!UNIFORM && VEC) {
#pragma unroll
        for (int v = 0; v < kBlk / 4; ++v) {
            r.v[v] = *reinterpret_cast<const float4*>(ph + b * kBlk + 4 * v);
            r.t[v] = *reinterpret_cast<const float4*>(th + b * kBlk + 4 * v);
        }
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
    // true when Bin(R', w/M) is certainly 0 for every R' <= Rf (see the header comment)
    __device__ __forceinline__ bool surely_zero(float wk, float Mk, uint32_t x) const
    {
        const float d = __builtin_fmaf((float)x, -2.3283064365386963e-10f, Bp);
        return A * wk <= d * Mk;
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

// POISSON selects the second form of Section 4 (the one Algorithm 3 prints): topic k of a task
// with Nf = mf * g copies gets an independent Poisson(Nf * w_k / mu) count, mu = P_{K-1}.  The scan
// is the same (drop test with the bound Nf and M_k = mu for every topic, the heaviest included);
// the machine then has no remaining count to carry: a queued topic starts its draw at once, a rate
// above 32 is cut into equal pieces that wait for the wave like the binomial pieces do.
template <bool UNIFORM, bool VEC, bool DEBUG, bool POISSON>
__global__ __launch_bounds__(kWave) void draw_kernel(DrawArgs a)
{
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    const int K = a.K;
    const int nblk = (K + kBlk - 1) / kBlk;
    constexpr int qw = 3;                                          // words per queue entry
    uint32_t* chk = lds;                                           // [nblk][64] checkpoints (binary32 bits)
    uint32_t* que = lds + (size_t)nblk * kWave;                    // [kQCap][qw][64], a ring per lane
    static_assert(kQCap <= 16, "two bits per ring slot in one register");
    uint32_t khi = 0;       // bits 9 and 10 of the topic queued in each ring slot (the entry holds the low nine)
    // [64] piece totals by owner lane: they take the place of the last block's checkpoint, which pass 2
    // reads first and never again (it is cleared right after that read, before any trip can run)
    uint32_t* acc = lds + (size_t)(nblk - 1) * kWave;

    // lanes past the end take the last task with zero copies: all loads stay valid, nothing is emitted
    const int64_t slot = (int64_t)blockIdx.x * kWave + lane;
    const bool live = slot < a.n;
    const int64_t row = live ? slot : a.n - 1;
    // order holds non-negative 32-bit ids: the high byte of tau is then a constant zero for the whole launch
    const int64_t tau = DEBUG ? a.ids[row] : (int64_t)(uint32_t)a.order[row];
    const int32_t d = a.t_doc[tau];
    const int32_t w = a.t_word[tau];
    const uint32_t N = POISSON ? (live ? 1u : 0u) : (live ? a.m * a.t_g[tau] : 0u);
    const float Nf = POISSON ? (live ? a.mf * (float)a.t_g[tau] : 0.0f) : (float)N;
    const float* __restrict__ th = UNIFORM ? nullptr : a.theta + (size_t)d * K;
    const float* __restrict__ ph = UNIFORM ? nullptr : a.phi + (size_t)w * K;
    uint32_t* __restrict__ out_d = DEBUG ? a.ndk + (size_t)row * K : a.ndk + (size_t)d * K;
    uint32_t* __restrict__ out_w = (DEBUG || a.nwk == nullptr) ? nullptr : a.nwk + (size_t)w * K;

    StreamKey key;
    key.seed_lo = a.seed_lo; key.seed_hi = a.seed_hi;
    key.tau_lo = (uint32_t)tau; key.tau_hi = (uint32_t)((uint64_t)tau >> 32) & 0xFFu;
    key.pass = a.pass;
    const PrimaryPre pre = primary_pre(key);

    // ---- pass 1: running sum, checkpoint before every block; heaviest topic (highest index among ties)
    float wmax = -1.0f;
    int kstar = 0;
    float mu = 0.0f;
    {
        float P = 0.0f;
        PhiBlock cur = load_phi<UNIFORM, VEC>(th, ph, 0);
        for (int b = 0; b < nblk; ++b) {
            PhiBlock nxt = cur;
            if (b + 1 < nblk) nxt = load_phi<UNIFORM, VEC>(th, ph, b + 1);
            chk[b * kWave + lane] = __float_as_uint(P);
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
        mu = P;
    }

    // ---- the conditional-binomial chain over the queued topics (descending k), a per-lane state
    // machine that lives across the whole scan
    uint32_t R = N;         // copies not yet placed (the heaviest topic keeps what is left at the end)
    int qh = 0, cnt = 0;    // ring queue: position of the oldest entry, entries queued
    int st = 0;             // 0: between binomials, 1: walking a single piece,
                            // 3: holds a binomial of several pieces, waiting for the wave to share it
    uint32_t bR = 0, L = 0, xw = 0;
    float sc = 0.f, r = 0.f, pm = 0.f, cdf = 0.f, u = 0.f;
    bool flip = false, stalled = false;
    int kk = 0;
    uint32_t busy = 0;      // trips in which this lane had work: its cost for the next ordering

    // Every placed count goes to the document's row at once.  The word's row is updated either the
    // same way or, when the launch has a pair list, later by word_reduce_kernel: the task records
    // (topic, count) in its slot of the list (slots are in word order), so that the scattered
    // updates of [V][K] become one streaming pass with all updates of a row close together.
    const int32_t slot_id = (DEBUG || a.pairs == nullptr || out_w == nullptr) ? -1 : a.t_slot[tau];
    uint32_t* __restrict__ pslot = slot_id < 0 ? nullptr : a.pairs + (size_t)slot_id * kPairWords;
    uint32_t npairs = 0;
    auto emit = [&](int k, uint32_t n) {
        atomicAdd(out_d + k, n);
        if (pslot) {
            if (npairs < (uint32_t)(kPairWords - 1)) pslot[1u + npairs] = (uint32_t)k | (n << kPairShift);
            else atomicAdd(out_w + k, n);                          // slot full: straight to the row
            npairs += 1;
        } else if (out_w) {
            atomicAdd(out_w + k, n);
        }
    };

    // Binomials cut into pieces.  The pieces are independent (own uniform each): those of all the
    // lanes in state 3 are numbered consecutively and dealt out over the 64 lanes; every owner
    // receives the total of its pieces through an LDS counter.
    auto pool = [&](uint64_t pend) {
        const uint32_t np = (st == 3) ? (POISSON ? bR : (bR + L - 1u) / L) : 0u;   // Poisson: bR holds the piece count
        uint32_t total = 0;
        for (uint64_t p = pend; p != 0; p &= p - 1) total += __shfl(np, __ffsll((unsigned long long)p) - 1);
        if (lane == 0) { SAME_COUNT(a, 6, 1); SAME_COUNT(a, 7, total); }
        for (uint32_t base = 0; base < total; base += kWave) {
            const uint32_t p = base + (uint32_t)lane;
            int owner = lane;
            uint32_t first = 0, off = 0;
            for (uint64_t q = pend; q != 0; q &= q - 1) {        // the last owner whose first piece is <= p
                const int src = __ffsll((unsigned long long)q) - 1;
                if (p >= off) { owner = src; first = off; }
                off += __shfl(np, src);
            }
            const uint32_t oR = __shfl(bR, owner), oL = __shfl(L, owner), onp = __shfl(np, owner);
            const float osc = __shfl(POISSON ? pm : sc, owner), orr = __shfl(r, owner), ou = __shfl(u, owner);
            const uint32_t ok = (uint32_t)__shfl(kk, owner);
            StreamKey okey = key;
            okey.tau_lo = __shfl(key.tau_lo, owner);
            okey.tau_hi = __shfl(key.tau_hi, owner);
            if (p < total) {
                const uint32_t jp = p - first;
                const uint32_t nj = POISSON ? 0xFFFFFFFFu : ((jp == onp - 1u) ? oR - jp * oL : oL);
                float pmj = POISSON ? osc : ipow(osc, nj);          // Poisson: the owner's exp(-rate)
                float uj = ou;
                if (jp > 0) {
                    uint32_t xb[4];
                    piece_block(okey, ok, (jp - 1u) >> 2, xb);
                    const uint32_t sel = (jp - 1u) & 3u;
                    uj = uniform_from_word(sel == 0u ? xb[0] : sel == 1u ? xb[1] : sel == 2u ? xb[2] : xb[3]);
                }
                uint32_t xj = 0;
                float cdfj = pmj;
                while (uj > cdfj && xj < nj) {
                    xj += 1;
                    pmj = pmj * orr;
                    if (!POISSON) pmj = pmj * (float)(nj - xj + 1u);
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
            const uint32_t part = acc[lane];
            acc[lane] = 0u;
            const uint32_t nk = (!POISSON && flip) ? bR - part : part;
            if (nk > 0) { emit(kk, nk); SAME_COUNT(a, 5, 1); }
            if (!POISSON) R -= nk;
            st = 0;
        }
        __syncthreads();
    };

    // One trip of the machine for the whole wave: lanes in state 0 take their next queued topic
    // (re-tested against the now exact remaining count), shared binomials are worked off when enough
    // of them wait or nothing else is in flight, walking lanes advance by kWalkSteps pmf steps.
    auto trip = [&]() {
        if (lane == 0) SAME_COUNT(a, 2, 1);
        busy += (st != 0 || (cnt > 0 && R > 0)) ? 1u : 0u;
        if (st == 0) {
            bool found = false;
            float wq = 0.f, Mq = 1.f;
            while (cnt > 0 && R > 0) {
                wq = __uint_as_float(que[(qh * qw + 0) * kWave + lane]);
                Mq = __uint_as_float(que[(qh * qw + 1) * kWave + lane]);
                const uint32_t xk = que[(qh * qw + 2) * kWave + lane];
                kk = (int)((xk & 511u) | (((khi >> (2 * qh)) & 3u) << 9));
                u = uniform_from_word(xk);
                qh = (qh + 1 == kQCap) ? 0 : qh + 1;
                --cnt;
                if (!POISSON && kk == kstar) continue;             // the scan does not single out the heaviest topic
                if (POISSON || !ZeroTest((float)R).surely_zero(wq, Mq, xk)) { found = true; break; }
            }
            if (R == 0) cnt = 0;                                   // nothing left to place: the rest is void
            if (found && POISSON) {
                const float scaled = Nf * wq;
                const float lam = scaled / Mq;
                if (lam > 0.0f) {
                    L = 0xFFFFFFFFu;                               // the walk has no upper end
                    if (lam <= 32.0f) {                            // one piece
                        r = lam;
                        const float pm0 = expneg(lam);
                        xw = 0; pm = pm0; cdf = pm0; stalled = false;
                        st = 1;
                    } else {                                       // equal pieces: shared by the wave
                        bR = (uint32_t)(lam / 32.0f) + 1u;
                        r = lam / (float)bR;
                        pm = expneg(r);
                        st = 3;
                    }
                }
            } else if (found) {
                const float q = wq / Mq;
                if (q >= 1.0f) {
                    emit(kk, R);
                    R = 0;
                    cnt = 0;
                } else if (q > 0.0f) {
                    flip = q > 0.5f;
                    const float qq = flip ? 1.0f - q : q;
                    sc = 1.0f - qq;
                    r = qq / sc;
                    bR = R;
                    SAME_COUNT(a, 3, 1);                           // binomials set up
                    if (((float)R * qq) <= kPieceMean) {                // one piece of R trials
                        L = R;
                        const float pm0 = ipow(sc, R);
                        xw = 0; pm = pm0; cdf = pm0; stalled = false;
                        st = 1;
                    } else {                                       // pieces of L trials: shared by the wave
                        L = (uint32_t)(kPieceMean / qq);
                        st = 3;
                    }
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
                const bool go = walking && !stalled && u > cdf && xw < L;
                const uint32_t xn = xw + 1u;
                float pmn = pm * r;
                if (!POISSON) pmn = pmn * (float)(L - xn + 1u);
                pmn = pmn * inv_int((float)xn);
                const float next = cdf + pmn;
                const bool still = next == cdf;
                if (go) SAME_COUNT(a, 4, 1);                       // walk steps
                xw = go ? xn : xw;
                pm = go ? pmn : pm;
                cdf = (go && !still) ? next : cdf;
                stalled = stalled || (go && still);
            }
            if (walking && (stalled || !(u > cdf && xw < L))) {   // the piece is finished
                const uint32_t nk = (!POISSON && flip) ? bR - xw : xw;
                if (nk > 0) { emit(kk, nk); SAME_COUNT(a, 5, 1); }   // nonzero counts
                if (!POISSON) R -= nk;
                st = 0;
            }
        }
    };

    // ---- pass 2: blocks from last to first
    {
        PhiBlock cur = load_phi<UNIFORM, VEC>(th, ph, nblk - 1);
        ZeroTest zt(POISSON ? Nf : (float)R);   // R bounds the remaining count from here on
        for (int b = nblk - 1; b >= 0; --b) {
            if (!__any(R > 0)) break;
            PhiBlock nxt = cur;
            if (b > 0) nxt = load_phi<UNIFORM, VEC>(th, ph, b - 1);
            float wv[kBlk], Pv[kBlk];
            block_weights<UNIFORM, VEC>(th, ph, cur, b, K, wv);
            cur = nxt;
            {
                float P = __uint_as_float(chk[b * kWave + lane]);
                if (b == nblk - 1) acc[lane] = 0u;
#pragma unroll
                for (int j = 0; j < kBlk; ++j) { P = P + wv[j]; Pv[j] = P; }
            }
#pragma unroll
            for (int g = kBlk / 4 - 1; g >= 0; --g) {
                uint32_t x[4];
                primary_block(key, pre, (uint32_t)(b * (kBlk / 4) + g), x);
#pragma unroll
                for (int j = 3; j >= 0; --j) {
                    const int k = b * kBlk + g * 4 + j;
                    const float wk = wv[g * 4 + j];
                    const float Mk = POISSON ? mu : Pv[g * 4 + j] + (k < kstar ? wmax : 0.0f);   // weight not yet decided at k
                    // a zero weight passes the test; the heaviest topic may be queued: the chain skips it
                    const bool cand = (VEC || k < K) && !zt.surely_zero(wk, Mk, x[j]);
                    if (cand) {
                        int e = qh + cnt;
                        e = e >= kQCap ? e - kQCap : e;
                        que[(e * qw + 0) * kWave + lane] = __float_as_uint(wk);
                        que[(e * qw + 1) * kWave + lane] = __float_as_uint(Mk);
                        que[(e * qw + 2) * kWave + lane] = (x[j] & ~511u) | ((uint32_t)k & 511u);   // the uniform uses the top 23 bits
                        khi = (khi & ~(3u << (2 * e))) | (((uint32_t)k >> 9) << (2 * e));
                        cnt += 1;
                        SAME_COUNT(a, 1, 1);                       // queued topics
                    }
                }
                // trips are run only while some lane could not take the next four topics
                if (__any(cnt > kQCap - 4)) {
                    do { trip(); } while (__any(cnt > kQCap - 4));
                    if (!POISSON) zt = ZeroTest((float)R);
                }
            }
        }
    }
    while (__any(st != 0 || (cnt > 0 && R > 0))) trip();
    if (!POISSON && R > 0) emit(kstar, R);
    if (pslot && live) pslot[0] = npairs < (uint32_t)(kPairWords - 1) ? npairs : (uint32_t)(kPairWords - 1);
    // The ordering key for the next pass: a running mean (weight 1/4 on this pass) predicts a task's next
    // cost a little better than this pass's cost alone.
    if (!DEBUG && live && a.cost) a.cost[tau] = (3u * a.cost[tau] + busy + 2u) >> 2;
}

// Adds the recorded pairs to the word rows.  Slots are in word order and exist only for words with
// at least kSlotMinTasks tasks: a workgroup takes kReduceChunk consecutive slots, sums the pairs of
// the first `rows` words it meets in an LDS table and sends the rest straight to [V][K]; the table is
// then added to the rows it stands for.  Threads start at different pairs of their slots: tasks of
// one word have their large counts at the same topics, and aligned walks would meet at one address.
constexpr int kReduceChunk = 2048;
constexpr int kSlotMinTasks = 32;
constexpr int kReduceThreads = 1024;    // two slots per thread: the kernel waits on its loads, many waves hide that

__global__ __launch_bounds__(kReduceThreads) void word_reduce_kernel(const uint32_t* __restrict__ pairs,
                                                          const int32_t* __restrict__ slot_word, int64_t n, int K,
                                                          int rows, uint32_t* __restrict__ nwk)
{
    extern __shared__ uint32_t tab[];                              // [rows][K]
    const int64_t s0 = (int64_t)blockIdx.x * kReduceChunk;
    const int64_t s1 = s0 + kReduceChunk < n ? s0 + kReduceChunk : n;
    const int32_t w0 = slot_word[s0];
    for (int i = threadIdx.x; i < rows * K; i += blockDim.x) tab[i] = 0u;
    __syncthreads();
    for (int64_t s = s0 + threadIdx.x; s < s1; s += blockDim.x) {
        const uint32_t* __restrict__ src = pairs + (size_t)s * kPairWords;
        const int32_t w = slot_word[s];
        const bool in_tab = w - w0 < rows;
        uint32_t* dst = in_tab ? tab + (size_t)(w - w0) * K : nwk + (size_t)w * K;
        const uint32_t cnt = src[0];
        uint32_t idx = ((threadIdx.x & 255u) * cnt) >> 8;          // start somewhere in [0, cnt)
        for (uint32_t i = 0; i < cnt; i += 4u) {                   // four loads in flight, then their updates
            uint32_t p[4];
#pragma unroll
            for (uint32_t j = 0; j < 4u; ++j) {
                p[j] = (i + j < cnt) ? src[1u + idx] : 0u;
                idx = idx + 1u >= cnt ? 0u : idx + 1u;
            }
#pragma unroll
            for (uint32_t j = 0; j < 4u; ++j)
                if (i + j < cnt) atomicAdd(dst + (p[j] & ((1u << kPairShift) - 1u)), p[j] >> kPairShift);
        }
    }
    __syncthreads();
    uint32_t* base = nwk + (size_t)w0 * K;                         // row w0 + r, topic k is at base[r*K + k]
    for (int i = threadIdx.x; i < rows * K; i += blockDim.x) {
        const uint32_t v = tab[i];
        if (v != 0u) atomicAdd(base + i, v);                       // only rows of real words hold counts
    }
}

inline int reduce_rows(int K) { const int r = 16384 / K; return r < 1 ? 1 : (r > 64 ? 64 : r); }

inline size_t draw_lds_bytes(int K)
{
    const int nblk = (K + kBlk - 1) / kBlk;
    return 4u * (size_t)kWave * (size_t)(nblk + 3 * kQCap);
}

}  // namespace same
