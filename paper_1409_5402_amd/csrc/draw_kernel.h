// Draw-and-scatter kernel of the SAME LDA sweep (Algorithm 3, the loop over document-word
// pairs; Section 4, multinomial form of the factored draw) for gfx950.
//
// Mapping: one lane per draw task (a group of tokens of one nonzero).  A lane walks the K
// topics of its task twice.
//   pass 1  accumulates the running sums P_k = w_0 + ... + w_k left to right
//           (w_k = theta[d][k] * phi[w][k]) and checkpoints P at every 16th topic in LDS;
//   pass 2  revisits the 16-topic blocks from the last to the first, rebuilds P_k inside the
//           block from its checkpoint, generates the topics' uniforms (one Philox block per 4
//           topics) and tests every topic: a topic whose uniform already proves that its
//           conditional binomial is 0 for ANY remaining count is dropped; the few others
//           are queued in LDS in chain order (descending k).
// The queue is then drained lane by lane: n_k ~ Bin(R, w_k / P_k), R -= n_k, with the exact
// division and the exact inversion sampler.  Deferring the (rare, expensive, serial) binomials
// to the drain keeps the 64 lanes of a wave converged during the two scans.
//
// The drop test is conservative and never changes a result.  For a single-piece binomial with
// R <= Rb trials and success probability q <= 1/2 the sampler returns 0 iff u <= (1-q)^R
// evaluated in binary32 by square-and-multiply; that value is >= 1 - Rb*(q + 2^-22)
// (Bernoulli's inequality plus at most 2R roundings of relative size 2^-24 and the rounding of
// 1-q).  The test uses an approximate quotient q~ (hardware reciprocal, relative error
// < 2^-21) and checks q~ <= 0.499 (so the sampler does not take its complement branch) and
// u + Rb*(q~*(1+1e-5) + 1e-6) <= 1 - 1e-5, which implies the former.
#pragma once
#include "rng_binom.h"

namespace same {

constexpr int kBlk = 16;    // topics per checkpoint block
constexpr int kQCap = 12;   // queued candidates per lane between drains (drain when > kQCap - 4)

struct DrawArgs {
    int64_t         n;          // tasks in this launch
    const int32_t*  t_doc;      // [n_tasks] document of the task
    const int32_t*  t_word;     // [n_tasks] word of the task
    const uint32_t* t_g;        // [n_tasks] tokens in the task's group
    const int64_t*  ids;        // debug launches: task ids to draw (else null: task = launch index)
    const float*    theta;      // [D][K]   (unused when weights are uniform)
    const float*    phi;        // [V][K]
    uint32_t*       ndk;        // [D][K]   (debug launches: [n][K] output rows)
    uint32_t*       nwk;        // [V][K] or null
    int32_t         K;
    uint32_t        m;
    uint32_t        seed_lo, seed_hi, pass;
};

template <bool UNIFORM>
__device__ __forceinline__ float weight(const float* __restrict__ th, const float* __restrict__ ph, int k)
{
    if (UNIFORM) return 1.0f;
    return th[k] * ph[k];
}

// Loads the 16 weights of block b (zero beyond K) into wv.
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

template <bool UNIFORM, bool VEC, bool DEBUG>
__global__ __launch_bounds__(256) void draw_kernel(DrawArgs a)
{
    extern __shared__ uint32_t lds[];
    const int T = blockDim.x;
    const int tid = threadIdx.x;
    const int K = a.K;
    const int nblk = (K + kBlk - 1) / kBlk;
    float*    chk = reinterpret_cast<float*>(lds);                 // [nblk][T]
    uint32_t* que = lds + (size_t)nblk * T;                        // [kQCap][3][T]

    // lanes past the end take the last task with zero copies: all loads stay valid, nothing is emitted
    const int64_t slot = (int64_t)blockIdx.x * T + tid;
    const bool live = slot < a.n;
    const int64_t row = live ? slot : a.n - 1;
    const int64_t tau = DEBUG ? a.ids[row] : row;
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

    // ---- pass 1: running sum, checkpoint before every block
    {
        float P = 0.0f;
        for (int b = 0; b < nblk; ++b) {
            chk[(size_t)b * T + tid] = P;
            float wv[kBlk];
            block_weights<UNIFORM, VEC>(th, ph, b, K, wv);
#pragma unroll
            for (int j = 0; j < kBlk; ++j) P = P + wv[j];
        }
    }

    uint32_t R = N;
    int cnt = 0;

    auto emit = [&](int k, uint32_t n) {
        atomicAdd(out_d + k, n);
        if (out_w) atomicAdd(out_w + k, n);
    };

    // drains the lane's queue in order (descending topic): the conditional-binomial chain
    auto drain = [&]() {
        for (int e = 0; __any(e < cnt && R > 0); ++e) {
            if (e < cnt && R > 0) {
                const float Pk = __uint_as_float(que[((size_t)e * 3 + 0) * T + tid]);
                const uint32_t x = que[((size_t)e * 3 + 1) * T + tid];
                const int k = (int)que[((size_t)e * 3 + 2) * T + tid];
                const float wk = weight<UNIFORM>(th, ph, k);
                const float q = wk / Pk;
                const uint32_t n = binom(R, q, uniform_from_word(x), key, (uint32_t)k);
                if (n > 0) emit(k, n);
                R -= n;
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
            float P = chk[(size_t)b * T + tid];
#pragma unroll
            for (int j = 0; j < kBlk; ++j) { P = P + wv[j]; Pv[j] = P; }
        }
        const float Rb = (float)R;   // bound on the remaining count until the next drain
#pragma unroll
        for (int g = kBlk / 4 - 1; g >= 0; --g) {
            uint32_t x[4];
            primary_block(key, (uint32_t)(b * (kBlk / 4) + g), x);
#pragma unroll
            for (int j = 3; j >= 0; --j) {
                const int k = b * kBlk + g * 4 + j;
                const float wk = wv[g * 4 + j];
                const float Pk = Pv[g * 4 + j];
                const float u = uniform_from_word(x[j]);
                const float qa = wk * __builtin_amdgcn_rcpf(Pk);
                const float tt = Rb * (qa * 1.00001f + 1.0e-6f);
                const bool surely_zero = (qa <= 0.499f) && ((u + tt) <= 0.99999f);
                const bool cand = (k > 0) && (wk > 0.0f) && !surely_zero;
                if (cand) {
                    que[((size_t)cnt * 3 + 0) * T + tid] = __float_as_uint(Pk);
                    que[((size_t)cnt * 3 + 1) * T + tid] = x[j];
                    que[((size_t)cnt * 3 + 2) * T + tid] = (uint32_t)k;
                    cnt += 1;
                }
            }
            if (__any(cnt > kQCap - 4)) drain();
        }
    }
    drain();
    if (R > 0) emit(0, R);
}

inline size_t draw_lds_bytes(int K, int threads)
{
    const int nblk = (K + kBlk - 1) / kBlk;
    return (size_t)threads * 4u * (size_t)(nblk + 3 * kQCap);
}

}  // namespace same
