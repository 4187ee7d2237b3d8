// Dense kernels around the draw: zeroing, topic totals, the parameter update of Eq. 6 /
// Algorithm 3 (add priors, normalise phi over words, blend) and the log-likelihood reduction.
// All are plain coalesced streams over [rows][K] matrices; every arithmetic step is one
// binary32 operation (no contraction), in the order stated next to it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rng_binom.h"

namespace same {

// Self-test: reciprocal of every integer in [1, 2^24) and the published Philox known answers.
__global__ void selftest_kernel(unsigned long long* __restrict__ failures)
{
    const uint32_t x = blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= 1u && x < (1u << 24)) {
        const float fx = (float)x;
        if (inv_int(fx) != 1.0f / fx) atomicAdd(failures, 1ull);
    }
    if (x < 3u) {
        const uint32_t in[3][6] = {{0u, 0u, 0u, 0u, 0u, 0u},
                                   {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu},
                                   {0x243f6a88u, 0x85a308d3u, 0x13198a2eu, 0x03707344u, 0xa4093822u, 0x299f31d0u}};
        const uint32_t want[3][4] = {{0x6627e8d5u, 0xe169c58du, 0xbc57ac4cu, 0x9b00dbd8u},
                                     {0x408f276du, 0x41c83b0eu, 0xa20bc7c6u, 0x6d5451fdu},
                                     {0xd16cfe09u, 0x94fdccebu, 0x5001e420u, 0x24126ea1u}};
        uint32_t out[4];
        philox4x32_10(in[x][0], in[x][1], in[x][2], in[x][3], in[x][4], in[x][5], out);
        for (int i = 0; i < 4; ++i) if (out[i] != want[x][i]) atomicAdd(failures, 1ull);
    }
}

__global__ void zero_u32_kernel(uint32_t* __restrict__ p, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

__global__ void zero_u64_kernel(unsigned long long* __restrict__ p, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0ull;
}

// Re-sorts the processing order of one document tile by descending cost (counting sort over 256
// cost buckets; ties land in arbitrary order, which only affects scheduling, never results).
__global__ __launch_bounds__(256) void reorder_kernel(const int32_t* __restrict__ tile_start,
                                                      const uint32_t* __restrict__ cost,
                                                      int32_t* __restrict__ order)
{
    __shared__ uint32_t bins[256];
    const int t0 = tile_start[blockIdx.x], t1 = tile_start[blockIdx.x + 1];
    bins[threadIdx.x] = 0u;
    __syncthreads();
    for (int i = t0 + (int)threadIdx.x; i < t1; i += 256) atomicAdd(&bins[min(cost[i], 255u)], 1u);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t acc = 0u;
        for (int b = 255; b >= 0; --b) { const uint32_t c = bins[b]; bins[b] = acc; acc += c; }
    }
    __syncthreads();
    for (int i = t0 + (int)threadIdx.x; i < t1; i += 256) {
        const uint32_t pos = atomicAdd(&bins[min(cost[i], 255u)], 1u);
        order[t0 + (int)pos] = i;
    }
}

// n_k = sum over words of n_wk[w][k], exact in 64-bit integers (any order gives the same value).
// Each block sums a slab of rows; thread t owns column (t mod K') of every row group.
__global__ void topic_totals_kernel(const uint32_t* __restrict__ nwk, int V, int K,
                                    unsigned long long* __restrict__ nk, int rows_per_block)
{
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(V, r0 + rows_per_block);
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
        unsigned long long acc = 0ull;
        for (int r = r0; r < r1; ++r) acc += nwk[(size_t)r * K + k];
        if (acc) atomicAdd(nk + k, acc);
    }
}

// theta = n_dk / m + alpha   (divide, then add)
__global__ void theta_update_kernel(const uint32_t* __restrict__ ndk, float* __restrict__ theta,
                                    size_t n, float mf, float alpha)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float avg = (float)ndk[i] / mf;
        theta[i] = avg + alpha;
    }
}

// phi_hat = (n_wk/m + beta) / (n_k/m + V*beta);  phi = rho == 1 ? phi_hat : (1-rho)*phi + rho*phi_hat
__global__ void phi_update_kernel(const uint32_t* __restrict__ nwk, const unsigned long long* __restrict__ nk,
                                  float* __restrict__ phi, size_t n, int K, float mf, float beta,
                                  float vbeta, float rho)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const float one_minus_rho = 1.0f - rho;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int k = (int)(i % (size_t)K);
        const float avg_k = (float)nk[k] / mf;
        const float den = avg_k + vbeta;
        const float avg = (float)nwk[i] / mf;
        const float num = avg + beta;
        const float hat = num / den;
        if (rho == 1.0f) {
            phi[i] = hat;
        } else {
            const float keep = one_minus_rho * phi[i];
            const float add = rho * hat;
            phi[i] = keep + add;
        }
    }
}

// log of each document's theta total (double, summed left to right)
__global__ void doc_log_total_kernel(const float* __restrict__ theta, int D, int K, double* __restrict__ out)
{
    const int d = blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= D) return;
    double s = 0.0;
    for (int k = 0; k < K; ++k) s += (double)theta[(size_t)d * K + k];
    out[d] = log(s);
}

// Per nonzero: c * (log(sum_k theta_dk phi_wk) - log theta total); the inner sum is the
// binary32 left-to-right running sum of the draw.  Block partial sums (double) go to part[].
__global__ __launch_bounds__(256) void loglik_kernel(int64_t nnz, const int32_t* __restrict__ nz_doc,
                                                     const int32_t* __restrict__ rowidx,
                                                     const float* __restrict__ val,
                                                     const float* __restrict__ theta,
                                                     const float* __restrict__ phi, int K,
                                                     const double* __restrict__ doc_log_total,
                                                     double* __restrict__ part)
{
    __shared__ double red[256];
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    double v = 0.0;
    if (i < nnz) {
        const int d = nz_doc[i];
        const float* th = theta + (size_t)d * K;
        const float* ph = phi + (size_t)rowidx[i] * K;
        float S;
        if ((K & 3) == 0) {                                        // 16-byte loads, the same order of additions (0 + x = x)
            S = 0.0f;
            for (int k = 0; k < K; k += 4) {
                const float4 t = *reinterpret_cast<const float4*>(th + k);
                const float4 p = *reinterpret_cast<const float4*>(ph + k);
                S = S + t.x * p.x;
                S = S + t.y * p.y;
                S = S + t.z * p.z;
                S = S + t.w * p.w;
            }
        } else {
            S = th[0] * ph[0];
            for (int k = 1; k < K; ++k) { const float wk = th[k] * ph[k]; S = S + wk; }
        }
        v = (double)val[i] * (log((double)S) - doc_log_total[d]);
    }
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}

// The normaliser of Algorithm 3 as a kernel of its own (Section 5.3: SDDMM, the product of two dense
// matrices evaluated at the nonzeros of a sparse one): mu[i] = sum_k theta[d][k] * phi[w][k].
// One wave per nonzero at a time, lanes across topics: a lane multiplies four consecutive topics
// (16-byte loads: the 64 lanes read a row's 1 KB in one instruction), the wave sums its 64 partial
// results inside rows of 16 lanes by DPP moves, the four row sums by lane reads.  A wave owns
// kSddmmChunk consecutive nonzeros (mostly one document: its theta row stays in cache) and keeps
// the loads of four of them in flight.
constexpr int kSddmmChunk = 32;

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v = dpp_add<0xB1>(v);      // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);      // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);     // row_half_mirror
    v = dpp_add<0x140>(v);     // row_mirror: every lane of a row of 16 holds the row's sum
    const int b = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
    return (r0 + r1) + (r2 + r3);
}

template <bool VEC>   // VEC: K is a multiple of 4
__global__ __launch_bounds__(256) void sddmm_kernel(const int32_t* __restrict__ nz_doc,
                                                    const int32_t* __restrict__ rowidx, int64_t nnz, int K,
                                                    const float* __restrict__ theta, const float* __restrict__ phi,
                                                    float* __restrict__ mu)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t i0 = wave * kSddmmChunk;
    const int64_t i1 = i0 + kSddmmChunk < nnz ? i0 + kSddmmChunk : nnz;
    for (int64_t i = i0; i < i1; i += 4) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i + j < i1) {                                      // uniform over the wave
                const float* __restrict__ t = theta + (size_t)nz_doc[i + j] * K;
                const float* __restrict__ p = phi + (size_t)rowidx[i + j] * K;
                if (VEC) {
                    for (int q = lane; q < (K >> 2); q += 64) {
                        const float4 a = *reinterpret_cast<const float4*>(t + 4 * q);
                        const float4 b = *reinterpret_cast<const float4*>(p + 4 * q);
                        acc[j] = __builtin_fmaf(a.x, b.x, acc[j]);
                        acc[j] = __builtin_fmaf(a.y, b.y, acc[j]);
                        acc[j] = __builtin_fmaf(a.z, b.z, acc[j]);
                        acc[j] = __builtin_fmaf(a.w, b.w, acc[j]);
                    }
                } else {
                    for (int k = lane; k < K; k += 64) acc[j] = __builtin_fmaf(t[k], p[k], acc[j]);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float total = wave_sum(acc[j]);
            if (i + j < i1 && lane == 0) mu[i + j] = total;
        }
    }
}

// K a multiple of 4 and at most 256: a row is one 16-byte load per lane.  The wave reads the ids of its
// kSddmmChunk nonzeros with one load (lane l those of nonzero l), then goes through them four at a time with
// the eight row loads of the next four in flight; every round issues the same loads (past the end of the matrix
// those of its last nonzero), so that the wait before a round's sums has a fixed number of younger loads behind it.
__global__ __launch_bounds__(256) void sddmm_small_kernel(const int32_t* __restrict__ nz_doc,
                                                          const int32_t* __restrict__ rowidx, int64_t nnz, int K,
                                                          const float* __restrict__ theta, const float* __restrict__ phi,
                                                          float* __restrict__ mu)
{
    static_assert(kSddmmChunk <= 64 && kSddmmChunk % 4 == 0, "one id per lane, rounds of four");
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t i0 = wave * kSddmmChunk;
    if (i0 >= nnz) return;                                         // the whole wave
    const int64_t mine = i0 + lane < nnz ? i0 + lane : nnz - 1;
    const int32_t my_d = nz_doc[mine], my_w = rowidx[mine];
    const int k = 4 * lane;
    const bool in = k < K;
    auto rows = [&](int r, float4 (&t)[4], float4 (&p)[4]) {      // the rows of round r (nonzeros 4r .. 4r+3 of the chunk)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int src = (4 * r + j) & (kSddmmChunk - 1);
            const int32_t dd = __builtin_amdgcn_readlane(my_d, src), ww = __builtin_amdgcn_readlane(my_w, src);
            t[j] = in ? *reinterpret_cast<const float4*>(theta + (size_t)dd * K + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            p[j] = in ? *reinterpret_cast<const float4*>(phi + (size_t)ww * K + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto sums = [&](int r, const float4 (&t)[4], const float4 (&p)[4]) {
        float total[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float acc = 0.f;
            acc = __builtin_fmaf(t[j].x, p[j].x, acc);
            acc = __builtin_fmaf(t[j].y, p[j].y, acc);
            acc = __builtin_fmaf(t[j].z, p[j].z, acc);
            acc = __builtin_fmaf(t[j].w, p[j].w, acc);
            total[j] = wave_sum(acc);
        }
        const int64_t i = i0 + 4 * r + lane;                       // lanes 0..3 write the round's four values
        const float v = lane == 0 ? total[0] : lane == 1 ? total[1] : lane == 2 ? total[2] : total[3];
        if (lane < 4 && i < nnz) mu[i] = v;
    };
    float4 ta[4], pa[4], tb[4], pb[4];
    rows(0, ta, pa);
    static_assert((kSddmmChunk / 4) % 2 == 0, "rounds in pairs");
#pragma unroll 1
    for (int r = 0; r < kSddmmChunk / 4; r += 2) {
        rows(r + 1, tb, pb);
        __builtin_amdgcn_sched_barrier(0);
        sums(r, ta, pa);
        __builtin_amdgcn_sched_barrier(0);
        rows(r + 2, ta, pa);                                       // the last one wraps to round 0: loaded, not used
        __builtin_amdgcn_sched_barrier(0);
        sums(r + 1, tb, pb);
        __builtin_amdgcn_sched_barrier(0);
    }
}

}  // namespace same
