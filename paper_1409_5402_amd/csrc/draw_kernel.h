// Draw-and-scatter kernel of the SAME LDA sweep (Algorithm 3, the loop over document-word pairs;
// Section 4, multinomial form of the factored draw) for gfx950.
//
// One wave per workgroup takes 64 draw tasks (a task: a group of tokens of one nonzero) through two
// phases.
//
// Scan (lanes across topics).  Two tasks at a time, one per half-wave: lane l of a half owns block l of
// its task's topics, T = 4*ceil(K/128) consecutive topics (T = 8 at K = 256: the 32 lanes read the
// task's phi row and its document's theta row as two 16-byte loads each), multiplies them
// (w_k = theta[d][k] * phi[w][k]) and adds the block's weights left to right.  The 32 block sums of a
// task go to LDS.  No random numbers are used here and nothing is kept per topic.  (For K = 512 and 1024 the
// lanes of a half read consecutive 16-byte pieces instead and share the blocks' sums: see COAL below.)
//
// Draw (one lane per task).  A lane first turns its task's block sums into running sums S_0..S_31 (left to
// right, so S_l is the cumulative weight at the end of block l and S_31 = mu, the normaliser of
// Algorithm 3).  The cumulative weight at topic k of block l is P_k = S_{l-1} + (running sum inside the
// block): topic k owns the interval (P_{k-1}, P_k] of (0, mu).  The N = m*g copies are N uniform points
// on (0, mu); they are placed from the top, one step per topic that receives copies.  With R copies
// left, all below U:
//   - the highest one sits at y = U * u^(1/R) (one uniform, the R-th root by the fixed log/exp
//     sequences of rng_binom.h);
//   - its block is the first l with S_l >= y (binary search in LDS); the lane reloads that one block's
//     theta and phi values, rebuilds its P_k and takes the first k with P_k >= y;
//   - the other R-1 copies are uniform below y: 1 + Binomial(R-1, (y - P_{k-1}) / y) copies go to k
//     (exact inversion sampler), the rest continue below U = P_{k-1}.
// The work of a task is proportional to the number of topics that receive copies, not to K, and the
// second visit of a row touches only the blocks that receive copies.
//
// Lanes differ in the number of steps and in the length of their pmf walks; the draw therefore runs as a
// per-lane state machine: every trip lets each lane either take its next step or advance its walk by
// a few terms, so lanes with long walks do not hold up lanes with many short steps.  A binomial that
// the sampler cuts into several pieces (independent, one uniform each) is handed to the whole wave,
// one piece per lane.  Two consecutive steps of a task share one Philox block.
#pragma once
#include <type_traits>
#include "scatter.h"

namespace same {

constexpr int kMaxBlocks = 32;                  // blocks of topics per task (= lanes of a half-wave)
constexpr int kSumStride = kMaxBlocks + 1;      // words between the block sums of two tasks in LDS: lanes that
                                                // read the same block of 64 different tasks hit 32 different banks

__host__ __device__ inline int block_len(int K) { return 4 * ((K + 127) / 128); }

// Rows of document counts a wave keeps in LDS: two up to K = 128, one up to K = 1024 (4 KB at most), none beyond.
// A second row at K = 256 would serve the waves that straddle two documents, but its kilobyte costs two of the
// fifteen waves a compute unit holds, which costs more.
__host__ __device__ inline int doc_rows(int K) { return K <= 128 ? 2 : (K <= 1024 ? 1 : 0); }

// The value of v in the next lower lane (lanes 0, 16, 32, 48 receive 0): a row shift inside the vector ALU.
__device__ __forceinline__ float from_lane_below(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x111, 0xf, 0xf, true));
}

// Position of the highest of R copies uniform on (0, U).
__device__ __forceinline__ float top_position(float U, uint32_t R, float u)
{
    const float a = -flog(u);
    const float z = a / (float)R;
    float e = expneg(z);
    e = e > 1.0f ? 1.0f : e;
    float y = (R == 1u) ? U * u : U * e;
    if (!(y > 0.0f)) y = U;
    return y;
}

#ifndef SAME_REFILL_MIN
#define SAME_REFILL_MIN 24
#endif
#ifndef SAME_WALK_ROUNDS
#define SAME_WALK_ROUNDS 1
#endif
constexpr int kRefillMin = SAME_REFILL_MIN;     // idle lanes that make the wave fetch new tasks
constexpr int kWalkRounds = SAME_WALK_ROUNDS;   // rounds of kWalkSteps pmf terms per trip, while some lane needs them

// VEC: K is a multiple of 4 (16-byte loads), else element-wise loads (TB = 0).  TB: 16-byte loads per matrix that
// a lane has in flight at a time: a block of T = 4 ceil(K / 128) topics is read in T / (4 TB) batches of TB loads
// per matrix, TB the largest of 1, 2, 4 that divides T / 4 (one batch of one up to K = 128, one of two up to 256,
// one of four from 385 to 512, two of four from 897 to 1024).  ONE: a block is a single batch.  KC > 0: the
// same kernel with the number of topics a constant (row addresses become shifts, the bounds of the loads vanish).
// COAL (KC = 128 n, n = 2, 4 or 8): in the scan a load covers 128 consecutive topics per half-wave, four per lane,
// instead of four topics of every lane's own block: a wave's load touches 8 cache lines, not 64 (blocks of 32
// topics are a whole line each, and the cache serves a load one line at a time: with 64 lines per load the kernel
// at K = 1024 was bound there, at half the speed).  The n lanes that hold a block then add its products in the
// same left-to-right order through a chain of lane-to-lane shifts; the block sums are the same bits.  The steps'
// reloads of single blocks stay as they are (a lane's block belongs to its own task).
//
// The launch positions are handed out in segments of kSegment consecutive positions through a counter in
// device memory (a.counter, zero at launch): a workgroup (one wave) takes a segment, its lanes take the
// segment's tasks as they become free, and when the segment is used up the wave takes the next one.  Tasks
// differ widely in the number of steps they need (one for most, a hundred for a few): a lane that waited
// for the slowest of 64 fixed tasks would idle most of the time, and a wave with a fixed share of the matrix
// would end with one lane busy.  Whenever kRefillMin lanes are idle the wave stops stepping, gives each idle
// lane the next position, scans the new tasks (two per instruction) and goes on.
#ifndef SAME_SEGMENT
#define SAME_SEGMENT 512
#endif
constexpr int kSegment = SAME_SEGMENT;

template <bool UNIFORM, bool VEC, bool DEBUG, int TB, bool ONE, int KC = 0, bool COAL = false>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(TB <= 2 ? 4 : 3))) void draw_kernel(DrawArgs a)
{
    extern __shared__ uint32_t lds[];
    float* sums = reinterpret_cast<float*>(lds);                   // [64 lanes][kSumStride]: block sums, then running sums
    uint32_t* acc = lds + kMaxBlocks;                              // piece totals by owner lane: lane l's is acc[l * kSumStride],
                                                                   // the word of its row of sums that pads the stride
    const int lane = threadIdx.x;
    const int K = KC > 0 ? KC : a.K;                              // KC: the number of topics where it is known at compile time
    const int T = (TB > 0 && ONE) ? 4 * TB : block_len(K);         // topics per block
    const int nb = (TB > 0 && !ONE) ? T / (4 * TB) : 1;            // batches of loads per block
    const int nblk = (K + T - 1) / T;                              // blocks in use (<= 32)
    const int half = lane >> 5, hl = lane & 31;
    // Rows of the new document counts kept in LDS while the wave works on their documents (the launch positions are
    // in storage order: the 64 lanes hold tasks of one or two documents at a time).  Counts are added here and
    // reach the matrix in one pass over the row when the wave has left the document; tasks of a document that
    // has no row here add to the matrix at once.
    uint32_t* stage = lds + (size_t)kWave * kSumStride + lane;     // [3][64] pairs on their way to the pair list
    uint32_t* rows = lds + (size_t)kWave * (kSumStride + 3);       // [n_rows][K]
    const int n_rows = DEBUG ? 0 : doc_rows(K);
    int tag0 = -1, tag1 = -1;                                      // the documents of rows 0 and 1 (wave-uniform), -1: free
    int myrow = -1;                                                // the row of this lane's document, -1: none
    for (int i = lane; i < n_rows * K; i += kWave) rows[i] = 0u;
    int32_t next = 0, end = 0;                                     // the wave's segment: positions not yet handed out
    bool drained = false;                                          // the counter has passed the last position
    uint32_t chunk_next = 0, chunk_end = 0;                        // the wave's share of the chunk pool not yet handed out
    bool pool_dry = a.chunks == nullptr;                           // the pool has no chunk left for this wave
    acc[lane * kSumStride] = 0u;

    // ---- the lane's current task
#ifdef SAME_STATS
    uint32_t R_task_g = 0;
#endif
    bool open = false;      // a task was taken and its slot of the pair list is not yet closed
    int32_t d = 0, w = 0;
    Scatter sc;
    sc.drow = 0; sc.wrow = kNone; sc.slot = kNone; sc.npairs = 0;
    StreamKey key;
    key.seed_lo = a.seed_lo; key.seed_hi = a.seed_hi; key.tau_lo = 0; key.tau_hi = 0; key.pass = a.pass;
    PrimaryPre pre = primary_pre(key);

    // ---- the draw of that task: a per-lane state machine
    uint32_t R = 0;         // copies not yet placed, all of them below U
    float U = 0.0f;
    int lt = 0;             // block that holds U
    int top = K;            // the copies left belong to topics below top
    uint32_t step = 0;      // steps taken: the next one uses words 2*(step & 1), +1 of block step >> 1
    uint32_t xs2 = 0, xs3 = 0;   // the second half of the last Philox block, for the odd step
    int st = 0;             // 0: between steps, 1: walking a single-piece binomial,
                            // 3: holds a binomial of several pieces, waiting for the wave to share it
    uint32_t bR = 0, L = 0, xw = 0, bstep = 0;
    float r = 0.f, lq = 0.f, pm = 0.f, cdf = 0.f, u = 0.f;
    bool flip = false, stalled = false;
    int kk = 0;

    // Adds row i of the LDS counts to the matrix row of document doc and clears it (whole wave).
    auto flush_row = [&](int i, int doc) {
        __syncthreads();
        for (int k = lane; k < K; k += kWave) {
            const uint32_t v = rows[i * K + k];
            if (v) { atomicAdd(a.ndk + (size_t)doc * K + k, v); rows[i * K + k] = 0u; }
        }
        __syncthreads();
    };

    // Idle lanes take the next positions, the wave scans the new tasks' block sums (two tasks at a time, one
    // per half-wave: lane hl of a half owns block hl), each new lane turns its sums into running sums.
    auto refill = [&](uint64_t idle_mask) {
        const bool idle = (idle_mask >> lane) & 1ull;
        if (idle && open) { sc.close(a, true, stage); open = false; }
        const int rank = (int)__popcll(idle_mask & ((1ull << lane) - 1ull));
        const int avail = end - next;
        const bool take = idle && rank < avail;
        if (take) {
            const int64_t pos = (int64_t)next + rank;
            const int64_t tau = DEBUG ? a.ids[pos] : pos;
            d = a.t_doc[tau];
            w = a.t_word[tau];
            R = a.m * a.t_g[tau];
#ifdef SAME_STATS
            R_task_g = a.t_g[tau];
#endif
            sc = make_scatter<DEBUG>(a, pos, tau, d, w);
            key.tau_lo = (uint32_t)tau; key.tau_hi = (uint32_t)((uint64_t)tau >> 32) & 0xFFu;
            pre = primary_pre(key);
            open = true;
            lt = nblk - 1; top = K; step = 0; st = 0;
        }
        const int n_idle = (int)__popcll(idle_mask);
        next += n_idle < avail ? n_idle : avail;
        uint64_t fresh = __ballot(take);
        if (n_rows > 0) {
            // lanes that keep working keep their row; a new task joins the row of its document if there is one;
            // documents that are new to the wave get the rows no lane uses any more, lowest document first
            if (idle) myrow = -1;
            if (take) myrow = d == tag0 ? 0 : ((n_rows > 1 && d == tag1) ? 1 : -1);
            for (int round = 0; round < n_rows; ++round) {
                const uint64_t used0 = __ballot(myrow == 0), used1 = __ballot(myrow == 1);
                const int free_row = used0 == 0 ? 0 : ((n_rows > 1 && used1 == 0) ? 1 : -1);
                int dn = (take && myrow < 0) ? d : 0x7FFFFFFF;         // the lowest new document without a row
                for (int o = 32; o > 0; o >>= 1) dn = min(dn, __shfl_xor(dn, o));
                if (dn == 0x7FFFFFFF) break;
                if (free_row < 0) {
                    // one row (n_rows == 1) in use: it goes to the new document if that one now has more lanes than
                    // the row's document has left; the lanes that stay behind add to the matrix directly from here on
                    if (n_rows != 1) break;
                    const int n_new = (int)__popcll((unsigned long long)__ballot(take && myrow < 0 && d == dn));
                    if (n_new <= (int)__popcll((unsigned long long)used0)) break;
                    flush_row(0, tag0);
                    if (myrow == 0) myrow = -1;
                    tag0 = dn;
                    if (take && d == dn) myrow = 0;
                    break;
                }
                const int old = free_row == 0 ? tag0 : tag1;
                if (old >= 0) flush_row(free_row, old);
                if (free_row == 0) tag0 = dn; else tag1 = dn;
                if (take && d == dn) myrow = free_row;
            }
        }
        if (UNIFORM) {
            // all weights are 1: block l holds min(T, K - l*T) topics
            if (take) for (int l = 0; l < nblk; ++l) sums[lane * kSumStride + l] = (float)(min(K, (l + 1) * T) - l * T);
        } else {
            const int k0 = hl * T;
            // the next pair of new lanes: one for each half-wave (the last one twice if their number is odd)
            auto pick = [&](uint64_t& rem) {
                const int la = __ffsll((unsigned long long)rem) - 1;
                rem &= rem - 1;
                int lb = la;
                if (rem) { lb = __ffsll((unsigned long long)rem) - 1; rem &= rem - 1; }
                return half ? lb : la;
            };
            if (VEC && TB > 0) {
                // Where every block is whole (K = 32 T: 256 at T = 8) the loads need no bounds.  Blocks of one batch
                // (ONE) and of two batches of four loads go through the pipeline in run(); blocks of other shapes load
                // the next batch into a second set of registers before the current one is summed (the load there sits
                // under a condition, and the compiler's wait then covers it too: no overlap, rare shapes).
                struct Item { int src, b; bool last, valid; };
                auto advance = [&](Item& it) {                     // the next (pair of tasks, batch) of this refill
                    if (it.valid && !it.last) { it.b += 1; it.last = it.b == nb - 1; return; }
                    if (fresh == 0) { it.valid = false; return; }
                    it.src = pick(fresh); it.b = 0; it.last = nb == 1; it.valid = true;
                };
                auto run = [&](auto whole) {
                    constexpr bool WHOLE = decltype(whole)::value;
                    auto issue = [&](float4* pv, float4* tv, const Item& it) {     // blocks of several batches
                        const int32_t pd = __shfl(d, it.src), pw = __shfl(w, it.src);
                        const int kb = COAL ? 128 * TB * it.b + 4 * hl : k0 + 4 * TB * it.b;
                        constexpr int kStep = COAL ? 128 : 4;      // topics between two loads of a lane
                        const float* __restrict__ tp = a.theta + (size_t)pd * K + kb;
                        const float* __restrict__ pp = a.phi + (size_t)pw * K + kb;
#pragma unroll
                        for (int c = 0; c < TB; ++c) {
                            if (WHOLE || kb + 4 * c < K) {
                                pv[c] = *reinterpret_cast<const float4*>(pp + kStep * c);
                                tv[c] = *reinterpret_cast<const float4*>(tp + kStep * c);
                            } else {
                                pv[c] = make_float4(0.f, 0.f, 0.f, 0.f);
                                tv[c] = make_float4(0.f, 0.f, 0.f, 0.f);
                            }
                        }
                    };
                    float rs = 0.0f;
                    auto consume = [&](const float4* pv, const float4* tv, const Item& it) {
                        if constexpr (COAL) {
                            // A load covers 128 consecutive topics of the task, four per lane: the kNL lanes that hold a block
                            // add its products left to right, the running sum handed from lane to lane.  Every lane
                            // runs all kNL stages; stage j is meaningful in the block's lane j, and the block's last lane
                            // ends with the same sum, rounded in the same order, as one lane that adds the block alone.
                            constexpr int kNL = KC / 128;
                            static_assert(!COAL || (KC >= 256 && KC % 128 == 0 && 16 % (KC / 128) == 0), "blocks must not straddle loads");
#pragma unroll
                            for (int c = 0; c < TB; ++c) {
                                const float x0 = tv[c].x * pv[c].x, x1 = tv[c].y * pv[c].y;
                                const float x2 = tv[c].z * pv[c].z, x3 = tv[c].w * pv[c].w;
                                float s = 0.0f;
#pragma unroll
                                for (int j = 0; j < kNL; ++j) {
                                    const float in = j == 0 ? 0.0f : from_lane_below(s);
                                    s = in + x0;
                                    s = s + x1;
                                    s = s + x2;
                                    s = s + x3;
                                }
                                if ((hl & (kNL - 1)) == kNL - 1)
                                    sums[it.src * kSumStride + (TB * it.b + c) * (32 / kNL) + hl / kNL] = s;
                            }
                            return;
                        }
#pragma unroll
                        for (int c = 0; c < TB; ++c) {
                            rs = rs + tv[c].x * pv[c].x;
                            rs = rs + tv[c].y * pv[c].y;
                            rs = rs + tv[c].z * pv[c].z;
                            rs = rs + tv[c].w * pv[c].w;
                        }
                        if (it.last) { sums[it.src * kSumStride + hl] = rs; rs = 0.0f; }
                    };
                    // Blocks of one batch, or of two (K = 1024).  The new tasks of a refill are worked off in runs whose
                    // document stays the same (a document's tasks are consecutive): the run's theta values are loaded once,
                    // one set of registers per batch, and the phi loads of the next batch are in flight while a batch is
                    // summed, in two sets used in turn (with two batches per block a set always holds the same batch).
                    // The loop has the same number of loads behind every sum on every path that reaches it: the
                    // compiler's wait then lets the younger loads fly.
                    auto pipeline = [&](auto batches) {
                        constexpr int NB = decltype(batches)::value;   // batches per block: 1 or 2
                        constexpr int N = 2;                       // sets of phi registers
                        constexpr int kStep = COAL ? 128 : 4;      // topics between two loads of a lane
                        constexpr int kBatch = COAL ? 128 * TB : 4 * TB;   // topics between two batches of a lane
                        const int kb0 = COAL ? 4 * hl : k0;
                        float4 pv[N][TB > 0 ? TB : 1], tv[NB][TB > 0 ? TB : 1];
                        int srcs[N];
                        int32_t held = -1;                         // the document whose theta values tv holds
                        int src_cur = 0;
                        const float* __restrict__ row_cur = a.phi; // the phi row of the pair whose batches are being issued
                        auto lane_of = [&](uint64_t m) { return __ffsll((unsigned long long)m) - 1; };
                        auto of_lane = [&](int32_t v, int l0, int l1) {    // v of lane l0 (first half-wave) or l1 (second)
                            const int32_t va = __builtin_amdgcn_readlane(v, l0), vb = __builtin_amdgcn_readlane(v, l1);
                            return half ? vb : va;
                        };
                        // batch i % NB of pair i / NB of the run goes to set i % N: with N = 2 and NB = 1 or 2 the batch
                        // of a set is known at compile time (j % NB)
                        auto issue_phi = [&](float4* p, int& src, int bt) {
                            if (bt == 0) {                         // the next pair of the run
                                const int l0 = lane_of(fresh);
                                fresh &= fresh - 1;
                                const int l1 = fresh ? lane_of(fresh) : l0;
                                fresh &= fresh - 1;
                                src_cur = half ? l1 : l0;
                                row_cur = a.phi + (size_t)of_lane(w, l0, l1) * K;
                            }
                            src = src_cur;
                            const int kb = kb0 + kBatch * bt;
#pragma unroll
                            for (int c = 0; c < TB; ++c)
                                p[c] = (WHOLE || kb + 4 * c < K) ? *reinterpret_cast<const float4*>(row_cur + kb + kStep * c)
                                                                  : make_float4(0.f, 0.f, 0.f, 0.f);
                        };
                        auto sum_batch = [&](const float4* p, int src, int bt) {
                            Item it{src, bt, bt == NB - 1, true};
                            consume(p, tv[bt], it);
                        };
                        while (fresh) {
                            const int32_t doc = __builtin_amdgcn_readlane(d, lane_of(fresh));
                            const uint64_t other = fresh & ~__ballot(d == doc);
                            const uint64_t lead = other ? fresh & ((other & (~other + 1ull)) - 1ull) : fresh;
                            const int lanes_in = (int)__popcll((unsigned long long)lead);
                            // pairs inside the document; a lane left over is scanned alone, as its own partner, when
                            // nothing else of its document is left
                            int pairs = lanes_in / 2;
                            uint64_t rest = 0;                     // new lanes set aside while this run is scanned
                            if (pairs == 0) { pairs = 1; rest = fresh & (fresh - 1); fresh &= ~rest; }
                            else {
                                rest = fresh & ~lead;
                                if (lanes_in & 1) rest |= 1ull << (63 - __clzll((unsigned long long)lead));
                                fresh &= ~rest;
                            }
                            const int P = pairs * NB;              // batches of the run
                            if (doc != held) {
                                const float* __restrict__ tp = a.theta + (size_t)doc * K;
#pragma unroll
                                for (int bt = 0; bt < NB; ++bt)
#pragma unroll
                                    for (int c = 0; c < TB; ++c) {
                                        const int kb = kb0 + kBatch * bt;
                                        tv[bt][c] = (WHOLE || kb + 4 * c < K) ? *reinterpret_cast<const float4*>(tp + kb + kStep * c)
                                                                               : make_float4(0.f, 0.f, 0.f, 0.f);
                                    }
                                held = doc;
                            }
                            issue_phi(pv[0], srcs[0], 0);          // P >= 1
                            int issued = 1;
                            while (P - issued >= N) {              // whole rounds: every sum has the loads of one batch behind it
#pragma unroll
                                for (int j = 0; j < N; ++j) {
                                    issue_phi(pv[(j + 1) % N], srcs[(j + 1) % N], (j + 1) % NB);
                                    __builtin_amdgcn_sched_barrier(0);     // the loads first, then the sum that waits
                                    sum_batch(pv[j], srcs[j], j % NB);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                                issued += N;
                            }
                            if (P - issued == 1) {                 // one batch not yet issued: it goes to set 1
                                issue_phi(pv[1], srcs[1], 1 % NB);
                                sum_batch(pv[0], srcs[0], 0);
                                sum_batch(pv[1], srcs[1], 1 % NB);
                            } else {
                                sum_batch(pv[0], srcs[0], 0);
                            }
                            fresh = rest;
                        }
                    };
                    if constexpr (ONE) {
                        pipeline(std::integral_constant<int, 1>{});
                        return;
                    } else if constexpr (TB == 4) {
                        if (nb == 2) {
                            pipeline(std::integral_constant<int, 2>{});
                            return;
                        }
                    }
                    float4 pa[TB > 0 ? TB : 1], ta[TB > 0 ? TB : 1], pb[TB > 0 ? TB : 1], tb[TB > 0 ? TB : 1];
                    Item cur{0, 0, false, false};
                    advance(cur);
                    if (cur.valid) issue(pa, ta, cur);
                    while (cur.valid) {
                        Item nxt = cur;
                        advance(nxt);
                        if (nxt.valid) issue(pb, tb, nxt);
                        consume(pa, ta, cur);
                        if (!nxt.valid) break;
                        cur = nxt;
                        advance(cur);
                        if (cur.valid) issue(pa, ta, cur);
                        consume(pb, tb, nxt);
                    }
                };
                if (nblk * T == K) run(std::true_type{}); else run(std::false_type{});
            } else {
                while (fresh) {
                    const int src = pick(fresh);
                    const int32_t pd = __shfl(d, src), pw = __shfl(w, src);
                    const float* __restrict__ tp = a.theta + (size_t)pd * K;
                    const float* __restrict__ pp = a.phi + (size_t)pw * K;
                    float rs = 0.0f;
                    if (VEC) {
                        for (int c = 0; c < T / 4; ++c) {
                            const int k = k0 + 4 * c;
                            if (k < K) {
                                const float4 x = *reinterpret_cast<const float4*>(pp + k);
                                const float4 t = *reinterpret_cast<const float4*>(tp + k);
                                rs = rs + t.x * x.x;
                                rs = rs + t.y * x.y;
                                rs = rs + t.z * x.z;
                                rs = rs + t.w * x.w;
                            }
                        }
                    } else {
                        for (int j = 0; j < T; ++j) {
                            const int k = k0 + j;
                            if (k < K) rs = rs + tp[k] * pp[k];
                        }
                    }
                    sums[src * kSumStride + hl] = rs;
                }
            }
        }
        __syncthreads();
        if (take) {
            float run = 0.0f;
            for (int l = 0; l < nblk; ++l) {
                run = run + sums[lane * kSumStride + l];
                sums[lane * kSumStride + l] = run;
            }
            U = run;
        }
    };

    // Binomials cut into pieces.  The pieces are independent (own uniform each): those of all the
    // lanes in state 3 are numbered consecutively and dealt out over the 64 lanes; every owner
    // receives the total of its pieces through an LDS counter.  Returns the owner's successes.
    auto pool = [&](uint64_t pend) -> uint32_t {
        const uint32_t np = (st == 3) ? (bR + L - 1u) / L : 0u;
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
            const float olq = __shfl(lq, owner), orr = __shfl(r, owner), ou = __shfl(u, owner);
            const uint32_t ostep = __shfl(bstep, owner);
            StreamKey okey = key;
            okey.tau_lo = __shfl(key.tau_lo, owner);
            okey.tau_hi = __shfl(key.tau_hi, owner);
            if (p < total) {
                const uint32_t jp = p - first;
                const uint32_t nj = (jp == onp - 1u) ? oR - jp * oL : oL;
                float pmj = expneg((float)nj * olq);               // no success among the piece's trials
                float uj = ou;
                if (jp > 0) {
                    uint32_t xb[4];
                    piece_block(okey, ostep, (jp - 1u) >> 2, xb);
                    const uint32_t sel = (jp - 1u) & 3u;
                    uj = uniform_from_word(sel == 0u ? xb[0] : sel == 1u ? xb[1] : sel == 2u ? xb[2] : xb[3]);
                }
                uint32_t xj = 0;
                float cdfj = pmj;
                while (uj > cdfj && xj < nj) {
                    xj += 1;
                    pmj = pmj * orr;
                    pmj = pmj * (float)(nj - xj + 1u);
                    pmj = pmj * inv_int((float)xj);
                    const float next_cdf = cdfj + pmj;
                    if (next_cdf == cdfj) break;
                    cdfj = next_cdf;
                }
                if (xj > 0) atomicAdd(acc + owner * kSumStride, xj);
            }
        }
        __syncthreads();
        uint32_t part = 0;
        if (st == 3) { part = acc[lane * kSumStride]; acc[lane * kSumStride] = 0u; }
        __syncthreads();
        return part;
    };

    // One trip of the machine for the whole wave.
    auto trip = [&]() {
        if (lane == 0) SAME_COUNT(a, 2, 1);
#ifdef SAME_STATS
        {   // lanes by what they do in this trip: step, walk on, wait for a shared pass, idle
            const uint64_t b_step = __ballot(st == 0 && R > 0), b_walk = __ballot(st == 1), b_wait = __ballot(st == 3);
            if (lane == 0) {
                SAME_COUNT(a, 8, __popcll((unsigned long long)b_step)); SAME_COUNT(a, 9, __popcll((unsigned long long)b_walk));
                SAME_COUNT(a, 10, __popcll((unsigned long long)b_wait));
                SAME_COUNT(a, 11, 64 - __popcll((unsigned long long)(b_step | b_walk | b_wait)));
            }
        }
#endif
        int ek = 0;             // the count this trip settles for this lane: en copies to topic ek
        uint32_t en = 0;
        if (st == 0 && R > 0) {
            SAME_COUNT(a, 1, 1);                                   // steps
            if (!(U > 0.0f)) {                                     // no weight left: a degenerate input
                ek = top > 0 ? top - 1 : 0; en = R;
                R = 0;
            } else {
                uint32_t xa, xb;
                if ((step & 1u) == 0u) {
                    uint32_t x[4];
                    primary_block(key, pre, step >> 1, x);
                    xa = x[0]; xb = x[1]; xs2 = x[2]; xs3 = x[3];
                } else {
                    xa = xs2; xb = xs3;
                }
                const float y = top_position(U, R, uniform_from_word(xa));
                // the first block whose cumulative weight reaches y (S_lt >= U >= y)
                int lo = 0, hi = lt;
#pragma unroll
                for (int it = 0; it < 5; ++it) {
                    const int mid = (lo + hi) >> 1;
                    const bool ge = sums[lane * kSumStride + mid] >= y;
                    hi = ge ? mid : hi;
                    lo = ge ? lo : (mid < hi ? mid + 1 : hi);
                }
                const int l = hi;
                const float base = l > 0 ? sums[lane * kSumStride + l - 1] : 0.0f;
                // inside the block: rebuild P_k from the block's weights, count the topics still below y
                const int k0 = l * T;
                const float* __restrict__ th = UNIFORM ? nullptr : a.theta + (size_t)d * K;   // the task's rows
                const float* __restrict__ ph = UNIFORM ? nullptr : a.phi + (size_t)w * K;
                int below = 0;
                float prev = base, rs = 0.0f;
                auto visit = [&](float wk) {
                    rs = rs + wk;
                    const float P = base + rs;
                    const bool lt_y = !(P >= y);
                    below += lt_y ? 1 : 0;
                    prev = lt_y ? P : prev;
                };
                if (UNIFORM) {
                    for (int j = 0; j < T; ++j) visit(k0 + j < K ? 1.0f : 0.0f);
                } else if (VEC && TB > 0) {
                    auto reload = [&](auto whole) {
                        constexpr bool WHOLE = decltype(whole)::value;
                        for (int b = 0; b < nb; ++b) {
                            const int kb = k0 + 4 * TB * b;
                            float4 pv[TB > 0 ? TB : 1], tv[TB > 0 ? TB : 1];
#pragma unroll
                            for (int c = 0; c < TB; ++c) {
                                const bool in = WHOLE || kb + 4 * c < K;
                                pv[c] = in ? *reinterpret_cast<const float4*>(ph + kb + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
                                tv[c] = in ? *reinterpret_cast<const float4*>(th + kb + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
                            }
#pragma unroll
                            for (int c = 0; c < TB; ++c) {
                                visit(tv[c].x * pv[c].x);
                                visit(tv[c].y * pv[c].y);
                                visit(tv[c].z * pv[c].z);
                                visit(tv[c].w * pv[c].w);
                            }
                        }
                    };
                    if (nblk * T == K) reload(std::true_type{}); else reload(std::false_type{});
                } else if (VEC) {
                    for (int c = 0; c < T / 4; ++c) {
                        const int k = k0 + 4 * c;
                        if (k < K) {
                            const float4 x = *reinterpret_cast<const float4*>(ph + k);
                            const float4 t = *reinterpret_cast<const float4*>(th + k);
                            visit(t.x * x.x);
                            visit(t.y * x.y);
                            visit(t.z * x.z);
                            visit(t.w * x.w);
                        }
                    }
                } else {
                    for (int j = 0; j < T; ++j) {
                        const int k = k0 + j;
                        if (k < K) visit(th[k] * ph[k]);
                    }
                }
                const int kend = min(k0 + T, top) - 1;            // the block's last topic not yet passed
                const int k = max(min(k0 + below, kend), 0);
                SAME_COUNT(a, 3, 1);                               // block reloads
                // the step's topic, its top copy, and the binomial of the copies that share the topic
                const uint32_t Rm = R - 1u;
                const float width = y - prev;
                const float q = width / y;
                kk = k;
                bstep = step;
                U = prev; lt = l; top = k; step += 1u;
                if (Rm == 0u || !(q > 0.0f)) {
                    ek = k; en = 1u;
                    R = Rm;
                } else if (q >= 1.0f) {
                    ek = k; en = R;
                    R = 0;
                } else {
                    flip = q > 0.5f;
                    const float qq = flip ? 1.0f - q : q;
                    const float s1 = 1.0f - qq;
                    r = qq / s1;
                    lq = log1m(qq);
                    bR = Rm;
                    R = Rm;                                        // the binomial's share comes off when it is known
                    u = uniform_from_word(xb);
                    if (((float)Rm * qq) <= kPieceMean) {          // one piece of Rm trials
                        L = Rm;
                        const float pm0 = expneg((float)Rm * lq);
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
            if (pend != 0 && (__popcll((unsigned long long)pend) >= kPoolMin || !__any(st == 1 || (st == 0 && R > 0)))) {
                const uint32_t part = pool(pend);
                if (st == 3) {
                    const uint32_t nk = flip ? bR - part : part;
                    ek = kk; en = 1u + nk;
                    R -= nk;
                    st = 0;
                    SAME_COUNT(a, 5, 1);
                }
            }
        }
        if (__any(st == 1)) {
            const bool walking = st == 1;
            bool more = walking && !stalled && u > cdf && xw < L;
            for (int round = 0; round < kWalkRounds && __any(more); ++round) {
                if (lane == 0) SAME_COUNT(a, 12, 1);               // rounds of pmf terms
#pragma unroll
                for (int i = 0; i < kWalkSteps; ++i) {
                    const uint32_t xn = xw + 1u;
                    float pmn = pm * r;
                    pmn = pmn * (float)(L - xn + 1u);
                    pmn = pmn * inv_int((float)xn);
                    const float next_cdf = cdf + pmn;
                    const bool still = next_cdf == cdf;
                    if (more) SAME_COUNT(a, 4, 1);                 // pmf terms
                    xw = more ? xn : xw;
                    pm = more ? pmn : pm;
                    cdf = (more && !still) ? next_cdf : cdf;
                    stalled = stalled || (more && still);
                    more = more && !still && u > cdf && xw < L;
                }
            }
            if (walking && !more) {                                // the binomial is known
                const uint32_t nk = flip ? bR - xw : xw;
                ek = kk; en = 1u + nk;
                R -= nk;
                st = 0;
                SAME_COUNT(a, 5, 1);
            }
        }
        if (!DEBUG && !pool_dry) {
            // lanes whose slot (or chunk) is full go on in a new chunk: the wave hands out consecutive chunks of its
            // share of the pool and takes the next kChunkBatch from the pool's counter when they do not suffice
            const bool need = en > 0u && sc.full();
            const uint64_t need_mask = __ballot(need);
            if (need_mask != 0) {
                const uint32_t cnt = (uint32_t)__popcll((unsigned long long)need_mask);
                if (chunk_end - chunk_next < cnt) {
                    uint32_t first = 0;
                    if (lane == 0) first = atomicAdd(a.chunk_counter, (uint32_t)kChunkBatch);
                    first = (uint32_t)__builtin_amdgcn_readfirstlane((int)first);
                    pool_dry = first >= a.n_chunks;
                    chunk_next = pool_dry ? 0u : first;
                    chunk_end = pool_dry ? 0u : (a.n_chunks - first < (uint32_t)kChunkBatch ? a.n_chunks : first + (uint32_t)kChunkBatch);
                    if (lane == 0) SAME_COUNT(a, 14, 1);               // batches of chunks taken
                }
                const uint32_t mine = chunk_next + (uint32_t)__popcll((unsigned long long)(need_mask & ((1ull << lane) - 1ull)));
                if (need && mine < chunk_end) { sc.extend(a, mine, stage); SAME_COUNT(a, 15, 1); }
                chunk_next = chunk_end - chunk_next < cnt ? chunk_end : chunk_next + cnt;
            }
        }
#ifdef SAME_STATS
        if (en > 0u && sc.full()) {                                // a count that goes straight to the word's row
            const uint32_t g = R_task_g;
            SAME_COUNT(a, 16 + min(5, 31 - __clz((int)max(g, 1u))), 1);
            SAME_COUNT(a, 22 + (w < 16 ? 0 : w < 256 ? 1 : w < 4096 ? 2 : 3), 1);
        }
#endif
        if (en > 0u) {
            if (myrow >= 0) { atomicAdd(rows + myrow * K + ek, en); sc.emit_word(a, ek, en, stage); }
            else sc.emit(a, ek, en, stage);
        }
    };

    for (;;) {
        const uint64_t idle_mask = __ballot(st == 0 && R == 0);
        if (!drained && (__popcll((unsigned long long)idle_mask) >= kRefillMin || idle_mask == ~0ull)) {
            if (next >= end) {                                     // the next segment (all lanes obtain the same value)
                uint32_t first = 0;
                if (lane == 0) first = atomicAdd(a.counter, (uint32_t)kSegment);
                first = (uint32_t)__builtin_amdgcn_readfirstlane((int)first);
                drained = (int64_t)first >= a.n;
                next = drained ? 0 : (int32_t)first;
                end = drained ? 0 : (int32_t)((int64_t)first + kSegment < a.n ? (int64_t)first + kSegment : a.n);
            }
            if (next < end) {
                if (lane == 0) SAME_COUNT(a, 13, 1);               // refills
                refill(idle_mask);
                continue;
            }
        }
        if (idle_mask == ~0ull) break;                             // nothing in flight and nothing left to take
        trip();
    }
    if (open) sc.close(a, true, stage);
    if (n_rows > 0 && tag0 >= 0) flush_row(0, tag0);
    if (n_rows > 1 && tag1 >= 0) flush_row(1, tag1);
}

inline size_t draw_lds_bytes(int K) { return 4u * ((size_t)kWave * (size_t)(kSumStride + 3) + (size_t)doc_rows(K) * (size_t)K); }

}  // namespace same
