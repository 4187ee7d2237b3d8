// What the two draw kernels (multinomial form: draw_kernel.h, Poisson form: poisson_kernel.h) share:
// the launch arguments, the scatter of a task's counts (Algorithm 3, the two accumulation lines) and
// the kernel that adds the recorded (topic, count) pairs to the word rows.
#pragma once
#include "rng_binom.h"

namespace same {

#ifndef SAME_WALK_STEPS
#define SAME_WALK_STEPS 8
#endif
#ifndef SAME_POOL_MIN
#define SAME_POOL_MIN 8
#endif
constexpr int kWave = 64;               // lanes per workgroup (one wave)
constexpr int kPairWords = 16;          // words of a pair-list slot: up to 15 (topic, count) pairs and a header
constexpr uint32_t kPairLink = 0x80000000u;   // header bit: the slot is full and the chunk named by the other bits goes on
constexpr int kChunkBatch = 256;        // chunks a wave takes from the pool at a time
constexpr int kPairShift = 11;          // a pair is topic | count << 11 (topics < 2048, counts < 2^21)
constexpr int kWalkSteps = SAME_WALK_STEPS;   // pmf steps per trip of a draw machine
constexpr float kPieceMean = 32.0f;     // a binomial / Poisson variable whose mean exceeds this is cut into pieces
constexpr int kPoolMin = SAME_POOL_MIN; // waiting multi-piece variables that trigger a pass shared by the wave

struct DrawArgs {
    int64_t         n;          // tasks in this launch
    uint32_t*       counter;    // multinomial form: first launch position not yet taken by a workgroup (zero at launch)
    const int32_t*  t_doc;      // [n_tasks] document of the task
    const int32_t*  t_word;     // [n_tasks] word of the task
    const uint32_t* t_g;        // [n_tasks] tokens in the task's group
    const int32_t*  order;      // Poisson form: [n_tasks] task id handled at each launch position
    uint32_t*       cost;       // Poisson form: [n_tasks] out: trips this task was busy for (null: not recorded)
    const int64_t*  ids;        // debug launches: task ids to draw instead (else null)
    const float*    theta;      // [D][K]   (unused when weights are uniform)
    const float*    phi;        // [V][K]
    uint32_t*       ndk;        // [D][K]   (debug launches: [n][K] output rows)
    uint32_t*       nwk;        // [V][K] or null
    uint32_t*       pairs;      // [n_slots][kPairWords] pair list in word order, or null (update nwk directly)
    const int32_t*  t_slot;     // [n_tasks] slot of each task in the pair list, -1 for a task without one
    uint32_t*       chunks;     // [n_chunks][kPairWords] pool of chunks that continue full slots, or null
    uint32_t*       chunk_counter;  // first chunk of the pool not yet taken by a wave (zero at launch)
    uint32_t        n_chunks;   // chunks in the pool (below 2^31)
    int32_t         K;
    uint32_t        m;          // copies per token (multinomial form)
    float           mf;         // copies per token (Poisson form: any positive real)
    uint32_t        seed_lo, seed_hi, pass;
    int32_t         V;          // rows of nwk that are words; the copies of the hot words' rows follow them
    const int16_t*  hot_of;     // [V] index of a hot word among the hot words, -1 for the others (null: no hot words)
#ifdef SAME_STATS
    unsigned long long* stats;  // profiling builds only: event counters
#endif
};

#ifdef SAME_STATS
#define SAME_COUNT(a, i, v) do { if ((a).stats) atomicAdd((a).stats + (i), (unsigned long long)(v)); } while (0)
#else
#define SAME_COUNT(a, i, v) do { } while (0)
#endif

// Rows of [V][K] that very many tasks update at once (the most frequent words: their tasks spread copies
// over many topics, fill their pair-list slot and send the rest straight to the row) are a bottleneck of
// their own: atomics on a handful of lines are served by a handful of memory channels, one after the other.
// Such a word therefore gets kHotCopies private copies of its row behind the matrix; a workgroup adds to the
// copy picked by its index, and hot_fold_kernel adds the copies to the word's row afterwards.
constexpr int kHotMax = 256;            // words that may be hot (those holding at least 1/256 of all tokens)
constexpr int kHotCopies = 32;          // copies of a hot word's row

// Where the counts of one task go.  Every placed count goes to the document's row at once (an atomic:
// several waves may hold tasks of one document).  The word's row is updated either the same way or, when
// the launch has a pair list, later by word_reduce_kernel: the task records (topic, count) in its slot of
// the list (slots are in word order), so that the scattered updates of [V][K] become one streaming pass
// with all updates of a row close together.  A slot is 16 words: 15 pairs and, last, a header.  A task that
// places more than 15 pairs (most tasks do while the posterior is still flat) continues in chunks of the same
// shape taken from a pool: the header of a full slot or chunk names the chunk that follows it, the header of
// the last one holds its number of pairs.  When the pool is used up the remaining counts go straight to the
// word's row.  Pairs are collected in LDS (stage: this lane's three words, kWave words apart) and written four
// at a time, the fourth from its register, with one 16-byte store: the memory system handles a 16-byte write
// as fast as a 4-byte one.
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint32_t kInPool = 0x80000000u;   // Scatter::slot: the index is one of the pool's chunks, not of the pair list's slots

// The struct holds row and slot numbers, not addresses: a lane keeps it for the whole life of its task, and
// registers decide how many waves a compute unit holds.
struct Scatter {
    uint32_t drow;      // row of a.ndk that takes the counts (the document; debug launches: the task's output row)
    uint32_t wrow;      // row of a.nwk that takes direct updates (the word, or this workgroup's copy of a hot word's row), kNone: none
    uint32_t slot;      // the slot (or, with kInPool, the chunk) the task is filling, kNone: none
    uint32_t npairs;    // pairs in it

    __device__ __forceinline__ uint32_t* slot_words(const DrawArgs& a) const
    {
        uint32_t* base = (slot & kInPool) ? a.chunks : a.pairs;
        return base + (size_t)(slot & ~kInPool) * kPairWords;
    }
    // words 4q .. 4q+3 of the slot: the three staged words and a fourth
    __device__ __forceinline__ void store_quad(const DrawArgs& a, uint32_t q, const uint32_t* stage, uint32_t fourth) const
    {
        uint4 v;
        v.x = stage[0]; v.y = stage[kWave]; v.z = stage[2 * kWave]; v.w = fourth;
        *reinterpret_cast<uint4*>(slot_words(a) + 4u * q) = v;
    }
    __device__ __forceinline__ void emit(const DrawArgs& a, int k, uint32_t n, uint32_t* stage)
    {
        atomicAdd(a.ndk + (size_t)drow * a.K + k, n);
        emit_word(a, k, n, stage);
    }
    // the word's half alone (the caller has added the count to the document's row itself)
    __device__ __forceinline__ void emit_word(const DrawArgs& a, int k, uint32_t n, uint32_t* stage)
    {
        if (slot != kNone) {
            if (npairs < (uint32_t)(kPairWords - 1)) {
                const uint32_t j = npairs & 3u;
                const uint32_t pair = (uint32_t)k | (n << kPairShift);
                if (j == 3u) store_quad(a, npairs >> 2, stage, pair);   // pairs 0-3, 4-7 or 8-11
                else stage[j * kWave] = pair;
                npairs += 1;
            } else {
                atomicAdd(a.nwk + (size_t)wrow * a.K + k, n);      // full and no chunk to go on with: straight to the row
            }
        } else if (wrow != kNone) {
            atomicAdd(a.nwk + (size_t)wrow * a.K + k, n);
        }
    }
    __device__ __forceinline__ bool full() const { return slot != kNone && npairs >= (uint32_t)(kPairWords - 1); }
    // a full slot (pairs 12-14 are still staged) goes on in chunk idx of the pool
    __device__ __forceinline__ void extend(const DrawArgs& a, uint32_t idx, uint32_t* stage)
    {
        store_quad(a, 3u, stage, kPairLink | idx);
        slot = kInPool | idx;
        npairs = 0;
    }
    // the staged pairs and the header of the last slot or chunk: how many pairs it holds
    __device__ __forceinline__ void close(const DrawArgs& a, bool live, uint32_t* stage) const
    {
        if (slot != kNone && live) {
            const uint32_t q = npairs >> 2;
            if (q == 3u) {                                         // the header shares the last quad
                store_quad(a, 3u, stage, npairs);
            } else {
                if ((npairs & 3u) != 0u) store_quad(a, q, stage, 0u);   // words past the last pair are never read
                slot_words(a)[kPairWords - 1] = npairs;
            }
        }
    }
};

template <bool DEBUG>
__device__ __forceinline__ Scatter make_scatter(const DrawArgs& a, int64_t row, int64_t tau, int32_t d, int32_t w)
{
    Scatter s;
    s.drow = DEBUG ? (uint32_t)row : (uint32_t)d;
    s.wrow = kNone;
    s.slot = kNone;
    if (!DEBUG && a.nwk != nullptr) {
        const int hot = a.hot_of ? (int)a.hot_of[w] : -1;
        s.wrow = hot < 0 ? (uint32_t)w : (uint32_t)a.V + (uint32_t)(blockIdx.x % kHotCopies) * (uint32_t)kHotMax + (uint32_t)hot;
        if (a.pairs != nullptr) {
            const int32_t slot_id = a.t_slot[tau];
            if (slot_id >= 0) s.slot = (uint32_t)slot_id;
        }
    }
    s.npairs = 0;
    return s;
}

// Adds the copies of the hot words' rows (rows V .. V + kHotCopies*kHotMax of the matrix) to the words' own
// rows and clears them.  Runs alone on its stream after the draw and the pair-list reduction.
__global__ void hot_fold_kernel(uint32_t* __restrict__ nwk, const int32_t* __restrict__ hot_word, int n_hot, int V, int K)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_hot * K) return;
    const int hw = i / K, k = i - hw * K;
    uint32_t total = 0;
    for (int c = 0; c < kHotCopies; ++c) {
        uint32_t* p = nwk + ((size_t)V + (size_t)c * kHotMax + (size_t)hw) * K + k;
        total += *p;
        *p = 0u;
    }
    if (total) nwk[(size_t)hot_word[hw] * K + k] += total;
}

// Adds the recorded pairs to the word rows.  Slots are in word order and exist only for words with
// at least kSlotMinTasks tasks: a workgroup takes kReduceChunk consecutive slots, sums the pairs of
// the first `rows` words it meets in an LDS table and sends the rest straight to [V][K]; the table is
// then added to the rows it stands for.  A thread reads a slot with four 16-byte loads and starts with the
// quad picked by its index: tasks of one word have their large counts at the same topics in the same places
// of their slots, and aligned walks would meet at one address.
constexpr int kReduceChunk = 2048;
constexpr int kSlotMinTasks = 2;         // (32 measured 1.5 % slower on the resident matrix and 5 % on a minibatch: the direct
                                        // updates of rare words are atomics on lines that have long left the cache)
constexpr int kReduceThreads = 1024;    // two slots per thread: the kernel waits on its loads, many waves hide that

__global__ __launch_bounds__(kReduceThreads) void word_reduce_kernel(const uint32_t* __restrict__ pairs,
                                                          const uint32_t* __restrict__ chunks, uint32_t n_chunks,
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
        const uint32_t t = threadIdx.x & 3u;                       // which quad of the slot this thread starts with
        for (;;) {                                                 // the slot, then the chunks that continue it
            const uint4* __restrict__ s4 = reinterpret_cast<const uint4*>(src);
            uint4 q[4];                                            // the whole slot: four 16-byte loads in flight
#pragma unroll
            for (uint32_t i = 0; i < 4u; ++i) q[i] = s4[(t + i) & 3u];
            const uint32_t head = t == 0u ? q[3].w : (t == 1u ? q[2].w : (t == 2u ? q[1].w : q[0].w));
            const bool linked = (head & kPairLink) != 0u;
            const uint32_t cnt = (linked || head > (uint32_t)(kPairWords - 1)) ? (uint32_t)(kPairWords - 1) : head;
#pragma unroll
            for (uint32_t i = 0; i < 4u; ++i) {
                const uint32_t first = 4u * ((t + i) & 3u);        // index of the quad's first pair
                const uint32_t p[4] = {q[i].x, q[i].y, q[i].z, q[i].w};
#pragma unroll
                for (uint32_t j = 0; j < 4u; ++j)
                    if (first + j < cnt) atomicAdd(dst + (p[j] & ((1u << kPairShift) - 1u)), p[j] >> kPairShift);
            }
            if (!linked || (head & ~kPairLink) >= n_chunks) break;
            src = chunks + (size_t)(head & ~kPairLink) * kPairWords;
        }
    }
    __syncthreads();
    // A word whose slots all lie in this workgroup's range is updated by no other workgroup of this launch (and
    // nothing else runs beside the launch): its row takes plain additions.  Only the first and the last word of
    // the range may share their rows with the neighbours.
    const int32_t w1 = slot_word[s1 - 1];                          // the last word of the range
    const bool first_shared = s0 > 0 && slot_word[s0 - 1] == w0;
    const bool last_shared = s1 < n && slot_word[s1] == w1;
    uint32_t* base = nwk + (size_t)w0 * K;                         // row w0 + r, topic k is at base[r*K + k]
    for (int i = threadIdx.x; i < rows * K; i += blockDim.x) {
        const uint32_t v = tab[i];
        if (v == 0u) continue;                                     // only rows of real words hold counts
        const int32_t w = w0 + i / K;
        if ((w == w0 && first_shared) || (w == w1 && last_shared)) atomicAdd(base + i, v);
        else base[i] += v;
    }
}

inline int reduce_rows(int K) { const int r = 16384 / K; return r < 1 ? 1 : (r > 64 ? 64 : r); }

}  // namespace same
