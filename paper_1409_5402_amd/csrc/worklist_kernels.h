// Device-side construction of the draw work list from a CSC matrix (columns = documents).
//
// A nonzero (d, w, c) stands for c tokens with identical conditionals; its tokens are drawn in
// groups ("tasks") of at most G.  These kernels validate the matrix and produce, without a host
// copy of the matrix: the document of every nonzero, the tasks (document, word, group size) in
// storage order, the first task of every tile of documents, and the slots of the word-ordered pair
// list.  The exclusive sums and the stable sort by word that this takes are kernels of this file too.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace same {

// Filled by the kernels below; first_bad is the smallest (index << 2 | code) over all defects found,
// ~0 if the matrix is sound: code 1 = column pointer decreases (index = document), 2 = word id out
// of range, 3 = count not an integer in [1, 2^24) (index = nonzero).
struct BuildStats {
    unsigned long long tokens;
    unsigned long long n_tasks;
    unsigned long long first_bad;
    unsigned long long max_doc_tokens;     // largest number of tokens in one document, and that document
    unsigned long long max_word_tokens;    // largest number of tokens of one word, and that word
    uint32_t max_doc, max_word;
    uint32_t max_group;
    uint32_t n_slots;
    uint32_t n_hot;                        // words holding at least 1/kHotMax of all tokens
};

__global__ void wl_init_stats(BuildStats* s)
{
    s->tokens = 0ull; s->n_tasks = 0ull; s->first_bad = ~0ull; s->max_group = 0u; s->n_slots = 0u;
    s->max_doc_tokens = 0ull; s->max_word_tokens = 0ull; s->max_doc = ~0u; s->max_word = ~0u; s->n_hot = 0u;
}

// Token totals per document and per word (the largest values the count matrices can reach are m times
// these).  Only entries that passed validation are counted.  Words: one thread per nonzero adds to one of
// kTokenStripes copies of the per-word array (the most frequent words would otherwise receive one atomic per
// document on a single address); wl_word_totals then adds the copies.  Documents: one thread per document.
constexpr int kTokenStripes = 32;

__global__ __launch_bounds__(256) void wl_word_tokens(const int32_t* __restrict__ rowidx, const float* __restrict__ val,
                                                      int64_t nnz, int32_t V, unsigned long long* __restrict__ stripes)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    unsigned long long* mine = stripes + (size_t)(blockIdx.x % kTokenStripes) * V;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nnz; i += stride) {
        const int32_t w = rowidx[i];
        const float c = val[i];
        if (w < 0 || w >= V || !(c >= 1.0f) || c >= 16777216.0f) continue;
        atomicAdd(mine + w, (unsigned long long)c);
    }
}

// word_tok[w] = sum of the copies; the largest one goes to the statistics (one atomic per workgroup).
__global__ __launch_bounds__(256) void wl_word_totals(const unsigned long long* __restrict__ stripes, int32_t V,
                                                      unsigned long long* __restrict__ word_tok, BuildStats* s)
{
    __shared__ unsigned long long sh[256];
    const int32_t w = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    unsigned long long tot = 0ull;
    if (w < V) {
        for (int c = 0; c < kTokenStripes; ++c) tot += stripes[(size_t)c * V + w];
        word_tok[w] = tot;
    }
    sh[threadIdx.x] = tot;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] = sh[threadIdx.x] > sh[threadIdx.x + off] ? sh[threadIdx.x] : sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0 && sh[0]) atomicMax(&s->max_word_tokens, sh[0]);
}

__global__ __launch_bounds__(256) void wl_doc_tokens(const int32_t* __restrict__ colptr, const int32_t* __restrict__ rowidx,
                                                     const float* __restrict__ val, int32_t D, int32_t V,
                                                     unsigned long long* __restrict__ doc_tok, BuildStats* s)
{
    __shared__ unsigned long long sh[256];
    const int32_t d = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    unsigned long long tot = 0ull;
    if (d < D) {
        for (int64_t i = colptr[d]; i < (int64_t)colptr[d + 1]; ++i) {
            const int32_t w = rowidx[i];
            const float c = val[i];
            if (w < 0 || w >= V || !(c >= 1.0f) || c >= 16777216.0f) continue;
            tot += (unsigned long long)c;
        }
        doc_tok[d] = tot;
    }
    sh[threadIdx.x] = tot;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] = sh[threadIdx.x] > sh[threadIdx.x + off] ? sh[threadIdx.x] : sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0 && sh[0]) atomicMax(&s->max_doc_tokens, sh[0]);
}

// Hot words: those that hold at least one part in hot_max of all tokens (so at most hot_max of them).  They are
// numbered in the order the threads arrive; the numbering only names the copies of their rows, no result
// depends on it.  hot_of[w] = number or -1; hot_word[number] = w.
__global__ void wl_hot_words(const unsigned long long* __restrict__ word_tok, int32_t V, int32_t hot_max,
                             int16_t* __restrict__ hot_of, int32_t* __restrict__ hot_word, BuildStats* s)
{
    const int32_t w = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (w >= V) return;
    int16_t idx = -1;
    if (word_tok[w] > 0ull && word_tok[w] * (unsigned long long)hot_max >= s->tokens) {
        const uint32_t at = atomicAdd(&s->n_hot, 1u);
        if (at < (uint32_t)hot_max) { idx = (int16_t)at; hot_word[at] = w; }
    }
    hot_of[w] = idx;
}

// The lowest document and word ids that attain the two maxima (for the error message).
__global__ void wl_token_argmax(const unsigned long long* __restrict__ doc_tok, int32_t D,
                                const unsigned long long* __restrict__ word_tok, int32_t V, BuildStats* s)
{
    const int32_t i = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i < D && doc_tok[i] == s->max_doc_tokens) atomicMin(&s->max_doc, (uint32_t)i);
    if (i < V && word_tok[i] == s->max_word_tokens) atomicMin(&s->max_word, (uint32_t)i);
}

__global__ void wl_check_cols(const int32_t* __restrict__ colptr, int32_t D, BuildStats* s)
{
    const int32_t d = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (d < D && colptr[d + 1] < colptr[d]) atomicMin(&s->first_bad, ((unsigned long long)d << 2) | 1ull);
}

// Per nonzero: its document (the last d with colptr[d] <= i), validity, number of tasks.
// ntask has nnz + 1 entries; the last one is set to 0 so that an exclusive sum over all of them
// ends with the total.
__global__ __launch_bounds__(256) void wl_scan_nonzeros(const int32_t* __restrict__ colptr,
                                                        const int32_t* __restrict__ rowidx,
                                                        const float* __restrict__ val, int32_t D, int64_t nnz,
                                                        int32_t V, uint32_t G, int32_t* __restrict__ nz_doc,
                                                        uint32_t* __restrict__ ntask, BuildStats* s)
{
    __shared__ unsigned long long sh_tok[256], sh_task[256];
    __shared__ uint32_t sh_max[256];
    unsigned long long tok = 0ull, tasks = 0ull;
    uint32_t gmax = 0u;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i <= nnz; i += stride) {
        if (i == nnz) { ntask[i] = 0u; break; }
        int32_t lo = 0, hi = D;                                    // colptr[lo] <= i < colptr[hi] when sound
        while (hi - lo > 1) { const int32_t mid = lo + (hi - lo) / 2; if ((int64_t)colptr[mid] <= i) lo = mid; else hi = mid; }
        nz_doc[i] = lo;
        const int32_t w = rowidx[i];
        const float c = val[i];
        uint32_t nt = 0u;
        if (w < 0 || w >= V) {
            atomicMin(&s->first_bad, ((unsigned long long)i << 2) | 2ull);
        } else if (!(c >= 1.0f) || c >= 16777216.0f || c != floorf(c)) {
            atomicMin(&s->first_bad, ((unsigned long long)i << 2) | 3ull);
        } else {
            const uint32_t ci = (uint32_t)c;
            nt = (ci + G - 1u) / G;
            tok += ci; tasks += nt;
            gmax = max(gmax, ci < G ? ci : G);
        }
        ntask[i] = nt;
    }
    sh_tok[threadIdx.x] = tok; sh_task[threadIdx.x] = tasks; sh_max[threadIdx.x] = gmax;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) {
            sh_tok[threadIdx.x] += sh_tok[threadIdx.x + off];
            sh_task[threadIdx.x] += sh_task[threadIdx.x + off];
            sh_max[threadIdx.x] = max(sh_max[threadIdx.x], sh_max[threadIdx.x + off]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (sh_tok[0]) atomicAdd(&s->tokens, sh_tok[0]);
        if (sh_task[0]) atomicAdd(&s->n_tasks, sh_task[0]);
        if (sh_max[0]) atomicMax(&s->max_group, sh_max[0]);
    }
}

// The tasks of every nonzero, consecutive from tbase[i]; the processing order starts as storage order.
__global__ void wl_expand(const int32_t* __restrict__ nz_doc, const int32_t* __restrict__ rowidx,
                          const float* __restrict__ val, const uint32_t* __restrict__ tbase, int64_t nnz, uint32_t G,
                          int32_t* __restrict__ t_doc, int32_t* __restrict__ t_word, uint32_t* __restrict__ t_g,
                          int32_t* __restrict__ order, uint32_t* __restrict__ cost)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nnz; i += stride) {
        const uint32_t t0 = tbase[i], t1 = tbase[i + 1];
        const int32_t d = nz_doc[i], w = rowidx[i];
        uint32_t left = (uint32_t)val[i];
        for (uint32_t t = t0; t < t1; ++t) {
            const uint32_t g = left < G ? left : G;
            t_doc[t] = d; t_word[t] = w; t_g[t] = g;
            order[t] = (int32_t)t; cost[t] = 0u;
            left -= g;
        }
    }
}

// tile_start[T] = first task of document tile T (tile_docs documents per tile), n_tiles + 1 entries.
__global__ void wl_tiles(const int32_t* __restrict__ colptr, const uint32_t* __restrict__ tbase, int32_t D,
                         int32_t tile_docs, int32_t n_tiles, int32_t* __restrict__ tile_start)
{
    const int32_t T = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (T > n_tiles) return;
    const int64_t d = (int64_t)T * tile_docs;
    tile_start[T] = (int32_t)tbase[colptr[d < D ? d : D]];
}

// ---- Exclusive sum of 32-bit counts.  A workgroup owns a tile of kScanTile consecutive items.  One launch adds up
// every tile, the tile totals are summed the same way (recursively, until one tile is left), and a last launch
// per level writes the items' exclusive sums from the tile's base.  All sums are modulo 2^32 (the callers' totals
// stay below 2^31).
constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;                                     // consecutive items per thread
constexpr int kScanTile = kScanThreads * kScanItems;

// sum over the workgroup; every thread receives it
__device__ __forceinline__ uint32_t wl_block_sum(uint32_t v, uint32_t* sh /* [kScanThreads / 64] */)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t t = 0;
    for (int i = 0; i < kScanThreads / 64; ++i) t += sh[i];
    __syncthreads();
    return t;
}

__global__ __launch_bounds__(kScanThreads) void wl_tile_sums(const uint32_t* __restrict__ in, size_t n, uint32_t* __restrict__ tile_sum)
{
    __shared__ uint32_t sh[kScanThreads / 64];
    const size_t first = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    uint32_t v = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) if (first + j < n) v += in[first + j];
    const uint32_t t = wl_block_sum(v, sh);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = t;
}

// out[i] = tile_base[tile of i] + sum of the items of the tile before i (tile_base null: zero, a single tile)
__global__ __launch_bounds__(kScanThreads) void wl_tile_scan(const uint32_t* __restrict__ in, size_t n, const uint32_t* __restrict__ tile_base,
                                                            uint32_t* __restrict__ out)
{
    __shared__ uint32_t wave_total[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const size_t first = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    uint32_t x[kScanItems];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) { x[j] = first + j < n ? in[first + j] : 0u; mine += x[j]; }
    uint32_t incl = mine;                                          // inclusive sum over the wave's lanes
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    if (lane == 63) wave_total[wv] = incl;
    __syncthreads();
    uint32_t base = tile_base ? tile_base[blockIdx.x] : 0u;
    for (int i = 0; i < wv; ++i) base += wave_total[i];
    uint32_t run = base + incl - mine;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (first + j < n) out[first + j] = run;
        run += x[j];
    }
}

// ---- Stable radix sort of (key, value) pairs by 8-bit digits, least significant first.  A workgroup owns a tile of
// kSortTile consecutive items, wave v of it the items [v * 1024, (v + 1) * 1024) of the tile, read 64 at a time (a row).
// Per pass: wl_sort_histogram counts the tile's items per digit into hist[digit][tile]; the exclusive sum of hist
// in that order is where each tile's run of each digit starts in the output; wl_sort_scatter places the items: a
// lane's position is the start of its (digit, tile) run, plus the items of the same digit in the waves before its
// own, in the earlier rows of its wave, and in the lower lanes of its row.  Items keep their order inside a digit:
// the sort is stable, and the passes from the lowest digit up sort by the whole key.
constexpr int kSortThreads = 256;
constexpr int kSortRows = 16;                                     // rows of 64 items per wave
constexpr int kSortTile = kSortThreads * kSortRows;               // 4096 items
constexpr int kSortDigits = 256;
static_assert(kSortThreads == kSortDigits, "thread d of a workgroup owns digit d");

__global__ __launch_bounds__(kSortThreads) void wl_sort_histogram(const int32_t* __restrict__ keys, int64_t n, int shift, uint32_t n_tiles,
                                                                 uint32_t* __restrict__ hist)
{
    __shared__ uint32_t h[kSortDigits];
    h[threadIdx.x] = 0u;
    __syncthreads();
    const int64_t first = (int64_t)blockIdx.x * kSortTile;
    for (int j = 0; j < kSortRows; ++j) {
        const int64_t i = first + (int64_t)j * kSortThreads + threadIdx.x;
        if (i < n) atomicAdd(&h[((uint32_t)keys[i] >> shift) & (kSortDigits - 1)], 1u);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * n_tiles + blockIdx.x] = h[threadIdx.x];
}

// vals_in null: the value of item i is i (the first pass sorts the identity)
__global__ __launch_bounds__(kSortThreads) void wl_sort_scatter(const int32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in,
                                                                int64_t n, int shift, uint32_t n_tiles, const uint32_t* __restrict__ start,
                                                                int32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out)
{
    __shared__ uint32_t cnt[kSortThreads / 64][kSortDigits];      // per wave and digit: items, then the next output position
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int v = 0; v < kSortThreads / 64; ++v) cnt[v][threadIdx.x] = 0u;
    __syncthreads();
    const int64_t first = (int64_t)blockIdx.x * kSortTile + (int64_t)wv * (kSortRows * 64) + lane;
    int32_t key[kSortRows], val[kSortRows];
#pragma unroll
    for (int j = 0; j < kSortRows; ++j) {
        const int64_t i = first + (int64_t)j * 64;
        const bool in = i < n;
        key[j] = in ? keys_in[i] : 0;
        val[j] = in ? (vals_in ? vals_in[i] : (int32_t)i) : 0;
        if (in) atomicAdd(&cnt[wv][((uint32_t)key[j] >> shift) & (kSortDigits - 1)], 1u);
    }
    __syncthreads();
    {   // thread d: where the waves' items of digit d start
        uint32_t pos = start[(size_t)threadIdx.x * n_tiles + blockIdx.x];
        for (int v = 0; v < kSortThreads / 64; ++v) { const uint32_t c = cnt[v][threadIdx.x]; cnt[v][threadIdx.x] = pos; pos += c; }
    }
    __syncthreads();
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < kSortRows; ++j) {
        const bool in = first + (int64_t)j * 64 < n;
        const uint32_t dgt = ((uint32_t)key[j] >> shift) & (kSortDigits - 1);
        uint64_t peers = __ballot(in);                             // the lanes of this row that hold the same digit
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const bool one = (dgt >> bit) & 1u;
            const uint64_t m = __ballot(one);
            peers &= one ? m : ~m;
        }
        if (in) {
            const uint32_t rank = (uint32_t)__popcll((unsigned long long)(peers & below));
            const uint32_t pos = cnt[wv][dgt] + rank;              // every peer reads the position before the first one moves it on
            if (rank == 0u) cnt[wv][dgt] = pos + (uint32_t)__popcll((unsigned long long)peers);
            if ((int64_t)pos < n) {                                // always true; keeps a wrong count from becoming a wild store
                keys_out[pos] = key[j];
                vals_out[pos] = val[j];
            }
        }
    }
}

// wstart[w] = first position of word w in the word-sorted task list (n for words beyond the last), V + 1 entries.
__global__ void wl_word_starts(const int32_t* __restrict__ keys, int32_t n, int32_t V, int32_t* __restrict__ wstart)
{
    const int32_t w = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (w > V) return;
    int32_t lo = 0, hi = n;                                        // first position with keys[pos] >= w
    while (lo < hi) { const int32_t mid = lo + (hi - lo) / 2; if (keys[mid] < w) lo = mid + 1; else hi = mid; }
    wstart[w] = lo;
}

// flag[i] = 1 if the word at sorted position i has at least min_tasks tasks (its tasks get slots).
__global__ void wl_slot_flags(const int32_t* __restrict__ keys, const int32_t* __restrict__ wstart, int64_t n,
                              int32_t min_tasks, uint32_t* __restrict__ flag)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i <= n; i += stride) {
        if (i == n) { flag[i] = 0u; break; }
        const int32_t w = keys[i];
        flag[i] = (wstart[w + 1] - wstart[w] >= min_tasks) ? 1u : 0u;
    }
}

// Slots in (word, task id) order: pos is the exclusive sum of flag (n + 1 entries, the last = number of slots).
__global__ void wl_slot_scatter(const int32_t* __restrict__ keys, const int32_t* __restrict__ tasks,
                                const uint32_t* __restrict__ flag, const uint32_t* __restrict__ pos, int64_t n,
                                int32_t* __restrict__ t_slot, int32_t* __restrict__ slot_word, BuildStats* s)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (flag[i]) { t_slot[tasks[i]] = (int32_t)pos[i]; slot_word[pos[i]] = keys[i]; }
        else t_slot[tasks[i]] = -1;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) s->n_slots = pos[n];
}

}  // namespace same
