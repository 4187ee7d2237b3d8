// Host side of the SAME LDA library: handle, validation, work-list construction, launches.
// Exports the C ABI declared in include/same_lda.h.
#include "../../include/same_lda.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "draw_kernel.h"
#include "gamma_kernels.h"
#include "poisson_kernel.h"
#include "update_kernels.h"
#include "vb_kernels.h"
#include "worklist_kernels.h"

namespace {

thread_local std::string g_init_error;

constexpr int32_t kTileDocs = 16;   // documents per tile of the processing order
#ifndef SAME_GRID_PER_CU
#define SAME_GRID_PER_CU 16
#endif
constexpr int64_t kDrawGrid = 256 * SAME_GRID_PER_CU;   // workgroups of the multinomial draw kernel: as many as are resident at once (sixteen waves per compute unit)
constexpr int kGammaRows = 64;      // rows of n_wk per workgroup of the sampled phi step

// Device copy of one sparse matrix plus its draw work list.
struct Matrix {
    int32_t D = 0;
    int64_t nnz = 0, n_tasks = 0;
    uint32_t max_group = 0;        // largest number of tokens in one task
    uint64_t max_doc_tokens = 0, max_word_tokens = 0;   // largest token total of one document / of one word
    int32_t max_doc = -1, max_word = -1;                // and where they occur
    bool with_words = false;       // its draws also accumulate word counts (a training matrix)
    double tokens = 0.0;
    int32_t*  t_doc = nullptr;     // [n_tasks]
    int32_t*  t_word = nullptr;    // [n_tasks]
    uint32_t* t_g = nullptr;       // [n_tasks]
    int32_t*  order = nullptr;     // [n_tasks] task id processed at each launch position
    int32_t*  tile_start = nullptr;// [n_tiles+1] first task id of every document tile
    uint32_t* cost = nullptr;      // [n_tasks] drain work each task reported in the last pass
    int32_t   n_tiles = 0;
    int32_t*  colptr = nullptr;    // [D+1]
    int32_t*  nz_doc = nullptr;    // [nnz]
    int32_t*  rowidx = nullptr;    // [nnz]
    float*    val = nullptr;       // [nnz]
    float*    theta = nullptr;     // [D][K]
    uint32_t* ndk = nullptr;       // [D][K]
    // pair list of the word-count update (training matrices only; absent if it did not fit)
    uint32_t* pairs = nullptr;     // [n_tasks][kPairWords]
    int64_t   n_slots = 0;         // tasks of frequent words, each with a slot
    int32_t*  t_slot = nullptr;    // [n_tasks] slot of each task (rank in (word, task id) order), -1 if none
    int32_t*  slot_word = nullptr; // [n_slots] word of each slot
    // hot words (training matrices only): their rows of the word-count matrix have private copies
    int16_t*  hot_of = nullptr;    // [V] number of a hot word, -1 for the others
    int32_t*  hot_word = nullptr;  // [kHotMax] the hot words by number
    int32_t   n_hot = 0;
};

}  // namespace

// Device blocks handed back by the library's own buffers are kept for the next request of similar
// size instead of being freed: a stream of minibatches then allocates nothing after its first steps
// (hipFree waits for the whole device).  Blocks are only put back once no enqueued work uses them.
struct BlockCache {
    std::unordered_map<void*, size_t> live;      // blocks handed out, with their size
    std::multimap<size_t, void*> spare;          // blocks waiting for reuse, by size
    size_t spare_bytes = 0, limit = (size_t)1 << 30;

    hipError_t get(void** p, size_t bytes)
    {
        bytes = (bytes + 255) & ~(size_t)255;
        if (bytes == 0) bytes = 256;
        auto it = spare.lower_bound(bytes);
        if (it != spare.end() && it->first <= 2 * bytes + 4096) {
            *p = it->second; live[*p] = it->first; spare_bytes -= it->first; spare.erase(it);
            return hipSuccess;
        }
        hipError_t e = hipMalloc(p, bytes);
        if (e != hipSuccess && !spare.empty()) {                   // give the spare blocks back and try again
            (void)hipGetLastError();
            clear_spare();
            e = hipMalloc(p, bytes);
        }
        if (e == hipSuccess) live[*p] = bytes;
        return e;
    }
    void put(void* p)
    {
        if (!p) return;
        auto it = live.find(p);
        if (it == live.end()) { hipFree(p); return; }
        spare.emplace(it->second, p); spare_bytes += it->second; live.erase(it);
        while (spare_bytes > limit && !spare.empty()) {            // drop the smallest blocks first
            auto sm = spare.begin();
            spare_bytes -= sm->first; hipFree(sm->second); spare.erase(sm);
        }
    }
    void clear_spare()
    {
        for (auto& kv : spare) hipFree(kv.second);
        spare.clear(); spare_bytes = 0;
    }
};

struct same_lda {
    int32_t V = 0, K = 0, G = 0;
    BlockCache cache;
    float alpha = 0.f, beta = 0.f;
    uint64_t seed = 0;
    int32_t pass = 0;              // next pass index of the training stream
    hipStream_t stream = nullptr;
    Matrix X;
    // the next minibatch, prepared on a second stream while the current one is swept
    Matrix staged;
    bool has_staged = false;
    int32_t staged_pass = 0;       // pass index its initial pass was drawn with
    int32_t staged_m = 0;
    hipStream_t copy_stream = nullptr;
    float* phi = nullptr;          // [V][K]
    uint32_t* nwk = nullptr;       // [V][K]
    unsigned long long* nk = nullptr;  // [K]
    uint32_t* draw_counter = nullptr;  // [3] counters of the draw kernel: segments and chunks taken by a launch on the handle's
                                       // stream, segments taken by a launch on the copy stream
    uint32_t* chunks = nullptr;        // pool of chunks that continue full pair-list slots (launches on the handle's stream)
    uint32_t n_chunks = 0;             // chunks allocated
    int64_t chunk_limit = -1;          // chunks a launch may use (-1: all of them); lowered by tests of the fallback
    double* gamma_partial = nullptr;   // [ceil(V / kGammaRows)][K] block sums of the sampled phi step
    float* gamma_total = nullptr;      // [K]
    double* vb_psi = nullptr;          // [K] psi of the column sums of lambda (variational E-step)
    bool timing = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> events;   // recorded, not yet read
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;     // free event pairs
    std::string error;
};

namespace {

int fail(same_lda* h, int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (h) h->error = buf; else g_init_error = buf;
    return code;
}

#define HIP_TRY(h, expr)                                                                         \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail(h, e_ == hipErrorOutOfMemory ? SAME_LDA_ENOMEM : SAME_LDA_EHIP,          \
                        "%s: %s", #expr, hipGetErrorString(e_));                                 \
    } while (0)

template <class T>
int dev_alloc(same_lda* h, T** p, size_t n)
{
    *p = nullptr;
    if (n == 0) return SAME_LDA_OK;
    HIP_TRY(h, h->cache.get(reinterpret_cast<void**>(p), n * sizeof(T)));
    return SAME_LDA_OK;
}

template <class T>
void dev_free(same_lda* h, T*& p)
{
    h->cache.put(p);
    p = nullptr;
}

// Only after every launch that uses M has completed.
void free_matrix(same_lda* h, Matrix& M)
{
    dev_free(h, M.colptr); dev_free(h, M.t_doc); dev_free(h, M.t_word); dev_free(h, M.t_g); dev_free(h, M.order);
    dev_free(h, M.tile_start); dev_free(h, M.cost); dev_free(h, M.nz_doc); dev_free(h, M.rowidx); dev_free(h, M.val);
    dev_free(h, M.theta); dev_free(h, M.ndk); dev_free(h, M.pairs); dev_free(h, M.t_slot); dev_free(h, M.slot_word);
    dev_free(h, M.hot_of); dev_free(h, M.hot_word);
    M = Matrix();
}

int grid_for(size_t n, int threads = 256, int cap = 256 * 32);

// Device temporaries of one build, handed back together at the end (after the build's stream has
// been waited for).
struct Temps {
    same_lda* h;
    hipStream_t st;
    std::vector<void*> ptrs;
    Temps(same_lda* handle, hipStream_t stream) : h(handle), st(stream) {}
    template <class T> hipError_t get(T** p, size_t n)
    {
        *p = nullptr;
        void* v = nullptr;
        const hipError_t e = h->cache.get(&v, (n ? n : 1) * sizeof(T));
        if (e == hipSuccess) { ptrs.push_back(v); *p = static_cast<T*>(v); }
        return e;
    }
    ~Temps() { (void)hipStreamSynchronize(st); for (void* v : ptrs) h->cache.put(v); }
};

// out[i] = in[0] + ... + in[i-1] for n items (worklist_kernels.h): tile totals, their exclusive sum by the same
// steps, then the tiles.  Temporaries come from tmp and are handed back with it.
hipError_t exclusive_sum(Temps& tmp, const uint32_t* in, uint32_t* out, size_t n, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    const size_t tiles = (n + same::kScanTile - 1) / same::kScanTile;
    uint32_t* tile_base = nullptr;
    if (tiles > 1) {
        uint32_t* tile_sum = nullptr;
        hipError_t e = tmp.get(&tile_sum, tiles);
        if (e == hipSuccess) e = tmp.get(&tile_base, tiles);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(same::wl_tile_sums, dim3((unsigned)tiles), dim3(same::kScanThreads), 0, st, in, n, tile_sum);
        e = exclusive_sum(tmp, tile_sum, tile_base, tiles, st);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(same::wl_tile_scan, dim3((unsigned)tiles), dim3(same::kScanThreads), 0, st, in, n, tile_base, out);
    return hipGetLastError();
}

// The pool of chunks that continue full pair-list slots (scatter.h).  A task places at most K pairs, 15 of them in
// its slot; eight chunks per slot cover a sweep from a flat posterior (a hundred copies of a token then reach some
// eighty topics), and a sweep that needs more sends the rest straight to the word rows.  The pool never takes more
// than a quarter of the free device memory.  A failed allocation leaves the handle without a pool.
void ensure_chunks(same_lda* h, int64_t n_slots)
{
    const int64_t per_slot_most = ((int64_t)h->K - 1) / (same::kPairWords - 1);      // ceil((K - 15) / 15), 0 up to K = 15
    const int64_t per_slot = per_slot_most < 8 ? per_slot_most : 8;
    int64_t want = n_slots * per_slot;
    if (want > 0) want += 64 * (int64_t)same::kChunkBatch;                            // unused ends of the waves' shares
    if (want > 0x7FFFFFFF) want = 0x7FFFFFFF;
    if (want <= (int64_t)h->n_chunks) return;
    want += want / 4;                                                                 // minibatches differ in size
    if (want > 0x7FFFFFFF) want = 0x7FFFFFFF;
    if (h->chunks) {
        // a sweep that is still running on the handle's stream (this may be the build of a staged minibatch on the
        // other stream) reads and writes the pool: it ends before the pool is replaced
        (void)hipStreamSynchronize(h->stream);
        (void)hipFree(h->chunks); h->chunks = nullptr; h->n_chunks = 0;
    }
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) { (void)hipGetLastError(); return; }
    const size_t chunk_bytes = (size_t)same::kPairWords * sizeof(uint32_t);
    if ((size_t)want > free_b / 4 / chunk_bytes) want = (int64_t)(free_b / 4 / chunk_bytes);
    if (want <= 0) return;
    void* p = nullptr;
    if (hipMalloc(&p, (size_t)want * chunk_bytes) != hipSuccess) { (void)hipGetLastError(); return; }
    h->chunks = static_cast<uint32_t*>(p);
    h->n_chunks = (uint32_t)want;
}

// Validates the matrix and builds its work list on the device (worklist_kernels.h).  The matrix may
// live on the host or on the device; it is copied once.  All work is enqueued on st; the call
// waits for st twice (to learn the number of tasks and of pair-list slots).
int build_matrix(same_lda* h, const same_lda_csc* X, int32_t V, int32_t K, int32_t G, Matrix& M, hipStream_t st,
                 bool with_pairs)
{
    if (!X) return fail(h, SAME_LDA_EINVAL, "matrix is null");
    if (X->D < 0 || X->V != V || X->nnz < 0 || X->nnz >= (int64_t)1 << 31)
        return fail(h, SAME_LDA_EINVAL, "bad matrix shape D=%d V=%d (expected V=%d) nnz=%lld", X->D, X->V, V,
                    (long long)X->nnz);
    if (!X->colptr || (X->nnz > 0 && (!X->rowidx || !X->val)))
        return fail(h, SAME_LDA_EINVAL, "matrix arrays are null");
    const int32_t D = X->D;
    const int64_t nnz = X->nnz;
    const hipMemcpyKind kind = X->on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    int32_t ends[2] = {0, 0};
    if (X->on_device) {
        HIP_TRY(h, hipMemcpy(&ends[0], X->colptr, 4, hipMemcpyDeviceToHost));
        HIP_TRY(h, hipMemcpy(&ends[1], X->colptr + D, 4, hipMemcpyDeviceToHost));
    } else {
        ends[0] = X->colptr[0]; ends[1] = X->colptr[D];
    }
    if (ends[0] != 0 || (int64_t)ends[1] != nnz)
        return fail(h, SAME_LDA_ECSC, "colptr[0]=%d colptr[D]=%d do not match nnz=%lld", ends[0], ends[1], (long long)nnz);

    M.D = D; M.nnz = nnz;
    int rc;
    if ((rc = dev_alloc(h, &M.colptr, (size_t)D + 1))) return rc;
    if ((rc = dev_alloc(h, &M.nz_doc, (size_t)nnz))) return rc;
    if ((rc = dev_alloc(h, &M.rowidx, (size_t)nnz))) return rc;
    if ((rc = dev_alloc(h, &M.val, (size_t)nnz))) return rc;
    HIP_TRY(h, hipMemcpyAsync(M.colptr, X->colptr, ((size_t)D + 1) * 4, kind, st));
    if (nnz) {
        HIP_TRY(h, hipMemcpyAsync(M.rowidx, X->rowidx, (size_t)nnz * 4, kind, st));
        HIP_TRY(h, hipMemcpyAsync(M.val, X->val, (size_t)nnz * 4, kind, st));
    }

    Temps tmp(h, st);
    same::BuildStats* d_stats = nullptr;
    uint32_t *ntask = nullptr, *tbase = nullptr;
    HIP_TRY(h, tmp.get(&d_stats, 1));
    HIP_TRY(h, tmp.get(&ntask, (size_t)nnz + 1));
    HIP_TRY(h, tmp.get(&tbase, (size_t)nnz + 1));
    hipLaunchKernelGGL(same::wl_init_stats, dim3(1), dim3(1), 0, st, d_stats);
    if (D > 0) hipLaunchKernelGGL(same::wl_check_cols, dim3((unsigned)((D + 255) / 256)), dim3(256), 0, st, M.colptr, D, d_stats);
    hipLaunchKernelGGL(same::wl_scan_nonzeros, dim3(grid_for((size_t)nnz + 1)), dim3(256), 0, st, M.colptr, M.rowidx,
                       M.val, D, nnz, V, (uint32_t)G, M.nz_doc, ntask, d_stats);
    // token totals per document and per word: they bound what the 32-bit count matrices must hold
    unsigned long long *doc_tok = nullptr, *word_tok = nullptr, *stripes = nullptr;
    HIP_TRY(h, tmp.get(&doc_tok, (size_t)D));
    HIP_TRY(h, tmp.get(&word_tok, (size_t)V));
    HIP_TRY(h, tmp.get(&stripes, (size_t)V * same::kTokenStripes));
    hipLaunchKernelGGL(same::zero_u64_kernel, dim3(grid_for((size_t)V * same::kTokenStripes)), dim3(256), 0, st, stripes,
                       (size_t)V * same::kTokenStripes);
    if (nnz > 0)
        hipLaunchKernelGGL(same::wl_word_tokens, dim3(grid_for((size_t)nnz)), dim3(256), 0, st, M.rowidx, M.val, nnz, V, stripes);
    hipLaunchKernelGGL(same::wl_word_totals, dim3((unsigned)((V + 255) / 256)), dim3(256), 0, st, stripes, V, word_tok, d_stats);
    if (D > 0) {
        hipLaunchKernelGGL(same::wl_doc_tokens, dim3((unsigned)((D + 255) / 256)), dim3(256), 0, st, M.colptr, M.rowidx,
                           M.val, D, V, doc_tok, d_stats);
        const int32_t most = D > V ? D : V;
        hipLaunchKernelGGL(same::wl_token_argmax, dim3((unsigned)((most + 255) / 256)), dim3(256), 0, st, doc_tok, D,
                           word_tok, V, d_stats);
        if (with_pairs) {                                      // the words whose rows get private copies (scatter.h)
            if ((rc = dev_alloc(h, &M.hot_of, (size_t)V))) return rc;
            if ((rc = dev_alloc(h, &M.hot_word, (size_t)same::kHotMax))) return rc;
            hipLaunchKernelGGL(same::wl_hot_words, dim3((unsigned)((V + 255) / 256)), dim3(256), 0, st, word_tok, V,
                               (int32_t)same::kHotMax, M.hot_of, M.hot_word, d_stats);
        }
    }
    HIP_TRY(h, hipGetLastError());
    same::BuildStats stats;
    HIP_TRY(h, hipMemcpyAsync(&stats, d_stats, sizeof(stats), hipMemcpyDeviceToHost, st));
    HIP_TRY(h, hipStreamSynchronize(st));
    if (stats.first_bad != ~0ull) {
        const long long where = (long long)(stats.first_bad >> 2);
        switch ((int)(stats.first_bad & 3ull)) {
            case 1:  return fail(h, SAME_LDA_ECSC, "colptr decreases at document %lld", where);
            case 2:  return fail(h, SAME_LDA_ECSC, "word id out of range at entry %lld", where);
            default: return fail(h, SAME_LDA_ECSC, "count at entry %lld is not an integer in [1, 2^24)", where);
        }
    }
    if (stats.n_tasks >= (1ull << 31))
        return fail(h, SAME_LDA_ECSC, "too many draw tasks (%llu); raise tokens_per_draw", stats.n_tasks);
    const size_t n = (size_t)stats.n_tasks;
    M.n_tasks = (int64_t)n; M.max_group = stats.max_group; M.tokens = (double)stats.tokens;
    M.max_doc_tokens = stats.max_doc_tokens; M.max_word_tokens = stats.max_word_tokens;
    M.max_doc = (int32_t)stats.max_doc; M.max_word = (int32_t)stats.max_word;
    M.n_hot = M.hot_of ? (int32_t)(stats.n_hot < (uint32_t)same::kHotMax ? stats.n_hot : (uint32_t)same::kHotMax) : 0;
    M.with_words = with_pairs;

    // Processing order: documents are taken in tiles of kTileDocs (the theta rows a wave touches stay
    // within one small tile); inside a tile the order starts as storage order and is re-sorted before
    // every sweep by the cost each task reported in the previous pass, so that the 64 lanes of a wave
    // run chains of similar length.  The order does not affect results: tasks are independent and
    // keyed by their id.
    M.n_tiles = (D + kTileDocs - 1) / kTileDocs;
    if ((rc = dev_alloc(h, &M.t_doc, n))) return rc;
    if ((rc = dev_alloc(h, &M.t_word, n))) return rc;
    if ((rc = dev_alloc(h, &M.t_g, n))) return rc;
    if ((rc = dev_alloc(h, &M.order, n))) return rc;
    if ((rc = dev_alloc(h, &M.cost, n))) return rc;
    if ((rc = dev_alloc(h, &M.tile_start, (size_t)M.n_tiles + 1))) return rc;
    if ((rc = dev_alloc(h, &M.theta, (size_t)D * K))) return rc;
    if ((rc = dev_alloc(h, &M.ndk, (size_t)D * K))) return rc;
    HIP_TRY(h, exclusive_sum(tmp, ntask, tbase, (size_t)nnz + 1, st));
    if (nnz)
        hipLaunchKernelGGL(same::wl_expand, dim3(grid_for((size_t)nnz)), dim3(256), 0, st, M.nz_doc, M.rowidx, M.val,
                           tbase, nnz, (uint32_t)G, M.t_doc, M.t_word, M.t_g, M.order, M.cost);
    hipLaunchKernelGGL(same::wl_tiles, dim3((unsigned)((M.n_tiles + 256) / 256)), dim3(256), 0, st, M.colptr, tbase, D,
                       kTileDocs, M.n_tiles, M.tile_start);
    HIP_TRY(h, hipGetLastError());

    // Pair list: slots in (word, task id) order for the tasks of frequent words: a stable radix sort of the tasks
    // by word (worklist_kernels.h), the words' ranges in the sorted list, a flag per task of a word with enough
    // tasks, the flags' exclusive sum.  Optional: without it the draw kernel updates the word rows directly.
    if (with_pairs && n > 0) {
        int bits = 1;
        while (((int64_t)1 << bits) < (int64_t)V) ++bits;
        const uint32_t tiles = (uint32_t)((n + same::kSortTile - 1) / same::kSortTile);
        const size_t cells = (size_t)same::kSortDigits * tiles;
        int32_t *kbuf[2] = {nullptr, nullptr}, *vbuf[2] = {nullptr, nullptr}, *wstart = nullptr;
        uint32_t *hist = nullptr, *hstart = nullptr, *flag = nullptr, *pos = nullptr;
        bool ok = tmp.get(&kbuf[0], n) == hipSuccess && tmp.get(&kbuf[1], n) == hipSuccess &&
                  tmp.get(&vbuf[0], n) == hipSuccess && tmp.get(&vbuf[1], n) == hipSuccess &&
                  tmp.get(&hist, cells) == hipSuccess && tmp.get(&hstart, cells) == hipSuccess &&
                  tmp.get(&wstart, (size_t)V + 1) == hipSuccess && tmp.get(&flag, n + 1) == hipSuccess &&
                  tmp.get(&pos, n + 1) == hipSuccess &&
                  h->cache.get(reinterpret_cast<void**>(&M.t_slot), n * 4) == hipSuccess &&
                  h->cache.get(reinterpret_cast<void**>(&M.slot_word), n * 4) == hipSuccess;
        if (ok) {
            const int32_t* kin = M.t_word;                         // the first pass reads the tasks' words and numbers them itself
            const int32_t* vin = nullptr;
            int to = 0;
            for (int shift = 0; shift < bits; shift += 8, to ^= 1) {
                hipLaunchKernelGGL(same::wl_sort_histogram, dim3(tiles), dim3(same::kSortThreads), 0, st, kin, (int64_t)n, shift, tiles, hist);
                HIP_TRY(h, exclusive_sum(tmp, hist, hstart, cells, st));
                hipLaunchKernelGGL(same::wl_sort_scatter, dim3(tiles), dim3(same::kSortThreads), 0, st, kin, vin, (int64_t)n, shift, tiles,
                                   hstart, kbuf[to], vbuf[to]);
                kin = kbuf[to]; vin = vbuf[to];
            }
            const int32_t* keys = kin;                             // words in ascending order, tasks of a word in task order
            const int32_t* tasks = vin;
            hipLaunchKernelGGL(same::wl_word_starts, dim3((unsigned)((V + 256) / 256)), dim3(256), 0, st, keys,
                               (int32_t)n, V, wstart);
            hipLaunchKernelGGL(same::wl_slot_flags, dim3(grid_for(n + 1)), dim3(256), 0, st, keys, wstart, (int64_t)n,
                               (int32_t)same::kSlotMinTasks, flag);
            HIP_TRY(h, exclusive_sum(tmp, flag, pos, n + 1, st));
            hipLaunchKernelGGL(same::wl_slot_scatter, dim3(grid_for(n)), dim3(256), 0, st, keys, tasks, flag, pos,
                               (int64_t)n, M.t_slot, M.slot_word, d_stats);
            HIP_TRY(h, hipGetLastError());
            HIP_TRY(h, hipMemcpyAsync(&stats, d_stats, sizeof(stats), hipMemcpyDeviceToHost, st));
            HIP_TRY(h, hipStreamSynchronize(st));
            M.n_slots = (int64_t)stats.n_slots;
            ok = M.n_slots > 0 &&
                 h->cache.get(reinterpret_cast<void**>(&M.pairs), (size_t)M.n_slots * same::kPairWords * sizeof(uint32_t)) == hipSuccess;
            if (ok) ensure_chunks(h, M.n_slots);
        }
        if (!ok) {
            (void)hipGetLastError();
            dev_free(h, M.pairs); dev_free(h, M.t_slot); dev_free(h, M.slot_word);
            M.n_slots = 0;
        }
    }
    HIP_TRY(h, hipStreamSynchronize(st));   // the temporaries are handed back on return
    // blocks worth keeping for the next matrix of this size: the matrix itself and the temporaries
    const size_t matrix_bytes = (size_t)nnz * 12 + n * 28 + (size_t)M.n_slots * 68 + (size_t)D * K * 8;
    if (h->cache.limit < 2 * matrix_bytes + ((size_t)1 << 30)) h->cache.limit = 2 * matrix_bytes + ((size_t)1 << 30);
    return SAME_LDA_OK;
}

int grid_for(size_t n, int threads, int cap)
{
    size_t g = (n + (size_t)threads - 1) / (size_t)threads;
    if (g < 1) g = 1;
    if (g > (size_t)cap) g = (size_t)cap;
    return (int)g;
}

// Copies per token of one pass: an integer (multinomial form) or a positive real (Poisson form).
struct Copies {
    uint32_t m = 1;
    float mf = 1.0f;
    bool poisson = false;
    static Copies whole(uint32_t m) { Copies c; c.m = m; c.mf = (float)m; return c; }
    static Copies real(float mf) { Copies c; c.m = 0; c.mf = mf; c.poisson = true; return c; }
};

// The count matrices are 32-bit: n_dk[d][k] can reach m * (tokens of document d) and n_wk[w][k]
// m * (tokens of word w) when one topic takes them all.  A pass places at most most * tokens + extra copies
// of a document or word (most = m, extra = 0 in the multinomial form; margins above the mean in the
// Poisson form, whose totals are random).
int check_accumulators(same_lda* h, double most, double extra, const Matrix& M)
{
    const double limit = 4294967296.0;
    if (most * (double)M.max_doc_tokens + extra >= limit)
        return fail(h, SAME_LDA_ECSC, "m * tokens of document %d = %g * %llu does not fit the 32-bit counts", M.max_doc,
                    most, (unsigned long long)M.max_doc_tokens);
    if (M.with_words && most * (double)M.max_word_tokens + extra >= limit)
        return fail(h, SAME_LDA_ECSC, "m * tokens of word %d = %g * %llu does not fit the 32-bit counts", M.max_word,
                    most, (unsigned long long)M.max_word_tokens);
    return SAME_LDA_OK;
}

int check_mf(same_lda* h, float m, const Matrix& M)
{
    if (!(m > 0.0f) || !std::isfinite(m)) return fail(h, SAME_LDA_EINVAL, "m must be a positive number (got %g)", (double)m);
    if ((double)m * (double)(M.max_group ? M.max_group : 1u) >= 4194304.0)
        return fail(h, SAME_LDA_ECSC, "m * largest token group = %g * %u must stay below 2^22", (double)m, M.max_group);
    // a Poisson total exceeds its mean: one percent and 2^16 copies above it are beyond any total that occurs
    return check_accumulators(h, 1.01 * (double)m, 65536.0, M);
}

int check_m(same_lda* h, int32_t m, const Matrix& M)
{
    if (m < 1) return fail(h, SAME_LDA_EINVAL, "m must be >= 1 (got %d)", m);
    if ((uint64_t)m * (uint64_t)(M.max_group ? M.max_group : 1u) >= (1ull << 24))
        return fail(h, SAME_LDA_ECSC, "m * largest token group = %d * %u must stay below 2^24", m, M.max_group);
    return check_accumulators(h, (double)m, 0.0, M);
}

// The multinomial kernel's counters for a launch on st, set to zero on st (a launch of its own, so that the
// events around the draw kernel bracket that kernel alone).  Launches on the copy stream have no pair list and
// therefore no use for the chunk pool: they run beside launches on the handle's stream, which own it.
int prepare_counter(same_lda* h, same::DrawArgs& a, hipStream_t st)
{
    const bool beside = st == h->copy_stream && st != h->stream;
    a.counter = beside ? h->draw_counter + 2 : h->draw_counter;
    a.chunk_counter = h->draw_counter + 1;
    if (beside || !a.pairs) { a.chunks = nullptr; a.n_chunks = 0; }
    hipLaunchKernelGGL(same::zero_u32_kernel, dim3(1), dim3(64), 0, st, a.counter, (size_t)(beside ? 1 : 2));
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

template <bool DEBUG>
int launch_draw(same_lda* h, const same::DrawArgs& a, bool uniform, bool poisson, hipStream_t st)
{
    if (a.n <= 0) return SAME_LDA_OK;
    const int T = same::kWave;
    dim3 block((unsigned)T);
    if (poisson) {
        const int64_t blocks = (a.n + T - 1) / T;
        if (blocks >= (int64_t)1 << 31) return fail(h, SAME_LDA_EINVAL, "too many draw tasks for one launch");
        dim3 grid((unsigned)blocks);
        const size_t lds = same::poisson_lds_bytes();
        if (a.K == 256)            hipLaunchKernelGGL((same::poisson_draw_kernel<true, DEBUG, 256>), grid, block, lds, st, a);
        else if (a.K % same::kBlk == 0) hipLaunchKernelGGL((same::poisson_draw_kernel<true, DEBUG>), grid, block, lds, st, a);
        else                       hipLaunchKernelGGL((same::poisson_draw_kernel<false, DEBUG>), grid, block, lds, st, a);
    } else {
        // Workgroups take segments of launch positions from a counter until none is left: as many workgroups as
        // the chip holds at once, so that it is full from the first moment to the last.
        const int64_t segments = (a.n + same::kSegment - 1) / same::kSegment;
        dim3 grid((unsigned)(segments < kDrawGrid ? segments : kDrawGrid));
        // blocks of 4 * ceil(K / 128) topics, read in batches of one, two or four 16-byte loads per matrix
        // (K = 512 and K = 1024: the scan reads a row 512 contiguous bytes per half-wave and load; at K = 256, where the
        // kernel is bound by vector-ALU issue, the extra additions of that form cost more than the fewer cache lines save)
        const size_t lds = same::draw_lds_bytes(a.K);
        const bool vec = a.K % 4 == 0;
        const int quads = same::block_len(a.K) / 4;                // 16-byte loads per block and matrix
        const int tb = quads % 4 == 0 ? 4 : (quads % 2 == 0 ? 2 : 1);
        const bool one = quads == tb;
        if (uniform)             hipLaunchKernelGGL((same::draw_kernel<true, false, DEBUG, 0, true>), grid, block, lds, st, a);
        else if (!vec)           hipLaunchKernelGGL((same::draw_kernel<false, false, DEBUG, 0, true>), grid, block, lds, st, a);
        else if (tb == 1 && one) hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 1, true>), grid, block, lds, st, a);
        else if (a.K == 256)     hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 2, true, 256>), grid, block, lds, st, a);
        else if (a.K == 1024)    hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 4, false, 1024, true>), grid, block, lds, st, a);
        else if (a.K == 512)     hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 4, true, 512, true>), grid, block, lds, st, a);
        else if (tb == 2 && one) hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 2, true>), grid, block, lds, st, a);
        else if (tb == 4 && one) hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 4, true>), grid, block, lds, st, a);
        else if (tb == 1)        hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 1, false>), grid, block, lds, st, a);
        else if (tb == 2)        hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 2, false>), grid, block, lds, st, a);
        else                     hipLaunchKernelGGL((same::draw_kernel<false, true, DEBUG, 4, false>), grid, block, lds, st, a);
    }
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

#ifdef SAME_STATS
unsigned long long* g_stats = nullptr;   // profiling builds only
#endif

same::DrawArgs draw_args(const same_lda* h, const Matrix& M, Copies c, uint32_t pass_word, bool with_words)
{
    same::DrawArgs a;
    a.n = M.n_tasks; a.counter = nullptr; a.t_doc = M.t_doc; a.t_word = M.t_word; a.t_g = M.t_g; a.order = M.order; a.cost = M.cost; a.ids = nullptr;
    a.theta = M.theta; a.phi = h->phi; a.ndk = M.ndk; a.nwk = with_words ? h->nwk : nullptr;
    // a pair holds a count below 2^(32 - kPairShift): m * largest group must fit
    // (a Poisson count may exceed its rate: four times the rate plus 128 is beyond any count the walk can return)
    const double most = (double)c.mf * (double)(M.max_group ? M.max_group : 1u);
    const bool pairs_fit = (c.poisson ? 4.0 * most + 128.0 : most) < (double)(1ull << (32 - same::kPairShift));
    a.pairs = (with_words && M.pairs && pairs_fit) ? M.pairs : nullptr;
    a.t_slot = M.t_slot;
    // the chunk pool continues full slots in the multinomial kernel
    const uint32_t usable = h->chunk_limit >= 0 && h->chunk_limit < (int64_t)h->n_chunks ? (uint32_t)h->chunk_limit : h->n_chunks;
    const bool pool = a.pairs && !c.poisson && h->chunks && usable > 0;
    a.chunks = pool ? h->chunks : nullptr;
    a.chunk_counter = nullptr;
    a.n_chunks = pool ? usable : 0u;
    a.K = h->K; a.m = c.m; a.mf = c.mf; a.seed_lo = (uint32_t)h->seed; a.seed_hi = (uint32_t)(h->seed >> 32);
    a.pass = pass_word;
    a.V = h->V;
    a.hot_of = (with_words && M.n_hot > 0) ? M.hot_of : nullptr;
#ifdef SAME_STATS
    a.stats = g_stats;
#endif
    return a;
}

uint32_t pass_word(int32_t pass_index, uint32_t domain) { return (domain << 28) | ((uint32_t)pass_index & 0x0FFFFFFFu); }

// The word-count matrix is followed by the private copies of the hot words' rows.
size_t nwk_elements(const same_lda* h) { return ((size_t)h->V + (size_t)same::kHotCopies * same::kHotMax) * h->K; }

int zero_u32(same_lda* h, uint32_t* p, size_t n, hipStream_t st)
{
    if (n == 0) return SAME_LDA_OK;
    hipLaunchKernelGGL(same::zero_u32_kernel, dim3(grid_for(n)), dim3(256), 0, st, p, n);
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

int update_theta(same_lda* h, Matrix& M, float m, hipStream_t st)
{
    const size_t n = (size_t)M.D * h->K;
    if (n == 0) return SAME_LDA_OK;
    hipLaunchKernelGGL(same::theta_update_kernel, dim3(grid_for(n)), dim3(256), 0, st, M.ndk, M.theta, n,
                       m, h->alpha);
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

int update_phi(same_lda* h, float m, float rho, hipStream_t st)
{
    const size_t n = (size_t)h->V * h->K;
    hipLaunchKernelGGL(same::zero_u64_kernel, dim3(1), dim3(256), 0, st, h->nk, (size_t)h->K);
    const int rows_per_block = 64;
    const int blocks = (h->V + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL(same::topic_totals_kernel, dim3(blocks), dim3(256), 0, st, h->nwk, h->V, h->K, h->nk,
                       rows_per_block);
    hipLaunchKernelGGL(same::phi_update_kernel, dim3(grid_for(n)), dim3(256), 0, st, h->nwk, h->nk, h->phi, n,
                       h->K, m, h->beta, (float)h->V * h->beta, rho);
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

// theta of M drawn from its Dirichlet conditional (unnormalised, mean n_dk/m + alpha).
int sample_theta(same_lda* h, Matrix& M, float m, uint32_t pword, hipStream_t st)
{
    const size_t n = (size_t)M.D * h->K;
    if (n == 0) return SAME_LDA_OK;
    hipLaunchKernelGGL(same::gamma_theta_kernel, dim3(grid_for(n)), dim3(256), 0, st, M.ndk, M.theta, n, h->K, m,
                       m * h->alpha, (uint32_t)h->seed, (uint32_t)(h->seed >> 32), pword);
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

// phi drawn from its Dirichlet conditionals: Gamma variables, their sums over words in a fixed order, division.
int sample_phi(same_lda* h, float m, uint32_t pword, hipStream_t st)
{
    const size_t n = (size_t)h->V * h->K;
    const int blocks = (h->V + kGammaRows - 1) / kGammaRows;
    // the topic totals are part of the readable state, kept current as after a collapsed update
    hipLaunchKernelGGL(same::zero_u64_kernel, dim3(1), dim3(256), 0, st, h->nk, (size_t)h->K);
    hipLaunchKernelGGL(same::topic_totals_kernel, dim3(blocks), dim3(256), 0, st, h->nwk, h->V, h->K, h->nk, kGammaRows);
    hipLaunchKernelGGL(same::gamma_phi_kernel, dim3(blocks), dim3(256), 0, st, h->nwk, h->phi, h->V, h->K,
                       m * h->beta, (uint32_t)h->seed, (uint32_t)(h->seed >> 32), pword, kGammaRows, h->gamma_partial);
    hipLaunchKernelGGL(same::gamma_phi_totals_kernel, dim3((h->K + 255) / 256), dim3(256), 0, st, h->gamma_partial,
                       blocks, h->K, h->gamma_total);
    hipLaunchKernelGGL(same::gamma_phi_normalise_kernel, dim3(grid_for(n)), dim3(256), 0, st, h->phi, n, h->K,
                       h->gamma_total);
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

// One pass of draws on M.  uniform: weights are all ones (initialisation).
int run_pass(same_lda* h, Matrix& M, Copies c, uint32_t pword, bool uniform, bool with_words, bool timed,
             hipStream_t st)
{
    int rc;
    if ((rc = zero_u32(h, M.ndk, (size_t)M.D * h->K, st))) return rc;
    if (with_words && (rc = zero_u32(h, h->nwk, nwk_elements(h), st))) return rc;   // the hot words' copies too
    if (!uniform && c.poisson && M.n_tiles > 0) {               // the Poisson kernel takes its tasks in cost order
        hipLaunchKernelGGL(same::reorder_kernel, dim3((unsigned)M.n_tiles), dim3(256), 0, st, M.tile_start, M.cost,
                           M.order);
        HIP_TRY(h, hipGetLastError());
    }
    same::DrawArgs a = draw_args(h, M, c, pword, with_words);
    if (!c.poisson && (rc = prepare_counter(h, a, st))) return rc;
    // the events bracket the draw kernel alone
    std::pair<hipEvent_t, hipEvent_t> ev{nullptr, nullptr};
    if (timed) {
        if (!h->pool.empty()) { ev = h->pool.back(); h->pool.pop_back(); }
        else {
            HIP_TRY(h, hipEventCreate(&ev.first));
            HIP_TRY(h, hipEventCreate(&ev.second));
        }
        HIP_TRY(h, hipEventRecord(ev.first, st));
    }
    if ((rc = launch_draw<false>(h, a, uniform, c.poisson, st))) return rc;
    if (timed) {
        HIP_TRY(h, hipEventRecord(ev.second, st));
        h->events.push_back(ev);
    }
    if (a.pairs && a.n > 0) {
        const int rows = same::reduce_rows(h->K);
        const int64_t blocks = (M.n_slots + same::kReduceChunk - 1) / same::kReduceChunk;
        hipLaunchKernelGGL(same::word_reduce_kernel, dim3((unsigned)blocks), dim3(same::kReduceThreads),
                           (size_t)rows * h->K * sizeof(uint32_t), st, a.pairs, a.chunks, a.n_chunks, M.slot_word, M.n_slots,
                           h->K, rows, h->nwk);
        HIP_TRY(h, hipGetLastError());
    }
    if (a.hot_of) {
        hipLaunchKernelGGL(same::hot_fold_kernel, dim3((unsigned)((M.n_hot * h->K + 255) / 256)), dim3(256), 0, st, h->nwk,
                           M.hot_word, M.n_hot, h->V, h->K);
        HIP_TRY(h, hipGetLastError());
    }
    return SAME_LDA_OK;
}

size_t state_bytes(const same_lda* h, int32_t which)
{
    switch (which) {
        case SAME_LDA_THETA: return (size_t)h->X.D * h->K * sizeof(float);
        case SAME_LDA_PHI:   return (size_t)h->V * h->K * sizeof(float);
        case SAME_LDA_NDK:   return (size_t)h->X.D * h->K * sizeof(uint32_t);
        case SAME_LDA_NWK:   return (size_t)h->V * h->K * sizeof(uint32_t);
        case SAME_LDA_NK:    return (size_t)h->K * sizeof(uint64_t);
        default:             return 0;
    }
}

void* state_ptr(same_lda* h, int32_t which)
{
    switch (which) {
        case SAME_LDA_THETA: return h->X.theta;
        case SAME_LDA_PHI:   return h->phi;
        case SAME_LDA_NDK:   return h->X.ndk;
        case SAME_LDA_NWK:   return h->nwk;
        case SAME_LDA_NK:    return h->nk;
        default:             return nullptr;
    }
}

}  // namespace

extern "C" {

int same_lda_init(same_lda_t** out, const same_lda_csc* X, int32_t K, float alpha, float beta, uint64_t seed,
                  int32_t m0, int32_t tokens_per_draw, void* hip_stream)
{
    if (!out) return fail(nullptr, SAME_LDA_EINVAL, "out is null");
    *out = nullptr;
    if (!X) return fail(nullptr, SAME_LDA_EINVAL, "matrix is null");
    if (K < 1 || K > 2048) return fail(nullptr, SAME_LDA_EINVAL, "K must be in [1, 2048] (got %d)", K);
    if (!(alpha > 0.f) || !(beta > 0.f) || !std::isfinite(alpha) || !std::isfinite(beta))
        return fail(nullptr, SAME_LDA_EINVAL, "alpha and beta must be positive and finite");
    if (X->V < 1) return fail(nullptr, SAME_LDA_EINVAL, "V must be >= 1 (got %d)", X->V);
    if (tokens_per_draw < 1) return fail(nullptr, SAME_LDA_EINVAL, "tokens_per_draw must be >= 1");
    same_lda* h = new (std::nothrow) same_lda();
    if (!h) return fail(nullptr, SAME_LDA_ENOMEM, "host allocation failed");
    h->V = X->V; h->K = K; h->G = tokens_per_draw; h->alpha = alpha; h->beta = beta; h->seed = seed;
    h->stream = static_cast<hipStream_t>(hip_stream);
    int rc = build_matrix(h, X, h->V, K, h->G, h->X, h->stream, true);
    if (!rc) rc = check_m(h, m0, h->X);
    if (!rc) rc = dev_alloc(h, &h->phi, (size_t)h->V * K);
    if (!rc) rc = dev_alloc(h, &h->nwk, nwk_elements(h));
    if (!rc) rc = dev_alloc(h, &h->nk, (size_t)K);
    if (!rc) rc = dev_alloc(h, &h->gamma_partial, (size_t)((h->V + kGammaRows - 1) / kGammaRows) * K);
    if (!rc) rc = dev_alloc(h, &h->gamma_total, (size_t)K);
    if (!rc) rc = dev_alloc(h, &h->vb_psi, (size_t)K);
    if (!rc) rc = dev_alloc(h, &h->draw_counter, (size_t)3);
    if (!rc) rc = run_pass(h, h->X, Copies::whole((uint32_t)m0), pass_word(0, 0), true, true, false, h->stream);
    if (!rc) rc = update_theta(h, h->X, (float)m0, h->stream);
    if (!rc) rc = update_phi(h, (float)m0, 1.0f, h->stream);
    if (!rc) { hipError_t e = hipStreamSynchronize(h->stream); if (e != hipSuccess) rc = fail(h, SAME_LDA_EHIP, "init: %s", hipGetErrorString(e)); }
    if (rc) { g_init_error = h->error; same_lda_free(h); return rc; }
    h->pass = 1;
    h->cache.clear_spare();                                // the build's temporaries: a single resident matrix needs them no more
    *out = h;
    return SAME_LDA_OK;
}

int same_lda_sweep(same_lda_t* h, int32_t m_t, float rho_t)
{
    if (!h) return SAME_LDA_EINVAL;
    if (!(rho_t > 0.f) || rho_t > 1.f) return fail(h, SAME_LDA_EINVAL, "rho must be in (0, 1] (got %g)", (double)rho_t);
    int rc = check_m(h, m_t, h->X);
    if (!rc) rc = run_pass(h, h->X, Copies::whole((uint32_t)m_t), pass_word(h->pass, 0), false, true, h->timing, h->stream);
    if (!rc) rc = update_theta(h, h->X, (float)m_t, h->stream);
    if (!rc) rc = update_phi(h, (float)m_t, rho_t, h->stream);
    if (!rc) h->pass += 1;
    return rc;
}

int same_lda_sweep_sampled(same_lda_t* h, int32_t m_t)
{
    if (!h) return SAME_LDA_EINVAL;
    int rc = check_m(h, m_t, h->X);
    if (!rc) rc = run_pass(h, h->X, Copies::whole((uint32_t)m_t), pass_word(h->pass, 0), false, true, h->timing, h->stream);
    if (!rc) rc = sample_theta(h, h->X, (float)m_t, pass_word(h->pass, 2), h->stream);
    if (!rc) rc = sample_phi(h, (float)m_t, pass_word(h->pass, 3), h->stream);
    if (!rc) h->pass += 1;
    return rc;
}

int same_lda_sweep_poisson(same_lda_t* h, float m_t, float rho_t)
{
    if (!h) return SAME_LDA_EINVAL;
    if (!(rho_t > 0.f) || rho_t > 1.f) return fail(h, SAME_LDA_EINVAL, "rho must be in (0, 1] (got %g)", (double)rho_t);
    int rc = check_mf(h, m_t, h->X);
    if (!rc) rc = run_pass(h, h->X, Copies::real(m_t), pass_word(h->pass, 0), false, true, h->timing, h->stream);
    if (!rc) rc = update_theta(h, h->X, m_t, h->stream);
    if (!rc) rc = update_phi(h, m_t, rho_t, h->stream);
    if (!rc) h->pass += 1;
    return rc;
}

int same_lda_stage_batch(same_lda_t* h, const same_lda_csc* X, int32_t m_init, int32_t sweeps_ahead)
{
    if (!h) return SAME_LDA_EINVAL;
    if (sweeps_ahead < 0) return fail(h, SAME_LDA_EINVAL, "sweeps_ahead must be >= 0");
    if (!h->copy_stream) HIP_TRY(h, hipStreamCreateWithFlags(&h->copy_stream, hipStreamNonBlocking));
    if (h->has_staged) { free_matrix(h, h->staged); h->has_staged = false; }
    Matrix M;
    int rc = build_matrix(h, X, h->V, h->K, h->G, M, h->copy_stream, true);
    if (!rc) rc = check_m(h, m_init, M);
    // the initial pass of the new documents needs neither phi nor the word counts: it can run now
    const int32_t pass = h->pass + sweeps_ahead;
    if (!rc) rc = run_pass(h, M, Copies::whole((uint32_t)m_init), pass_word(pass, 0), true, false, false, h->copy_stream);
    if (!rc) rc = update_theta(h, M, (float)m_init, h->copy_stream);
    if (!rc) { hipError_t e = hipStreamSynchronize(h->copy_stream); if (e != hipSuccess) rc = fail(h, SAME_LDA_EHIP, "stage_batch: %s", hipGetErrorString(e)); }
    if (rc) { (void)hipStreamSynchronize(h->copy_stream); free_matrix(h, M); return rc; }
    h->staged = M; h->has_staged = true; h->staged_pass = pass; h->staged_m = m_init;
    return SAME_LDA_OK;
}

int same_lda_commit_batch(same_lda_t* h)
{
    if (!h) return SAME_LDA_EINVAL;
    if (!h->has_staged) return fail(h, SAME_LDA_EINVAL, "no staged batch to commit");
    HIP_TRY(h, hipStreamSynchronize(h->stream));           // the old matrix may still be in use
    free_matrix(h, h->X);
    h->X = h->staged;
    h->staged = Matrix(); h->has_staged = false;
    int rc = SAME_LDA_OK;
    if (h->staged_pass != h->pass) {                       // not the announced number of sweeps: draw the initial pass again
        rc = run_pass(h, h->X, Copies::whole((uint32_t)h->staged_m), pass_word(h->pass, 0), true, false, false, h->stream);
        if (!rc) rc = update_theta(h, h->X, (float)h->staged_m, h->stream);
        if (!rc) HIP_TRY(h, hipStreamSynchronize(h->stream));
    }
    if (!rc) h->pass += 1;
    return rc;
}

int same_lda_set_batch(same_lda_t* h, const same_lda_csc* X, int32_t m_init)
{
    if (!h) return SAME_LDA_EINVAL;
    HIP_TRY(h, hipStreamSynchronize(h->stream));           // a device matrix written on this stream is complete
    int rc = same_lda_stage_batch(h, X, m_init, 0);
    if (!rc) rc = same_lda_commit_batch(h);
    return rc;
}

int same_lda_loglik(same_lda_t* h, const same_lda_csc* Xtest, int32_t foldin_sweeps, int32_t m_eval, double* ll_per_word)
{
    if (!h) return SAME_LDA_EINVAL;
    if (!ll_per_word || foldin_sweeps < 0) return fail(h, SAME_LDA_EINVAL, "bad loglik arguments");
    Matrix M;
    int rc = build_matrix(h, Xtest, h->V, h->K, h->G, M, h->stream, false);
    if (!rc) rc = check_m(h, m_eval, M);
    double* doc_log = nullptr; double* part = nullptr;
    const int nblocks = (int)((M.nnz + 255) / 256);
    if (!rc) rc = dev_alloc(h, &doc_log, (size_t)M.D);
    if (!rc) rc = dev_alloc(h, &part, (size_t)nblocks);
    if (!rc) rc = run_pass(h, M, Copies::whole((uint32_t)m_eval), pass_word(0, 1), true, false, false, h->stream);
    if (!rc) rc = update_theta(h, M, (float)m_eval, h->stream);
    for (int32_t s = 1; !rc && s <= foldin_sweeps; ++s) {
        rc = run_pass(h, M, Copies::whole((uint32_t)m_eval), pass_word(s, 1), false, false, false, h->stream);
        if (!rc) rc = update_theta(h, M, (float)m_eval, h->stream);
    }
    double total = 0.0;
    if (!rc && M.nnz > 0) {
        hipLaunchKernelGGL(same::doc_log_total_kernel, dim3((M.D + 255) / 256), dim3(256), 0, h->stream, M.theta,
                           M.D, h->K, doc_log);
        hipLaunchKernelGGL(same::loglik_kernel, dim3(nblocks), dim3(256), 0, h->stream, M.nnz, M.nz_doc, M.rowidx,
                           M.val, M.theta, h->phi, h->K, doc_log, part);
        std::vector<double> part_h((size_t)nblocks);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) e = hipMemcpyAsync(part_h.data(), part, (size_t)nblocks * 8, hipMemcpyDeviceToHost, h->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) rc = fail(h, SAME_LDA_EHIP, "loglik: %s", hipGetErrorString(e));
        for (double v : part_h) total += v;
    } else if (!rc) {
        hipError_t e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) rc = fail(h, SAME_LDA_EHIP, "loglik: %s", hipGetErrorString(e));
    }
    if (!rc) *ll_per_word = M.tokens > 0.0 ? total / M.tokens : 0.0;
    if (rc) (void)hipStreamSynchronize(h->stream);         // nothing enqueued may still use the blocks handed back
    dev_free(h, doc_log); dev_free(h, part);
    free_matrix(h, M);
    return rc;
}

void same_lda_free(same_lda_t* h)
{
    if (!h) return;
    hipStreamSynchronize(h->stream);
    free_matrix(h, h->X);
    if (h->has_staged) free_matrix(h, h->staged);
    if (h->copy_stream) { hipStreamSynchronize(h->copy_stream); hipStreamDestroy(h->copy_stream); }
    dev_free(h, h->phi); dev_free(h, h->nwk); dev_free(h, h->nk);
    dev_free(h, h->gamma_partial); dev_free(h, h->gamma_total); dev_free(h, h->draw_counter); dev_free(h, h->vb_psi);
    if (h->chunks) (void)hipFree(h->chunks);
    h->cache.clear_spare();
    for (auto& e : h->events) { hipEventDestroy(e.first); hipEventDestroy(e.second); }
    for (auto& e : h->pool) { hipEventDestroy(e.first); hipEventDestroy(e.second); }
    delete h;
}

int same_lda_get(same_lda_t* h, int32_t which, void* dst, size_t bytes, int32_t dst_on_device)
{
    if (!h) return SAME_LDA_EINVAL;
    const size_t want = state_bytes(h, which);
    if (!state_ptr(h, which) && want) return fail(h, SAME_LDA_EINVAL, "unknown selector %d", which);
    if (which < SAME_LDA_THETA || which > SAME_LDA_NK) return fail(h, SAME_LDA_EINVAL, "unknown selector %d", which);
    if (bytes != want || (!dst && want)) return fail(h, SAME_LDA_EINVAL, "selector %d needs %zu bytes (got %zu)", which, want, bytes);
    if (want) HIP_TRY(h, hipMemcpyAsync(dst, state_ptr(h, which), want, dst_on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return SAME_LDA_OK;
}

int same_lda_set(same_lda_t* h, int32_t which, const void* src, size_t bytes, int32_t src_on_device)
{
    if (!h) return SAME_LDA_EINVAL;
    if (which != SAME_LDA_THETA && which != SAME_LDA_PHI) return fail(h, SAME_LDA_EINVAL, "only theta and phi can be set");
    const size_t want = state_bytes(h, which);
    if (bytes != want || (!src && want)) return fail(h, SAME_LDA_EINVAL, "selector %d needs %zu bytes (got %zu)", which, want, bytes);
    if (want) HIP_TRY(h, hipMemcpyAsync(state_ptr(h, which), src, want, src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return SAME_LDA_OK;
}

int same_lda_get_pass(const same_lda_t* h, int32_t* pass_index)
{
    if (!h || !pass_index) return SAME_LDA_EINVAL;
    *pass_index = h->pass;
    return SAME_LDA_OK;
}

int same_lda_set_pass(same_lda_t* h, int32_t pass_index)
{
    if (!h) return SAME_LDA_EINVAL;
    if (pass_index < 0 || pass_index >= (1 << 28)) return fail(h, SAME_LDA_EINVAL, "pass index out of range");
    h->pass = pass_index;
    return SAME_LDA_OK;
}

int same_lda_task_count(const same_lda_t* h, int64_t* count)
{
    if (!h || !count) return SAME_LDA_EINVAL;
    *count = h->X.n_tasks;
    return SAME_LDA_OK;
}

namespace {
// Device memory of same_lda_debug_draw_noalloc: the segment counter of the draw kernel, the staged task ids and
// the count rows.  One copy per GPU (a file-scope device array), kept until the process ends.
constexpr int32_t kNoAllocMaxTasks = 4096;
constexpr size_t kNoAllocMaxCounts = (size_t)1 << 20;
struct NoAllocScratch {
    uint32_t counter[64];
    int64_t  ids[kNoAllocMaxTasks];
    uint32_t counts[kNoAllocMaxCounts];
};
}  // namespace

static __device__ __align__(256) unsigned char scratch[sizeof(NoAllocScratch)];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];      // the array's address on each device, once asked for
std::mutex g_scratch_mutex;

// The address of the current device's copy of `scratch` (its name is a host-side stand-in, not a device address).
int scratch_of_current_device(same_lda* h, NoAllocScratch** out)
{
    int dev = -1;
    HIP_TRY(h, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(h, SAME_LDA_EINVAL, "device %d is beyond the %d this library keeps scratch for", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(h, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<NoAllocScratch*>(g_scratch_ptr[dev]);
    return SAME_LDA_OK;
}

int debug_draw(same_lda_t* h, Copies c, const int64_t* task_ids, int32_t n, uint32_t* counts_out)
{
    if (n < 0 || (n > 0 && (!task_ids || !counts_out))) return fail(h, SAME_LDA_EINVAL, "bad debug_draw arguments");
    int rc = c.poisson ? check_mf(h, c.mf, h->X) : check_m(h, (int32_t)c.m, h->X);
    if (rc || n == 0) return rc;
    for (int32_t i = 0; i < n; ++i)
        if (task_ids[i] < 0 || task_ids[i] >= h->X.n_tasks) return fail(h, SAME_LDA_EINVAL, "task id %lld out of range", (long long)task_ids[i]);
    int64_t* ids_d = nullptr; uint32_t* out_d = nullptr;
    rc = dev_alloc(h, &ids_d, (size_t)n);
    if (!rc) rc = dev_alloc(h, &out_d, (size_t)n * h->K);
    if (!rc) {
        hipError_t e = hipMemcpyAsync(ids_d, task_ids, (size_t)n * 8, hipMemcpyHostToDevice, h->stream);
        if (e != hipSuccess) rc = fail(h, SAME_LDA_EHIP, "debug_draw: %s", hipGetErrorString(e));
    }
    if (!rc) rc = zero_u32(h, out_d, (size_t)n * h->K, h->stream);
    if (!rc) {
        same::DrawArgs a = draw_args(h, h->X, c, pass_word(h->pass, 0), false);
        a.n = n; a.ids = ids_d; a.ndk = out_d; a.nwk = nullptr; a.cost = nullptr;
        if (!c.poisson) rc = prepare_counter(h, a, h->stream);
        if (!rc) rc = launch_draw<true>(h, a, false, c.poisson, h->stream);
    }
    if (!rc) {
        hipError_t e = hipMemcpyAsync(counts_out, out_d, (size_t)n * h->K * 4, hipMemcpyDeviceToHost, h->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) rc = fail(h, SAME_LDA_EHIP, "debug_draw: %s", hipGetErrorString(e));
    }
    if (rc) (void)hipStreamSynchronize(h->stream);
    dev_free(h, ids_d); dev_free(h, out_d);
    return rc;
}
}  // namespace

int same_lda_debug_draw(same_lda_t* h, int32_t m_t, const int64_t* task_ids, int32_t n, uint32_t* counts_out)
{
    if (!h) return SAME_LDA_EINVAL;
    if (m_t < 1) return fail(h, SAME_LDA_EINVAL, "m must be >= 1 (got %d)", m_t);
    return debug_draw(h, Copies::whole((uint32_t)m_t), task_ids, n, counts_out);
}

int same_lda_debug_draw_noalloc(same_lda_t* h, int32_t m_t, const int64_t* task_ids, int32_t n, uint32_t* counts_out)
{
    if (!h) return SAME_LDA_EINVAL;
    if (m_t < 1) return fail(h, SAME_LDA_EINVAL, "m must be >= 1 (got %d)", m_t);
    if (n < 0 || (n > 0 && (!task_ids || !counts_out))) return fail(h, SAME_LDA_EINVAL, "bad debug_draw arguments");
    if (n > kNoAllocMaxTasks || (size_t)n * (size_t)h->K > kNoAllocMaxCounts)
        return fail(h, SAME_LDA_EINVAL, "debug_draw_noalloc takes at most %d tasks and %zu counts (tasks * K) per call (got %d tasks, K = %d)",
                    kNoAllocMaxTasks, kNoAllocMaxCounts, n, h->K);
    int rc = check_m(h, m_t, h->X);
    if (rc || n == 0) return rc;
    for (int32_t i = 0; i < n; ++i)
        if (task_ids[i] < 0 || task_ids[i] >= h->X.n_tasks) return fail(h, SAME_LDA_EINVAL, "task id %lld out of range", (long long)task_ids[i]);
    NoAllocScratch* S = nullptr;
    if ((rc = scratch_of_current_device(h, &S))) return rc;
    const size_t counts = (size_t)n * h->K;
    HIP_TRY(h, hipMemcpyAsync(S->ids, task_ids, (size_t)n * 8, hipMemcpyHostToDevice, h->stream));
    if ((rc = zero_u32(h, S->counts, counts, h->stream))) return rc;             // the array keeps the last call's contents
    same::DrawArgs a = draw_args(h, h->X, Copies::whole((uint32_t)m_t), pass_word(h->pass, 0), false);
    a.n = n; a.ids = S->ids; a.ndk = S->counts; a.nwk = nullptr; a.cost = nullptr;
    a.counter = S->counter;
    if ((rc = zero_u32(h, S->counter, 1, h->stream))) return rc;
    if ((rc = launch_draw<true>(h, a, false, false, h->stream))) return rc;
    HIP_TRY(h, hipMemcpyAsync(counts_out, S->counts, counts * 4, hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return SAME_LDA_OK;
}

int same_lda_debug_chunk_limit(same_lda_t* h, int64_t max_chunks, int64_t* chunks_in_use)
{
    if (!h) return SAME_LDA_EINVAL;
    h->chunk_limit = max_chunks < 0 ? -1 : max_chunks;
    if (chunks_in_use)
        *chunks_in_use = h->chunk_limit >= 0 && h->chunk_limit < (int64_t)h->n_chunks ? h->chunk_limit : (int64_t)h->n_chunks;
    return SAME_LDA_OK;
}

int same_lda_debug_draw_poisson(same_lda_t* h, float m_t, const int64_t* task_ids, int32_t n, uint32_t* counts_out)
{
    if (!h) return SAME_LDA_EINVAL;
    return debug_draw(h, Copies::real(m_t), task_ids, n, counts_out);
}

int same_lda_sddmm(same_lda_t* h, float* mu_out, int32_t out_on_device)
{
    if (!h) return SAME_LDA_EINVAL;
    const Matrix& M = h->X;
    if (M.nnz == 0) return SAME_LDA_OK;
    if (!mu_out) return fail(h, SAME_LDA_EINVAL, "mu_out is null");
    float* dst = mu_out;
    if (!out_on_device) { int rc = dev_alloc(h, &dst, (size_t)M.nnz); if (rc) return rc; }
    const int waves_per_block = 4;
    const int64_t waves = (M.nnz + same::kSddmmChunk - 1) / same::kSddmmChunk;
    const int64_t blocks = (waves + waves_per_block - 1) / waves_per_block;
    std::pair<hipEvent_t, hipEvent_t> ev{nullptr, nullptr};
    if (h->timing) {
        if (!h->pool.empty()) { ev = h->pool.back(); h->pool.pop_back(); }
        else { HIP_TRY(h, hipEventCreate(&ev.first)); HIP_TRY(h, hipEventCreate(&ev.second)); }
        HIP_TRY(h, hipEventRecord(ev.first, h->stream));
    }
    if (h->K % 4 == 0 && h->K <= 256)
        hipLaunchKernelGGL(same::sddmm_small_kernel, dim3((unsigned)blocks), dim3(64 * waves_per_block), 0, h->stream,
                           M.nz_doc, M.rowidx, M.nnz, h->K, M.theta, h->phi, dst);
    else if (h->K % 4 == 0)
        hipLaunchKernelGGL(same::sddmm_kernel<true>, dim3((unsigned)blocks), dim3(64 * waves_per_block), 0, h->stream,
                           M.nz_doc, M.rowidx, M.nnz, h->K, M.theta, h->phi, dst);
    else
        hipLaunchKernelGGL(same::sddmm_kernel<false>, dim3((unsigned)blocks), dim3(64 * waves_per_block), 0, h->stream,
                           M.nz_doc, M.rowidx, M.nnz, h->K, M.theta, h->phi, dst);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && h->timing) { e = hipEventRecord(ev.second, h->stream); if (e == hipSuccess) h->events.push_back(ev); }
    if (e == hipSuccess && !out_on_device) {
        e = hipMemcpyAsync(mu_out, dst, (size_t)M.nnz * 4, hipMemcpyDeviceToHost, h->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    }
    if (!out_on_device) dev_free(h, dst);
    if (e != hipSuccess) return fail(h, SAME_LDA_EHIP, "sddmm: %s", hipGetErrorString(e));
    return SAME_LDA_OK;
}

int same_lda_vb_exp_elog_beta(same_lda_t* h, const float* lambda, float* b_out, float* shift_out)
{
    if (!h) return SAME_LDA_EINVAL;
    if (!lambda || !b_out || !shift_out) return fail(h, SAME_LDA_EINVAL, "vb_exp_elog_beta: lambda, b_out and shift_out must be device pointers");
    static_assert(same::kVbRows == kGammaRows, "the column sums reuse the block-sum buffer of the sampled phi step");
    const int blocks = (h->V + same::kVbRows - 1) / same::kVbRows;
    hipLaunchKernelGGL(same::vb_colsum_kernel, dim3(blocks), dim3(256), 0, h->stream, lambda, h->V, h->K, h->gamma_partial);
    hipLaunchKernelGGL(same::vb_colpsi_kernel, dim3((h->K + 255) / 256), dim3(256), 0, h->stream, h->gamma_partial, blocks, h->K,
                       h->vb_psi);
    hipLaunchKernelGGL(same::vb_exp_elog_beta_kernel, dim3((unsigned)((h->V + 3) / 4)), dim3(256), 0, h->stream, lambda, h->V, h->K,
                       h->vb_psi, b_out, shift_out);
    HIP_TRY(h, hipGetLastError());
    return SAME_LDA_OK;
}

int same_lda_vb_estep(same_lda_t* h, const float* b, const float* shift, float alpha, int32_t iters, float* gamma,
                      float* log_mu_out)
{
    if (!h) return SAME_LDA_EINVAL;
    const Matrix& M = h->X;
    if (!(alpha > 0.f) || !std::isfinite(alpha)) return fail(h, SAME_LDA_EINVAL, "alpha must be positive and finite (got %g)", (double)alpha);
    if (iters < 0) return fail(h, SAME_LDA_EINVAL, "iters must be >= 0 (got %d)", iters);
    if (M.D == 0 || iters == 0) return SAME_LDA_OK;
    if (!b || !gamma) return fail(h, SAME_LDA_EINVAL, "vb_estep: b and gamma must be device pointers");
    const int waves_per_block = 4;
    const unsigned blocks = (unsigned)((M.D + waves_per_block - 1) / waves_per_block);
    std::pair<hipEvent_t, hipEvent_t> ev{nullptr, nullptr};
    if (h->timing) {
        if (!h->pool.empty()) { ev = h->pool.back(); h->pool.pop_back(); }
        else { HIP_TRY(h, hipEventCreate(&ev.first)); HIP_TRY(h, hipEventCreate(&ev.second)); }
        HIP_TRY(h, hipEventRecord(ev.first, h->stream));
    }
    const int K = h->K;
    const dim3 grid(blocks), block(64 * waves_per_block);
#define SAME_VB_LAUNCH(CH) hipLaunchKernelGGL(same::vb_estep_kernel<CH>, grid, block, 0, h->stream, M.colptr, M.rowidx, M.val, \
                                              M.D, K, b, shift, alpha, iters, gamma, log_mu_out)
    if (K % 4 != 0)
        hipLaunchKernelGGL(same::vb_estep_any_kernel, grid, block, (size_t)waves_per_block * (2 * K + (K + 1) / 2) * sizeof(double), h->stream, M.colptr,
                           M.rowidx, M.val, M.D, K, b, shift, alpha, iters, gamma, log_mu_out);
    else if (K <= 256)  SAME_VB_LAUNCH(1);
    else if (K <= 512)  SAME_VB_LAUNCH(2);
    else if (K <= 1024) SAME_VB_LAUNCH(4);
    else                SAME_VB_LAUNCH(8);
#undef SAME_VB_LAUNCH
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && h->timing) { e = hipEventRecord(ev.second, h->stream); if (e == hipSuccess) h->events.push_back(ev); }
    if (e != hipSuccess) return fail(h, SAME_LDA_EHIP, "vb_estep: %s", hipGetErrorString(e));
    return SAME_LDA_OK;
}

int same_lda_set_timing(same_lda_t* h, int32_t enabled)
{
    if (!h) return SAME_LDA_EINVAL;
    h->timing = enabled != 0;
    return SAME_LDA_OK;
}

int same_lda_get_timing(same_lda_t* h, double* draw_ms_total, int64_t* launches)
{
    if (!h || !draw_ms_total || !launches) return SAME_LDA_EINVAL;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    double total = 0.0;
    for (auto& e : h->events) {
        float ms = 0.f;
        HIP_TRY(h, hipEventElapsedTime(&ms, e.first, e.second));
        total += (double)ms;
        h->pool.push_back(e);
    }
    *draw_ms_total = total;
    *launches = (int64_t)h->events.size();
    h->events.clear();
    return SAME_LDA_OK;
}

namespace {
// The work list's exclusive sum and stable radix sort on a seeded array of a million items over several tiles with a
// ragged end: sums against the host's, the sorted pairs must be the input's pairs in (key, position) order.
int selftest_sort_and_sum(int64_t* bad)
{
    const size_t n = 1000003;
    const int32_t V = 70001;                                       // 17 bits: three passes
    std::vector<int32_t> keys(n);
    std::vector<uint32_t> cnt(n);
    uint32_t x = 12345u;
    for (size_t i = 0; i < n; ++i) { x = x * 1664525u + 1013904223u; keys[i] = (int32_t)((x >> 8) % (uint32_t)V); cnt[i] = (x >> 28); }
    same_lda* h = new (std::nothrow) same_lda();
    if (!h) return fail(nullptr, SAME_LDA_ENOMEM, "host allocation failed");
    int rc = SAME_LDA_OK;
    int64_t wrong = 0;
    {
        Temps tmp(h, nullptr);
        const uint32_t tiles = (uint32_t)((n + same::kSortTile - 1) / same::kSortTile);
        const size_t cells = (size_t)same::kSortDigits * tiles;
        int32_t *kin = nullptr, *kb[2] = {nullptr, nullptr}, *vb[2] = {nullptr, nullptr};
        uint32_t *hist = nullptr, *hstart = nullptr, *cin = nullptr, *cout = nullptr;
        hipError_t e = tmp.get(&kin, n);
        if (e == hipSuccess) e = tmp.get(&kb[0], n);
        if (e == hipSuccess) e = tmp.get(&kb[1], n);
        if (e == hipSuccess) e = tmp.get(&vb[0], n);
        if (e == hipSuccess) e = tmp.get(&vb[1], n);
        if (e == hipSuccess) e = tmp.get(&hist, cells);
        if (e == hipSuccess) e = tmp.get(&hstart, cells);
        if (e == hipSuccess) e = tmp.get(&cin, n);
        if (e == hipSuccess) e = tmp.get(&cout, n);
        if (e == hipSuccess) e = hipMemcpy(kin, keys.data(), n * 4, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(cin, cnt.data(), n * 4, hipMemcpyHostToDevice);
        const int32_t* k = kin;
        const int32_t* v = nullptr;
        int to = 0;
        for (int shift = 0; e == hipSuccess && shift < 17; shift += 8, to ^= 1) {
            hipLaunchKernelGGL(same::wl_sort_histogram, dim3(tiles), dim3(same::kSortThreads), 0, nullptr, k, (int64_t)n, shift, tiles, hist);
            e = exclusive_sum(tmp, hist, hstart, cells, nullptr);
            if (e != hipSuccess) break;
            hipLaunchKernelGGL(same::wl_sort_scatter, dim3(tiles), dim3(same::kSortThreads), 0, nullptr, k, v, (int64_t)n, shift, tiles, hstart,
                               kb[to], vb[to]);
            k = kb[to]; v = vb[to];
        }
        if (e == hipSuccess) e = exclusive_sum(tmp, cin, cout, n, nullptr);
        std::vector<int32_t> ks(n), vs(n);
        std::vector<uint32_t> sums(n);
        if (e == hipSuccess) e = hipMemcpy(ks.data(), k, n * 4, hipMemcpyDeviceToHost);
        if (e == hipSuccess) e = hipMemcpy(vs.data(), v, n * 4, hipMemcpyDeviceToHost);
        if (e == hipSuccess) e = hipMemcpy(sums.data(), cout, n * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) rc = fail(nullptr, SAME_LDA_EHIP, "selftest: %s", hipGetErrorString(e));
        else {
            uint32_t run = 0;
            for (size_t i = 0; i < n; ++i) {
                if (sums[i] != run) ++wrong;
                run += cnt[i];
                const int32_t src = vs[i];
                if (src < 0 || (size_t)src >= n || keys[(size_t)src] != ks[i]) { ++wrong; continue; }
                if (i > 0 && (ks[i] < ks[i - 1] || (ks[i] == ks[i - 1] && vs[i] <= vs[i - 1]))) ++wrong;   // a permutation follows
            }
        }
    }
    h->cache.clear_spare();
    delete h;
    *bad = wrong;
    return rc;
}
}  // namespace

int same_lda_selftest(int64_t* failures)
{
    if (!failures) return fail(nullptr, SAME_LDA_EINVAL, "failures is null");
    unsigned long long* d = nullptr;
    unsigned long long got = 0;
    HIP_TRY(nullptr, hipMalloc(reinterpret_cast<void**>(&d), sizeof(unsigned long long)));
    hipError_t e = hipMemset(d, 0, sizeof(unsigned long long));
    if (e == hipSuccess) {
        hipLaunchKernelGGL(same::selftest_kernel, dim3((1u << 24) / 256u), dim3(256), 0, nullptr, d);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpy(&got, d, sizeof got, hipMemcpyDeviceToHost);
    hipFree(d);
    if (e != hipSuccess) return fail(nullptr, SAME_LDA_EHIP, "selftest: %s", hipGetErrorString(e));
    int64_t bad = 0;
    const int rc = selftest_sort_and_sum(&bad);
    if (rc) return rc;
    *failures = (int64_t)got + bad;
    return SAME_LDA_OK;
}

int same_lda_synchronize(same_lda_t* h)
{
    if (!h) return SAME_LDA_EINVAL;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return SAME_LDA_OK;
}

#ifdef SAME_STATS
// Profiling builds only: device array of 8 event counters filled by the draw kernel.
void same_lda_stats_buffer(unsigned long long* device_counters) { g_stats = device_counters; }
#endif

const char* same_lda_last_error(const same_lda_t* h)
{
    return h ? h->error.c_str() : g_init_error.c_str();
}

}  // extern "C"
