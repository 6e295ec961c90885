// C ABI of the library (see include/lda_mi355x.h): argument checks, the state
// machine, device allocations and the host-side tiling tables.  All arithmetic of
// the method runs in the kernels of alias.hip, sweep.hip, rebuild.hip, loglik.hip.
#include <algorithm>
#include <atomic>
#include <cstring>

#include "common.hpp"
#include "doc_tile.hpp"

namespace lda {

static thread_local std::string g_init_error;

int fail(lda_ctx* c, int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    g_init_error = buf;
    return code;
}

int device_malloc(lda_ctx* c, void** p, size_t bytes, const char* what)
{
    *p = nullptr;
    if (bytes == 0) bytes = 1;
    if (c->opt.dev_alloc) {
        *p = c->opt.dev_alloc(bytes, c->opt.alloc_user);
        if (!*p)
            return fail(c, LDA_ERR_OOM, "the caller's allocator returned NULL for %zu bytes (%s)",
                        bytes, what);
        return LDA_OK;
    }
    const hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) {
        *p = nullptr;
        (void)hipGetLastError();
        return fail(c, LDA_ERR_OOM, "device allocation of %zu bytes for %s failed: %s", bytes, what,
                    hipGetErrorString(e));
    }
    return LDA_OK;
}

void device_free(lda_ctx* c, void* p)
{
    if (!p) return;
    if (c->opt.dev_free) c->opt.dev_free(p, c->opt.alloc_user);
    else (void)hipFree(p);
}

namespace {

// bytes of list memory of the alias builder for n entries with the mass cache
size_t alias_list_bytes_host(size_t n) { return 8 * (n + 1) + 4 * n + 4 * n; }

int setup_hybrid(lda_ctx* c, const std::vector<int32_t>& woff);

template <class T>
int dev_alloc(lda_ctx* c, T** p, size_t count, const char* what)
{
    return device_malloc(c, p, count, what);
}

template <class T>
void dev_free(lda_ctx* c, T*& p)
{
    device_free(c, p);
    p = nullptr;
}

void free_all(lda_ctx* c)
{
    dev_free(c, c->d_word); dev_free(c, c->d_doff); dev_free(c, c->d_z); dev_free(c, c->d_znew);
    dev_free(c, c->d_gid); dev_free(c, c->d_wpos); dev_free(c, c->d_xmap); dev_free(c, c->d_zt); dev_free(c, c->d_rec);
    dev_free(c, c->d_row_items); dev_free(c, c->d_mix_items); dev_free(c, c->d_gather_pieces);
    for (int i = 0; i < 3; ++i) dev_free(c, c->d_sort_words[i]);
    dev_free(c, c->d_long_words); dev_free(c, c->d_long_base); dev_free(c, c->d_long_tiles); dev_free(c, c->d_fill_tiles);
    dev_free(c, c->d_long_part); dev_free(c, c->d_long_dcount); dev_free(c, c->d_long_dstart);
    dev_free(c, c->d_long_cursor); dev_free(c, c->d_long_nnzd); dev_free(c, c->d_long_lofs);
    dev_free(c, c->d_nk_part); dev_free(c, c->d_nk_tiles); dev_free(c, c->d_nk_ranges);
    for (hipEvent_t& e : c->pass_ev) {
        if (e) (void)hipEventDestroy(e);
        e = nullptr;
    }
    if (c->side_stream) (void)hipStreamSynchronize(c->side_stream);
    if (c->side_fork) (void)hipEventDestroy(c->side_fork);
    if (c->side_join) (void)hipEventDestroy(c->side_join);
    if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
    c->side_fork = c->side_join = nullptr;
    c->side_stream = nullptr;
    dev_free(c, c->d_woff); dev_free(c, c->d_nkw); dev_free(c, c->d_nk);
    dev_free(c, c->d_alias); dev_free(c, c->d_cap); dev_free(c, c->d_chunk_doc); dev_free(c, c->d_chunk_tok); dev_free(c, c->d_tokdoc); dev_free(c, c->d_chunk_doc2); dev_free(c, c->d_chunk_tok2); dev_free(c, c->d_tokdoc2); dev_free(c, c->d_long_doc);
    dev_free(c, c->d_long_slot); dev_free(c, c->d_long_keys); dev_free(c, c->d_long_cnts); dev_free(c, c->d_long_first);
    dev_free(c, c->d_tiles); dev_free(c, c->d_multi_words); dev_free(c, c->d_partial); dev_free(c, c->d_row);
    dev_free(c, c->d_flag);
    dev_free(c, c->d_dense_alias_words);
    for (int i = 0; i < kMixClasses; ++i) dev_free(c, c->d_mix_class[i]);
    dev_free(c, c->d_sparse_words); dev_free(c, c->d_compact_words); dev_free(c, c->d_sp_off);
    dev_free(c, c->d_sp_topic); dev_free(c, c->d_sp_count); dev_free(c, c->d_sp_nnz); dev_free(c, c->d_hs_off);
    dev_free(c, c->d_hs); dev_free(c, c->d_ma); dev_free(c, c->d_metaA); c->d_metaB = nullptr;
    dev_free(c, c->d_beta_alias); dev_free(c, c->d_beta_hdr); dev_free(c, c->d_big_ws);
}

}  // namespace

// Once per process and device, before the first allocation of the first context: take a large
// block from the driver and give it back.  Observed on this GPU, not explained: the arrays of
// the first process that allocates on a freshly started device make the sweep's gathers about
// 4 % slower than the same arrays of any later process -- and equally fast once 16 GB have
// been allocated and freed (or are merely held) beforehand; 8 GB give half of the effect, 1 GB
// none.  Where the driver places the long-lived arrays seems to matter, and this changes it.
// Only with the library's own allocator; a failure is ignored.
static void prime_device_heap()
{
    static std::atomic<uint64_t> primed{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) {
        (void)hipGetLastError();
        return;
    }
    if (primed.fetch_or(1ull << dev) & (1ull << dev)) return;
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) {
        (void)hipGetLastError();
        return;
    }
    const size_t want = std::min<size_t>((size_t)16 << 30, free_b / 2);
    if (want < ((size_t)1 << 30)) return;
    void* p = nullptr;
    if (hipMalloc(&p, want) == hipSuccess) (void)hipFree(p);
    else (void)hipGetLastError();
}

int fork_side_stream(lda_ctx* c)
{
    if (c->side_pending) {
        const int rc = join_side_stream(c);
        if (rc != LDA_OK) return rc;
    }
    if (!c->side_stream) {
        LDA_HIP(c, hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking));
        LDA_HIP(c, hipEventCreateWithFlags(&c->side_fork, hipEventDisableTiming));
        LDA_HIP(c, hipEventCreateWithFlags(&c->side_join, hipEventDisableTiming));
    }
    LDA_HIP(c, hipEventRecord(c->side_fork, c->stream));
    LDA_HIP(c, hipStreamWaitEvent(c->side_stream, c->side_fork, 0));
    return LDA_OK;
}

int side_stream_done(lda_ctx* c)
{
    LDA_HIP(c, hipEventRecord(c->side_join, c->side_stream));
    c->side_pending = true;
    return LDA_OK;
}

int join_side_stream(lda_ctx* c)
{
    if (!c->side_pending) return LDA_OK;
    c->side_pending = false;
    LDA_HIP(c, hipStreamWaitEvent(c->stream, c->side_join, 0));
    return LDA_OK;
}

namespace {

template <class T>
int upload(lda_ctx* c, T** dst, const std::vector<T>& v, const char* what)
{
    int rc = dev_alloc(c, dst, v.size(), what);
    if (rc != LDA_OK) return rc;
    if (!v.empty()) {
        hipError_t e = hipMemcpy(*dst, v.data(), sizeof(T) * v.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) return fail(c, LDA_ERR_HIP, "upload of %s: %s", what, hipGetErrorString(e));
    }
    return LDA_OK;
}

// A mixture word with a dense row whose tokens fit one rebuild tile gets its list of
// non-zeros from the workgroup that histograms the row; the others from a compaction
// pass over the row (needs h_wcount, h_wkind).
bool list_from_rebuild(const lda_ctx* c, int32_t w)
{
    return c->hybrid && (c->h_wkind[w] & 3) == 1 && c->h_wcount[w] <= c->rebuild_tile_tokens &&
           c->K <= max_rebuild_topics();
}

// Word classes, list / hash-row offsets, work lists and buffers of the hybrid store.
// woff: host copy of the word segment offsets.
int setup_hybrid(lda_ctx* c, const std::vector<int32_t>& woff)
{
    const int32_t V = c->V, K = c->K, H = c->H;
    const int32_t min_count = c->opt.dense_alias_min_count;
    c->h_wcount.resize(V);
    c->h_wkind.resize(V);
    c->h_sp_off.assign((size_t)V + 1, 0);
    c->h_hs_off.assign((size_t)V + 1, 0);
    std::vector<int32_t> dense_alias, mix, sparse, compact, list_only, mixc[kMixClasses];
    std::vector<uint4> meta(2 * (size_t)V, make_uint4(0u, 0u, 0u, 0u));
    const int32_t lds_max = max_lds_table_entries();
    uint64_t list_total = 0, hash_total = 0;
    for (int32_t w = 0; w < V; ++w) {
        const int32_t cw = woff[w + 1] - woff[w];
        c->h_wcount[w] = cw;
        const bool dense_row = w < H;
        const bool dense_alias_w = (min_count == 0) || (cw >= min_count);
        if (dense_alias_w && !dense_row)
            return fail(c, LDA_ERR_ARG,
                        "lda_init: word %d (count %d) would draw from a dense table but has no dense "
                        "row; raise dense_alias_min_count or dense_rows", w, cw);
        uint8_t kind = (dense_row ? 1 : 0) | (dense_alias_w ? 2 : 0);
        c->h_wkind[w] = kind;
        c->h_sp_off[w] = (uint32_t)list_total;
        c->h_hs_off[w] = (uint32_t)hash_total;
        uint32_t lg = 0;
        if (dense_alias_w) {
            dense_alias.push_back(w);
        } else {
            if ((uint32_t)cw >> kMixCountBits)
                return fail(c, LDA_ERR_UNSUPPORTED,
                            "lda_init: word %d has %d tokens; a word with 2^%u tokens or more must "
                            "draw from a dense table (dense_alias_min_count)", w, cw, kMixCountBits);
            const int32_t cap = std::min(cw, K);
            list_total += (uint64_t)cap;
            mix.push_back(w);
            int cl = 0;
            while (kMixClassCap[cl] >= 0 && cap > (kMixClassCap[cl] ? kMixClassCap[cl] : lds_max)) ++cl;
            mixc[cl].push_back(w);
            if (dense_row) {
                if (!list_from_rebuild(c, w)) {
                    compact.push_back(w);
                } else if (K <= kMixRowTopics && cw >= kMixRowMinTokens) {
                    kind |= (uint8_t)kKindListOnly;  // served from its list everywhere
                    c->h_wkind[w] = kind;
                    list_only.push_back(w);
                }
            } else {
                sparse.push_back(w);
                uint32_t hcap = 2;
                while (hcap < 2u * (uint32_t)cap) hcap <<= 1;
                while ((1u << lg) < hcap) ++lg;
                hash_total += hcap;
            }
        }
        meta[2 * (size_t)w + 1] = make_uint4(c->h_sp_off[w], c->h_hs_off[w], lg, kind);
        if (list_total > 0x7FFFFFFFull || hash_total > 0xFFFFFFFFull)
            return fail(c, LDA_ERR_UNSUPPORTED, "lda_init: sparse rows exceed 2^31 entries");
    }
    c->h_sp_off[V] = (uint32_t)list_total;
    c->h_hs_off[V] = (uint32_t)hash_total;
    c->total_list = (int64_t)list_total;
    c->total_hash = (int64_t)hash_total;
    c->n_dense_alias = (int32_t)dense_alias.size();
    c->n_mix = (int32_t)mix.size();
    c->n_list_only = (int32_t)list_only.size();
    sparse.insert(sparse.end(), list_only.begin(), list_only.end());  // d_sparse_words: see common.hpp
    c->n_sparse = (int32_t)sparse.size();
    c->n_compact = (int32_t)compact.size();
    if (c->n_dense_alias > 0 && K > lds_max && (double)H * (double)K > 4.0e9)
        return fail(c, LDA_ERR_UNSUPPORTED, "lda_init: dense tables for %d words at K = %d", H, K);

    int rc;
#define UP(field, vec, what) do { rc = upload(c, &c->field, vec, what); if (rc != LDA_OK) return rc; } while (0)
    UP(d_dense_alias_words, dense_alias, "dense-table words");
    UP(d_sparse_words, sparse, "sparse-row words");
    UP(d_compact_words, compact, "compaction words");
    {  // the tables built in the global workspace: largest list first (see alias_mix_big_kernel)
        std::vector<int32_t>& big = mixc[kMixClasses - 1];
        std::stable_sort(big.begin(), big.end(), [&](int32_t a, int32_t b) {
            return c->h_sp_off[a + 1] - c->h_sp_off[a] > c->h_sp_off[b + 1] - c->h_sp_off[b];
        });
    }
    for (int i = 0; i < kMixClasses; ++i) {
        c->n_mix_class[i] = (int32_t)mixc[i].size();
        UP(d_mix_class[i], mixc[i], "mixture class");
    }
    UP(d_sp_off, c->h_sp_off, "list offsets");
    UP(d_hs_off, c->h_hs_off, "hash offsets");
    UP(d_metaA, meta, "word descriptors");
    c->d_metaB = c->d_metaA + 1;
#undef UP
#define AL(field, count, what) do { rc = dev_alloc(c, &c->field, (size_t)(count), what); if (rc != LDA_OK) return rc; } while (0)
    AL(d_sp_topic, list_total, "sparse rows");
    AL(d_sp_count, list_total, "sparse rows");
    AL(d_sp_nnz, V, "sparse rows");
    AL(d_hs, hash_total, "hash rows");
    AL(d_ma, list_total, "mixture tables");
    AL(d_beta_alias, (size_t)K + 2, "beta table");  // read in aligned pairs
    AL(d_beta_hdr, 2, "beta table");
    LDA_HIP(c, hipMemsetAsync(c->d_sp_nnz, 0, sizeof(int32_t) * (size_t)V, c->stream));
    // global list memory for tables too large for LDS
    const bool need_big = (K > lds_max && (c->n_dense_alias > 0 || c->n_mix > 0)) ||
                          c->n_mix_class[kMixClasses - 1] > 0;
    if (need_big) {
        c->big_ws_stride = (alias_list_bytes_host((size_t)K) + 255) / 256 * 256;
        // one workgroup per compute unit when 12 GB allow it (K = 10^6: 256 x 40 MB)
        int64_t wg = (int64_t)(12.0e9 / (double)c->big_ws_stride);
        c->n_big_wg = (int32_t)std::max<int64_t>(1, std::min<int64_t>(256, wg));
        AL(d_big_ws, c->big_ws_stride * ((size_t)c->n_big_wg + 1), "table workspace");
    }
#undef AL
    return setup_sparse_rows(c, woff);
}


// Greedy tiling of the documents: consecutive documents are grouped while they
// fit cap_tokens tokens and cap_docs documents.  A document longer than
// max_doc (<= cap_tokens) becomes a tile of its own and is also listed as "long".
void build_doc_tiles(const std::vector<int32_t>& doff, int64_t D, int32_t cap_tokens,
                     int32_t cap_docs, int32_t max_doc, std::vector<int32_t>& chunk_doc,
                     std::vector<int32_t>& long_doc)
{
    chunk_doc.clear();
    long_doc.clear();
    chunk_doc.push_back(0);
    int32_t cur_tok = 0, cur_docs = 0;
    for (int64_t d = 0; d < D; ++d) {
        const int32_t L = doff[d + 1] - doff[d];
        if (L > max_doc) {
            if (cur_docs > 0) chunk_doc.push_back((int32_t)d);
            chunk_doc.push_back((int32_t)d + 1);
            long_doc.push_back((int32_t)d);
            cur_tok = 0;
            cur_docs = 0;
            continue;
        }
        if (cur_docs > 0 && (cur_tok + L > cap_tokens || cur_docs + 1 > cap_docs)) {
            chunk_doc.push_back((int32_t)d);
            cur_tok = 0;
            cur_docs = 0;
        }
        cur_tok += L;
        cur_docs += 1;
    }
    if (cur_docs > 0) chunk_doc.push_back((int32_t)D);
}

}  // namespace
}  // namespace lda

using namespace lda;

extern "C" {

int lda_init(lda_ctx** out, int64_t D, int32_t V, int32_t K, const int64_t* doc_offsets,
             const int32_t* word_ids, double alpha, double beta, uint64_t seed,
             const lda_options* opt)
{
    if (!out) return fail(nullptr, LDA_ERR_ARG, "lda_init: out is NULL");
    *out = nullptr;
    if (!doc_offsets || !word_ids) return fail(nullptr, LDA_ERR_ARG, "lda_init: NULL corpus pointer");
    if (D < 1 || D > 2147483646LL) return fail(nullptr, LDA_ERR_ARG, "lda_init: D out of range");
    if (V < 1 || K < 1) return fail(nullptr, LDA_ERR_ARG, "lda_init: V and K must be >= 1");
    if (!(alpha > 0.0) || !(beta > 0.0) || !(alpha < 1e300) || !(beta < 1e300))
        return fail(nullptr, LDA_ERR_ARG, "lda_init: alpha and beta must be positive and finite");
    if (doc_offsets[0] != 0) return fail(nullptr, LDA_ERR_ARG, "lda_init: doc_offsets[0] != 0");
    for (int64_t d = 0; d < D; ++d)
        if (doc_offsets[d + 1] < doc_offsets[d])
            return fail(nullptr, LDA_ERR_ARG, "lda_init: doc_offsets decreases at %lld", (long long)d);
    const int64_t N = doc_offsets[D];
    if (N < 1) return fail(nullptr, LDA_ERR_ARG, "lda_init: empty corpus");
    // token positions are 32-bit; kernels look up to a few thousand positions past a segment's end
    // in their loop conditions, so the margin keeps every such sum representable
    if (N > 2147483647LL - (1LL << 20))
        return fail(nullptr, LDA_ERR_ARG, "lda_init: N must be at most 2^31 - 2^20 - 1 tokens");
    lda_options o{};
    if (opt) o = *opt;
    if (o.proposal_mode < 0 || o.proposal_mode > 2)
        return fail(nullptr, LDA_ERR_ARG, "lda_init: proposal_mode must be 0, 1 or 2");
    if (o.dense_rows < -1 || o.dense_alias_min_count < 0 || o.sweep_chunk_tokens < 0 ||
        o.sweep_block_threads < 0 || o.rebuild_tile_tokens < 0 || o.time_sweep_passes < 0 ||
        o.time_sweep_passes > 1)
        return fail(nullptr, LDA_ERR_ARG, "lda_init: option out of range");
    if (o.doc_refresh < 0 || o.doc_refresh > 1)
        return fail(nullptr, LDA_ERR_ARG, "lda_init: doc_refresh must be 0 or 1");
    if (o.stream_block_tokens < 0 || (o.stream_block_tokens > 0 && o.doc_refresh))
        return fail(nullptr, LDA_ERR_ARG, "lda_init: stream_block_tokens must be >= 0, and 0 with doc_refresh");
    for (int i = 0; i < 5; ++i)
        if (o.reserved[i] != 0) return fail(nullptr, LDA_ERR_ARG, "lda_init: reserved option set");
    if (o.record_bucket_tokens < -1 ||
        (o.record_bucket_tokens > 0 && (o.record_bucket_tokens & (o.record_bucket_tokens - 1)) != 0))
        return fail(nullptr, LDA_ERR_ARG, "lda_init: record_bucket_tokens must be a power of two");
    if ((o.dev_alloc == nullptr) != (o.dev_free == nullptr))
        return fail(nullptr, LDA_ERR_ARG, "lda_init: dev_alloc and dev_free must be set together");
    // The kernels of the all-dense case keep a whole row or table in LDS; beyond their K the
    // general ones (topic ranges, tables in a global workspace) take over, with every row dense.
    const bool hybrid = (o.dense_rows != 0) || (o.dense_alias_min_count != 0) ||
                        K > max_alias_topics() || K > max_rebuild_topics();
    const int32_t H = o.dense_rows < 0 ? 0 : (o.dense_rows == 0 ? V : std::min(o.dense_rows, V));
    if (K > kMaxPackedTopics)
        return fail(nullptr, LDA_ERR_UNSUPPORTED, "lda_init: K must be < 2^20 - 1");
    if ((double)H * (double)K > 1.0e10)
        return fail(nullptr, LDA_ERR_UNSUPPORTED, "lda_init: %d dense rows of %d topics are too large",
                    H, K);

    lda_ctx* c = new (std::nothrow) lda_ctx();
    if (!c) return fail(nullptr, LDA_ERR_OOM, "lda_init: host allocation failed");
    c->D = D; c->N = N; c->V = V; c->K = K;
    c->alpha = alpha; c->beta = beta;
    c->alphabar = (double)K * alpha;
    c->betabar = (double)V * beta;
    c->seed = seed;
    c->opt = o;
    c->hybrid = hybrid;
    c->H = H;
    {   // order of the records the sweep's two passes exchange (layout.hip, launch_layout)
        int32_t bucket = o.record_bucket_tokens;
        // default: buckets for a large corpus on the all-dense store, where the doc pass gains
        // more than the word pass and the rebuild lose (measured: 7 * 10^8 tokens gain, 10^8
        // tokens and the hybrid store lose a few percent)
        if (bucket == 0) bucket = (H == V && N >= ((int64_t)1 << 28)) ? (1 << 22) : -1;
        if (o.stream_block_tokens > 0) bucket = -1;  // the two-pass sweep's records do not exist
        c->record_bucket_shift = 0;
        if (bucket > 0 && (int64_t)bucket < N)
            while ((1 << c->record_bucket_shift) < bucket) ++c->record_bucket_shift;
        else
            c->record_bucket_shift = -1;  // one bucket
    }
    c->stream = reinterpret_cast<hipStream_t>(o.hip_stream);

    // sweep tiling parameters (LDS: 12 bytes per token + 4 per document).  A packed n_kd
    // slot holds counts up to 4095, a token's slot index takes 12 bits and its document index
    // one byte, which bound the tile.
    // default tile: 1024 tokens / 512 threads, for every K (with n_k gathered from L2 instead
    // of copied to LDS, 512-token tiles of 256 threads were a fifth slower at K = 10^5)
    c->chunk_tokens = o.sweep_chunk_tokens > 0 ? o.sweep_chunk_tokens : 1024;
    c->chunk_tokens = std::max(64, std::min((c->chunk_tokens / 64) * 64, (int)kMaxTileTokens / 64 * 64));
    c->chunk_docs = std::max(16, std::min(255, c->chunk_tokens / 4));
    c->sweep_block = o.sweep_block_threads > 0 ? o.sweep_block_threads
                                               : (o.sweep_chunk_tokens == 0 ? 512 : 256);
    c->sweep_block = std::max(64, std::min(1024, (c->sweep_block / 64) * 64));
    // a thread carries at most 8 tokens of its tile
    c->sweep_block = std::max(c->sweep_block, ((c->chunk_tokens + 7) / 8 + 63) / 64 * 64);
    const int32_t tile_tokens = o.rebuild_tile_tokens > 0 ? o.rebuild_tile_tokens : 262144;
    c->rebuild_tile_tokens = tile_tokens;

    int rc = LDA_OK;
    auto bail = [&](int code) {
        free_all(c);
        delete c;
        return code;
    };

    try {
        c->h_doff.resize((size_t)D + 1);
    } catch (...) {
        return bail(fail(nullptr, LDA_ERR_OOM, "lda_init: host allocation failed"));
    }
    for (int64_t d = 0; d <= D; ++d) c->h_doff[d] = (int32_t)doc_offsets[d];
    for (int64_t d = 0; d < D; ++d) c->longest_doc = std::max(c->longest_doc, c->h_doff[d + 1] - c->h_doff[d]);
    if (o.doc_refresh && (hybrid || c->longest_doc > refresh_sweep_max_doc()))
        return bail(fail(nullptr, LDA_ERR_UNSUPPORTED,
                         "lda_init: doc_refresh needs the all-dense store with dense tables and "
                         "documents of at most %d tokens", refresh_sweep_max_doc()));

    std::vector<int32_t> chunk_doc;
    std::vector<int64_t> long_slot;
    build_doc_tiles(c->h_doff, D, c->chunk_tokens, c->chunk_docs, c->chunk_tokens, chunk_doc,
                    c->h_long_doc);
    c->n_chunks = (int32_t)chunk_doc.size() - 1;
    // chains of one or two steps leave room for 768-thread workgroups on tiles of 1536 tokens
    // (measured: 7 % faster doc pass at K = 10 000); longer chains need the registers
    std::vector<int32_t> chunk_doc2;
    if (o.sweep_chunk_tokens == 0 && o.sweep_block_threads == 0 && o.stream_block_tokens == 0) {
        std::vector<int32_t> same_long;
        c->chunk_tokens2 = 1536;
        c->chunk_docs2 = 255;
        c->sweep_block2 = 768;
        build_doc_tiles(c->h_doff, D, c->chunk_tokens2, c->chunk_docs2, c->chunk_tokens, chunk_doc2,
                        same_long);
        c->n_chunks2 = (int32_t)chunk_doc2.size() - 1;
    }
    c->n_long = (int32_t)c->h_long_doc.size();
    long_slot.resize((size_t)c->n_long + 1);
    long_slot[0] = 0;
    for (int32_t i = 0; i < c->n_long; ++i) {
        const int32_t d = c->h_long_doc[i];
        long_slot[i + 1] = long_slot[i] + 2 * (int64_t)(c->h_doff[d + 1] - c->h_doff[d]);
    }
    c->long_slots = long_slot[c->n_long];

    const size_t VK = (size_t)H * (size_t)K;  // dense rows (all V of them in the all-dense mode)
    bool any_dense_alias = true;  // refined below in the hybrid mode
#define TRY(x) do { rc = (x); if (rc != LDA_OK) return bail(rc); } while (0)
#define TRY_HIP(call)                                                                     \
    do {                                                                                  \
        hipError_t e__ = (call);                                                          \
        if (e__ != hipSuccess)                                                            \
            return bail(fail(nullptr, LDA_ERR_HIP, "%s: %s", #call, hipGetErrorString(e__))); \
    } while (0)
    if (!o.dev_alloc) prime_device_heap();
    TRY(dev_alloc(c, &c->d_word, (size_t)N, "word ids"));
    TRY(dev_alloc(c, &c->d_doff, (size_t)D + 1, "document offsets"));
    TRY(dev_alloc(c, &c->d_z, (size_t)N, "z"));
    TRY(dev_alloc(c, &c->d_znew, (size_t)N, "z (next)"));
    TRY(dev_alloc(c, &c->d_gid, (size_t)N, "word-major order"));
    TRY(dev_alloc(c, &c->d_wpos, (size_t)N, "word-major positions"));
    TRY(dev_alloc(c, &c->d_zt, (size_t)N, "word-major z"));
    c->zt_ints = (size_t)N;
    c->zt_pack16 = K <= 65536;
    c->zt_mask = c->zt_pack16 ? 0xFFFFu : 0xFFFFFFFFu;
    TRY(dev_alloc(c, &c->d_woff, (size_t)V + 1, "word offsets"));
    TRY(dev_alloc(c, &c->d_nkw, VK, "n_kw"));
    // rows of list-only words (kKindListOnly) are never written: all zero from here on
    if (hybrid) TRY_HIP(hipMemsetAsync(c->d_nkw, 0, sizeof(int32_t) * VK, c->stream));
    TRY(dev_alloc(c, &c->d_nk, (size_t)K + 3, "n_k"));  // read 16 bytes at a time by the doc pass
    TRY(dev_alloc(c, &c->d_cap, (size_t)V, "alias capacities"));
    TRY(dev_alloc(c, &c->d_chunk_doc, chunk_doc.size(), "document tiles"));
    TRY(dev_alloc(c, &c->d_chunk_tok, chunk_doc.size(), "document tiles"));
    TRY(dev_alloc(c, &c->d_tokdoc, (size_t)N, "token document indices"));
    if (c->n_chunks2 > 0) {
        TRY(dev_alloc(c, &c->d_chunk_doc2, chunk_doc2.size(), "document tiles"));
        TRY(dev_alloc(c, &c->d_chunk_tok2, chunk_doc2.size(), "document tiles"));
        TRY(dev_alloc(c, &c->d_tokdoc2, (size_t)N, "token document indices"));
    }
    TRY(dev_alloc(c, &c->d_long_doc, (size_t)c->n_long, "long documents"));
    TRY(dev_alloc(c, &c->d_long_slot, (size_t)c->n_long + 1, "long document slots"));
    TRY(dev_alloc(c, &c->d_long_keys, (size_t)c->long_slots, "long document tables"));
    TRY(dev_alloc(c, &c->d_long_cnts, (size_t)c->long_slots, "long document tables"));
    TRY(dev_alloc(c, &c->d_long_first, (size_t)c->long_slots, "long document tables"));
    c->n_partial = std::max(std::max(c->n_chunks, c->n_long), 4096);
    TRY(dev_alloc(c, &c->d_partial, (size_t)c->n_partial, "partial sums"));
    TRY(dev_alloc(c, &c->d_row, (size_t)K, "row staging"));
    TRY(dev_alloc(c, &c->d_flag, 4, "flags"));

    TRY_HIP(hipMemcpyAsync(c->d_word, word_ids, sizeof(int32_t) * (size_t)N, hipMemcpyHostToDevice,
                           c->stream));
    TRY_HIP(hipMemcpyAsync(c->d_doff, c->h_doff.data(), sizeof(int32_t) * ((size_t)D + 1),
                           hipMemcpyHostToDevice, c->stream));
    TRY_HIP(hipMemcpyAsync(c->d_chunk_doc, chunk_doc.data(), sizeof(int32_t) * chunk_doc.size(),
                           hipMemcpyHostToDevice, c->stream));
    std::vector<int32_t> chunk_tok(chunk_doc.size()), chunk_tok2(chunk_doc2.size());
    for (size_t i = 0; i < chunk_doc.size(); ++i) chunk_tok[i] = c->h_doff[chunk_doc[i]];
    for (size_t i = 0; i < chunk_doc2.size(); ++i) chunk_tok2[i] = c->h_doff[chunk_doc2[i]];
    TRY_HIP(hipMemcpyAsync(c->d_chunk_tok, chunk_tok.data(), sizeof(int32_t) * chunk_tok.size(),
                           hipMemcpyHostToDevice, c->stream));
    if (c->n_chunks2 > 0) {
        TRY_HIP(hipMemcpyAsync(c->d_chunk_doc2, chunk_doc2.data(), sizeof(int32_t) * chunk_doc2.size(),
                               hipMemcpyHostToDevice, c->stream));
        TRY_HIP(hipMemcpyAsync(c->d_chunk_tok2, chunk_tok2.data(), sizeof(int32_t) * chunk_tok2.size(),
                               hipMemcpyHostToDevice, c->stream));
    }
    if (c->n_long > 0)
        TRY_HIP(hipMemcpyAsync(c->d_long_doc, c->h_long_doc.data(), sizeof(int32_t) * c->n_long,
                               hipMemcpyHostToDevice, c->stream));
    TRY_HIP(hipMemcpyAsync(c->d_long_slot, long_slot.data(), sizeof(int64_t) * long_slot.size(),
                           hipMemcpyHostToDevice, c->stream));
    TRY_HIP(hipStreamSynchronize(c->stream));

    bool ok = true;
    TRY(launch_check_range(c, c->d_word, N, 0, V, &ok));
    if (!ok) return bail(fail(nullptr, LDA_ERR_ARG, "lda_init: a word id is outside [0, V)"));

    TRY(launch_layout(c, word_ids));
    TRY(launch_tokdoc(c));

    // rebuild tiles from the word segment offsets
    std::vector<int32_t> woff((size_t)V + 1);
    TRY_HIP(hipMemcpy(woff.data(), c->d_woff, sizeof(int32_t) * ((size_t)V + 1),
                      hipMemcpyDeviceToHost));
    if (hybrid) {
        TRY(setup_hybrid(c, woff));
        any_dense_alias = c->n_dense_alias > 0;
    }
    TRY(setup_split_sweep(c, woff));
    TRY(dev_alloc(c, &c->d_alias, any_dense_alias ? VK : 1, "alias tables"));
    std::vector<RebuildTile> tiles;
    std::vector<int32_t> multi;
    tiles.reserve((size_t)H + 1024);
    for (int32_t w = 0; w < H; ++w) {
        const int32_t b = woff[w], e = woff[w + 1];
        if (e - b <= tile_tokens) {
            const int32_t form = !list_from_rebuild(c, w) ? 0 : ((c->h_wkind[w] & kKindListOnly) ? 3 : 2);
            tiles.push_back(RebuildTile{w, b, e, form});
        } else {
            multi.push_back(w);
            for (int32_t p = b; p < e; p += tile_tokens)
                tiles.push_back(RebuildTile{w, p, std::min(e, p + tile_tokens), 1});
        }
    }
    c->n_tiles = (int32_t)tiles.size();
    c->n_multi_words = (int32_t)multi.size();
    TRY(dev_alloc(c, &c->d_tiles, tiles.size(), "rebuild tiles"));
    TRY(dev_alloc(c, &c->d_multi_words, multi.size(), "multi-tile words"));
    TRY_HIP(hipMemcpy(c->d_tiles, tiles.data(), sizeof(RebuildTile) * tiles.size(),
                      hipMemcpyHostToDevice));
    if (!multi.empty())
        TRY_HIP(hipMemcpy(c->d_multi_words, multi.data(), sizeof(int32_t) * multi.size(),
                          hipMemcpyHostToDevice));

    TRY(hybrid ? launch_rebuild_hybrid(c) : launch_rebuild(c));
    TRY_HIP(hipStreamSynchronize(c->stream));
    if (o.stream_block_tokens > 0) {
        rc = enter_streamed_mode(c, chunk_doc);
        if (rc != LDA_OK) {
            leave_streamed_mode(c);
            return bail(rc);
        }
    }
#undef TRY
#undef TRY_HIP
    c->state = COUNTS_VALID;
    c->sweep_index = 0;
    *out = c;
    return LDA_OK;
}

int lda_build_alias(lda_ctx* c)
{
    if (!c) return LDA_ERR_ARG;
    if (c->state != COUNTS_VALID && c->state != ALIAS_VALID)
        return fail(c, LDA_ERR_STATE, "lda_build_alias: counts are stale (call lda_rebuild_counts)");
    int rc;
    if (c->hybrid) {
        rc = launch_alias_build_hybrid(c);
    } else {
        rc = launch_alias_build(c);
    }
    if (rc == LDA_OK) c->state = ALIAS_VALID;
    return rc;
}

int lda_sweep(lda_ctx* c, int32_t mh_steps)
{
    if (!c) return LDA_ERR_ARG;
    if (mh_steps < 1) return fail(c, LDA_ERR_ARG, "lda_sweep: mh_steps must be >= 1");
    if (c->state != ALIAS_VALID)
        return fail(c, LDA_ERR_STATE, "lda_sweep: needs fresh alias tables (call lda_build_alias)");
    if (c->sweep_index == 0xFFFFFFFEu) return fail(c, LDA_ERR_STATE, "lda_sweep: sweep index exhausted");
    int rc;
    if (c->streamed) {
        rc = launch_sweep_streamed(c, mh_steps);
        c->pass_ev_recorded = false;
        if (rc != LDA_OK) return rc;
        std::swap(c->h_z, c->h_znew);
        c->sweep_index += 1;
        c->state = SWEPT;
        c->prev_valid = false;
        return LDA_OK;
    }
    if (c->opt.doc_refresh) {
        rc = launch_sweep_doc_refresh(c, mh_steps, c->longest_doc);
        c->zt_current = false;  // only the doc-major assignment is written
        c->td_valid = false;
        c->pass_ev_recorded = false;
    } else if (split_sweep_supported(c, mh_steps)) {
        rc = launch_sweep_split(c, mh_steps);
    } else {
        rc = c->hybrid ? launch_sweep_hybrid(c, mh_steps) : launch_sweep(c, mh_steps);
        c->zt_current = false;  // the fused kernels write the doc-major assignment only
        c->td_valid = false;
        c->pass_ev_recorded = false;
    }
    if (rc != LDA_OK) return rc;
    std::swap(c->d_z, c->d_znew);
    c->sweep_index += 1;
    c->state = SWEPT;
    c->prev_valid = true;
    return LDA_OK;
}

int lda_sweep_pass_ms(lda_ctx* c, float* word_pass_ms, float* doc_pass_ms)
{
    if (!c) return LDA_ERR_ARG;
    if (!word_pass_ms || !doc_pass_ms) return fail(c, LDA_ERR_ARG, "lda_sweep_pass_ms: NULL pointer");
    if (!c->opt.time_sweep_passes || !c->pass_ev_recorded)
        return fail(c, LDA_ERR_STATE, "lda_sweep_pass_ms: no timed two-pass sweep has run");
    LDA_HIP(c, hipEventSynchronize(c->pass_ev[2]));
    LDA_HIP(c, hipEventElapsedTime(word_pass_ms, c->pass_ev[0], c->pass_ev[1]));
    LDA_HIP(c, hipEventElapsedTime(doc_pass_ms, c->pass_ev[1], c->pass_ev[2]));
    return LDA_OK;
}

int lda_rebuild_counts(lda_ctx* c)
{
    if (!c) return LDA_ERR_ARG;
    const int rc = c->hybrid ? launch_rebuild_hybrid(c) : launch_rebuild(c);
    if (rc == LDA_OK) c->state = COUNTS_VALID;
    c->prev_valid = false;
    return rc;
}

int lda_update_counts(lda_ctx* c)
{
    if (!c) return LDA_ERR_ARG;
    if (c->streamed)
        return fail(c, LDA_ERR_UNSUPPORTED, "lda_update_counts: not with streamed data blocks");
    if (c->hybrid)
        return fail(c, LDA_ERR_UNSUPPORTED,
                    "lda_update_counts: needs the all-dense store with dense tables (lists and hash "
                    "rows are only made by lda_rebuild_counts)");
    if (c->state != SWEPT || !c->prev_valid)
        return fail(c, LDA_ERR_STATE, "lda_update_counts: needs the state left by lda_sweep");
    const int rc = launch_update_counts(c);
    c->prev_valid = false;
    if (rc == LDA_OK) c->state = COUNTS_VALID;
    return rc;
}

int lda_loglik(lda_ctx* c, double* total, double* doc_part, double* word_part)
{
    if (!c) return LDA_ERR_ARG;
    if (!total) return fail(c, LDA_ERR_ARG, "lda_loglik: total is NULL");
    if (c->state != COUNTS_VALID && c->state != ALIAS_VALID)
        return fail(c, LDA_ERR_STATE, "lda_loglik: counts are stale (call lda_rebuild_counts)");
    double d = 0.0, w = 0.0;
    const int rc = launch_loglik(c, &d, &w);
    if (rc != LDA_OK) return rc;
    if (doc_part) *doc_part = d;
    if (word_part) *word_part = w;
    *total = d + w;
    return LDA_OK;
}

int64_t lda_num_tokens(const lda_ctx* c) { return c ? c->N : -1; }
int64_t lda_sweep_index(const lda_ctx* c) { return c ? (int64_t)c->sweep_index : -1; }

int lda_get_z(lda_ctx* c, int32_t* z)
{
    if (!c) return LDA_ERR_ARG;
    if (!z) return fail(c, LDA_ERR_ARG, "lda_get_z: NULL buffer");
    if (c->streamed) return streamed_get_z(c, z);
    LDA_HIP(c, hipMemcpyAsync(z, c->d_z, sizeof(int32_t) * (size_t)c->N, hipMemcpyDeviceToHost,
                              c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    return LDA_OK;
}

int lda_set_z(lda_ctx* c, const int32_t* z, int64_t next_sweep_index)
{
    if (!c) return LDA_ERR_ARG;
    if (!z) return fail(c, LDA_ERR_ARG, "lda_set_z: NULL buffer");
    if (next_sweep_index < 0 || next_sweep_index > 0xFFFFFFFELL)
        return fail(c, LDA_ERR_ARG, "lda_set_z: sweep index out of range");
    if (c->streamed) {
        const int rc = streamed_set_z(c, z);
        if (rc != LDA_OK) return rc;
        c->td_valid = false;
        c->prev_valid = false;
        c->sweep_index = (uint32_t)next_sweep_index;
        c->state = SWEPT;
        return LDA_OK;
    }
    // stage in the spare buffer, validate, then adopt
    LDA_HIP(c, hipMemcpyAsync(c->d_znew, z, sizeof(int32_t) * (size_t)c->N, hipMemcpyHostToDevice,
                              c->stream));
    bool ok = true;
    const int rc = launch_check_range(c, c->d_znew, c->N, 0, c->K, &ok);
    if (rc != LDA_OK) return rc;
    if (!ok) return fail(c, LDA_ERR_ARG, "lda_set_z: a topic is outside [0, K)");
    std::swap(c->d_z, c->d_znew);
    c->zt_current = false;
    c->td_valid = false;
    c->prev_valid = false;
    c->sweep_index = (uint32_t)next_sweep_index;
    c->state = SWEPT;
    return LDA_OK;
}

int lda_get_nk(lda_ctx* c, int32_t* nk)
{
    if (!c) return LDA_ERR_ARG;
    if (!nk) return fail(c, LDA_ERR_ARG, "lda_get_nk: NULL buffer");
    if (c->state == SWEPT) return fail(c, LDA_ERR_STATE, "lda_get_nk: counts are stale");
    LDA_HIP(c, hipMemcpyAsync(nk, c->d_nk, sizeof(int32_t) * (size_t)c->K, hipMemcpyDeviceToHost,
                              c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    return LDA_OK;
}

int lda_get_nkw_row(lda_ctx* c, int32_t w, int32_t* row)
{
    if (!c) return LDA_ERR_ARG;
    if (!row || w < 0 || w >= c->V) return fail(c, LDA_ERR_ARG, "lda_get_nkw_row: bad argument");
    if (c->state == SWEPT) return fail(c, LDA_ERR_STATE, "lda_get_nkw_row: counts are stale");
    if (c->hybrid && (!(c->h_wkind[w] & 1) || (c->h_wkind[w] & kKindListOnly))) {  // densify its list
        int32_t nnz = 0;
        LDA_HIP(c, hipMemcpyAsync(&nnz, c->d_sp_nnz + w, sizeof(int32_t), hipMemcpyDeviceToHost,
                                  c->stream));
        LDA_HIP(c, hipStreamSynchronize(c->stream));
        std::vector<int32_t> t((size_t)nnz), n((size_t)nnz);
        if (nnz > 0) {
            LDA_HIP(c, hipMemcpy(t.data(), c->d_sp_topic + c->h_sp_off[w], sizeof(int32_t) * nnz,
                                 hipMemcpyDeviceToHost));
            LDA_HIP(c, hipMemcpy(n.data(), c->d_sp_count + c->h_sp_off[w], sizeof(int32_t) * nnz,
                                 hipMemcpyDeviceToHost));
        }
        memset(row, 0, sizeof(int32_t) * (size_t)c->K);
        for (int32_t i = 0; i < nnz; ++i) row[t[i]] = n[i];
        return LDA_OK;
    }
    LDA_HIP(c, hipMemcpyAsync(row, c->d_nkw + (size_t)w * (size_t)c->K,
                              sizeof(int32_t) * (size_t)c->K, hipMemcpyDeviceToHost, c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    return LDA_OK;
}

int lda_get_ndk_row(lda_ctx* c, int64_t d, int32_t* row)
{
    if (!c) return LDA_ERR_ARG;
    if (!row || d < 0 || d >= c->D) return fail(c, LDA_ERR_ARG, "lda_get_ndk_row: bad argument");
    const int rc = launch_ndk_row(c, d);
    if (rc != LDA_OK) return rc;
    LDA_HIP(c, hipMemcpyAsync(row, c->d_row, sizeof(int32_t) * (size_t)c->K, hipMemcpyDeviceToHost,
                              c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    return LDA_OK;
}

int lda_get_alias_row(lda_ctx* c, int32_t w, uint32_t* split, uint32_t* alias, uint32_t* cap)
{
    if (!c) return LDA_ERR_ARG;
    if (!split || !alias || !cap || w < 0 || w >= c->V)
        return fail(c, LDA_ERR_ARG, "lda_get_alias_row: bad argument");
    if (c->state != ALIAS_VALID) return fail(c, LDA_ERR_STATE, "lda_get_alias_row: no valid tables");
    if (c->hybrid && !(c->h_wkind[w] & 2))
        return fail(c, LDA_ERR_ARG, "lda_get_alias_row: word %d draws from the mixture", w);
    std::vector<uint4> h((size_t)c->K);
    LDA_HIP(c, hipMemcpyAsync(h.data(), c->d_alias + (size_t)w * (size_t)c->K,
                              sizeof(uint4) * (size_t)c->K, hipMemcpyDeviceToHost, c->stream));
    if (c->hybrid) {
        uint4 m;
        LDA_HIP(c, hipMemcpyAsync(&m, c->d_metaA + 2 * (size_t)w, sizeof(uint4), hipMemcpyDeviceToHost, c->stream));
        LDA_HIP(c, hipStreamSynchronize(c->stream));
        *cap = m.y;
    } else {
        LDA_HIP(c, hipMemcpyAsync(cap, c->d_cap + w, sizeof(uint32_t), hipMemcpyDeviceToHost,
                                  c->stream));
    }
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    for (int32_t k = 0; k < c->K; ++k) {
        split[k] = h[k].x;
        alias[k] = h[k].y;
    }
    return LDA_OK;
}

int lda_get_sparse_table(lda_ctx* c, int32_t w, int32_t cap_entries, int32_t* n, int32_t* topics,
                         uint32_t* split, int32_t* alias_topic, uint32_t* cap, uint64_t* mass)
{
    if (!c) return LDA_ERR_ARG;
    if (!n || w < 0 || w >= c->V || cap_entries < 0)
        return fail(c, LDA_ERR_ARG, "lda_get_sparse_table: bad argument");
    if (c->state != ALIAS_VALID) return fail(c, LDA_ERR_STATE, "lda_get_sparse_table: no valid tables");
    if (!c->hybrid || (c->h_wkind[w] & 2))
        return fail(c, LDA_ERR_ARG, "lda_get_sparse_table: word %d draws from a dense table", w);
    uint4 m;
    LDA_HIP(c, hipMemcpyAsync(&m, c->d_metaA + 2 * (size_t)w, sizeof(uint4), hipMemcpyDeviceToHost, c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    *n = (int32_t)m.x;
    if (cap) *cap = m.y;
    if (mass) *mass = ((uint64_t)m.w << 32) | m.z;
    if ((int32_t)m.x <= cap_entries && m.x > 0 && topics && split && alias_topic) {
        std::vector<uint4> e((size_t)m.x);
        LDA_HIP(c, hipMemcpy(e.data(), c->d_ma + (size_t)c->h_sp_off[w],
                             sizeof(uint4) * e.size(), hipMemcpyDeviceToHost));
        for (uint32_t i = 0; i < m.x; ++i) {
            int32_t cnt;
            split[i] = e[i].x;
            unpack_mix_bin(e[i], true, topics[i], cnt);
            unpack_mix_bin(e[i], false, alias_topic[i], cnt);
        }
    }
    return LDA_OK;
}

int lda_get_beta_table(lda_ctx* c, uint32_t* split, uint32_t* alias, uint32_t* cap, uint64_t* mass)
{
    if (!c) return LDA_ERR_ARG;
    if (!split || !alias || !cap || !mass) return fail(c, LDA_ERR_ARG, "lda_get_beta_table: NULL buffer");
    if (c->state != ALIAS_VALID || !c->hybrid || c->n_mix == 0)
        return fail(c, LDA_ERR_STATE, "lda_get_beta_table: no mixture tables");
    std::vector<uint2> e((size_t)c->K);
    uint64_t hdr[2];
    LDA_HIP(c, hipMemcpyAsync(e.data(), c->d_beta_alias, sizeof(uint2) * (size_t)c->K,
                              hipMemcpyDeviceToHost, c->stream));
    LDA_HIP(c, hipMemcpyAsync(hdr, c->d_beta_hdr, sizeof(hdr), hipMemcpyDeviceToHost, c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    for (int32_t k = 0; k < c->K; ++k) {
        split[k] = e[k].x;
        alias[k] = e[k].y;
    }
    *mass = hdr[0];
    *cap = (uint32_t)hdr[1];
    return LDA_OK;
}

int lda_sync(lda_ctx* c)
{
    if (!c) return LDA_ERR_ARG;
    if (c->streamed) return streamed_sync(c);
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    return LDA_OK;
}

const char* lda_last_error(const lda_ctx* c)
{
    return c ? c->err.c_str() : g_init_error.c_str();
}

void lda_destroy(lda_ctx* c)
{
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    leave_streamed_mode(c);
    free_all(c);
    delete c;
}

}  // extern "C"
