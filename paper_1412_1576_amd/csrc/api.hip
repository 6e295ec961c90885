// C ABI of the library (see include/lda_mi355x.h): argument checks, the state
// machine, device allocations and the host-side tiling tables.  All arithmetic of
// the method runs in the kernels of alias.hip, sweep.hip, rebuild.hip, loglik.hip.
#include <algorithm>
#include <cstring>

#include "common.hpp"
#include "doc_tile.hpp"

namespace lda {

static thread_local std::string g_init_error;

void set_init_error(const char* msg) { g_init_error = msg; }

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

namespace {

template <class T>
int dev_alloc(lda_ctx* c, T** p, size_t count, const char* what)
{
    *p = nullptr;
    const size_t bytes = sizeof(T) * (count ? count : 1);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(p), bytes);
    if (e != hipSuccess) {
        *p = nullptr;
        (void)hipGetLastError();
        return fail(c, LDA_ERR_OOM, "device allocation of %zu bytes for %s failed: %s", bytes, what,
                    hipGetErrorString(e));
    }
    return LDA_OK;
}

template <class T>
void dev_free(T*& p)
{
    if (p) (void)hipFree(p);
    p = nullptr;
}

void free_all(lda_ctx* c)
{
    dev_free(c->d_word); dev_free(c->d_doff); dev_free(c->d_z); dev_free(c->d_znew);
    dev_free(c->d_gid); dev_free(c->d_woff); dev_free(c->d_nkw); dev_free(c->d_nk);
    dev_free(c->d_alias); dev_free(c->d_cap); dev_free(c->d_chunk_doc); dev_free(c->d_tokdoc); dev_free(c->d_long_doc);
    dev_free(c->d_long_slot); dev_free(c->d_long_keys); dev_free(c->d_long_cnts);
    dev_free(c->d_tiles); dev_free(c->d_multi_words); dev_free(c->d_partial); dev_free(c->d_row);
    dev_free(c->d_flag);
}

// Greedy tiling of the documents: consecutive documents are grouped while they
// fit cap_tokens tokens and cap_docs documents.  A document longer than
// cap_tokens becomes a tile of its own and is also listed as "long".
void build_doc_tiles(const std::vector<int32_t>& doff, int64_t D, int32_t cap_tokens,
                     int32_t cap_docs, std::vector<int32_t>& chunk_doc,
                     std::vector<int32_t>& long_doc)
{
    chunk_doc.clear();
    long_doc.clear();
    chunk_doc.push_back(0);
    int32_t cur_tok = 0, cur_docs = 0;
    for (int64_t d = 0; d < D; ++d) {
        const int32_t L = doff[d + 1] - doff[d];
        if (L > cap_tokens) {
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
    if (N > 2147483646LL) return fail(nullptr, LDA_ERR_ARG, "lda_init: N must be < 2^31 - 1");
    lda_options o{};
    if (opt) o = *opt;
    if (o.proposal_mode < 0 || o.proposal_mode > 2)
        return fail(nullptr, LDA_ERR_ARG, "lda_init: proposal_mode must be 0, 1 or 2");
    if (o.dense_rows < 0 || o.dense_alias_min_count < 0 || o.sweep_chunk_tokens < 0 ||
        o.sweep_block_threads < 0 || o.rebuild_tile_tokens < 0)
        return fail(nullptr, LDA_ERR_ARG, "lda_init: negative option");
    for (int i = 0; i < 9; ++i)
        if (o.reserved[i] != 0) return fail(nullptr, LDA_ERR_ARG, "lda_init: reserved option set");
    if (o.dense_rows != 0 || o.dense_alias_min_count != 0)
        return fail(nullptr, LDA_ERR_UNSUPPORTED,
                    "lda_init: hybrid rows / mixture proposal are not available in this build");
    if (K > kMaxPackedTopics)
        return fail(nullptr, LDA_ERR_UNSUPPORTED, "lda_init: K must be < 2^20");
    if (K > max_alias_topics() || K > max_rebuild_topics())
        return fail(nullptr, LDA_ERR_UNSUPPORTED, "lda_init: K = %d exceeds the dense-path limit %d",
                    K, std::min(max_alias_topics(), max_rebuild_topics()));
    if ((double)V * (double)K > 4.0e10)
        return fail(nullptr, LDA_ERR_UNSUPPORTED, "lda_init: dense V*K too large");

    lda_ctx* c = new (std::nothrow) lda_ctx();
    if (!c) return fail(nullptr, LDA_ERR_OOM, "lda_init: host allocation failed");
    c->D = D; c->N = N; c->V = V; c->K = K;
    c->alpha = alpha; c->beta = beta;
    c->alphabar = (double)K * alpha;
    c->betabar = (double)V * beta;
    c->seed = seed;
    c->opt = o;
    c->stream = reinterpret_cast<hipStream_t>(o.hip_stream);

    // sweep tiling parameters (LDS: 12 bytes per token + 4 per document).  A packed n_kd
    // slot holds counts up to 4095, a token's slot index takes 12 bits and its document index
    // one byte, which bound the tile.
    c->chunk_tokens = o.sweep_chunk_tokens > 0 ? o.sweep_chunk_tokens : 512;
    c->chunk_tokens = std::max(64, std::min((c->chunk_tokens / 64) * 64, (int)kMaxTileTokens / 64 * 64));
    c->chunk_docs = std::max(16, std::min(255, c->chunk_tokens / 4));
    c->sweep_block = o.sweep_block_threads > 0 ? o.sweep_block_threads : 256;
    c->sweep_block = std::max(64, std::min(1024, (c->sweep_block / 64) * 64));
    // a thread carries at most 8 tokens of its tile
    c->sweep_block = std::max(c->sweep_block, ((c->chunk_tokens + 7) / 8 + 63) / 64 * 64);
    const int32_t tile_tokens = o.rebuild_tile_tokens > 0 ? o.rebuild_tile_tokens : 262144;

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

    std::vector<int32_t> chunk_doc;
    std::vector<int64_t> long_slot;
    build_doc_tiles(c->h_doff, D, c->chunk_tokens, c->chunk_docs, chunk_doc, c->h_long_doc);
    c->n_chunks = (int32_t)chunk_doc.size() - 1;
    c->n_long = (int32_t)c->h_long_doc.size();
    long_slot.resize((size_t)c->n_long + 1);
    long_slot[0] = 0;
    for (int32_t i = 0; i < c->n_long; ++i) {
        const int32_t d = c->h_long_doc[i];
        long_slot[i + 1] = long_slot[i] + 2 * (int64_t)(c->h_doff[d + 1] - c->h_doff[d]);
    }
    c->long_slots = long_slot[c->n_long];

    const size_t VK = (size_t)V * (size_t)K;
#define TRY(x) do { rc = (x); if (rc != LDA_OK) return bail(rc); } while (0)
#define TRY_HIP(call)                                                                     \
    do {                                                                                  \
        hipError_t e__ = (call);                                                          \
        if (e__ != hipSuccess)                                                            \
            return bail(fail(nullptr, LDA_ERR_HIP, "%s: %s", #call, hipGetErrorString(e__))); \
    } while (0)
    TRY(dev_alloc(c, &c->d_word, (size_t)N, "word ids"));
    TRY(dev_alloc(c, &c->d_doff, (size_t)D + 1, "document offsets"));
    TRY(dev_alloc(c, &c->d_z, (size_t)N, "z"));
    TRY(dev_alloc(c, &c->d_znew, (size_t)N, "z (next)"));
    TRY(dev_alloc(c, &c->d_gid, (size_t)N, "word-major order"));
    TRY(dev_alloc(c, &c->d_woff, (size_t)V + 1, "word offsets"));
    TRY(dev_alloc(c, &c->d_nkw, VK, "n_kw"));
    TRY(dev_alloc(c, &c->d_nk, (size_t)K, "n_k"));
    TRY(dev_alloc(c, &c->d_alias, VK, "alias tables"));
    TRY(dev_alloc(c, &c->d_cap, (size_t)V, "alias capacities"));
    TRY(dev_alloc(c, &c->d_chunk_doc, chunk_doc.size(), "document tiles"));
    TRY(dev_alloc(c, &c->d_tokdoc, (size_t)N, "token document indices"));
    TRY(dev_alloc(c, &c->d_long_doc, (size_t)c->n_long, "long documents"));
    TRY(dev_alloc(c, &c->d_long_slot, (size_t)c->n_long + 1, "long document slots"));
    TRY(dev_alloc(c, &c->d_long_keys, (size_t)c->long_slots, "long document tables"));
    TRY(dev_alloc(c, &c->d_long_cnts, (size_t)c->long_slots, "long document tables"));
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
    std::vector<RebuildTile> tiles;
    std::vector<int32_t> multi;
    tiles.reserve((size_t)V + 1024);
    for (int32_t w = 0; w < V; ++w) {
        const int32_t b = woff[w], e = woff[w + 1];
        if (e - b <= tile_tokens) {
            tiles.push_back(RebuildTile{w, b, e, 0});
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

    TRY(launch_rebuild(c));
    TRY_HIP(hipStreamSynchronize(c->stream));
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
    const int rc = launch_alias_build(c);
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
    const int rc = launch_sweep(c, mh_steps);
    if (rc != LDA_OK) return rc;
    std::swap(c->d_z, c->d_znew);
    c->sweep_index += 1;
    c->state = SWEPT;
    return LDA_OK;
}

int lda_rebuild_counts(lda_ctx* c)
{
    if (!c) return LDA_ERR_ARG;
    const int rc = launch_rebuild(c);
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
    // stage in the spare buffer, validate, then adopt
    LDA_HIP(c, hipMemcpyAsync(c->d_znew, z, sizeof(int32_t) * (size_t)c->N, hipMemcpyHostToDevice,
                              c->stream));
    bool ok = true;
    const int rc = launch_check_range(c, c->d_znew, c->N, 0, c->K, &ok);
    if (rc != LDA_OK) return rc;
    if (!ok) return fail(c, LDA_ERR_ARG, "lda_set_z: a topic is outside [0, K)");
    std::swap(c->d_z, c->d_znew);
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
    std::vector<uint4> h((size_t)c->K);
    LDA_HIP(c, hipMemcpyAsync(h.data(), c->d_alias + (size_t)w * (size_t)c->K,
                              sizeof(uint4) * (size_t)c->K, hipMemcpyDeviceToHost, c->stream));
    LDA_HIP(c, hipMemcpyAsync(cap, c->d_cap + w, sizeof(uint32_t), hipMemcpyDeviceToHost, c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    for (int32_t k = 0; k < c->K; ++k) {
        split[k] = h[k].x;
        alias[k] = h[k].y;
    }
    return LDA_OK;
}

int lda_sync(lda_ctx* c)
{
    if (!c) return LDA_ERR_ARG;
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
    free_all(c);
    delete c;
}

}  // extern "C"
