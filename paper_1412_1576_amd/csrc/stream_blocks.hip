// Streamed data blocks (LightLDA Sec. 3: the corpus is cut into data blocks that are brought
// in one after the other while the model stays put; Sec. 6 "Token and Topic Indicator
// Storage", Fig. 7: loading the next block overlaps the sampling of the current one).
// Selected by lda_options.stream_block_tokens.
//
// Here the "disk" is pinned host memory and the model -- n_kw in its dense or hybrid form,
// n_k, the word-proposal tables -- stays in HBM.  A block is a run of whole document tiles of
// about stream_block_tokens tokens.  What travels with a block, every sweep, is its
// document-major token data: word ids, topics, and two static per-token indices (the token's
// place in the corpus-wide word-major order, its document's index inside its tile), 13 bytes
// per token to the device and 4 bytes per token (the new topics) back.  Two device buffers
// alternate: while the sweep kernel works on one, the next block is copied into the other on
// a stream of the library's own and the previous block's topics are copied out on a third
// (all of default priority, ordered by events).
//
// The sweep kernel of this mode is the fused one (sweep.hip): it needs no word-major
// arrays of the block, which would have to travel too, and a streamed sweep is bound by the
// host link, not by the kernel.  Tokens keep their corpus-wide positions -- the kernels are
// handed block buffers shifted by the block's first token -- so the Philox counters, and with
// them every result, are those of the resident run, bit for bit.
//
// The one per-token array that stays resident is the word-major copy of z (4 bytes per
// token): every block scatters its new topics into it, and the count rebuild -- dense rows,
// sparse rows, n_k -- runs on it unchanged once the last block is through.
#include <algorithm>
#include <cstring>

#include "common.hpp"
#include "doc_tile.hpp"

namespace lda {

namespace {

template <class T>
T* shifted(T* buf, int64_t first)  // buf[0] is element `first` of the corpus-wide array
{
    return reinterpret_cast<T*>(reinterpret_cast<uintptr_t>(buf) - (uintptr_t)first * sizeof(T));
}

int wait(lda_ctx* c, hipStream_t s, hipEvent_t e)
{
    LDA_HIP(c, hipStreamWaitEvent(s, e, 0));
    return LDA_OK;
}

// block b's token data into buffer k, on the load stream
int load_block(lda_ctx* c, int b, int k, bool with_words)
{
    const StreamBlock& B = c->blocks[b];
    BlockBuffer& U = c->buf[k];
    const size_t n = (size_t)(B.g1 - B.g0);
    hipStream_t s = c->load_stream;
    LDA_HIP(c, hipMemcpyAsync(U.z, c->h_z + B.g0, sizeof(int32_t) * n, hipMemcpyHostToDevice, s));
    LDA_HIP(c, hipMemcpyAsync(U.tokdoc, c->h_tokdoc + B.g0, n, hipMemcpyHostToDevice, s));
    if (with_words) {
        LDA_HIP(c, hipMemcpyAsync(U.word, c->h_word + B.g0, sizeof(int32_t) * n, hipMemcpyHostToDevice, s));
        LDA_HIP(c, hipMemcpyAsync(U.wpos, c->h_wpos + B.g0, sizeof(int32_t) * n, hipMemcpyHostToDevice, s));
    }
    LDA_HIP(c, hipEventRecord(U.loaded, s));
    return LDA_OK;
}

// Runs `work(b, k)` for every block on the context's stream, block b + 1 being loaded while
// block b is worked on.  store: the buffer's znew goes back to h_znew afterwards.
template <class Work>
int for_each_block(lda_ctx* c, bool with_words, bool store, Work work)
{
    int rc;
    // the buffers are free and h_z is complete once the previous pass has stored everything
    if (c->stored_all_recorded && (rc = wait(c, c->load_stream, c->stored_all)) != LDA_OK) return rc;
    // (nothing on the context's stream holds the loads back: the first blocks of a sweep travel
    // while the tables are still being built)
    const int nb = (int)c->blocks.size();
    for (int b = 0; b < nb; ++b) {
        const int k = b & 1;
        BlockBuffer& U = c->buf[k];
        if (b >= 2) {  // the buffer's previous block is worked on and, if it goes back, stored
            if ((rc = wait(c, c->load_stream, U.computed)) != LDA_OK) return rc;
            if (store && (rc = wait(c, c->load_stream, U.stored)) != LDA_OK) return rc;
        }
        if ((rc = load_block(c, b, k, with_words)) != LDA_OK) return rc;
        if ((rc = wait(c, c->stream, U.loaded)) != LDA_OK) return rc;
        if ((rc = work(b, k)) != LDA_OK) return rc;
        LDA_HIP(c, hipEventRecord(U.computed, c->stream));
        if (store) {
            const StreamBlock& B = c->blocks[b];
            if ((rc = wait(c, c->store_stream, U.computed)) != LDA_OK) return rc;
            LDA_HIP(c, hipMemcpyAsync(c->h_znew + B.g0, U.znew, sizeof(int32_t) * (size_t)(B.g1 - B.g0),
                                      hipMemcpyDeviceToHost, c->store_stream));
            LDA_HIP(c, hipEventRecord(U.stored, c->store_stream));
        }
    }
    // the next pass may reuse the buffers when this one has computed (and stored) everything
    LDA_HIP(c, hipEventRecord(c->pass_end, c->stream));
    if ((rc = wait(c, c->store_stream, c->pass_end)) != LDA_OK) return rc;
    LDA_HIP(c, hipEventRecord(c->stored_all, c->store_stream));
    c->stored_all_recorded = true;
    return LDA_OK;
}

// binds the block's buffers as the context's token arrays for the duration of `launch`
template <class Launch>
int with_block_bound(lda_ctx* c, int b, int k, Launch launch)
{
    const StreamBlock& B = c->blocks[b];
    const BlockBuffer& U = c->buf[k];
    int32_t *word = c->d_word, *z = c->d_z, *znew = c->d_znew, *chunk_doc = c->d_chunk_doc;
    uint8_t* tokdoc = c->d_tokdoc;
    const int32_t n_chunks = c->n_chunks;
    c->d_word = shifted(U.word, B.g0);
    c->d_z = shifted(U.z, B.g0);
    c->d_znew = shifted(U.znew, B.g0);
    c->d_tokdoc = shifted(U.tokdoc, B.g0);
    c->d_chunk_doc = chunk_doc + B.c0;
    c->n_chunks = B.c1 - B.c0;
    const int rc = launch();
    c->d_word = word; c->d_z = z; c->d_znew = znew; c->d_tokdoc = tokdoc;
    c->d_chunk_doc = chunk_doc; c->n_chunks = n_chunks;
    return rc;
}

}  // namespace

// Cuts the corpus into blocks of whole tiles, moves the per-token arrays to pinned host memory
// and leaves two block buffers on the device.  Called at the end of lda_init, with the whole
// corpus still resident (the layout of a corpus that does not fit would be made block by
// block on the host side of this boundary; not built).
int enter_streamed_mode(lda_ctx* c, const std::vector<int32_t>& chunk_doc)
{
    if (c->n_long > 0)
        return fail(c, LDA_ERR_UNSUPPORTED, "lda_init: stream_block_tokens needs documents of at most %d tokens",
                    c->chunk_tokens);
    const int64_t target = c->opt.stream_block_tokens;
    int64_t most = 0;
    {
        StreamBlock B{0, 0, 0, 0};
        for (int32_t ch = 0; ch < c->n_chunks; ++ch) {
            const int64_t end = c->h_doff[chunk_doc[ch + 1]];
            if (end - B.g0 >= target || ch + 1 == c->n_chunks) {
                B.c1 = ch + 1;
                B.g1 = end;
                if (B.g1 > B.g0) c->blocks.push_back(B);
                most = std::max(most, B.g1 - B.g0);
                B = StreamBlock{ch + 1, ch + 1, end, end};
            }
        }
    }
    if (c->blocks.empty()) return fail(c, LDA_ERR_ARG, "lda_init: no tokens to stream");
    c->max_block_tokens = most;
    const size_t N = (size_t)c->N;
    LDA_HIP(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_word), sizeof(int32_t) * N, hipHostMallocDefault));
    LDA_HIP(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_z), sizeof(int32_t) * N, hipHostMallocDefault));
    LDA_HIP(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_znew), sizeof(int32_t) * N, hipHostMallocDefault));
    LDA_HIP(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_wpos), sizeof(int32_t) * N, hipHostMallocDefault));
    LDA_HIP(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_tokdoc), N, hipHostMallocDefault));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    LDA_HIP(c, hipMemcpy(c->h_word, c->d_word, sizeof(int32_t) * N, hipMemcpyDeviceToHost));
    LDA_HIP(c, hipMemcpy(c->h_z, c->d_z, sizeof(int32_t) * N, hipMemcpyDeviceToHost));
    LDA_HIP(c, hipMemcpy(c->h_wpos, c->d_wpos, sizeof(int32_t) * N, hipMemcpyDeviceToHost));
    LDA_HIP(c, hipMemcpy(c->h_tokdoc, c->d_tokdoc, N, hipMemcpyDeviceToHost));
    // the per-token arrays leave the device; d_zt (the word-major z) stays
    device_free(c, c->d_word); c->d_word = nullptr;
    device_free(c, c->d_z); c->d_z = nullptr;
    device_free(c, c->d_znew); c->d_znew = nullptr;
    device_free(c, c->d_gid); c->d_gid = nullptr;
    device_free(c, c->d_wpos); c->d_wpos = nullptr;
    device_free(c, c->d_tokdoc); c->d_tokdoc = nullptr;
    for (BlockBuffer& U : c->buf) {
        LDA_ALLOC(c, &U.word, (size_t)most, "block buffer");
        LDA_ALLOC(c, &U.z, (size_t)most, "block buffer");
        LDA_ALLOC(c, &U.znew, (size_t)most, "block buffer");
        LDA_ALLOC(c, &U.wpos, (size_t)most, "block buffer");
        LDA_ALLOC(c, &U.tokdoc, (size_t)most, "block buffer");
        LDA_HIP(c, hipEventCreateWithFlags(&U.loaded, hipEventDisableTiming));
        LDA_HIP(c, hipEventCreateWithFlags(&U.computed, hipEventDisableTiming));
        LDA_HIP(c, hipEventCreateWithFlags(&U.stored, hipEventDisableTiming));
    }
    LDA_HIP(c, hipStreamCreateWithFlags(&c->load_stream, hipStreamNonBlocking));
    LDA_HIP(c, hipStreamCreateWithFlags(&c->store_stream, hipStreamNonBlocking));
    LDA_HIP(c, hipEventCreateWithFlags(&c->pass_begin, hipEventDisableTiming));
    LDA_HIP(c, hipEventCreateWithFlags(&c->pass_end, hipEventDisableTiming));
    LDA_HIP(c, hipEventCreateWithFlags(&c->stored_all, hipEventDisableTiming));
    c->streamed = true;
    return LDA_OK;
}

void leave_streamed_mode(lda_ctx* c)
{
    if (c->load_stream) (void)hipStreamSynchronize(c->load_stream);
    if (c->store_stream) (void)hipStreamSynchronize(c->store_stream);
    for (BlockBuffer& U : c->buf) {
        device_free(c, U.word); device_free(c, U.z); device_free(c, U.znew);
        device_free(c, U.wpos); device_free(c, U.tokdoc);
        if (U.loaded) (void)hipEventDestroy(U.loaded);
        if (U.computed) (void)hipEventDestroy(U.computed);
        if (U.stored) (void)hipEventDestroy(U.stored);
        U = BlockBuffer{};
    }
    for (hipEvent_t* e : {&c->pass_begin, &c->pass_end, &c->stored_all}) {
        if (*e) (void)hipEventDestroy(*e);
        *e = nullptr;
    }
    if (c->load_stream) (void)hipStreamDestroy(c->load_stream);
    if (c->store_stream) (void)hipStreamDestroy(c->store_stream);
    c->load_stream = c->store_stream = nullptr;
    if (c->h_word) (void)hipHostFree(c->h_word);
    if (c->h_z) (void)hipHostFree(c->h_z);
    if (c->h_znew) (void)hipHostFree(c->h_znew);
    if (c->h_wpos) (void)hipHostFree(c->h_wpos);
    if (c->h_tokdoc) (void)hipHostFree(c->h_tokdoc);
    c->h_word = c->h_z = c->h_znew = c->h_wpos = nullptr;
    c->h_tokdoc = nullptr;
}

// One sweep over all blocks; the new topics end up in h_znew (the caller swaps) and in the
// word-major copy.
int launch_sweep_streamed(lda_ctx* c, int32_t mh_steps)
{
    const int rc = for_each_block(c, true, true, [&](int b, int k) {
        int r = with_block_bound(c, b, k, [&]() {
            return c->hybrid ? launch_sweep_hybrid(c, mh_steps) : launch_sweep(c, mh_steps);
        });
        if (r != LDA_OK) return r;
        const StreamBlock& B = c->blocks[b];
        return launch_scatter_word_major(c, c->buf[k].znew, c->buf[k].wpos, B.g1 - B.g0);
    });
    if (rc != LDA_OK) return rc;
    c->zt_current = true;
    c->td_valid = false;
    return LDA_OK;
}

// Doc part of the log-likelihood: partial[tile] for every tile, block by block.
int launch_loglik_doc_streamed(lda_ctx* c, double* d_partial)
{
    return for_each_block(c, false, false, [&](int b, int k) {
        const StreamBlock& B = c->blocks[b];
        return with_block_bound(c, b, k, [&]() { return launch_loglik_doc_tiles(c, d_partial + B.c0); });
    });
}

// The assignment of the corpus from / to the pinned copy.
int streamed_get_z(lda_ctx* c, int32_t* z)
{
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->store_stream));
    std::memcpy(z, c->h_z, sizeof(int32_t) * (size_t)c->N);
    return LDA_OK;
}

int streamed_set_z(lda_ctx* c, const int32_t* z)
{
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->store_stream));
    for (int64_t g = 0; g < c->N; ++g)
        if (z[g] < 0 || z[g] >= c->K) return fail(c, LDA_ERR_ARG, "lda_set_z: a topic is outside [0, K)");
    std::memcpy(c->h_z, z, sizeof(int32_t) * (size_t)c->N);
    // the word-major copy, block by block (the topics travel as a block's z)
    const int rc = for_each_block(c, true, false, [&](int b, int k) {
        const StreamBlock& B = c->blocks[b];
        return launch_scatter_word_major(c, c->buf[k].z, c->buf[k].wpos, B.g1 - B.g0);
    });
    if (rc != LDA_OK) return rc;
    c->zt_current = true;
    return LDA_OK;
}

// z of document d in a block buffer, shifted so that the n_kd accessor's kernel finds it at
// its corpus-wide position
int streamed_doc_z(lda_ctx* c, int64_t d, const int32_t** z_shifted)
{
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->store_stream));
    LDA_HIP(c, hipStreamSynchronize(c->load_stream));
    const int64_t g0 = c->h_doff[d], g1 = c->h_doff[d + 1];
    if (g1 > g0)
        LDA_HIP(c, hipMemcpy(c->buf[0].z, c->h_z + g0, sizeof(int32_t) * (size_t)(g1 - g0), hipMemcpyHostToDevice));
    *z_shifted = shifted(c->buf[0].z, g0);
    return LDA_OK;
}

int streamed_sync(lda_ctx* c)
{
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->load_stream));
    LDA_HIP(c, hipStreamSynchronize(c->store_stream));
    return LDA_OK;
}

}  // namespace lda
