// Shared declarations of the gfx950 LightLDA library: context, launch helpers,
// and the small device routines every kernel uses (Philox4x32-10, mulhi).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/lda_mi355x.h"

namespace lda {

constexpr int kWave = 64;

enum State { COUNTS_VALID = 1, ALIAS_VALID = 2, SWEPT = 3 };

// One rebuild work item: a slice [p0, p1) of word w's word-major segment.
// Mixture tables are launched by size class so that a small table does not reserve a large
// table's LDS: list capacity of each class, 0 = the largest that fits LDS, -1 = any size (built
// in the global workspace).
constexpr int kMixClasses = 8;
constexpr int32_t kMixClassCap[kMixClasses] = {64, 256, 1024, 2048, 4096, 8192, 0, -1};

struct RebuildTile {
    int32_t w;
    int32_t p0;
    int32_t p1;
    int32_t multi;  // 1: the word has several tiles (row pre-zeroed, merged by atomics);
                    // 2: single tile of a mixture word, whose list of non-zeros is written too;
                    // 3: single tile of a list-only word (kKindListOnly): the list, not the row
};

// A tile of a partition pass (sparse_rows.hip): source positions [p0, p1) of segment seg (a
// long word, or the whole of z)
struct PartTile {
    int32_t seg;
    int32_t p0, p1;
};

// Streamed data blocks (stream_blocks.hip): tiles [c0, c1) = tokens [g0, g1) of the corpus
struct StreamBlock {
    int32_t c0, c1;
    int64_t g0, g1;
};

// One of the two device buffers a block is loaded into
struct BlockBuffer {
    int32_t* word = nullptr;
    int32_t* z = nullptr;
    int32_t* znew = nullptr;
    int32_t* wpos = nullptr;
    uint8_t* tokdoc = nullptr;
    hipEvent_t loaded = nullptr, computed = nullptr, stored = nullptr;
};

}  // namespace lda

struct lda_ctx {
    // problem
    int64_t D = 0, N = 0;
    int32_t V = 0, K = 0;
    double alpha = 0, beta = 0, alphabar = 0, betabar = 0;
    uint64_t seed = 0;
    lda_options opt{};
    hipStream_t stream = nullptr;
    int state = 0;
    uint32_t sweep_index = 0;
    bool prev_valid = false;  // d_znew holds the assignment before the last sweep
    int32_t longest_doc = 0;  // tokens of the longest document
    std::string err;

    // corpus, document-major (CSR order)
    int32_t* d_word = nullptr;  // [N] word id of token g
    int32_t* d_doff = nullptr;  // [D+1] token offset of document d
    int32_t* d_z = nullptr;     // [N] snapshot assignment
    int32_t* d_znew = nullptr;  // [N] next assignment
    // word-major view
    int32_t* d_gid = nullptr;   // [N] CSR position of the p-th token in word-major order
    int32_t* d_wpos = nullptr;  // [N] position of token g's records in zt / rec: its word-major
                                //     position (inverse of gid), mapped through d_xmap if set
    int32_t* d_xmap = nullptr;  // [N] word-major position -> record position (NULL: identity)
    int32_t record_bucket_shift = -1;  // records ordered by (CSR position >> shift, word-major
                                       // position); -1: by word-major position alone
    // Word-major token records of 2^zt_shift ints.  Fields: the token's z, then the topic that
    // doc step i of the coming sweep proposes for it (when td_valid); one int per field, or,
    // with zt_pack16 (K <= 65536), two 16-bit fields per int.  The z field is the low
    // zt_mask bits of the record's first int.
    int32_t* d_zt = nullptr;
    size_t zt_ints = 0;         // allocated ints
    int32_t zt_shift = 0;
    bool zt_pack16 = false;
    uint32_t zt_mask = 0xFFFFFFFFu;
    bool zt_current = false;    // record [0] equals d_z
    bool td_valid = false;      // the stored doc proposals are those of sweep td_sweep, drawn
    uint32_t td_sweep = 0;      //   from d_z, for a chain of td_nw word and td_nd doc steps
    int32_t td_nw = 0, td_nd = 0;
    // Word-pass output, word-major, 2^rec_shift ints per token (sweep_split.hip)
    int32_t* d_rec = nullptr;
    size_t rec_ints = 0;
    // Work lists of the word pass: items (w, p0, n, 0) whose rows are staged in LDS, and
    // pieces (w0, w1, p0, n) of several short words whose rows are gathered
    int4* d_row_items = nullptr;
    int4* d_mix_items = nullptr;  // items (w, p0, n, 0) of mixture words whose row is rebuilt in LDS
    int4* d_gather_pieces = nullptr;
    int32_t n_row_items = 0, n_mix_items = 0, n_gather_pieces = 0;
    // option time_sweep_passes: events before the word pass, between the passes and after
    // the doc pass's tile kernel
    hipEvent_t pass_ev[3] = {nullptr, nullptr, nullptr};
    bool pass_ev_recorded = false;
    int32_t* d_woff = nullptr;  // [V+1] segment offsets
    // model
    int32_t* d_nkw = nullptr;   // [V*K] word-topic counts (dense rows)
    int32_t* d_nk = nullptr;    // [K]
    uint4* d_alias = nullptr;   // [V*K] (split, alias, n_kw[bin], n_kw[alias]) per bin
    uint32_t* d_cap = nullptr;  // [V] bin capacity of the word's table
    // sweep tiling: chunk c covers documents [chunk_doc[c], chunk_doc[c+1])
    int32_t* d_chunk_doc = nullptr;
    int32_t* d_chunk_tok = nullptr;  // [n_chunks+1] first token of chunk c (= doff[chunk_doc[c]])
    uint8_t* d_tokdoc = nullptr;     // [N] index of the token's document inside its tile
    int32_t n_chunks = 0;
    int32_t chunk_tokens = 0, chunk_docs = 0, sweep_block = 0;
    // second tiling of the same documents with larger tiles, used by the doc pass of chains
    // of at most two steps (n_chunks2 == 0: not built).  A document is "long" under both
    // tilings when it exceeds chunk_tokens.
    int32_t* d_chunk_doc2 = nullptr;
    int32_t* d_chunk_tok2 = nullptr;
    uint8_t* d_tokdoc2 = nullptr;
    int32_t n_chunks2 = 0;
    int32_t chunk_tokens2 = 0, chunk_docs2 = 0, sweep_block2 = 0;
    // documents too long for an LDS tile: hashed in a global workspace
    int32_t* d_long_doc = nullptr;     // [n_long] document ids
    int64_t* d_long_slot = nullptr;    // [n_long+1] first hash slot of each long document
    int32_t* d_long_keys = nullptr;    // [total slots]
    int32_t* d_long_cnts = nullptr;
    int32_t* d_long_first = nullptr;   // [total slots] log-likelihood: first token of every topic
    int32_t n_long = 0;
    int64_t long_slots = 0;
    std::vector<int32_t> h_long_doc;
    // rebuild tiling
    lda::RebuildTile* d_tiles = nullptr;
    int32_t n_tiles = 0;
    int32_t rebuild_tile_tokens = 0;
    int32_t* d_multi_words = nullptr;  // words that own several tiles
    int32_t n_multi_words = 0;
    // hybrid store / mixture proposal (Sec. 4.2 and 5); all null in the all-dense mode
    bool hybrid = false;
    int32_t H = 0;                       // word ids [0, H) own a dense n_kw row
    int32_t* d_dense_alias_words = nullptr;  // words that draw from a dense K-bin table
    int32_t n_dense_alias = 0;
    int32_t n_mix = 0;                   // words that draw from the mixture
    // the mixture words by list capacity (kMixClassCap; the last class is built in the global
    // workspace)
    int32_t* d_mix_class[lda::kMixClasses] = {};
    int32_t n_mix_class[lda::kMixClasses] = {};
    int32_t* d_sparse_words = nullptr;   // words whose n_kw row lives as a list: sparse rows and
                                         // list-only words (the log-likelihood sums over these lists)
    int32_t n_sparse = 0;
    int32_t n_list_only = 0;             // words marked kKindListOnly
    int32_t* d_compact_words = nullptr;  // mixture words with a dense row (list made by compaction)
    int32_t n_compact = 0;
    uint32_t* d_sp_off = nullptr;        // [V+1] first list entry of word w (capacity min(c_w, K))
    int32_t* d_sp_topic = nullptr;       // non-zero topics of the word, ascending
    int32_t* d_sp_count = nullptr;       // their counts
    int32_t* d_sp_nnz = nullptr;         // [V] entries in use
    uint32_t* d_hs_off = nullptr;        // [V+1] first hash slot of word w (power-of-two capacity)
    uint2* d_hs = nullptr;               // (topic, count) slots, topic = -1: empty
    uint4* d_ma = nullptr;               // mixture tables: one packed bin per list entry
    // one 32-byte record per word, [2w] = (entries n, capacity C, QS low, QS high) rewritten by
    // every table build, [2w+1] = (list offset, hash offset, log2 hash slots, kind) fixed
    uint4* d_metaA = nullptr;            // [2V]
    uint4* d_metaB = nullptr;            // = d_metaA + 1 (not owned)
    uint2* d_beta_alias = nullptr;       // [K] shared table of the beta term (split, alias)
    uint64_t* d_beta_hdr = nullptr;      // [2] QB, capacity
    unsigned char* d_big_ws = nullptr;   // list memory of the workgroups that build big tables
    size_t big_ws_stride = 0;
    int32_t n_big_wg = 0;                // the shared beta table has one more slot of its own
    // the one-workgroup build of a large beta table runs beside the other table kernels
    hipStream_t side_stream = nullptr;
    hipEvent_t side_fork = nullptr, side_join = nullptr;
    bool side_pending = false;           // side_join recorded, not yet waited for
    int64_t total_list = 0, total_hash = 0;
    std::vector<int32_t> h_wcount;       // corpus frequency of every word
    std::vector<uint8_t> h_wkind;        // bit 0: dense row, bit 1: dense proposal table,
                                         // bit 2 (kKindListOnly): the dense row is allotted but
                                         // not kept -- see kKindListOnly
    std::vector<uint32_t> h_sp_off, h_hs_off;
    // sparse-row rebuild (sparse_rows.hip): words sorted in LDS, in three size classes; longer
    // words partitioned by topic range in d_long_part (segment of long word i at d_long_base[i])
    int32_t* d_sort_words[3] = {};
    int32_t n_sort_words[3] = {};
    int32_t* d_long_words = nullptr;
    uint32_t* d_long_base = nullptr;
    lda::PartTile* d_long_tiles = nullptr;
    lda::PartTile* d_fill_tiles = nullptr;  // tiles over the places of the long words' lists
    int32_t n_long_words = 0, n_long_tiles = 0, n_fill_tiles = 0;
    uint32_t long_word_tokens = 0;
    uint32_t max_hash_row = 0;           // slots of the largest hash row that is filled by atomics
    bool clear_all_hash_rows = false;    // those rows own most of d_hs: clear it in one go
    int32_t* d_long_part = nullptr;
    uint32_t* d_long_dcount = nullptr;   // [n_long_words * ranges] tokens per range (zero between rebuilds)
    uint32_t* d_long_dstart = nullptr;   // [n_long_words * (ranges + 1)]
    uint32_t* d_long_cursor = nullptr;
    uint32_t* d_long_nnzd = nullptr;     // non-zero topics per range
    uint32_t* d_long_lofs = nullptr;     // their exclusive prefix: list position of a range
    // n_k for very large K: z partitioned by topic range
    int32_t* d_nk_part = nullptr;
    lda::PartTile* d_nk_tiles = nullptr;
    int32_t n_nk_tiles = 0;
    uint32_t* d_nk_ranges = nullptr;
    // streamed data blocks: the per-token arrays live in pinned host memory and pass through two
    // device buffers; d_word, d_z, d_znew, d_gid, d_wpos, d_tokdoc are then NULL between calls
    bool streamed = false;
    std::vector<lda::StreamBlock> blocks;
    int64_t max_block_tokens = 0;
    int32_t *h_word = nullptr, *h_z = nullptr, *h_znew = nullptr, *h_wpos = nullptr;
    uint8_t* h_tokdoc = nullptr;
    lda::BlockBuffer buf[2];
    hipStream_t load_stream = nullptr, store_stream = nullptr;
    hipEvent_t pass_begin = nullptr, pass_end = nullptr, stored_all = nullptr;
    bool stored_all_recorded = false;
    // scratch
    double* d_partial = nullptr;       // per-block partial sums (log-likelihood)
    int32_t n_partial = 0;
    int32_t* d_row = nullptr;          // [max(K,1)] row staging for accessors
    int32_t* d_flag = nullptr;         // [4] validation flags
    // host copies of small layouts
    std::vector<int32_t> h_doff;
};

namespace lda {

int fail(lda_ctx* c, int code, const char* fmt, ...);

// Device memory of a context: the caller's allocator (lda_options) or hipMalloc / hipFree.
// device_malloc returns LDA_OK or records LDA_ERR_OOM; *p is NULL on failure.
int device_malloc(lda_ctx* c, void** p, size_t bytes, const char* what);
void device_free(lda_ctx* c, void* p);

template <class T>
int device_malloc(lda_ctx* c, T** p, size_t count, const char* what)
{
    return device_malloc(c, reinterpret_cast<void**>(p), sizeof(T) * (count ? count : 1), what);
}

#define LDA_ALLOC(ctx, ptr, count, what)                                                  \
    do {                                                                                  \
        const int rc__ = lda::device_malloc((ctx), (ptr), (size_t)(count), (what));       \
        if (rc__ != LDA_OK) return rc__;                                                  \
    } while (0)

#define LDA_HIP(ctx, call)                                                              \
    do {                                                                                \
        hipError_t e__ = (call);                                                        \
        if (e__ != hipSuccess)                                                          \
            return lda::fail((ctx), e__ == hipErrorOutOfMemory ? LDA_ERR_OOM : LDA_ERR_HIP, \
                             "%s: %s (%s:%d)", #call, hipGetErrorString(e__), __FILE__, __LINE__); \
    } while (0)

// launchers implemented in the kernel files
int launch_layout(lda_ctx* c, const int32_t* h_word);      // word-major order, woff, z init
int launch_alias_build(lda_ctx* c);
int launch_alias_build_hybrid(lda_ctx* c);
int launch_rebuild_hybrid(lda_ctx* c);
int launch_sweep_hybrid(lda_ctx* c, int32_t mh_steps);
int launch_loglik_word_hybrid(lda_ctx* c, double* word_part);
// A second stream of the library's own (default priority) for kernels that can run beside
// the caller's stream: fork (the side stream waits for everything queued on the caller's
// stream so far), launch on c->side_stream, side_stream_done, and later join (the caller's
// stream waits for the side stream).  One fork may be pending at a time.
int fork_side_stream(lda_ctx* c);
int side_stream_done(lda_ctx* c);
int join_side_stream(lda_ctx* c);
int max_lds_table_entries();  // largest alias table built in LDS

// Up to this many topics the doc pass keeps a copy of n_k in every workgroup's LDS.
constexpr int32_t kNkLdsTopics = 16384;

// slot of topic t in a hash row of 2^lg slots (multiplicative hashing, top bits)
__host__ __device__ inline uint32_t row_hash_slot(int32_t t, uint32_t lg)
{
    return ((uint32_t)t * 0x9E3779B1u) >> (32u - lg);
}

// A bin of a mixture word's own table in 16 bytes: the split height and, for each
// of its two outcomes, the topic (20 bits) and the word's count of it (28 bits).
constexpr uint32_t kMixTopicBits = 20, kMixCountBits = 28;
__host__ __device__ inline uint4 pack_mix_bin(uint32_t split, int32_t t_own, int32_t t_other,
                                              int32_t n_own, int32_t n_other)
{
    return make_uint4(split, (uint32_t)t_own | ((uint32_t)n_own << kMixTopicBits),
                      (uint32_t)t_other | ((uint32_t)n_other << kMixTopicBits),
                      ((uint32_t)n_own >> 12) | (((uint32_t)n_other >> 12) << 16));
}
// A mixture word with a dense row, at least kMixRowMinTokens tokens, K <= kMixRowTopics and a
// segment that fits one rebuild tile is served everywhere from its list of non-zeros: the
// word pass rebuilds its row in LDS from the list, the table build reads the list, the
// log-likelihood sums over it.  Rewriting its K-entry dense row at every count rebuild would
// be the largest write of the rebuild (c3: 5.4 of 6.4 GB) for nobody to read, so the row is
// left untouched (all zero since lda_init) and the word is marked with this bit; the rare
// lookup outside the word pass (fused sweep) searches the word's mixture table, whose bins
// are its non-zero topics in ascending order.
constexpr uint32_t kKindListOnly = 4u;
constexpr int32_t kMixRowTopics = 16384;   // largest K whose n_kw row a mixture item keeps in LDS
constexpr int32_t kMixRowMinTokens = 128;

__host__ __device__ inline void unpack_mix_bin(const uint4& e, bool own, int32_t& topic,
                                               int32_t& count)
{
    const uint32_t sel = own ? e.y : e.z;
    const uint32_t hi = own ? (e.w & 0xFFFFu) : (e.w >> 16);
    topic = (int32_t)(sel & ((1u << kMixTopicBits) - 1u));
    count = (int32_t)((sel >> kMixTopicBits) | (hi << 12));
}
int launch_sweep(lda_ctx* c, int32_t mh_steps);
// Sweep with the doc side refreshed after every token (sweep_refresh.hip)
int refresh_sweep_max_doc();
int launch_sweep_doc_refresh(lda_ctx* c, int32_t mh_steps, int32_t longest_doc);
// Two-pass sweep (word pass over word-major tokens, doc pass over document tiles)
bool split_sweep_supported(const lda_ctx* c, int32_t mh_steps);
int setup_split_sweep(lda_ctx* c, const std::vector<int32_t>& woff);
int launch_sweep_split(lda_ctx* c, int32_t mh_steps);
int launch_tokdoc(lda_ctx* c);                               // per-token document index in its tile
int launch_rebuild(lda_ctx* c);
int launch_update_counts(lda_ctx* c);  // n_kw, n_k by +-1 for the tokens the last sweep moved
int setup_sparse_rows(lda_ctx* c, const std::vector<int32_t>& woff);
int launch_sparse_rows(lda_ctx* c);   // lists, list lengths and hash rows of the sparse-row words
int launch_nk_by_ranges(lda_ctx* c);  // n_k when K is too large for a few LDS histograms over z
int launch_loglik(lda_ctx* c, double* doc_part, double* word_part);
int launch_loglik_doc_tiles(lda_ctx* c, double* d_partial);  // partial[tile] of the bound tiles
// zw[wpos[i]] = z[i], i < n: topics into the word-major copy
int launch_scatter_word_major(lda_ctx* c, const int32_t* z, const int32_t* wpos, int64_t n);
// streamed data blocks (stream_blocks.hip)
int enter_streamed_mode(lda_ctx* c, const std::vector<int32_t>& chunk_doc);
void leave_streamed_mode(lda_ctx* c);
int launch_sweep_streamed(lda_ctx* c, int32_t mh_steps);
int launch_loglik_doc_streamed(lda_ctx* c, double* d_partial);
int streamed_get_z(lda_ctx* c, int32_t* z);
int streamed_set_z(lda_ctx* c, const int32_t* z);
int streamed_doc_z(lda_ctx* c, int64_t d, const int32_t** z_shifted);
int streamed_sync(lda_ctx* c);
int launch_ndk_row(lda_ctx* c, int64_t d);                  // dense n_dk row into c->d_row
int launch_check_range(lda_ctx* c, const int32_t* d_vals, int64_t n, int32_t lo, int32_t hi,
                       bool* ok);
int max_alias_topics();    // largest K the dense alias kernel handles
int max_rebuild_topics();  // largest K the count-rebuild tiles handle

// ------------------------------------------------------------------------------------
// device helpers
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t mulhi32(uint32_t a, uint32_t b) { return __umulhi(a, b); }

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies,
// the key advanced by Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        // full 64-bit products: one multiply instruction yields both halves
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// (x + 1/2) / 2^32: uniform in (0,1), exact in fp64
__device__ __forceinline__ double unit_open(uint32_t x)
{
    return ((double)x + 0.5) * (1.0 / 4294967296.0);
}

}  // namespace lda
