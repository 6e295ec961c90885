/*
 * lda_mi355x.h -- C ABI of the MI355X (gfx950) LightLDA sweep library.
 *
 * The library runs the data-parallel hot path of LightLDA (arXiv 1412.1576):
 * the O(1) cycle Metropolis-Hastings sweep over all tokens of a corpus
 * (Sec. 4.2-4.3, Eq. 6-13), the per-word alias tables it draws from
 * (Sec. 4.2, Fig. 2), and the rebuild of the count tables n_kd, n_kw, n_k
 * (Sec. 3, text after Eq. 1).  Every step runs in hand-written HIP kernels on
 * one GPU; the host side only marshals arguments.
 *
 * Semantics fixed by this library (the paper leaves them open):
 *   - Snapshot sweeps: every token of a sweep reads the assignment z and all
 *     counts as of the start of the sweep (the limit of the paper's immutable
 *     model slice with delayed updates, Sec. 6 "Multi-thread Efficiency").
 *     A token's own contribution is removed at its snapshot topic.
 *   - One MH step is one proposal plus one accept test; step j of a token is a
 *     word-proposal for even j and a doc-proposal for odd j (Eq. 13).
 *   - Randomness is Philox4x32-10 with key = seed and counter
 *     (token id low, token id high, sweep index, step index), so results do not
 *     depend on launch geometry.  Acceptance ratios are evaluated in fp64 with
 *     separately rounded operations.
 *
 * Conventions
 *   - All pointers in the signatures are HOST pointers unless stated otherwise.
 *     The library copies what it needs; the caller keeps ownership of its buffers
 *     and may free them as soon as a call returns.
 *   - Token order at the boundary is the caller's CSR (document-major) order:
 *     token g is word_ids[g]; document d owns g in [doc_offsets[d], doc_offsets[d+1]).
 *   - Return value 0 (LDA_OK) on success, a negative LDA_ERR_* otherwise; no call
 *     throws.  lda_last_error() returns a message for the last failure.
 *   - lda_build_alias, lda_sweep and lda_rebuild_counts enqueue work on the
 *     context's HIP stream and return; accessors and lda_loglik synchronise.
 *     (lda_build_alias may run part of its kernels on a second stream of the
 *     library's own, of default priority, forked from and joined to the context's
 *     stream by events: work queued after the call still sees every table.  With
 *     stream_block_tokens the copies of the blocks run on two more such streams;
 *     lda_sync waits for them too.)
 *   - A context is not thread-safe.  Calls must follow the state machine
 *       COUNTS_VALID --lda_build_alias--> ALIAS_VALID --lda_sweep--> SWEPT
 *       SWEPT --lda_rebuild_counts--> COUNTS_VALID
 *     and return LDA_ERR_STATE otherwise.
 */
#ifndef LDA_MI355X_H
#define LDA_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LDA_OK 0
#define LDA_ERR_ARG (-1)         /* bad pointer, size, id out of range, alpha/beta <= 0, ... */
#define LDA_ERR_STATE (-2)       /* call out of order */
#define LDA_ERR_OOM (-3)         /* host or device allocation failed */
#define LDA_ERR_HIP (-4)         /* a HIP runtime call or kernel launch failed */
#define LDA_ERR_UNSUPPORTED (-5) /* valid request outside what this build supports */

typedef struct lda_ctx lda_ctx; /* opaque; owns all device memory of one corpus */

/* Options for lda_init.  A zeroed struct (or a NULL pointer) selects the defaults. */
typedef struct lda_options {
    void* hip_stream;              /* hipStream_t all work is enqueued on; NULL: the null stream */
    /* Device allocator of the caller (e.g. a framework's caching allocator); both NULL: hipMalloc
       and hipFree.  When set, every device buffer of the context -- at lda_init and the ones
       that later calls grow or create on first use -- comes from dev_alloc(bytes, alloc_user),
       which returns device memory aligned to 256 bytes or NULL (reported as LDA_ERR_OOM), and
       goes back through dev_free(ptr, alloc_user), at lda_destroy at the latest.  The
       callbacks run on the thread that calls the library; setting only one is LDA_ERR_ARG.
       rocprim's temporary storage is requested through them as well. */
    void* (*dev_alloc)(size_t bytes, void* alloc_user);
    void (*dev_free)(void* ptr, void* alloc_user);
    void* alloc_user;
    int32_t dense_rows;            /* hybrid store (Sec. 5): word ids [0, dense_rows) keep a dense n_kw
                                      row, the others a sorted (topic, count) list plus a hash row;
                                      0: every row dense; -1: no dense row */
    int32_t dense_alias_min_count; /* words with corpus frequency >= this draw from a dense K-bin
                                      table, the others from the sparsified mixture (Sec. 4.2);
                                      0: every word uses the dense table.  A word that draws from a
                                      dense table must have a dense row (LDA_ERR_ARG otherwise). */
    int32_t proposal_mode;         /* 0: cycle word,doc,word,... (Eq. 13); 1: word only; 2: doc only */
    int32_t sweep_chunk_tokens;    /* tuning: tokens per sweep workgroup tile; 0: default */
    int32_t sweep_block_threads;   /* tuning: threads per sweep workgroup; 0: default */
    int32_t rebuild_tile_tokens;   /* tuning: tokens per count-rebuild tile; 0: default */
    int32_t time_sweep_passes;     /* 1: lda_sweep records HIP events around its two passes on the
                                      context's stream (read them with lda_sweep_pass_ms) */
    int32_t record_bucket_tokens;  /* tuning: the per-token records the two passes of a sweep
                                      exchange are ordered by buckets of this many consecutive
                                      tokens (a power of two), inside a bucket by word; 0: default
                                      (2^22 when every n_kw row is dense and the corpus has at
                                      least 2^28 tokens, else one bucket);
                                      -1: one bucket (plain word order) */
    int32_t doc_refresh;           /* 1: lda_sweep refreshes the doc side after every token (Sec. 4.2,
                                      footnote 4): the tokens of a document are visited in order
                                      and each sees, in n_kd and in the doc-proposal's draw, the
                                      topics its predecessors of the same sweep were just given;
                                      the word side stays at the snapshot (Sec. 6).  All-dense
                                      store with dense tables, documents of at most 4096 tokens,
                                      at most 4 steps (LDA_ERR_UNSUPPORTED otherwise).  0: every
                                      token reads the snapshot (the default, and the fast path) */
    int32_t stream_block_tokens;   /* > 0: streamed data blocks (Sec. 3; Sec. 6, Fig. 7).  The model
                                      stays on the device; the per-token arrays move to pinned
                                      host memory when lda_init is done and every lda_sweep brings
                                      them in block by block -- runs of whole documents of about
                                      this many tokens, the next block loading while the current
                                      one is swept -- and takes the new topics back.  4 bytes per
                                      token stay resident (the word-major copy of z that the count
                                      rebuild reads).  Results are those of the resident run, bit
                                      for bit.  lda_init itself still holds the whole corpus on
                                      the device once.  Not with doc_refresh (LDA_ERR_ARG), not
                                      with documents longer than a sweep tile, not
                                      lda_update_counts (LDA_ERR_UNSUPPORTED).  0: resident */
    int32_t reserved[5];           /* must be zero */
} lda_options;

/*
 * lda_init -- take a corpus and set up the sampler state (problem statement: Sec. 3).
 *   D            number of documents (>= 1); empty documents are legal
 *   V, K         vocabulary size and number of topics (>= 1); K <= 2^20 - 2; dense rows and
 *                dense tables are limited to 10^10 and 4 * 10^9 entries (LDA_ERR_UNSUPPORTED)
 *   doc_offsets  [D+1] host, doc_offsets[0] = 0, non-decreasing, N = doc_offsets[D] in [1, 2^31 - 2^20 - 1]
 *   word_ids     [N] host, each in [0, V)
 *   alpha, beta  symmetric Dirichlet parameters (> 0) of Eq. (1)
 *   seed         Philox key
 * Copies the corpus to the device, builds the word-major token order and the
 * document tiling, draws the initial assignment z[g] = floor(x0 * K / 2^32) from
 * the Philox counter (g, 0xFFFFFFFF, 0) and counts n_kw, n_k.  On success
 * *out is a new context in state COUNTS_VALID with sweep index 0.
 */
int lda_init(lda_ctx** out, int64_t D, int32_t V, int32_t K, const int64_t* doc_offsets,
             const int32_t* word_ids, double alpha, double beta, uint64_t seed,
             const lda_options* opt);

/*
 * lda_build_alias -- word-proposal tables of Eq. (6) for every word, from the
 * current counts: per bin a split point and an alias (Sec. 4.2, Fig. 2), plus the
 * bin capacity of the table.  Words of the dense form get one table over all K
 * topics; words of the mixture form (Sec. 4.2, the sparsified table) one table
 * over their non-zero topics, and all of them share one table over
 * beta/(n_k + V beta).  COUNTS_VALID -> ALIAS_VALID.
 */
int lda_build_alias(lda_ctx* ctx);

/*
 * lda_sweep -- one sweep: for every token mh_steps (>= 1) Metropolis-Hastings
 * steps alternating the word-proposal (Eq. 6-8) and the doc-proposal
 * (Eq. 9-12) against the conditional of Eq. (4), all reads from the snapshot.
 * Uses the context's sweep index as Philox counter word 2 and increments it.
 * ALIAS_VALID -> SWEPT (the counts no longer match z).
 */
int lda_sweep(lda_ctx* ctx, int32_t mh_steps);

/*
 * lda_sweep_pass_ms -- device time of the last sweep's two passes, from the HIP events
 * recorded with the option time_sweep_passes: *word_pass_ms covers the word pass (every
 * kernel that evaluates the word side of the chains, Eq. 6-8, in word-major order),
 * *doc_pass_ms the one kernel that runs the accept tests over the document tiles.
 * Waits for the events.  LDA_ERR_STATE if the option is off, no sweep has run, or the
 * last sweep ran as one fused kernel (more than 4 steps, word-only or doc-only chains of
 * several steps, tiles of more than 4 tokens per thread).
 */
int lda_sweep_pass_ms(lda_ctx* ctx, float* word_pass_ms, float* doc_pass_ms);

/*
 * lda_rebuild_counts -- recount n_kw (per-word histogram of the word-major
 * token segments: dense rows, and for words without a dense row the sorted
 * (topic, count) list and hash row of Sec. 5) and n_k from the current
 * assignment; the per-document counts n_kd are formed inside the sweep from the
 * document's assignments.  SWEPT (or any state) -> COUNTS_VALID.
 */
int lda_rebuild_counts(lda_ctx* ctx);

/*
 * lda_update_counts -- the counts after a sweep by the paper's own rule (Sec. 3, text after
 * Eq. 1; applied late as in Sec. 6, "Multi-thread Efficiency"): for every token the last
 * lda_sweep moved from topic a to topic b, n_kw[w][a] and n_k[a] lose one, n_kw[w][b] and
 * n_k[b] gain one.  Same tables as lda_rebuild_counts, bit for bit; cheaper when few tokens
 * move (late in training), dearer when most do.  Needs the state SWEPT reached by lda_sweep
 * (not by lda_set_z: LDA_ERR_STATE) and the all-dense store with dense tables for every word
 * (LDA_ERR_UNSUPPORTED otherwise: lists and hash rows are only made by the recount).
 * SWEPT -> COUNTS_VALID.
 */
int lda_update_counts(lda_ctx* ctx);

/*
 * lda_loglik -- log p(w, z | alpha, beta) of the collapsed model, the metric of
 * Sec. 7 ("doc-likelihood" + "word-likelihood"); fp64.  Needs valid counts.
 * doc_part / word_part may be NULL.  Synchronises.
 */
int lda_loglik(lda_ctx* ctx, double* total, double* doc_part, double* word_part);

/*
 * lda_loglik_noalloc -- lda_loglik for callers that cannot allocate: code under HIP graph
 * capture around it, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels, same summation order and therefore the same value as lda_loglik; the
 * per-block partial sums go to a static device array of the library (2^20 doubles = 8 MB,
 * held by every GPU the library runs on until the process ends) instead of the context's
 * own buffer, and the host side stages them through the stack.  The call makes no device or
 * host allocation.  The context's device must be the current device.
 *   - LDA_ERR_UNSUPPORTED when the context needs more partial sums than the array holds
 *     (one per document tile: more than 2^20 tiles, or long documents); use lda_loglik then.
 *   - All contexts on one GPU share the array: two calls that overlap on one GPU (two
 *     host threads, two streams) race on it and must be serialised by the caller.  Nothing in
 *     the array needs to be zero on entry; every element that is read was written by the
 *     same call.
 */
int lda_loglik_noalloc(lda_ctx* ctx, double* total, double* doc_part, double* word_part);

/* ---- accessors (parity checks, checkpoint / warm start of Sec. 6); all synchronise ---- */
int64_t lda_num_tokens(const lda_ctx* ctx);
int64_t lda_sweep_index(const lda_ctx* ctx);
/* z [N] in CSR token order. */
int lda_get_z(lda_ctx* ctx, int32_t* z);
/* Replace the assignment (each z[g] in [0,K)) and the next sweep index (< 2^32-1); -> SWEPT. */
int lda_set_z(lda_ctx* ctx, const int32_t* z, int64_t next_sweep_index);
/* nk [K]; needs valid counts. */
int lda_get_nk(lda_ctx* ctx, int32_t* nk);
/* Dense copy of row w of the word-topic table, row [K]; needs valid counts. */
int lda_get_nkw_row(lda_ctx* ctx, int32_t w, int32_t* row);
/* Dense copy of row d of the doc-topic table as the sweep kernel forms it, row [K]. */
int lda_get_ndk_row(lda_ctx* ctx, int64_t d, int32_t* row);
/* Dense-form table of word w: split [K], alias [K], *cap = bin capacity; needs ALIAS_VALID. */
int lda_get_alias_row(lda_ctx* ctx, int32_t w, uint32_t* split, uint32_t* alias, uint32_t* cap);

/* Mixture-form tables (Sec. 4.2, the sparsified word-proposal); need ALIAS_VALID.
 * lda_get_sparse_table: the table of word w over its non-zero topics.  *n = number of entries;
 * when *n <= cap_entries the entries are written: topics[i] ascending, split[i], and
 * alias_topic[i] = the topic bin i falls through to.  *cap = bin capacity, *mass = integer mass
 * QS_w of the sparse term.  LDA_ERR_ARG if the word draws from a dense table.
 * lda_get_beta_table: the table over beta/(n_k + V beta) shared by all words, split [K],
 * alias [K] (topic indices), its capacity and integer mass QB. */
int lda_get_sparse_table(lda_ctx* ctx, int32_t w, int32_t cap_entries, int32_t* n, int32_t* topics,
                         uint32_t* split, int32_t* alias_topic, uint32_t* cap, uint64_t* mass);
int lda_get_beta_table(lda_ctx* ctx, uint32_t* split, uint32_t* alias, uint32_t* cap,
                       uint64_t* mass);

/* Wait for all work enqueued by this context. */
int lda_sync(lda_ctx* ctx);
/* Message of the last error of this context (ctx == NULL: of the last failed lda_init on this
 * thread).  The string is owned by the library and valid until the next call. */
const char* lda_last_error(const lda_ctx* ctx);
/* Free the context and all its device memory.  NULL is allowed. */
void lda_destroy(lda_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* LDA_MI355X_H */
