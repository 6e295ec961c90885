// The fused cycle Metropolis-Hastings sweep (LightLDA Sec. 4.2-4.3, Eq. 6-13).
//
// Work is tiled by documents: a workgroup stages a run of consecutive documents
// in LDS (their snapshot z values and one n_kd hash table per document), so the
// whole document side of every step -- the doc-proposal's "copy the topic of a
// random token of the document" (Eq. 12) and the n_kd factors of the ratios --
// is served from LDS.  The word side (alias bin, n_kw, n_k) is gathered from
// HBM/L2.  Every token runs its mh_steps fused in registers and writes one int.
// An alias bin carries the word-topic counts of its two possible outcomes, so a
// word step costs one gather for the draw and the proposed topic's n_kw together.
#include "common.hpp"
#include "doc_tile.hpp"
#include "word_side.hpp"

namespace lda {

struct SweepArgs {
    const int32_t* word;
    const int32_t* z;
    int32_t* znew;
    const int32_t* doff;
    const int32_t* chunk_doc;
    const uint8_t* tokdoc;  // index of each token's document inside its tile
    const int32_t* nkw;
    const int32_t* nk;
    const uint4* alias;     // (split, alias, n_kw[bin], n_kw[alias]) per bin
    const uint32_t* cap;
    int32_t K;
    int32_t mh_steps;
    int32_t mode;
    int32_t cap_tokens;
    double alpha, beta, alphabar, betabar;
    uint32_t seed_lo, seed_hi, sweep;
    // hybrid store / mixture proposal (null in the all-dense mode)
    const uint4* metaA;       // word w at [2w]: (entries n, capacity C, QS low, QS high)
    const uint4* metaB;       // = metaA + 1, word w at [2w]: (list offset, hash offset, log2 slots, kind)
    const uint4* ma;          // mixture bins, two uint4 per list entry
    const uint2* hs;          // hash rows (topic, count)
    const uint2* beta_alias;  // shared beta-term table
    const uint64_t* beta_hdr; // QB, capacity
    // long documents
    const int32_t* long_doc;
    const int64_t* long_slot;
    int32_t* long_keys;
    int32_t* long_cnts;
};

// A token's document as the chain sees it: n_kd of an arbitrary topic, and the
// topic and n_kd of the document's j-th token.
struct TileDocView {  // document staged in an LDS tile
    PackedDocTable tab;
    const uint32_t* zs;  // the document's packed (topic | slot << 20) entries
    int32_t L;
    __device__ __forceinline__ int32_t count(int32_t k) const { return tab.count(k); }
    __device__ __forceinline__ void token(uint32_t j, int32_t& topic, int32_t& nd) const
    {
        const uint32_t v = zs[j];
        topic = (int32_t)(v & kTopicMask);
        nd = tab.count_at(v >> kTopicBits);
    }
};

struct LongDocView {  // document hashed in the global workspace
    GlobalDocTable tab;
    const int32_t* z;
    int32_t L;
    __device__ __forceinline__ int32_t count(int32_t k) const { return tab.count(k); }
    __device__ __forceinline__ void token(uint32_t j, int32_t& topic, int32_t& nd) const
    {
        topic = z[j];
        nd = tab.count(topic);
    }
};

// The chains of T tokens of one thread, advanced together.
//
// Interleaving T independent chains stage by stage keeps T gathers in flight per
// lane; every stage below is a fully unrolled loop over the T tokens, so all state
// lives in registers.  doc[u] is token u's document, own[u] its position in it,
// w[u] its word, g[u] its CSR position (the Philox counter).  The accept test is
// evaluated without branching; a step with t == s leaves the state unchanged.
template <int T, class DocView>
__device__ __forceinline__ void mh_chains(const SweepArgs& A, const DocView (&doc)[T],
                                          const uint32_t (&own)[T], const int32_t (&w)[T],
                                          const uint32_t (&g)[T], int32_t (&s)[T])
{
#pragma clang fp contract(off)
    const int32_t K = A.K;
    size_t wk[T];
    uint32_t capw[T];
    int32_t z0[T], nds[T], nws[T], nks[T];
#pragma unroll
    for (int u = 0; u < T; ++u) {
        doc[u].token(own[u], z0[u], nds[u]);
        s[u] = z0[u];
        wk[u] = (size_t)w[u] * (size_t)K;
        capw[u] = A.cap[w[u]];
        nws[u] = A.nkw[wk[u] + (size_t)z0[u]];
        nks[u] = A.nk[z0[u]];
    }
    for (int32_t j = 0; j < A.mh_steps; ++j) {
        const bool word_step = (A.mode == 0) ? ((j & 1) == 0) : (A.mode == 1);
        uint32_t x2[T];
        int32_t t[T], ndt[T], nwt[T], nkt[T];
        if (word_step) {
            // Fig. 2: uniform bin, uniform height, keep the bin or take its alias;
            // the bin brings n_kw of both outcomes along
            uint32_t bin[T], rr[T];
            uint4 e[T];
#pragma unroll
            for (int u = 0; u < T; ++u) {
                uint32_t x[4];
                philox4x32_10(g[u], 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
                x2[u] = x[2];
                bin[u] = mulhi32(x[0], (uint32_t)K);
                rr[u] = mulhi32(x[1], capw[u]);
                e[u] = A.alias[wk[u] + bin[u]];
            }
#pragma unroll
            for (int u = 0; u < T; ++u) {
                const bool keep = rr[u] < e[u].x;
                t[u] = keep ? (int32_t)bin[u] : (int32_t)e[u].y;
                nwt[u] = keep ? (int32_t)e[u].z : (int32_t)e[u].w;
                nkt[u] = A.nk[t[u]];
            }
#pragma unroll
            for (int u = 0; u < T; ++u) ndt[u] = doc[u].count(t[u]);
        } else {
            // Eq. (9), (12): a random token of the document, or a uniform topic
#pragma unroll
            for (int u = 0; u < T; ++u) {
                uint32_t x[4];
                philox4x32_10(g[u], 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
                x2[u] = x[2];
                const double u0 = unit_open(x[0]);
                const double Ld = (double)doc[u].L;
                if (u0 * (Ld + A.alphabar) < Ld) {
                    doc[u].token(mulhi32(x[1], (uint32_t)doc[u].L), t[u], ndt[u]);
                } else {
                    t[u] = (int32_t)mulhi32(x[1], (uint32_t)K);
                    ndt[u] = doc[u].count(t[u]);
                }
                nkt[u] = A.nk[t[u]];
                nwt[u] = nws[u];
                if (t[u] != s[u]) nwt[u] = A.nkw[wk[u] + (size_t)t[u]];
            }
        }
#pragma unroll
        for (int u = 0; u < T; ++u) {
            const int32_t ms = (s[u] == z0[u]) ? 1 : 0;
            const int32_t mt = (t[u] == z0[u]) ? 1 : 0;
            // Eq. (4) ratio p(t)/p(s), the token removed at its snapshot topic
            double num = (double)(ndt[u] - mt) + A.alpha;
            num = num * ((double)(nwt[u] - mt) + A.beta);
            num = num * ((double)(nks[u] - ms) + A.betabar);
            double den = (double)(nds[u] - ms) + A.alpha;
            den = den * ((double)(nws[u] - ms) + A.beta);
            den = den * ((double)(nkt[u] - mt) + A.betabar);
            if (word_step) {  // Eq. (8): times p_w(s)/p_w(t)
                num = num * ((double)nws[u] + A.beta);
                num = num * ((double)nkt[u] + A.betabar);
                den = den * ((double)nwt[u] + A.beta);
                den = den * ((double)nks[u] + A.betabar);
            } else {          // Eq. (11): times p_d(s)/p_d(t)
                num = num * ((double)nds[u] + A.alpha);
                den = den * ((double)ndt[u] + A.alpha);
            }
            const double uu = unit_open(x2[u]);
            const bool accept = (t[u] != s[u]) && (uu * den < num);
            s[u] = accept ? t[u] : s[u];
            nds[u] = accept ? ndt[u] : nds[u];
            nws[u] = accept ? nwt[u] : nws[u];
            nks[u] = accept ? nkt[u] : nks[u];
        }
    }
}

// ---- hybrid store -----------------------------------------------------------------------
// Chains with the hybrid word side: dense tables for the head words, the
// sparsified mixture (Sec. 4.2) for the others.  Same structure as mh_chains.
// The three forms of a word step (dense table, sparse term, shared beta term)
// differ only in the address of the one 16-byte record they gather and in how it
// is decoded, so every lane issues the same load.
template <int T, int STORE, class DocView>
__device__ __forceinline__ void mh_chains_hybrid(const SweepArgs& A, const DocView (&doc)[T],
                                                 const uint32_t (&own)[T], const int32_t (&w)[T],
                                                 const uint32_t (&g)[T], int32_t (&s)[T])
{
#pragma clang fp contract(off)
    const uint32_t K = (uint32_t)A.K;
    const BetaTable bt = load_beta_table(A);
    WordSide wv[T];
    int32_t z0[T], nds[T], nws[T], nks[T];
#pragma unroll
    for (int u = 0; u < T; ++u) {
        doc[u].token(own[u], z0[u], nds[u]);
        s[u] = z0[u];
        wv[u] = load_word<STORE>(A, w[u]);
    }
#pragma unroll
    for (int u = 0; u < T; ++u) {
        nws[u] = nkw_lookup<STORE>(wv[u], z0[u]);
        nks[u] = A.nk[z0[u]];
    }
    for (int32_t j = 0; j < A.mh_steps; ++j) {
        const bool word_step = (A.mode == 0) ? ((j & 1) == 0) : (A.mode == 1);
        uint32_t x2[T];
        int32_t t[T], ndt[T], nwt[T], nkt[T];
        if (word_step) {
            WordDraw d[T];
            uint4 e[T];
            bool known[T];
#pragma unroll
            for (int u = 0; u < T; ++u) {
                uint32_t x[4];
                philox4x32_10(g[u], 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
                x2[u] = x[2];
                e[u] = *word_draw_address(wv[u], bt, K, x[0], x[1], x[3], d[u]);
            }
#pragma unroll
            for (int u = 0; u < T; ++u) {
                known[u] = word_draw_decode(d[u], e[u], t[u], nwt[u]);
                nkt[u] = A.nk[t[u]];
            }
#pragma unroll
            for (int u = 0; u < T; ++u) {
                if (!known[u]) nwt[u] = nkw_lookup<STORE>(wv[u], t[u]);
                ndt[u] = doc[u].count(t[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < T; ++u) {
                uint32_t x[4];
                philox4x32_10(g[u], 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
                x2[u] = x[2];
                const double u0 = unit_open(x[0]);
                const double Ld = (double)doc[u].L;
                if (u0 * (Ld + A.alphabar) < Ld) {
                    doc[u].token(mulhi32(x[1], (uint32_t)doc[u].L), t[u], ndt[u]);
                } else {
                    t[u] = (int32_t)mulhi32(x[1], K);
                    ndt[u] = doc[u].count(t[u]);
                }
                nkt[u] = A.nk[t[u]];
                nwt[u] = nws[u];
                if (t[u] != s[u]) nwt[u] = nkw_lookup<STORE>(wv[u], t[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < T; ++u) {
            const int32_t ms = (s[u] == z0[u]) ? 1 : 0;
            const int32_t mt = (t[u] == z0[u]) ? 1 : 0;
            double num = (double)(ndt[u] - mt) + A.alpha;
            num = num * ((double)(nwt[u] - mt) + A.beta);
            num = num * ((double)(nks[u] - ms) + A.betabar);
            double den = (double)(nds[u] - ms) + A.alpha;
            den = den * ((double)(nws[u] - ms) + A.beta);
            den = den * ((double)(nkt[u] - mt) + A.betabar);
            if (word_step) {  // Eq. (8)
                num = num * ((double)nws[u] + A.beta);
                num = num * ((double)nkt[u] + A.betabar);
                den = den * ((double)nwt[u] + A.beta);
                den = den * ((double)nks[u] + A.betabar);
            } else {          // Eq. (11)
                num = num * ((double)nds[u] + A.alpha);
                den = den * ((double)ndt[u] + A.alpha);
            }
            const double uu = unit_open(x2[u]);
            const bool accept = (t[u] != s[u]) && (uu * den < num);
            s[u] = accept ? t[u] : s[u];
            nds[u] = accept ? ndt[u] : nds[u];
            nws[u] = accept ? nwt[u] : nws[u];
            nks[u] = accept ? nkt[u] : nks[u];
        }
    }
}

// T = tokens per thread; a tile has at most T * blockDim.x tokens.  MAXB bounds
// the block size so that small blocks may use more registers per thread.
template <int T, int MAXB, int STORE>
__global__ __launch_bounds__(MAXB) void sweep_tiles_kernel(SweepArgs A)
{
    extern __shared__ int32_t smem[];
    const int32_t c = blockIdx.x;
    const int32_t d0 = A.chunk_doc[c], d1 = A.chunk_doc[c + 1];
    const int32_t ntok = A.doff[d1] - A.doff[d0];
    if (ntok > A.cap_tokens || ntok == 0) return;  // a long document (other kernel) / nothing
    const DocTile tile = load_doc_tile(smem, A.cap_tokens, A.z, A.doff, A.tokdoc, d0, d1);
    TileDocView doc[T];
    uint32_t own[T], g[T];
    int32_t w[T], s[T];
    bool live[T];
#pragma unroll
    for (int u = 0; u < T; ++u) {
        // lanes past the end of the tile redo its last token and drop the result:
        // no lane is ever masked off inside the chains
        int32_t i = (int32_t)threadIdx.x + u * (int32_t)blockDim.x;
        live[u] = i < tile.ntok;
        if (!live[u]) i = tile.ntok - 1;
        g[u] = (uint32_t)(tile.tok0 + i);
        const int32_t dl = (int32_t)A.tokdoc[g[u]];
        const int32_t b = tile.sdoff[dl];
        doc[u].L = tile.sdoff[dl + 1] - b;
        doc[u].tab = tile.table(dl);
        doc[u].zs = tile.zs + b;
        own[u] = (uint32_t)(i - b);
        w[u] = A.word[g[u]];
    }
    if constexpr (STORE != 0)
        mh_chains_hybrid<T, STORE>(A, doc, own, w, g, s);
    else
        mh_chains<T>(A, doc, own, w, g, s);
#pragma unroll
    for (int u = 0; u < T; ++u)
        if (live[u]) A.znew[g[u]] = s[u];
}

template <int STORE>
__global__ __launch_bounds__(1024) void sweep_long_docs_kernel(SweepArgs A)
{
    constexpr int T = 2;
    const int32_t d = A.long_doc[blockIdx.x];
    const int32_t tok0 = A.doff[d];
    const int32_t Ld = A.doff[d + 1] - tok0;
    const int64_t s0 = A.long_slot[blockIdx.x];
    const GlobalDocTable table =
        load_long_doc(A.long_keys + s0, A.long_cnts + s0, A.z + tok0, Ld);
    for (int32_t base = 0; base < Ld; base += T * (int32_t)blockDim.x) {
        LongDocView doc[T];
        uint32_t own[T], g[T];
        int32_t w[T], s[T];
        bool live[T];
#pragma unroll
        for (int u = 0; u < T; ++u) {
            int32_t i = base + (int32_t)threadIdx.x + u * (int32_t)blockDim.x;
            live[u] = i < Ld;
            if (!live[u]) i = Ld - 1;
            doc[u].tab = table;
            doc[u].z = A.z + tok0;
            doc[u].L = Ld;
            own[u] = (uint32_t)i;
            g[u] = (uint32_t)(tok0 + i);
            w[u] = A.word[g[u]];
        }
        if constexpr (STORE != 0)
            mh_chains_hybrid<T, STORE>(A, doc, own, w, g, s);
        else
            mh_chains<T>(A, doc, own, w, g, s);
#pragma unroll
        for (int u = 0; u < T; ++u)
            if (live[u]) A.znew[g[u]] = s[u];
    }
}

template <int T, int MAXB, int STORE>
int launch_tiles_tb(lda_ctx* c, const SweepArgs& A, size_t lds)
{
    auto kern = sweep_tiles_kernel<T, MAXB, STORE>;
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3(c->n_chunks), dim3(c->sweep_block), lds, c->stream, A);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

template <int T, int STORE>
int launch_tiles_t(lda_ctx* c, const SweepArgs& A, size_t lds)
{
    if (c->sweep_block <= 256) return launch_tiles_tb<T, 256, STORE>(c, A, lds);
    if (c->sweep_block <= 512) return launch_tiles_tb<T, 512, STORE>(c, A, lds);
    return launch_tiles_tb<T, 1024, STORE>(c, A, lds);
}

template <int STORE>
int launch_tiles(lda_ctx* c, const SweepArgs& A, size_t lds)
{
    const int tpt = (c->chunk_tokens + c->sweep_block - 1) / c->sweep_block;
    if (tpt <= 1) return launch_tiles_t<1, STORE>(c, A, lds);
    if (tpt <= 2) return launch_tiles_t<2, STORE>(c, A, lds);
    if (tpt <= 4) return launch_tiles_t<4, STORE>(c, A, lds);
    if (tpt <= 6) return launch_tiles_t<6, STORE>(c, A, lds);
    if (tpt <= 8) return launch_tiles_t<8, STORE>(c, A, lds);
    return fail(c, LDA_ERR_ARG, "sweep: more than 8 tokens per thread (tile %d, block %d)",
                c->chunk_tokens, c->sweep_block);
}

// tokdoc[g] = index of token g's document inside its tile (0 for long documents)
__global__ __launch_bounds__(256) void tokdoc_kernel(const int32_t* __restrict__ doff,
                                                     const int32_t* __restrict__ chunk_doc,
                                                     int32_t cap_tokens,
                                                     uint8_t* __restrict__ tokdoc)
{
    const int32_t c = blockIdx.x;
    const int32_t d0 = chunk_doc[c], d1 = chunk_doc[c + 1];
    const int32_t tok0 = doff[d0], ntok = doff[d1] - tok0;
    const bool is_long = ntok > cap_tokens;
    for (int32_t i = threadIdx.x; i < ntok; i += blockDim.x) {
        int32_t lo = 0, hi = d1 - d0;  // doff[d0+lo] - tok0 <= i < doff[d0+hi] - tok0
        while (hi - lo > 1) {
            const int32_t mid = (lo + hi) >> 1;
            if (doff[d0 + mid] - tok0 <= i) lo = mid; else hi = mid;
        }
        tokdoc[tok0 + i] = is_long ? (uint8_t)0 : (uint8_t)lo;
    }
}

int launch_tokdoc(lda_ctx* c)
{
    if (c->n_chunks > 0) {
        hipLaunchKernelGGL(tokdoc_kernel, dim3(c->n_chunks), dim3(256), 0, c->stream, c->d_doff,
                           c->d_chunk_doc, c->chunk_tokens, c->d_tokdoc);
        LDA_HIP(c, hipGetLastError());
    }
    if (c->n_chunks2 > 0) {
        hipLaunchKernelGGL(tokdoc_kernel, dim3(c->n_chunks2), dim3(256), 0, c->stream, c->d_doff,
                           c->d_chunk_doc2, c->chunk_tokens2, c->d_tokdoc2);
        LDA_HIP(c, hipGetLastError());
    }
    return LDA_OK;
}

static SweepArgs make_sweep_args(lda_ctx* c, int32_t mh_steps)
{
    SweepArgs A{};
    A.word = c->d_word; A.z = c->d_z; A.znew = c->d_znew; A.doff = c->d_doff;
    A.chunk_doc = c->d_chunk_doc; A.tokdoc = c->d_tokdoc; A.nkw = c->d_nkw; A.nk = c->d_nk;
    A.alias = c->d_alias; A.cap = c->d_cap; A.K = c->K; A.mh_steps = mh_steps;
    A.mode = c->opt.proposal_mode; A.cap_tokens = c->chunk_tokens;
    A.alpha = c->alpha; A.beta = c->beta; A.alphabar = c->alphabar; A.betabar = c->betabar;
    A.seed_lo = (uint32_t)c->seed; A.seed_hi = (uint32_t)(c->seed >> 32); A.sweep = c->sweep_index;
    A.metaA = c->d_metaA; A.metaB = c->d_metaB; A.ma = c->d_ma; A.hs = c->d_hs;
    A.beta_alias = c->d_beta_alias; A.beta_hdr = c->d_beta_hdr;
    A.long_doc = c->d_long_doc; A.long_slot = c->d_long_slot;
    A.long_keys = c->d_long_keys; A.long_cnts = c->d_long_cnts;
    return A;
}

template <int STORE>
static int launch_sweep_store(lda_ctx* c, int32_t mh_steps)
{
    const SweepArgs A = make_sweep_args(c, mh_steps);
    const size_t lds = doc_tile_lds_bytes(c->chunk_tokens, c->chunk_docs);
    if (c->n_chunks > 0) {
        const int rc = launch_tiles<STORE>(c, A, lds);
        if (rc != LDA_OK) return rc;
    }
    if (c->n_long > 0) {
        hipLaunchKernelGGL(sweep_long_docs_kernel<STORE>, dim3(c->n_long), dim3(1024), 0,
                           c->stream, A);
        LDA_HIP(c, hipGetLastError());
    }
    return LDA_OK;
}

int launch_sweep(lda_ctx* c, int32_t mh_steps) { return launch_sweep_store<0>(c, mh_steps); }

int launch_sweep_hybrid(lda_ctx* c, int32_t mh_steps)
{
    return c->H == c->V ? launch_sweep_store<1>(c, mh_steps) : launch_sweep_store<2>(c, mh_steps);
}

// ---- n_kd accessor: the row exactly as the sweep kernels form it -------------------

__global__ __launch_bounds__(256) void ndk_row_tile_kernel(const int32_t* z, const int32_t* doff,
                                                           int32_t d, int32_t cap_tokens,
                                                           int32_t K, int32_t* row)
{
    extern __shared__ int32_t smem[];
    const DocTile T = load_doc_tile(smem, cap_tokens, z, doff, nullptr, d, d + 1);
    const PackedDocTable tab = T.table(0);
    for (int32_t k = threadIdx.x; k < K; k += blockDim.x) row[k] = T.ntok > 0 ? tab.count(k) : 0;
}

__global__ __launch_bounds__(1024) void ndk_row_long_kernel(const int32_t* z, const int32_t* doff,
                                                            int32_t d, int32_t* keys,
                                                            int32_t* cnts, int32_t K, int32_t* row)
{
    const int32_t tok0 = doff[d];
    const int32_t L = doff[d + 1] - tok0;
    const GlobalDocTable tab = load_long_doc(keys, cnts, z + tok0, L);
    for (int32_t k = threadIdx.x; k < K; k += blockDim.x) row[k] = tab.count(k);
}

int launch_ndk_row(lda_ctx* c, int64_t d)
{
    const int32_t L = c->h_doff[d + 1] - c->h_doff[d];
    const int32_t* z = c->d_z;
    if (c->streamed) {  // the document's topics come from the pinned copy
        const int rc = streamed_doc_z(c, d, &z);
        if (rc != LDA_OK) return rc;
    }
    if (L <= c->chunk_tokens) {
        const size_t lds = doc_tile_lds_bytes(c->chunk_tokens, c->chunk_docs);
        if (lds > 48 * 1024)
            LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(ndk_row_tile_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(ndk_row_tile_kernel, dim3(1), dim3(256), lds, c->stream, z,
                           c->d_doff, (int32_t)d, c->chunk_tokens, c->K, c->d_row);
    } else {
        // the d-th long document's workspace slice
        int64_t s0 = -1;
        std::vector<int64_t> slot(c->n_long + 1);
        LDA_HIP(c, hipMemcpy(slot.data(), c->d_long_slot, sizeof(int64_t) * (c->n_long + 1),
                             hipMemcpyDeviceToHost));
        for (int32_t i = 0; i < c->n_long; ++i)
            if (c->h_long_doc[i] == (int32_t)d) s0 = slot[i];
        if (s0 < 0) return fail(c, LDA_ERR_HIP, "long document %lld has no workspace", (long long)d);
        hipLaunchKernelGGL(ndk_row_long_kernel, dim3(1), dim3(1024), 0, c->stream, c->d_z,
                           c->d_doff, (int32_t)d, c->d_long_keys + s0, c->d_long_cnts + s0, c->K,
                           c->d_row);
    }
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
