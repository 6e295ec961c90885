// Two-pass form of the cycle Metropolis-Hastings sweep (LightLDA Sec. 4.2-4.3, Eq. 6-13).
//
// A proposal never depends on the chain's current state: a word-proposal draw is a
// function of the word's table and the token's random numbers (Fig. 2), a
// doc-proposal draw of the document's snapshot assignment (Eq. 12).  The word side of
// a token's chain -- its alias draws and every n_kw its ratios will need -- can
// therefore be evaluated before the accept tests, in word-major order, where all
// accesses of a word fall into that word's own rows:
//
//   word pass  word-major.  Frequent words: a workgroup stages the word's n_kw row and
//              its table in LDS and serves a run of the word's tokens from there
//              (one coalesced read of the rows per 65536 tokens instead of three random
//              128-byte lines per token).  Short words: the rows are gathered; the
//              word's tokens are processed together, so its lines are reused in L2.
//              Output: one record per token (n_kw at its snapshot topic, the proposed
//              topic and its n_kw for every word step, n_kw at every doc proposal).
//   doc pass   document tiles in LDS as in the fused kernel; the word side of a token is
//              the one record gathered from its word-major position.  Runs every accept
//              test (Eq. 8, 11) in order and writes the new assignment.  Its tail draws
//              the doc proposals of the NEXT sweep from the tile's new assignment and
//              writes (z, proposals) to the token's word-major record, which is what
//              the next word pass and the count rebuild read: no separate scatter pass.
//
// The arithmetic, the random numbers and their use are those of the fused kernel
// (sweep.hip), so the result is bit-identical.
#include <algorithm>

#include "common.hpp"
#include "doc_tile.hpp"
#include "word_side.hpp"
#include "xcd.hpp"

namespace lda {

namespace {

constexpr int32_t kRowItemTokens = 65536;  // tokens a workgroup serves from one staging of the rows
constexpr int32_t kRowMinTokens = 2048;    // words with fewer tokens are gathered
// Tokens of a gather piece.  Small on purpose: a piece is one workgroup, some 200 of them are
// in flight on an XCD, and what they gather from -- the hash rows and tables of their words --
// has to fit that XCD's 4 MB of L2 to be reused by a word's later tokens.  With 4096-token
// pieces the words in flight held 30 MB and three of four gathers missed.
constexpr int32_t kPieceTokens = 512;
constexpr int32_t kPieceWords = 4096;      // words of a gather piece (their offsets sit in LDS)

constexpr int pow2_shift(int n)
{
    int s = 0;
    while ((1 << s) < n) ++s;
    return s;
}

// Shape of a chain of NW word steps and ND doc steps: all word steps (ND = 0), all
// doc steps (NW = 0), or alternating starting with a word step (Eq. 13).
template <int NW, int ND>
struct Chain {
    static_assert(NW + ND >= 1 && (ND == 0 || NW == 0 || NW == ND || NW == ND + 1), "chain shape");
    static constexpr int M = NW + ND;
    static constexpr int rec_shift = pow2_shift(1 + 2 * NW + ND);
    static constexpr int R = 1 << rec_shift;  // ints of a word-pass record
    __host__ __device__ static constexpr bool is_word(int j)
    {
        return ND == 0 ? true : (NW == 0 ? false : (j & 1) == 0);
    }
    __host__ __device__ static constexpr int index(int j) { return (ND == 0 || NW == 0) ? j : j / 2; }
    __host__ __device__ static constexpr int word_step(int i) { return ND == 0 ? i : 2 * i; }
    __host__ __device__ static constexpr int doc_step(int i) { return NW == 0 ? i : 2 * i + 1; }
    // word-pass record: [0] n_kw[z0]; [1 + 2i], [2 + 2i] topic and n_kw of word step i;
    // [1 + 2 NW + i] n_kw of doc step i's proposal
    __host__ __device__ static constexpr int rec_topic(int i) { return 1 + 2 * i; }
    __host__ __device__ static constexpr int rec_doc(int i) { return 1 + 2 * NW + i; }
};

// A word step's record carries, above the proposed topic (topics take kTopicBits bits), the top
// bits of the random word x2 that decides the step's accept test.  The word pass has that
// Philox output anyway (the draw uses the same call); the doc pass can then decide almost
// every test from the two ends of the interval the bits leave open and needs the generator
// only when the ends disagree.
constexpr int kHintShift = kTopicBits;
constexpr uint32_t kHintSpan = (1u << kHintShift) - 1u;  // x2 is in [hint << shift, (hint << shift) | span]
__device__ __forceinline__ int32_t topic_with_hint(int32_t t, uint32_t x2)
{
    return (int32_t)((uint32_t)t | (x2 & ~kHintSpan));
}

template <int R>
__device__ __forceinline__ void load_ints(const int32_t* __restrict__ p, int32_t (&v)[R])
{
    if constexpr (R == 1) {
        v[0] = p[0];
    } else if constexpr (R == 2) {
        const int2 a = *reinterpret_cast<const int2*>(p);
        v[0] = a.x; v[1] = a.y;
    } else {
#pragma unroll
        for (int q = 0; q < R / 4; ++q) {
            const int4 a = reinterpret_cast<const int4*>(p)[q];
            v[4 * q] = a.x; v[4 * q + 1] = a.y; v[4 * q + 2] = a.z; v[4 * q + 3] = a.w;
        }
    }
}

template <int R>
__device__ __forceinline__ void store_ints(int32_t* __restrict__ p, const int32_t (&v)[R])
{
    if constexpr (R == 1) {
        p[0] = v[0];
    } else if constexpr (R == 2) {
        *reinterpret_cast<int2*>(p) = make_int2(v[0], v[1]);
    } else {
#pragma unroll
        for (int q = 0; q < R / 4; ++q)
            reinterpret_cast<int4*>(p)[q] = make_int4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    }
}

struct SplitArgs {
    const int32_t* z;
    int32_t* znew;
    const int32_t* doff;
    const int32_t* chunk_doc;
    const int32_t* chunk_tok;  // doff[chunk_doc[c]]: a tile's tokens without the second lookup
    const uint8_t* tokdoc;
    const int32_t* wpos;
    const int32_t* xmap;  // word-major position -> record position (NULL: identity)
    const int32_t* gid;
    const int32_t* woff;
    const int32_t* nkw;
    const int32_t* nk;
    const uint4* alias;  // (split, alias, n_kw[bin], n_kw[alias]) per bin
    const uint32_t* cap;
    int32_t* zt;
    int32_t zt_pack16;  // topics fit 16 bits: two fields of a (z, doc proposals) record per int
    int32_t* rec;
    const int4* row_items;
    const int4* pieces;
    int32_t n_chunks, n_row_items, n_pieces;
    int32_t K, cap_tokens;
    int32_t max_doc_tokens;  // a longer document is a tile of its own, left to the long-document kernel
    int32_t doc_block;       // threads per workgroup of the doc pass
    int32_t tile_lds_ints;  // ints of a document tile in LDS (the n_k copy follows it)
    double alpha, beta, alphabar, betabar;
    uint32_t seed_lo, seed_hi, sweep;
    // hybrid store / mixture proposal (null in the all-dense mode)
    const uint4* metaA;
    const uint4* metaB;
    const uint4* ma;
    const uint2* hs;
    const uint2* beta_alias;
    const uint64_t* beta_hdr;
    const uint32_t* sp_off;
    const int32_t* sp_topic;
    const int32_t* sp_count;
    const int32_t* sp_nnz;
    const int4* mix_items;
    int32_t n_mix_items;
    const int32_t* long_doc;
    const int64_t* long_slot;
    int32_t* long_keys;
    int32_t* long_cnts;
};

// ints of a token's (z, doc proposals) record with nd doc proposals: one int per field, or,
// when every topic fits 16 bits, two fields per int; rounded up to a power of two
constexpr int zt_record_shift(int nd, bool pack16) { return pow2_shift(pack16 ? (2 + nd) / 2 : 1 + nd); }

// v[0] = z, v[1 + i] = the topic doc step i proposes, of the token whose records are at p
template <int ND>
__device__ __forceinline__ void load_zt(const SplitArgs& A, size_t p, int32_t (&v)[1 + ND])
{
    if (A.zt_pack16) {
        constexpr int W = 1 << zt_record_shift(ND, true);
        int32_t w[W];
        load_ints<W>(A.zt + p * W, w);
#pragma unroll
        for (int k = 0; k <= ND; ++k) v[k] = (int32_t)(((uint32_t)w[k >> 1] >> (16 * (k & 1))) & 0xFFFFu);
    } else {
        constexpr int W = 1 << zt_record_shift(ND, false);
        int32_t w[W];
        load_ints<W>(A.zt + p * W, w);
#pragma unroll
        for (int k = 0; k <= ND; ++k) v[k] = w[k];
    }
}

template <int ND>
__device__ __forceinline__ void store_zt(const SplitArgs& A, size_t p, const int32_t (&v)[1 + ND])
{
    if (A.zt_pack16) {
        constexpr int W = 1 << zt_record_shift(ND, true);
        int32_t w[W];
#pragma unroll
        for (int k = 0; k < W; ++k) w[k] = 0;
#pragma unroll
        for (int k = 0; k <= ND; ++k) w[k >> 1] |= (int32_t)((uint32_t)v[k] << (16 * (k & 1)));
        store_ints<W>(A.zt + p * W, w);
    } else {
        constexpr int W = 1 << zt_record_shift(ND, false);
        int32_t w[W];
#pragma unroll
        for (int k = 0; k < W; ++k) w[k] = 0;
#pragma unroll
        for (int k = 0; k <= ND; ++k) w[k] = v[k];
        store_ints<W>(A.zt + p * W, w);
    }
}

// The word pass's inputs of U tokens of a thread, fetched stage by stage: record position
// (a load of its own when the records are bucketed) and CSR position, then the packed
// (z, doc proposals) record.  Whether there is an xmap and how the record is packed is the
// same for the whole launch; with_record_layout() dispatches on both once, outside the loops,
// so that the loops are straight-line code in which the U loads of a stage are issued back
// to back.  (With the two tests inside, every token's loads were issued and awaited one after
// the other: eight dependent round trips per round of four tokens instead of two.)
template <int ND, int U, bool XM, bool P16>
struct TokenFetch {
    static constexpr int W = 1 << zt_record_shift(ND, P16);
    size_t q[U];
    uint32_t g[U];
    int32_t w[U][W];
    template <bool GID>
    __device__ __forceinline__ void positions(const SplitArgs& A, const int32_t (&p)[U])
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (XM) q[u] = (size_t)A.xmap[p[u]]; else q[u] = (size_t)p[u];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (GID) g[u] = (uint32_t)A.gid[p[u]]; else g[u] = 0u;
        }
    }
    __device__ __forceinline__ void records(const SplitArgs& A)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) load_ints<W>(A.zt + q[u] * W, w[u]);
    }
    // v[0] = z, v[1 + i] = the topic doc step i proposes
    __device__ __forceinline__ void decode(int u, int32_t (&v)[1 + ND]) const
    {
#pragma unroll
        for (int k = 0; k <= ND; ++k) {
            if constexpr (P16) v[k] = (int32_t)(((uint32_t)w[u][k >> 1] >> (16 * (k & 1))) & 0xFFFFu);
            else v[k] = w[u][k];
        }
    }
};

template <bool B>
struct Flag { static constexpr bool value = B; };

template <class F>
__device__ __forceinline__ void with_record_layout(const SplitArgs& A, F&& f)
{
    if (A.xmap) {
        if (A.zt_pack16) f(Flag<true>{}, Flag<true>{}); else f(Flag<true>{}, Flag<false>{});
    } else {
        if (A.zt_pack16) f(Flag<false>{}, Flag<true>{}); else f(Flag<false>{}, Flag<false>{});
    }
}

constexpr int32_t kRowItemRun = 8, kMixItemRun = 16, kPieceRun = 256;

// Eq. (9), (12): the topic of a random token of the document, or a uniform topic.
// zat(j) is the snapshot topic of the document's j-th token.
template <class ZAt>
__device__ __forceinline__ int32_t doc_proposal(uint32_t x0, uint32_t x1, int32_t L, int32_t K,
                                                double alphabar, ZAt zat)
{
#pragma clang fp contract(off)
    const double u0 = unit_open(x0);
    const double Ld = (double)L;
    if (u0 * (Ld + alphabar) < Ld) return zat(mulhi32(x1, (uint32_t)L));
    return (int32_t)mulhi32(x1, (uint32_t)K);
}

// (z, doc proposals of sweep A.sweep) of every token, from the doc-major snapshot.
// Needed when no doc pass has left them behind: first sweep, after lda_set_z, or when
// the chain shape changes.  One workgroup per document tile.
template <int NW, int ND>
__global__ __launch_bounds__(256) void doc_proposals_kernel(SplitArgs A)
{
    using C = Chain<NW, ND>;
    const int32_t c = xcd_contiguous(A.n_chunks);
    if (c >= A.n_chunks) return;
    const int32_t d0 = A.chunk_doc[c], d1 = A.chunk_doc[c + 1];
    const int32_t tok0 = A.doff[d0], ntok = A.doff[d1] - tok0;
    for (int32_t i = threadIdx.x; i < ntok; i += blockDim.x) {
        const uint32_t g = (uint32_t)(tok0 + i);
        int32_t row[1 + ND];
        row[0] = A.z[g];
        if constexpr (ND > 0) {
            const int32_t d = d0 + (int32_t)A.tokdoc[g];  // a long document is a tile of its own
            const int32_t b = A.doff[d], L = A.doff[d + 1] - b;
#pragma unroll
            for (int k = 0; k < ND; ++k) {
                uint32_t x[4];
                philox4x32_10(g, 0u, A.sweep, (uint32_t)C::doc_step(k), A.seed_lo, A.seed_hi, x);
                row[1 + k] = doc_proposal(x[0], x[1], L, A.K, A.alphabar,
                                          [&](uint32_t j) { return A.z[b + (int32_t)j]; });
            }
        }
        store_zt<ND>(A, (size_t)A.wpos[g], row);
    }
}

// ---- word pass -----------------------------------------------------------------------

// One item = up to kRowItemTokens consecutive tokens of one word.
template <int NW, int ND>
__global__ __launch_bounds__(1024) void word_pass_rows_kernel(SplitArgs A)
{
    using C = Chain<NW, ND>;
    extern __shared__ int32_t smem[];
    uint2* __restrict__ tab = reinterpret_cast<uint2*>(smem);  // [K] (split, alias)
    int32_t* __restrict__ row = smem + 2 * (size_t)A.K;        // [K] n_kw
    const int32_t it_i = xcd_runs(kRowItemRun);
    if (it_i >= A.n_row_items) return;
    const int4 it = A.row_items[it_i];  // (w, p0, n, 0)
    const int32_t K = A.K;
    const size_t wk = (size_t)it.x * (size_t)K;
    const int tid = threadIdx.x, nt = blockDim.x;
    {
        // staging: S entries of a thread in flight together
        constexpr int S = 4;
        for (int32_t k0 = tid; k0 < K; k0 += S * nt) {
            int32_t rv[S];
            uint2 ev[S];
#pragma unroll
            for (int q = 0; q < S; ++q) {
                const int32_t k = k0 + q * nt < K ? k0 + q * nt : K - 1;
                rv[q] = A.nkw[wk + k];
                if constexpr (NW > 0) ev[q] = *reinterpret_cast<const uint2*>(&A.alias[wk + k]);
            }
#pragma unroll
            for (int q = 0; q < S; ++q) {
                const int32_t k = k0 + q * nt < K ? k0 + q * nt : K - 1;  // past the end: the last entry again
                row[k] = rv[q];
                if constexpr (NW > 0) tab[k] = ev[q];
            }
        }
    }
    __syncthreads();
    const uint32_t capw = A.cap[it.x];
    with_record_layout(A, [&](auto xm, auto p16) {
        // U tokens per thread and round, their loads issued together stage by stage
        constexpr int U = 4;
        for (int32_t i0 = 0; i0 < it.z; i0 += U * nt) {
            int32_t p[U];
            bool live[U];
            TokenFetch<ND, U, decltype(xm)::value, decltype(p16)::value> f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int32_t i = i0 + u * nt + tid;
                live[u] = i < it.z;
                if (!live[u]) i = it.z - 1;  // redo the item's last token, drop the result
                p[u] = it.y + i;
            }
            f.template positions<(NW > 0)>(A, p);
            f.records(A);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int32_t zt[1 + ND], out[C::R];
                f.decode(u, zt);
#pragma unroll
                for (int k = 0; k < C::R; ++k) out[k] = 0;
                out[0] = row[zt[0]];
#pragma unroll
                for (int k = 0; k < NW; ++k) {
                    // Fig. 2: uniform bin, uniform height, keep the bin or take its alias
                    uint32_t x[4];
                    philox4x32_10(f.g[u], 0u, A.sweep, (uint32_t)C::word_step(k), A.seed_lo, A.seed_hi, x);
                    const uint32_t bin = mulhi32(x[0], (uint32_t)K);
                    const uint32_t rr = mulhi32(x[1], capw);
                    const uint2 e = tab[bin];
                    const int32_t t = (rr < e.x) ? (int32_t)bin : (int32_t)e.y;
                    out[C::rec_topic(k)] = topic_with_hint(t, x[2]);
                    out[C::rec_topic(k) + 1] = row[t];
                }
#pragma unroll
                for (int k = 0; k < ND; ++k) out[C::rec_doc(k)] = row[zt[1 + k]];
                if (live[u]) store_ints<C::R>(A.rec + (f.q[u] << C::rec_shift), out);
            }
        }
    });
}

// The word of word-major position p inside a piece: the last w with off[w] <= p, where
// off[0..nwords] are the piece's word offsets (off[0] <= p < off[nwords]).
__device__ __forceinline__ int32_t piece_word(const int32_t* off, int32_t nwords, int32_t p)
{
    int32_t lo = 0, hi = nwords;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (off[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

// One piece = tokens [p0, p0 + n) that belong to words [w0, w1).  STORE 0: every word
// has a dense row and a dense table; 1, 2: hybrid store (word_side.hpp).  The hybrid
// form advances U tokens per thread together, stage by stage, so that their gathers
// (word record, first probe of every n_kw lookup, table bin) are in flight at once.
template <int NW, int ND, int STORE>
__global__ __launch_bounds__(256) void word_pass_gather_kernel(SplitArgs A)
{
    using C = Chain<NW, ND>;
    __shared__ int32_t soff[kPieceWords + 1];
    const int32_t pc_i = xcd_runs(kPieceRun);
    if (pc_i >= A.n_pieces) return;
    const int4 pc = A.pieces[pc_i];  // (w0, w1, p0, n)
    const int32_t nwords = pc.y - pc.x;
    const int32_t K = A.K;
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int32_t i = tid; i <= nwords; i += nt) soff[i] = A.woff[pc.x + i];
    __syncthreads();
    if constexpr (STORE == 0) {
        with_record_layout(A, [&](auto xm, auto p16) {
            constexpr int U = 4;
            for (int32_t i0 = 0; i0 < pc.w; i0 += U * nt) {
                int32_t p[U], zt[U][1 + ND], out[U][C::R];
                size_t wk[U];
                uint32_t capw[U];
                bool live[U];
                TokenFetch<ND, U, decltype(xm)::value, decltype(p16)::value> f;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    int32_t i = i0 + u * nt + tid;
                    live[u] = i < pc.w;
                    if (!live[u]) i = pc.w - 1;  // redo the piece's last token, drop the result
                    p[u] = pc.z + i;
                }
                f.template positions<(NW > 0)>(A, p);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int32_t w = pc.x + piece_word(soff, nwords, p[u]);
                    wk[u] = (size_t)w * (size_t)K;
                    capw[u] = (NW > 0) ? A.cap[w] : 0u;
                }
                f.records(A);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    f.decode(u, zt[u]);
#pragma unroll
                    for (int k = 0; k < C::R; ++k) out[u][k] = 0;
                }
                // every gather of the round before the first use
                uint4 e[NW > 0 ? NW : 1][U];
                uint32_t bin[NW > 0 ? NW : 1][U], rr[NW > 0 ? NW : 1][U], hint[NW > 0 ? NW : 1][U];
#pragma unroll
                for (int k = 0; k < NW; ++k) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        uint32_t x[4];
                        philox4x32_10(f.g[u], 0u, A.sweep, (uint32_t)C::word_step(k), A.seed_lo, A.seed_hi, x);
                        bin[k][u] = mulhi32(x[0], (uint32_t)K);
                        rr[k][u] = mulhi32(x[1], capw[u]);
                        hint[k][u] = x[2];
                        e[k][u] = A.alias[wk[u] + bin[k][u]];  // brings n_kw of both outcomes along
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    out[u][0] = A.nkw[wk[u] + (size_t)zt[u][0]];
#pragma unroll
                    for (int k = 0; k < ND; ++k) out[u][C::rec_doc(k)] = A.nkw[wk[u] + (size_t)zt[u][1 + k]];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int k = 0; k < NW; ++k) {
                        const bool keep = rr[k][u] < e[k][u].x;
                        out[u][C::rec_topic(k)] =
                            topic_with_hint(keep ? (int32_t)bin[k][u] : (int32_t)e[k][u].y, hint[k][u]);
                        out[u][C::rec_topic(k) + 1] = keep ? (int32_t)e[k][u].z : (int32_t)e[k][u].w;
                    }
                    if (live[u]) store_ints<C::R>(A.rec + (f.q[u] << C::rec_shift), out[u]);
                }
            }
        });
    } else {
        BetaTable bt{};
        if constexpr (NW > 0) bt = load_beta_table(A);
        with_record_layout(A, [&](auto xm, auto p16) {
            constexpr int U = 2;
            for (int32_t i0 = 0; i0 < pc.w; i0 += U * nt) {
                int32_t p[U], w[U], zt[U][1 + ND], out[U][C::R];
                bool live[U];
                WordMeta meta[U];
                WordSide wv[U];
                TokenFetch<ND, U, decltype(xm)::value, decltype(p16)::value> f;
                // stage 1: positions (and CSR positions), the words by bisection of the piece's
                // offsets in LDS, then every word record and token record
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    // lanes past the end of the piece redo its last token and drop the result
                    int32_t i = i0 + u * nt + tid;
                    live[u] = i < pc.w;
                    if (!live[u]) i = pc.w - 1;
                    p[u] = pc.z + i;
                }
                f.template positions<(NW > 0)>(A, p);
#pragma unroll
                for (int u = 0; u < U; ++u) w[u] = pc.x + piece_word(soff, nwords, p[u]);
#pragma unroll
                for (int u = 0; u < U; ++u) meta[u] = load_word_meta(A, w[u]);
                f.records(A);
                uint32_t kinds = 0;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    wv[u] = word_from_meta<STORE>(A, w[u], meta[u]);
                    kinds |= wv[u].kind;
                    f.decode(u, zt[u]);
#pragma unroll
                    for (int k = 0; k < C::R; ++k) out[u][k] = 0;
                }
                if (__any(kinds & kKindListOnly)) {
                    // a word whose row is not kept: its lookups search its mixture table
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        out[u][0] = nkw_lookup<STORE>(wv[u], zt[u][0]);
#pragma unroll
                        for (int k = 0; k < ND; ++k) out[u][C::rec_doc(k)] = nkw_lookup<STORE>(wv[u], zt[u][1 + k]);
#pragma unroll
                        for (int k = 0; k < NW; ++k) {
                            uint32_t x[4];
                            philox4x32_10(f.g[u], 0u, A.sweep, (uint32_t)C::word_step(k), A.seed_lo, A.seed_hi, x);
                            WordDraw d;
                            const uint4 e = *word_draw_address(wv[u], bt, (uint32_t)K, x[0], x[1], x[3], d);
                            int32_t t, nwt;
                            if (!word_draw_decode(d, e, t, nwt)) nwt = nkw_lookup<STORE>(wv[u], t);
                            out[u][C::rec_topic(k)] = topic_with_hint(t, x[2]);
                            out[u][C::rec_topic(k) + 1] = nwt;
                        }
                        if (live[u]) store_ints<C::R>(A.rec + (f.q[u] << C::rec_shift), out[u]);
                    }
                    continue;
                }
                // stage 2: the first probe of every n_kw lookup and the table bin of every draw
                NkwFetch pr[U][1 + ND];
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int k = 0; k <= ND; ++k) pr[u][k] = nkw_fetch_begin<STORE>(wv[u], zt[u][k]);
                WordDraw d[NW > 0 ? NW : 1][U];
                uint4 e[NW > 0 ? NW : 1][U];
                uint32_t hint[NW > 0 ? NW : 1][U];
#pragma unroll
                for (int k = 0; k < NW; ++k) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        uint32_t x[4];
                        philox4x32_10(f.g[u], 0u, A.sweep, (uint32_t)C::word_step(k), A.seed_lo, A.seed_hi, x);
                        e[k][u] = *word_draw_address(wv[u], bt, (uint32_t)K, x[0], x[1], x[3], d[k][u]);
                        hint[k][u] = x[2];
                    }
                }
                // stage 3: the proposals; a draw from the beta term still needs its n_kw
                int32_t t[NW > 0 ? NW : 1][U], nwt[NW > 0 ? NW : 1][U];
                bool known[NW > 0 ? NW : 1][U];
                NkwFetch pb[NW > 0 ? NW : 1][U];
#pragma unroll
                for (int k = 0; k < NW; ++k) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        known[k][u] = word_draw_decode(d[k][u], e[k][u], t[k][u], nwt[k][u]);
                        if (!known[k][u]) pb[k][u] = nkw_fetch_begin<STORE>(wv[u], t[k][u]);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int k = 0; k < NW; ++k) {
                        if (!known[k][u]) nwt[k][u] = nkw_fetch_finish<STORE>(wv[u], t[k][u], pb[k][u]);
                        out[u][C::rec_topic(k)] = topic_with_hint(t[k][u], hint[k][u]);
                        out[u][C::rec_topic(k) + 1] = nwt[k][u];
                    }
                    out[u][0] = nkw_fetch_finish<STORE>(wv[u], zt[u][0], pr[u][0]);
#pragma unroll
                    for (int k = 0; k < ND; ++k)
                        out[u][C::rec_doc(k)] = nkw_fetch_finish<STORE>(wv[u], zt[u][1 + k], pr[u][1 + k]);
                    if (live[u]) store_ints<C::R>(A.rec + (f.q[u] << C::rec_shift), out[u]);
                }
            }
        });
    }
}

// One item = up to kRowItemTokens consecutive tokens of one mixture word that has a dense
// n_kw row.  The row is rebuilt in LDS from the word's list of non-zeros (8 bytes per
// non-zero instead of 4 K bytes from memory), so every n_kw lookup is an LDS read; the
// draw gathers one bin of the word's own table or of the shared beta table.
template <int NW, int ND>
__global__ __launch_bounds__(512) void word_pass_mix_rows_kernel(SplitArgs A)
{
    using C = Chain<NW, ND>;
    extern __shared__ int32_t smem[];
    int32_t* __restrict__ row = smem;  // [K] n_kw
    const int32_t it_i = xcd_runs(kMixItemRun);
    if (it_i >= A.n_mix_items) return;
    const int4 it = A.mix_items[it_i];  // (w, p0, n, 0)
    const int32_t K = A.K, w = it.x;
    const int tid = threadIdx.x, nt = blockDim.x;
    with_record_layout(A, [&](auto xm, auto p16) {
        constexpr int U = 2;
        int32_t p[U];
        bool live[U];
        TokenFetch<ND, U, decltype(xm)::value, decltype(p16)::value> f;
        auto place = [&](int32_t i0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int32_t i = i0 + u * nt + tid;
                live[u] = i < it.z;
                if (!live[u]) i = it.z - 1;  // redo the item's last token, drop the result
                p[u] = it.y + i;
            }
        };
        // The first round's token loads and the thread's first list entry are requested before
        // the row is built: they do not depend on it, and its two barriers hide their latency.
        place(0);
        f.template positions<(NW > 0)>(A, p);
        f.records(A);
        const size_t off = A.sp_off[w];
        const int32_t nnz = A.sp_nnz[w];
        const int32_t i_first = tid < nnz ? tid : (nnz > 0 ? nnz - 1 : 0);
        int32_t tp0 = 0, ct0 = 0;
        if (nnz > 0) {
            tp0 = A.sp_topic[off + i_first];
            ct0 = A.sp_count[off + i_first];
        }
        const WordSide wv = load_word<1>(A, w);
        BetaTable bt{};
        if constexpr (NW > 0) bt = load_beta_table(A);
        for (int32_t k = tid; k < K; k += nt) row[k] = 0;
        __syncthreads();
        if (nnz > 0) row[tp0] = ct0;  // threads past the list's end repeat its last entry
        for (int32_t i = tid + nt; i < nnz; i += nt) row[A.sp_topic[off + i]] = A.sp_count[off + i];
        __syncthreads();
        for (int32_t i0 = 0;;) {
            int32_t zt[U][1 + ND], out[U][C::R];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                f.decode(u, zt[u]);
#pragma unroll
                for (int k = 0; k < C::R; ++k) out[u][k] = 0;
                out[u][0] = row[zt[u][0]];
            }
#pragma unroll
            for (int k = 0; k < NW; ++k) {
                WordDraw d[U];
                uint4 e[U];
                uint32_t hint[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    uint32_t x[4];
                    philox4x32_10(f.g[u], 0u, A.sweep, (uint32_t)C::word_step(k), A.seed_lo, A.seed_hi, x);
                    e[u] = *word_draw_address(wv, bt, (uint32_t)K, x[0], x[1], x[3], d[u]);
                    hint[u] = x[2];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    int32_t t, nwt;
                    if (!word_draw_decode(d[u], e[u], t, nwt)) nwt = row[t];
                    out[u][C::rec_topic(k)] = topic_with_hint(t, hint[u]);
                    out[u][C::rec_topic(k) + 1] = nwt;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int k = 0; k < ND; ++k) out[u][C::rec_doc(k)] = row[zt[u][1 + k]];
                if (live[u]) store_ints<C::R>(A.rec + (f.q[u] << C::rec_shift), out[u]);
            }
            i0 += U * nt;
            if (i0 >= it.z) break;
            place(i0);
            f.template positions<(NW > 0)>(A, p);
            f.records(A);
        }
    });
}

// ---- doc pass ------------------------------------------------------------------------

struct TileDoc {  // document staged in an LDS tile
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

struct LongDoc {  // document hashed in the global workspace
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

// The chains of T tokens of one thread, advanced together stage by stage.  doc[u] is
// token u's document, g[u] its CSR position (the Philox counter), r[u] its word-pass record, z0[u] its snapshot topic and nd0[u] = n_kd of it.
template <int NW, int ND, int T, class DocView>
__device__ __forceinline__ void doc_pass_chains(const SplitArgs& A, const DocView (&doc)[T],
                                                const uint32_t (&g)[T],
                                                const int32_t (&r)[T][Chain<NW, ND>::R],
                                                const int32_t (&z0)[T], const int32_t (&nd0)[T],
                                                const int32_t* __restrict__ nk, int32_t (&s)[T])
{
#pragma clang fp contract(off)
    using C = Chain<NW, ND>;
    int32_t nds[T], nws[T], nks[T];
#pragma unroll
    for (int u = 0; u < T; ++u) {
        nds[u] = nd0[u];
        s[u] = z0[u];
        nks[u] = nk[z0[u]];
        nws[u] = r[u][0];
    }
    // Proposals do not depend on the chain's state, so every step's proposal, its n_kd probe
    // and its n_k gather are issued before the first accept test: one round trip to L2
    // for all of them instead of one per step.
    uint32_t x2[C::M][T];
    int32_t t[C::M][T], ndt[C::M][T], nwt[C::M][T], nkt[C::M][T];
#pragma unroll
    for (int j = 0; j < C::M; ++j) {
        const bool word_step = C::is_word(j);
        const int i = C::index(j);
#pragma unroll
        for (int u = 0; u < T; ++u) {
            if (word_step) {
                // the record's topic int: the topic, and above it the top bits of x2
                x2[j][u] = (uint32_t)r[u][C::rec_topic(i)] & ~kHintSpan;
                t[j][u] = (int32_t)((uint32_t)r[u][C::rec_topic(i)] & kHintSpan);
                nwt[j][u] = r[u][C::rec_topic(i) + 1];
                ndt[j][u] = doc[u].count(t[j][u]);
            } else {
                uint32_t x[4];
                philox4x32_10(g[u], 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
                x2[j][u] = x[2];
                const double u0 = unit_open(x[0]);
                const double Ld = (double)doc[u].L;
                if (u0 * (Ld + A.alphabar) < Ld) {
                    doc[u].token(mulhi32(x[1], (uint32_t)doc[u].L), t[j][u], ndt[j][u]);
                } else {
                    t[j][u] = (int32_t)mulhi32(x[1], (uint32_t)A.K);
                    ndt[j][u] = doc[u].count(t[j][u]);
                }
                nwt[j][u] = r[u][C::rec_doc(i)];
            }
            nkt[j][u] = nk[t[j][u]];
        }
    }
#pragma unroll
    for (int j = 0; j < C::M; ++j) {
        const bool word_step = C::is_word(j);
#pragma unroll
        for (int u = 0; u < T; ++u) {
            const int32_t tt = t[j][u], nd_t = ndt[j][u], nw_t = nwt[j][u], nk_t = nkt[j][u];
            const int32_t ms = (s[u] == z0[u]) ? 1 : 0;
            const int32_t mt = (tt == z0[u]) ? 1 : 0;
            // Eq. (4) ratio p(t)/p(s), the token removed at its snapshot topic
            double num = (double)(nd_t - mt) + A.alpha;
            num = num * ((double)(nw_t - mt) + A.beta);
            num = num * ((double)(nks[u] - ms) + A.betabar);
            double den = (double)(nds[u] - ms) + A.alpha;
            den = den * ((double)(nws[u] - ms) + A.beta);
            den = den * ((double)(nk_t - mt) + A.betabar);
            if (word_step) {  // Eq. (8): times p_w(s)/p_w(t)
                num = num * ((double)nws[u] + A.beta);
                num = num * ((double)nk_t + A.betabar);
                den = den * ((double)nw_t + A.beta);
                den = den * ((double)nks[u] + A.betabar);
            } else {          // Eq. (11): times p_d(s)/p_d(t)
                num = num * ((double)nds[u] + A.alpha);
                den = den * ((double)nd_t + A.alpha);
            }
            bool accept;
            if (word_step) {
                // x2 is known up to its low bits.  The test is monotone in x2 (a rounded product
                // of a positive number is monotone), so if both ends of the interval agree the
                // test is decided; if they differ in any lane, the wave draws the number itself.
                const bool at_low = unit_open(x2[j][u]) * den < num;
                const bool at_high = unit_open(x2[j][u] | kHintSpan) * den < num;
                accept = at_high;
                if (__any((at_low != at_high) && (tt != s[u]))) {
                    uint32_t x[4];
                    philox4x32_10(g[u], 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
                    accept = unit_open(x[2]) * den < num;
                }
            } else {
                accept = unit_open(x2[j][u]) * den < num;
            }
            accept = accept && (tt != s[u]);
            s[u] = accept ? tt : s[u];
            nds[u] = accept ? nd_t : nds[u];
            nws[u] = accept ? nw_t : nws[u];
            nks[u] = accept ? nk_t : nks[u];
        }
    }
}

// What a thread holds of its T tokens of one tile before the tile is staged.
template <int T, int R>
struct TileTokens {
    int32_t d0, d1, tok0, ntok;  // uniform over the workgroup
    bool valid;                  // uniform: a tile this kernel handles
    uint32_t g[T];
    int32_t wp[T], idx[T], z0[T], dl[T], r[T][R];
    int32_t doc_end;             // doff of the thread's own document of the tile (clamped to the last)
    bool live[T];
};

// first half of a tile's loads: the tile's bounds and, per token, the word-major position
template <int T, int R>
__device__ __forceinline__ void tile_issue_positions(const SplitArgs& A, int32_t c, TileTokens<T, R>& t)
{
    t.valid = c < A.n_chunks;
    if (!t.valid) return;
    t.d0 = A.chunk_doc[c];
    t.d1 = A.chunk_doc[c + 1];
    t.tok0 = A.chunk_tok[c];
    t.ntok = A.chunk_tok[c + 1] - t.tok0;
    // nothing / a long document (the long-document kernel's)
    t.valid = !(t.ntok == 0 || (t.d1 - t.d0 == 1 && t.ntok > A.max_doc_tokens));
    if (!t.valid) return;
#pragma unroll
    for (int u = 0; u < T; ++u) {
        // lanes past the end of the tile redo its last token and drop the result
        int32_t i = (int32_t)threadIdx.x + u * (int32_t)blockDim.x;
        t.live[u] = i < t.ntok;
        if (!t.live[u]) i = t.ntok - 1;
        t.idx[u] = i;
        t.g[u] = (uint32_t)(t.tok0 + i);
        t.wp[u] = __builtin_nontemporal_load(&A.wpos[t.g[u]]);
    }
    // Loads return in the order they were issued: what the staging of the documents needs is
    // requested before the record gather, so that the staging does not wait for the gather.
#pragma unroll
    for (int u = 0; u < T; ++u) {
        t.z0[u] = __builtin_nontemporal_load(&A.z[t.g[u]]);
        t.dl[u] = (int32_t)__builtin_nontemporal_load(&A.tokdoc[t.g[u]]);
    }
    const int32_t nd = t.d1 - t.d0;
    t.doc_end = A.doff[t.d0 + ((int32_t)threadIdx.x < nd ? (int32_t)threadIdx.x : nd)];
}

// second half: the word-pass records (one random line per token)
template <int T, int R, int RS>
__device__ __forceinline__ void tile_issue_records(const SplitArgs& A, TileTokens<T, R>& t)
{
    if (!t.valid) return;
#pragma unroll
    for (int u = 0; u < T; ++u) load_ints<R>(A.rec + ((size_t)t.wp[u] << RS), t.r[u]);
}

// Stage the tile as load_doc_tile does (doc_tile.hpp: same LDS layout, same tables) but keep
// what each thread learns about its own tokens in registers -- the thread that inserts a
// token into its document's table is the one that runs its chain --, run the chains, write
// the new assignment, and from it draw the doc proposals of the next sweep.
template <int NW, int ND, int T>
__device__ __forceinline__ void tile_process(const SplitArgs& A, int32_t* smem,
                                             const int32_t* __restrict__ nk,
                                             const TileTokens<T, Chain<NW, ND>::R>& t)
{
    using C = Chain<NW, ND>;
    DocTile tile;
    tile.zs = reinterpret_cast<uint32_t*>(smem);
    tile.tab = reinterpret_cast<uint32_t*>(smem + A.cap_tokens);
    tile.sdoff = smem + 3 * (size_t)A.cap_tokens;
    tile.nd = t.d1 - t.d0;
    tile.tok0 = t.tok0;
    tile.ntok = t.ntok;
    int32_t nd0[T], s[T];
    uint32_t slot[T];
    // document offsets inside the tile: a thread's first one was requested with its tokens
    if ((int32_t)threadIdx.x <= tile.nd) tile.sdoff[threadIdx.x] = t.doc_end - t.tok0;
    for (int32_t i = threadIdx.x + blockDim.x; i <= tile.nd; i += blockDim.x) tile.sdoff[i] = A.doff[t.d0 + i] - t.tok0;
#pragma unroll
    for (int u = 0; u < T; ++u) {
        if (t.live[u]) {
            tile.zs[t.idx[u]] = (uint32_t)t.z0[u];
            reinterpret_cast<uint2*>(tile.tab)[t.idx[u]] = make_uint2(kEmptySlot, kEmptySlot);
        }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < T; ++u) {
        if (t.live[u]) {
            slot[u] = tile.table(t.dl[u]).insert(t.z0[u]);
            tile.zs[t.idx[u]] = (uint32_t)t.z0[u] | (slot[u] << kTopicBits);  // own element only
        }
    }
    __syncthreads();
    TileDoc doc[T];
#pragma unroll
    for (int u = 0; u < T; ++u) {
        const int32_t b = tile.sdoff[t.dl[u]];
        doc[u].L = tile.sdoff[t.dl[u] + 1] - b;
        doc[u].tab = tile.table(t.dl[u]);
        doc[u].zs = tile.zs + b;
        if (!t.live[u]) slot[u] = tile.zs[t.idx[u]] >> kTopicBits;  // a clone of the last token
        nd0[u] = doc[u].tab.count_at(slot[u]);
    }
    doc_pass_chains<NW, ND, T>(A, doc, t.g, t.r, t.z0, nd0, nk, s);
#pragma unroll
    for (int u = 0; u < T; ++u)
        if (t.live[u]) __builtin_nontemporal_store(s[u], &A.znew[t.g[u]]);
    // the tile's new assignment replaces the staged snapshot; from it, the doc proposals
    // of the next sweep
    __syncthreads();
#pragma unroll
    for (int u = 0; u < T; ++u)
        if (t.live[u]) tile.zs[t.idx[u]] = (uint32_t)s[u];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < T; ++u) {
        if (!t.live[u]) continue;
        int32_t row[1 + ND];
        row[0] = s[u];
#pragma unroll
        for (int k = 0; k < ND; ++k) {
            uint32_t x[4];
            philox4x32_10(t.g[u], 0u, A.sweep + 1u, (uint32_t)C::doc_step(k), A.seed_lo, A.seed_hi, x);
            const uint32_t* zs = doc[u].zs;
            row[1 + k] = doc_proposal(x[0], x[1], doc[u].L, A.K, A.alphabar,
                                      [&](uint32_t j) { return (int32_t)zs[j]; });
        }
        store_zt<ND>(A, (size_t)t.wp[u], row);
    }
}

// One workgroup per document tile; a thread runs the chains of up to T of its tokens,
// interleaved.  Chains of up to two steps with up to two tokens per thread are compiled for
// a fixed number of waves per SIMD (7 in blocks of up to 256 threads, 6 up to 768): one more
// resident workgroup per CU hides more of the gather latency than the few registers it
// costs.  Longer chains take the registers they need: two interleaved four-step chains use
// about 100, one uses 62, which is why the launcher gives them one token per thread.
//
// NKL: the workgroup keeps a copy of n_k in LDS behind the tile (K <= kNkLdsTopics).  The
// three n_k reads of a token are otherwise three separate requests to L2 (the array is larger
// than the L1), and the rate of such requests, not their bytes, is what bounded this kernel:
// without them it ran 14.8 instead of 22.7 ms on the benchmark workload.
template <int NW, int ND, int T, int MAXB, bool NKL>
__global__ __launch_bounds__(MAXB, (T <= 2 && NW + ND <= 2) ? (MAXB <= 256 ? 7 : (MAXB <= 768 ? 6 : 1)) : 1) void doc_pass_tiles_kernel(SplitArgs A)
{
    using C = Chain<NW, ND>;
    extern __shared__ int32_t smem[];
    const int32_t* __restrict__ nk = A.nk;
    const int32_t c = xcd_contiguous(A.n_chunks);
    if (c >= A.n_chunks) return;
    // Order of the requests: the token streams the staging needs, the first part of n_k, then
    // the word-pass records (one random line per token, addressed by the first stream).  Loads
    // complete in order, so the n_k copy and the staging of the documents go ahead while the
    // gather is still on its way; the chains are the first to need it.
    TileTokens<T, C::R> t;
    tile_issue_positions<T, C::R>(A, c, t);
    if (!t.valid) return;  // uniform over the workgroup
    if constexpr (NKL) {
        // 16 bytes per load (n_k is allocated, and the LDS copy sized, up to the next multiple of
        // 4 topics); the first kNkAhead loads of a thread are in flight together.  Threads past
        // the end repeat the last element: same value to the same place, no branch.
        constexpr int kNkAhead = 4;
        const int32_t nq = (A.K + 3) / 4;
        int32_t* nk_lds = smem + A.tile_lds_ints;
        const int4* __restrict__ src = reinterpret_cast<const int4*>(A.nk);
        int4* dst = reinterpret_cast<int4*>(nk_lds);
        int4 ahead[kNkAhead];
        int32_t at[kNkAhead];
#pragma unroll
        for (int b = 0; b < kNkAhead; ++b) {
            const int32_t k = (int32_t)threadIdx.x + b * (int32_t)blockDim.x;
            at[b] = k < nq ? k : nq - 1;
            ahead[b] = src[at[b]];
        }
        tile_issue_records<T, C::R, C::rec_shift>(A, t);
#pragma unroll
        for (int b = 0; b < kNkAhead; ++b) dst[at[b]] = ahead[b];
        for (int32_t k = threadIdx.x + kNkAhead * blockDim.x; k < nq; k += blockDim.x) dst[k] = src[k];
        nk = nk_lds;  // the staging's first barrier makes it visible
    } else {
        tile_issue_records<T, C::R, C::rec_shift>(A, t);
    }
    tile_process<NW, ND, T>(A, smem, nk, t);
}

template <int NW, int ND>
__global__ __launch_bounds__(1024) void doc_pass_long_kernel(SplitArgs A)
{
    using C = Chain<NW, ND>;
    constexpr int T = 2;
    const int32_t d = A.long_doc[blockIdx.x];
    const int32_t tok0 = A.doff[d];
    const int32_t Ld = A.doff[d + 1] - tok0;
    const int64_t s0 = A.long_slot[blockIdx.x];
    const GlobalDocTable table = load_long_doc(A.long_keys + s0, A.long_cnts + s0, A.z + tok0, Ld);
    for (int32_t base = 0; base < Ld; base += T * (int32_t)blockDim.x) {
        LongDoc doc[T];
        uint32_t own[T], g[T];
        int32_t wp[T], s[T];
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
            wp[u] = A.wpos[g[u]];
        }
        int32_t r[T][C::R];
#pragma unroll
        for (int u = 0; u < T; ++u) load_ints<C::R>(A.rec + ((size_t)wp[u] << C::rec_shift), r[u]);
        int32_t z0[T], nd0[T];
#pragma unroll
        for (int u = 0; u < T; ++u) doc[u].token(own[u], z0[u], nd0[u]);
        doc_pass_chains<NW, ND, T>(A, doc, g, r, z0, nd0, A.nk, s);
#pragma unroll
        for (int u = 0; u < T; ++u)
            if (live[u])
                __hip_atomic_store(&A.znew[g[u]], s[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();  // the document's new assignment is complete
    for (int32_t i = threadIdx.x; i < Ld; i += blockDim.x) {
        const uint32_t g = (uint32_t)(tok0 + i);
        int32_t row[1 + ND];
        row[0] = __hip_atomic_load(&A.znew[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int k = 0; k < ND; ++k) {
            uint32_t x[4];
            philox4x32_10(g, 0u, A.sweep + 1u, (uint32_t)C::doc_step(k), A.seed_lo, A.seed_hi, x);
            row[1 + k] = doc_proposal(x[0], x[1], Ld, A.K, A.alphabar, [&](uint32_t j) {
                return __hip_atomic_load(&A.znew[tok0 + (int32_t)j], __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
            });
        }
        store_zt<ND>(A, (size_t)A.wpos[g], row);
    }
}

// ---- launch --------------------------------------------------------------------------

template <class Kern>
int raise_lds_limit(lda_ctx* c, Kern kern, size_t lds)
{
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    return LDA_OK;
}

template <int NW, int ND, int T, int MAXB, bool NKL>
int launch_doc_tiles_as(lda_ctx* c, const SplitArgs& A, size_t lds)
{
    auto kern = doc_pass_tiles_kernel<NW, ND, T, MAXB, NKL>;
    const int rc = raise_lds_limit(c, kern, lds);
    if (rc != LDA_OK) return rc;
    hipLaunchKernelGGL(kern, dim3(xcd_grid(A.n_chunks)), dim3(A.doc_block), lds, c->stream, A);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

template <int NW, int ND, int T>
int launch_doc_tiles(lda_ctx* c, const SplitArgs& A, size_t lds)
{
    if (c->K <= kNkLdsTopics) {  // with the workgroup's own copy of n_k
        lds += sizeof(int32_t) * (size_t)((c->K + 3) / 4 * 4);
        if (A.doc_block <= 256) return launch_doc_tiles_as<NW, ND, T, 256, true>(c, A, lds);
        if (A.doc_block <= 768) return launch_doc_tiles_as<NW, ND, T, 768, true>(c, A, lds);
        return launch_doc_tiles_as<NW, ND, T, 1024, true>(c, A, lds);
    }
    if (A.doc_block <= 256) return launch_doc_tiles_as<NW, ND, T, 256, false>(c, A, lds);
    return launch_doc_tiles_as<NW, ND, T, 1024, false>(c, A, lds);
}

int tokens_per_thread(const SplitArgs& A)
{
    return (A.cap_tokens + A.doc_block - 1) / A.doc_block;
}

template <int NW, int ND>
int launch_chain(lda_ctx* c, const SplitArgs& A, bool need_proposals)
{
    int rc;
    const bool timed = c->opt.time_sweep_passes != 0;
    if (timed) {
        for (hipEvent_t& e : c->pass_ev)
            if (!e) LDA_HIP(c, hipEventCreate(&e));
        LDA_HIP(c, hipEventRecord(c->pass_ev[0], c->stream));
    }
    if (need_proposals) {
        hipLaunchKernelGGL((doc_proposals_kernel<NW, ND>), dim3(xcd_grid(A.n_chunks)), dim3(256), 0,
                           c->stream, A);
        LDA_HIP(c, hipGetLastError());
    }
    if (c->n_row_items > 0) {
        auto kern = word_pass_rows_kernel<NW, ND>;
        const size_t lds = sizeof(int32_t) * 3 * (size_t)c->K;
        if ((rc = raise_lds_limit(c, kern, lds)) != LDA_OK) return rc;
        hipLaunchKernelGGL(kern, dim3(xcd_runs_grid(c->n_row_items, kRowItemRun)), dim3(1024), lds, c->stream, A);
        LDA_HIP(c, hipGetLastError());
    }
    if (c->n_mix_items > 0) {
        auto kern = word_pass_mix_rows_kernel<NW, ND>;
        const size_t lds = sizeof(int32_t) * (size_t)c->K;
        if ((rc = raise_lds_limit(c, kern, lds)) != LDA_OK) return rc;
        hipLaunchKernelGGL(kern, dim3(xcd_runs_grid(c->n_mix_items, kMixItemRun)), dim3(512), lds, c->stream, A);
        LDA_HIP(c, hipGetLastError());
    }
    if (c->n_gather_pieces > 0) {
        const dim3 grid(xcd_runs_grid(c->n_gather_pieces, kPieceRun));
        if (!c->hybrid)
            hipLaunchKernelGGL((word_pass_gather_kernel<NW, ND, 0>), grid, dim3(256), 0, c->stream, A);
        else if (c->H == c->V)
            hipLaunchKernelGGL((word_pass_gather_kernel<NW, ND, 1>), grid, dim3(256), 0, c->stream, A);
        else
            hipLaunchKernelGGL((word_pass_gather_kernel<NW, ND, 2>), grid, dim3(256), 0, c->stream, A);
        LDA_HIP(c, hipGetLastError());
    }
    if (timed) LDA_HIP(c, hipEventRecord(c->pass_ev[1], c->stream));
    if (A.n_chunks > 0) {
        const size_t lds = sizeof(int32_t) * (size_t)A.tile_lds_ints;
        const int tpt = tokens_per_thread(A);
        rc = tpt <= 1 ? launch_doc_tiles<NW, ND, 1>(c, A, lds)
           : tpt <= 2 ? launch_doc_tiles<NW, ND, 2>(c, A, lds)
                      : launch_doc_tiles<NW, ND, 4>(c, A, lds);
        if (rc != LDA_OK) return rc;
    }
    if (timed) {
        LDA_HIP(c, hipEventRecord(c->pass_ev[2], c->stream));
        c->pass_ev_recorded = true;
    }
    if (c->n_long > 0) {
        hipLaunchKernelGGL((doc_pass_long_kernel<NW, ND>), dim3(c->n_long), dim3(1024), 0, c->stream,
                           A);
        LDA_HIP(c, hipGetLastError());
    }
    return LDA_OK;
}

// word and doc steps of a chain of mh_steps steps under proposal mode `mode`
void chain_shape(int32_t mode, int32_t mh_steps, int32_t& nw, int32_t& nd)
{
    if (mode == 1) { nw = mh_steps; nd = 0; }
    else if (mode == 2) { nw = 0; nd = mh_steps; }
    else { nw = (mh_steps + 1) / 2; nd = mh_steps / 2; }
}

template <class T>
int grow(lda_ctx* c, T** p, size_t* have, size_t need, const char* what)
{
    if (*have >= need) return LDA_OK;
    device_free(c, *p);
    *p = nullptr;
    *have = 0;
    const int rc = device_malloc(c, p, need, what);
    if (rc != LDA_OK) return rc;
    *have = need;
    return LDA_OK;
}

}  // namespace

// Chains of 1..4 steps in the cycle mode (and the one-step word chain), tiles of at most
// 4 tokens per thread; everything else runs the fused kernel.
bool split_sweep_supported(const lda_ctx* c, int32_t mh_steps)
{
    if (mh_steps < 1 || mh_steps > 4) return false;
    if (c->opt.proposal_mode == 2 || (c->opt.proposal_mode == 1 && mh_steps != 1)) return false;
    return (c->chunk_tokens + c->sweep_block - 1) / c->sweep_block <= 4;
}

// Work lists of the word pass from the word segment offsets.
int setup_split_sweep(lda_ctx* c, const std::vector<int32_t>& woff)
{
    std::vector<int4> items, mix_items, pieces;
    const int32_t V = c->V;
    int32_t w0 = -1;  // first word of the open piece
    auto close_piece = [&](int32_t w_end) {
        if (w0 >= 0 && woff[w_end] > woff[w0])
            pieces.push_back(make_int4(w0, w_end, woff[w0], woff[w_end] - woff[w0]));
        w0 = -1;
    };
    // rows are staged for frequent words with a dense row and a dense table of at most
    // max_alias_topics() bins (12 bytes of LDS per topic)
    const bool rows_fit = c->K <= max_alias_topics();
    for (int32_t w = 0; w < V; ++w) {
        const int32_t b = woff[w], n = woff[w + 1] - b;
        const bool dense_dense = !c->hybrid || (c->h_wkind[w] & 3) == 3;
        if (n >= kRowMinTokens && rows_fit && dense_dense) {
            close_piece(w);
            for (int32_t p = b; p < b + n; p += kRowItemTokens)
                items.push_back(make_int4(w, p, std::min(kRowItemTokens, b + n - p), 0));
            continue;
        }
        // a mixture word with a dense row of at most kMixRowTopics topics and enough
        // tokens to pay for clearing an LDS row
        if (c->hybrid && (c->h_wkind[w] & 3) == 1 && c->K <= kMixRowTopics && n >= kMixRowMinTokens) {
            close_piece(w);
            for (int32_t p = b; p < b + n; p += kRowItemTokens)
                mix_items.push_back(make_int4(w, p, std::min(kRowItemTokens, b + n - p), 0));
            continue;
        }
        if (n > kPieceTokens) {  // a long word that cannot be staged: pieces of its own
            close_piece(w);
            for (int32_t p = b; p < b + n; p += kPieceTokens)
                pieces.push_back(make_int4(w, w + 1, p, std::min(kPieceTokens, b + n - p)));
            continue;
        }
        if (w0 >= 0 && (woff[w + 1] - woff[w0] > kPieceTokens || w + 1 - w0 > kPieceWords))
            close_piece(w);
        if (w0 < 0) w0 = w;
    }
    close_piece(V);
    c->n_row_items = (int32_t)items.size();
    c->n_mix_items = (int32_t)mix_items.size();
    if (!mix_items.empty()) {
        LDA_ALLOC(c, &c->d_mix_items, mix_items.size(), "word-pass work list");
        LDA_HIP(c, hipMemcpy(c->d_mix_items, mix_items.data(), sizeof(int4) * mix_items.size(),
                             hipMemcpyHostToDevice));
    }
    c->n_gather_pieces = (int32_t)pieces.size();
    if (!items.empty()) {
        LDA_ALLOC(c, &c->d_row_items, items.size(), "word-pass work list");
        LDA_HIP(c, hipMemcpy(c->d_row_items, items.data(), sizeof(int4) * items.size(),
                             hipMemcpyHostToDevice));
    }
    if (!pieces.empty()) {
        LDA_ALLOC(c, &c->d_gather_pieces, pieces.size(), "word-pass work list");
        LDA_HIP(c, hipMemcpy(c->d_gather_pieces, pieces.data(), sizeof(int4) * pieces.size(),
                             hipMemcpyHostToDevice));
    }
    return LDA_OK;
}

int launch_sweep_split(lda_ctx* c, int32_t mh_steps)
{
    int32_t nw, nd;
    chain_shape(c->opt.proposal_mode, mh_steps, nw, nd);
    const int zt_shift = zt_record_shift(nd, c->zt_pack16), rec_shift = pow2_shift(1 + 2 * nw + nd);
    int rc;
    if (c->zt_shift != zt_shift || c->zt_ints < ((size_t)c->N << zt_shift)) {
        c->zt_current = false;
        c->td_valid = false;
        if ((rc = grow(c, &c->d_zt, &c->zt_ints, ((size_t)c->N << zt_shift), "word-major records")) != LDA_OK)
            return rc;
        c->zt_shift = zt_shift;
    }
    if ((rc = grow(c, &c->d_rec, &c->rec_ints, (size_t)c->N << rec_shift, "word-pass records")) != LDA_OK)
        return rc;
    const bool have = c->zt_current &&
                      (nd == 0 || (c->td_valid && c->td_sweep == c->sweep_index && c->td_nw == nw &&
                                   c->td_nd == nd));
    SplitArgs A{};
    A.z = c->d_z; A.znew = c->d_znew; A.doff = c->d_doff; A.chunk_doc = c->d_chunk_doc; A.chunk_tok = c->d_chunk_tok;
    A.tokdoc = c->d_tokdoc; A.wpos = c->d_wpos; A.xmap = c->d_xmap; A.gid = c->d_gid; A.woff = c->d_woff;
    A.nkw = c->d_nkw; A.nk = c->d_nk; A.alias = c->d_alias; A.cap = c->d_cap;
    A.zt = c->d_zt; A.zt_pack16 = c->zt_pack16 ? 1 : 0; A.rec = c->d_rec; A.row_items = c->d_row_items; A.pieces = c->d_gather_pieces;
    A.n_chunks = c->n_chunks; A.n_row_items = c->n_row_items; A.n_pieces = c->n_gather_pieces;
    A.K = c->K; A.cap_tokens = c->chunk_tokens; A.max_doc_tokens = c->chunk_tokens;
    A.doc_block = c->sweep_block;
    // (rounded up to 16 bytes: the copy of n_k behind the tile is moved as int4)
    auto tile_ints = [](int32_t tokens, int32_t docs) {
        return (int32_t)((doc_tile_lds_bytes(tokens, docs) / sizeof(int32_t) + 3) / 4 * 4);
    };
    A.tile_lds_ints = tile_ints(c->chunk_tokens, c->chunk_docs);
    if (nw + nd <= 2 && c->n_chunks2 > 0) {  // short chains: the tiling with larger tiles
        A.chunk_doc = c->d_chunk_doc2; A.chunk_tok = c->d_chunk_tok2; A.tokdoc = c->d_tokdoc2;
        A.n_chunks = c->n_chunks2;
        A.cap_tokens = c->chunk_tokens2; A.doc_block = c->sweep_block2;
        A.tile_lds_ints = tile_ints(c->chunk_tokens2, c->chunk_docs2);
    } else if (c->n_chunks2 > 0) {
        // longer chains (default tiles): one token per thread keeps the chain's registers low
        // enough for two 1024-thread workgroups per CU (4 steps: 28.9 instead of 33.4 ms)
        A.doc_block = std::min(1024, (c->chunk_tokens + 63) / 64 * 64);
    }
    A.alpha = c->alpha; A.beta = c->beta; A.alphabar = c->alphabar; A.betabar = c->betabar;
    A.seed_lo = (uint32_t)c->seed; A.seed_hi = (uint32_t)(c->seed >> 32); A.sweep = c->sweep_index;
    A.metaA = c->d_metaA; A.metaB = c->d_metaB; A.ma = c->d_ma; A.hs = c->d_hs;
    A.beta_alias = c->d_beta_alias; A.beta_hdr = c->d_beta_hdr;
    A.sp_off = c->d_sp_off; A.sp_topic = c->d_sp_topic; A.sp_count = c->d_sp_count;
    A.sp_nnz = c->d_sp_nnz; A.mix_items = c->d_mix_items; A.n_mix_items = c->n_mix_items;
    A.long_doc = c->d_long_doc; A.long_slot = c->d_long_slot;
    A.long_keys = c->d_long_keys; A.long_cnts = c->d_long_cnts;
    // from here on the records are being rewritten: valid again only if every launch succeeds
    c->zt_current = false;
    c->td_valid = false;
    if (nw == 1 && nd == 0) rc = launch_chain<1, 0>(c, A, !have);
    else if (nw == 1 && nd == 1) rc = launch_chain<1, 1>(c, A, !have);
    else if (nw == 2 && nd == 1) rc = launch_chain<2, 1>(c, A, !have);
    else if (nw == 2 && nd == 2) rc = launch_chain<2, 2>(c, A, !have);
    else rc = fail(c, LDA_ERR_UNSUPPORTED, "two-pass sweep: chain of %d word and %d doc steps", nw, nd);
    if (rc != LDA_OK) return rc;
    // the doc pass left (new z, doc proposals of the next sweep) in the records
    c->zt_current = true;
    c->td_valid = true;
    c->td_sweep = c->sweep_index + 1u;
    c->td_nw = nw;
    c->td_nd = nd;
    return LDA_OK;
}

}  // namespace lda
