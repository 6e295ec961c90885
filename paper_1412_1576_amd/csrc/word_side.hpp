// The word side of a token under the hybrid store (LightLDA Sec. 4.2 and 5): where the
// word's proposal table and n_kw row live, one n_kw lookup, and one word-proposal draw
// from the dense table or from the sparsified mixture.  Shared by the fused sweep and
// the word pass of the two-pass sweep.
//
// STORE: 1 = every word has a dense n_kw row, some draw from the mixture;
//        2 = sparse (hash) rows as well.
// Args is a kernel argument block with the members metaA, metaB, alias, ma, hs, nkw, K.
#pragma once

#include "common.hpp"

namespace lda {

struct WordSide {
    const uint4* tab;  // the word's own table: K dense bins, or its mixture bins
    const void* row;   // dense n_kw row (int32[K]), or hash row (uint2[2^lg]) in store 2
    uint32_t n, C;     // bins and capacity of the own table
    uint32_t kind;     // bit 0: dense n_kw row, bit 1: dense proposal table, bit 2: the row is
                       // not kept (kKindListOnly): lookups search the word's mixture table
    uint32_t lg;
    uint64_t QS;       // integer mass of the sparse term (mixture form)
};

// The word's 32-byte record as loaded, and what it says, in two steps: a caller that
// serves several tokens at once issues all their loads before it looks at any of them.
struct WordMeta {
    uint4 a, b;
};

template <class Args>
__device__ __forceinline__ WordMeta load_word_meta(const Args& A, int32_t w)
{
    return WordMeta{A.metaA[2 * (size_t)w], A.metaB[2 * (size_t)w]};
}

template <int STORE, class Args>
__device__ __forceinline__ WordSide word_from_meta(const Args& A, int32_t w, const WordMeta& m)
{
    const uint4 a = m.a, b = m.b;
    WordSide v;
    v.kind = b.w;
    v.lg = b.z;
    v.C = a.y;
    v.QS = ((uint64_t)a.w << 32) | a.z;
    const size_t wk = (size_t)w * (size_t)A.K;
    const bool dense_tab = (b.w & 2u) != 0;
    v.n = dense_tab ? (uint32_t)A.K : a.x;
    v.tab = dense_tab ? A.alias + wk : A.ma + b.x;
    if (STORE == 2 && !(b.w & 1u))
        v.row = A.hs + b.y;
    else
        v.row = A.nkw + wk;
    return v;
}

template <int STORE, class Args>
__device__ __forceinline__ WordSide load_word(const Args& A, int32_t w)
{
    return word_from_meta<STORE>(A, w, load_word_meta(A, w));
}

// n_kw[w][t] of a list-only word: bin i of its mixture table carries its i-th non-zero topic
// (ascending) and that topic's count
__device__ __forceinline__ int32_t nkw_from_table(const WordSide& v, int32_t t)
{
    uint32_t lo = 0, hi = v.n;  // first bin whose topic is >= t
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        int32_t topic, count;
        unpack_mix_bin(v.tab[mid], true, topic, count);
        if (topic < t) lo = mid + 1; else hi = mid;
    }
    if (lo == v.n) return 0;
    int32_t topic, count;
    unpack_mix_bin(v.tab[lo], true, topic, count);
    return topic == t ? count : 0;
}

// n_kw[w][t]: dense row, or the word's hash row (Sec. 5)
template <int STORE>
__device__ __forceinline__ int32_t nkw_lookup(const WordSide& v, int32_t t)
{
    if (v.kind & kKindListOnly) return nkw_from_table(v, t);
    if (STORE != 2 || (v.kind & 1u)) return static_cast<const int32_t*>(v.row)[t];
    const uint2* __restrict__ row = static_cast<const uint2*>(v.row);
    const uint32_t mask = (1u << v.lg) - 1u;
    uint32_t s = row_hash_slot(t, v.lg);
    for (uint32_t i = 0; i <= mask; ++i) {
        const uint2 e = row[s];
        if (e.x == (uint32_t)t) return (int32_t)e.y;
        if (e.x == 0xFFFFFFFFu) return 0;
        s = (s + 1) & mask;
    }
    return 0;
}

// The same lookup in two halves, so that a caller can keep several in flight: the first
// half issues the load of the dense entry or of the first hash slot, the second half
// resolves it (and probes on in the rare case the first slot holds another topic).
struct NkwProbe {
    uint2 e;
    uint32_t slot;
};

template <int STORE>
__device__ __forceinline__ NkwProbe nkw_probe_begin(const WordSide& v, int32_t t)
{
    NkwProbe p;
    if (v.kind & kKindListOnly) {  // resolved here; nkw_probe_finish returns it
        p.slot = 0;
        p.e = make_uint2((uint32_t)nkw_from_table(v, t), 0u);
    } else if (STORE != 2 || (v.kind & 1u)) {
        p.slot = 0;
        p.e = make_uint2((uint32_t) static_cast<const int32_t*>(v.row)[t], 0u);
    } else {
        p.slot = row_hash_slot(t, v.lg);
        p.e = static_cast<const uint2*>(v.row)[p.slot];
    }
    return p;
}

template <int STORE>
__device__ __forceinline__ int32_t nkw_probe_finish(const WordSide& v, int32_t t, const NkwProbe& p)
{
    if (STORE != 2 || (v.kind & (1u | kKindListOnly))) return (int32_t)p.e.x;
    if (p.e.x == (uint32_t)t) return (int32_t)p.e.y;
    if (p.e.x == 0xFFFFFFFFu) return 0;
    const uint2* __restrict__ row = static_cast<const uint2*>(v.row);
    const uint32_t mask = (1u << v.lg) - 1u;
    uint32_t s = (p.slot + 1) & mask;
    for (uint32_t i = 1; i <= mask; ++i) {
        const uint2 e = row[s];
        if (e.x == (uint32_t)t) return (int32_t)e.y;
        if (e.x == 0xFFFFFFFFu) return 0;
        s = (s + 1) & mask;
    }
    return 0;
}

// The lookup as two dword loads from one computed address, whatever the kind of row (not for
// list-only words): no branch between the loads of a round, so they are issued back to back.
// Dense row: both loads read n_kw[t]; hash row: the slot's topic and count.
struct NkwFetch {
    uint32_t key, val, slot;
};

template <int STORE>
__device__ __forceinline__ NkwFetch nkw_fetch_begin(const WordSide& v, int32_t t)
{
    const bool dense = STORE != 2 || (v.kind & 1u);
    NkwFetch f;
    f.slot = dense ? 0u : row_hash_slot(t, v.lg);
    const uint32_t* __restrict__ base = static_cast<const uint32_t*>(v.row);
    const size_t i = dense ? (size_t)t : 2 * (size_t)f.slot;
    f.key = base[i];
    f.val = base[dense ? i : i + 1];
    return f;
}

template <int STORE>
__device__ __forceinline__ int32_t nkw_fetch_finish(const WordSide& v, int32_t t, const NkwFetch& f)
{
    if (STORE != 2 || (v.kind & 1u)) return (int32_t)f.key;
    if (f.key == (uint32_t)t) return (int32_t)f.val;
    if (f.key == 0xFFFFFFFFu) return 0;
    const uint2* __restrict__ row = static_cast<const uint2*>(v.row);
    const uint32_t mask = (1u << v.lg) - 1u;
    uint32_t s = (f.slot + 1) & mask;
    for (uint32_t i = 1; i <= mask; ++i) {
        const uint2 e = row[s];
        if (e.x == (uint32_t)t) return (int32_t)e.y;
        if (e.x == 0xFFFFFFFFu) return 0;
        s = (s + 1) & mask;
    }
    return 0;
}

// The shared table of the mixture's beta term: (split, alias) bins read as aligned pairs.
struct BetaTable {
    const uint4* pairs;
    uint64_t QB;
    uint32_t C;
};

template <class Args>
__device__ __forceinline__ BetaTable load_beta_table(const Args& A)
{
    return BetaTable{reinterpret_cast<const uint4*>(A.beta_alias), A.beta_hdr[0],
                     (uint32_t)A.beta_hdr[1]};
}

// A word-proposal draw in two halves, so that a caller can keep several gathers in
// flight.  The three forms of a draw (dense table, sparse term, shared beta term)
// differ only in the address of the one 16-byte record they gather and in how it is
// decoded, so every lane issues the same load.
struct WordDraw {
    uint32_t bin, rr;
    uint32_t form;  // 0 dense table, 1 sparse term, 2 beta term
};

// x0, x1: bin and height; x3 picks the mixture's term by its integer mass
__device__ __forceinline__ const uint4* word_draw_address(const WordSide& wv, const BetaTable& bt,
                                                          uint32_t K, uint32_t x0, uint32_t x1,
                                                          uint32_t x3, WordDraw& d)
{
#pragma clang fp contract(off)
    const double u3 = unit_open(x3);
    const bool sparse_term = u3 * (double)(wv.QS + bt.QB) < (double)wv.QS;
    d.form = (wv.kind & 2u) ? 0u : (sparse_term ? 1u : 2u);
    const bool beta_term = d.form == 2u;
    d.bin = mulhi32(x0, beta_term ? K : wv.n);
    d.rr = mulhi32(x1, beta_term ? bt.C : wv.C);
    return beta_term ? bt.pairs + (d.bin >> 1) : wv.tab + d.bin;
}

// The proposed topic; n_kw of it unless the draw came from the beta term (returns
// false: the caller looks it up).
__device__ __forceinline__ bool word_draw_decode(const WordDraw& d, const uint4& e, int32_t& t,
                                                 int32_t& nwt)
{
    const bool odd = (d.form == 2u) && (d.bin & 1u);  // beta table: two 8-byte bins per record
    const bool keep = d.rr < (odd ? e.z : e.x);
    int32_t tm, nm;
    unpack_mix_bin(e, keep, tm, nm);
    const int32_t td = keep ? (int32_t)d.bin : (int32_t)(odd ? e.w : e.y);
    t = (d.form == 1u) ? tm : td;
    nwt = (d.form == 1u) ? nm : (keep ? (int32_t)e.z : (int32_t)e.w);
    return d.form != 2u;
}

}  // namespace lda
