// Word-proposal tables (LightLDA Sec. 4.2, Eq. 6, Fig. 2).
//
// Dense form: one table per word over all K topics, weights (n_kw + beta)/(n_k + betabar).
// Mixture form (the paper's sparsified table): per word a table over its non-zero
// topics only, weights n_kw/(n_k + betabar), plus one table shared by all words over
// beta/(n_k + betabar); the sweep picks the term by the two integer masses QS_w and QB.
// Every table is built by one workgroup with the generic builder of alias_build.hpp;
// tables too large for LDS use a global workspace.
#include <algorithm>

#include "alias_build.hpp"

namespace lda {

namespace {

__device__ __forceinline__ uint64_t quantise40(double a)
{
    return (uint64_t)floor(a * 1099511627776.0);
}

// dense form: entry k is topic k
struct DenseSrc {
    const int32_t* __restrict__ row;
    const int32_t* __restrict__ nk;
    double beta, betabar;
    __device__ __forceinline__ uint64_t q0(int32_t k) const
    {
#pragma clang fp contract(off)
        return quantise40(((double)row[k] + beta) / ((double)nk[k] + betabar));
    }
};

// A dense bin also carries the word-topic counts of its two outcomes, so the sweep's
// accept test needs no second gather.
struct DenseSink {
    uint4* __restrict__ out;
    const int32_t* __restrict__ row;
    struct Loaded { int32_t own, other; };
    __device__ __forceinline__ Loaded load(int32_t k, uint32_t al) const
    {
        return Loaded{row[k], row[al]};
    }
    __device__ __forceinline__ void store(int32_t k, uint32_t split, uint32_t al,
                                          const Loaded& v) const
    {
        out[k] = make_uint4(split, al, (uint32_t)v.own, (uint32_t)v.other);
    }
};

// sparse term of the mixture: entry i is the word's i-th non-zero topic (ascending)
struct SparseSrc {
    const int32_t* __restrict__ topic;
    const int32_t* __restrict__ count;
    const int32_t* __restrict__ nk;
    double betabar;
    __device__ __forceinline__ uint64_t q0(int32_t i) const
    {
#pragma clang fp contract(off)
        return quantise40((double)count[i] / ((double)nk[topic[i]] + betabar));
    }
};

// mixture bin: (split, own topic, alias topic, n_kw[own]) and (n_kw[alias], -, -, -)
struct SparseSink {
    uint4* __restrict__ out;
    const int32_t* __restrict__ topic;
    const int32_t* __restrict__ count;
    struct Loaded { int32_t t_own, t_other, n_own, n_other; };
    __device__ __forceinline__ Loaded load(int32_t i, uint32_t al) const
    {
        return Loaded{topic[i], topic[al], count[i], count[al]};
    }
    __device__ __forceinline__ void store(int32_t i, uint32_t split, uint32_t,
                                          const Loaded& v) const
    {
        out[i] = pack_mix_bin(split, v.t_own, v.t_other, v.n_own, v.n_other);
    }
};

// shared beta term of the mixture: entry k is topic k
struct BetaSrc {
    const int32_t* __restrict__ nk;
    double beta, betabar;
    __device__ __forceinline__ uint64_t q0(int32_t k) const
    {
#pragma clang fp contract(off)
        return quantise40(beta / ((double)nk[k] + betabar));
    }
};

struct BetaSink {
    uint2* __restrict__ out;
    struct Loaded {};
    __device__ __forceinline__ Loaded load(int32_t, uint32_t) const { return Loaded{}; }
    __device__ __forceinline__ void store(int32_t k, uint32_t split, uint32_t al,
                                          const Loaded&) const
    {
        out[k] = make_uint2(split, al);
    }
};

struct DenseArgs {
    const int32_t* words;  // NULL: word = block index
    int32_t n_words;
    const int32_t* nkw;
    const int32_t* nk;
    int32_t K;
    double beta, betabar;
    uint4* alias;
    uint32_t* cap;   // nullable
    uint4* metaA;    // nullable; word w at [2w]
    int32_t use_cache;
    unsigned char* ws;  // GLOBAL: list memory, ws_stride bytes per workgroup
    size_t ws_stride;
};

template <bool GLOBAL>
__device__ __forceinline__ void dense_table(const DenseArgs& a, int32_t w, unsigned char* lists)
{
    const int32_t K = a.K;
    const int32_t* row = a.nkw + (size_t)w * (size_t)K;
    DenseSrc src{row, a.nk, a.beta, a.betabar};
    DenseSink sink{a.alias + (size_t)w * (size_t)K, row};
    uint64_t Q0;
    uint32_t C;
    build_alias_table<GLOBAL>(K, src, sink, lists, a.use_cache != 0, Q0, C);
    if (threadIdx.x == 0) {
        if (a.cap) a.cap[w] = C;
        if (a.metaA) a.metaA[2 * (size_t)w] = make_uint4((uint32_t)K, C, 0u, 0u);
    }
}

// one workgroup per word, lists in LDS
__global__ __launch_bounds__(1024) void alias_dense_lds_kernel(DenseArgs a)
{
    extern __shared__ unsigned char smem_raw[];
    const int32_t w = a.words ? a.words[blockIdx.x] : (int32_t)blockIdx.x;
    dense_table<false>(a, w, smem_raw);
}

// persistent workgroups, lists in a global workspace (K too large for LDS)
__global__ __launch_bounds__(1024) void alias_dense_big_kernel(DenseArgs a)
{
    unsigned char* lists = a.ws + (size_t)blockIdx.x * a.ws_stride;
    for (int32_t i = blockIdx.x; i < a.n_words; i += gridDim.x) {
        const int32_t w = a.words ? a.words[i] : i;
        dense_table<true>(a, w, lists);
        ListMem<true>::barrier();
    }
}

struct MixArgs {
    const int32_t* words;
    int32_t n_words;
    const uint32_t* sp_off;
    const int32_t* sp_topic;
    const int32_t* sp_count;
    const int32_t* sp_nnz;
    const int32_t* nk;
    double betabar;
    uint4* ma;
    uint4* metaA;
    int32_t use_cache;
    unsigned char* ws;
    size_t ws_stride;
    int32_t* next;  // big tables: work counter, zero at launch
};

template <bool GLOBAL>
__device__ __forceinline__ void mix_table(const MixArgs& a, int32_t w, unsigned char* lists)
{
    const int32_t n = a.sp_nnz[w];
    if (n <= 0) {  // a word without tokens is never drawn from
        if (threadIdx.x == 0) a.metaA[2 * (size_t)w] = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
    const size_t off = a.sp_off[w];
    SparseSrc src{a.sp_topic + off, a.sp_count + off, a.nk, a.betabar};
    SparseSink sink{a.ma + off, a.sp_topic + off, a.sp_count + off};
    uint64_t QS;
    uint32_t C;
    build_alias_table<GLOBAL>(n, src, sink, lists, a.use_cache != 0, QS, C);
    if (threadIdx.x == 0)
        a.metaA[2 * (size_t)w] = make_uint4((uint32_t)n, C, (uint32_t)QS, (uint32_t)(QS >> 32));
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void alias_mix_lds_kernel(MixArgs a)
{
    extern __shared__ unsigned char smem_raw[];
    mix_table<false>(a, a.words[blockIdx.x], smem_raw);
}

__global__ __launch_bounds__(1024) void alias_mix_big_kernel(MixArgs a)
{
    // The tables differ in size by orders of magnitude and are listed largest first: a
    // workgroup takes its first table by its index and every further one from a counter.
    __shared__ int32_t s_next;
    unsigned char* lists = a.ws + (size_t)blockIdx.x * a.ws_stride;
    int32_t i = blockIdx.x;
    while (i < a.n_words) {
        mix_table<true>(a, a.words[i], lists);
        ListMem<true>::barrier();
        if (threadIdx.x == 0) s_next = (int32_t)gridDim.x + atomicAdd(a.next, 1);
        __syncthreads();
        i = s_next;
        __syncthreads();
    }
}

__global__ void set_i32_kernel(int32_t* p, int32_t v) { *p = v; }

template <bool GLOBAL>
__global__ __launch_bounds__(1024) void alias_beta_kernel(const int32_t* nk, int32_t K, double beta,
                                                          double betabar, uint2* out,
                                                          uint64_t* hdr, int32_t use_cache,
                                                          unsigned char* ws)
{
    extern __shared__ unsigned char smem_raw[];
    unsigned char* lists = GLOBAL ? ws : smem_raw;
    BetaSrc src{nk, beta, betabar};
    BetaSink sink{out};
    uint64_t QB;
    uint32_t C;
    build_alias_table<GLOBAL>(K, src, sink, lists, use_cache != 0, QB, C);
    if (threadIdx.x == 0) {
        hdr[0] = QB;
        hdr[1] = C;
    }
}

// Non-zero topics of a dense row, ascending, into the word's list (a mixture word
// that keeps a dense row).  One workgroup per word; every wave owns a contiguous run of
// topics, counts its non-zeros, and after one barrier places them (the second read of the
// run comes from L2).  Four loads per lane are in flight.
__global__ __launch_bounds__(1024) void compact_rows_kernel(const int32_t* __restrict__ words,
                                                            const int32_t* __restrict__ nkw,
                                                            int32_t K,
                                                            const uint32_t* __restrict__ sp_off,
                                                            int32_t* __restrict__ sp_topic,
                                                            int32_t* __restrict__ sp_count,
                                                            int32_t* __restrict__ sp_nnz)
{
    __shared__ uint32_t wcnt[16];
    const int32_t w = words[blockIdx.x];
    const int32_t* __restrict__ row = nkw + (size_t)w * (size_t)K;
    const size_t off = sp_off[w];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int32_t chunk = (((K + nw - 1) / nw) + kWave - 1) & ~(kWave - 1);
    const int32_t kb0 = (wv * chunk < K) ? wv * chunk : K;
    const int32_t kb1 = (kb0 + chunk < K) ? kb0 + chunk : K;
    uint32_t cnt = 0;
    int32_t kb = kb0;
    for (; kb + 4 * kWave <= kb1; kb += 4 * kWave) {
        int32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = row[kb + u * kWave + lane];
#pragma unroll
        for (int u = 0; u < 4; ++u) cnt += (uint32_t)__popcll(__ballot(v[u] > 0));
    }
    for (; kb < kb1; kb += kWave) {
        const int32_t k = kb + lane;
        const int32_t v = (k < kb1) ? row[k] : 0;
        cnt += (uint32_t)__popcll(__ballot(v > 0));
    }
    if (lane == 0) wcnt[wv] = cnt;
    __syncthreads();
    uint32_t pos = 0, total = 0;
    for (int i = 0; i < nw; ++i) {
        if (i < wv) pos += wcnt[i];
        total += wcnt[i];
    }
    auto place = [&](int32_t k, int32_t v) {
        const uint64_t mask = __ballot(v > 0);
        if (v > 0) {
            const size_t p = off + pos + rank_below(mask);
            sp_topic[p] = k;
            sp_count[p] = v;
        }
        pos += (uint32_t)__popcll(mask);
    };
    kb = kb0;
    for (; kb + 4 * kWave <= kb1; kb += 4 * kWave) {
        int32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = row[kb + u * kWave + lane];
#pragma unroll
        for (int u = 0; u < 4; ++u) place(kb + u * kWave + lane, v[u]);
    }
    for (; kb < kb1; kb += kWave) {
        const int32_t k = kb + lane;
        place(k, (k < kb1) ? row[k] : 0);
    }
    if (threadIdx.x == 0) sp_nnz[w] = (int32_t)total;
}

template <class Kern>
int set_lds(lda_ctx* c, Kern kern, size_t lds)
{
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    return LDA_OK;
}

constexpr size_t kLdsLimit = 160 * 1024 - 1024;  // 160 KiB per workgroup, room for statics

// LDS bytes and cache flag for a table of n entries
void lds_plan(size_t n, size_t& bytes, int32_t& use_cache)
{
    use_cache = alias_list_bytes(n, true) <= kLdsLimit ? 1 : 0;
    bytes = alias_list_bytes(n, use_cache != 0);
}

}  // namespace

int max_lds_table_entries() { return 12 * 1024; }
int max_alias_topics() { return 12 * 1024; }

// all-dense mode: every word, lists in LDS
int launch_alias_build(lda_ctx* c)
{
    const int32_t K = c->K;
    if (K > max_lds_table_entries())
        return fail(c, LDA_ERR_UNSUPPORTED, "dense alias build in LDS supports K <= %d",
                    max_lds_table_entries());
    int nw = (K + kWave - 1) / kWave;
    if (nw > kMaxWaves) nw = kMaxWaves;
    size_t lds;
    int32_t use_cache;
    lds_plan((size_t)K, lds, use_cache);
    int rc = set_lds(c, alias_dense_lds_kernel, lds);
    if (rc != LDA_OK) return rc;
    DenseArgs a{};
    a.words = nullptr; a.n_words = c->V; a.nkw = c->d_nkw; a.nk = c->d_nk; a.K = K;
    a.beta = c->beta; a.betabar = c->betabar; a.alias = c->d_alias; a.cap = c->d_cap;
    a.metaA = nullptr; a.use_cache = use_cache;
    hipLaunchKernelGGL(alias_dense_lds_kernel, dim3(c->V), dim3(nw * kWave), lds, c->stream, a);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

namespace {

// Mixture tables of the words in `words` whose list capacity is at most cap_entries
// (cap_entries = 0: any size, built in the global workspace).
int launch_alias_mix_class(lda_ctx* c, hipStream_t stream, const int32_t* words, int32_t n_words,
                           int32_t cap_entries)
{
    if (n_words <= 0) return LDA_OK;
    MixArgs a{};
    a.words = words; a.n_words = n_words; a.sp_off = c->d_sp_off; a.sp_topic = c->d_sp_topic;
    a.sp_count = c->d_sp_count; a.sp_nnz = c->d_sp_nnz; a.nk = c->d_nk; a.betabar = c->betabar;
    a.ma = c->d_ma; a.metaA = c->d_metaA;
    if (cap_entries > 0) {
        size_t lds;
        lds_plan((size_t)cap_entries, lds, a.use_cache);
        // Tables of a few thousand entries are few per CU (their lists fill the LDS), so each
        // gets more waves: the time of one table, not the number in flight, bounds such a class.
        // (c3: 2.95 -> 2.57 ms for all tables, c4: 10.9 -> 10.1)
        if (cap_entries >= 2048) {
            int rc = set_lds(c, alias_mix_lds_kernel<1024>, lds);
            if (rc != LDA_OK) return rc;
            int threads = cap_entries / 4;
            threads = threads < 256 ? 256 : (threads > 1024 ? 1024 : threads / kWave * kWave);
            hipLaunchKernelGGL(alias_mix_lds_kernel<1024>, dim3(n_words), dim3(threads), lds, stream, a);
        } else {
            int rc = set_lds(c, alias_mix_lds_kernel<256>, lds);
            if (rc != LDA_OK) return rc;
            // small tables: half a wave's worth of entries per lane-round keeps more tables in
            // flight (two waves per table up to 1024 entries; c2 0.62 -> 0.51 ms, c4 10.0 -> 9.6)
            int threads = ((cap_entries + kWave - 1) / kWave) * kWave;
            threads = std::max(64, std::min(threads, 256) / 2 / kWave * kWave);
            hipLaunchKernelGGL(alias_mix_lds_kernel<256>, dim3(n_words), dim3(threads), lds, stream, a);
        }
    } else {
        a.use_cache = 1; a.ws = c->d_big_ws; a.ws_stride = c->big_ws_stride;
        a.next = c->d_flag + 1;
        hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, stream, a.next, 0);
        LDA_HIP(c, hipGetLastError());
        const int grid = n_words < c->n_big_wg ? n_words : c->n_big_wg;
        hipLaunchKernelGGL(alias_mix_big_kernel, dim3(grid), dim3(1024), 0, stream, a);
    }
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

// the shared beta table and the mixture tables that are built in LDS, in this order on `stream`
int launch_small_mixture_tables(lda_ctx* c, hipStream_t stream)
{
    const int32_t K = c->K;
    const int lds_max = max_lds_table_entries();
    int rc;
    if (K <= lds_max) {
        size_t lds;
        int32_t use_cache;
        lds_plan((size_t)K, lds, use_cache);
        rc = set_lds(c, alias_beta_kernel<false>, lds);
        if (rc != LDA_OK) return rc;
        int nw = (K + kWave - 1) / kWave;
        if (nw > kMaxWaves) nw = kMaxWaves;
        hipLaunchKernelGGL(alias_beta_kernel<false>, dim3(1), dim3(nw * kWave), lds, stream, c->d_nk,
                           K, c->beta, c->betabar, c->d_beta_alias, c->d_beta_hdr, use_cache, nullptr);
    } else {  // one workgroup, with a slot of list memory of its own
        hipLaunchKernelGGL(alias_beta_kernel<true>, dim3(1), dim3(1024), 0, stream, c->d_nk, K,
                           c->beta, c->betabar, c->d_beta_alias, c->d_beta_hdr, 1,
                           c->d_big_ws + c->big_ws_stride * (size_t)c->n_big_wg);
    }
    LDA_HIP(c, hipGetLastError());
    for (int cl = 0; cl < kMixClasses; ++cl) {
        const int32_t cap = kMixClassCap[cl];
        if (cap < 0) continue;  // the class of the global workspace
        rc = launch_alias_mix_class(c, stream, c->d_mix_class[cl], c->n_mix_class[cl],
                                    cap ? cap : lds_max);
        if (rc != LDA_OK) return rc;
    }
    return LDA_OK;
}

}  // namespace

// Hybrid mode: the shared beta table, dense tables of the head words, mixture tables of the
// rest.  Two chains of kernels run side by side: on a second stream of the library's own the
// beta table (one workgroup, milliseconds when K is large) and the many small tables built in
// LDS; on the caller's stream the dense tables and the tables built in the global workspace.
// The second stream is forked from the caller's by an event and joined at the end.
int launch_alias_build_hybrid(lda_ctx* c)
{
    const int32_t K = c->K;
    const int lds_max = max_lds_table_entries();
    int rc;
    if (c->n_compact > 0) {  // lists the mixture tables below are built from
        hipLaunchKernelGGL(compact_rows_kernel, dim3(c->n_compact), dim3(K <= 4096 ? 256 : 1024), 0,
                           c->stream, c->d_compact_words, c->d_nkw, K, c->d_sp_off, c->d_sp_topic,
                           c->d_sp_count, c->d_sp_nnz);
        LDA_HIP(c, hipGetLastError());
    }
    if (c->n_mix > 0) {
        if ((rc = fork_side_stream(c)) != LDA_OK) return rc;
        rc = launch_small_mixture_tables(c, c->side_stream);
        const int rd = side_stream_done(c);
        if (rc != LDA_OK || rd != LDA_OK) {
            (void)join_side_stream(c);
            return rc != LDA_OK ? rc : rd;
        }
    }
    if (c->n_dense_alias > 0) {
        DenseArgs a{};
        a.words = c->d_dense_alias_words; a.n_words = c->n_dense_alias; a.nkw = c->d_nkw;
        a.nk = c->d_nk; a.K = K; a.beta = c->beta; a.betabar = c->betabar; a.alias = c->d_alias;
        a.cap = c->d_cap; a.metaA = c->d_metaA;
        if (K <= lds_max) {
            size_t lds;
            lds_plan((size_t)K, lds, a.use_cache);
            rc = set_lds(c, alias_dense_lds_kernel, lds);
            if (rc == LDA_OK) {
                int nw = (K + kWave - 1) / kWave;
                if (nw > kMaxWaves) nw = kMaxWaves;
                hipLaunchKernelGGL(alias_dense_lds_kernel, dim3(c->n_dense_alias), dim3(nw * kWave),
                                   lds, c->stream, a);
            }
        } else {
            a.use_cache = 1; a.ws = c->d_big_ws; a.ws_stride = c->big_ws_stride;
            const int grid = c->n_dense_alias < c->n_big_wg ? c->n_dense_alias : c->n_big_wg;
            hipLaunchKernelGGL(alias_dense_big_kernel, dim3(grid), dim3(1024), 0, c->stream, a);
            rc = LDA_OK;
        }
        if (rc == LDA_OK && hipGetLastError() != hipSuccess)
            rc = fail(c, LDA_ERR_HIP, "launch of the dense table build failed");
    } else {
        rc = LDA_OK;
    }
    if (rc == LDA_OK)
        rc = launch_alias_mix_class(c, c->stream, c->d_mix_class[kMixClasses - 1],
                                    c->n_mix_class[kMixClasses - 1], 0);
    const int rj = join_side_stream(c);
    return rc != LDA_OK ? rc : rj;
}

}  // namespace lda
