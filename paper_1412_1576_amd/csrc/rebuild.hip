// Count rebuild (LightLDA Sec. 3: the sufficient statistics n_kw and n_k).
//
// n_kw: tokens are laid out word-major, so every word's tokens are one
// contiguous segment.  z is first scattered into that order (one random 4-byte
// write per token, cheaper than a 128-byte line per gathered token); a workgroup
// then histograms a tile of a segment in LDS and writes the dense row.  Words whose segment is longer than one tile are split
// over several workgroups whose partial histograms are merged into a
// pre-zeroed row with integer atomics (order-free, hence exact).
// n_k: an LDS-privatised histogram of z over all tokens (for very large K over a copy of z
// partitioned by topic range, sparse_rows.hip).
#include <algorithm>

#include "common.hpp"
#include "xcd.hpp"

namespace lda {

namespace {

// zw[p] = topic of the p-th token in word-major order: zw[wpos[g]] = z[g].
//
// A word's tokens are ordered by document, so while g advances the writes into
// one word's segment are sequential: a 128-byte line of zw is completed by 32
// writes that are close in g.  Workgroups are dealt round-robin to the 8 XCDs,
// each with its own L2; every XCD therefore takes one contiguous eighth of the
// token range and walks it in order, so that the partially written lines of the
// frequent words stay in that XCD's L2 until they are full instead of being
// written back piecemeal by eight caches.
constexpr int kScatterPerThread = 1;
constexpr int kScatterBlock = 1024;

__global__ __launch_bounds__(1024) void scatter_wm_kernel(const int32_t* __restrict__ z,
                                                         const int32_t* __restrict__ wpos,
                                                         int64_t N, int32_t* __restrict__ zw,
                                                         int32_t sh)
{
    const int64_t per_xcd = (N + kXcds - 1) / kXcds;
    const int xcd = blockIdx.x % kXcds;
    const int64_t j = blockIdx.x / kXcds;
    const int64_t lo = xcd * per_xcd;
    const int64_t hi = (lo + per_xcd < N) ? lo + per_xcd : N;
    const int64_t base = lo + j * (int64_t)(blockDim.x * kScatterPerThread);
#pragma unroll
    for (int u = 0; u < kScatterPerThread; ++u) {
        const int64_t g = base + u * (int64_t)blockDim.x + threadIdx.x;
        if (g < hi)
            zw[(size_t)__builtin_nontemporal_load(&wpos[g]) << sh] = __builtin_nontemporal_load(&z[g]);
    }
}

// blockIdx.x: tile; blockIdx.y: range of `span` topics (one range when the row fits LDS)
constexpr int32_t kTileRun = 32;

__global__ __launch_bounds__(1024) void nkw_tiles_kernel(const RebuildTile* __restrict__ tiles,
                                                         int32_t n_tiles,
                                                         const int32_t* __restrict__ zw,
                                                         int32_t sh, uint32_t zmask, int32_t K,
                                                         int32_t span,
                                                         int32_t* __restrict__ nkw,
                                                         const uint32_t* __restrict__ sp_off,
                                                         int32_t* __restrict__ sp_topic,
                                                         int32_t* __restrict__ sp_count,
                                                         int32_t* __restrict__ sp_nnz,
                                                         const int32_t* __restrict__ xmap)
{
    extern __shared__ int32_t hist[];
    __shared__ uint32_t wcnt[16];
    // runs of consecutive tiles (neighbouring words) share an XCD and with it the lines of
    // the records they read
    const int32_t ti = xcd_runs(kTileRun);
    if (ti >= n_tiles) return;
    const RebuildTile t = tiles[ti];
    const int32_t k0 = (int32_t)blockIdx.y * span;
    const int32_t nk_r = ((k0 + span < K) ? k0 + span : K) - k0;
    const int tid = threadIdx.x, nt = blockDim.x;
    auto count = [&](int32_t rec) {
        const uint32_t r = ((uint32_t)rec & zmask) - (uint32_t)k0;
        if (r < (uint32_t)nk_r) atomicAdd(&hist[r], 1);
    };
    auto at = [&](int32_t p) -> size_t { return xmap ? (size_t)xmap[p] : (size_t)p; };
    int32_t p = t.p0 + tid;
    // The thread's first records are requested before the histogram is cleared: most tiles are
    // short (a word of a thousand tokens), and the clearing and its barrier then hide the two
    // dependent round trips instead of preceding them.  Threads past the end repeat the last.
    int32_t first[2] = {0, 0};
    if (t.p1 > t.p0) {  // (a word without tokens has an empty tile)
        size_t q[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) q[u] = at(p + u * nt < t.p1 ? p + u * nt : t.p1 - 1);
#pragma unroll
        for (int u = 0; u < 2; ++u) first[u] = __builtin_nontemporal_load(&zw[q[u] << sh]);
    }
    for (int32_t k = tid; k < nk_r; k += nt) hist[k] = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (p + u * nt < t.p1) count(first[u]);
    p += 2 * nt;
    for (; p + 3 * nt < t.p1; p += 4 * nt) {  // four loads in flight per thread
        size_t q[4];
        int32_t rec[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) q[u] = at(p + u * nt);
#pragma unroll
        for (int u = 0; u < 4; ++u) rec[u] = __builtin_nontemporal_load(&zw[q[u] << sh]);
#pragma unroll
        for (int u = 0; u < 4; ++u) count(rec[u]);
    }
    for (; p < t.p1; p += nt) count(zw[at(p) << sh]);
    __syncthreads();
    int32_t* __restrict__ row = nkw + (size_t)t.w * (size_t)K + (size_t)k0;
    if (t.multi == 1) {
        for (int32_t k = tid; k < nk_r; k += nt) {
            const int32_t v = hist[k];
            if (v) atomicAdd(&row[k], v);
        }
    } else if (t.multi >= 2) {
        // the whole row is here (one tile, one topic range): write it and the list of its
        // non-zero topics, ascending
        const size_t off = sp_off[t.w];
        const int lane = tid & 63, wv = tid >> 6, nw = nt >> 6;
        // every wave owns a contiguous run of topics: count its non-zeros, then place them
        const int32_t chunk = (((nk_r + nw - 1) / nw) + 63) & ~63;
        const int32_t kb0 = wv * chunk;
        const int32_t kb1 = (kb0 + chunk < nk_r) ? kb0 + chunk : nk_r;
        uint32_t cnt = 0;
        for (int32_t kb = kb0; kb < kb1; kb += 64) {
            const int32_t k = kb + lane;
            const int32_t v = (k < kb1) ? hist[k] : 0;
            if (k < kb1 && t.multi == 2) row[k] = v;  // 3: the row is not kept
            cnt += (uint32_t)__popcll(__ballot(v > 0));
        }
        if (lane == 0) wcnt[wv] = cnt;
        __syncthreads();
        uint32_t base = 0, pos = 0;
        for (int i = 0; i < nw; ++i) {
            if (i < wv) pos += wcnt[i];
            base += wcnt[i];
        }
        for (int32_t kb = kb0; kb < kb1; kb += 64) {
            const int32_t k = kb + lane;
            const int32_t v = (k < kb1) ? hist[k] : 0;
            const uint64_t mask = __ballot(v > 0);
            if (v > 0) {
                const size_t p = off + pos + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
                sp_topic[p] = k;
                sp_count[p] = v;
            }
            pos += (uint32_t)__popcll(mask);
        }
        if (tid == 0) sp_nnz[t.w] = (int32_t)base;
    } else {
        for (int32_t k = tid; k < nk_r; k += nt) row[k] = hist[k];
    }
}

__global__ __launch_bounds__(256) void zero_rows_kernel(const int32_t* __restrict__ words,
                                                        int32_t K, int32_t* __restrict__ nkw)
{
    int32_t* __restrict__ row = nkw + (size_t)words[blockIdx.x] * (size_t)K;
    for (int32_t k = threadIdx.x; k < K; k += blockDim.x) row[k] = 0;
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* __restrict__ p, int64_t n,
                                                       int32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

constexpr int32_t kNkRangeTopics = 36864;  // 144 KB of LDS counters per workgroup

// n_k: each block histograms a contiguous slice of z in LDS, then adds its non-zero bins to
// the (pre-zeroed) global row.  For K beyond one LDS histogram blockIdx.y selects a range of
// `span` topics and every range reads all of z.
__global__ __launch_bounds__(1024) void nk_hist_ranges_kernel(const int32_t* __restrict__ z,
                                                              int64_t N, int32_t K, int32_t span,
                                                              int32_t* __restrict__ nk)
{
    extern __shared__ int32_t hist[];
    const int32_t k0 = (int32_t)blockIdx.y * span;
    const int32_t k1 = (k0 + span < K) ? k0 + span : K;
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int32_t k = tid; k < k1 - k0; k += nt) hist[k] = 0;
    __syncthreads();
    // blocks own runs of whole int4s; two int4 loads per thread are in flight together (one
    // dword per thread and iteration left the kernel bound by load latency)
    const int64_t n4 = N / 4;
    const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
    const int64_t b = (int64_t)blockIdx.x * per;
    const int64_t e = (b + per < n4) ? b + per : n4;
    using v4i = int32_t __attribute__((ext_vector_type(4)));
    const v4i* __restrict__ z4 = reinterpret_cast<const v4i*>(z);
    auto count = [&](int32_t t) {
        if (t >= k0 && t < k1) atomicAdd(&hist[t - k0], 1);
    };
    int64_t i = b + tid;
    for (; i + nt < e; i += 2 * (int64_t)nt) {
        const v4i a = __builtin_nontemporal_load(&z4[i]);
        const v4i c = __builtin_nontemporal_load(&z4[i + nt]);
        count(a.x); count(a.y); count(a.z); count(a.w);
        count(c.x); count(c.y); count(c.z); count(c.w);
    }
    if (i < e) {
        const v4i a = __builtin_nontemporal_load(&z4[i]);
        count(a.x); count(a.y); count(a.z); count(a.w);
    }
    if (blockIdx.x == 0 && tid < (int)(N - 4 * n4)) count(z[4 * n4 + tid]);
    __syncthreads();
    for (int32_t k = tid; k < k1 - k0; k += nt) {
        const int32_t v = hist[k];
        if (v) atomicAdd(&nk[k0 + k], v);
    }
}

// The paper's incremental rule (Sec. 3): a token that moved from topic a to topic b takes one
// from n_kw[w][a], n_k[a] and gives one to n_kw[w][b], n_k[b].  Integer atomics, so the result
// equals the recount whatever the order.  The deltas of n_k are summed per workgroup in LDS
// first (the all-dense store has K <= max_alias_topics()).
__global__ __launch_bounds__(1024) void update_counts_kernel(const int32_t* __restrict__ z,
                                                            const int32_t* __restrict__ zprev,
                                                            const int32_t* __restrict__ word,
                                                            int64_t N, int32_t K,
                                                            int32_t* __restrict__ nkw,
                                                            int32_t* __restrict__ nk)
{
    extern __shared__ int32_t dk[];
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int32_t k = tid; k < K; k += nt) dk[k] = 0;
    __syncthreads();
    const int64_t per = (N + gridDim.x - 1) / gridDim.x;
    const int64_t b = (int64_t)blockIdx.x * per;
    const int64_t e = (b + per < N) ? b + per : N;
    for (int64_t g = b + tid; g < e; g += nt) {
        const int32_t to = __builtin_nontemporal_load(&z[g]);
        const int32_t from = __builtin_nontemporal_load(&zprev[g]);
        if (to == from) continue;
        int32_t* __restrict__ row = nkw + (size_t)word[g] * (size_t)K;
        atomicSub(&row[from], 1);
        atomicAdd(&row[to], 1);
        atomicSub(&dk[from], 1);
        atomicAdd(&dk[to], 1);
    }
    __syncthreads();
    for (int32_t k = tid; k < K; k += nt) {
        const int32_t v = dk[k];
        if (v) atomicAdd(&nk[k], v);
    }
}

}  // namespace

int launch_update_counts(lda_ctx* c)
{
    if (c->K > kNkRangeTopics)
        return fail(c, LDA_ERR_UNSUPPORTED, "lda_update_counts supports K <= %d", kNkRangeTopics);
    int64_t blocks = (c->N + 65535) / 65536;
    blocks = std::max<int64_t>(1, std::min<int64_t>(blocks, 2048));
    const size_t lds = sizeof(int32_t) * (size_t)c->K;
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(update_counts_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(update_counts_kernel, dim3((unsigned)blocks), dim3(1024), lds, c->stream, c->d_z,
                       c->d_znew, c->d_word, c->N, c->K, c->d_nkw, c->d_nk);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

int max_rebuild_topics() { return 36 * 1024; }

namespace {

// word-major copy of z, then the dense rows by LDS histograms over topic ranges
int launch_dense_rows(lda_ctx* c)
{
    const int32_t K = c->K;
    if (!c->zt_current) {  // the sweep's doc pass may have written the new assignment already
        const int rc = launch_scatter_word_major(c, c->d_z, c->d_wpos, c->N);
        if (rc != LDA_OK) return rc;
        c->zt_current = true;
        c->td_valid = false;  // any stored doc proposals belong to another assignment
    }
    if (c->n_tiles == 0) return LDA_OK;
    const int32_t nr = (K + max_rebuild_topics() - 1) / max_rebuild_topics();
    const int32_t span = (((K + nr - 1) / nr) + 63) / 64 * 64;
    const size_t lds = sizeof(int32_t) * (size_t)span;
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(nkw_tiles_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    if (c->n_multi_words > 0) {
        hipLaunchKernelGGL(zero_rows_kernel, dim3(c->n_multi_words), dim3(256), 0, c->stream,
                           c->d_multi_words, K, c->d_nkw);
        LDA_HIP(c, hipGetLastError());
    }
    hipLaunchKernelGGL(nkw_tiles_kernel, dim3(xcd_runs_grid(c->n_tiles, kTileRun), (K + span - 1) / span),
                       dim3(span <= 512 ? 256 : (span <= 16384 ? 512 : 1024)), lds, c->stream, c->d_tiles,
                       c->n_tiles, c->d_zt,
                       c->zt_shift, c->zt_mask, K, span,
                       c->d_nkw, c->d_sp_off, c->d_sp_topic, c->d_sp_count, c->d_sp_nnz, c->d_xmap);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}


// n_k by LDS histograms (K <= 8 * kNkRangeTopics)
int launch_nk_hist(lda_ctx* c)
{
    const int32_t K = c->K;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(64), dim3(256), 0, c->stream, c->d_nk, (int64_t)K, 0);
    LDA_HIP(c, hipGetLastError());
    const int32_t nr = (K + kNkRangeTopics - 1) / kNkRangeTopics;
    const int32_t span = (K + nr - 1) / nr;
    int64_t blocks = (c->N + 65535) / 65536;
    const int64_t most = nr > 1 ? 512 : 2048;
    if (blocks > most) blocks = most;
    if (blocks < 1) blocks = 1;
    const size_t lds = sizeof(int32_t) * (size_t)span;
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(nk_hist_ranges_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(nk_hist_ranges_kernel, dim3((unsigned)blocks, (unsigned)nr), dim3(1024), lds,
                       c->stream, c->streamed ? c->d_zt : c->d_z, c->N, K, span, c->d_nk);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace

int launch_scatter_word_major(lda_ctx* c, const int32_t* z, const int32_t* wpos, int64_t n)
{
    if (n <= 0) return LDA_OK;
    const int64_t per_xcd = (n + kXcds - 1) / kXcds;
    const int64_t per_block = kScatterBlock * kScatterPerThread;
    const int64_t blocks = ((per_xcd + per_block - 1) / per_block) * kXcds;
    hipLaunchKernelGGL(scatter_wm_kernel, dim3((unsigned)blocks), dim3(kScatterBlock), 0, c->stream, z, wpos,
                       n, c->d_zt, c->zt_shift);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

int launch_rebuild(lda_ctx* c)
{
    const int32_t K = c->K;
    if (K > max_rebuild_topics())
        return fail(c, LDA_ERR_UNSUPPORTED, "count rebuild supports K <= %d", max_rebuild_topics());
    int rc = launch_dense_rows(c);
    if (rc != LDA_OK) return rc;
    return launch_nk_hist(c);
}

// Hybrid store (LightLDA Sec. 5): dense rows for the head words as above; for every other word
// a list of its non-zero (topic, count) pairs in ascending topic order plus an open-addressing
// hash row (load <= 1/2) for random lookups, both made word by word from the word's own
// segment of the word-major order (sparse_rows.hip).
int launch_rebuild_hybrid(lda_ctx* c)
{
    const int32_t K = c->K;
    // ---- word-major copy of z and the dense head rows ----
    {
        const int rc = launch_dense_rows(c);
        if (rc != LDA_OK) return rc;
    }
    // ---- sparse rows: lists, lengths and hash rows (sparse_rows.hip) ----
    if (c->V > c->H) {
        const int rc = launch_sparse_rows(c);
        if (rc != LDA_OK) return rc;
    }
    // ---- n_k ----
    if (K > 8 * kNkRangeTopics) return launch_nk_by_ranges(c);
    return launch_nk_hist(c);
}

}  // namespace lda
