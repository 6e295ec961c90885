// Count rebuild of the hybrid store's sparse rows (LightLDA Sec. 5: words of the long tail keep
// their non-zero (topic, count) pairs instead of a dense row) and of n_k when K exceeds what a
// few LDS histograms cover.  Everything is a segmented histogram: the tokens of a word are one
// contiguous segment of the word-major order, so no global sort is needed.
//
//   short words (at most kSortMaxTokens tokens): one workgroup per word sorts the word's topics
//     in LDS (bitonic network), turns runs of equal topics into (topic, count) pairs in
//     ascending order -- the word's list -- and inserts every pair into the word's hash row.
//     Work is proportional to the word's tokens, not to K.
//   long words: their tokens are first partitioned by topic range (kRangeTopics topics per
//     range, order inside a range irrelevant: only counts matter) with a counting pass, a scan
//     and a scatter pass; a workgroup per (word, range) then histograms its sub-segment in LDS,
//     once to count the range's non-zero topics and, after a scan of those counts, once more
//     to write them at their place in the list and into the hash row.
//   n_k for very large K: z partitioned by topic range the same way, then LDS histograms of
//     the ranges added to n_k.
#include <algorithm>

#include "common.hpp"

namespace lda {

namespace {

constexpr int kRangeShift = 13;
constexpr int32_t kRangeTopics = 1 << kRangeShift;  // topics per range: 32 KB of LDS counters
constexpr int32_t kPartTile = 16384;                // tokens per workgroup of the partition passes
constexpr int32_t kNkChunk = 1 << 18;               // tokens per workgroup of the n_k range histograms
// words sorted in LDS, by tokens: up to 256 by one wave, up to 2048 by 256 threads, up to 4096
// by 1024 threads; longer words are partitioned by topic range
constexpr int32_t kSortTokensA = 256, kSortTokensB = 2048, kSortMaxTokens = 4096;

// Where the topic of position p is read from: word-major records (z in the low bits of the
// record's first int, positions mapped through xmap when the records are bucketed) or plain z.
struct TopicSource {
    const int32_t* src;
    const int32_t* xmap;
    int32_t sh;
    uint32_t mask;
    __device__ __forceinline__ int32_t at(int32_t p) const
    {
        const size_t q = xmap ? (size_t)xmap[p] : (size_t)p;
        return (int32_t)((uint32_t)src[q << sh] & mask);
    }
};

// ---- short words: LDS sort + run lengths -------------------------------------------------

// One 64-bit compare-and-swap per probe claims an empty slot (topic 0xFFFFFFFF, count 0) and
// fills it: a single transaction on the row's line instead of a claim plus a store.
__device__ __forceinline__ void hash_row_insert(uint2* __restrict__ row, uint32_t cap, int32_t topic,
                                                uint32_t count)
{
    const uint32_t lg = 31u - (uint32_t)__clz((int)cap);  // cap is a power of two
    uint32_t slot = row_hash_slot(topic, lg);
    const unsigned long long empty = 0xFFFFFFFFull;       // .x in the low half
    const unsigned long long entry = (unsigned long long)(uint32_t)topic | ((unsigned long long)count << 32);
    for (uint32_t i = 0; i < cap; ++i) {
        if (atomicCAS(reinterpret_cast<unsigned long long*>(&row[slot]), empty, entry) == empty) return;
        slot = (slot + 1) & (cap - 1);
    }
}

// Orders the LDS accesses of one wave (compiler and hardware) without a workgroup barrier and
// without waiting for the wave's global loads.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// BLOCK threads per word, WORDS words per workgroup (WORDS > 1 only with BLOCK = 64: every
// wave then works on a word of its own and never meets a workgroup barrier); a word has at
// most BLOCK * EPT tokens.  The hash rows of words with more than 2048 tokens have been
// cleared (those of shorter words are written whole).
//
// Bitonic network over n2 = 2^m >= n keys in LDS.  Wave v owns the pairs [v P, (v + 1) P) of
// every stage, P = n2 / 2 / waves: in the stages with distance j <= P both keys of such a
// pair lie in the wave's own block of 2 P keys, so only the few stages with j > P need a
// workgroup barrier before and after; the others order the wave's own LDS accesses.
template <int BLOCK, int EPT, int WORDS>
__global__ __launch_bounds__(BLOCK * WORDS) void sparse_sort_words_kernel(
    const int32_t* __restrict__ words, int32_t n_words, TopicSource T,
    const int32_t* __restrict__ woff, const uint32_t* __restrict__ sp_off,
    int32_t* __restrict__ sp_topic, int32_t* __restrict__ sp_count, int32_t* __restrict__ sp_nnz,
    const uint32_t* __restrict__ hs_off, uint2* __restrict__ hs)
{
    static_assert(WORDS == 1 || BLOCK == 64, "several words per workgroup: one wave each");
    constexpr int CAP = BLOCK * EPT;
    constexpr int NW = BLOCK / 64;
    constexpr bool LDSROW = CAP <= 2048;  // row of 2 CAP slots (16 CAP bytes) beside the keys
    __shared__ uint2 rowl_all[LDSROW ? WORDS : 1][LDSROW ? 2 * CAP : 1];
    __shared__ uint32_t keys_all[WORDS][CAP];
    __shared__ int32_t first_all[WORDS][CAP];  // first[r] = position of the first token of run r
    __shared__ int32_t wsum[NW + 1];
    const int sub = (int)threadIdx.x / BLOCK, tid = (int)threadIdx.x % BLOCK;
    const int32_t wi = (int32_t)blockIdx.x * WORDS + sub;
    if (wi >= n_words) return;  // WORDS > 1: a whole wave leaves, no barrier follows
    uint32_t* __restrict__ keys = keys_all[sub];
    int32_t* __restrict__ first = first_all[sub];
    auto sync = [&](bool wide) {
        if (BLOCK > 64 && wide) __syncthreads(); else wave_lds_sync();
    };
    const int32_t w = words[wi];
    const int32_t b = woff[w], n = woff[w + 1] - b;
    if (n == 0) {  // uniform over the word's threads: an empty list and an empty row
        uint2* __restrict__ row0 = hs + hs_off[w];
        for (uint32_t i = tid; i < hs_off[w + 1] - hs_off[w]; i += BLOCK) row0[i] = make_uint2(0xFFFFFFFFu, 0u);
        if (tid == 0) sp_nnz[w] = 0;
        return;
    }
    int32_t n2 = 2;
    while (n2 < n) n2 <<= 1;
    for (int32_t i = tid; i < n2; i += BLOCK) keys[i] = i < n ? (uint32_t)T.at(b + i) : 0xFFFFFFFFu;
    sync(true);
    const int32_t half = n2 >> 1;
    const int32_t P = half >= NW ? half / NW : 1;
    const int lane = tid & 63, wv = tid >> 6;
    const int32_t pb = wv * P, pe = (pb + P < half) ? pb + P : half;
    for (int32_t k = 2; k <= n2; k <<= 1) {
        for (int32_t j = k >> 1; j > 0; j >>= 1) {
            for (int32_t i = pb + lane; i < pe; i += 64) {
                const int32_t l = 2 * i - (i & (j - 1));  // the pair (l, l + j)
                const uint32_t x = keys[l], y = keys[l + j];
                const bool up = (l & k) == 0;
                if ((x > y) == up) {
                    keys[l] = y;
                    keys[l + j] = x;
                }
            }
            const int32_t jn = j > 1 ? (j >> 1) : k;  // distance of the next stage
            sync(j > P || jn > P);
        }
    }
    sync(true);
    // thread t owns positions [t * per, t * per + per): heads of runs counted, then placed
    const int32_t per = (n2 + BLOCK - 1) / BLOCK;
    const int32_t i0 = tid * per, i1 = min(i0 + per, n);
    int32_t heads = 0;
    for (int32_t i = i0; i < i1; ++i) heads += (i == 0 || keys[i] != keys[i - 1]) ? 1 : 0;
    // exclusive prefix over the threads
    int32_t incl = heads;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t v = __shfl_up(incl, d, 64);
        if (lane >= d) incl += v;
    }
    int32_t base = 0, total;
    if constexpr (NW == 1) {
        total = __shfl(incl, 63, 64);
    } else {
        if (lane == 63) wsum[wv] = incl;
        __syncthreads();
        total = 0;
        for (int i = 0; i < NW; ++i) {
            if (i < wv) base += wsum[i];
            total += wsum[i];
        }
    }
    int32_t r = base + incl - heads;
    for (int32_t i = i0; i < i1; ++i) {
        if (i == 0 || keys[i] != keys[i - 1]) first[r++] = i;
    }
    sync(true);
    const size_t off = sp_off[w];
    uint2* __restrict__ row = hs + hs_off[w];
    const uint32_t cap = hs_off[w + 1] - hs_off[w];
    if constexpr (LDSROW) {
        // the hash row (at most 2 CAP slots) is filled in LDS and written out whole, empty slots
        // included: no global atomics, and the row needs no clearing beforehand
        uint2* __restrict__ rl = rowl_all[sub];
        const uint32_t lg = 31u - (uint32_t)__clz((int)cap);
        for (uint32_t i = tid; i < cap; i += BLOCK) rl[i] = make_uint2(0xFFFFFFFFu, 0u);
        sync(true);
        for (int32_t q = tid; q < total; q += BLOCK) {
            const int32_t s = first[q], e = (q + 1 < total) ? first[q + 1] : n;
            const int32_t topic = (int32_t)keys[s];
            sp_topic[off + q] = topic;
            sp_count[off + q] = e - s;
            uint32_t slot = row_hash_slot(topic, lg);
            for (uint32_t i = 0; i < cap; ++i) {
                if (atomicCAS(&rl[slot].x, 0xFFFFFFFFu, (uint32_t)topic) == 0xFFFFFFFFu) {
                    rl[slot].y = (uint32_t)(e - s);
                    break;
                }
                slot = (slot + 1) & (cap - 1);
            }
        }
        sync(true);
        for (uint32_t i = tid; i < cap; i += BLOCK) row[i] = rl[i];
    } else {
        for (int32_t q = tid; q < total; q += BLOCK) {
            const int32_t s = first[q], e = (q + 1 < total) ? first[q + 1] : n;
            const int32_t topic = (int32_t)keys[s];
            sp_topic[off + q] = topic;
            sp_count[off + q] = e - s;
            hash_row_insert(row, cap, topic, (uint32_t)(e - s));
        }
    }
    if (tid == 0) sp_nnz[w] = total;
}

// ---- partition by topic range ----------------------------------------------------------------

// dcount[seg * nd + d] += tokens of the tile whose topic lies in range d
__global__ __launch_bounds__(1024) void range_count_kernel(const PartTile* __restrict__ tiles,
                                                          TopicSource T, int32_t nd,
                                                          uint32_t* __restrict__ dcount)
{
    __shared__ uint32_t cnt[128];
    const PartTile t = tiles[blockIdx.x];
    const int tid = threadIdx.x;
    if (tid < 128) cnt[tid] = 0;
    __syncthreads();
    for (int32_t p = t.p0 + tid; p < t.p1; p += blockDim.x) atomicAdd(&cnt[T.at(p) >> kRangeShift], 1u);
    __syncthreads();
    if (tid < nd && cnt[tid]) atomicAdd(&dcount[(size_t)t.seg * nd + tid], cnt[tid]);
}

// dstart[seg * (nd + 1) + d] = base[seg] + tokens of the segment in ranges < d (d = 0..nd);
// cursor = the same; dcount is cleared for the next rebuild.  One wave per segment, nd <= 128.
__global__ __launch_bounds__(64) void range_scan_kernel(int32_t nd, const uint32_t* __restrict__ base,
                                                        uint32_t* __restrict__ dcount,
                                                        uint32_t* __restrict__ dstart,
                                                        uint32_t* __restrict__ cursor)
{
    const int32_t seg = blockIdx.x;
    const int lane = threadIdx.x;
    uint32_t run = base[seg];
    for (int32_t d0 = 0; d0 < nd; d0 += 64) {
        const int32_t d = d0 + lane;
        const uint32_t v = d < nd ? dcount[(size_t)seg * nd + d] : 0u;
        uint32_t incl = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const uint32_t u = __shfl_up(incl, s, 64);
            if (lane >= s) incl += u;
        }
        if (d < nd) {
            dstart[(size_t)seg * (nd + 1) + d] = run + incl - v;
            cursor[(size_t)seg * nd + d] = run + incl - v;
            dcount[(size_t)seg * nd + d] = 0u;
        }
        run += __shfl(incl, 63, 64);
    }
    if (lane == 0) dstart[(size_t)seg * (nd + 1) + nd] = run;
}

// part[...] = the tile's topics, each in its range's part of the segment (any order inside)
__global__ __launch_bounds__(1024) void range_scatter_kernel(const PartTile* __restrict__ tiles,
                                                            TopicSource T, int32_t nd,
                                                            uint32_t* __restrict__ cursor,
                                                            int32_t* __restrict__ part)
{
    __shared__ uint32_t cnt[128], gbase[128];
    const PartTile t = tiles[blockIdx.x];
    const int tid = threadIdx.x;
    if (tid < 128) cnt[tid] = 0;
    __syncthreads();
    // a thread's tokens, their ranks inside the tile's share of each range
    constexpr int E = kPartTile / 1024;
    int32_t topic[E];
    uint32_t rank[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int32_t p = t.p0 + e * 1024 + tid;
        topic[e] = p < t.p1 ? T.at(p) : -1;
    }
#pragma unroll
    for (int e = 0; e < E; ++e)
        if (topic[e] >= 0) rank[e] = atomicAdd(&cnt[topic[e] >> kRangeShift], 1u);
    __syncthreads();
    if (tid < nd && cnt[tid]) gbase[tid] = atomicAdd(&cursor[(size_t)t.seg * nd + tid], cnt[tid]);
    __syncthreads();
#pragma unroll
    for (int e = 0; e < E; ++e)
        if (topic[e] >= 0) part[gbase[topic[e] >> kRangeShift] + rank[e]] = topic[e];
}

// ---- long words: one workgroup per (word, range) ---------------------------------------------

// EMIT false: nnzd[lw * nd + d] = non-zero topics of the range.  EMIT true: the range's
// (topic, count) pairs, ascending, at list position lofs[lw * (nd + 1) + d].
template <bool EMIT>
__global__ __launch_bounds__(256) void long_word_ranges_kernel(
    const int32_t* __restrict__ long_words, int32_t nd, const uint32_t* __restrict__ dstart,
    const int32_t* __restrict__ part, uint32_t* __restrict__ nnzd,
    const uint32_t* __restrict__ lofs, const uint32_t* __restrict__ sp_off,
    int32_t* __restrict__ sp_topic, int32_t* __restrict__ sp_count)
{
    __shared__ int32_t hist[kRangeTopics];
    __shared__ int32_t wsum[4];
    const int32_t lw = blockIdx.x / nd, d = blockIdx.x % nd;
    const int tid = threadIdx.x;
    const uint32_t b = dstart[(size_t)lw * (nd + 1) + d], e = dstart[(size_t)lw * (nd + 1) + d + 1];
    if (b == e) {
        if (!EMIT && tid == 0) nnzd[(size_t)lw * nd + d] = 0u;
        return;
    }
    for (int32_t k = tid; k < kRangeTopics; k += 256) hist[k] = 0;
    __syncthreads();
    const int32_t k0 = d << kRangeShift;
    for (uint32_t i = b + tid; i < e; i += 256) atomicAdd(&hist[part[i] - k0], 1);
    __syncthreads();
    // every wave owns a contiguous quarter of the bins and walks it 64 bins at a time: the
    // non-zero bins of a step are ranked by a ballot, so their pairs go to consecutive places
    constexpr int per_wave = kRangeTopics / 4;
    const int lane = tid & 63, wv = tid >> 6;
    int32_t cnt = 0;
    for (int32_t kb = wv * per_wave; kb < (wv + 1) * per_wave; kb += 64)
        cnt += (int32_t)__popcll(__ballot(hist[kb + lane] > 0));
    if (lane == 0) wsum[wv] = cnt;
    __syncthreads();
    int32_t base = 0, total = 0;
    for (int i = 0; i < 4; ++i) {
        if (i < wv) base += wsum[i];
        total += wsum[i];
    }
    if constexpr (!EMIT) {
        if (tid == 0) nnzd[(size_t)lw * nd + d] = (uint32_t)total;
    } else {
        const int32_t w = long_words[lw];
        size_t pos = (size_t)sp_off[w] + lofs[(size_t)lw * (nd + 1) + d] + (size_t)base;
        for (int32_t kb = wv * per_wave; kb < (wv + 1) * per_wave; kb += 64) {
            const int32_t v = hist[kb + lane];
            const uint64_t mask = __ballot(v > 0);
            if (v > 0) {
                const size_t q = pos + (size_t)__popcll(mask & ((1ull << lane) - 1ull));
                sp_topic[q] = k0 + kb + lane;
                sp_count[q] = v;
            }
            pos += (size_t)__popcll(mask);
        }
    }
}

// The hash rows of the long words from their lists, one thread per list entry: a tile covers
// kFillTile places of one word's list (p0 = first place, seg = the word), of which the first
// sp_nnz[w] are in use.  (Inserting from the workgroups that write the lists made every thread
// wait for up to 32 atomics in turn: 22.7 instead of 4 + 9 ms at K = 10^6.)
constexpr int32_t kFillTile = 4096;

__global__ __launch_bounds__(256) void long_word_hash_rows_kernel(
    const PartTile* __restrict__ tiles, const int32_t* __restrict__ sp_nnz,
    const uint32_t* __restrict__ sp_off, const int32_t* __restrict__ sp_topic,
    const int32_t* __restrict__ sp_count, const uint32_t* __restrict__ hs_off, uint2* __restrict__ hs)
{
    const PartTile t = tiles[blockIdx.x];
    const int32_t w = t.seg, n = sp_nnz[w];
    const int32_t e1 = t.p1 < n ? t.p1 : n;
    const size_t off = sp_off[w];
    uint2* __restrict__ row = hs + hs_off[w];
    const uint32_t cap = hs_off[w + 1] - hs_off[w];
    for (int32_t e = t.p0 + (int32_t)threadIdx.x; e < e1; e += 256)
        hash_row_insert(row, cap, sp_topic[off + e], (uint32_t)sp_count[off + e]);
}

// lofs[lw * (nd + 1) + d] = non-zero topics of the word in ranges < d; sp_nnz[w] = all of them
__global__ __launch_bounds__(64) void long_word_offsets_kernel(const int32_t* __restrict__ long_words,
                                                               int32_t nd,
                                                               const uint32_t* __restrict__ nnzd,
                                                               uint32_t* __restrict__ lofs,
                                                               int32_t* __restrict__ sp_nnz)
{
    const int32_t lw = blockIdx.x;
    const int lane = threadIdx.x;
    uint32_t run = 0;
    for (int32_t d0 = 0; d0 < nd; d0 += 64) {
        const int32_t d = d0 + lane;
        const uint32_t v = d < nd ? nnzd[(size_t)lw * nd + d] : 0u;
        uint32_t incl = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const uint32_t u = __shfl_up(incl, s, 64);
            if (lane >= s) incl += u;
        }
        if (d < nd) lofs[(size_t)lw * (nd + 1) + d] = run + incl - v;
        run += __shfl(incl, 63, 64);
    }
    if (lane == 0) {
        lofs[(size_t)lw * (nd + 1) + nd] = run;
        sp_nnz[long_words[lw]] = (int32_t)run;
    }
}

// ---- n_k from the partitioned z ---------------------------------------------------------------

// blockIdx.y: range; blockIdx.x: chunk of kNkChunk tokens of the range's part.  n_k is zero on entry.
__global__ __launch_bounds__(1024) void nk_ranges_kernel(const uint32_t* __restrict__ dstart,
                                                        const int32_t* __restrict__ part, int32_t K,
                                                        int32_t* __restrict__ nk)
{
    __shared__ int32_t hist[kRangeTopics];
    const int32_t d = blockIdx.y;
    const uint32_t b = dstart[d] + (uint32_t)blockIdx.x * (uint32_t)kNkChunk;
    const uint32_t end = dstart[d + 1];
    if (b >= end) return;
    const uint32_t e = (end - b > (uint32_t)kNkChunk) ? b + (uint32_t)kNkChunk : end;
    const int tid = threadIdx.x;
    for (int32_t k = tid; k < kRangeTopics; k += 1024) hist[k] = 0;
    __syncthreads();
    const int32_t k0 = d << kRangeShift;
    for (uint32_t i = b + tid; i < e; i += 1024) atomicAdd(&hist[part[i] - k0], 1);
    __syncthreads();
    for (int32_t k = tid; k < kRangeTopics; k += 1024) {
        const int32_t v = hist[k];
        if (v && k0 + k < K) atomicAdd(&nk[k0 + k], v);
    }
}

// Empties the hash rows of the listed words: blockIdx.y = word, blockIdx.x = piece of
// kClearPiece slots of its row (pieces past the row's end return at once).
constexpr uint32_t kClearPiece = 1u << 16;

__global__ __launch_bounds__(256) void clear_hash_rows_kernel(const int32_t* __restrict__ words,
                                                              const uint32_t* __restrict__ hs_off,
                                                              uint2* __restrict__ hs)
{
    const int32_t w = words[blockIdx.y];
    const uint32_t cap = hs_off[w + 1] - hs_off[w];
    const uint32_t b = blockIdx.x * kClearPiece;
    if (b >= cap) return;
    const uint32_t e = (cap - b > kClearPiece) ? b + kClearPiece : cap;
    uint2* __restrict__ row = hs + hs_off[w];
    for (uint32_t i = b + threadIdx.x; i < e; i += 256) row[i] = make_uint2(0xFFFFFFFFu, 0u);
}

__global__ __launch_bounds__(256) void clear_all_hash_rows_kernel(uint2* __restrict__ hs, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        hs[i] = make_uint2(0xFFFFFFFFu, 0u);
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* __restrict__ p, int64_t n, uint32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

unsigned blocks_for(int64_t n, int block, unsigned most)
{
    int64_t b = (n + block - 1) / block;
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>(b, most));
}

int32_t range_count(int32_t K) { return (K + kRangeTopics - 1) / kRangeTopics; }

template <class T>
int upload_vec(lda_ctx* c, T** dst, const std::vector<T>& v, const char* what)
{
    const int rc = device_malloc(c, dst, v.size(), what);
    if (rc != LDA_OK) return rc;
    if (!v.empty())
        LDA_HIP(c, hipMemcpy(*dst, v.data(), sizeof(T) * v.size(), hipMemcpyHostToDevice));
    return LDA_OK;
}

TopicSource word_major_source(const lda_ctx* c)
{
    return TopicSource{c->d_zt, c->d_xmap, c->zt_shift, c->zt_mask};
}

}  // namespace

// Work lists and buffers of the sparse-row rebuild; woff: host copy of the word offsets.
int setup_sparse_rows(lda_ctx* c, const std::vector<int32_t>& woff)
{
    const int32_t H = c->H, V = c->V;
    std::vector<int32_t> cls[3], longw;
    std::vector<uint32_t> base;
    std::vector<PartTile> tiles, fill;
    uint32_t total = 0;
    for (int32_t w = H; w < V; ++w) {
        const int32_t n = woff[w + 1] - woff[w];
        if (n <= kSortTokensA) cls[0].push_back(w);
        else if (n <= kSortTokensB) cls[1].push_back(w);
        else if (n <= kSortMaxTokens) cls[2].push_back(w);
        else {
            const int32_t lw = (int32_t)longw.size();
            longw.push_back(w);
            base.push_back(total);
            for (int32_t p = woff[w]; p < woff[w + 1]; p += kPartTile)
                tiles.push_back(PartTile{lw, p, std::min(p + kPartTile, woff[w + 1])});
            total += (uint32_t)n;
            const int32_t places = std::min(n, c->K);  // capacity of the word's list
            for (int32_t e = 0; e < places; e += kFillTile)
                fill.push_back(PartTile{w, e, std::min(e + kFillTile, places)});
        }
    }
    int rc;
    for (int i = 0; i < 3; ++i) {
        c->n_sort_words[i] = (int32_t)cls[i].size();
        if ((rc = upload_vec(c, &c->d_sort_words[i], cls[i], "short sparse-row words")) != LDA_OK) return rc;
    }
    c->max_hash_row = 0;
    uint64_t atomically_filled = 0;  // slots of the rows of class 2 and of the long words
    for (int32_t w = H; w < V; ++w) {
        const uint32_t cap = c->h_hs_off[w + 1] - c->h_hs_off[w];
        if (woff[w + 1] - woff[w] > kSortTokensB) {
            c->max_hash_row = std::max(c->max_hash_row, cap);
            atomically_filled += cap;
        }
    }
    c->clear_all_hash_rows = 2 * atomically_filled > (uint64_t)c->total_hash;
    c->n_long_words = (int32_t)longw.size();
    c->n_long_tiles = (int32_t)tiles.size();
    c->n_fill_tiles = (int32_t)fill.size();
    c->long_word_tokens = total;
    if (c->n_long_words > 0) {
        const size_t nd = (size_t)range_count(c->K), nl = longw.size();
        if ((rc = upload_vec(c, &c->d_long_words, longw, "long sparse-row words")) != LDA_OK) return rc;
        if ((rc = upload_vec(c, &c->d_long_base, base, "long sparse-row words")) != LDA_OK) return rc;
        if ((rc = upload_vec(c, &c->d_long_tiles, tiles, "partition tiles")) != LDA_OK) return rc;
        if ((rc = upload_vec(c, &c->d_fill_tiles, fill, "hash row tiles")) != LDA_OK) return rc;
        LDA_ALLOC(c, &c->d_long_part, (size_t)total, "partitioned topics");
        LDA_ALLOC(c, &c->d_long_dcount, nl * nd, "range counts");
        LDA_ALLOC(c, &c->d_long_dstart, nl * (nd + 1), "range offsets");
        LDA_ALLOC(c, &c->d_long_cursor, nl * nd, "range cursors");
        LDA_ALLOC(c, &c->d_long_nnzd, nl * nd, "range non-zeros");
        LDA_ALLOC(c, &c->d_long_lofs, nl * (nd + 1), "range list offsets");
        LDA_HIP(c, hipMemsetAsync(c->d_long_dcount, 0, sizeof(uint32_t) * nl * nd, c->stream));
    }
    return LDA_OK;
}

// Lists, list lengths and hash rows of every word without a dense row, from the word-major z.
int launch_sparse_rows(lda_ctx* c)
{
    if (c->V <= c->H) return LDA_OK;
    const TopicSource T = word_major_source(c);
    // rows that are filled by global atomics start empty: class 2 and the long words, word by
    // word, or the whole array at once when they own most of it
    const unsigned pieces = (unsigned)((c->max_hash_row + kClearPiece - 1) / kClearPiece);
    if (c->clear_all_hash_rows) {
        hipLaunchKernelGGL(clear_all_hash_rows_kernel, dim3(blocks_for(c->total_hash, 256, 65536)), dim3(256),
                           0, c->stream, c->d_hs, c->total_hash);
        LDA_HIP(c, hipGetLastError());
    } else if (pieces > 0) {
        if (c->n_sort_words[2] > 0)
            hipLaunchKernelGGL(clear_hash_rows_kernel, dim3(pieces, c->n_sort_words[2]), dim3(256), 0,
                               c->stream, c->d_sort_words[2], c->d_hs_off, c->d_hs);
        if (c->n_long_words > 0)
            hipLaunchKernelGGL(clear_hash_rows_kernel, dim3(pieces, c->n_long_words), dim3(256), 0, c->stream,
                               c->d_long_words, c->d_hs_off, c->d_hs);
        LDA_HIP(c, hipGetLastError());
    }
#define LDA_SORT(i, BLOCK, EPT, WORDS)                                                                 \
    if (c->n_sort_words[i] > 0) {                                                                      \
        hipLaunchKernelGGL((sparse_sort_words_kernel<BLOCK, EPT, WORDS>),                              \
                           dim3((c->n_sort_words[i] + WORDS - 1) / WORDS), dim3(BLOCK * WORDS), 0,     \
                           c->stream, c->d_sort_words[i], c->n_sort_words[i], T, c->d_woff, c->d_sp_off, \
                           c->d_sp_topic, c->d_sp_count, c->d_sp_nnz, c->d_hs_off, c->d_hs);           \
        LDA_HIP(c, hipGetLastError());                                                                 \
    }
    LDA_SORT(0, 64, kSortTokensA / 64, 4)
    LDA_SORT(1, 256, kSortTokensB / 256, 1)
    LDA_SORT(2, 1024, kSortMaxTokens / 1024, 1)
#undef LDA_SORT
    if (c->n_long_words > 0) {
        const int32_t nd = range_count(c->K), nl = c->n_long_words;
        const PartTile* tiles = c->d_long_tiles;
        hipLaunchKernelGGL(range_count_kernel, dim3(c->n_long_tiles), dim3(1024), 0, c->stream, tiles, T,
                           nd, c->d_long_dcount);
        hipLaunchKernelGGL(range_scan_kernel, dim3(nl), dim3(64), 0, c->stream, nd, c->d_long_base,
                           c->d_long_dcount, c->d_long_dstart, c->d_long_cursor);
        hipLaunchKernelGGL(range_scatter_kernel, dim3(c->n_long_tiles), dim3(1024), 0, c->stream, tiles, T,
                           nd, c->d_long_cursor, c->d_long_part);
        hipLaunchKernelGGL((long_word_ranges_kernel<false>), dim3((unsigned)nl * nd), dim3(256), 0, c->stream,
                           c->d_long_words, nd, c->d_long_dstart, c->d_long_part, c->d_long_nnzd,
                           c->d_long_lofs, c->d_sp_off, c->d_sp_topic, c->d_sp_count);
        hipLaunchKernelGGL(long_word_offsets_kernel, dim3(nl), dim3(64), 0, c->stream, c->d_long_words, nd,
                           c->d_long_nnzd, c->d_long_lofs, c->d_sp_nnz);
        hipLaunchKernelGGL((long_word_ranges_kernel<true>), dim3((unsigned)nl * nd), dim3(256), 0, c->stream,
                           c->d_long_words, nd, c->d_long_dstart, c->d_long_part, c->d_long_nnzd,
                           c->d_long_lofs, c->d_sp_off, c->d_sp_topic, c->d_sp_count);
        hipLaunchKernelGGL(long_word_hash_rows_kernel, dim3(c->n_fill_tiles), dim3(256), 0, c->stream,
                           c->d_fill_tiles, c->d_sp_nnz, c->d_sp_off, c->d_sp_topic, c->d_sp_count,
                           c->d_hs_off, c->d_hs);
        LDA_HIP(c, hipGetLastError());
    }
    return LDA_OK;
}

// n_k for K beyond what LDS histograms over all of z cover in a few passes: z partitioned by
// topic range, then one LDS histogram per chunk of a range.  (One global atomic per token, the
// alternative, runs at about 27 G atomics/s: 18.6 ms for 5e8 tokens.)
int launch_nk_by_ranges(lda_ctx* c)
{
    const int32_t nd = range_count(c->K);
    const int64_t N = c->N;
    if (!c->d_nk_part) {
        std::vector<PartTile> tiles;
        for (int64_t p = 0; p < N; p += kPartTile)
            tiles.push_back(PartTile{0, (int32_t)p, (int32_t)std::min<int64_t>(p + kPartTile, N)});
        c->n_nk_tiles = (int32_t)tiles.size();
        int rc = upload_vec(c, &c->d_nk_tiles, tiles, "partition tiles");
        if (rc != LDA_OK) return rc;
        LDA_ALLOC(c, &c->d_nk_part, (size_t)N, "partitioned topics");
        LDA_ALLOC(c, &c->d_nk_ranges, 3 * (size_t)nd + 2, "range counts");  // counts, cursors, base, offsets
        LDA_HIP(c, hipMemsetAsync(c->d_nk_ranges, 0, sizeof(uint32_t) * (3 * (size_t)nd + 2), c->stream));
    }
    uint32_t* dcount = c->d_nk_ranges;
    uint32_t* cursor = dcount + nd;
    uint32_t* base = cursor + nd;      // one zero
    uint32_t* dstart = base + 1;       // nd + 1 entries
    // any order of the topics will do: the word-major copy when z itself is not resident
    const TopicSource T{c->streamed ? c->d_zt : c->d_z, nullptr, 0, 0xFFFFFFFFu};
    const PartTile* tiles = c->d_nk_tiles;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(c->K, 256, 1024)), dim3(256), 0, c->stream,
                       reinterpret_cast<uint32_t*>(c->d_nk), (int64_t)c->K, 0u);
    hipLaunchKernelGGL(range_count_kernel, dim3(c->n_nk_tiles), dim3(1024), 0, c->stream, tiles, T, nd, dcount);
    hipLaunchKernelGGL(range_scan_kernel, dim3(1), dim3(64), 0, c->stream, nd, base, dcount, dstart, cursor);
    hipLaunchKernelGGL(range_scatter_kernel, dim3(c->n_nk_tiles), dim3(1024), 0, c->stream, tiles, T, nd,
                       cursor, c->d_nk_part);
    // a range may hold all N tokens; chunks past a range's end return at once
    const unsigned chunks = (unsigned)((N + kNkChunk - 1) / kNkChunk);
    hipLaunchKernelGGL(nk_ranges_kernel, dim3(chunks, (unsigned)nd), dim3(1024), 0, c->stream, dstart,
                       c->d_nk_part, c->K, c->d_nk);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
