// One-time layout work of lda_init: the word-major token order (LightLDA Sec. 6,
// "Tuning the Structure-Aware Model Parallelization", item 3: tokens sorted by
// word so that each word's tokens are contiguous), the segment offsets, the
// initial assignment, and input validation.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_run_length_encode.hpp>

#include "common.hpp"

namespace lda {

namespace {

__global__ __launch_bounds__(256) void iota_kernel(int32_t* __restrict__ p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = (int32_t)i;
}

// woff[w] = first position p with sorted_word[p] >= w, w = 0..V
__global__ __launch_bounds__(256) void word_offsets_kernel(const int32_t* __restrict__ sorted_word,
                                                           int64_t n, int32_t V,
                                                           int32_t* __restrict__ woff)
{
    const int32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w > V) return;
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (sorted_word[mid] < w) lo = mid + 1; else hi = mid;
    }
    woff[w] = (int32_t)lo;
}

// z[g] = floor(x0 * K / 2^32), Philox counter (g, 0, 0xFFFFFFFF, 0)
__global__ __launch_bounds__(256) void init_z_kernel(int32_t* __restrict__ z, int64_t n, int32_t K,
                                                     uint32_t seed_lo, uint32_t seed_hi)
{
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n;
         g += (int64_t)gridDim.x * blockDim.x) {
        uint32_t x[4];
        philox4x32_10((uint32_t)g, (uint32_t)((uint64_t)g >> 32), 0xFFFFFFFFu, 0u, seed_lo, seed_hi,
                      x);
        z[g] = (int32_t)mulhi32(x[0], (uint32_t)K);
    }
}

__global__ __launch_bounds__(256) void check_range_kernel(const int32_t* __restrict__ v, int64_t n,
                                                          int32_t lo, int32_t hi,
                                                          int32_t* __restrict__ bad)
{
    bool any = false;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t x = v[i];
        any |= (x < lo) | (x >= hi);
    }
    if (any) atomicOr(bad, 1);
}

// wpos[gid[p]] = p
__global__ __launch_bounds__(256) void invert_kernel(const int32_t* __restrict__ gid, int64_t n,
                                                     int32_t* __restrict__ wpos)
{
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n;
         p += (int64_t)gridDim.x * blockDim.x)
        wpos[gid[p]] = (int32_t)p;
}

// keys[p] = bucket of the token at word-major position p (its CSR position >> shift)
__global__ __launch_bounds__(256) void bucket_keys_kernel(const int32_t* __restrict__ gid, int64_t n,
                                                          int shift, int32_t* __restrict__ keys)
{
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n;
         p += (int64_t)gridDim.x * blockDim.x)
        keys[p] = gid[p] >> shift;
}

// wpos[g] = xmap[wpos[g]]
__global__ __launch_bounds__(256) void compose_kernel(int32_t* __restrict__ wpos, int64_t n,
                                                      const int32_t* __restrict__ xmap)
{
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n;
         g += (int64_t)gridDim.x * blockDim.x)
        wpos[g] = xmap[wpos[g]];
}

// n_k[k] = number of entries equal to k in the ascending array `sorted`
__global__ __launch_bounds__(256) void nk_from_sorted_kernel(const int32_t* __restrict__ sorted,
                                                             int64_t n, int32_t K,
                                                             int32_t* __restrict__ nk)
{
    const int32_t k = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (k >= K) return;
    int64_t bound[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {  // first position whose key is >= k + j
        int64_t lo = 0, hi = n;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (sorted[mid] < k + j) lo = mid + 1; else hi = mid;
        }
        bound[j] = lo;
    }
    nk[k] = (int32_t)(bound[1] - bound[0]);
}

// ---- sparse rows by one global sort (words without a dense row are the ids >= H, so their
// tokens are the word-major positions [p0, N)) ---------------------------------------------

// wloc[i] = (word of position p0 + i) - H: the last w >= H with woff[w] <= p0 + i
__global__ __launch_bounds__(256) void sparse_wloc_kernel(const int32_t* __restrict__ woff, int32_t H,
                                                          int32_t V, int64_t p0, int64_t n,
                                                          uint32_t* __restrict__ wloc)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t p = p0 + i;
        int32_t lo = H, hi = V;  // woff[lo] <= p < woff[hi]
        while (hi - lo > 1) {
            const int32_t mid = lo + ((hi - lo) >> 1);
            if (woff[mid] <= p) lo = mid; else hi = mid;
        }
        wloc[i] = (uint32_t)(lo - H);
    }
}

// key = (word - H) << tb | topic
__global__ __launch_bounds__(256) void sparse_keys_kernel(const int32_t* __restrict__ zt, int32_t sh,
                                                          uint32_t zmask,
                                                          const uint32_t* __restrict__ wloc,
                                                          int64_t p0, int64_t n, int32_t tb,
                                                          const int32_t* __restrict__ xmap,
                                                          uint64_t* __restrict__ keys)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const size_t q = xmap ? (size_t)xmap[p0 + i] : (size_t)(p0 + i);
        keys[i] = ((uint64_t)wloc[i] << tb) | (uint64_t)((uint32_t)zt[q << sh] & zmask);
    }
}

// first[wl] = index of the first run (distinct key) of word H + wl, wl = 0..n_words
__global__ __launch_bounds__(256) void sparse_first_run_kernel(const uint64_t* __restrict__ uniq,
                                                               const int32_t* __restrict__ n_runs,
                                                               int32_t n_words, int32_t tb,
                                                               int32_t* __restrict__ first)
{
    const int32_t wl = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (wl > n_words) return;
    const uint64_t key = (uint64_t)wl << tb;
    int32_t lo = 0, hi = *n_runs;
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (uniq[mid] < key) lo = mid + 1; else hi = mid;
    }
    first[wl] = lo;
}

// run r is entry r - first[word] of its word's list; it also goes into the word's hash row
// (cleared beforehand), one thread per entry so that a word with a million entries is
// filled by as many threads
__global__ __launch_bounds__(256) void sparse_lists_kernel(const uint64_t* __restrict__ uniq,
                                                           const uint32_t* __restrict__ counts,
                                                           const int32_t* __restrict__ n_runs,
                                                           const int32_t* __restrict__ first,
                                                           int32_t tb, int32_t H,
                                                           const uint32_t* __restrict__ sp_off,
                                                           int32_t* __restrict__ sp_topic,
                                                           int32_t* __restrict__ sp_count,
                                                           const uint32_t* __restrict__ hs_off,
                                                           uint2* __restrict__ hs)
{
    const int64_t nr = *n_runs;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < nr;
         r += (int64_t)gridDim.x * blockDim.x) {
        const uint64_t key = uniq[r];
        const uint32_t wl = (uint32_t)(key >> tb);
        const int32_t w = H + (int32_t)wl;
        const int32_t topic = (int32_t)(key & ((1ull << tb) - 1ull));
        const uint32_t count = counts[r];
        const size_t pos = (size_t)sp_off[w] + (size_t)(r - first[wl]);
        sp_topic[pos] = topic;
        sp_count[pos] = (int32_t)count;
        uint2* __restrict__ row = hs + hs_off[w];
        const uint32_t cap = hs_off[w + 1] - hs_off[w];  // a power of two, at least twice the entries
        const uint32_t lg = 31u - (uint32_t)__clz((int)cap);
        uint32_t slot = row_hash_slot(topic, lg);
        for (uint32_t i = 0; i < cap; ++i) {
            if (atomicCAS(&row[slot].x, 0xFFFFFFFFu, (uint32_t)topic) == 0xFFFFFFFFu) {
                row[slot].y = count;
                break;
            }
            slot = (slot + 1) & (cap - 1);
        }
    }
}

// list lengths from the first-run indices
__global__ __launch_bounds__(256) void sparse_nnz_kernel(const int32_t* __restrict__ first,
                                                         int32_t n_words, int32_t H,
                                                         int32_t* __restrict__ sp_nnz)
{
    const int32_t wl = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (wl < n_words) sp_nnz[H + wl] = first[wl + 1] - first[wl];
}

__global__ __launch_bounds__(256) void clear_hash_kernel(uint2* __restrict__ hs, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        hs[i] = make_uint2(0xFFFFFFFFu, 0u);
}

unsigned grid_for(int64_t n, int block, unsigned cap = 8192)
{
    int64_t b = (n + block - 1) / block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

}  // namespace

int launch_check_range(lda_ctx* c, const int32_t* d_vals, int64_t n, int32_t lo, int32_t hi,
                       bool* ok)
{
    int32_t zero = 0, bad = 0;
    LDA_HIP(c, hipMemcpyAsync(c->d_flag, &zero, sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    hipLaunchKernelGGL(check_range_kernel, dim3(grid_for(n, 256)), dim3(256), 0, c->stream, d_vals,
                       n, lo, hi, c->d_flag);
    LDA_HIP(c, hipGetLastError());
    LDA_HIP(c, hipMemcpyAsync(&bad, c->d_flag, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    LDA_HIP(c, hipStreamSynchronize(c->stream));
    *ok = (bad == 0);
    return LDA_OK;
}

// n_k for K beyond what LDS histograms cover in a few passes over z: radix sort of z, then
// the run length of every topic by bisection.  (One global atomic per token, the
// alternative, runs at about 27 G atomics/s: 18.6 ms for 5e8 tokens against 5 ms for this.)
int launch_nk_by_sort(lda_ctx* c)
{
    const int64_t N = c->N;
    int end_bit = 1;
    while (end_bit < 31 && (1LL << end_bit) < (long long)c->K) ++end_bit;
    if (!c->d_sort_keys) {
        size_t bytes = 0;
        LDA_HIP(c, rocprim::radix_sort_keys(nullptr, bytes, c->d_z, c->d_z, (size_t)N, 0u,
                                            (unsigned)end_bit, c->stream));
        LDA_ALLOC(c, &c->d_sort_keys, N, "sorted topics");
        LDA_ALLOC(c, reinterpret_cast<unsigned char**>(&c->d_sort_tmp), bytes, "sort workspace");
        c->sort_tmp_bytes = bytes;
    }
    size_t bytes = c->sort_tmp_bytes;
    LDA_HIP(c, rocprim::radix_sort_keys(c->d_sort_tmp, bytes, c->d_z, c->d_sort_keys, (size_t)N, 0u,
                                        (unsigned)end_bit, c->stream));
    hipLaunchKernelGGL(nk_from_sorted_kernel, dim3((c->K + 255) / 256), dim3(256), 0, c->stream,
                       c->d_sort_keys, N, c->K, c->d_nk);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

// Sorted (topic, count) lists, their lengths and the hash rows of every word without a dense
// row, from one radix sort of (word, topic) keys over their tokens and a run-length encoding.
int launch_sparse_lists_by_sort(lda_ctx* c)
{
    const int32_t H = c->H, V = c->V, n_words = V - H;
    const int64_t p0 = c->h_sparse_p0, n = c->N - p0;
    if (n_words <= 0) return LDA_OK;
    int tb = 1, wb = 1;
    while (tb < 31 && (1LL << tb) < (long long)c->K) ++tb;
    while (wb < 31 && (1LL << wb) < (long long)n_words) ++wb;
    if (!c->d_sp_first) {
        LDA_ALLOC(c, &c->d_sp_first, (size_t)n_words + 2, "first runs");
        LDA_ALLOC(c, &c->d_sp_nruns, 2, "run count");
        LDA_HIP(c, hipMemsetAsync(c->d_sp_nruns, 0, sizeof(int32_t) * 2, c->stream));
        const size_t m = (size_t)(n > 0 ? n : 1);
        LDA_ALLOC(c, &c->d_sp_wloc, m, "tail word indices");
        LDA_ALLOC(c, &c->d_sp_keys, m, "(word, topic) keys");
        LDA_ALLOC(c, &c->d_sp_sorted, m, "sorted keys");
        LDA_ALLOC(c, &c->d_sp_runlen, m, "run lengths");
        size_t b1 = 0, b2 = 0;
        LDA_HIP(c, rocprim::radix_sort_keys(nullptr, b1, c->d_sp_keys, c->d_sp_sorted, (size_t)n, 0u,
                                            (unsigned)(tb + wb), c->stream));
        LDA_HIP(c, rocprim::run_length_encode(nullptr, b2, c->d_sp_sorted, (size_t)n, c->d_sp_keys,
                                              c->d_sp_runlen, c->d_sp_nruns, c->stream));
        c->sp_tmp_bytes = b1 > b2 ? b1 : b2;
        LDA_ALLOC(c, reinterpret_cast<unsigned char**>(&c->d_sp_tmp), c->sp_tmp_bytes, "sort workspace");
        if (n > 0) {
            hipLaunchKernelGGL(sparse_wloc_kernel, dim3(grid_for(n, 256)), dim3(256), 0, c->stream,
                               c->d_woff, H, V, p0, n, c->d_sp_wloc);
            LDA_HIP(c, hipGetLastError());
        }
    }
    if (n > 0) {
        hipLaunchKernelGGL(sparse_keys_kernel, dim3(grid_for(n, 256)), dim3(256), 0, c->stream, c->d_zt,
                           c->zt_shift, c->zt_mask, c->d_sp_wloc, p0, n, tb, c->d_xmap, c->d_sp_keys);
        LDA_HIP(c, hipGetLastError());
        size_t bytes = c->sp_tmp_bytes;
        LDA_HIP(c, rocprim::radix_sort_keys(c->d_sp_tmp, bytes, c->d_sp_keys, c->d_sp_sorted, (size_t)n,
                                            0u, (unsigned)(tb + wb), c->stream));
        bytes = c->sp_tmp_bytes;
        // the distinct keys overwrite the unsorted ones
        LDA_HIP(c, rocprim::run_length_encode(c->d_sp_tmp, bytes, c->d_sp_sorted, (size_t)n,
                                              c->d_sp_keys, c->d_sp_runlen, c->d_sp_nruns, c->stream));
    }
    hipLaunchKernelGGL(sparse_first_run_kernel, dim3((n_words + 1 + 255) / 256), dim3(256), 0, c->stream,
                       c->d_sp_keys, c->d_sp_nruns, n_words, tb, c->d_sp_first);
    LDA_HIP(c, hipGetLastError());
    hipLaunchKernelGGL(sparse_nnz_kernel, dim3((n_words + 255) / 256), dim3(256), 0, c->stream,
                       c->d_sp_first, n_words, H, c->d_sp_nnz);
    LDA_HIP(c, hipGetLastError());
    if (c->total_hash > 0) {
        hipLaunchKernelGGL(clear_hash_kernel, dim3(grid_for(c->total_hash, 256, 65536)), dim3(256), 0,
                           c->stream, c->d_hs, c->total_hash);
        LDA_HIP(c, hipGetLastError());
    }
    if (n > 0) {
        hipLaunchKernelGGL(sparse_lists_kernel, dim3(grid_for(n, 256, 65536)), dim3(256), 0, c->stream,
                           c->d_sp_keys, c->d_sp_runlen, c->d_sp_nruns, c->d_sp_first, tb, H, c->d_sp_off,
                           c->d_sp_topic, c->d_sp_count, c->d_hs_off, c->d_hs);
        LDA_HIP(c, hipGetLastError());
    }
    return LDA_OK;
}

namespace {

// Record order of the sweep's exchange.  The word pass writes one record per token and reads
// one; the doc pass gathers and scatters them.  In plain word-major order the records of a
// rare word are spread over the whole array, so the doc pass's access to them is a miss in
// every cache.  Ordering the records by buckets of 2^shift consecutive tokens of the corpus
// (inside a bucket by word-major position) confines the doc pass, which walks the corpus in
// order, to one bucket's records at a time -- a window of some tens of megabytes that the
// memory-side cache holds -- while the word pass still meets the records of a word in
// ascending order, now as one run per bucket.
//   xmap[p] = rank of word-major position p under the key (gid[p] >> shift, p)
//   wpos[g] = xmap[wpos[g]]
int build_record_order(lda_ctx* c)
{
    const int64_t N = c->N;
    const int shift = c->record_bucket_shift;
    int32_t *keys = nullptr, *keys_sorted = nullptr, *pos = nullptr, *pos_sorted = nullptr;
    void* tmp = nullptr;
    auto release = [&]() {
        device_free(c, keys);
        device_free(c, keys_sorted);
        device_free(c, pos);
        device_free(c, pos_sorted);
        device_free(c, tmp);
    };
    int rc = device_malloc(c, &keys, (size_t)N, "record order");
    if (rc == LDA_OK) rc = device_malloc(c, &keys_sorted, (size_t)N, "record order");
    if (rc == LDA_OK) rc = device_malloc(c, &pos, (size_t)N, "record order");
    if (rc == LDA_OK) rc = device_malloc(c, &pos_sorted, (size_t)N, "record order");
    if (rc == LDA_OK) rc = device_malloc(c, &c->d_xmap, (size_t)N, "record order");
    if (rc != LDA_OK) {
        release();
        return rc;
    }
    hipLaunchKernelGGL(bucket_keys_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, c->d_gid, N,
                       shift, keys);
    hipLaunchKernelGGL(iota_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, pos, N);
    int end_bit = 1;
    while (end_bit < 31 && (1LL << end_bit) < ((long long)(N - 1) >> shift) + 1) ++end_bit;
    size_t tmp_bytes = 0;
    // stable: inside a bucket the word-major positions stay ascending
    hipError_t e = rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys, keys_sorted, pos, pos_sorted,
                                             (size_t)N, 0u, (unsigned)end_bit, c->stream);
    if (e == hipSuccess && (rc = device_malloc(c, &tmp, tmp_bytes, "record order")) != LDA_OK) {
        release();
        return rc;
    }
    if (e == hipSuccess)
        e = rocprim::radix_sort_pairs(tmp, tmp_bytes, keys, keys_sorted, pos, pos_sorted, (size_t)N, 0u,
                                      (unsigned)end_bit, c->stream);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(invert_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, pos_sorted, N,
                           c->d_xmap);
        hipLaunchKernelGGL(compose_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, c->d_wpos, N,
                           c->d_xmap);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    release();
    if (e != hipSuccess) return fail(c, LDA_ERR_HIP, "record order: %s", hipGetErrorString(e));
    return LDA_OK;
}

}  // namespace

int launch_layout(lda_ctx* c, const int32_t* /*h_word*/)
{
    const int64_t N = c->N;
    // stable radix sort of (word, CSR position) pairs: positions of one word stay ascending
    int32_t *keys_out = nullptr, *vals_in = nullptr;
    void* tmp = nullptr;
    auto release = [&]() {
        device_free(c, tmp);
        device_free(c, keys_out);
        device_free(c, vals_in);
    };
    int rc = device_malloc(c, &keys_out, (size_t)N, "layout sort");
    if (rc == LDA_OK) rc = device_malloc(c, &vals_in, (size_t)N, "layout sort");
    if (rc != LDA_OK) {
        release();
        return rc;
    }
    hipLaunchKernelGGL(iota_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, vals_in, N);
    int end_bit = 1;
    while (end_bit < 31 && (1LL << end_bit) < (long long)c->V) ++end_bit;
    size_t tmp_bytes = 0;
    hipError_t e = rocprim::radix_sort_pairs(nullptr, tmp_bytes, c->d_word, keys_out, vals_in,
                                             c->d_gid, (size_t)N, 0u, (unsigned)end_bit, c->stream);
    if (e == hipSuccess && (rc = device_malloc(c, &tmp, tmp_bytes, "layout sort")) != LDA_OK) {
        release();
        return rc;
    }
    if (e == hipSuccess)
        e = rocprim::radix_sort_pairs(tmp, tmp_bytes, c->d_word, keys_out, vals_in, c->d_gid,
                                      (size_t)N, 0u, (unsigned)end_bit, c->stream);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(word_offsets_kernel, dim3((c->V + 1 + 255) / 256), dim3(256), 0,
                           c->stream, keys_out, N, c->V, c->d_woff);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    release();
    if (e != hipSuccess)
        return fail(c, LDA_ERR_HIP, "layout sort: %s", hipGetErrorString(e));

    hipLaunchKernelGGL(invert_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, c->d_gid, N,
                       c->d_wpos);
    LDA_HIP(c, hipGetLastError());
    if (c->record_bucket_shift >= 0) {
        const int rc2 = build_record_order(c);
        if (rc2 != LDA_OK) return rc2;
    }
    hipLaunchKernelGGL(init_z_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, c->d_z, N,
                       c->K, (uint32_t)c->seed, (uint32_t)(c->seed >> 32));
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
