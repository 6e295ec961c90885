// One-time layout work of lda_init: the word-major token order (LightLDA Sec. 6,
// "Tuning the Structure-Aware Model Parallelization", item 3: tokens sorted by
// word so that each word's tokens are contiguous), the segment offsets, the
// initial assignment, and input validation.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

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
