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
        LDA_HIP(c, hipMalloc(reinterpret_cast<void**>(&c->d_sort_keys), sizeof(int32_t) * (size_t)N));
        LDA_HIP(c, hipMalloc(&c->d_sort_tmp, bytes ? bytes : 1));
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

int launch_layout(lda_ctx* c, const int32_t* /*h_word*/)
{
    const int64_t N = c->N;
    // stable radix sort of (word, CSR position) pairs: positions of one word stay ascending
    int32_t *keys_out = nullptr, *vals_in = nullptr;
    LDA_HIP(c, hipMalloc(&keys_out, sizeof(int32_t) * N));
    if (hipMalloc(&vals_in, sizeof(int32_t) * N) != hipSuccess) {
        (void)hipFree(keys_out);
        return fail(c, LDA_ERR_OOM, "layout: device allocation of %lld bytes failed",
                    (long long)(sizeof(int32_t) * N));
    }
    hipLaunchKernelGGL(iota_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, vals_in, N);
    int end_bit = 1;
    while (end_bit < 31 && (1LL << end_bit) < (long long)c->V) ++end_bit;
    size_t tmp_bytes = 0;
    void* tmp = nullptr;
    hipError_t e = rocprim::radix_sort_pairs(nullptr, tmp_bytes, c->d_word, keys_out, vals_in,
                                             c->d_gid, (size_t)N, 0u, (unsigned)end_bit, c->stream);
    if (e == hipSuccess) e = hipMalloc(&tmp, tmp_bytes > 0 ? tmp_bytes : 1);
    if (e == hipSuccess)
        e = rocprim::radix_sort_pairs(tmp, tmp_bytes, c->d_word, keys_out, vals_in, c->d_gid,
                                      (size_t)N, 0u, (unsigned)end_bit, c->stream);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(word_offsets_kernel, dim3((c->V + 1 + 255) / 256), dim3(256), 0,
                           c->stream, keys_out, N, c->V, c->d_woff);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    (void)hipFree(tmp);
    (void)hipFree(keys_out);
    (void)hipFree(vals_in);
    if (e != hipSuccess)
        return fail(c, e == hipErrorOutOfMemory ? LDA_ERR_OOM : LDA_ERR_HIP, "layout sort: %s",
                    hipGetErrorString(e));

    hipLaunchKernelGGL(invert_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, c->d_gid, N,
                       c->d_wpos);
    LDA_HIP(c, hipGetLastError());
    hipLaunchKernelGGL(init_z_kernel, dim3(grid_for(N, 256)), dim3(256), 0, c->stream, c->d_z, N,
                       c->K, (uint32_t)c->seed, (uint32_t)(c->seed >> 32));
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
