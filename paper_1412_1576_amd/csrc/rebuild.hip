// Count rebuild (LightLDA Sec. 3: the sufficient statistics n_kw and n_k).
//
// n_kw: tokens are laid out word-major, so every word's tokens are one
// contiguous segment; a workgroup histograms a tile of a segment in LDS
// (gathering each token's new topic through the word-major -> CSR map) and
// writes the dense row.  Words whose segment is longer than one tile are split
// over several workgroups whose partial histograms are merged into a
// pre-zeroed row with integer atomics (order-free, hence exact).
// n_k: an LDS-privatised histogram of z over all tokens.
#include "common.hpp"

namespace lda {

namespace {

__global__ __launch_bounds__(1024) void nkw_tiles_kernel(const RebuildTile* __restrict__ tiles,
                                                         const int32_t* __restrict__ gid,
                                                         const int32_t* __restrict__ z,
                                                         int32_t K, int32_t* __restrict__ nkw)
{
    extern __shared__ int32_t hist[];
    const RebuildTile t = tiles[blockIdx.x];
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int32_t k = tid; k < K; k += nt) hist[k] = 0;
    __syncthreads();
    for (int32_t p = t.p0 + tid; p < t.p1; p += nt) atomicAdd(&hist[z[gid[p]]], 1);
    __syncthreads();
    int32_t* __restrict__ row = nkw + (size_t)t.w * (size_t)K;
    if (t.multi) {
        for (int32_t k = tid; k < K; k += nt) {
            const int32_t v = hist[k];
            if (v) atomicAdd(&row[k], v);
        }
    } else {
        for (int32_t k = tid; k < K; k += nt) row[k] = hist[k];
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

// n_k: each block histograms a contiguous slice of z in LDS, then adds its
// non-zero bins to the (pre-zeroed) global row.
__global__ __launch_bounds__(1024) void nk_hist_kernel(const int32_t* __restrict__ z, int64_t N,
                                                       int32_t K, int32_t* __restrict__ nk)
{
    extern __shared__ int32_t hist[];
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int32_t k = tid; k < K; k += nt) hist[k] = 0;
    __syncthreads();
    const int64_t per = (N + gridDim.x - 1) / gridDim.x;
    const int64_t b = (int64_t)blockIdx.x * per;
    const int64_t e = (b + per < N) ? b + per : N;
    for (int64_t i = b + tid; i < e; i += nt) atomicAdd(&hist[z[i]], 1);
    __syncthreads();
    for (int32_t k = tid; k < K; k += nt) {
        const int32_t v = hist[k];
        if (v) atomicAdd(&nk[k], v);
    }
}

}  // namespace

int max_rebuild_topics() { return 36 * 1024; }

int launch_rebuild(lda_ctx* c)
{
    const int32_t K = c->K;
    if (K > max_rebuild_topics())
        return fail(c, LDA_ERR_UNSUPPORTED, "count rebuild supports K <= %d", max_rebuild_topics());
    const size_t lds = sizeof(int32_t) * (size_t)K;
    if (lds > 48 * 1024) {
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(nkw_tiles_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(nk_hist_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    }
    if (c->n_multi_words > 0) {
        hipLaunchKernelGGL(zero_rows_kernel, dim3(c->n_multi_words), dim3(256), 0, c->stream,
                           c->d_multi_words, K, c->d_nkw);
        LDA_HIP(c, hipGetLastError());
    }
    // block size: small rows do not need 1024 threads
    int block = 1024;
    if (K <= 512) block = 256;
    hipLaunchKernelGGL(nkw_tiles_kernel, dim3(c->n_tiles), dim3(block), lds, c->stream, c->d_tiles,
                       c->d_gid, c->d_z, K, c->d_nkw);
    LDA_HIP(c, hipGetLastError());

    hipLaunchKernelGGL(fill_i32_kernel, dim3(64), dim3(256), 0, c->stream, c->d_nk, (int64_t)K, 0);
    LDA_HIP(c, hipGetLastError());
    int64_t blocks = (c->N + 65535) / 65536;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(nk_hist_kernel, dim3((unsigned)blocks), dim3(1024), lds, c->stream, c->d_z,
                       c->N, K, c->d_nk);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
