// Log-likelihood log p(w, z | alpha, beta) of the collapsed LDA model, the
// convergence metric of LightLDA Sec. 7 (doc-likelihood + word-likelihood):
//   doc  = sum_d [ lgG(K a) - lgG(L_d + K a) + sum_{k: n_kd>0} (lgG(n_kd + a) - lgG(a)) ]
//   word = sum_k [ lgG(V b) - lgG(n_k + V b) ] + sum_{w,k: n_kw>0} (lgG(n_kw + b) - lgG(b))
// fp64 throughout; every block reduces in a fixed tree and writes one partial,
// the host adds the partials in index order with compensation.
#include "common.hpp"
#include "doc_tile.hpp"

namespace lda {

namespace {

__device__ __forceinline__ double block_sum_f64(double v, double* wtot)
{
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int nw = (blockDim.x + kWave - 1) >> 6;
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    __syncthreads();
    if (lane == 0) wtot[wv] = v;
    __syncthreads();
    double s = 0.0;
    for (int i = 0; i < nw; ++i) s += wtot[i];
    return s;
}

// doc part over LDS document tiles: one partial per tile
__global__ __launch_bounds__(1024) void loglik_doc_tiles_kernel(
    const int32_t* __restrict__ z, const int32_t* __restrict__ doff,
    const int32_t* __restrict__ chunk_doc, const uint8_t* __restrict__ tokdoc, int32_t cap_tokens,
    double alpha, double alphabar, double lg_alpha, double lg_alphabar,
    double* __restrict__ partial)
{
    extern __shared__ int32_t smem[];
    __shared__ double wtot[16];
    const int32_t c = blockIdx.x;
    const int32_t d0 = chunk_doc[c], d1 = chunk_doc[c + 1];
    double acc = 0.0;
    if (doff[d1] - doff[d0] <= cap_tokens) {
        const DocTile T = load_doc_tile(smem, cap_tokens, z, doff, tokdoc, d0, d1);
        for (int32_t i = threadIdx.x; i < T.nd; i += blockDim.x)
            acc += lg_alphabar - lgamma((double)(T.sdoff[i + 1] - T.sdoff[i]) + alphabar);
        for (int32_t i = threadIdx.x; i < 2 * T.ntok; i += blockDim.x) {
            const uint32_t v = T.tab[i];
            if (v != kEmptySlot) acc += lgamma((double)(v >> kTopicBits) + alpha) - lg_alpha;
        }
    }
    const double s = block_sum_f64(acc, wtot);
    if (threadIdx.x == 0) partial[c] = s;
}

__global__ __launch_bounds__(1024) void loglik_long_docs_kernel(
    const int32_t* __restrict__ z, const int32_t* __restrict__ doff,
    const int32_t* __restrict__ long_doc, const int64_t* __restrict__ long_slot, int32_t* keys,
    int32_t* cnts, double alpha, double alphabar, double lg_alpha, double lg_alphabar,
    double* __restrict__ partial)
{
    __shared__ double wtot[16];
    const int32_t d = long_doc[blockIdx.x];
    const int32_t tok0 = doff[d];
    const int32_t L = doff[d + 1] - tok0;
    const int64_t s0 = long_slot[blockIdx.x];
    const GlobalDocTable tab = load_long_doc(keys + s0, cnts + s0, z + tok0, L);
    double acc = 0.0;
    if (threadIdx.x == 0) acc += lg_alphabar - lgamma((double)L + alphabar);
    for (uint32_t i = threadIdx.x; i < tab.slots; i += blockDim.x)
        if (GlobalDocTable::ld(&tab.keys[i]) != kEmptyKey)
            acc += lgamma((double)GlobalDocTable::ld(&tab.cnts[i]) + alpha) - lg_alpha;
    const double s = block_sum_f64(acc, wtot);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// word part: grid-stride over the dense table, one partial per block
__global__ __launch_bounds__(256) void loglik_word_kernel(const int32_t* __restrict__ nkw,
                                                          int64_t total, double beta,
                                                          double lg_beta,
                                                          double* __restrict__ partial)
{
    __shared__ double wtot[4];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = nkw[i];
        if (v > 0) acc += lgamma((double)v + beta) - lg_beta;
    }
    const double s = block_sum_f64(acc, wtot);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

__global__ __launch_bounds__(256) void loglik_nk_kernel(const int32_t* __restrict__ nk, int32_t K,
                                                        double betabar, double lg_betabar,
                                                        double* __restrict__ partial)
{
    __shared__ double wtot[4];
    double acc = 0.0;
    for (int32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < K; k += gridDim.x * blockDim.x)
        acc += lg_betabar - lgamma((double)nk[k] + betabar);
    const double s = block_sum_f64(acc, wtot);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// word part over the sparse rows: one wave per word of the list, grid-stride
__global__ __launch_bounds__(256) void loglik_sparse_kernel(const int32_t* __restrict__ words,
                                                            int32_t n_words,
                                                            const uint32_t* __restrict__ sp_off,
                                                            const int32_t* __restrict__ sp_count,
                                                            const int32_t* __restrict__ sp_nnz,
                                                            double beta, double lg_beta,
                                                            double* __restrict__ partial)
{
    __shared__ double wtot[4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    double acc = 0.0;
    for (int32_t i = wave; i < n_words; i += nwaves) {
        const int32_t w = words[i];
        const int32_t nnz = sp_nnz[w];
        const int32_t* __restrict__ cnt = sp_count + sp_off[w];
        for (int32_t e = lane; e < nnz; e += kWave) acc += lgamma((double)cnt[e] + beta) - lg_beta;
    }
    const double s = block_sum_f64(acc, wtot);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// compensated (Neumaier) sum of the partials in index order
double host_sum(const std::vector<double>& v, size_t n)
{
    double s = 0.0, comp = 0.0;
    for (size_t i = 0; i < n; ++i) {
        const double x = v[i], t = s + x;
        comp += (fabs(s) >= fabs(x)) ? (s - t) + x : (x - t) + s;
        s = t;
    }
    return s + comp;
}

}  // namespace

int launch_loglik(lda_ctx* c, double* doc_part, double* word_part)
{
    const double lga = lgamma(c->alpha), lgab = lgamma(c->alphabar);
    const double lgb = lgamma(c->beta), lgbb = lgamma(c->betabar);
    std::vector<double> h((size_t)c->n_partial);
    double doc = 0.0, word = 0.0;

    if (c->n_chunks > 0) {
        const size_t lds = doc_tile_lds_bytes(c->chunk_tokens, c->chunk_docs);
        if (lds > 48 * 1024)
            LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(loglik_doc_tiles_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(loglik_doc_tiles_kernel, dim3(c->n_chunks), dim3(c->sweep_block), lds,
                           c->stream, c->d_z, c->d_doff, c->d_chunk_doc, c->d_tokdoc, c->chunk_tokens,
                           c->alpha, c->alphabar, lga, lgab, c->d_partial);
        LDA_HIP(c, hipGetLastError());
        LDA_HIP(c, hipMemcpyAsync(h.data(), c->d_partial, sizeof(double) * c->n_chunks,
                                  hipMemcpyDeviceToHost, c->stream));
        LDA_HIP(c, hipStreamSynchronize(c->stream));
        doc += host_sum(h, (size_t)c->n_chunks);
    }
    if (c->n_long > 0) {
        hipLaunchKernelGGL(loglik_long_docs_kernel, dim3(c->n_long), dim3(1024), 0, c->stream,
                           c->d_z, c->d_doff, c->d_long_doc, c->d_long_slot, c->d_long_keys,
                           c->d_long_cnts, c->alpha, c->alphabar, lga, lgab, c->d_partial);
        LDA_HIP(c, hipGetLastError());
        LDA_HIP(c, hipMemcpyAsync(h.data(), c->d_partial, sizeof(double) * c->n_long,
                                  hipMemcpyDeviceToHost, c->stream));
        LDA_HIP(c, hipStreamSynchronize(c->stream));
        doc += host_sum(h, (size_t)c->n_long);
    }
    {
        const int blocks = 4096;
        const int64_t dense_rows = c->hybrid ? c->H : c->V;
        if (dense_rows > 0) {
            hipLaunchKernelGGL(loglik_word_kernel, dim3(blocks), dim3(256), 0, c->stream, c->d_nkw,
                               dense_rows * (int64_t)c->K, c->beta, lgb, c->d_partial);
            LDA_HIP(c, hipGetLastError());
            LDA_HIP(c, hipMemcpyAsync(h.data(), c->d_partial, sizeof(double) * blocks,
                                      hipMemcpyDeviceToHost, c->stream));
            LDA_HIP(c, hipStreamSynchronize(c->stream));
            word += host_sum(h, blocks);
        }
        if (c->hybrid && c->n_sparse > 0) {
            hipLaunchKernelGGL(loglik_sparse_kernel, dim3(blocks), dim3(256), 0, c->stream,
                               c->d_sparse_words, c->n_sparse, c->d_sp_off, c->d_sp_count,
                               c->d_sp_nnz, c->beta, lgb, c->d_partial);
            LDA_HIP(c, hipGetLastError());
            LDA_HIP(c, hipMemcpyAsync(h.data(), c->d_partial, sizeof(double) * blocks,
                                      hipMemcpyDeviceToHost, c->stream));
            LDA_HIP(c, hipStreamSynchronize(c->stream));
            word += host_sum(h, blocks);
        }
        const int kb = 64;
        hipLaunchKernelGGL(loglik_nk_kernel, dim3(kb), dim3(256), 0, c->stream, c->d_nk, c->K,
                           c->betabar, lgbb, c->d_partial);
        LDA_HIP(c, hipGetLastError());
        LDA_HIP(c, hipMemcpyAsync(h.data(), c->d_partial, sizeof(double) * kb,
                                  hipMemcpyDeviceToHost, c->stream));
        LDA_HIP(c, hipStreamSynchronize(c->stream));
        word += host_sum(h, kb);
    }
    *doc_part = doc;
    *word_part = word;
    return LDA_OK;
}

}  // namespace lda
