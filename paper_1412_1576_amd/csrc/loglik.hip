// Log-likelihood log p(w, z | alpha, beta) of the collapsed LDA model, the
// convergence metric of LightLDA Sec. 7 (doc-likelihood + word-likelihood):
//   doc  = sum_d [ lgG(K a) - lgG(L_d + K a) + sum_{k: n_kd>0} (lgG(n_kd + a) - lgG(a)) ]
//   word = sum_k [ lgG(V b) - lgG(n_k + V b) ] + sum_{w,k: n_kw>0} (lgG(n_kw + b) - lgG(b))
// fp64 throughout; every block reduces in a fixed tree and writes one partial,
// the host adds the partials in index order with compensation.  Which slot of a document's
// hash table a topic lands in depends on the order in which the threads' inserts win, so the
// doc part is summed per token instead of per slot: the term of (document, topic) is added
// by the first token of the document that has the topic.  Every run adds the same terms in
// the same order and returns the same bits.
#include <algorithm>
#include <mutex>

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
    int32_t cap_docs, double alpha, double alphabar, double lg_alpha, double lg_alphabar,
    double* __restrict__ partial)
{
    extern __shared__ int32_t smem[];
    __shared__ double wtot[16];
    const int32_t c = blockIdx.x;
    const int32_t d0 = chunk_doc[c], d1 = chunk_doc[c + 1];
    double acc = 0.0;
    if (doff[d1] - doff[d0] <= cap_tokens) {
        const DocTile T = load_doc_tile(smem, cap_tokens, z, doff, tokdoc, d0, d1);
        // first[s] = the lowest token of the tile whose topic sits in slot s
        int32_t* first = smem + doc_tile_lds_bytes(cap_tokens, cap_docs) / sizeof(int32_t);
        for (int32_t i = threadIdx.x; i < 2 * T.ntok; i += blockDim.x) first[i] = 0x7FFFFFFF;
        __syncthreads();
        auto slot_of = [&](int32_t i) {
            const int32_t dl = tokdoc ? (int32_t)tokdoc[T.tok0 + i] : find_doc(T.sdoff, T.nd, i);
            return 2 * T.sdoff[dl] + (int32_t)(T.zs[i] >> kTopicBits);
        };
        for (int32_t i = threadIdx.x; i < T.ntok; i += blockDim.x) atomicMin(&first[slot_of(i)], i);
        __syncthreads();
        for (int32_t i = threadIdx.x; i < T.nd; i += blockDim.x)
            acc += lg_alphabar - lgamma((double)(T.sdoff[i + 1] - T.sdoff[i]) + alphabar);
        for (int32_t i = threadIdx.x; i < T.ntok; i += blockDim.x) {
            const int32_t s = slot_of(i);
            if (first[s] == i) acc += lgamma((double)(T.tab[s] >> kTopicBits) + alpha) - lg_alpha;
        }
    }
    const double s = block_sum_f64(acc, wtot);
    if (threadIdx.x == 0) partial[c] = s;
}

__global__ __launch_bounds__(1024) void loglik_long_docs_kernel(
    const int32_t* __restrict__ z, const int32_t* __restrict__ doff,
    const int32_t* __restrict__ long_doc, const int64_t* __restrict__ long_slot, int32_t* keys,
    int32_t* cnts, int32_t* first_all, double alpha, double alphabar, double lg_alpha,
    double lg_alphabar, double* __restrict__ partial)
{
    __shared__ double wtot[16];
    const int32_t d = long_doc[blockIdx.x];
    const int32_t tok0 = doff[d];
    const int32_t L = doff[d + 1] - tok0;
    const int64_t s0 = long_slot[blockIdx.x];
    const GlobalDocTable tab = load_long_doc(keys + s0, cnts + s0, z + tok0, L);
    // first[s] = the lowest token of the document whose topic sits in slot s
    int32_t* first = first_all + s0;
    for (uint32_t i = threadIdx.x; i < tab.slots; i += blockDim.x)
        __hip_atomic_store(&first[i], 0x7FFFFFFF, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    for (int32_t i = threadIdx.x; i < L; i += blockDim.x) atomicMin(&first[tab.slot_of(z[tok0 + i])], i);
    __syncthreads();
    double acc = 0.0;
    if (threadIdx.x == 0) acc += lg_alphabar - lgamma((double)L + alphabar);
    for (int32_t i = threadIdx.x; i < L; i += blockDim.x) {
        const uint32_t s = tab.slot_of(z[tok0 + i]);
        if (GlobalDocTable::ld(&first[s]) == i)
            acc += lgamma((double)GlobalDocTable::ld(&tab.cnts[s]) + alpha) - lg_alpha;
    }
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

// compensated (Neumaier) sum, terms added in the order given
struct CompensatedSum {
    double s = 0.0, comp = 0.0;
    void add(double x)
    {
        const double t = s + x;
        comp += (fabs(s) >= fabs(x)) ? (s - t) + x : (x - t) + s;
        s = t;
    }
    double value() const { return s + comp; }
};

// Sum of the n partials at d_partial in index order.  Staged through `host` (a buffer of
// host_cap doubles owned by the caller) a piece at a time, so the result does not depend on
// host_cap.  Waits for the stream.
int sum_partials(lda_ctx* c, const double* d_partial, size_t n, double* host, size_t host_cap,
                 double* out)
{
    CompensatedSum acc;
    for (size_t i0 = 0; i0 < n; i0 += host_cap) {
        const size_t m = (n - i0 < host_cap) ? n - i0 : host_cap;
        LDA_HIP(c, hipMemcpyAsync(host, d_partial + i0, sizeof(double) * m, hipMemcpyDeviceToHost,
                                  c->stream));
        LDA_HIP(c, hipStreamSynchronize(c->stream));
        for (size_t i = 0; i < m; ++i) acc.add(host[i]);
    }
    *out = acc.value();
    return LDA_OK;
}

// Scratch of lda_loglik_noalloc: the per-block partial sums of the kernels above.  One copy
// of the array per GPU, at an address that hipGetSymbolAddress reports for the current
// device; host code uses that address, never the array's name.
constexpr size_t kStaticPartials = (size_t)1 << 20;  // 8 MB
static __device__ __align__(256) double g_static_partials[kStaticPartials];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};

// Device address of g_static_partials on the current device (looked up once per device).
int static_partials(lda_ctx* c, double** out)
{
    int dev = -1;
    LDA_HIP(c, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(c, LDA_ERR_UNSUPPORTED, "lda_loglik_noalloc: device index %d", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        LDA_HIP(c, hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_partials)));
        if (!p) return fail(c, LDA_ERR_HIP, "lda_loglik_noalloc: no address for the static scratch");
        g_scratch_ptr[dev] = static_cast<double*>(p);
    }
    *out = g_scratch_ptr[dev];
    return LDA_OK;
}

// The log-likelihood with the partial sums in d_partial (device memory of at least
// max(n_chunks, n_long, 4096) doubles) and host staging in `h` (h_cap doubles).
int run_loglik(lda_ctx* c, double* d_partial, double* h, size_t h_cap, double* doc_part,
               double* word_part)
{
    const double lga = lgamma(c->alpha), lgab = lgamma(c->alphabar);
    const double lgb = lgamma(c->beta), lgbb = lgamma(c->betabar);
    double doc = 0.0, word = 0.0, part = 0.0;
    int rc;

    if (c->n_chunks > 0) {
        rc = c->streamed ? launch_loglik_doc_streamed(c, d_partial) : launch_loglik_doc_tiles(c, d_partial);
        if (rc != LDA_OK) return rc;
        if ((rc = sum_partials(c, d_partial, (size_t)c->n_chunks, h, h_cap, &part)) != LDA_OK) return rc;
        doc += part;
    }
    if (c->n_long > 0) {
        hipLaunchKernelGGL(loglik_long_docs_kernel, dim3(c->n_long), dim3(1024), 0, c->stream,
                           c->d_z, c->d_doff, c->d_long_doc, c->d_long_slot, c->d_long_keys,
                           c->d_long_cnts, c->d_long_first, c->alpha, c->alphabar, lga, lgab, d_partial);
        LDA_HIP(c, hipGetLastError());
        if ((rc = sum_partials(c, d_partial, (size_t)c->n_long, h, h_cap, &part)) != LDA_OK) return rc;
        doc += part;
    }
    {
        const int blocks = 4096;
        const int64_t dense_rows = c->hybrid ? c->H : c->V;
        if (dense_rows > 0) {
            hipLaunchKernelGGL(loglik_word_kernel, dim3(blocks), dim3(256), 0, c->stream, c->d_nkw,
                               dense_rows * (int64_t)c->K, c->beta, lgb, d_partial);
            LDA_HIP(c, hipGetLastError());
            if ((rc = sum_partials(c, d_partial, blocks, h, h_cap, &part)) != LDA_OK) return rc;
            word += part;
        }
        if (c->hybrid && c->n_sparse > 0) {
            hipLaunchKernelGGL(loglik_sparse_kernel, dim3(blocks), dim3(256), 0, c->stream,
                               c->d_sparse_words, c->n_sparse, c->d_sp_off, c->d_sp_count,
                               c->d_sp_nnz, c->beta, lgb, d_partial);
            LDA_HIP(c, hipGetLastError());
            if ((rc = sum_partials(c, d_partial, blocks, h, h_cap, &part)) != LDA_OK) return rc;
            word += part;
        }
        const int kb = 64;
        hipLaunchKernelGGL(loglik_nk_kernel, dim3(kb), dim3(256), 0, c->stream, c->d_nk, c->K,
                           c->betabar, lgbb, d_partial);
        LDA_HIP(c, hipGetLastError());
        if ((rc = sum_partials(c, d_partial, kb, h, h_cap, &part)) != LDA_OK) return rc;
        word += part;
    }
    *doc_part = doc;
    *word_part = word;
    return LDA_OK;
}

}  // namespace

// doc part of the tiles the context's token arrays are bound to: partial[tile]
int launch_loglik_doc_tiles(lda_ctx* c, double* d_partial)
{
    const double lga = lgamma(c->alpha), lgab = lgamma(c->alphabar);
    const size_t lds = doc_tile_lds_bytes(c->chunk_tokens, c->chunk_docs) +
                       sizeof(int32_t) * 2 * (size_t)c->chunk_tokens;
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(loglik_doc_tiles_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(loglik_doc_tiles_kernel, dim3(c->n_chunks), dim3(c->sweep_block), lds, c->stream,
                       c->d_z, c->d_doff, c->d_chunk_doc, c->d_tokdoc, c->chunk_tokens, c->chunk_docs,
                       c->alpha, c->alphabar, lga, lgab, d_partial);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

int launch_loglik(lda_ctx* c, double* doc_part, double* word_part)
{
    std::vector<double> h((size_t)c->n_partial);
    return run_loglik(c, c->d_partial, h.data(), h.size(), doc_part, word_part);
}

}  // namespace lda

using namespace lda;

extern "C" int lda_loglik_noalloc(lda_ctx* c, double* total, double* doc_part, double* word_part)
{
    if (!c) return LDA_ERR_ARG;
    if (!total) return fail(c, LDA_ERR_ARG, "lda_loglik_noalloc: total is NULL");
    if (c->state != COUNTS_VALID && c->state != ALIAS_VALID)
        return fail(c, LDA_ERR_STATE, "lda_loglik_noalloc: counts are stale (call lda_rebuild_counts)");
    const size_t need = (size_t)std::max(std::max(c->n_chunks, c->n_long), 4096);
    if (need > kStaticPartials)
        return fail(c, LDA_ERR_UNSUPPORTED,
                    "lda_loglik_noalloc: %zu partial sums (one per document tile) exceed the static "
                    "scratch of %zu; use lda_loglik", need, kStaticPartials);
    double* scratch = nullptr;
    int rc = static_partials(c, &scratch);
    if (rc != LDA_OK) return rc;
    double staging[2048];  // host side: on the stack
    double d = 0.0, w = 0.0;
    rc = run_loglik(c, scratch, staging, sizeof(staging) / sizeof(staging[0]), &d, &w);
    if (rc != LDA_OK) return rc;
    if (doc_part) *doc_part = d;
    if (word_part) *word_part = w;
    *total = d + w;
    return LDA_OK;
}
