// The fused cycle Metropolis-Hastings sweep (LightLDA Sec. 4.2-4.3, Eq. 6-13).
//
// Work is tiled by documents: a workgroup stages a run of consecutive documents
// in LDS (their snapshot z values and one n_kd hash table per document), so the
// whole document side of every step -- the doc-proposal's "copy the topic of a
// random token of the document" (Eq. 12) and the n_kd factors of the ratios --
// is served from LDS.  The word side (alias bin, n_kw, n_k) is gathered from
// HBM/L2.  Every token runs its mh_steps fused in registers and writes one int.
#include "common.hpp"
#include "doc_tile.hpp"

namespace lda {

struct SweepArgs {
    const int32_t* word;
    const int32_t* z;
    int32_t* znew;
    const int32_t* doff;
    const int32_t* chunk_doc;
    const int32_t* nkw;
    const int32_t* nk;
    const uint2* alias;
    const uint32_t* cap;
    int32_t K;
    int32_t mh_steps;
    int32_t mode;
    int32_t cap_tokens;
    double alpha, beta, alphabar, betabar;
    uint32_t seed_lo, seed_hi, sweep;
    // long documents
    const int32_t* long_doc;
    const int64_t* long_slot;
    int32_t* long_keys;
    int32_t* long_cnts;
};

// One token's chain.  `tab` answers n_kd lookups, zdoc[j] is the snapshot topic
// of the document's j-th token, L the document length.
template <class Table>
__device__ __forceinline__ int32_t mh_chain(const SweepArgs& A, const Table& tab,
                                            const int32_t* zdoc, int32_t L, int32_t w, uint32_t g,
                                            int32_t z0)
{
#pragma clang fp contract(off)
    const int32_t K = A.K;
    const int32_t* __restrict__ row = A.nkw + (size_t)w * (size_t)K;
    const uint2* __restrict__ arow = A.alias + (size_t)w * (size_t)K;
    const uint32_t capw = A.cap[w];
    int32_t s = z0;
    int32_t nds = tab.count(z0);
    int32_t nws = row[z0];
    int32_t nks = A.nk[z0];
    for (int32_t j = 0; j < A.mh_steps; ++j) {
        uint32_t x[4];
        philox4x32_10(g, 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
        const bool word_step = (A.mode == 0) ? ((j & 1) == 0) : (A.mode == 1);
        int32_t t;
        if (word_step) {
            // Fig. 2: uniform bin, uniform height, keep the bin or take its alias
            const uint32_t bin = mulhi32(x[0], (uint32_t)K);
            const uint32_t rr = mulhi32(x[1], capw);
            const uint2 e = arow[bin];
            t = (rr < e.x) ? (int32_t)bin : (int32_t)e.y;
        } else {
            // Eq. (9), (12): a random token of the document, or a uniform topic
            const double u0 = unit_open(x[0]);
            if (u0 * ((double)L + A.alphabar) < (double)L)
                t = zdoc[mulhi32(x[1], (uint32_t)L)];
            else
                t = (int32_t)mulhi32(x[1], (uint32_t)K);
        }
        if (t != s) {
            const int32_t ndt = tab.count(t);
            const int32_t nwt = row[t];
            const int32_t nkt = A.nk[t];
            const int32_t ms = (s == z0) ? 1 : 0;
            const int32_t mt = (t == z0) ? 1 : 0;
            // Eq. (4) ratio p(t)/p(s), the token removed at its snapshot topic
            double num = (double)(ndt - mt) + A.alpha;
            num = num * ((double)(nwt - mt) + A.beta);
            num = num * ((double)(nks - ms) + A.betabar);
            double den = (double)(nds - ms) + A.alpha;
            den = den * ((double)(nws - ms) + A.beta);
            den = den * ((double)(nkt - mt) + A.betabar);
            if (word_step) {  // Eq. (8): times p_w(s)/p_w(t)
                num = num * ((double)nws + A.beta);
                num = num * ((double)nkt + A.betabar);
                den = den * ((double)nwt + A.beta);
                den = den * ((double)nks + A.betabar);
            } else {          // Eq. (11): times p_d(s)/p_d(t)
                num = num * ((double)nds + A.alpha);
                den = den * ((double)ndt + A.alpha);
            }
            const double u = unit_open(x[2]);
            if (u * den < num) {
                s = t;
                nds = ndt;
                nws = nwt;
                nks = nkt;
            }
        }
    }
    return s;
}

__global__ __launch_bounds__(1024) void sweep_tiles_kernel(SweepArgs A)
{
    extern __shared__ int32_t smem[];
    const int32_t c = blockIdx.x;
    const int32_t d0 = A.chunk_doc[c], d1 = A.chunk_doc[c + 1];
    if (A.doff[d1] - A.doff[d0] > A.cap_tokens) return;  // a long document: other kernel
    const DocTile T = load_doc_tile(smem, A.cap_tokens, A.z, A.doff, d0, d1);
    for (int32_t i = threadIdx.x; i < T.ntok; i += blockDim.x) {
        const int32_t dl = find_doc(T.sdoff, T.nd, i);
        const int32_t b = T.sdoff[dl];
        const int32_t L = T.sdoff[dl + 1] - b;
        const uint32_t g = (uint32_t)(T.tok0 + i);
        A.znew[g] = mh_chain(A, T.table(dl), T.zs + b, L, A.word[g], g, T.zs[i]);
    }
}

__global__ __launch_bounds__(1024) void sweep_long_docs_kernel(SweepArgs A)
{
    const int32_t d = A.long_doc[blockIdx.x];
    const int32_t tok0 = A.doff[d];
    const int32_t L = A.doff[d + 1] - tok0;
    const int64_t s0 = A.long_slot[blockIdx.x];
    const DocTable<true> tab = load_long_doc(A.long_keys + s0, A.long_cnts + s0, A.z + tok0, L);
    for (int32_t i = threadIdx.x; i < L; i += blockDim.x) {
        const uint32_t g = (uint32_t)(tok0 + i);
        A.znew[g] = mh_chain(A, tab, A.z + tok0, L, A.word[g], g, A.z[g]);
    }
}

int launch_sweep(lda_ctx* c, int32_t mh_steps)
{
    SweepArgs A{};
    A.word = c->d_word; A.z = c->d_z; A.znew = c->d_znew; A.doff = c->d_doff;
    A.chunk_doc = c->d_chunk_doc; A.nkw = c->d_nkw; A.nk = c->d_nk; A.alias = c->d_alias;
    A.cap = c->d_cap; A.K = c->K; A.mh_steps = mh_steps; A.mode = c->opt.proposal_mode;
    A.cap_tokens = c->chunk_tokens;
    A.alpha = c->alpha; A.beta = c->beta; A.alphabar = c->alphabar; A.betabar = c->betabar;
    A.seed_lo = (uint32_t)c->seed; A.seed_hi = (uint32_t)(c->seed >> 32); A.sweep = c->sweep_index;
    A.long_doc = c->d_long_doc; A.long_slot = c->d_long_slot;
    A.long_keys = c->d_long_keys; A.long_cnts = c->d_long_cnts;
    const size_t lds = doc_tile_lds_bytes(c->chunk_tokens, c->chunk_docs);
    if (c->n_chunks > 0) {
        if (lds > 48 * 1024)
            LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_tiles_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(sweep_tiles_kernel, dim3(c->n_chunks), dim3(c->sweep_block), lds,
                           c->stream, A);
        LDA_HIP(c, hipGetLastError());
    }
    if (c->n_long > 0) {
        hipLaunchKernelGGL(sweep_long_docs_kernel, dim3(c->n_long), dim3(1024), 0, c->stream, A);
        LDA_HIP(c, hipGetLastError());
    }
    return LDA_OK;
}

// ---- n_kd accessor: the row exactly as the sweep kernels form it -------------------

__global__ __launch_bounds__(256) void ndk_row_tile_kernel(const int32_t* z, const int32_t* doff,
                                                           int32_t d, int32_t cap_tokens,
                                                           int32_t K, int32_t* row)
{
    extern __shared__ int32_t smem[];
    const DocTile T = load_doc_tile(smem, cap_tokens, z, doff, d, d + 1);
    const DocTable<false> tab = T.table(0);
    for (int32_t k = threadIdx.x; k < K; k += blockDim.x) row[k] = T.ntok > 0 ? tab.count(k) : 0;
}

__global__ __launch_bounds__(1024) void ndk_row_long_kernel(const int32_t* z, const int32_t* doff,
                                                            int32_t d, int32_t* keys,
                                                            int32_t* cnts, int32_t K, int32_t* row)
{
    const int32_t tok0 = doff[d];
    const int32_t L = doff[d + 1] - tok0;
    const DocTable<true> tab = load_long_doc(keys, cnts, z + tok0, L);
    for (int32_t k = threadIdx.x; k < K; k += blockDim.x) row[k] = tab.count(k);
}

int launch_ndk_row(lda_ctx* c, int64_t d)
{
    const int32_t L = c->h_doff[d + 1] - c->h_doff[d];
    if (L <= c->chunk_tokens) {
        const size_t lds = doc_tile_lds_bytes(c->chunk_tokens, c->chunk_docs);
        if (lds > 48 * 1024)
            LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(ndk_row_tile_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(ndk_row_tile_kernel, dim3(1), dim3(256), lds, c->stream, c->d_z,
                           c->d_doff, (int32_t)d, c->chunk_tokens, c->K, c->d_row);
    } else {
        // the d-th long document's workspace slice
        int64_t s0 = -1;
        std::vector<int64_t> slot(c->n_long + 1);
        LDA_HIP(c, hipMemcpy(slot.data(), c->d_long_slot, sizeof(int64_t) * (c->n_long + 1),
                             hipMemcpyDeviceToHost));
        for (int32_t i = 0; i < c->n_long; ++i)
            if (c->h_long_doc[i] == (int32_t)d) s0 = slot[i];
        if (s0 < 0) return fail(c, LDA_ERR_HIP, "long document %lld has no workspace", (long long)d);
        hipLaunchKernelGGL(ndk_row_long_kernel, dim3(1), dim3(1024), 0, c->stream, c->d_z,
                           c->d_doff, (int32_t)d, c->d_long_keys + s0, c->d_long_cnts + s0, c->K,
                           c->d_row);
    }
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
