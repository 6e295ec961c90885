// Sweep with the doc side refreshed after every token (LightLDA Sec. 4.2, footnote 4: the
// doc-proposal is not frozen during a document but follows its assignments token by token) and the word side -- n_kw, n_k, the word-proposal tables -- kept at the snapshot
// (Sec. 6, the immutable model slice).  Selected by lda_options.doc_refresh.
//
// The tokens of a document are visited in order, so a document is a sequential chain; the
// documents are independent.  One wave per document: the document's current assignment sits
// in the wave's part of the LDS, n_kd of a topic is a ballot count over it, and everything
// that does not depend on the document's state -- the Philox numbers of every step, the
// word-proposal draws with their n_kw and n_k -- is computed 64 tokens at a time, one token
// per lane, before those tokens take their turns one after the other.
#include <algorithm>

#include "common.hpp"

namespace lda {

namespace {

constexpr int kRefreshWaves = 4;           // documents per workgroup
constexpr int32_t kRefreshMaxDoc = 4096;   // tokens of the longest document (16 KB of LDS per wave)

struct RefreshArgs {
    const int32_t* word;
    const int32_t* z;
    int32_t* znew;
    const int32_t* doff;
    const int32_t* nkw;
    const int32_t* nk;
    const uint4* alias;  // (split, alias, n_kw[bin], n_kw[alias]) per bin
    const uint32_t* cap;
    int32_t D, K, mode, lds_doc;
    double alpha, beta, alphabar, betabar;
    uint32_t seed_lo, seed_hi, sweep;
};

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// n_kd of topic k in the document whose current assignment is zs[0..L): every lane gets it
__device__ __forceinline__ int32_t doc_count(const int32_t* zs, int32_t L, int lane, int32_t k)
{
    int32_t c = 0;
    for (int32_t b = 0; b < L; b += 64) {
        const int32_t v = (b + lane < L) ? zs[b + lane] : -1;
        c += (int32_t)__popcll(__ballot(v == k));
    }
    return c;
}

template <int M>
__global__ __launch_bounds__(64 * kRefreshWaves) void sweep_doc_refresh_kernel(RefreshArgs A)
{
#pragma clang fp contract(off)
    extern __shared__ int32_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int32_t d = (int32_t)blockIdx.x * kRefreshWaves + wave;
    if (d >= A.D) return;  // a whole wave leaves; no workgroup barrier follows
    const int32_t b = A.doff[d], L = A.doff[d + 1] - b;
    if (L == 0) return;
    int32_t* __restrict__ zs = smem + (size_t)wave * A.lds_doc;
    for (int32_t i = lane; i < L; i += 64) zs[i] = A.z[b + i];
    wave_lds_sync();
    const int32_t K = A.K;
    const double Ld = (double)L;
    for (int32_t base = 0; base < L; base += 64) {
        // ---- one token per lane: what its chain needs from the snapshot ----
        const int32_t i = (base + lane < L) ? base + lane : L - 1;  // lanes past the end: a clone
        const uint32_t g = (uint32_t)(b + i);
        const int32_t w = A.word[g];
        const int32_t z0 = A.z[g];
        const size_t wk = (size_t)w * (size_t)K;
        const uint32_t capw = A.cap[w];
        const int32_t nw_z0 = A.nkw[wk + (size_t)z0];
        const int32_t nk_z0 = A.nk[z0];
        uint32_t x0[M], x1[M], x2[M];
        int32_t tw[M], nwt[M], nkt[M];
#pragma unroll
        for (int j = 0; j < M; ++j) {
            const bool word_step = (A.mode == 0) ? ((j & 1) == 0) : (A.mode == 1);
            uint32_t x[4];
            philox4x32_10(g, 0u, A.sweep, (uint32_t)j, A.seed_lo, A.seed_hi, x);
            x0[j] = x[0]; x1[j] = x[1]; x2[j] = x[2];
            tw[j] = 0; nwt[j] = 0; nkt[j] = 0;
            if (word_step) {  // Fig. 2: uniform bin, uniform height, keep the bin or take its alias
                const uint32_t bin = mulhi32(x[0], (uint32_t)K);
                const uint32_t rr = mulhi32(x[1], capw);
                const uint4 e = A.alias[wk + bin];
                const bool keep = rr < e.x;
                tw[j] = keep ? (int32_t)bin : (int32_t)e.y;
                nwt[j] = keep ? (int32_t)e.z : (int32_t)e.w;
                nkt[j] = A.nk[tw[j]];
            }
        }
        // ---- the tokens take their turns ----
        const int32_t turns = (L - base < 64) ? L - base : 64;
        for (int32_t q = 0; q < turns; ++q) {
            const int32_t z0q = __shfl(z0, q, 64);
            const size_t wkq = (size_t)__shfl(w, q, 64) * (size_t)K;
            int32_t s = z0q;
            int32_t nds = doc_count(zs, L, lane, z0q);
            int32_t nws = __shfl(nw_z0, q, 64);
            int32_t nks = __shfl(nk_z0, q, 64);
#pragma unroll
            for (int j = 0; j < M; ++j) {
                const bool word_step = (A.mode == 0) ? ((j & 1) == 0) : (A.mode == 1);
                int32_t t, nw_t, nk_t;
                if (word_step) {
                    t = __shfl(tw[j], q, 64);
                    nw_t = __shfl(nwt[j], q, 64);
                    nk_t = __shfl(nkt[j], q, 64);
                } else {  // Eq. (9), (12) on the document as it stands now
                    const double u0 = unit_open(__shfl(x0[j], q, 64));
                    const uint32_t x1q = __shfl(x1[j], q, 64);
                    if (u0 * (Ld + A.alphabar) < Ld) t = zs[mulhi32(x1q, (uint32_t)L)];
                    else t = (int32_t)mulhi32(x1q, (uint32_t)K);
                    nw_t = A.nkw[wkq + (size_t)t];
                    nk_t = A.nk[t];
                }
                const int32_t nd_t = doc_count(zs, L, lane, t);
                const int32_t ms = (s == z0q) ? 1 : 0;
                const int32_t mt = (t == z0q) ? 1 : 0;
                // Eq. (4) ratio p(t)/p(s), the token removed at its snapshot topic
                double num = (double)(nd_t - mt) + A.alpha;
                num = num * ((double)(nw_t - mt) + A.beta);
                num = num * ((double)(nks - ms) + A.betabar);
                double den = (double)(nds - ms) + A.alpha;
                den = den * ((double)(nws - ms) + A.beta);
                den = den * ((double)(nk_t - mt) + A.betabar);
                if (word_step) {  // Eq. (8): times p_w(s)/p_w(t)
                    num = num * ((double)nws + A.beta);
                    num = num * ((double)nk_t + A.betabar);
                    den = den * ((double)nw_t + A.beta);
                    den = den * ((double)nks + A.betabar);
                } else {          // Eq. (11): times p_d(s)/p_d(t)
                    num = num * ((double)nds + A.alpha);
                    den = den * ((double)nd_t + A.alpha);
                }
                const double uu = unit_open(__shfl(x2[j], q, 64));
                const bool accept = (t != s) && (uu * den < num);
                s = accept ? t : s;
                nds = accept ? nd_t : nds;
                nws = accept ? nw_t : nws;
                nks = accept ? nk_t : nks;
            }
            if (lane == 0) {
                zs[base + q] = s;  // the rest of the document sees the move
                A.znew[b + base + q] = s;
            }
            wave_lds_sync();
        }
    }
}

}  // namespace

int refresh_sweep_max_doc() { return kRefreshMaxDoc; }

int launch_sweep_doc_refresh(lda_ctx* c, int32_t mh_steps, int32_t longest_doc)
{
    if (c->hybrid)
        return fail(c, LDA_ERR_UNSUPPORTED, "lda_sweep with doc_refresh needs the all-dense store");
    if (mh_steps > 4)
        return fail(c, LDA_ERR_UNSUPPORTED, "lda_sweep with doc_refresh: at most 4 steps");
    RefreshArgs A{};
    A.word = c->d_word; A.z = c->d_z; A.znew = c->d_znew; A.doff = c->d_doff;
    A.nkw = c->d_nkw; A.nk = c->d_nk; A.alias = c->d_alias; A.cap = c->d_cap;
    A.D = (int32_t)c->D; A.K = c->K; A.mode = c->opt.proposal_mode;
    A.lds_doc = std::max(64, (longest_doc + 63) / 64 * 64);
    A.alpha = c->alpha; A.beta = c->beta; A.alphabar = c->alphabar; A.betabar = c->betabar;
    A.seed_lo = (uint32_t)c->seed; A.seed_hi = (uint32_t)(c->seed >> 32); A.sweep = c->sweep_index;
    const size_t lds = sizeof(int32_t) * (size_t)kRefreshWaves * (size_t)A.lds_doc;
    const dim3 grid((unsigned)((c->D + kRefreshWaves - 1) / kRefreshWaves)), block(64 * kRefreshWaves);
#define LDA_REFRESH(M)                                                                              \
    do {                                                                                            \
        if (lds > 48 * 1024)                                                                        \
            LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_doc_refresh_kernel<M>), \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));  \
        hipLaunchKernelGGL(sweep_doc_refresh_kernel<M>, grid, block, lds, c->stream, A);            \
    } while (0)
    if (mh_steps == 1) LDA_REFRESH(1);
    else if (mh_steps == 2) LDA_REFRESH(2);
    else if (mh_steps == 3) LDA_REFRESH(3);
    else LDA_REFRESH(4);
#undef LDA_REFRESH
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
