// Word-proposal alias tables (LightLDA Sec. 4.2, Eq. 6, Fig. 2), one workgroup
// per word.
//
// The table is defined on integers so that this parallel build is exact:
//   a_k  = (n_kw + beta) / (n_k + betabar)                  (fp64, one division)
//   q0_k = floor(a_k * 2^40),  Q0 = sum q0_k
//   sh   = smallest shift with (Q0 >> sh) < K * 2^31
//   q_k  = max(1, q0_k >> sh), Q = sum q_k, C = ceil(Q / K), pad = K*C - Q
//   m_k  = q_k + (k < pad)                                   (sum m_k = K*C)
// Bins with m_k < C ("lights", ascending k, exclusive deficit sums Delta_a) are
// topped up by bins with m_k >= C ("heavies", ascending k, inclusive excess sums
// X_b).  Pairing the two ascending lists greedily has the closed form
//   light a : split = m,  alias = heavy b with b = min{b : X_b > Delta_a}
//   heavy b : a = min{a : Delta_a >= X_b}, split = C + X_b - Delta_a,
//             alias = next heavy if split < C, else itself
// so the build is prefix sums over the two lists and one binary search per bin.
#include "common.hpp"

namespace lda {

namespace {

constexpr int kMaxWaves = 16;

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v)
{
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, d, kWave);
        const uint32_t hi = __shfl_xor((uint32_t)(v >> 32), d, kWave);
        v += ((uint64_t)hi << 32) | lo;
    }
    return v;
}

// Inclusive prefix sum over the 64 lanes with DPP row shifts and row broadcasts
// (no LDS traffic): shifts by 1, 2, 3 of the input, then 4 and 8 inside each row of
// 16 lanes, then the last lane of row 0 / 2 into row 1 / 3 and lane 31 into rows 2, 3.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t v)
{
    const int x = (int)v;
    int r = x;
    r += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);  // row_shr:1
    r += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);  // row_shr:2
    r += __builtin_amdgcn_update_dpp(0, x, 0x113, 0xf, 0xf, false);  // row_shr:3
    r += __builtin_amdgcn_update_dpp(0, r, 0x114, 0xf, 0xe, false);  // row_shr:4, lanes 4..15
    r += __builtin_amdgcn_update_dpp(0, r, 0x118, 0xf, 0xc, false);  // row_shr:8, lanes 8..15
    r += __builtin_amdgcn_update_dpp(0, r, 0x142, 0xa, 0xf, false);  // row_bcast:15 -> rows 1, 3
    r += __builtin_amdgcn_update_dpp(0, r, 0x143, 0xc, 0xf, false);  // row_bcast:31 -> rows 2, 3
    return (uint32_t)r;
}

// 64-bit inclusive prefix sum of values < 2^46: the low 26 bits and the rest are
// summed separately (64 terms cannot overflow 32 bits) and recombined.
__device__ __forceinline__ uint64_t wave_inclusive_scan_u64(uint64_t v)
{
    const uint32_t lo = wave_inclusive_scan_u32((uint32_t)v & 0x3FFFFFFu);
    const uint32_t hi = wave_inclusive_scan_u32((uint32_t)(v >> 26));
    return ((uint64_t)hi << 26) + (uint64_t)lo;
}

__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int lane)
{
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// First index in [lo, hi] at which the monotone predicate holds; pred(hi) is known
// to hold.  lo, hi are wave-uniform and all 64 lanes take part: a window of 64
// consecutive indices first (partners of neighbouring bins are close), then 64-ary
// narrowing of what is left.
template <class Pred>
__device__ __forceinline__ uint32_t wave_first_true(uint32_t lo, uint32_t hi, int lane, Pred pred)
{
    {
        const uint32_t top = (hi - lo > 63u) ? lo + 63u : hi;
        uint32_t idx = lo + (uint32_t)lane;
        if (idx > top) idx = top;
        const uint64_t mask = __ballot(pred(idx));
        if (mask != 0) return lo + (uint32_t)(__ffsll((unsigned long long)mask) - 1);
        lo = top + 1;  // top < hi here, because pred(hi) holds
    }
    for (;;) {
        const uint32_t step = (hi - lo) / 63u + 1u;
        uint32_t idx = lo + (uint32_t)lane * step;
        if (idx > hi) idx = hi;
        const uint64_t mask = __ballot(pred(idx));  // lane 63 sits on hi: never empty
        const uint32_t f = (uint32_t)(__ffsll((unsigned long long)mask) - 1);
        const uint32_t cand = lo + f * step;
        if (step == 1u) return cand < hi ? cand : hi;
        hi = cand < hi ? cand : hi;
        if (f > 0) lo = lo + (f - 1u) * step + 1u;
    }
}

// number of set bits of `mask` below this lane
__device__ __forceinline__ uint32_t rank_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// floor(a_k * 2^40) for bin k of the word: the only floating-point step
__device__ __forceinline__ uint64_t bin_q0(const int32_t* __restrict__ row,
                                           const int32_t* __restrict__ nk, int32_t k, double beta,
                                           double betabar)
{
#pragma clang fp contract(off)
    const double a = ((double)row[k] + beta) / ((double)nk[k] + betabar);
    return (uint64_t)floor(a * 1099511627776.0);
}

// One workgroup per word.  Wave v owns the contiguous bins [v*S, (v+1)*S), visited
// 64 at a time, so global loads and stores are coalesced and bins are met in
// ascending order.  The quantised weights are kept in LDS as 32-bit values when
// the table leaves room (recomputed by division when they do not fit).
__global__ __launch_bounds__(1024) void alias_dense_kernel(const int32_t* __restrict__ nkw,
                                                           const int32_t* __restrict__ nk,
                                                           int32_t K, double beta, double betabar,
                                                           uint4* __restrict__ alias,
                                                           uint32_t* __restrict__ cap,
                                                           int32_t use_cache)
{
    extern __shared__ unsigned char smem_raw[];
    // dx[0..A]   : Delta_a (exclusive deficit sums of the lights, dx[A] = total)
    // dx[K-b]    : X_b     (inclusive excess sums of the heavies), b = 0..B-1, A + B = K
    uint64_t* dx = reinterpret_cast<uint64_t*>(smem_raw);
    uint32_t* hidx = reinterpret_cast<uint32_t*>(dx + (K + 1));  // hidx[b] = bin of heavy b
    // qc[k] = q0_k saturated to 32 bits, kept for the later passes when LDS has room
    // (0xFFFFFFFF: does not fit, recompute)
    uint32_t* qc = hidx + K;
    __shared__ uint64_t w_a[kMaxWaves], w_b[kMaxWaves];
    __shared__ uint32_t w_c[kMaxWaves];

    const int32_t w = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int32_t* __restrict__ row = nkw + (size_t)w * (size_t)K;
    uint4* __restrict__ out = alias + (size_t)w * (size_t)K;
    const int32_t S = (((K + nw - 1) / nw + kWave - 1) / kWave) * kWave;  // bins per wave
    const int32_t kb = wv * S;
    const int32_t ke = (kb + S < K) ? kb + S : K;

    // pass 1: Q0 and, for the usual case of no shift, Q
    uint64_t p0 = 0, p1 = 0;
#pragma unroll 4
    for (int32_t k = kb + lane; k < ke; k += kWave) {
        const uint64_t q0 = bin_q0(row, nk, k, beta, betabar);
        if (use_cache) qc[k] = (q0 < 0xFFFFFFFFull) ? (uint32_t)q0 : 0xFFFFFFFFu;
        p0 += q0;
        p1 += (q0 < 1) ? 1 : q0;
    }
    p0 = wave_sum_u64(p0);
    p1 = wave_sum_u64(p1);
    if (lane == 0) { w_a[wv] = p0; w_b[wv] = p1; }
    __syncthreads();
    uint64_t Q0 = 0, Q = 0;
    for (int i = 0; i < nw; ++i) { Q0 += w_a[i]; Q += w_b[i]; }
    int sh = 0;
    while ((Q0 >> sh) >= ((uint64_t)K << 31)) ++sh;
    if (sh > 0) {  // uniform over the block
        p1 = 0;
        for (int32_t k = kb + lane; k < ke; k += kWave) {
            uint64_t q = use_cache ? (uint64_t)qc[k] : 0xFFFFFFFFull;
            if (q == 0xFFFFFFFFull) q = bin_q0(row, nk, k, beta, betabar);
            q >>= sh;
            p1 += (q < 1) ? 1 : q;
        }
        p1 = wave_sum_u64(p1);
        __syncthreads();
        if (lane == 0) w_b[wv] = p1;
        __syncthreads();
        Q = 0;
        for (int i = 0; i < nw; ++i) Q += w_b[i];
    }
    const uint64_t C = (Q + (uint64_t)K - 1) / (uint64_t)K;
    const uint64_t pad = (uint64_t)K * C - Q;
    auto mass = [&](int32_t k) -> uint64_t {
        uint64_t q = use_cache ? (uint64_t)qc[k] : 0xFFFFFFFFull;
        if (q == 0xFFFFFFFFull) q = bin_q0(row, nk, k, beta, betabar);
        q >>= sh;
        if (q < 1) q = 1;
        return q + (((uint64_t)k < pad) ? 1u : 0u);
    };

    // pass 2: per-wave totals (lights, their deficit, the heavies' excess)
    uint32_t lc = 0;
    uint64_t df = 0, ex = 0;
    for (int32_t k = kb + lane; k < ke; k += kWave) {
        const uint64_t m = mass(k);
        if (m < C) { lc += 1; df += C - m; } else { ex += m - C; }
    }
    df = wave_sum_u64(df);
    ex = wave_sum_u64(ex);
    lc = (uint32_t)wave_sum_u64(lc);
    __syncthreads();  // w_a / w_b of pass 1 are no longer read
    if (lane == 0) { w_a[wv] = df; w_b[wv] = ex; w_c[wv] = lc; }
    __syncthreads();
    uint32_t a_run = 0, A = 0;
    uint64_t d_run = 0, x_run = 0, d_tot = 0;
    for (int i = 0; i < nw; ++i) {
        if (i < wv) { a_run += w_c[i]; d_run += w_a[i]; x_run += w_b[i]; }
        A += w_c[i];
        d_tot += w_a[i];
    }
    const uint32_t B = (uint32_t)K - A;
    uint32_t b_run = (uint32_t)kb - a_run;
    if (threadIdx.x == 0) {
        dx[A] = d_tot;
        cap[w] = (uint32_t)C;
    }
    const uint32_t a_wave = a_run, b_wave = b_run;

    // pass 3: the two ascending lists with their running sums
    for (int32_t k0 = kb; k0 < ke; k0 += kWave) {
        const int32_t k = k0 + lane;
        const bool valid = k < ke;
        const uint64_t m = valid ? mass(k) : C;
        const bool light = valid && m < C;
        const bool heavy = valid && !light;
        const uint64_t lmask = __ballot(light);
        const uint64_t dinc = wave_inclusive_scan_u64(light ? C - m : 0ull);
        const uint64_t xinc = wave_inclusive_scan_u64(heavy ? m - C : 0ull);
        const uint32_t la = rank_below(lmask);
        if (light) {
            dx[a_run + la] = d_run + dinc - (C - m);
        } else if (heavy) {
            const uint32_t b = b_run + ((uint32_t)lane - la);
            dx[K - b] = x_run + xinc;
            hidx[b] = (uint32_t)k;
        }
        const uint32_t nl = (uint32_t)__popcll(lmask);
        const uint32_t nv = (uint32_t)((ke - k0 < kWave) ? ke - k0 : kWave);
        a_run += nl;
        b_run += nv - nl;
        d_run += readlane_u64(dinc, kWave - 1);
        x_run += readlane_u64(xinc, kWave - 1);
    }
    __syncthreads();

    // pass 4: pair them.  Within a wave the ranks of one kind only grow and the
    // partner index is monotone in the rank.  Per round the whole wave searches the
    // partner of the last light (heavy) starting from the previous round's result;
    // every lane then searches only between those two bounds.
    a_run = a_wave;
    b_run = b_wave;
    uint32_t b_prev = 0;  // partner of the last light met so far
    uint32_t a_prev = 0;  // partner of the last heavy met so far
    for (int32_t k0 = kb; k0 < ke; k0 += kWave) {
        const int32_t k = k0 + lane;
        const bool valid = k < ke;
        const uint64_t m = valid ? mass(k) : C;
        const bool light = valid && m < C;
        const bool heavy = valid && !light;
        const uint64_t lmask = __ballot(light);
        const uint64_t hmask = __ballot(heavy);
        const uint32_t la = rank_below(lmask);
        const uint32_t b_own = b_run + ((uint32_t)lane - la);
        // own list entry: Delta_a of a light, X_b of a heavy
        uint64_t own = 0;
        if (light) own = dx[a_run + la];
        if (heavy) own = dx[K - b_own];
        uint32_t b_hi = b_prev, a_hi = a_prev;
        if (lmask != 0) {  // uniform
            const uint64_t delta_last = readlane_u64(own, 63 - __clzll((unsigned long long)lmask));
            // first b with X_b > delta; X_{B-1} = total deficit > every delta
            b_hi = wave_first_true(b_prev, B - 1, lane,
                                   [&](uint32_t i) { return dx[K - i] > delta_last; });
        }
        if (hmask != 0) {  // uniform
            const uint64_t x_last = readlane_u64(own, 63 - __clzll((unsigned long long)hmask));
            // first a with Delta_a >= X; Delta_A = total excess >= every X
            a_hi = wave_first_true(a_prev, A, lane, [&](uint32_t i) { return dx[i] >= x_last; });
        }
        uint32_t split = 0, al = 0;
        if (light) {
            uint32_t lo = b_prev, hi = b_hi;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (dx[K - mid] > own) hi = mid; else lo = mid + 1;
            }
            split = (uint32_t)m;
            al = hidx[lo];
        } else if (heavy) {
            uint32_t lo = a_prev, hi = a_hi;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (dx[mid] >= own) hi = mid; else lo = mid + 1;
            }
            const uint64_t sp = C + own - dx[lo];
            split = (uint32_t)sp;
            al = (sp < C) ? hidx[b_own + 1] : (uint32_t)k;
        }
        // the bin also carries the counts of its two outcomes for the sweep's accept test
        if (valid) out[k] = make_uint4(split, al, (uint32_t)row[k], (uint32_t)row[al]);
        b_prev = b_hi;
        a_prev = a_hi;
        const uint32_t nl = (uint32_t)__popcll(lmask);
        const uint32_t nv = (uint32_t)((ke - k0 < kWave) ? ke - k0 : kWave);
        a_run += nl;
        b_run += nv - nl;
    }
}

}  // namespace

int max_alias_topics() { return 12 * 1024; }

int launch_alias_build(lda_ctx* c)
{
    const int32_t K = c->K;
    if (K > max_alias_topics())
        return fail(c, LDA_ERR_UNSUPPORTED, "dense alias build supports K <= %d", max_alias_topics());
    int nw = (K + kWave - 1) / kWave;
    if (nw > kMaxWaves) nw = kMaxWaves;
    size_t lds = sizeof(uint64_t) * ((size_t)K + 1) + sizeof(uint32_t) * (size_t)K;
    // room for the 4-byte mass cache next to the lists?  (160 KiB of LDS per workgroup)
    const size_t lds_limit = 160 * 1024 - 1024;
    const int32_t use_cache = (lds + sizeof(uint32_t) * (size_t)K <= lds_limit) ? 1 : 0;
    if (use_cache) lds += sizeof(uint32_t) * (size_t)K;
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(alias_dense_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(alias_dense_kernel, dim3(c->V), dim3(nw * kWave), lds, c->stream, c->d_nkw,
                       c->d_nk, K, c->beta, c->betabar, c->d_alias, c->d_cap, use_cache);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
