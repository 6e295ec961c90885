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

__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int delta)
{
    const uint32_t lo = __shfl_up((uint32_t)v, delta, kWave);
    const uint32_t hi = __shfl_up((uint32_t)(v >> 32), delta, kWave);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, int lane)
{
    const uint32_t lo = __shfl((uint32_t)v, lane, kWave);
    const uint32_t hi = __shfl((uint32_t)(v >> 32), lane, kWave);
    return ((uint64_t)hi << 32) | lo;
}

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

__device__ __forceinline__ uint64_t wave_inclusive_scan_u64(uint64_t v, int lane)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint64_t o = shfl_up_u64(v, d);
        if (lane >= d) v += o;
    }
    return v;
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
// ascending order.  Masses are recomputed in every pass instead of being kept: the
// division is cheaper than the registers or LDS it would take.
__global__ __launch_bounds__(1024) void alias_dense_kernel(const int32_t* __restrict__ nkw,
                                                           const int32_t* __restrict__ nk,
                                                           int32_t K, double beta, double betabar,
                                                           uint2* __restrict__ alias,
                                                           uint32_t* __restrict__ cap)
{
    extern __shared__ unsigned char smem_raw[];
    // dx[0..A]   : Delta_a (exclusive deficit sums of the lights, dx[A] = total)
    // dx[K-b]    : X_b     (inclusive excess sums of the heavies), b = 0..B-1, A + B = K
    uint64_t* dx = reinterpret_cast<uint64_t*>(smem_raw);
    uint32_t* hidx = reinterpret_cast<uint32_t*>(dx + (K + 1));  // hidx[b] = bin of heavy b
    __shared__ uint64_t w_a[kMaxWaves], w_b[kMaxWaves];
    __shared__ uint32_t w_c[kMaxWaves];

    const int32_t w = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int32_t* __restrict__ row = nkw + (size_t)w * (size_t)K;
    uint2* __restrict__ out = alias + (size_t)w * (size_t)K;
    const int32_t S = (((K + nw - 1) / nw + kWave - 1) / kWave) * kWave;  // bins per wave
    const int32_t kb = wv * S;
    const int32_t ke = (kb + S < K) ? kb + S : K;

    // pass 1: Q0 and, for the usual case of no shift, Q
    uint64_t p0 = 0, p1 = 0;
    for (int32_t k = kb + lane; k < ke; k += kWave) {
        const uint64_t q0 = bin_q0(row, nk, k, beta, betabar);
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
            const uint64_t q = bin_q0(row, nk, k, beta, betabar) >> sh;
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
        uint64_t q = bin_q0(row, nk, k, beta, betabar) >> sh;
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
        const uint64_t dinc = wave_inclusive_scan_u64(light ? C - m : 0ull, lane);
        const uint64_t xinc = wave_inclusive_scan_u64(heavy ? m - C : 0ull, lane);
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
        d_run += shfl_u64(dinc, kWave - 1);
        x_run += shfl_u64(xinc, kWave - 1);
    }
    __syncthreads();

    // pass 4: pair them
    a_run = a_wave;
    b_run = b_wave;
    for (int32_t k0 = kb; k0 < ke; k0 += kWave) {
        const int32_t k = k0 + lane;
        const bool valid = k < ke;
        const uint64_t m = valid ? mass(k) : C;
        const bool light = valid && m < C;
        const uint64_t lmask = __ballot(light);
        const uint32_t la = rank_below(lmask);
        if (valid) {
            uint32_t split, al;
            if (light) {
                const uint64_t delta = dx[a_run + la];
                // first b in [0, B) with X_b > delta; X_{B-1} = total deficit > delta
                uint32_t lo = 0, hi = B - 1;
                while (lo < hi) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (dx[K - mid] > delta) hi = mid; else lo = mid + 1;
                }
                split = (uint32_t)m;
                al = hidx[lo];
            } else {
                const uint32_t b = b_run + ((uint32_t)lane - la);
                const uint64_t X = dx[K - b];
                // first a in [0, A] with Delta_a >= X; Delta_A = total excess >= X
                uint32_t lo = 0, hi = A;
                while (lo < hi) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (dx[mid] >= X) hi = mid; else lo = mid + 1;
                }
                const uint64_t sp = C + X - dx[lo];
                split = (uint32_t)sp;
                al = (sp < C) ? hidx[b + 1] : (uint32_t)k;
            }
            out[k] = make_uint2(split, al);
        }
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
    const size_t lds = sizeof(uint64_t) * ((size_t)K + 1) + sizeof(uint32_t) * (size_t)K;
    if (lds > 48 * 1024)
        LDA_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(alias_dense_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(alias_dense_kernel, dim3(c->V), dim3(nw * kWave), lds, c->stream, c->d_nkw,
                       c->d_nk, K, c->beta, c->betabar, c->d_alias, c->d_cap);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace lda
