// Generic alias-table builder (LightLDA Sec. 4.2, Fig. 2) for one workgroup.
//
// The table is defined on integers so that a parallel build is exact.  Given the
// quantised weights q0_i = floor(weight_i * 2^40) of n entries:
//   Q0 = sum q0_i,  sh = smallest shift with (Q0 >> sh) < n * 2^31
//   q_i = max(1, q0_i >> sh), Q = sum q_i, C = ceil(Q / n), pad = n*C - Q
//   m_i = q_i + (i < pad)                                    (sum m_i = n*C)
// Entries with m_i < C ("lights", ascending i, exclusive deficit sums Delta_a) are
// topped up by entries with m_i >= C ("heavies", ascending i, inclusive excess sums
// X_b).  Pairing the two ascending lists greedily has the closed form
//   light a : split = m,  alias = heavy b with b = min{b : X_b > Delta_a}
//   heavy b : a = min{a : Delta_a >= X_b}, split = C + X_b - Delta_a,
//             alias = next heavy if split < C, else itself
// so the build is prefix sums over the two lists and bounded searches.
//
// Src supplies q0(i); Sink gathers what entry i's output needs (load) and writes the
// entry (store), once per entry.  The
// working lists live either in LDS or, for tables too large for it, in a global
// workspace private to the workgroup (GLOBAL = true: accesses bypass the L1; the
// workgroup barrier orders them, no device-wide fence is needed or wanted -- on this
// GPU a device-scope release writes back the whole L2).
#pragma once

#include "common.hpp"

namespace lda {

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


template <bool GLOBAL>
struct ListMem {
    __device__ __forceinline__ static uint64_t ld(const uint64_t* p)
    {
        if constexpr (GLOBAL)
            return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            return *p;
    }
    __device__ __forceinline__ static uint32_t ld(const uint32_t* p)
    {
        if constexpr (GLOBAL)
            return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            return *p;
    }
    __device__ __forceinline__ static void st(uint64_t* p, uint64_t v)
    {
        if constexpr (GLOBAL)
            __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            *p = v;
    }
    __device__ __forceinline__ static void st(uint32_t* p, uint32_t v)
    {
        if constexpr (GLOBAL)
            __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            *p = v;
    }
    __device__ __forceinline__ static void barrier()
    {
        __syncthreads();
    }
};

// Bytes of list memory for a table of n entries (with / without the mass cache).
__host__ __device__ inline size_t alias_list_bytes(size_t n, bool with_cache)
{
    return sizeof(uint64_t) * (n + 1) + sizeof(uint32_t) * n + (with_cache ? sizeof(uint32_t) * n : 0);
}

// Builds one table with all threads of the block (blockDim.x a multiple of 64, at
// most 1024).  lists: alias_list_bytes(n, use_cache) bytes, 8-byte aligned.  Wave v
// owns the contiguous entries [v*S, (v+1)*S), visited 64 at a time, so accesses by
// Src/Sink are coalesced and entries are met in ascending order.  Returns the
// pre-shift sum Q0 and the capacity C to every thread.  Ends with a barrier-free
// tail: callers synchronise before reusing `lists`.
template <bool GLOBAL, class Src, class Sink>
__device__ __forceinline__ void build_alias_table(int32_t n, const Src& src, const Sink& sink,
                                                  unsigned char* lists, bool use_cache,
                                                  uint64_t& Q0_out, uint32_t& C_out)
{
    using M = ListMem<GLOBAL>;
    // dx[0..A]   : Delta_a (exclusive deficit sums of the lights, dx[A] = total)
    // dx[n-b]    : X_b     (inclusive excess sums of the heavies), b = 0..B-1, A + B = n
    uint64_t* dx = reinterpret_cast<uint64_t*>(lists);
    uint32_t* hidx = reinterpret_cast<uint32_t*>(dx + (n + 1));  // hidx[b] = entry of heavy b
    // qc[i] = q0_i saturated to 32 bits, kept for the later passes when there is room
    // (0xFFFFFFFF: does not fit, recompute)
    uint32_t* qc = hidx + n;
    __shared__ uint64_t w_a[kMaxWaves], w_b[kMaxWaves];
    __shared__ uint32_t w_c[kMaxWaves];

    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int32_t S = (((n + nw - 1) / nw + kWave - 1) / kWave) * kWave;  // entries per wave
    const int32_t kb = wv * S;
    const int32_t ke = (kb + S < n) ? kb + S : n;

    // pass 1: Q0 and, for the usual case of no shift, Q
    uint64_t p0 = 0, p1 = 0;
#pragma unroll 4
    for (int32_t k = kb + lane; k < ke; k += kWave) {
        const uint64_t q0 = src.q0(k);
        if (use_cache) M::st(&qc[k], (q0 < 0xFFFFFFFFull) ? (uint32_t)q0 : 0xFFFFFFFFu);
        p0 += q0;
        p1 += (q0 < 1) ? 1 : q0;
    }
    p0 = wave_sum_u64(p0);
    p1 = wave_sum_u64(p1);
    __syncthreads();  // a previous table's use of w_a / w_b / w_c is over
    if (lane == 0) { w_a[wv] = p0; w_b[wv] = p1; }
    __syncthreads();
    uint64_t Q0 = 0, Q = 0;
    for (int i = 0; i < nw; ++i) { Q0 += w_a[i]; Q += w_b[i]; }
    int sh = 0;
    while ((Q0 >> sh) >= ((uint64_t)n << 31)) ++sh;
    auto quant = [&](int32_t k) -> uint64_t {
        uint64_t q = use_cache ? (uint64_t)M::ld(&qc[k]) : 0xFFFFFFFFull;
        if (q == 0xFFFFFFFFull) q = src.q0(k);
        return q;
    };
    if (sh > 0) {  // uniform over the block
        p1 = 0;
        for (int32_t k = kb + lane; k < ke; k += kWave) {
            const uint64_t q = quant(k) >> sh;
            p1 += (q < 1) ? 1 : q;
        }
        p1 = wave_sum_u64(p1);
        __syncthreads();
        if (lane == 0) w_b[wv] = p1;
        __syncthreads();
        Q = 0;
        for (int i = 0; i < nw; ++i) Q += w_b[i];
    }
    const uint64_t C = (Q + (uint64_t)n - 1) / (uint64_t)n;
    const uint64_t pad = (uint64_t)n * C - Q;
    auto mass = [&](int32_t k) -> uint64_t {
        uint64_t q = quant(k) >> sh;
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
    const uint32_t B = (uint32_t)n - A;
    uint32_t b_run = (uint32_t)kb - a_run;
    if (threadIdx.x == 0) M::st(&dx[A], d_tot);
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
            M::st(&dx[a_run + la], d_run + dinc - (C - m));
        } else if (heavy) {
            const uint32_t b = b_run + ((uint32_t)lane - la);
            M::st(&dx[n - b], x_run + xinc);
            M::st(&hidx[b], (uint32_t)k);
        }
        const uint32_t nl = (uint32_t)__popcll(lmask);
        const uint32_t nv = (uint32_t)((ke - k0 < kWave) ? ke - k0 : kWave);
        a_run += nl;
        b_run += nv - nl;
        d_run += readlane_u64(dinc, kWave - 1);
        x_run += readlane_u64(xinc, kWave - 1);
    }
    M::barrier();

    // pass 4: pair them.  Within a wave the ranks of one kind only grow and the
    // partner index is monotone in the rank.  Per round the whole wave searches the
    // partner of the last light (heavy) starting from the previous round's result;
    // every lane then searches only between those two bounds.
    a_run = a_wave;
    b_run = b_wave;
    uint32_t b_prev = 0;  // partner of the last light met so far
    uint32_t a_prev = 0;  // partner of the last heavy met so far
    // Lists in global memory: every probe of a search is a round trip to L2, and a round's
    // searches are a chain of them.  The 64 list entries that follow the previous round's
    // result are therefore read once, by the whole wave, and kept in a window in LDS; when
    // the round's last partner lies inside the window (the usual case) every lane's own
    // search runs on the window.
    __shared__ uint64_t s_win[GLOBAL ? kMaxWaves * 2 * kWave : 1];
    uint64_t* const xwin = s_win + (GLOBAL ? wv * 2 * kWave : 0);  // X of heavies b_prev + i
    uint64_t* const dwin = xwin + (GLOBAL ? kWave : 0);            // Delta of lights a_prev + i
    typename Sink::Loaded pend_v{};
    int32_t pend_k = -1;
    uint32_t pend_split = 0, pend_al = 0;
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
        if (light) own = M::ld(&dx[a_run + la]);
        if (heavy) own = M::ld(&dx[n - b_own]);
        uint32_t b_hi = b_prev, a_hi = a_prev;
        bool xwin_ok = false, dwin_ok = false;  // uniform: the round's partners are in the window
        if (lmask != 0) {  // uniform
            const uint64_t delta_last = readlane_u64(own, 63 - __clzll((unsigned long long)lmask));
            // first b with X_b > delta; X_{B-1} = total deficit > every delta
            uint32_t from = b_prev;
            if constexpr (GLOBAL) {
                const uint32_t top = (B - 1 - b_prev > 63u) ? b_prev + 63u : B - 1;
                const uint32_t idx = (b_prev + (uint32_t)lane < top) ? b_prev + (uint32_t)lane : top;
                const uint64_t xv = M::ld(&dx[n - idx]);
                const uint64_t hit = __ballot(xv > delta_last);
                if (hit != 0) {
                    b_hi = b_prev + (uint32_t)(__ffsll((unsigned long long)hit) - 1);
                    xwin[lane] = xv;
                    xwin_ok = true;
                } else {
                    from = top + 1;  // top < B - 1 here, because X_{B-1} > delta
                }
            }
            if (!xwin_ok)
                b_hi = wave_first_true(from, B - 1, lane,
                                       [&](uint32_t i) { return M::ld(&dx[n - i]) > delta_last; });
        }
        if (hmask != 0) {  // uniform
            const uint64_t x_last = readlane_u64(own, 63 - __clzll((unsigned long long)hmask));
            // first a with Delta_a >= X; Delta_A = total excess >= every X
            uint32_t from = a_prev;
            if constexpr (GLOBAL) {
                const uint32_t top = (A - a_prev > 63u) ? a_prev + 63u : A;
                const uint32_t idx = (a_prev + (uint32_t)lane < top) ? a_prev + (uint32_t)lane : top;
                const uint64_t dv = M::ld(&dx[idx]);
                const uint64_t hit = __ballot(dv >= x_last);
                if (hit != 0) {
                    a_hi = a_prev + (uint32_t)(__ffsll((unsigned long long)hit) - 1);
                    dwin[lane] = dv;
                    dwin_ok = true;
                } else {
                    from = top + 1;  // top < A here, because Delta_A >= X
                }
            }
            if (!dwin_ok)
                a_hi = wave_first_true(from, A, lane,
                                       [&](uint32_t i) { return M::ld(&dx[i]) >= x_last; });
        }
        if constexpr (GLOBAL) __builtin_amdgcn_wave_barrier();  // windows written before they are read
        uint32_t split = 0, al = 0;
        if (light) {
            uint32_t lo = b_prev, hi = b_hi;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                const uint64_t x = (GLOBAL && xwin_ok) ? xwin[mid - b_prev] : M::ld(&dx[n - mid]);
                if (x > own) hi = mid; else lo = mid + 1;
            }
            split = (uint32_t)m;
            al = M::ld(&hidx[lo]);
        } else if (heavy) {
            uint32_t lo = a_prev, hi = a_hi;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                const uint64_t d = (GLOBAL && dwin_ok) ? dwin[mid - a_prev] : M::ld(&dx[mid]);
                if (d >= own) hi = mid; else lo = mid + 1;
            }
            const uint64_t sp = C + own - ((GLOBAL && dwin_ok) ? dwin[lo - a_prev] : M::ld(&dx[lo]));
            split = (uint32_t)sp;
            al = (sp < C) ? M::ld(&hidx[b_own + 1]) : (uint32_t)k;
        }
        // An entry's output needs values gathered from global memory (the counts of its
        // two outcomes); the gathers are issued now and the entry is stored one round
        // later, so their latency overlaps the next round's searches.
        typename Sink::Loaded cur_v{};
        if (valid) cur_v = sink.load(k, al);
        if (pend_k >= 0) sink.store(pend_k, pend_split, pend_al, pend_v);
        pend_k = valid ? k : -1;
        pend_split = split;
        pend_al = al;
        pend_v = cur_v;
        b_prev = b_hi;
        a_prev = a_hi;
        const uint32_t nl = (uint32_t)__popcll(lmask);
        const uint32_t nv = (uint32_t)((ke - k0 < kWave) ? ke - k0 : kWave);
        a_run += nl;
        b_run += nv - nl;
    }
    if (pend_k >= 0) sink.store(pend_k, pend_split, pend_al, pend_v);
    Q0_out = Q0;
    C_out = (uint32_t)C;
}

}  // namespace lda
