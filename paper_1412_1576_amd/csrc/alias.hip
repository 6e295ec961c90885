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
// so the build is two block-wide prefix sums and one binary search per bin.
#include "common.hpp"

namespace lda {

namespace {

constexpr int kMaxWaves = 16;

struct Tri {
    uint32_t c;  // lights
    uint64_t d;  // deficit of lights
    uint64_t x;  // excess of heavies
};

__device__ __forceinline__ Tri tri_add(const Tri& a, const Tri& b)
{
    return Tri{a.c + b.c, a.d + b.d, a.x + b.x};
}

__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int delta)
{
    const uint32_t lo = __shfl_up((uint32_t)v, delta, kWave);
    const uint32_t hi = __shfl_up((uint32_t)(v >> 32), delta, kWave);
    return ((uint64_t)hi << 32) | lo;
}

// Exclusive prefix of v over the block in thread order; total = sum over the block.
// wtot is LDS scratch for kMaxWaves entries.  Contains two barriers.
__device__ __forceinline__ Tri block_exclusive_scan(Tri v, Tri& total, Tri* wtot)
{
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int nw = (blockDim.x + kWave - 1) >> 6;
    Tri inc = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        Tri o;
        o.c = __shfl_up(inc.c, d, kWave);
        o.d = shfl_up_u64(inc.d, d);
        o.x = shfl_up_u64(inc.x, d);
        if (lane >= d) inc = tri_add(inc, o);
    }
    __syncthreads();  // previous use of wtot is over
    if (lane == kWave - 1) wtot[wv] = inc;
    __syncthreads();
    Tri before{0u, 0ull, 0ull}, all{0u, 0ull, 0ull};
    for (int i = 0; i < nw; ++i) {
        const Tri t = wtot[i];
        if (i < wv) before = tri_add(before, t);
        all = tri_add(all, t);
    }
    total = all;
    Tri ex = tri_add(before, inc);
    ex.c -= v.c; ex.d -= v.d; ex.x -= v.x;
    return ex;
}

__device__ __forceinline__ uint64_t block_sum_u64(uint64_t v, uint64_t* wtot)
{
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int nw = (blockDim.x + kWave - 1) >> 6;
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, d, kWave);
        const uint32_t hi = __shfl_xor((uint32_t)(v >> 32), d, kWave);
        v += ((uint64_t)hi << 32) | lo;
    }
    __syncthreads();
    if (lane == 0) wtot[wv] = v;
    __syncthreads();
    uint64_t s = 0;
    for (int i = 0; i < nw; ++i) s += wtot[i];
    return s;
}

// R = bins per thread (bin k = r * blockDim.x + tid), K <= R * blockDim.x.
template <int R>
__global__ __launch_bounds__(1024) void alias_dense_kernel(const int32_t* __restrict__ nkw,
                                                           const int32_t* __restrict__ nk,
                                                           int32_t K, double beta, double betabar,
                                                           uint2* __restrict__ alias,
                                                           uint32_t* __restrict__ cap)
{
#pragma clang fp contract(off)
    extern __shared__ unsigned char smem_raw[];
    // dx[0..A]   : Delta_a (exclusive deficit sums of the lights, dx[A] = total)
    // dx[K-b]    : X_b     (inclusive excess sums of the heavies), b = 0..B-1, A + B = K
    uint64_t* dx = reinterpret_cast<uint64_t*>(smem_raw);
    uint32_t* hidx = reinterpret_cast<uint32_t*>(dx + (K + 1));  // hidx[b] = bin of heavy b
    __shared__ Tri wtot[kMaxWaves];
    __shared__ uint64_t wsum[kMaxWaves];

    const int32_t w = blockIdx.x;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int32_t* __restrict__ row = nkw + (size_t)w * (size_t)K;
    uint2* __restrict__ out = alias + (size_t)w * (size_t)K;

    uint64_t m[R];
    uint64_t part = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int32_t k = r * nt + tid;
        m[r] = 0;
        if (k < K) {
            const double a = ((double)row[k] + beta) / ((double)nk[k] + betabar);
            m[r] = (uint64_t)floor(a * 1099511627776.0);
            part += m[r];
        }
    }
    const uint64_t Q0 = block_sum_u64(part, wsum);
    int sh = 0;
    while ((Q0 >> sh) >= ((uint64_t)K << 31)) ++sh;
    part = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int32_t k = r * nt + tid;
        if (k < K) {
            uint64_t q = m[r] >> sh;
            if (q < 1) q = 1;
            m[r] = q;
            part += q;
        }
    }
    const uint64_t Q = block_sum_u64(part, wsum);
    const uint64_t C = (Q + (uint64_t)K - 1) / (uint64_t)K;
    const uint64_t pad = (uint64_t)K * C - Q;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int32_t k = r * nt + tid;
        if (k < K && (uint64_t)k < pad) m[r] += 1;
    }

    // split into lights / heavies in ascending k, with running sums
    uint32_t pos[R];
    Tri carry{0u, 0ull, 0ull};
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int32_t k = r * nt + tid;
        const bool valid = k < K;
        const bool light = valid && m[r] < C;
        const bool heavy = valid && !light;
        Tri v{light ? 1u : 0u, light ? C - m[r] : 0ull, heavy ? m[r] - C : 0ull};
        Tri total;
        Tri ex = block_exclusive_scan(v, total, wtot);
        ex = tri_add(ex, carry);
        pos[r] = 0;
        if (light) {
            pos[r] = ex.c;
            dx[ex.c] = ex.d;
        } else if (heavy) {
            const uint32_t b = (uint32_t)k - ex.c;
            pos[r] = b;
            dx[K - b] = ex.x + v.x;
            hidx[b] = (uint32_t)k;
        }
        carry = tri_add(carry, total);
    }
    const uint32_t A = carry.c;
    const uint32_t B = (uint32_t)K - A;
    if (tid == 0) {
        dx[A] = carry.d;
        cap[w] = (uint32_t)C;
    }
    __syncthreads();

#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int32_t k = r * nt + tid;
        if (k >= K) continue;
        uint32_t split, al;
        if (m[r] < C) {
            const uint64_t delta = dx[pos[r]];
            // first b in [0, B) with X_b > delta; X_{B-1} = total deficit > delta
            uint32_t lo = 0, hi = B - 1;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (dx[K - mid] > delta) hi = mid; else lo = mid + 1;
            }
            split = (uint32_t)m[r];
            al = hidx[lo];
        } else {
            const uint32_t b = pos[r];
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
}

template <int R>
int launch_r(lda_ctx* c, int block, size_t lds)
{
    auto kern = alias_dense_kernel<R>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return fail(c, LDA_ERR_HIP, "hipFuncSetAttribute(alias, %zu): %s", lds,
                        hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, dim3(c->V), dim3(block), lds, c->stream, c->d_nkw, c->d_nk, c->K,
                       c->beta, c->betabar, c->d_alias, c->d_cap);
    LDA_HIP(c, hipGetLastError());
    return LDA_OK;
}

}  // namespace

int max_alias_topics() { return 12 * 1024; }

int launch_alias_build(lda_ctx* c)
{
    const int32_t K = c->K;
    if (K > max_alias_topics())
        return fail(c, LDA_ERR_UNSUPPORTED, "dense alias build supports K <= %d", max_alias_topics());
    int block = 1024;
    if (K <= 1024) block = ((K + kWave - 1) / kWave) * kWave;
    const int R = (K + block - 1) / block;
    const size_t lds = sizeof(uint64_t) * ((size_t)K + 1) + sizeof(uint32_t) * (size_t)K;
    if (R <= 1) return launch_r<1>(c, block, lds);
    if (R <= 2) return launch_r<2>(c, block, lds);
    if (R <= 3) return launch_r<3>(c, block, lds);
    if (R <= 4) return launch_r<4>(c, block, lds);
    if (R <= 6) return launch_r<6>(c, block, lds);
    if (R <= 8) return launch_r<8>(c, block, lds);
    if (R <= 10) return launch_r<10>(c, block, lds);
    return launch_r<12>(c, block, lds);
}

}  // namespace lda
