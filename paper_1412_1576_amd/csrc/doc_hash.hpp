// Per-document topic counts n_kd as a small open-addressing hash table.
//
// The doc-topic row of a document with L tokens has at most L non-zeros, so it
// is kept as 2L (topic, count) slots (load factor <= 1/2), built from the
// document's assignments when a workgroup picks the document up.  Short
// documents live in LDS next to the document's z values; documents too long for
// an LDS tile use the same code on a global-memory workspace.
#pragma once

#include "common.hpp"

namespace lda {

constexpr int32_t kEmptyKey = -1;

__device__ __forceinline__ uint32_t topic_hash(int32_t k) { return (uint32_t)k * 0x9E3779B1u; }

// GLOBAL = false: keys/cnts point into LDS.  GLOBAL = true: they point into
// device memory that other lanes of the workgroup update with atomics, so reads
// go through agent-scope atomic loads (they must not be served from a stale L1 line).
template <bool GLOBAL>
struct DocTable {
    int32_t* keys;
    int32_t* cnts;
    uint32_t slots;  // 2 * L >= 2

    __device__ __forceinline__ static int32_t ld(const int32_t* p)
    {
        if constexpr (GLOBAL)
            return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            return *p;
    }

    __device__ __forceinline__ void insert(int32_t k) const
    {
        uint32_t s = mulhi32(topic_hash(k), slots);
        for (uint32_t n = 0; n < slots; ++n) {
            const int32_t prev = atomicCAS(&keys[s], kEmptyKey, k);
            if (prev == kEmptyKey || prev == k) {
                atomicAdd(&cnts[s], 1);
                return;
            }
            s = (s + 1 == slots) ? 0u : s + 1;
        }
    }

    // n_kd of topic k (0 when the document has no token of it).  At most `slots`
    // probes; an empty slot always exists because the load factor is <= 1/2.
    __device__ __forceinline__ int32_t count(int32_t k) const
    {
        uint32_t s = mulhi32(topic_hash(k), slots);
        for (uint32_t n = 0; n < slots; ++n) {
            const int32_t key = ld(&keys[s]);
            if (key == k) return ld(&cnts[s]);
            if (key == kEmptyKey) return 0;
            s = (s + 1 == slots) ? 0u : s + 1;
        }
        return 0;
    }
};

// Index of the document that owns local token i: the last dl with sdoff[dl] <= i,
// where sdoff[0..nd] are the chunk-relative document offsets (sdoff[nd] > i).
__device__ __forceinline__ int32_t find_doc(const int32_t* sdoff, int32_t nd, int32_t i)
{
    int32_t lo = 0, hi = nd;  // sdoff[lo] <= i < sdoff[hi]
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (sdoff[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace lda
