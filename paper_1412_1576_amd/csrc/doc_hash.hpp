// Per-document topic counts n_kd as a small open-addressing hash table.
//
// The doc-topic row of a document with L tokens has at most L non-zeros, so it
// is kept in 2L slots (load factor <= 1/2), built from the document's
// assignments when a workgroup picks the document up.  Documents that fit an LDS
// tile pack (count << 20 | topic) into one 32-bit slot next to the document's z
// values, and every token remembers the slot of its own topic, so the counts of
// a token's own topic and of a topic copied from another token of the document
// need no probing.  Documents too long for a tile keep (topic, count) in two
// arrays of a global-memory workspace.
#pragma once

#include "common.hpp"

namespace lda {

constexpr int32_t kEmptyKey = -1;
constexpr uint32_t kEmptySlot = 0xFFFFFFFFu;
constexpr int kTopicBits = 20;                       // packed slots: topic < 2^20 - 1
constexpr uint32_t kTopicMask = (1u << kTopicBits) - 1u;
constexpr int32_t kMaxPackedTopics = (1 << kTopicBits) - 1;
constexpr int32_t kMaxPackedCount = (1 << (32 - kTopicBits)) - 1;  // 4095 tokens per document
constexpr int32_t kMaxTileTokens = 2016;  // a token's slot index (< 2 * tile tokens) takes 12 bits

// Bucket of topic k in a table of `buckets` < 2^16 two-slot buckets.  Both
// multiplies are 24-bit (full rate on the vector ALU): a 16-bit golden-ratio
// multiplier spreads k, the middle 16 bits of the product are scaled to [0, buckets).
__device__ __forceinline__ uint32_t packed_bucket(int32_t k, uint32_t buckets)
{
    const uint32_t h = (__umul24((uint32_t)k, 40503u) >> 4) & 0xFFFFu;
    return __umul24(h, buckets) >> 16;
}

// LDS table of one document: L buckets of two packed slots (load factor <= 1/2),
// probed one whole bucket (one 8-byte LDS read) at a time.
struct PackedDocTable {
    uint32_t* tab;     // 8-byte aligned
    uint32_t buckets;  // = L, 1 <= buckets <= 2047

    // Adds one token of topic k; returns the slot (relative to tab) that holds k.
    __device__ __forceinline__ uint32_t insert(int32_t k) const
    {
        uint32_t b = packed_bucket(k, buckets);
        const uint32_t fresh = (1u << kTopicBits) | (uint32_t)k;
        for (uint32_t n = 0; n < buckets; ++n) {
#pragma unroll
            for (uint32_t j = 0; j < 2; ++j) {
                const uint32_t s = 2 * b + j;
                const uint32_t prev = atomicCAS(&tab[s], kEmptySlot, fresh);
                if (prev == kEmptySlot) return s;
                if ((prev & kTopicMask) == (uint32_t)k) {
                    atomicAdd(&tab[s], 1u << kTopicBits);
                    return s;
                }
            }
            b = (b + 1 == buckets) ? 0u : b + 1;
        }
        return 0;  // not reached: at most L distinct topics in 2L slots
    }

    // n_kd of topic k (0 when the document has no token of it).  Slots of a bucket
    // fill in order, so an empty slot ends the search.
    __device__ __forceinline__ int32_t count(int32_t k) const
    {
        uint32_t b = packed_bucket(k, buckets);
        int32_t result = 0;
        for (uint32_t n = 0; n < buckets; ++n) {
            const uint2 v = reinterpret_cast<const uint2*>(tab)[b];
            // an empty slot never matches: its topic field is 2^20 - 1 > any topic
            const bool hit0 = (v.x & kTopicMask) == (uint32_t)k;
            const bool hit1 = (v.y & kTopicMask) == (uint32_t)k;
            if (hit0) result = (int32_t)(v.x >> kTopicBits);
            if (hit1) result = (int32_t)(v.y >> kTopicBits);
            if (hit0 || hit1 || v.x == kEmptySlot || v.y == kEmptySlot) break;
            b = (b + 1 == buckets) ? 0u : b + 1;
        }
        return result;
    }

    // count of the topic stored in a known slot (as returned by insert)
    __device__ __forceinline__ int32_t count_at(uint32_t slot) const
    {
        return (int32_t)(tab[slot] >> kTopicBits);
    }
};

__device__ __forceinline__ uint32_t topic_hash(int32_t k) { return (uint32_t)k * 0x9E3779B1u; }

// Global-memory table of one long document.  Other lanes of the workgroup update
// it with atomics, so reads go through agent-scope atomic loads (they must not be
// served from a stale L1 line).
struct GlobalDocTable {
    int32_t* keys;
    int32_t* cnts;
    uint32_t slots;  // 2 * L

    __device__ __forceinline__ static int32_t ld(const int32_t* p)
    {
        return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

    // slot that holds topic k, which must be in the table
    __device__ __forceinline__ uint32_t slot_of(int32_t k) const
    {
        uint32_t s = mulhi32(topic_hash(k), slots);
        for (uint32_t n = 0; n < slots; ++n) {
            if (ld(&keys[s]) == k) return s;
            s = (s + 1 == slots) ? 0u : s + 1;
        }
        return 0;
    }

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
// where sdoff[0..nd] are the tile-relative document offsets (sdoff[nd] > i).
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
