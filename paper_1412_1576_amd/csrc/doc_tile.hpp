// A workgroup's tile of consecutive documents staged in LDS: the documents'
// snapshot assignments, their tile-relative offsets and one n_kd hash table per
// document (doc_hash.hpp).  Used by the sweep, the doc-likelihood and the
// n_kd accessor, so all three see the same tables.
#pragma once

#include "doc_hash.hpp"

namespace lda {

struct DocTile {
    uint32_t* zs;    // [cap_tokens]   per token: snapshot topic | slot of that topic << 20
                     //                (slot relative to the document's table)
    uint32_t* tab;   // [2*cap_tokens] packed slots, document d owns [2*sdoff[d], 2*sdoff[d+1])
    int32_t* sdoff;  // [cap_docs+1]   token offsets relative to the tile start
    int32_t nd;      // documents in the tile
    int32_t ntok;    // tokens in the tile
    int32_t tok0;    // CSR position of the tile's first token

    __device__ __forceinline__ PackedDocTable table(int32_t dl) const
    {
        const int32_t b = sdoff[dl];
        return PackedDocTable{tab + 2 * b, (uint32_t)(sdoff[dl + 1] - b)};
    }
};

__host__ __device__ inline size_t doc_tile_lds_bytes(int32_t cap_tokens, int32_t cap_docs)
{
    return sizeof(int32_t) * ((size_t)3 * cap_tokens + cap_docs + 1);
}

// Stage documents [d0, d1) and build their tables.  tokdoc[g] is the index of
// token g's document inside its tile (NULL: found by binary search).  STREAM: read z
// and tokdoc with the non-temporal hint (a caller that wants its L2 for other data).
// All threads of the block must call it; it ends with a barrier.
template <bool STREAM = false>
__device__ __forceinline__ DocTile load_doc_tile(int32_t* smem, int32_t cap_tokens,
                                                 const int32_t* __restrict__ z,
                                                 const int32_t* __restrict__ doff,
                                                 const uint8_t* __restrict__ tokdoc, int32_t d0,
                                                 int32_t d1)
{
    DocTile t;
    t.zs = reinterpret_cast<uint32_t*>(smem);
    t.tab = reinterpret_cast<uint32_t*>(smem + cap_tokens);
    t.sdoff = smem + 3 * (size_t)cap_tokens;
    t.nd = d1 - d0;
    t.tok0 = doff[d0];
    t.ntok = doff[d1] - t.tok0;
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int32_t i = tid; i <= t.nd; i += nt) t.sdoff[i] = doff[d0 + i] - t.tok0;
    for (int32_t i = tid; i < t.ntok; i += nt) {
        t.zs[i] = (uint32_t)(STREAM ? __builtin_nontemporal_load(&z[t.tok0 + i]) : z[t.tok0 + i]);
        reinterpret_cast<uint2*>(t.tab)[i] = make_uint2(kEmptySlot, kEmptySlot);
    }
    __syncthreads();
    for (int32_t i = tid; i < t.ntok; i += nt) {
        const int32_t dl = tokdoc ? (int32_t)(STREAM ? __builtin_nontemporal_load(&tokdoc[t.tok0 + i])
                                                     : tokdoc[t.tok0 + i])
                                  : find_doc(t.sdoff, t.nd, i);
        const uint32_t zi = t.zs[i];
        t.zs[i] = zi | (t.table(dl).insert((int32_t)zi) << kTopicBits);  // own element only
    }
    __syncthreads();
    return t;
}

// A document too long for an LDS tile: its table lives in a global workspace
// (keys/cnts of 2*L slots), cleared and filled by the calling workgroup.
__device__ __forceinline__ GlobalDocTable load_long_doc(int32_t* keys, int32_t* cnts,
                                                        const int32_t* __restrict__ zdoc,
                                                        int32_t L)
{
    GlobalDocTable tab{keys, cnts, (uint32_t)(2u * (uint32_t)L)};
    const int tid = threadIdx.x, nt = blockDim.x;
    for (uint32_t i = tid; i < tab.slots; i += nt) {
        __hip_atomic_store(&keys[i], kEmptyKey, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&cnts[i], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    for (int32_t i = tid; i < L; i += nt) tab.insert(zdoc[i]);
    __syncthreads();
    return tab;
}

}  // namespace lda
