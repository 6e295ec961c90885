// Mapping of workgroups to work items that respects the 8 XCDs of the device, each of which
// has its own L2.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace lda {

constexpr int kXcds = 8;

// Workgroups are dealt to the 8 XCDs round-robin.  Handing each XCD one contiguous run of
// the items keeps neighbouring items -- which touch neighbouring word-major records -- in
// one L2.  Returns an index that may lie past the last item.
__device__ __forceinline__ int32_t xcd_contiguous(int32_t n_items)
{
    const int32_t per = (n_items + kXcds - 1) / kXcds;
    return (int32_t)(blockIdx.x % kXcds) * per + (int32_t)(blockIdx.x / kXcds);
}

inline unsigned xcd_grid(int32_t n_items) { return (unsigned)((n_items + kXcds - 1) / kXcds * kXcds); }

// The word pass's work lists are in word order, and the cost of an item depends on its
// word's class (frequent words are served from LDS or L2, rare ones miss), so contiguous
// eighths would leave the XCDs unevenly loaded.  Runs of `run` consecutive items are dealt
// to the XCDs in turn instead: neighbours still share an L2, every XCD sees every class.
__device__ __forceinline__ int32_t xcd_runs(int32_t run)
{
    const int32_t xcd = (int32_t)(blockIdx.x % kXcds), seq = (int32_t)(blockIdx.x / kXcds);
    return ((seq / run) * kXcds + xcd) * run + seq % run;
}

inline unsigned xcd_runs_grid(int32_t n_items, int32_t run)
{
    const int32_t runs = (n_items + run - 1) / run;
    return (unsigned)((runs + kXcds - 1) / kXcds * kXcds * run);
}

}  // namespace lda
