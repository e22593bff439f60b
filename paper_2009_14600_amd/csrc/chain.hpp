// Single-pass prefix sums across the blocks of one launch ("chained scan with decoupled look-back"):
// every block publishes the aggregate of its slice, then adds up the aggregates of the blocks before
// it (one wave reads 64 predecessors at a time) until it meets a block whose inclusive prefix is
// already known.  Used for the per-tile-row counts -> offsets steps (paper Section 4.1: Algorithm 1's
// counts-to-offsets steps), which are too small to be worth three launches and too slow on a single CU.
//
// Forward progress: blocks are dispatched in index order, so the predecessors a block waits for are
// running or finished.  The wait is bounded all the same: after kChainSpinLimit polls a block gives
// up, raises *error and carries on with a wrong prefix, so every wave exits whatever happens and the
// host turns the flag into an error code.  Aggregates must stay below 2^40 (wave_inclusive_scan64).
#pragma once

#include "common.hpp"

namespace tsp {

constexpr int kChainValues = 3;
constexpr unsigned kChainSpinLimit = 1u << 22;

struct __attribute__((aligned(128))) ChainSlot {
    unsigned long long aggregate[kChainValues];
    unsigned long long inclusive[kChainValues];
    unsigned int flag;      // (epoch << 2) | state; state 1: aggregate valid, 2: inclusive valid
};

#ifdef __HIPCC__
// Called by every thread of the block (blockDim.x >= 64).  `mine` holds the block's aggregates (the
// same values in every thread).  Returns in `prefix` the sum of the aggregates of blocks 0..b-1.
// lds: kChainValues words of scratch.
__device__ __forceinline__ void chain_exclusive_prefix(ChainSlot *slots, unsigned epoch, const unsigned long long *mine,
                                                      unsigned long long *prefix, uint64_t *lds,
                                                      int64_t *error) {
    const int b = blockIdx.x;
    const unsigned tag = epoch << 2;
    if (threadIdx.x < 64) {                       // wave 0 does the chain work
        const int lane = threadIdx.x;
        unsigned long long run[kChainValues] = {0, 0, 0};
        if (b == 0) {
            if (lane == 0) {
                for (int q = 0; q < kChainValues; ++q) slots[0].inclusive[q] = mine[q];
                __hip_atomic_store(&slots[0].flag, tag | 2u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else {
            if (lane == 0) {
                for (int q = 0; q < kChainValues; ++q) slots[b].aggregate[q] = mine[q];
                __hip_atomic_store(&slots[b].flag, tag | 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            }
            int top = b - 1;                      // highest predecessor not yet accounted for
            bool done = false;
            unsigned spins = 0;
            while (!done) {
                const int p = top - lane;         // lane l looks at predecessor top - l
                unsigned f = tag | 2u;            // lanes before block 0 act as "inclusive zero"
                if (p >= 0) f = __hip_atomic_load(&slots[p].flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                const bool ready = (f & ~3u) == tag && (f & 3u) != 0;
                const unsigned long long not_ready = __ballot(!ready);
                const unsigned long long closed = __ballot(ready && (f & 3u) == 2u);
                // usable lanes: from lane 0 up to the first lane that is not ready or holds an inclusive value
                const int first_open = not_ready ? __ffsll((long long)not_ready) - 1 : 64;
                const int first_closed = closed ? __ffsll((long long)closed) - 1 : 64;
                if (first_closed < first_open) {
                    // lanes 0..first_closed-1 contribute aggregates, lane first_closed its inclusive value
#pragma unroll
                    for (int q = 0; q < kChainValues; ++q) {
                        unsigned long long v = 0;
                        if (p >= 0 && lane < first_closed) v = slots[p].aggregate[q];
                        if (p >= 0 && lane == first_closed) v = slots[p].inclusive[q];
                        run[q] += wave_inclusive_scan64(v);
                    }
                    done = true;
                } else if (first_open == 64) {
                    // all 64 predecessors hold aggregates only: take them and look further back
#pragma unroll
                    for (int q = 0; q < kChainValues; ++q) run[q] += wave_inclusive_scan64(slots[p].aggregate[q]);
                    top -= 64;
                } else {
                    if (++spins > kChainSpinLimit) {
                        if (lane == 0) *error = 1;
                        done = true;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            if (lane == 63) {                     // lane 63 holds the wave totals
                for (int q = 0; q < kChainValues; ++q) slots[b].inclusive[q] = run[q] + mine[q];
                __hip_atomic_store(&slots[b].flag, tag | 2u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (lane == 63)
            for (int q = 0; q < kChainValues; ++q) lds[q] = run[q];
    }
    __syncthreads();
    for (int q = 0; q < kChainValues; ++q) prefix[q] = lds[q];
}
#endif

}  // namespace tsp
