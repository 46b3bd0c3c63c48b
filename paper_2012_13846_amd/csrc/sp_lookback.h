// Single-pass device-wide prefix sums over the workgroups of ONE launch ("decoupled look-back"): a workgroup
// publishes the sum of its own items, adds up what its predecessors published and publishes its inclusive prefix,
// so that later workgroups stop looking back there.  Replaces "count kernel, scan kernels, emit kernel" by one
// kernel that counts, ranks and emits.  A chain carries a small vector of sums (one per kernel offset, or one).
//
// Storage: desc[i * n_tiles + t], one 64-bit word per (sum i, tile t), holding a 2-bit state and the value:
//   0 nothing yet | 1 the tile's own sum | 2 the inclusive prefix (sums of tiles 0..t).     (must start at 0)
// State and value travel in one word, written and read with relaxed device-scope atomics: no fences (a release
// fence writes the whole L2 back on this chip: measured 0.5 us per workgroup, serialised).
//
// Tile = workgroup index.  Workgroups are handed to each XCD in index order, so the lowest-numbered unfinished
// workgroup is always resident (its XCD started it before any later one) and waits for nobody that has not
// finished: the waits below always end.  (A ticket from an atomic counter would not need that argument, but
// one atomic per workgroup on ONE address costs ~0.5 us each across the XCDs.)  The waits are bounded all the
// same: a wait that exceeds kSpinLimit polls sets an error bit and gives up, so the grid drains whatever happens.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sp {

constexpr unsigned kSpinLimit = 1u << 22;  // polls of ~1 us: seconds, far beyond any real wait
constexpr int kErrLookback = 4;            // error bit: a look-back wait gave up
constexpr int kMaxChainWidth = 160;

struct Chain {
    unsigned long long* desc;  // [width][n_tiles]
    int64_t n_tiles;           // row pitch of desc
    int width;                 // sums per tile
};

constexpr unsigned long long kDescOwn = 1ull << 62, kDescPrefix = 2ull << 62, kDescValue = (1ull << 62) - 1ull;

__device__ __forceinline__ unsigned long long load_desc(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_desc(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by ALL threads of the workgroup (blockDim.x >= 64, a multiple of 64).  s_own[0..width): this tile's sums
// (shared memory, written before the call; a __syncthreads() inside precedes their first use).  On return
// s_excl[0..width) holds the sums of all earlier tiles and the tile's inclusive prefix has been published.
// s_state: 2 * kMaxChainWidth ints of shared memory.  err: device error word.
__device__ __forceinline__ void chain_lookback(const Chain& c, int tile, const int* s_own, int* s_excl, int* s_state,
                                               int32_t* err) {
    const int tid = threadIdx.x, nthreads = blockDim.x, lane = tid & 63;
    int* s_end = s_state;                     // per sum: the window still to look at is tiles [end - 64, end); 0 = done
    __syncthreads();
    for (int i = tid; i < c.width; i += nthreads) {
        s_excl[i] = 0;
        s_end[i] = tile;
        if (tile > 0) store_desc(c.desc + (int64_t)i * c.n_tiles + tile, kDescOwn | (unsigned long long)(unsigned)s_own[i]);
    }
    __syncthreads();
    if (tile > 0 && tid < 64) {
        // wavefront 0 walks every sum's chain; lane l looks at tile end - 1 - l
        for (unsigned spins = 0;; ++spins) {
            bool all_done = true;
            for (int i0 = 0; i0 < c.width; i0 += 8) {
                unsigned long long v[8];
                int end[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {  // the loads of 8 chains go out together
                    const int i = i0 + j;
                    end[j] = i < c.width ? s_end[i] : 0;
                    const int t = end[j] - 1 - lane;
                    v[j] = kDescPrefix;        // before tile 0: an inclusive prefix of 0
                    if (end[j] > 0 && t >= 0) v[j] = load_desc(c.desc + (int64_t)i * c.n_tiles + t);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (end[j] <= 0) continue;  // uniform: this sum is complete (or past the width)
                    const int state = (int)(v[j] >> 62);
                    const unsigned long long have_pre = __ballot(state == 2);
                    const unsigned long long missing = __ballot(state == 0);
                    const int first_pre = have_pre ? __ffsll((long long)have_pre) - 1 : 64;
                    const unsigned long long needed = first_pre >= 63 ? ~0ull : ((2ull << first_pre) - 1ull);
                    if (missing & needed) {  // a tile nearer than the nearest prefix has nothing yet: ask again
                        all_done = false;
                        continue;
                    }
                    int sum = lane <= first_pre ? (int)(v[j] & kDescValue) : 0;
#pragma unroll
                    for (int d = 32; d > 0; d >>= 1) sum += __shfl_xor(sum, d, 64);
                    if (lane == 0) {
                        s_excl[i0 + j] += sum;
                        s_end[i0 + j] = first_pre < 64 ? 0 : end[j] - 64;  // no prefix in the window: go on further back
                    }
                    if (first_pre >= 64) all_done = false;
                }
            }
            if (all_done) break;
            if (spins > kSpinLimit) {
                if (lane == 0) atomicOr(err, kErrLookback);
                break;  // gave up: results are garbage, the error bit says so
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    __syncthreads();
    for (int i = tid; i < c.width; i += nthreads)
        store_desc(c.desc + (int64_t)i * c.n_tiles + tile, kDescPrefix | (unsigned long long)(unsigned)(s_excl[i] + s_own[i]));
}

}  // namespace sp
