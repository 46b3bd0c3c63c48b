// Device-side open-addressing hash table on 64-bit packed coordinates (the GPU hashmap of Sec. III-B,
// used for the insertions and searches of step 2).  Linear probing; keys are 8 bytes, so the 16 slots
// after the home slot share one 128-byte line and a probe sequence almost always stays inside it.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sp {

constexpr uint64_t kEmptyKey = ~0ull;
constexpr int32_t kNoRow = 0x7fffffff;

// b in [0, 65536), x,y,z in [-32768, 32768).  Returns false when the row cannot be packed.
__device__ __forceinline__ bool pack_key(int32_t b, int32_t x, int32_t y, int32_t z, uint64_t* key) {
    const uint32_t ux = (uint32_t)(x + 32768), uy = (uint32_t)(y + 32768), uz = (uint32_t)(z + 32768);
    const bool ok = ((uint32_t)b < 65536u) & (ux < 65536u) & (uy < 65536u) & (uz < 65536u);
    *key = ((uint64_t)(uint32_t)b << 48) | ((uint64_t)ux << 32) | ((uint64_t)uy << 16) | (uint64_t)uz;
    return ok;
}

__device__ __forceinline__ uint32_t hash_key(uint64_t k) {
    // 64-bit finaliser (xor-shift-multiply), folded to 32 bits
    k ^= k >> 33;
    k *= 0xff51afd7ed558ccdull;
    k ^= k >> 33;
    k *= 0xc4ceb9fe1a85ec53ull;
    k ^= k >> 33;
    return (uint32_t)k;
}

// Insert-or-find.  Returns the slot of `key`, or -1 if the table is full (never at load factor <= 0.5).
__device__ __forceinline__ int64_t hash_insert(unsigned long long* __restrict__ keys, uint32_t cap, uint64_t key) {
    const uint32_t mask = cap - 1;
    uint32_t slot = hash_key(key) & mask;
    for (uint32_t probe = 0; probe < cap; ++probe) {
        unsigned long long cur = keys[slot];
        if (cur == key) return slot;
        if (cur == kEmptyKey) {
            unsigned long long prev = atomicCAS(&keys[slot], (unsigned long long)kEmptyKey, (unsigned long long)key);
            if (prev == kEmptyKey || prev == key) return slot;
        }
        slot = (slot + 1) & mask;
    }
    return -1;
}

// Row index stored for `key`, or -1 when absent.
__device__ __forceinline__ int32_t hash_find(const unsigned long long* __restrict__ keys,
                                             const int32_t* __restrict__ vals, uint32_t cap, uint64_t key) {
    const uint32_t mask = cap - 1;
    uint32_t slot = hash_key(key) & mask;
    for (uint32_t probe = 0; probe < cap; ++probe) {
        unsigned long long cur = keys[slot];
        if (cur == key) return vals[slot];
        if (cur == kEmptyKey) return -1;
        slot = (slot + 1) & mask;
    }
    return -1;
}

}  // namespace sp
