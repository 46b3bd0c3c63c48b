// Device-side open-addressing hash table on 64-bit packed coordinates (the GPU hashmap of Sec. III-B,
// used for the insertions and searches of step 2).  One slot is 16 bytes {key, first, row}, so a search
// resolves key and row with a single 16-byte access.
//
// The table is made of buckets of 4 slots (64 bytes).  Four coordinates that are neighbours along z (same b,
// x, y, same z / (4 * lattice step)) hash to the same bucket and have the slot given by their position in
// that group of four as home slot; collisions are resolved by plain linear probing over all slots, so the
// table fills evenly even when the coordinates use one position only (a plane of constant z).  The kernel-map search
// asks for a voxel's neighbours along z in one thread, so its 2-3 searches usually fall into one 64-byte line
// instead of 2-3 random ones: these searches are bound by the rate of random line fetches.
// zshift = floor(log2(lattice step)): which two bits of z number the four group members.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sp {

constexpr uint64_t kEmptyKey = ~0ull;
constexpr int32_t kNoRow = 0x7fffffff;

struct __align__(16) HashSlot {
    unsigned long long key;  // packed (b,x,y,z) or kEmptyKey
    int32_t first;           // smallest source row that carried this key (atomicMin while inserting)
    int32_t row;             // row number of the key among the distinct coordinates
};

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

// home bucket and slot position of a key (cap slots = cap / 4 buckets, cap a power of two >= 4)
__device__ __forceinline__ void hash_home(uint64_t key, uint32_t cap, int zshift, uint32_t* bucket, uint32_t* pos) {
    *pos = (uint32_t)(key >> zshift) & 3u;
    *bucket = hash_key(key & ~(3ull << zshift)) & (cap / 4 - 1);
}

// Insert-or-find.  Returns the slot of `key`, or -1 if the table is full (never at load factor <= 0.5).
// *fresh: this call put the key in (otherwise it was there, or arrived from another thread meanwhile).
__device__ __forceinline__ int64_t hash_insert(HashSlot* __restrict__ tab, uint32_t cap, int zshift, uint64_t key,
                                               bool* fresh) {
    uint32_t bucket, pos;
    hash_home(key, cap, zshift, &bucket, &pos);
    uint32_t slot = bucket * 4 + pos;
    *fresh = false;
    for (uint32_t probe = 0; probe < cap; ++probe) {
        unsigned long long cur = tab[slot].key;
        if (cur == key) return slot;
        if (cur == kEmptyKey) {
            unsigned long long prev = atomicCAS(&tab[slot].key, (unsigned long long)kEmptyKey, (unsigned long long)key);
            *fresh = prev == kEmptyKey;
            if (prev == kEmptyKey || prev == key) return slot;
        }
        slot = (slot + 1) & (cap - 1);
    }
    return -1;
}

// Row number stored for `key`, or -1 when absent.  One 16-byte load per probed slot.
__device__ __forceinline__ int32_t hash_find(const HashSlot* __restrict__ tab, uint32_t cap, int zshift, uint64_t key) {
    uint32_t bucket, pos;
    hash_home(key, cap, zshift, &bucket, &pos);
    uint32_t slot = bucket * 4 + pos;
    for (uint32_t probe = 0; probe < cap; ++probe) {
        const uint4 raw = *reinterpret_cast<const uint4*>(&tab[slot]);
        const unsigned long long cur = ((unsigned long long)raw.y << 32) | raw.x;
        if (cur == key) return (int32_t)raw.w;
        if (cur == kEmptyKey) return -1;
        slot = (slot + 1) & (cap - 1);
    }
    return -1;
}

}  // namespace sp
