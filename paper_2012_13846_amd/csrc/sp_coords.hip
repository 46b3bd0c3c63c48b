// Coordinate sets: hash insertion, duplicate merging in first-occurrence order, strided (coarser)
// coordinate generation.  Sec. III-B: sparse tensor definition and step 1.
//
// Five launches: fill the table; insert every row (slot.first = smallest row carrying the key); count the
// first occurrences per 1024-row block; number them (each block adds up the counts of the blocks before
// it, then ranks its own rows with ballots) and write coordinates + row numbers; read the row numbers
// back per source row (the inverse map).
#include "sp_hash.h"
#include "sp_internal.h"

namespace sp {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerThread = 4;
constexpr int kBlockRows = kThreads * kRowsPerThread;  // rows numbered by one block

__device__ __forceinline__ int32_t floor_to_multiple(int32_t v, int32_t s) {
    int32_t q = v / s;
    if ((v % s != 0) && (v < 0)) --q;  // s > 0: true floor, not truncation
    return q * s;
}

__device__ __forceinline__ int4 load_row(const int4* __restrict__ src, int64_t i, int32_t floor_step) {
    int4 c = src[i];
    if (floor_step > 1) {
        c.y = floor_to_multiple(c.y, floor_step);
        c.z = floor_to_multiple(c.z, floor_step);
        c.w = floor_to_multiple(c.w, floor_step);
    }
    return c;
}

__global__ __launch_bounds__(kThreads) void fill_table_kernel(HashSlot* __restrict__ tab, uint32_t cap,
                                                              int32_t* __restrict__ small, int n_small) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < cap) {
        uint4 v;
        v.x = 0xffffffffu;
        v.y = 0xffffffffu;
        v.z = (uint32_t)kNoRow;
        v.w = (uint32_t)-1;
        *reinterpret_cast<uint4*>(&tab[i]) = v;
    }
    if (i < (uint32_t)n_small) small[i] = 0;
}

// Every source row inserts its key; slot.first becomes the smallest source row carrying that key.
__global__ __launch_bounds__(kThreads) void insert_kernel(const int4* __restrict__ src, int64_t n, int32_t floor_step,
                                                          HashSlot* __restrict__ tab, uint32_t cap, int zshift,
                                                          int32_t* __restrict__ slot_of, int32_t* __restrict__ err, int always) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const int4 c = load_row(src, i, floor_step);
    uint64_t key;
    if (!pack_key(c.x, c.y, c.z, c.w, &key)) {
        atomicOr(err, 1);
        slot_of[i] = -1;
        return;
    }
    bool fresh;
    const int64_t slot = hash_insert(tab, cap, zshift, key, &fresh);
    if (slot < 0) {
        atomicOr(err, 2);
        slot_of[i] = -1;
        return;
    }
    // A duplicate that sees a smaller row already recorded has nothing to add (the value only ever decreases).
    // Looking first costs a round trip and saves an atomic: measured 5 us slower on 157 k rows, 50 us faster
    // on 4.1 M rows (where the atomics' throughput binds), so the host asks for it from 1 M rows (always = 0).
    if (always || fresh || __builtin_nontemporal_load(&tab[slot].first) > (int32_t)i) atomicMin(&tab[slot].first, (int32_t)i);
    slot_of[i] = (int32_t)slot;
}

__device__ __forceinline__ bool is_first(const HashSlot* __restrict__ tab, const int32_t* __restrict__ slot_of,
                                         int64_t i, int64_t n) {
    if (i >= n) return false;
    const int32_t s = slot_of[i];
    return s >= 0 && tab[s].first == (int32_t)i;
}

// Block b counts the first occurrences among rows [b*1024, b*1024+1024) and keeps them as one bit per row
// (first_mask[row / 64]), so that the numbering pass does not have to look every row up in the table again.
__global__ __launch_bounds__(kThreads) void count_first_kernel(const HashSlot* __restrict__ tab,
                                                               const int32_t* __restrict__ slot_of, int64_t n,
                                                               int32_t* __restrict__ block_counts,
                                                               unsigned long long* __restrict__ first_mask) {
    __shared__ int s_cnt[kThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kBlockRows;
    int c = 0;
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const unsigned long long m = __ballot(is_first(tab, slot_of, base + j * kThreads + threadIdx.x, n));
        if ((threadIdx.x & 63) == 0) first_mask[(base + j * kThreads + threadIdx.x) >> 6] = m;
        c += __popcll(m);
    }
    if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) block_counts[blockIdx.x] = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
}

// Block b numbers its first occurrences: rank = (firsts in earlier blocks) + (firsts before it in this
// block, row order).  Writes the (floored) coordinates at that rank and the rank into the table slot.
// block_base: if `scanned`, block_counts already holds exclusive prefixes.
__global__ __launch_bounds__(kThreads) void emit_first_kernel(const int4* __restrict__ src, int64_t n,
                                                              int32_t floor_step, HashSlot* __restrict__ tab,
                                                              const int32_t* __restrict__ slot_of,
                                                              const int32_t* __restrict__ block_counts, int scanned,
                                                              const unsigned long long* __restrict__ first_mask,
                                                              int4* __restrict__ coords, int32_t* __restrict__ total) {
    __shared__ int s_red[kThreads / 64];
    __shared__ int s_row[kRowsPerThread][kThreads / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // firsts in the blocks before this one
    int before = 0;
    if (scanned) {
        before = block_counts[blockIdx.x];
    } else {
        int s = 0;
        for (int b = threadIdx.x; b < (int)blockIdx.x; b += kThreads) s += block_counts[b];
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) s += __shfl_down(s, d, 64);
        if (lane == 0) s_red[w] = s;
        __syncthreads();
        before = s_red[0] + s_red[1] + s_red[2] + s_red[3];
    }
    const int64_t base = (int64_t)blockIdx.x * kBlockRows;
    bool f[kRowsPerThread];
    int pos[kRowsPerThread];
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const unsigned long long m = first_mask[(base + j * kThreads + threadIdx.x) >> 6];
        f[j] = (m >> lane) & 1ull;
        pos[j] = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) s_row[j][w] = __popcll(m);
    }
    __syncthreads();
    int run = before;
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        int mine = run;
        for (int ww = 0; ww < kThreads / 64; ++ww) {
            if (ww < w) mine += s_row[j][ww];
            run += s_row[j][ww];
        }
        if (f[j]) {
            const int64_t i = base + j * kThreads + threadIdx.x;
            const int32_t r = mine + pos[j];
            coords[r] = load_row(src, i, floor_step);
            tab[slot_of[i]].row = r;
        }
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *total = run;
}

__global__ __launch_bounds__(kThreads) void inverse_kernel(const HashSlot* __restrict__ tab,
                                                           const int32_t* __restrict__ slot_of, int64_t n,
                                                           int32_t* __restrict__ inverse) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const int32_t s = slot_of[i];
    inverse[i] = s >= 0 ? tab[s].row : -1;
}

inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

int coords_build_impl(const int32_t* d_src, int64_t n_src, int32_t floor_step, int32_t tensor_stride, hipStream_t s,
                      sp_coords_t** out) {
    if (n_src >= (int64_t)1 << 30) return fail(SP_ERR_INVALID_ARG, "too many rows (%lld)", (long long)n_src);
    std::unique_ptr<sp_coords> c(new sp_coords);
    c->n_raw = n_src;
    c->ts = tensor_stride;
    uint32_t cap = 1024;
    while ((int64_t)cap < 2 * n_src) cap <<= 1;
    c->tab.cap = cap;
    for (int t = tensor_stride; t > 1; t >>= 1) ++c->tab.zshift;
    c->tab.slots = dev_alloc((size_t)cap * sizeof(HashSlot), s);
    c->coords = dev_alloc((size_t)(n_src ? n_src : 1) * 16, s);
    c->inverse = dev_alloc((size_t)(n_src ? n_src : 1) * 4, s);
    Buf slot_of = dev_alloc((size_t)(n_src ? n_src : 1) * 4, s);
    const int64_t nb = (n_src + kBlockRows - 1) / kBlockRows;
    Buf block_counts = dev_alloc((size_t)(nb ? nb : 1) * 4, s);
    Buf first_mask = dev_alloc((size_t)(nb ? nb : 1) * (kBlockRows / 64) * 8, s);
    Buf small = dev_alloc(8, s);  // [0] total, [1] error bits
    if (!c->tab.slots || !c->coords || !c->inverse || !slot_of || !block_counts || !first_mask || !small) return SP_ERR_ALLOC;
    HashSlot* tab = ptr<HashSlot>(c->tab.slots);
    int32_t* d_small = ptr<int32_t>(small);

    hipLaunchKernelGGL(fill_table_kernel, dim3(blocks_for(cap, kThreads)), dim3(kThreads), 0, s, tab, cap, d_small, 2);
    int32_t host_small[2] = {0, 0};
    if (n_src > 0) {
        const int4* src = reinterpret_cast<const int4*>(d_src);
        hipLaunchKernelGGL(insert_kernel, dim3(blocks_for(n_src, kThreads)), dim3(kThreads), 0, s, src, n_src,
                           floor_step, tab, cap, c->tab.zshift, ptr<int32_t>(slot_of), d_small + 1, n_src < (1 << 20) ? 1 : 0);
        hipLaunchKernelGGL(count_first_kernel, dim3((unsigned)nb), dim3(kThreads), 0, s, tab, ptr<int32_t>(slot_of),
                           n_src, ptr<int32_t>(block_counts), ptr<unsigned long long>(first_mask));
        int scanned = 0;
        if (nb > 4096) {  // too many blocks for every block to add up its predecessors: scan the counts first
            ScanJob job;
            job.data = ptr<int32_t>(block_counts);
            job.n = nb;
            SP_TRY(exclusive_scan_jobs(&job, 1, s));
            scanned = 1;
        }
        hipLaunchKernelGGL(emit_first_kernel, dim3((unsigned)nb), dim3(kThreads), 0, s, src, n_src, floor_step, tab,
                           ptr<int32_t>(slot_of), ptr<int32_t>(block_counts), scanned,
                           ptr<unsigned long long>(first_mask), ptr<int4>(c->coords), d_small);
        SP_HIP(hipGetLastError());
    }
    // the host only waits for N; the inverse array is filled behind the read-back, while the host wakes up
    SP_TRY(read_back(host_small, d_small, 8, s, [&]() {
        if (n_src > 0)
            hipLaunchKernelGGL(inverse_kernel, dim3(blocks_for(n_src, kThreads)), dim3(kThreads), 0, s, tab,
                               ptr<int32_t>(slot_of), n_src, ptr<int32_t>(c->inverse));
    }));
    SP_HIP(hipGetLastError());
    if (host_small[1] & 1)
        return fail(SP_ERR_RANGE, "a coordinate is outside 0 <= b < 65536, -32768 <= x,y,z < 32768");
    if (host_small[1] & 2) return fail(SP_ERR_TABLE_FULL, "hash table overflow");
    c->n = host_small[0];
    *out = c.release();
    return SP_OK;
}

}  // namespace sp

extern "C" {

int sp_coords_build(const int32_t* d_raw, int64_t n_raw, int32_t tensor_stride, void* stream, sp_coords_t** out) {
    if (!out) return sp::fail(SP_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (n_raw < 0) return sp::fail(SP_ERR_INVALID_ARG, "n_raw < 0");
    if (n_raw > 0 && !d_raw) return sp::fail(SP_ERR_INVALID_ARG, "d_raw is NULL");
    if (tensor_stride < 1) return sp::fail(SP_ERR_INVALID_ARG, "tensor_stride < 1");
    if (((uintptr_t)d_raw & 15) != 0) return sp::fail(SP_ERR_INVALID_ARG, "d_raw must be 16-byte aligned");
    return sp::coords_build_impl(d_raw, n_raw, 1, tensor_stride, (hipStream_t)stream, out);
}

int sp_coords_size(const sp_coords_t* c, int64_t* n, int32_t* tensor_stride) {
    if (!c) return sp::fail(SP_ERR_INVALID_ARG, "coords handle is NULL");
    if (n) *n = c->n;
    if (tensor_stride) *tensor_stride = c->ts;
    return SP_OK;
}

int sp_coords_data(const sp_coords_t* c, const int32_t** d_coords, const int32_t** d_inverse, int64_t* n_raw) {
    if (!c) return sp::fail(SP_ERR_INVALID_ARG, "coords handle is NULL");
    if (d_coords) *d_coords = sp::ptr<int32_t>(c->coords);
    if (d_inverse) *d_inverse = sp::ptr<int32_t>(c->inverse);
    if (n_raw) *n_raw = c->n_raw;
    return SP_OK;
}

int sp_coords_destroy(sp_coords_t* c) {
    if (!c) return SP_OK;
    if (c->ref.fetch_sub(1) == 1) delete c;
    return SP_OK;
}

}  // extern "C"
