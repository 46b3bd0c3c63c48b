// Coordinate sets: hash insertion, duplicate merging in first-occurrence order, strided (coarser)
// coordinate generation.  Sec. III-B: sparse tensor definition and step 1.
#include "sp_hash.h"
#include "sp_internal.h"

namespace sp {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ int32_t floor_to_multiple(int32_t v, int32_t s) {
    int32_t q = v / s;
    if ((v % s != 0) && (v < 0)) --q;  // s > 0: true floor, not truncation
    return q * s;
}

__global__ __launch_bounds__(kThreads) void fill_table_kernel(unsigned long long* __restrict__ keys,
                                                              int32_t* __restrict__ vals, uint32_t cap) {
    uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < cap) {
        keys[i] = kEmptyKey;
        vals[i] = kNoRow;
    }
}

__global__ __launch_bounds__(kThreads) void zero_i32_kernel(int32_t* __restrict__ p, int n) {
    int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Every source row inserts its key; the slot's value becomes the smallest source row carrying that key.
__global__ __launch_bounds__(kThreads) void insert_kernel(const int4* __restrict__ src, int64_t n, int32_t floor_step,
                                                          unsigned long long* __restrict__ keys,
                                                          int32_t* __restrict__ vals, uint32_t cap,
                                                          int32_t* __restrict__ slot_of, int32_t* __restrict__ err) {
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    int4 c = src[i];
    if (floor_step > 1) {
        c.y = floor_to_multiple(c.y, floor_step);
        c.z = floor_to_multiple(c.z, floor_step);
        c.w = floor_to_multiple(c.w, floor_step);
    }
    uint64_t key;
    if (!pack_key(c.x, c.y, c.z, c.w, &key)) {
        atomicOr(err, 1);
        slot_of[i] = -1;
        return;
    }
    int64_t slot = hash_insert(keys, cap, key);
    if (slot < 0) {
        atomicOr(err, 2);
        slot_of[i] = -1;
        return;
    }
    atomicMin(&vals[slot], (int32_t)i);
    slot_of[i] = (int32_t)slot;
}

__global__ __launch_bounds__(kThreads) void flag_first_kernel(const int32_t* __restrict__ slot_of,
                                                              const int32_t* __restrict__ vals, int64_t n,
                                                              int32_t* __restrict__ flags) {
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    int32_t s = slot_of[i];
    flags[i] = (s >= 0 && vals[s] == (int32_t)i) ? 1 : 0;
}

// First occurrences write their (floored) row at their rank and relabel the table slot with that rank.
// `flags` was fixed by the previous kernel, so relabelling in place cannot disturb another thread's test.
__global__ __launch_bounds__(kThreads) void emit_first_kernel(const int4* __restrict__ src, int64_t n,
                                                              int32_t floor_step, const int32_t* __restrict__ slot_of,
                                                              const int32_t* __restrict__ flags,
                                                              const int32_t* __restrict__ rank,
                                                              int4* __restrict__ coords, int32_t* __restrict__ vals) {
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n || !flags[i]) return;
    int4 c = src[i];
    if (floor_step > 1) {
        c.y = floor_to_multiple(c.y, floor_step);
        c.z = floor_to_multiple(c.z, floor_step);
        c.w = floor_to_multiple(c.w, floor_step);
    }
    int32_t r = rank[i];
    coords[r] = c;
    vals[slot_of[i]] = r;
}

__global__ __launch_bounds__(kThreads) void inverse_kernel(const int32_t* __restrict__ slot_of,
                                                           const int32_t* __restrict__ vals, int64_t n,
                                                           int32_t* __restrict__ inverse) {
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    int32_t s = slot_of[i];
    inverse[i] = s >= 0 ? vals[s] : -1;
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

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
    c->tab.keys = dev_alloc((size_t)cap * 8);
    c->tab.vals = dev_alloc((size_t)cap * 4);
    c->coords = dev_alloc((size_t)(n_src ? n_src : 1) * 16);
    c->inverse = dev_alloc((size_t)(n_src ? n_src : 1) * 4);
    Buf slot_of = dev_alloc((size_t)(n_src ? n_src : 1) * 4);
    Buf flags = dev_alloc((size_t)(n_src ? n_src : 1) * 4);
    Buf small = dev_alloc(8);  // [0] total, [1] error bits
    if (!c->tab.keys || !c->tab.vals || !c->coords || !c->inverse || !slot_of || !flags || !small) return SP_ERR_ALLOC;
    auto* keys = ptr<unsigned long long>(c->tab.keys);
    auto* vals = ptr<int32_t>(c->tab.vals);
    int32_t* d_small = ptr<int32_t>(small);

    hipLaunchKernelGGL(fill_table_kernel, dim3(blocks_for(cap)), dim3(kThreads), 0, s, keys, vals, cap);
    hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(kThreads), 0, s, d_small, 2);
    int32_t host_small[2] = {0, 0};
    if (n_src > 0) {
        const int4* src = reinterpret_cast<const int4*>(d_src);
        hipLaunchKernelGGL(insert_kernel, dim3(blocks_for(n_src)), dim3(kThreads), 0, s, src, n_src, floor_step, keys,
                           vals, cap, ptr<int32_t>(slot_of), d_small + 1);
        hipLaunchKernelGGL(flag_first_kernel, dim3(blocks_for(n_src)), dim3(kThreads), 0, s, ptr<int32_t>(slot_of),
                           vals, n_src, ptr<int32_t>(flags));
        Buf rank = dev_alloc((size_t)n_src * 4);
        if (!rank) return SP_ERR_ALLOC;
        SP_TRY(exclusive_scan_i32(ptr<int32_t>(flags), ptr<int32_t>(rank), n_src, d_small, s));
        hipLaunchKernelGGL(emit_first_kernel, dim3(blocks_for(n_src)), dim3(kThreads), 0, s, src, n_src, floor_step,
                           ptr<int32_t>(slot_of), ptr<int32_t>(flags), ptr<int32_t>(rank),
                           ptr<int4>(c->coords), vals);
        hipLaunchKernelGGL(inverse_kernel, dim3(blocks_for(n_src)), dim3(kThreads), 0, s, ptr<int32_t>(slot_of), vals,
                           n_src, ptr<int32_t>(c->inverse));
        SP_HIP(hipGetLastError());
    }
    SP_TRY(read_back(host_small, d_small, 8, s));
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
