// Coordinate sets: hash insertion, duplicate merging in first-occurrence order, strided (coarser)
// coordinate generation.  Sec. III-B: sparse tensor definition and step 1.
//
// Four launches, no host round trip: (1) reset the table and the bookkeeping words; (2) insert every row
// (slot.first = smallest row carrying the key); (3) number the first occurrences in row order in a single pass
// (every block of 1024 rows counts its first occurrences, gets the count of all earlier blocks by decoupled
// look-back, ranks its rows with ballots, writes coordinates + row numbers; the last block writes the row count
// N to device memory for later kernels and to a mail slot for the host); (4) read the row numbers back per
// source row (the inverse map).  The host learns N when it first asks (coords_resolve).
#include <algorithm>

#include "sp_hash.h"
#include "sp_internal.h"
#include "sp_lookback.h"

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

// the source row count: a host value, or a count in device memory that the host has not seen yet
__device__ __forceinline__ int64_t row_count(int64_t n_host, const int32_t* __restrict__ d_n) {
    return d_n ? (int64_t)*d_n : n_host;
}

// table slots <- empty; meta words and look-back words <- 0
__global__ __launch_bounds__(kThreads) void reset_kernel(HashSlot* __restrict__ tab, uint32_t cap,
                                                         int32_t* __restrict__ meta, unsigned long long* __restrict__ desc,
                                                         int64_t n_desc) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < cap) {
        uint4 v;
        v.x = 0xffffffffu;
        v.y = 0xffffffffu;
        v.z = (uint32_t)kNoRow;
        v.w = (uint32_t)-1;
        *reinterpret_cast<uint4*>(&tab[i]) = v;
    }
    if (i < kMetaWords) meta[i] = 0;
    if (i < n_desc) desc[i] = 0ull;
}

// Every source row inserts its key; slot.first becomes the smallest source row carrying that key.
__global__ __launch_bounds__(kThreads) void insert_kernel(const int4* __restrict__ src, int64_t n_host,
                                                          const int32_t* __restrict__ d_n, int32_t floor_step,
                                                          HashSlot* __restrict__ tab, uint32_t cap, int zshift,
                                                          int32_t* __restrict__ slot_of, int32_t* __restrict__ err, int always) {
    const int64_t n = row_count(n_host, d_n);
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

// Block t numbers the first occurrences among rows [t*1024, t*1024+1024): rank = (first
// occurrences in earlier blocks, by look-back) + (those before it in this block, row order).  Writes the
// (floored) coordinates at that rank and the rank into the table slot.  The block holding the last rows
// delivers the total.
__global__ __launch_bounds__(kThreads) void number_kernel(const int4* __restrict__ src, int64_t n_host,
                                                          const int32_t* __restrict__ d_n, int32_t floor_step,
                                                          HashSlot* __restrict__ tab, const int32_t* __restrict__ slot_of,
                                                          Chain chain, int32_t* __restrict__ meta, int4* __restrict__ coords,
                                                          uint32_t* __restrict__ mail, uint32_t mail_seq) {
    __shared__ int s_own[1], s_excl[1], s_state[2];
    __shared__ int s_row[kRowsPerThread][kThreads / 64];
    const int64_t n = row_count(n_host, d_n);
    const int64_t nb = (n + kBlockRows - 1) / kBlockRows;
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (t >= nb) {
        if (t == 0 && threadIdx.x == 0) {  // no rows at all: block 0 reports N = 0
            meta[kMetaN] = 0;
            if (mail) {
                mail[0] = 0u;
                mail[1] = (uint32_t)meta[kMetaErr];
                __threadfence_system();
                __hip_atomic_store(mail + kMailSeqWord, mail_seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
        return;
    }
    const int64_t base = (int64_t)t * kBlockRows;
    bool f[kRowsPerThread];
    int pos[kRowsPerThread];
#pragma unroll
    for (int j = 0; j < kRowsPerThread; ++j) {
        const int64_t i = base + j * kThreads + threadIdx.x;
        bool first = false;
        if (i < n) {
            const int32_t s = slot_of[i];
            first = s >= 0 && tab[s].first == (int32_t)i;
        }
        const unsigned long long m = __ballot(first);
        f[j] = first;
        pos[j] = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) s_row[j][w] = __popcll(m);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int c = 0;
        for (int j = 0; j < kRowsPerThread; ++j)
            for (int ww = 0; ww < kThreads / 64; ++ww) c += s_row[j][ww];
        s_own[0] = c;
    }
    chain_lookback(chain, t, s_own, s_excl, s_state, meta + kMetaErr);
    int run = s_excl[0];
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
    if (t == nb - 1 && threadIdx.x == 0) {
        meta[kMetaN] = run;
        if (mail) {
            mail[0] = (uint32_t)run;
            mail[1] = (uint32_t)__hip_atomic_load(meta + kMetaErr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __threadfence_system();
            __hip_atomic_store(mail + kMailSeqWord, mail_seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

__global__ __launch_bounds__(kThreads) void inverse_kernel(const HashSlot* __restrict__ tab,
                                                           const int32_t* __restrict__ slot_of, int64_t n_host,
                                                           const int32_t* __restrict__ d_n, int32_t* __restrict__ inverse) {
    const int64_t n = row_count(n_host, d_n);
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const int32_t s = slot_of[i];
    inverse[i] = s >= 0 ? tab[s].row : -1;
}

inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

int coords_build_impl(const int32_t* d_src, int64_t n_src, const int32_t* d_n_src, int32_t floor_step,
                      int32_t tensor_stride, hipStream_t s, sp_coords_t** out) {
    if (n_src >= (int64_t)1 << 30) return fail(SP_ERR_INVALID_ARG, "too many rows (%lld)", (long long)n_src);
    std::unique_ptr<sp_coords> c(new sp_coords);
    c->n_raw = n_src;
    c->ts = tensor_stride;
    c->stream = s;
    uint32_t cap = 1024;
    while ((int64_t)cap < 2 * n_src) cap <<= 1;
    c->tab.cap = cap;
    for (int t = tensor_stride; t > 1; t >>= 1) ++c->tab.zshift;
    const int64_t nb = (n_src + kBlockRows - 1) / kBlockRows;
    c->tab.slots = dev_alloc((size_t)cap * sizeof(HashSlot), s);
    c->coords = dev_alloc((size_t)(n_src ? n_src : 1) * 16, s);
    c->inverse = dev_alloc((size_t)(n_src ? n_src : 1) * 4, s);
    c->meta = dev_alloc(kMetaWords * 4, s);
    Buf slot_of = dev_alloc((size_t)(n_src ? n_src : 1) * 4, s);
    Buf chain_mem = dev_alloc((size_t)(nb ? nb : 1) * 8, s);  // one look-back word per numbering block
    if (!c->tab.slots || !c->coords || !c->inverse || !c->meta || !slot_of || !chain_mem) return SP_ERR_ALLOC;
    HashSlot* tab = ptr<HashSlot>(c->tab.slots);
    int32_t* meta = ptr<int32_t>(c->meta);
    Chain chain;
    chain.desc = ptr<unsigned long long>(chain_mem);
    chain.n_tiles = nb ? nb : 1;
    chain.width = 1;
    const bool mailed = mail_acquire(&c->mail);

    hipLaunchKernelGGL(reset_kernel, dim3(blocks_for(std::max<int64_t>(cap, nb), kThreads)), dim3(kThreads), 0, s, tab, cap, meta,
                       chain.desc, nb);
    const int4* src = reinterpret_cast<const int4*>(d_src);
    if (n_src > 0)
        hipLaunchKernelGGL(insert_kernel, dim3(blocks_for(n_src, kThreads)), dim3(kThreads), 0, s, src, n_src, d_n_src,
                           floor_step, tab, cap, c->tab.zshift, ptr<int32_t>(slot_of), meta + kMetaErr,
                           n_src < (1 << 20) ? 1 : 0);
    hipLaunchKernelGGL(number_kernel, dim3((unsigned)(nb ? nb : 1)), dim3(kThreads), 0, s, src, n_src, d_n_src, floor_step, tab,
                       ptr<int32_t>(slot_of), chain, meta, ptr<int4>(c->coords), mailed ? c->mail.d : (uint32_t*)nullptr,
                       c->mail.seq);
    c->mail.armed = mailed;
    c->mail.stream = s;
    if (n_src > 0)
        hipLaunchKernelGGL(inverse_kernel, dim3(blocks_for(n_src, kThreads)), dim3(kThreads), 0, s, tab, ptr<int32_t>(slot_of),
                           n_src, d_n_src, ptr<int32_t>(c->inverse));
    SP_HIP(hipGetLastError());
    if (!mailed) {  // no mail slot free: wait here, the old way
        int32_t h[2] = {0, 0};
        SP_TRY(read_back(h, meta, 8, s));
        c->n = h[0];
        c->status = (h[1] & 1) ? SP_ERR_RANGE : (h[1] & 2) ? SP_ERR_TABLE_FULL : (h[1] & kErrLookback) ? SP_ERR_HIP : SP_OK;
        c->resolved = true;
    }
    *out = c.release();
    return SP_OK;
}

static int status_message(int status) {
    if (status == SP_ERR_RANGE) return fail(SP_ERR_RANGE, "a coordinate is outside 0 <= b < 65536, -32768 <= x,y,z < 32768");
    if (status == SP_ERR_TABLE_FULL) return fail(SP_ERR_TABLE_FULL, "hash table overflow");
    if (status == SP_ERR_HIP) return fail(SP_ERR_HIP, "internal: a look-back wait gave up");
    return status;
}

int coords_resolve(const sp_coords_t* c) {
    std::lock_guard<std::mutex> lk(c->mu);
    if (!c->resolved) {
        SP_TRY(mail_wait(c->mail, c->stream));
        const uint32_t n = c->mail.h[0], e = c->mail.h[1];
        c->n = (int64_t)n;
        c->status = (e & 1) ? SP_ERR_RANGE : (e & 2) ? SP_ERR_TABLE_FULL : (e & kErrLookback) ? SP_ERR_HIP : SP_OK;
        c->resolved = true;
        mail_release(&c->mail);
    }
    return status_message(c->status);
}

}  // namespace sp

sp_coords::~sp_coords() {
    sp::mail_release(&mail);
    if (src_of) sp_coords_destroy(src_of);
}

extern "C" {

int sp_coords_build(const int32_t* d_raw, int64_t n_raw, int32_t tensor_stride, void* stream, sp_coords_t** out) {
    if (!out) return sp::fail(SP_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (n_raw < 0) return sp::fail(SP_ERR_INVALID_ARG, "n_raw < 0");
    if (n_raw > 0 && !d_raw) return sp::fail(SP_ERR_INVALID_ARG, "d_raw is NULL");
    if (tensor_stride < 1) return sp::fail(SP_ERR_INVALID_ARG, "tensor_stride < 1");
    if (((uintptr_t)d_raw & 15) != 0) return sp::fail(SP_ERR_INVALID_ARG, "d_raw must be 16-byte aligned");
    return sp::coords_build_impl(d_raw, n_raw, nullptr, 1, tensor_stride, (hipStream_t)stream, out);
}

int sp_coords_size(const sp_coords_t* c, int64_t* n, int32_t* tensor_stride) {
    if (!c) return sp::fail(SP_ERR_INVALID_ARG, "coords handle is NULL");
    if (tensor_stride) *tensor_stride = c->ts;
    if (n) {
        SP_TRY(sp::coords_resolve(c));
        *n = c->n;
    }
    return SP_OK;
}

int sp_coords_data(const sp_coords_t* c, const int32_t** d_coords, const int32_t** d_inverse, int64_t* n_raw) {
    if (!c) return sp::fail(SP_ERR_INVALID_ARG, "coords handle is NULL");
    if (d_coords) *d_coords = sp::ptr<int32_t>(c->coords);
    if (d_inverse) *d_inverse = sp::ptr<int32_t>(c->inverse);
    if (n_raw) {
        *n_raw = c->n_raw;
        if (c->src_of) {  // derived from a set whose row count may have been unknown then: its rows are the source rows
            SP_TRY(sp::coords_resolve(c->src_of));
            *n_raw = c->src_of->n;
        }
    }
    return SP_OK;
}

int sp_coords_destroy(sp_coords_t* c) {
    if (!c) return SP_OK;
    if (c->ref.fetch_sub(1) == 1) delete c;
    return SP_OK;
}

}  // extern "C"
