// Pooling over a kernel map: Eq. 2 with the weighted sum replaced by a reduction over the same neighbour set
// (the pooling layers that sit between the SparseConv blocks, Sec. III figure caption).  Both directions are
// destination-row stationary walks of the neighbour table: no atomics, fixed order, reproducible bits.
//   forward:  y[o,c]  = max / sum / mean over k with i = nbr_out[k][o] >= 0 of x[i,c]
//   backward: dx[i,c] = sum over k with o = nbr_in[k][i] >= 0 of  dy[o,c] * (max: the link is the one that gave
//             the maximum | sum: 1 | mean: 1 / links of o)
// Memory bound: a row of c channels is gathered once per link.
#include <mutex>

#include "sp_internal.h"

namespace sp {
namespace {

typedef uint16_t bf16_t;
constexpr int kThreads = 256;
constexpr uint8_t kNoArg = 255;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ void from_f32(float f, float* o) { *o = f; }
__device__ __forceinline__ void from_f32(float f, bf16_t* o) {  // round to nearest even; NaN stays NaN
    uint32_t u = __float_as_uint(f);
    *o = (u & 0x7fffffffu) > 0x7f800000u ? (bf16_t)((u >> 16) | 0x40) : (bf16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// V channels (16 bytes) of one row
template <typename T, int V>
struct Vec {
    T v[V];
};
template <typename T, int V>
__device__ __forceinline__ Vec<T, V> load_vec(const T* p) {
    Vec<T, V> r;
    if constexpr (V * sizeof(T) == 16) {
        const uint4 raw = *reinterpret_cast<const uint4*>(p);
        __builtin_memcpy(&r, &raw, 16);
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) r.v[i] = p[i];
    }
    return r;
}
template <typename T, int V>
__device__ __forceinline__ void store_vec(T* p, const Vec<T, V>& r) {
    if constexpr (V * sizeof(T) == 16) {
        uint4 raw;
        __builtin_memcpy(&raw, &r, 16);
        *reinterpret_cast<uint4*>(p) = raw;
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) p[i] = r.v[i];
    }
}

// links per destination row of a neighbour table
__global__ __launch_bounds__(kThreads) void link_count_kernel(const int32_t* __restrict__ nbr, int64_t n_rows, int kvol,
                                                              int32_t* __restrict__ cnt) {
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r >= n_rows) return;
    int c = 0;
    for (int k = 0; k < kvol; ++k) c += nbr[(int64_t)k * n_rows + r] >= 0 ? 1 : 0;
    cnt[r] = c;
}

// Thread = (destination row, piece of V channels); c = pieces * V.  Offsets are visited in ascending TRUE
// offset number (a table derived by the stride-1 symmetry holds offset kvol-1-kk in block kk), so that among
// equal maxima the lowest offset number wins.
template <typename T, int V, int MODE>
__global__ __launch_bounds__(kThreads) void pool_fwd_kernel(const int32_t* __restrict__ nbr, int64_t n_rows, int kvol,
                                                            int flip, const T* __restrict__ x, int c, int pieces,
                                                            T* __restrict__ y, uint8_t* __restrict__ arg) {
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= n_rows * pieces) return;
    const int64_t row = t / pieces;
    const int c0 = (int)(t % pieces) * V;
    float acc[V];
    uint8_t best[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
        acc[i] = 0.f;
        best[i] = kNoArg;
    }
    int links = 0;
    for (int k = 0; k < kvol; ++k) {
        const int kk = flip ? kvol - 1 - k : k;
        const int32_t src = nbr[(int64_t)kk * n_rows + row];
        if (src < 0) continue;
        ++links;
        const Vec<T, V> v = load_vec<T, V>(x + (size_t)src * c + c0);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float f = to_f32(v.v[i]);
            if constexpr (MODE == SP_POOL_MAX) {
                if (best[i] == kNoArg || f > acc[i]) {
                    acc[i] = f;
                    best[i] = (uint8_t)k;
                }
            } else {
                acc[i] += f;
            }
        }
    }
    Vec<T, V> out;
    const float scale = (MODE == SP_POOL_AVG && links > 0) ? 1.f / (float)links : 1.f;
#pragma unroll
    for (int i = 0; i < V; ++i) from_f32(MODE == SP_POOL_AVG ? acc[i] * scale : acc[i], &out.v[i]);
    store_vec<T, V>(y + (size_t)row * c + c0, out);
    if (MODE == SP_POOL_MAX && arg) {
#pragma unroll
        for (int i = 0; i < V; ++i) arg[(size_t)row * c + c0 + i] = best[i];
    }
}

// Thread = (input row, piece).  nbr is the input side's table: nbr[kk][i] = output row linked at (table block kk).
template <typename T, int V, int MODE>
__global__ __launch_bounds__(kThreads) void pool_bwd_kernel(const int32_t* __restrict__ nbr, int64_t n_rows, int kvol,
                                                            int flip, const T* __restrict__ dy, const uint8_t* __restrict__ arg,
                                                            const int32_t* __restrict__ link_cnt, int c, int pieces,
                                                            T* __restrict__ dx) {
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= n_rows * pieces) return;
    const int64_t row = t / pieces;
    const int c0 = (int)(t % pieces) * V;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    for (int k = 0; k < kvol; ++k) {
        const int kk = flip ? kvol - 1 - k : k;
        const int32_t o = nbr[(int64_t)kk * n_rows + row];
        if (o < 0) continue;
        const Vec<T, V> g = load_vec<T, V>(dy + (size_t)o * c + c0);
        if constexpr (MODE == SP_POOL_MAX) {
            const uint8_t* a = arg + (size_t)o * c + c0;
#pragma unroll
            for (int i = 0; i < V; ++i)
                if (a[i] == (uint8_t)k) acc[i] += to_f32(g.v[i]);
        } else if constexpr (MODE == SP_POOL_AVG) {
            const float scale = 1.f / (float)link_cnt[o];  // o has at least this link
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] += to_f32(g.v[i]) * scale;
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] += to_f32(g.v[i]);
        }
    }
    Vec<T, V> out;
#pragma unroll
    for (int i = 0; i < V; ++i) from_f32(acc[i], &out.v[i]);
    store_vec<T, V>(dx + (size_t)row * c + c0, out);
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

template <typename T, int V>
int fwd_typed(const MapSide& side, int kvol, const void* x, void* y, uint8_t* arg, int c, int mode, hipStream_t s) {
    const int pieces = c / V;
    const int64_t n = side.n_rows * pieces;
    if (n == 0) return SP_OK;
    const dim3 g(blocks_for(n)), b(kThreads);
    const int32_t* nbr = ptr<int32_t>(side.nbr);
    const int flip = side.flip ? 1 : 0;
#define SP_GO(M)                                                                                                    \
    hipLaunchKernelGGL((pool_fwd_kernel<T, V, M>), g, b, 0, s, nbr, side.n_rows, kvol, flip, static_cast<const T*>(x), c, \
                       pieces, static_cast<T*>(y), arg)
    if (mode == SP_POOL_MAX) SP_GO(SP_POOL_MAX);
    else if (mode == SP_POOL_AVG) SP_GO(SP_POOL_AVG);
    else SP_GO(SP_POOL_SUM);
#undef SP_GO
    SP_HIP(hipGetLastError());
    return SP_OK;
}

template <typename T, int V>
int bwd_typed(const MapSide& side, int kvol, const void* dy, const uint8_t* arg, const int32_t* cnt, void* dx, int c,
              int mode, hipStream_t s) {
    const int pieces = c / V;
    const int64_t n = side.n_rows * pieces;
    if (n == 0) return SP_OK;
    const dim3 g(blocks_for(n)), b(kThreads);
    const int32_t* nbr = ptr<int32_t>(side.nbr);
    const int flip = side.flip ? 1 : 0;
#define SP_GO(M)                                                                                                     \
    hipLaunchKernelGGL((pool_bwd_kernel<T, V, M>), g, b, 0, s, nbr, side.n_rows, kvol, flip, static_cast<const T*>(dy), arg, \
                       cnt, c, pieces, static_cast<T*>(dx))
    if (mode == SP_POOL_MAX) SP_GO(SP_POOL_MAX);
    else if (mode == SP_POOL_AVG) SP_GO(SP_POOL_AVG);
    else SP_GO(SP_POOL_SUM);
#undef SP_GO
    SP_HIP(hipGetLastError());
    return SP_OK;
}

int check_pool_args(const sp_kmap_t* m, const void* a, int64_t rows_a, const void* b, int64_t rows_b, int c, int mode,
                    sp_dtype dt) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (c < 1 || c > 65536) return fail(SP_ERR_INVALID_ARG, "bad channel count");
    if (dt != SP_F32 && dt != SP_BF16) return fail(SP_ERR_INVALID_ARG, "bad dtype");
    if (mode != SP_POOL_MAX && mode != SP_POOL_AVG && mode != SP_POOL_SUM) return fail(SP_ERR_INVALID_ARG, "bad pooling mode");
    if (m->kvol > 254) return fail(SP_ERR_UNSUPPORTED, "kernel volume above 254");
    if ((!a && rows_a > 0) || (!b && rows_b > 0)) return fail(SP_ERR_INVALID_ARG, "a feature pointer is NULL");
    return SP_OK;
}

// 16-byte vectors when the channel count and the pointers allow it, else one channel per thread
bool vector_ok(const void* a, const void* b, int c, sp_dtype dt) {
    const int v = dt == SP_F32 ? 4 : 8;
    return c % v == 0 && (((uintptr_t)a | (uintptr_t)b) & 15) == 0;
}

}  // namespace
}  // namespace sp

using namespace sp;

extern "C" {

int sp_pool_fwd(const sp_kmap_t* m, const void* d_x, void* d_y, uint8_t* d_arg, int32_t c, sp_pool_mode mode, sp_dtype dt,
                void* stream) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    SP_TRY(kmap_resolve(m));
    SP_TRY(check_pool_args(m, d_x, m->n_in, d_y, m->n_out, c, mode, dt));
    hipStream_t s = (hipStream_t)stream;
    const MapSide& side = m->out_side;
    if (vector_ok(d_x, d_y, c, dt))
        return dt == SP_F32 ? fwd_typed<float, 4>(side, m->kvol, d_x, d_y, d_arg, c, mode, s)
                            : fwd_typed<bf16_t, 8>(side, m->kvol, d_x, d_y, d_arg, c, mode, s);
    return dt == SP_F32 ? fwd_typed<float, 1>(side, m->kvol, d_x, d_y, d_arg, c, mode, s)
                        : fwd_typed<bf16_t, 1>(side, m->kvol, d_x, d_y, d_arg, c, mode, s);
}

int sp_pool_bwd(const sp_kmap_t* m, const void* d_dy, const uint8_t* d_arg, void* d_dx, int32_t c, sp_pool_mode mode,
                sp_dtype dt, void* stream) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    SP_TRY(kmap_resolve(m));
    SP_TRY(check_pool_args(m, d_dy, m->n_out, d_dx, m->n_in, c, mode, dt));
    if (mode == SP_POOL_MAX && !d_arg && m->n_out > 0) return fail(SP_ERR_INVALID_ARG, "max pooling backward needs d_arg");
    hipStream_t s = (hipStream_t)stream;
    const MapSide& side = m->in_side;
    const int32_t* cnt = nullptr;
    if (mode == SP_POOL_AVG && m->n_out > 0) {
        // links per output row: counted once per handle, on the first call that needs them
        std::lock_guard<std::mutex> lk(m->cache_mu);
        if (!m->out_link_cnt) {
            m->out_link_cnt = dev_alloc((size_t)m->n_out * 4, s);
            if (!m->out_link_cnt) return SP_ERR_ALLOC;
            hipLaunchKernelGGL(link_count_kernel, dim3(blocks_for(m->n_out)), dim3(kThreads), 0, s,
                               ptr<int32_t>(m->out_side.nbr), m->n_out, m->kvol, ptr<int32_t>(m->out_link_cnt));
            SP_HIP(hipGetLastError());
        }
        cnt = ptr<int32_t>(m->out_link_cnt);
    }
    if (vector_ok(d_dy, d_dx, c, dt))
        return dt == SP_F32 ? bwd_typed<float, 4>(side, m->kvol, d_dy, d_arg, cnt, d_dx, c, mode, s)
                            : bwd_typed<bf16_t, 8>(side, m->kvol, d_dy, d_arg, cnt, d_dx, c, mode, s);
    return dt == SP_F32 ? bwd_typed<float, 1>(side, m->kvol, d_dy, d_arg, cnt, d_dx, c, mode, s)
                        : bwd_typed<bf16_t, 1>(side, m->kvol, d_dy, d_arg, cnt, d_dx, c, mode, s);
}

}  // extern "C"
