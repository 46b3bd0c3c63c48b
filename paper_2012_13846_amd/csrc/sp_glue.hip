// The layers between sparse convolutions of a sparse-tensor network (Sec. III, caption of the partition
// overview figure: batch normalisation, activation and pooling between SparseConv blocks; Sec. IV-A: a
// 40-category classifier): training-mode batch normalisation (+ReLU) over the rows of a sparse tensor,
// per-cloud global average pooling, a linear layer and the mean softmax cross-entropy, each with its
// backward pass.  All are streaming / reduction kernels over [N][C] row-major features; reductions are
// two-level (per-block partial sums in fp32, combined in fp64 in a fixed order): no atomics, reproducible.
#include <algorithm>
#include <type_traits>

#include "sp_internal.h"

namespace sp {
namespace {

typedef uint16_t bf16_t;
constexpr int kThreads = 256;
constexpr int kSlabRows = 512;  // rows reduced by one block

__device__ __forceinline__ float ld(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld(const bf16_t* p, size_t i) { return __uint_as_float((uint32_t)p[i] << 16); }
__device__ __forceinline__ void st(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st(bf16_t* p, size_t i, float v) {
    uint32_t u = __float_as_uint(v);
    p[i] = (u & 0x7fffffffu) > 0x7f800000u ? (bf16_t)((u >> 16) | 0x40) : (bf16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// Threads of a block form a (cb x ry) grid over (channel, row): cb = 32, 64, 128 or 256 channels side by
// side (coalesced), ry = 256 / cb rows at a time.  Channels beyond cb are covered by a loop.
__host__ __device__ inline int channel_block(int c) { return c <= 32 ? 32 : (c <= 64 ? 64 : (c <= 128 ? 128 : 256)); }

// partial[blk][q][c] = sum over the block's rows of f_q(row, c), q < 2.
// MODE 0: (x, x^2).  MODE 1: (dyh, dyh * xhat) with dyh = dy masked by y > 0 when relu.
template <typename T, int MODE>
__global__ __launch_bounds__(kThreads) void column_sums_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                               const T* __restrict__ dy, int64_t n, int c,
                                                               const float* __restrict__ mean,
                                                               const float* __restrict__ rstd, int relu,
                                                               float* __restrict__ partial) {
    __shared__ float red[2][kThreads];
    const int cb = channel_block(c), ry = kThreads / cb;
    const int cx = threadIdx.x % cb, r0 = threadIdx.x / cb;
    const int64_t row_beg = (int64_t)blockIdx.x * kSlabRows;
    const int64_t row_end = row_beg + kSlabRows < n ? row_beg + kSlabRows : n;
    for (int ch = cx; ch < c + cb - 1 - (c + cb - 1) % cb; ch += cb) {  // uniform trip count over the block
        float s0 = 0.f, s1 = 0.f;
        if (ch < c) {
            // MODE 0 sums deviations from the channel's first row (a shift close to the mean keeps
            // E[d^2] - E[d]^2 free of cancellation; a single row gives variance exactly 0)
            const float m = MODE == 1 ? mean[ch] : ld(x, (size_t)ch), rs = MODE == 1 ? rstd[ch] : 0.f;
            for (int64_t r = row_beg + r0; r < row_end; r += ry) {
                const size_t i = (size_t)r * c + ch;
                if (MODE == 0) {
                    const float v = ld(x, i) - m;
                    s0 += v;
                    s1 += v * v;
                } else {
                    float g = ld(dy, i);
                    if (relu && !(ld(y, i) > 0.f)) g = 0.f;
                    s0 += g;
                    s1 += g * (ld(x, i) - m) * rs;
                }
            }
        }
        red[0][threadIdx.x] = s0;
        red[1][threadIdx.x] = s1;
        __syncthreads();
        if (r0 == 0 && ch < c) {
            float t0 = 0.f, t1 = 0.f;
            for (int j = 0; j < ry; ++j) {
                t0 += red[0][j * cb + cx];
                t1 += red[1][j * cb + cx];
            }
            partial[((size_t)blockIdx.x * 2 + 0) * c + ch] = t0;
            partial[((size_t)blockIdx.x * 2 + 1) * c + ch] = t1;
        }
        __syncthreads();
    }
}

// Adds the block partials in double, in a fixed order: 32 interleaved running sums per channel (block b goes
// to sum b % 32), then added 0..31.  Block = 32 channels x 32 slices.
// MODE 0: mean / rstd (the partials are sums of deviations from `shift[ch]`).  MODE 1: dbeta (sum 0) /
// dgamma (sum 1).
template <int MODE, typename T>
__global__ __launch_bounds__(1024) void column_sums_final_kernel(const float* __restrict__ partial, int64_t nblk,
                                                                 int64_t n, int c, float eps,
                                                                 const T* __restrict__ shift,
                                                                 float* __restrict__ out0,
                                                                 float* __restrict__ out1) {
    __shared__ double red[2][32][32];
    const int cx = threadIdx.x & 31, slice = threadIdx.x >> 5;
    const int ch = blockIdx.x * 32 + cx;
    double s0 = 0.0, s1 = 0.0;
    if (ch < c)
        for (int64_t b = slice; b < nblk; b += 32) {
            s0 += (double)partial[((size_t)b * 2 + 0) * c + ch];
            s1 += (double)partial[((size_t)b * 2 + 1) * c + ch];
        }
    red[0][slice][cx] = s0;
    red[1][slice][cx] = s1;
    __syncthreads();
    if (slice != 0 || ch >= c) return;
    s0 = red[0][0][cx];
    s1 = red[1][0][cx];
    for (int j = 1; j < 32; ++j) {
        s0 += red[0][j][cx];
        s1 += red[1][j][cx];
    }
    if (MODE == 0) {
        const double md = n > 0 ? s0 / (double)n : 0.0;     // mean deviation from the shift
        double var = n > 0 ? s1 / (double)n - md * md : 0.0;  // biased variance
        if (var < 0.0) var = 0.0;
        out0[ch] = (float)(md + (n > 0 ? (double)ld(shift, (size_t)ch) : 0.0));
        out1[ch] = (float)(1.0 / sqrt(var + (double)eps));
    } else {
        out0[ch] = (float)s0;
        out1[ch] = (float)s1;
    }
}

// ---- 16-byte-vector versions for channel counts that are a multiple of 16 bytes --------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <typename T>
struct Vec {
    static constexpr int kN = 16 / sizeof(T);  // elements per 16 bytes
    float v[kN];
};
__device__ __forceinline__ void unpack(const u32x4& r, Vec<float>& o) {
#pragma unroll
    for (int i = 0; i < 4; ++i) o.v[i] = __uint_as_float(r[i]);
}
__device__ __forceinline__ void unpack(const u32x4& r, Vec<bf16_t>& o) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o.v[2 * i] = __uint_as_float(r[i] << 16);
        o.v[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ uint32_t bf16_bits(float v) {
    const uint32_t u = __float_as_uint(v);
    return (u & 0x7fffffffu) > 0x7f800000u ? ((u >> 16) | 0x40) : ((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ u32x4 pack(const Vec<float>& o) {
    return u32x4{__float_as_uint(o.v[0]), __float_as_uint(o.v[1]), __float_as_uint(o.v[2]), __float_as_uint(o.v[3])};
}
__device__ __forceinline__ u32x4 pack(const Vec<bf16_t>& o) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = bf16_bits(o.v[2 * i]) | (bf16_bits(o.v[2 * i + 1]) << 16);
    return r;
}
template <typename T>
__device__ __forceinline__ Vec<T> load_vec(const T* p, size_t elem) {
    Vec<T> o;
    unpack(*reinterpret_cast<const u32x4*>(p + elem), o);
    return o;
}

// Same sums as column_sums_kernel.  Thread = (row lane, 16-byte channel group); tpr = c / kN threads cover a
// row, 256 / tpr rows are read per pass (tpr need not divide 256: the spare threads idle).  The block's rows
// are rows [blockIdx.x * rows_per_block, ...).  Row lanes are added in lane order.
template <typename T, int MODE>
__global__ __launch_bounds__(kThreads) void column_sums_vec_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                                   const T* __restrict__ dy, int64_t n, int c,
                                                                   int64_t rows_per_block,
                                                                   const float* __restrict__ mean,
                                                                   const float* __restrict__ rstd, int relu,
                                                                   float* __restrict__ partial) {
    constexpr int kN = Vec<T>::kN;
    extern __shared__ float red[];  // [2][row lanes][c]
    const int tpr = c / kN, lanes = kThreads / tpr;
    const int cg = threadIdx.x % tpr, rl = threadIdx.x / tpr;
    const int64_t row_beg = (int64_t)blockIdx.x * rows_per_block;
    const int64_t row_end = row_beg + rows_per_block < n ? row_beg + rows_per_block : n;
    float s0[kN], s1[kN], m[kN], rs[kN];
#pragma unroll
    for (int i = 0; i < kN; ++i) s0[i] = s1[i] = m[i] = rs[i] = 0.f;
    if (rl < lanes) {
        if (MODE == 0) {
            // sums of deviations from the channel's first row (a shift close to the mean keeps
            // E[d^2] - E[d]^2 free of cancellation; a single row gives variance exactly 0)
            const Vec<T> f = load_vec(x, (size_t)cg * kN);
#pragma unroll
            for (int i = 0; i < kN; ++i) m[i] = f.v[i];
        } else {
#pragma unroll
            for (int i = 0; i < kN; ++i) {
                m[i] = mean[cg * kN + i];
                rs[i] = rstd[cg * kN + i];
            }
        }
        auto raw = [&](const T* p, size_t e) { return *reinterpret_cast<const u32x4*>(p + e); };
        auto add_row = [&](const u32x4& rx, const u32x4& rg, const u32x4& ry) __attribute__((always_inline)) {
            Vec<T> xv, gv, yv;
            unpack(rx, xv);
            if (MODE == 0) {
#pragma unroll
                for (int i = 0; i < kN; ++i) {
                    const float v = xv.v[i] - m[i];
                    s0[i] += v;
                    s1[i] += v * v;
                }
            } else {
                unpack(rg, gv);
                unpack(ry, yv);
#pragma unroll
                for (int i = 0; i < kN; ++i) {
                    float g = gv.v[i];
                    if (relu && !(yv.v[i] > 0.f)) g = 0.f;
                    s0[i] += g;
                    s1[i] += g * (xv.v[i] - m[i]) * rs[i];
                }
            }
        };
        // 4 rows' loads are requested before the first is used (the rows are still added in row order)
        int64_t r = row_beg + rl;
        for (; r + 3 * (int64_t)lanes < row_end; r += 4 * lanes) {
            u32x4 rx[4], rg[4], ry[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const size_t e = (size_t)(r + u * lanes) * c + (size_t)cg * kN;
                rx[u] = raw(x, e);
                if (MODE == 1) {
                    rg[u] = raw(dy, e);
                    ry[u] = relu ? raw(y, e) : rg[u];
                } else {
                    rg[u] = ry[u] = rx[u];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) add_row(rx[u], rg[u], ry[u]);
        }
        for (; r < row_end; r += lanes) {
            const size_t e = (size_t)r * c + (size_t)cg * kN;
            const u32x4 rx = raw(x, e);
            const u32x4 rg = MODE == 1 ? raw(dy, e) : rx;
            const u32x4 ry = MODE == 1 && relu ? raw(y, e) : rg;
            add_row(rx, rg, ry);
        }
#pragma unroll
        for (int i = 0; i < kN; ++i) {
            red[(0 * lanes + rl) * c + cg * kN + i] = s0[i];
            red[(1 * lanes + rl) * c + cg * kN + i] = s1[i];
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 2 * c; e += kThreads) {
        const int q = e / c, ch = e % c;
        float t = 0.f;
        for (int j = 0; j < lanes; ++j) t += red[(q * lanes + j) * c + ch];
        partial[((size_t)blockIdx.x * 2 + q) * c + ch] = t;
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_apply_vec_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                                int64_t chunks, int c, const float* __restrict__ gamma,
                                                                const float* __restrict__ beta,
                                                                const float* __restrict__ mean,
                                                                const float* __restrict__ rstd, int relu) {
    constexpr int kN = Vec<T>::kN;
    // the grid stride is cut to a multiple of the 16-byte groups per row, so a thread stays on its channels
    const int tpr = c / kN;
    const int64_t stride = (int64_t)gridDim.x * kThreads / tpr * tpr;
    const int64_t i0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i0 >= stride) return;
    const int ch = (int)(i0 % tpr) * kN;
    float m[kN], k[kN], g[kN], b[kN];
#pragma unroll
    for (int j = 0; j < kN; ++j) {
        m[j] = mean[ch + j];
        k[j] = rstd[ch + j];
        g[j] = gamma[ch + j];
        b[j] = beta[ch + j];
    }
    for (int64_t i = i0; i < chunks; i += stride) {
        const Vec<T> xv = load_vec(x, (size_t)i * kN);
        Vec<T> o;
#pragma unroll
        for (int j = 0; j < kN; ++j) {
            float v = (xv.v[j] - m[j]) * k[j] * g[j] + b[j];
            if (relu) v = fmaxf(v, 0.f);
            o.v[j] = v;
        }
        *reinterpret_cast<u32x4*>(y + (size_t)i * kN) = pack(o);
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_vec_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                                    const T* __restrict__ dy, T* __restrict__ dx,
                                                                    int64_t n, int c, const float* __restrict__ gamma,
                                                                    const float* __restrict__ mean,
                                                                    const float* __restrict__ rstd,
                                                                    const float* __restrict__ dgamma,
                                                                    const float* __restrict__ dbeta, int relu) {
    constexpr int kN = Vec<T>::kN;
    const int64_t chunks = n * c / kN;
    const float inv_n = 1.f / (float)n;
    const int tpr = c / kN;
    const int64_t stride = (int64_t)gridDim.x * kThreads / tpr * tpr;
    const int64_t i0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i0 >= stride) return;
    const int ch = (int)(i0 % tpr) * kN;
    float m[kN], k[kN], ga[kN], dg[kN], db[kN];
#pragma unroll
    for (int j = 0; j < kN; ++j) {
        m[j] = mean[ch + j];
        k[j] = rstd[ch + j];
        ga[j] = gamma[ch + j];
        dg[j] = dgamma[ch + j];
        db[j] = dbeta[ch + j];
    }
    for (int64_t i = i0; i < chunks; i += stride) {
        const size_t e = (size_t)i * kN;
        const Vec<T> xv = load_vec(x, e), gv = load_vec(dy, e);
        Vec<T> yv = gv;
        if (relu) yv = load_vec(y, e);
        Vec<T> o;
#pragma unroll
        for (int j = 0; j < kN; ++j) {
            float g = gv.v[j];
            if (relu && !(yv.v[j] > 0.f)) g = 0.f;
            const float xhat = (xv.v[j] - m[j]) * k[j];
            o.v[j] = ga[j] * k[j] * (g - (db[j] + xhat * dg[j]) * inv_n);
        }
        *reinterpret_cast<u32x4*>(dx + (size_t)i * kN) = pack(o);
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(const T* __restrict__ x, T* __restrict__ y, int64_t total,
                                                            int c, const float* __restrict__ gamma,
                                                            const float* __restrict__ beta,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ rstd, int relu) {
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int ch = (int)(i % c);
        float v = (ld(x, i) - mean[ch]) * rstd[ch] * gamma[ch] + beta[ch];
        if (relu) v = fmaxf(v, 0.f);
        st(y, i, v);
    }
}

// dx = gamma * rstd / N * (N * dyh - dbeta - xhat * dgamma)
template <typename T>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                                const T* __restrict__ dy, T* __restrict__ dx,
                                                                int64_t n, int c, const float* __restrict__ gamma,
                                                                const float* __restrict__ mean,
                                                                const float* __restrict__ rstd,
                                                                const float* __restrict__ dgamma,
                                                                const float* __restrict__ dbeta, int relu) {
    const int64_t total = n * c;
    const float inv_n = 1.f / (float)n;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int ch = (int)(i % c);
        float g = ld(dy, i);
        if (relu && !(ld(y, i) > 0.f)) g = 0.f;
        const float xhat = (ld(x, i) - mean[ch]) * rstd[ch];
        st(dx, i, gamma[ch] * rstd[ch] * (g - (dbeta[ch] + xhat * dgamma[ch]) * inv_n));
    }
}

// Per-cloud sums: thread (cx, r0) owns the LDS cells [r0][b][cx]; partial[blk][b][c], cnt_partial[blk][b].
template <typename T>
__global__ __launch_bounds__(kThreads) void pool_partial_kernel(const int4* __restrict__ coords,
                                                                const T* __restrict__ x, int64_t n, int c, int nb,
                                                                float* __restrict__ partial,
                                                                int32_t* __restrict__ cnt_partial) {
    extern __shared__ float s_acc[];  // [ry][nb][cb] floats, then [ry][nb] ints
    const int cb = channel_block(c), ry = kThreads / cb;
    const int cx = threadIdx.x % cb, r0 = threadIdx.x / cb;
    int* s_cnt = reinterpret_cast<int*>(s_acc + (size_t)ry * nb * cb);
    const int64_t row_beg = (int64_t)blockIdx.x * kSlabRows;
    const int64_t row_end = row_beg + kSlabRows < n ? row_beg + kSlabRows : n;
    for (int ch0 = 0; ch0 < c; ch0 += cb) {
        for (int i = threadIdx.x; i < ry * nb * cb; i += kThreads) s_acc[i] = 0.f;
        for (int i = threadIdx.x; i < ry * nb; i += kThreads) s_cnt[i] = 0;
        __syncthreads();
        const int ch = ch0 + cx;
        for (int64_t r = row_beg + r0; r < row_end; r += ry) {
            const int b = coords[r].x;
            if ((unsigned)b < (unsigned)nb) {
                if (ch < c) s_acc[((size_t)r0 * nb + b) * cb + cx] += ld(x, (size_t)r * c + ch);
                if (cx == 0 && ch0 == 0) s_cnt[r0 * nb + b] += 1;
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < nb * cb; i += kThreads) {
            const int b = i / cb, cc = i % cb;
            if (ch0 + cc < c) {
                float t = 0.f;
                for (int j = 0; j < ry; ++j) t += s_acc[((size_t)j * nb + b) * cb + cc];
                partial[((size_t)blockIdx.x * nb + b) * c + ch0 + cc] = t;
            }
        }
        if (ch0 == 0)
            for (int b = threadIdx.x; b < nb; b += kThreads) {
                int t = 0;
                for (int j = 0; j < ry; ++j) t += s_cnt[j * nb + b];
                cnt_partial[(size_t)blockIdx.x * nb + b] = t;
            }
        __syncthreads();
    }
}

// 16-byte-vector version: thread = (row lane, 16-byte channel group); a thread keeps the running sums of the
// cloud its rows are currently in and adds them to its own LDS cells [row lane][cloud][channels] when the
// cloud changes (rows of one cloud are usually contiguous, so that is rare).  Row lanes are added in lane
// order.  LDS: lanes * nb * c floats, the host checks that it fits.
template <typename T>
__global__ __launch_bounds__(kThreads) void pool_partial_vec_kernel(const int4* __restrict__ coords,
                                                                    const T* __restrict__ x, int64_t n, int c, int nb,
                                                                    int slab, float* __restrict__ partial,
                                                                    int32_t* __restrict__ cnt_partial) {
    constexpr int kN = Vec<T>::kN;
    extern __shared__ float s_acc[];  // [lanes][nb][c] floats, then [lanes][nb] ints
    const int tpr = c / kN, lanes = kThreads / tpr;
    const int cg = threadIdx.x % tpr, rl = threadIdx.x / tpr;
    int* s_cnt = reinterpret_cast<int*>(s_acc + (size_t)lanes * nb * c);
    for (int i = threadIdx.x; i < lanes * nb * c; i += kThreads) s_acc[i] = 0.f;
    for (int i = threadIdx.x; i < lanes * nb; i += kThreads) s_cnt[i] = 0;
    __syncthreads();
    const int64_t row_beg = (int64_t)blockIdx.x * slab;
    const int64_t row_end = row_beg + slab < n ? row_beg + slab : n;
    if (rl < lanes) {
        float acc[kN];
#pragma unroll
        for (int i = 0; i < kN; ++i) acc[i] = 0.f;
        int cur = -1, cnt = 0;
        auto flush = [&]() {
            if (cur >= 0) {
                float* cell = s_acc + ((size_t)rl * nb + cur) * c + cg * kN;
#pragma unroll
                for (int i = 0; i < kN; ++i) {
                    cell[i] += acc[i];
                    acc[i] = 0.f;
                }
                if (cg == 0) s_cnt[rl * nb + cur] += cnt;
            }
            cnt = 0;
        };
        for (int64_t r = row_beg + rl; r < row_end; r += lanes) {
            const int b = coords[r].x;
            const Vec<T> xv = load_vec(x, (size_t)r * c + (size_t)cg * kN);
            if ((unsigned)b >= (unsigned)nb) continue;
            if (b != cur) {
                flush();
                cur = b;
            }
#pragma unroll
            for (int i = 0; i < kN; ++i) acc[i] += xv.v[i];
            ++cnt;
        }
        flush();
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nb * c; i += kThreads) {
        float t = 0.f;
        for (int j = 0; j < lanes; ++j) t += s_acc[(size_t)j * nb * c + i];
        partial[(size_t)blockIdx.x * nb * c + i] = t;
    }
    for (int b = threadIdx.x; b < nb; b += kThreads) {
        int t = 0;
        for (int j = 0; j < lanes; ++j) t += s_cnt[j * nb + b];
        cnt_partial[(size_t)blockIdx.x * nb + b] = t;
    }
}

__global__ __launch_bounds__(1024) void pool_final_kernel(const float* __restrict__ partial,
                                                              const int32_t* __restrict__ cnt_partial, int64_t nblk,
                                                              int c, int nb, float* __restrict__ out,
                                                              float* __restrict__ counts) {
    // block = 32 (cloud, channel) elements x 32 slices of the row blocks; slices are added in order
    __shared__ double red[32][32];
    __shared__ long long redc[32][32];
    const int ex = threadIdx.x & 31, slice = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + ex;
    const bool live = i < nb * c;
    const int b = live ? i / c : 0;
    double s = 0.0;
    long long cnt = 0;
    if (live)
        for (int64_t k = slice; k < nblk; k += 32) {
            s += (double)partial[(size_t)k * nb * c + i];
            cnt += cnt_partial[(size_t)k * nb + b];
        }
    red[slice][ex] = s;
    redc[slice][ex] = cnt;
    __syncthreads();
    if (slice != 0 || !live) return;
    for (int j = 1; j < 32; ++j) {
        s += red[j][ex];
        cnt += redc[j][ex];
    }
    out[i] = cnt > 0 ? (float)(s / (double)cnt) : 0.f;
    if (i % c == 0) counts[b] = (float)cnt;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void pool_bwd_kernel(const int4* __restrict__ coords,
                                                            const float* __restrict__ dout,
                                                            const float* __restrict__ counts, T* __restrict__ dx,
                                                            int64_t n, int c, int nb) {
    const int64_t total = n * c;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int64_t r = i / c;
        const int ch = (int)(i % c);
        const int b = coords[r].x;
        float v = 0.f;
        if ((unsigned)b < (unsigned)nb) v = dout[(size_t)b * c + ch] / fmaxf(counts[b], 1.f);
        st(dx, i, v);
    }
}

// 16-byte-vector version: one thread per 16 bytes of dx
template <typename T>
__global__ __launch_bounds__(kThreads) void pool_bwd_vec_kernel(const int4* __restrict__ coords,
                                                                const float* __restrict__ dout,
                                                                const float* __restrict__ counts, T* __restrict__ dx,
                                                                int64_t n, int c, int nb) {
    constexpr int kN = Vec<T>::kN;
    const int tpr = c / kN;
    const int64_t chunks = n * tpr;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < chunks; i += (int64_t)gridDim.x * kThreads) {
        const int64_t r = i / tpr;
        const int ch = (int)(i % tpr) * kN;
        const int b = coords[r].x;
        Vec<T> o;
        const bool live = (unsigned)b < (unsigned)nb;
#pragma unroll
        for (int j = 0; j < kN; ++j) o.v[j] = live ? dout[(size_t)b * c + ch + j] / fmaxf(counts[b], 1.f) : 0.f;
        *reinterpret_cast<u32x4*>(dx + (size_t)i * kN) = pack(o);
    }
}

__global__ __launch_bounds__(kThreads) void linear_fwd_kernel(const float* __restrict__ in,
                                                              const float* __restrict__ w,
                                                              const float* __restrict__ bias, int nb, int c, int m,
                                                              float* __restrict__ out) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= nb * m) return;
    const int b = i / m, j = i % m;
    // 4 interleaved running sums (k % 4), added 0+1+2+3: four independent load/fma chains instead of one
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    const float* x = in + (size_t)b * c;
    const float* wr = w + (size_t)j * c;
    int k = 0;
    for (; k + 4 <= c; k += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) s[u] = fmaf(x[k + u], wr[k + u], s[u]);
    }
    for (; k < c; ++k) s[k & 3] = fmaf(x[k], wr[k], s[k & 3]);
    out[i] = (bias ? bias[j] : 0.f) + (((s[0] + s[1]) + s[2]) + s[3]);
}

// one launch for the three gradients: [0, nb*c) din, [nb*c, nb*c + m*c) dw, then m entries of dbias
__global__ __launch_bounds__(kThreads) void linear_bwd_kernel(const float* __restrict__ in,
                                                              const float* __restrict__ w,
                                                              const float* __restrict__ dout, int nb, int c, int m,
                                                              float* __restrict__ din, float* __restrict__ dw,
                                                              float* __restrict__ dbias) {
    int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < nb * c) {
        const int b = i / c, k = i % c;
        float s = 0.f;
        for (int j = 0; j < m; ++j) s = fmaf(dout[(size_t)b * m + j], w[(size_t)j * c + k], s);
        din[i] = s;
        return;
    }
    i -= nb * c;
    if (i < m * c) {
        const int j = i / c, k = i % c;
        float s = 0.f;
        for (int b = 0; b < nb; ++b) s = fmaf(dout[(size_t)b * m + j], in[(size_t)b * c + k], s);
        dw[i] = s;
        return;
    }
    i -= m * c;
    if (i < m) {
        float s = 0.f;
        for (int b = 0; b < nb; ++b) s += dout[(size_t)b * m + i];
        dbias[i] = s;
    }
}

// one block; thread b handles cloud b, then thread 0 adds the per-cloud losses in order
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(const float* __restrict__ logits,
                                                              const int32_t* __restrict__ labels, int nb, int m,
                                                              float* __restrict__ loss, float* __restrict__ dlogits,
                                                              float* __restrict__ per_cloud) {
    for (int b = threadIdx.x; b < nb; b += kThreads) {
        const float* z = logits + (size_t)b * m;
        float mx = z[0];
        for (int j = 1; j < m; ++j) mx = fmaxf(mx, z[j]);
        float se = 0.f;
        for (int j = 0; j < m; ++j) se += expf(z[j] - mx);
        const float lse = logf(se) + mx;
        const int lab = labels[b];
        per_cloud[b] = ((unsigned)lab < (unsigned)m) ? lse - z[lab] : 0.f;
        for (int j = 0; j < m; ++j)
            dlogits[(size_t)b * m + j] = (expf(z[j] - lse) - (j == lab ? 1.f : 0.f)) / (float)nb;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int b = 0; b < nb; ++b) s += (double)per_cloud[b];
        *loss = nb > 0 ? (float)(s / (double)nb) : 0.f;
    }
}

inline unsigned stream_blocks(int64_t total) {
    int64_t b = (total + kThreads - 1) / kThreads;
    return (unsigned)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

// vector kernels: whole 16-byte groups per row, at most 256 of them, 16-byte aligned base pointers
template <typename T>
bool vec_ok(int c, const void* p0, const void* p1, const void* p2, const void* p3) {
    constexpr int kN = 16 / (int)sizeof(T);
    const uintptr_t bits = (uintptr_t)p0 | (uintptr_t)p1 | (uintptr_t)p2 | (uintptr_t)p3;
    return c % kN == 0 && c / kN <= kThreads && (bits & 15) == 0;
}
// rows per block of the vector column sums: at most 512 blocks, at least 256 rows each
inline int64_t vec_rows_per_block(int64_t n) {
    const int64_t r = (n + 511) / 512;
    return r < 256 ? 256 : r;
}

template <typename T>
int bn_fwd_typed(const void* x, int64_t n, int c, const float* gamma, const float* beta, float eps, int relu, void* y,
                 float* mean, float* rstd, hipStream_t s) {
    const bool vec = vec_ok<T>(c, x, y, nullptr, nullptr);
    const int64_t rpb = vec ? vec_rows_per_block(n) : kSlabRows;
    const int64_t nblk = (n + rpb - 1) / rpb;
    Buf partial = dev_alloc((size_t)(nblk ? nblk : 1) * 2 * c * 4, s);
    if (!partial) return SP_ERR_ALLOC;
    if (nblk > 0) {
        if (vec) {
            const int lanes = kThreads / (c / (16 / (int)sizeof(T)));
            hipLaunchKernelGGL((column_sums_vec_kernel<T, 0>), dim3((unsigned)nblk), dim3(kThreads),
                               (size_t)2 * lanes * c * 4, s, static_cast<const T*>(x), (const T*)nullptr,
                               (const T*)nullptr, n, c, rpb, (const float*)nullptr, (const float*)nullptr, 0,
                               ptr<float>(partial));
        } else {
            hipLaunchKernelGGL((column_sums_kernel<T, 0>), dim3((unsigned)nblk), dim3(kThreads), 0, s,
                               static_cast<const T*>(x), (const T*)nullptr, (const T*)nullptr, n, c,
                               (const float*)nullptr, (const float*)nullptr, 0, ptr<float>(partial));
        }
    }
    hipLaunchKernelGGL((column_sums_final_kernel<0, T>), dim3((c + 31) / 32), dim3(1024), 0, s, ptr<float>(partial),
                       nblk, n, c, eps, static_cast<const T*>(x), mean, rstd);
    if (n > 0) {
        if (vec)
            hipLaunchKernelGGL(bn_apply_vec_kernel<T>, dim3(stream_blocks(n * c / (16 / (int64_t)sizeof(T)))),
                               dim3(kThreads), 0, s, static_cast<const T*>(x), static_cast<T*>(y),
                               n * c / (16 / (int64_t)sizeof(T)), c, gamma, beta, mean, rstd, relu);
        else
            hipLaunchKernelGGL(bn_apply_kernel<T>, dim3(stream_blocks(n * c)), dim3(kThreads), 0, s,
                               static_cast<const T*>(x), static_cast<T*>(y), n * c, c, gamma, beta, mean, rstd, relu);
    }
    SP_HIP(hipGetLastError());
    return SP_OK;
}

template <typename T>
int bn_bwd_typed(const void* x, const void* y, const void* dy, int64_t n, int c, const float* gamma, const float* mean,
                 const float* rstd, int relu, void* dx, float* dgamma, float* dbeta, hipStream_t s) {
    const bool vec = vec_ok<T>(c, x, y, dy, dx);
    const int64_t rpb = vec ? vec_rows_per_block(n) : kSlabRows;
    const int64_t nblk = (n + rpb - 1) / rpb;
    Buf partial = dev_alloc((size_t)(nblk ? nblk : 1) * 2 * c * 4, s);
    if (!partial) return SP_ERR_ALLOC;
    if (nblk > 0) {
        if (vec) {
            const int lanes = kThreads / (c / (16 / (int)sizeof(T)));
            hipLaunchKernelGGL((column_sums_vec_kernel<T, 1>), dim3((unsigned)nblk), dim3(kThreads),
                               (size_t)2 * lanes * c * 4, s, static_cast<const T*>(x), static_cast<const T*>(y),
                               static_cast<const T*>(dy), n, c, rpb, mean, rstd, relu, ptr<float>(partial));
        } else {
            hipLaunchKernelGGL((column_sums_kernel<T, 1>), dim3((unsigned)nblk), dim3(kThreads), 0, s,
                               static_cast<const T*>(x), static_cast<const T*>(y), static_cast<const T*>(dy), n, c, mean,
                               rstd, relu, ptr<float>(partial));
        }
    }
    hipLaunchKernelGGL((column_sums_final_kernel<1, T>), dim3((c + 31) / 32), dim3(1024), 0, s, ptr<float>(partial),
                       nblk, n, c, 0.f, (const T*)nullptr, dbeta, dgamma);
    if (n > 0) {
        if (vec)
            hipLaunchKernelGGL(bn_bwd_apply_vec_kernel<T>, dim3(stream_blocks(n * c / (16 / (int64_t)sizeof(T)))),
                               dim3(kThreads), 0, s, static_cast<const T*>(x), static_cast<const T*>(y),
                               static_cast<const T*>(dy), static_cast<T*>(dx), n, c, gamma, mean, rstd, dgamma, dbeta,
                               relu);
        else
            hipLaunchKernelGGL(bn_bwd_apply_kernel<T>, dim3(stream_blocks(n * c)), dim3(kThreads), 0, s,
                               static_cast<const T*>(x), static_cast<const T*>(y), static_cast<const T*>(dy),
                               static_cast<T*>(dx), n, c, gamma, mean, rstd, dgamma, dbeta, relu);
    }
    SP_HIP(hipGetLastError());
    return SP_OK;
}

template <typename T>
int pool_fwd_typed(const int32_t* coords, const void* x, int64_t n, int c, int nb, float* out, float* counts,
                   hipStream_t s) {
    const int cb = channel_block(c), ry = kThreads / cb;
    const size_t lds = (size_t)ry * nb * cb * 4 + (size_t)ry * nb * 4;
    if (lds > 64 * 1024) return fail(SP_ERR_UNSUPPORTED, "too many clouds for the pooling kernel (%d)", nb);
    constexpr int kN = 16 / (int)sizeof(T);
    const int vlanes = c % kN == 0 && c / kN <= kThreads ? kThreads / (c / kN) : 0;
    const size_t vlds = (size_t)vlanes * nb * c * 4 + (size_t)vlanes * nb * 4;
    const bool vec = vlanes > 0 && vlds <= 64 * 1024 && ((uintptr_t)x & 15) == 0;
    // rows per block: the vector kernel is latency bound per block, so it takes smaller slabs (more blocks),
    // but no more than 1024 blocks for the final sums to add up
    int64_t slab = kSlabRows;
    if (vec) slab = std::max<int64_t>(128, (n + 1023) / 1024);
    const int64_t nblk = (n + slab - 1) / slab;
    Buf partial = dev_alloc((size_t)(nblk ? nblk : 1) * nb * c * 4, s);
    Buf cnt = dev_alloc((size_t)(nblk ? nblk : 1) * nb * 4, s);
    if (!partial || !cnt) return SP_ERR_ALLOC;
    if (nblk > 0) {
        if (vec)
            hipLaunchKernelGGL(pool_partial_vec_kernel<T>, dim3((unsigned)nblk), dim3(kThreads), vlds, s,
                               reinterpret_cast<const int4*>(coords), static_cast<const T*>(x), n, c, nb, (int)slab,
                               ptr<float>(partial), ptr<int32_t>(cnt));
        else
            hipLaunchKernelGGL(pool_partial_kernel<T>, dim3((unsigned)nblk), dim3(kThreads), lds, s,
                               reinterpret_cast<const int4*>(coords), static_cast<const T*>(x), n, c, nb,
                               ptr<float>(partial), ptr<int32_t>(cnt));
    }
    hipLaunchKernelGGL(pool_final_kernel, dim3((nb * c + 31) / 32), dim3(1024), 0, s, ptr<float>(partial),
                       ptr<int32_t>(cnt), nblk, c, nb, out, counts);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

int check_rows(const void* a, int64_t n, int c, sp_dtype dt) {
    if (n < 0 || c < 1 || c > 65536) return fail(SP_ERR_INVALID_ARG, "bad row or channel count");
    if (dt != SP_F32 && dt != SP_BF16) return fail(SP_ERR_INVALID_ARG, "bad dtype");
    if (n > 0 && !a) return fail(SP_ERR_INVALID_ARG, "a feature pointer is NULL");
    return SP_OK;
}

}  // namespace
}  // namespace sp

using namespace sp;

extern "C" {

int sp_bn_relu_fwd(const void* d_x, int64_t n, int32_t c, const float* d_gamma, const float* d_beta, float eps,
                   int32_t relu, void* d_y, float* d_mean, float* d_rstd, sp_dtype dt, void* stream) {
    SP_TRY(check_rows(d_x, n, c, dt));
    if (!d_gamma || !d_beta || !d_mean || !d_rstd || (n > 0 && !d_y))
        return fail(SP_ERR_INVALID_ARG, "a parameter/statistics pointer is NULL");
    return dt == SP_F32 ? bn_fwd_typed<float>(d_x, n, c, d_gamma, d_beta, eps, relu, d_y, d_mean, d_rstd, (hipStream_t)stream)
                        : bn_fwd_typed<bf16_t>(d_x, n, c, d_gamma, d_beta, eps, relu, d_y, d_mean, d_rstd, (hipStream_t)stream);
}

int sp_bn_relu_bwd(const void* d_x, const void* d_y, const void* d_dy, int64_t n, int32_t c, const float* d_gamma,
                   const float* d_mean, const float* d_rstd, int32_t relu, void* d_dx, float* d_dgamma,
                   float* d_dbeta, sp_dtype dt, void* stream) {
    SP_TRY(check_rows(d_x, n, c, dt));
    if (!d_gamma || !d_mean || !d_rstd || !d_dgamma || !d_dbeta || (n > 0 && (!d_dy || !d_dx || (relu && !d_y))))
        return fail(SP_ERR_INVALID_ARG, "a parameter/gradient pointer is NULL");
    return dt == SP_F32 ? bn_bwd_typed<float>(d_x, d_y, d_dy, n, c, d_gamma, d_mean, d_rstd, relu, d_dx, d_dgamma, d_dbeta, (hipStream_t)stream)
                        : bn_bwd_typed<bf16_t>(d_x, d_y, d_dy, n, c, d_gamma, d_mean, d_rstd, relu, d_dx, d_dgamma, d_dbeta, (hipStream_t)stream);
}

int sp_pool_avg_fwd(const int32_t* d_coords, const void* d_x, int64_t n, int32_t c, int32_t n_clouds, float* d_out,
                    float* d_counts, sp_dtype dt, void* stream) {
    SP_TRY(check_rows(d_x, n, c, dt));
    if (n_clouds < 1 || !d_out || !d_counts || (n > 0 && !d_coords))
        return fail(SP_ERR_INVALID_ARG, "bad cloud count or NULL pointer");
    return dt == SP_F32 ? pool_fwd_typed<float>(d_coords, d_x, n, c, n_clouds, d_out, d_counts, (hipStream_t)stream)
                        : pool_fwd_typed<bf16_t>(d_coords, d_x, n, c, n_clouds, d_out, d_counts, (hipStream_t)stream);
}

int sp_pool_avg_bwd(const int32_t* d_coords, const float* d_dout, const float* d_counts, int64_t n, int32_t c,
                    int32_t n_clouds, void* d_dx, sp_dtype dt, void* stream) {
    SP_TRY(check_rows(d_dx, n, c, dt));
    if (n_clouds < 1 || !d_dout || !d_counts || (n > 0 && !d_coords))
        return fail(SP_ERR_INVALID_ARG, "bad cloud count or NULL pointer");
    if (n == 0) return SP_OK;
    hipStream_t s = (hipStream_t)stream;
    const int kn = dt == SP_F32 ? 4 : 8;
    const bool vec = c % kn == 0 && ((uintptr_t)d_dx & 15) == 0;
    if (dt == SP_F32 && vec)
        hipLaunchKernelGGL(pool_bwd_vec_kernel<float>, dim3(stream_blocks(n * c / kn)), dim3(kThreads), 0, s,
                           reinterpret_cast<const int4*>(d_coords), d_dout, d_counts, static_cast<float*>(d_dx), n, c,
                           n_clouds);
    else if (dt == SP_F32)
        hipLaunchKernelGGL(pool_bwd_kernel<float>, dim3(stream_blocks(n * c)), dim3(kThreads), 0, s,
                           reinterpret_cast<const int4*>(d_coords), d_dout, d_counts, static_cast<float*>(d_dx), n, c,
                           n_clouds);
    else if (vec)
        hipLaunchKernelGGL(pool_bwd_vec_kernel<bf16_t>, dim3(stream_blocks(n * c / kn)), dim3(kThreads), 0, s,
                           reinterpret_cast<const int4*>(d_coords), d_dout, d_counts, static_cast<bf16_t*>(d_dx), n, c,
                           n_clouds);
    else
        hipLaunchKernelGGL(pool_bwd_kernel<bf16_t>, dim3(stream_blocks(n * c)), dim3(kThreads), 0, s,
                           reinterpret_cast<const int4*>(d_coords), d_dout, d_counts, static_cast<bf16_t*>(d_dx), n, c,
                           n_clouds);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

int sp_linear_fwd(const float* d_in, const float* d_w, const float* d_bias, int32_t n_clouds, int32_t c, int32_t m,
                  float* d_out, void* stream) {
    if (n_clouds < 1 || c < 1 || m < 1 || !d_in || !d_w || !d_out) return fail(SP_ERR_INVALID_ARG, "bad linear arguments");
    hipLaunchKernelGGL(linear_fwd_kernel, dim3((n_clouds * m + kThreads - 1) / kThreads), dim3(kThreads), 0,
                       (hipStream_t)stream, d_in, d_w, d_bias, n_clouds, c, m, d_out);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

int sp_linear_bwd(const float* d_in, const float* d_w, const float* d_dout, int32_t n_clouds, int32_t c, int32_t m,
                  float* d_din, float* d_dw, float* d_dbias, void* stream) {
    if (n_clouds < 1 || c < 1 || m < 1 || !d_in || !d_w || !d_dout || !d_din || !d_dw || !d_dbias)
        return fail(SP_ERR_INVALID_ARG, "bad linear arguments");
    const int total = n_clouds * c + m * c + m;
    hipLaunchKernelGGL(linear_bwd_kernel, dim3((total + kThreads - 1) / kThreads), dim3(kThreads), 0,
                       (hipStream_t)stream, d_in, d_w, d_dout, n_clouds, c, m, d_din, d_dw, d_dbias);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

int sp_softmax_ce(const float* d_logits, const int32_t* d_labels, int32_t n_clouds, int32_t m, float* d_loss,
                  float* d_dlogits, void* stream) {
    if (n_clouds < 1 || m < 1 || !d_logits || !d_labels || !d_loss || !d_dlogits)
        return fail(SP_ERR_INVALID_ARG, "bad cross-entropy arguments");
    Buf per_cloud = dev_alloc((size_t)n_clouds * 4, (hipStream_t)stream);
    if (!per_cloud) return SP_ERR_ALLOC;
    hipLaunchKernelGGL(softmax_ce_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)stream, d_logits, d_labels, n_clouds,
                       m, d_loss, d_dlogits, ptr<float>(per_cloud));
    SP_HIP(hipGetLastError());
    return SP_OK;
}

}  // extern "C"
