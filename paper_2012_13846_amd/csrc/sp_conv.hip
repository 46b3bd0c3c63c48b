// Step 3 of the generalized sparse convolution (Eq. 2) and its input gradient, as one gather-GEMM kernel.
//
// One workgroup owns a tile of destination rows (output rows for the forward pass, input rows for the data
// gradient) and a slice of destination channels.  It keeps the tile's fp32 accumulator in LDS.  For every
// kernel offset it takes the tile's compacted link list (source row, destination row), gathers the source
// feature rows into LDS, multiplies 16-link blocks with the offset's weight matrix on the matrix cores and
// adds each result row into the accumulator row of its destination.  A destination row belongs to exactly
// one workgroup and appears at most once per offset, so nothing is atomic and the summation order is
// fixed (results are reproducible run to run).  The accumulator is written once, rounded once.
#include <type_traits>

#include "sp_internal.h"

namespace sp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t bf16_t;  // storage

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even; NaN stays NaN
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
    return (bf16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

struct GatherArgs {
    const int32_t* tl_off;
    const int32_t* tl_src;
    const uint16_t* tl_row;
    const void* f;   // source features [n_src][CC]
    const void* w;   // weights [kvol][co_total][CC] (contraction index fastest)
    void* g;         // destination features [n_rows][co_total]
    int64_t n_rows;
    int kvol;
    int co_total;
    int flip;        // weight matrix of list k is kvol-1-k
};

// ---------------------------------------------------------------------------------------------------------
// T: float or bf16_t.  CC: contraction channels.  COT: destination channels per workgroup (16, 32 or 64).
// TR: destination rows per workgroup (64, 128 or 256).  4 wavefronts: COT/16 of them side by side over the
// channel slice, the rest over alternating 16-link blocks.
// ---------------------------------------------------------------------------------------------------------
template <typename T, int CC, int COT, int TR>
struct GatherCfg {
    static constexpr int kElt = sizeof(T);
    static constexpr int kNCS = COT / 16;            // wavefronts across channels
    static constexpr int kNBS = 4 / kNCS;            // wavefronts across link blocks
    static constexpr int kRowBytes = CC * kElt + 16; // staged row + 16 B pad (keeps b128 reads conflict-poor)
    static constexpr int kChunkRaw = (32 * 1024) / kRowBytes;
    static constexpr int kChunk0 = kChunkRaw > TR ? TR : kChunkRaw;
    static constexpr int kChunk = (kChunk0 / (16 * kNBS)) * (16 * kNBS) > 0 ? (kChunk0 / (16 * kNBS)) * (16 * kNBS) : 16 * kNBS;
    static constexpr int kAccStride = COT + 4;       // floats
    static constexpr int kPiecesPerRow = CC * kElt / 16;
    static constexpr size_t kLds = (size_t)TR * kAccStride * 4 + (size_t)kChunk * kRowBytes + (size_t)kChunk * 2;
};

template <typename T, int CC, int COT, int TR>
__global__ __launch_bounds__(256) void gather_mma_kernel(GatherArgs a) {
    using Cfg = GatherCfg<T, CC, COT, TR>;
    constexpr bool kIsF32 = std::is_same<T, float>::value;
    constexpr int kGroup = kIsF32 ? 16 : 32;  // contraction channels consumed per A/B fragment load
    constexpr int kGroups = CC / kGroup;
    static_assert(CC % kGroup == 0, "contraction channels must fill whole fragment groups");
    static_assert(COT == 16 || COT == 32 || COT == 64, "bad channel tile");

    extern __shared__ __align__(16) unsigned char smem[];
    float* acc = reinterpret_cast<float*>(smem);
    unsigned char* abuf = smem + (size_t)TR * Cfg::kAccStride * 4;
    uint16_t* s_row = reinterpret_cast<uint16_t*>(abuf + (size_t)Cfg::kChunk * Cfg::kRowBytes);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cs = wave % Cfg::kNCS, bs = wave / Cfg::kNCS;
    const int n16 = lane & 15, g = lane >> 4;
    constexpr int kPerTile = kTileRows / TR;             // workgroups per 256-row tile
    const int64_t tile = blockIdx.x / kPerTile;
    const int q0 = (blockIdx.x % kPerTile) * (TR / 64);  // first 64-row sub-tile of this workgroup
    constexpr int kNQ = TR / 64;
    const int co0 = blockIdx.y * COT;

    for (int i = tid; i < TR * Cfg::kAccStride; i += 256) acc[i] = 0.f;

    const T* __restrict__ F = static_cast<const T*>(a.f);
    const T* __restrict__ W = static_cast<const T*>(a.w);

    for (int kk = 0; kk < a.kvol; ++kk) {
        const int64_t ob = (tile * a.kvol + kk) * kSubTiles + q0;
        const int beg = a.tl_off[ob], end = a.tl_off[ob + kNQ];
        if (beg == end) continue;
        const int wk = a.flip ? a.kvol - 1 - kk : kk;
        // this wavefront's weight slice: B[cc][n16] = W[wk][co0 + cs*16 + n16][cc]
        const T* wrow = W + ((size_t)wk * a.co_total + co0 + cs * 16 + n16) * CC;
        f32x4 bf[kIsF32 ? kGroups : 1];
        bf16x8 bh[kIsF32 ? 1 : kGroups];
#pragma unroll
        for (int s = 0; s < kGroups; ++s) {
            if constexpr (kIsF32)
                bf[s] = *reinterpret_cast<const f32x4*>(wrow + s * 16 + g * 4);
            else
                bh[s] = *reinterpret_cast<const bf16x8*>(wrow + s * 32 + g * 8);
        }
        for (int c0 = beg; c0 < end; c0 += Cfg::kChunk) {
            const int m = min(Cfg::kChunk, end - c0);
            __syncthreads();  // everyone is done with the previous staging buffer and its accumulator updates
            for (int idx = tid; idx < m * Cfg::kPiecesPerRow; idx += 256) {
                const int p = idx / Cfg::kPiecesPerRow, piece = idx % Cfg::kPiecesPerRow;
                const int32_t src = a.tl_src[c0 + p];
                const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(F) +
                                                                ((size_t)src * CC * Cfg::kElt + piece * 16));
                *reinterpret_cast<uint4*>(abuf + (size_t)p * Cfg::kRowBytes + piece * 16) = v;
            }
            if (tid < m) s_row[tid] = (uint16_t)(a.tl_row[c0 + tid] - q0 * 64);
            __syncthreads();
            const int nblk = (m + 15) >> 4;
            for (int blk = bs; blk < nblk; blk += Cfg::kNBS) {
                f32x4 d = {0.f, 0.f, 0.f, 0.f};
                const unsigned char* arow = abuf + (size_t)(blk * 16 + n16) * Cfg::kRowBytes;
#pragma unroll
                for (int s = 0; s < kGroups; ++s) {
                    if constexpr (kIsF32) {
                        const f32x4 av = *reinterpret_cast<const f32x4*>(arow + (s * 16 + g * 4) * 4);
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(av[0], bf[s][0], d, 0, 0, 0);
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(av[1], bf[s][1], d, 0, 0, 0);
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(av[2], bf[s][2], d, 0, 0, 0);
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(av[3], bf[s][3], d, 0, 0, 0);
                    } else {
                        const bf16x8 av = *reinterpret_cast<const bf16x8*>(arow + (s * 32 + g * 8) * 2);
                        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh[s], d, 0, 0, 0);
                    }
                }
                // d[j] is link blk*16 + 4*g + j, channel n16 of this wavefront's slice
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int p = blk * 16 + g * 4 + j;
                    if (p < m) acc[(int)s_row[p] * Cfg::kAccStride + cs * 16 + n16] += d[j];
                }
            }
        }
    }
    __syncthreads();
    const int64_t row0 = tile * kTileRows + q0 * 64;
    constexpr int kQuads = COT / 4;
    for (int idx = tid; idx < TR * kQuads; idx += 256) {
        const int r = idx / kQuads, c4 = (idx % kQuads) * 4;
        const int64_t row = row0 + r;
        if (row >= a.n_rows) continue;
        const f32x4 v = *reinterpret_cast<const f32x4*>(acc + r * Cfg::kAccStride + c4);
        if constexpr (kIsF32) {
            *reinterpret_cast<f32x4*>(static_cast<float*>(a.g) + row * a.co_total + co0 + c4) = v;
        } else {
            ushort4 o;
            o.x = f32_to_bf16(v[0]);
            o.y = f32_to_bf16(v[1]);
            o.z = f32_to_bf16(v[2]);
            o.w = f32_to_bf16(v[3]);
            *reinterpret_cast<ushort4*>(static_cast<bf16_t*>(a.g) + row * a.co_total + co0 + c4) = o;
        }
    }
}

// Plain kernel for channel counts the matrix-core kernel does not take: one thread per (row, channel),
// walking the neighbour table.  Weights as stored, W[kvol][cout][cin]; (w_cc, w_co) are the element strides
// of the contraction / destination channel inside one offset's matrix.
template <typename T>
__global__ __launch_bounds__(256) void gather_plain_kernel(const int32_t* __restrict__ nbr, int64_t n_rows, int kvol,
                                                           int flip, const T* __restrict__ F, const T* __restrict__ W,
                                                           T* __restrict__ G, int cc, int co, int w_cc, int w_co) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_rows * co) return;
    const int64_t row = idx / co;
    const int c = (int)(idx % co);
    float acc = 0.f;
    for (int kk = 0; kk < kvol; ++kk) {
        const int32_t src = nbr[(int64_t)kk * n_rows + row];
        if (src < 0) continue;
        const int wk = flip ? kvol - 1 - kk : kk;
        const T* wp = W + (size_t)wk * cc * co + (size_t)c * w_co;
        const T* fp = F + (size_t)src * cc;
        for (int j = 0; j < cc; ++j) {
            if constexpr (std::is_same<T, float>::value)
                acc = fmaf(wp[(size_t)j * w_cc], fp[j], acc);
            else
                acc = fmaf(bf16_to_f32(wp[(size_t)j * w_cc]), bf16_to_f32(fp[j]), acc);
        }
    }
    if constexpr (std::is_same<T, float>::value)
        G[idx] = acc;
    else
        G[idx] = f32_to_bf16(acc);
}

// W[kvol][cout][cin] -> Wt[kvol][cin][cout]
template <typename T>
__global__ __launch_bounds__(256) void transpose_w_kernel(const T* __restrict__ w, T* __restrict__ wt, int kvol,
                                                          int cout, int cin) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t per = (int64_t)cout * cin;
    if (idx >= per * kvol) return;
    const int k = (int)(idx / per);
    const int rem = (int)(idx % per);
    const int ci = rem / cout, co = rem % cout;  // destination order
    wt[idx] = w[(size_t)k * per + (size_t)co * cin + ci];
}

template <typename T, int CC, int COT, int TR>
int launch_gather(const GatherArgs& a, hipStream_t s) {
    using Cfg = GatherCfg<T, CC, COT, TR>;
    auto kern = gather_mma_kernel<T, CC, COT, TR>;
    static bool attr_set = false;  // one-time opt-in to > 64 KB of dynamic LDS
    if (!attr_set) {
        SP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)Cfg::kLds));
        attr_set = true;
    }
    const int64_t ntiles = (a.n_rows + kTileRows - 1) / kTileRows;
    dim3 grid((unsigned)(ntiles * (kTileRows / TR)), (unsigned)(a.co_total / COT));
    hipLaunchKernelGGL(kern, grid, dim3(256), Cfg::kLds, s, a);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

template <typename T, int CC>
int dispatch_co(const GatherArgs& a, hipStream_t s) {
    // rows per workgroup: keep the accumulator + staging within ~64 KB so two workgroups share a CU
    if (a.co_total % 64 == 0) return launch_gather<T, CC, 64, 128>(a, s);
    if (a.co_total % 32 == 0) return launch_gather<T, CC, 32, 128>(a, s);
    return launch_gather<T, CC, 16, 128>(a, s);
}

template <typename T>
int dispatch_cc(int cc, const GatherArgs& a, hipStream_t s) {
    switch (cc) {
        case 16:
            if constexpr (std::is_same<T, float>::value) return dispatch_co<T, 16>(a, s);
            break;
        case 32: return dispatch_co<T, 32>(a, s);
        case 64: return dispatch_co<T, 64>(a, s);
        case 128: return dispatch_co<T, 128>(a, s);
        case 256: return dispatch_co<T, 256>(a, s);
        default: break;
    }
    return SP_ERR_UNSUPPORTED;
}

bool mma_shape_ok(int cc, int co, sp_dtype dt) {
    if (co % 16 != 0) return false;
    if (dt == SP_F32) return cc == 16 || cc == 32 || cc == 64 || cc == 128 || cc == 256;
    return cc == 32 || cc == 64 || cc == 128 || cc == 256;
}

}  // namespace

// side: which rows are destinations.  w_transposed = false: W[k][co][cc] as stored (forward);
// true: the stored W is [k][cc][co] (data gradient), transposed into pool memory first for the MFMA path.
int conv_gather(const MapSide& side, int kvol, const void* d_f, const void* d_w, bool w_transposed, void* d_g, int cc,
                int co, sp_dtype dt, hipStream_t s) {
    if (side.n_rows == 0) return SP_OK;
    const size_t elt = dt == SP_F32 ? 4 : 2;
    if (mma_shape_ok(cc, co, dt)) {
        Buf wt;
        const void* w_use = d_w;
        if (w_transposed) {
            const int64_t n = (int64_t)kvol * cc * co;
            wt = dev_alloc((size_t)n * elt);
            if (!wt) return SP_ERR_ALLOC;
            // stored matrix is [cout = cc][cin = co]; the kernel wants [co][cc]
            if (dt == SP_F32)
                hipLaunchKernelGGL(transpose_w_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                                   static_cast<const float*>(d_w), ptr<float>(wt), kvol, cc, co);
            else
                hipLaunchKernelGGL(transpose_w_kernel<bf16_t>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                                   static_cast<const bf16_t*>(d_w), ptr<bf16_t>(wt), kvol, cc, co);
            w_use = wt->p;
        }
        GatherArgs a;
        a.tl_off = ptr<int32_t>(side.tl_off);
        a.tl_src = ptr<int32_t>(side.tl_src);
        a.tl_row = ptr<uint16_t>(side.tl_row);
        a.f = d_f;
        a.w = w_use;
        a.g = d_g;
        a.n_rows = side.n_rows;
        a.kvol = kvol;
        a.co_total = co;
        a.flip = side.flip ? 1 : 0;
        return dt == SP_F32 ? dispatch_cc<float>(cc, a, s) : dispatch_cc<bf16_t>(cc, a, s);
    }
    const int64_t n = side.n_rows * co;
    const int w_cc = w_transposed ? co : 1, w_co = w_transposed ? 1 : cc;
    if (dt == SP_F32)
        hipLaunchKernelGGL(gather_plain_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           ptr<int32_t>(side.nbr), side.n_rows, kvol, side.flip ? 1 : 0, static_cast<const float*>(d_f),
                           static_cast<const float*>(d_w), static_cast<float*>(d_g), cc, co, w_cc, w_co);
    else
        hipLaunchKernelGGL(gather_plain_kernel<bf16_t>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           ptr<int32_t>(side.nbr), side.n_rows, kvol, side.flip ? 1 : 0,
                           static_cast<const bf16_t*>(d_f), static_cast<const bf16_t*>(d_w),
                           static_cast<bf16_t*>(d_g), cc, co, w_cc, w_co);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

}  // namespace sp

using namespace sp;

namespace {
// a: source features (rows_a), b: weights, c: destination (rows_c); a zero-sized buffer may be NULL
int check_conv_args(const sp_kmap_t* m, const void* a, int64_t rows_a, const void* b, const void* c, int64_t rows_c,
                    int cin, int cout, sp_dtype dt) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (cin < 1 || cout < 1 || cin > 4096 || cout > 4096) return fail(SP_ERR_INVALID_ARG, "bad channel count");
    if (dt != SP_F32 && dt != SP_BF16) return fail(SP_ERR_INVALID_ARG, "bad dtype");
    if (!b || (!a && rows_a > 0) || (!c && rows_c > 0))
        return fail(SP_ERR_INVALID_ARG, "a feature/weight pointer is NULL");
    if ((((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 15) != 0)
        return fail(SP_ERR_INVALID_ARG, "feature/weight pointers must be 16-byte aligned");
    return SP_OK;
}
}  // namespace

extern "C" {

int sp_conv_fwd(const sp_kmap_t* m, const void* d_x, const void* d_w, void* d_y, int32_t cin, int32_t cout,
                sp_dtype dt, void* stream) {
    SP_TRY(check_conv_args(m, d_x, m ? m->n_in : 0, d_w, d_y, m ? m->n_out : 0, cin, cout, dt));
    return conv_gather(m->out_side, m->kvol, d_x, d_w, false, d_y, cin, cout, dt, (hipStream_t)stream);
}

int sp_conv_bwd_data(const sp_kmap_t* m, const void* d_dy, const void* d_w, void* d_dx, int32_t cin, int32_t cout,
                     sp_dtype dt, void* stream) {
    SP_TRY(check_conv_args(m, d_dy, m ? m->n_out : 0, d_w, d_dx, m ? m->n_in : 0, cin, cout, dt));
    return conv_gather(m->in_side, m->kvol, d_dy, d_w, true, d_dx, cout, cin, dt, (hipStream_t)stream);
}

}  // extern "C"
