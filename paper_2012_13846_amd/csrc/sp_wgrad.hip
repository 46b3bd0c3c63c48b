// Weight gradient of Eq. 2: dW_k[co][ci] = sum over the links (i,o) of offset k of dY[o][co] * X[i][ci].
//
// Per offset this is a GEMM whose contraction runs over that offset's link list.  The lists of all offsets
// are cut into chunks; one workgroup reduces one chunk into a partial Cout x Cin block on the matrix cores,
// and a second kernel adds the partials of each offset in a fixed order.  No atomics: the result is
// reproducible run to run.
//
// The contraction index (the link) is the row index of both gathered operands, while memory is contiguous
// along channels: both operands reach the matrix cores transposed.  The staged kernel gathers rows with
// coalesced 16-byte loads into LDS (double buffered, one barrier per step) and reads MFMA fragments from
// there: fp32 with one 4-byte read per lane (lane = channel, links in lane groups), bf16 with the LDS
// transpose read, which hands a lane 4 consecutive links of one channel out of row-major storage.
#include <type_traits>

#include "sp_internal.h"

namespace sp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;

__device__ __forceinline__ float load_f32(const float* p) { return *p; }
__device__ __forceinline__ float load_f32(const bf16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

// Which (offset, chunk) a work item is: items are numbered offset by offset, ceil(count/chunk) per offset.
struct Item {
    int k;
    int64_t beg, end;
};
__device__ __forceinline__ Item locate_item(const int32_t* __restrict__ koff, int kvol, int chunk, int item) {
    Item it;
    int first = 0;
    for (int k = 0; k < kvol; ++k) {
        const int cnt = koff[k + 1] - koff[k];
        const int ni = (cnt + chunk - 1) / chunk;
        if (item < first + ni) {
            it.k = k;
            it.beg = (int64_t)koff[k] + (int64_t)(item - first) * chunk;
            it.end = min(it.beg + chunk, (int64_t)koff[k + 1]);
            return it;
        }
        first += ni;
    }
    it.k = -1;
    it.beg = it.end = 0;
    return it;
}

// grid (items, cout/COB, cin/CIB); 4 wavefronts each take every 4th group of 4 links of the chunk.
// MFMA 16x16x4: A[m = channel of dY][kk = link], B[kk = link][n = channel of X].
template <typename T, int COB, int CIB>
__global__ __launch_bounds__(256) void wgrad_partial_kernel(const int32_t* __restrict__ pair_in,
                                                            const int32_t* __restrict__ pair_out,
                                                            const int32_t* __restrict__ koff, int kvol, int chunk,
                                                            const T* __restrict__ X, const T* __restrict__ dY, int cin,
                                                            int cout, float* __restrict__ part) {
    constexpr int NCO = COB / 16, NCI = CIB / 16;
    __shared__ float red[COB * CIB];
    const Item it = locate_item(koff, kvol, chunk, blockIdx.x);
    if (it.k < 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int co0 = blockIdx.y * COB, ci0 = blockIdx.z * CIB;

    f32x4 acc[NCO][NCI];
#pragma unroll
    for (int a = 0; a < NCO; ++a)
#pragma unroll
        for (int b = 0; b < NCI; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Software pipeline in super-steps of kU steps (kU * 4 links per wavefront): the rows of super-step s+1
    // and the link indices of super-step s+2 are requested before the MFMAs of super-step s are issued.
    constexpr int kU = 4;
    const int64_t first_p = it.beg + wave * 4 + g;  // this lane's link in step 0; step j is 16*j further
    auto load_idx = [&](int64_t p, int32_t (&o)[kU], int32_t (&i)[kU]) {
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const bool live = p + 16 * u < it.end;
            o[u] = live ? pair_out[p + 16 * u] : -1;
            i[u] = live ? pair_in[p + 16 * u] : 0;
        }
    };
    auto load_rows = [&](const int32_t (&o)[kU], const int32_t (&i)[kU], float (&av)[kU][NCO], float (&bv)[kU][NCI]) {
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const bool live = o[u] >= 0;
            const T* dyp = dY + (size_t)(live ? o[u] : 0) * cout + co0 + n16;
            const T* xp = X + (size_t)(live ? i[u] : 0) * cin + ci0 + n16;
#pragma unroll
            for (int a = 0; a < NCO; ++a) av[u][a] = live ? load_f32(dyp + a * 16) : 0.f;
#pragma unroll
            for (int b = 0; b < NCI; ++b) bv[u][b] = live ? load_f32(xp + b * 16) : 0.f;
        }
    };
    int32_t o2[kU], i2[kU];
    float av[kU][NCO], bv[kU][NCI];
    {
        int32_t o1[kU], i1[kU];
        load_idx(first_p, o1, i1);
        load_idx(first_p + 16 * kU, o2, i2);
        load_rows(o1, i1, av, bv);
    }
    for (int64_t p = first_p; p - g < it.end; p += 16 * kU) {
        float an[kU][NCO], bn[kU][NCI];
        int32_t o3[kU], i3[kU];
        load_idx(p + 32 * kU, o3, i3);
        load_rows(o2, i2, an, bn);
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int a = 0; a < NCO; ++a)
#pragma unroll
                for (int b = 0; b < NCI; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][a], bv[u][b], acc[a][b], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
#pragma unroll
            for (int a = 0; a < NCO; ++a) av[u][a] = an[u][a];
#pragma unroll
            for (int b = 0; b < NCI; ++b) bv[u][b] = bn[u][b];
            o2[u] = o3[u];
            i2[u] = i3[u];
        }
    }
    // acc[a][b][j] is element (co = a*16 + 4*g + j, ci = b*16 + n16); add the 4 wavefronts in order
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int a = 0; a < NCO; ++a)
#pragma unroll
                for (int b = 0; b < NCI; ++b)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int e = (a * 16 + g * 4 + j) * CIB + b * 16 + n16;
                        red[e] = (w == 0 ? 0.f : red[e]) + acc[a][b][j];
                    }
        }
        __syncthreads();
    }
    float* dst = part + (size_t)blockIdx.x * cout * cin;
    for (int e = tid; e < COB * CIB; e += 256) {
        const int co = e / CIB, ci = e % CIB;
        dst[(size_t)(co0 + co) * cin + ci0 + ci] = red[e];
    }
}

// dW[k][e] = sum of the partials of offset k's items, in a fixed order: 4 interleaved running sums per
// element (one per wavefront of the block), each over every 4th item, then added 0+1+2+3.
// grid (per/64, kvol), block 256 = 64 elements x 4 item groups.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part,
                                                           const int32_t* __restrict__ koff, int kvol, int chunk,
                                                           int per, float* __restrict__ dw) {
    __shared__ float red[4][64];
    const int k = blockIdx.y;
    const int el = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + el;
    int first = 0;
    for (int j = 0; j < k; ++j) first += (koff[j + 1] - koff[j] + chunk - 1) / chunk;
    const int ni = (koff[k + 1] - koff[k] + chunk - 1) / chunk;
    float s0 = 0.f, s1 = 0.f;
    if (e < per) {
        const float* p = part + (size_t)first * per + e;
        int it = grp;
        for (; it + 4 < ni; it += 8) {  // two independent loads in flight
            s0 += p[(size_t)it * per];
            s1 += p[(size_t)(it + 4) * per];
        }
        if (it < ni) s0 += p[(size_t)it * per];
    }
    red[grp][el] = s0 + s1;
    __syncthreads();
    if (grp == 0 && e < per) dw[(size_t)k * per + e] = ((red[0][el] + red[1][el]) + red[2][el]) + red[3][el];
}


// ---------------------------------------------------------------------------------------------------------
// Staged kernel.  Tile COB x CIB of dW per workgroup; WCO x WCI x WK wavefronts: the tile is cut WCO x WCI
// ways and each step's 32*WK links WK ways.  grid (items, cout/COB, cin/CIB).
// ---------------------------------------------------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T, int COB, int CIB, int WCO, int WCI, int WK>
struct StagedCfg {
    static constexpr int kElt = sizeof(T);
    static constexpr int kWaves = WCO * WCI * WK, kThreads = 64 * kWaves;
    static constexpr int kS = 32 * WK;                     // links per step
    static constexpr int kPad = 16 * kElt;                 // row pad: fragment reads of 4 rows hit disjoint banks
    static constexpr int kPA = COB * kElt + kPad, kPB = CIB * kElt + kPad;  // staged row pitch of dY / X rows
    static constexpr int kPiecesA = COB * kElt / 16, kPiecesB = CIB * kElt / 16;  // 16-byte pieces per row
    static constexpr int kLoadsA = (kS * kPiecesA + kThreads - 1) / kThreads;
    static constexpr int kLoadsB = (kS * kPiecesB + kThreads - 1) / kThreads;
    static constexpr int kBufBytes = kS * (kPA + kPB);
    static constexpr int kTA = COB / WCO / 16, kTB = CIB / WCI / 16;  // 16x16 tiles per wavefront
    static constexpr int kRedBytes = WK > 1 ? COB * CIB * 4 : 0;
    static constexpr int kLds = 2 * kBufBytes > kRedBytes ? 2 * kBufBytes : kRedBytes;
    static_assert(COB % (16 * WCO) == 0 && CIB % (16 * WCI) == 0, "tile split");
};

struct StagedArgs {
    const int32_t* pair_in;
    const int32_t* pair_out;
    const int32_t* koff;
    const void* x;
    const void* dy;
    float* part;
    int kvol, chunk, cin, cout;
    uint32_t x_bytes, dy_bytes, pair_bytes;  // buffer sizes (< 2 GiB each)
};

template <typename T, int COB, int CIB, int WCO, int WCI, int WK>
__global__ __launch_bounds__(64 * WCO * WCI * WK) void wgrad_staged_kernel(StagedArgs a) {
    using Cfg = StagedCfg<T, COB, CIB, WCO, WCI, WK>;
    constexpr bool kIsF32 = std::is_same<T, float>::value;
    constexpr int kTA = Cfg::kTA, kTB = Cfg::kTB, kPA = Cfg::kPA, kPB = Cfg::kPB, kS = Cfg::kS;
    constexpr int kLoadsA = Cfg::kLoadsA, kLoadsB = Cfg::kLoadsB, kThreads = Cfg::kThreads;
    extern __shared__ __align__(16) unsigned char smem[];

    const Item it = locate_item(a.koff, a.kvol, a.chunk, blockIdx.x);
    if (it.k < 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wci = (wave / WK) % WCI, wco = wave / (WK * WCI);
    const int n16 = lane & 15, g = lane >> 4;
    const int co0 = blockIdx.y * COB, ci0 = blockIdx.z * CIB;

    // Buffer addressing: a lane whose link lies past the chunk's end asks for an offset outside the buffer
    // and gets zeros, so the loop body has no branch around a load.
    constexpr int kRsrcFlags = 0x00020000;
    constexpr uint32_t kOutside = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.x), 0, (int)a.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rDY = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.dy), 0, (int)a.dy_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rPI =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(a.pair_in), 0, (int)a.pair_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rPO =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(a.pair_out), 0, (int)a.pair_bytes, kRsrcFlags);
    const uint32_t rowbytes_a = (uint32_t)a.cout * Cfg::kElt, rowbytes_b = (uint32_t)a.cin * Cfg::kElt;
    const uint32_t col_a = (uint32_t)co0 * Cfg::kElt, col_b = (uint32_t)ci0 * Cfg::kElt;

    // this thread's pieces of a step: piece q = tid + j * kThreads of the dY rows, likewise of the X rows
    struct Regs {
        int ia[kLoadsA], ib[kLoadsB];      // gathered row numbers
        u32x4 va[kLoadsA], vb[kLoadsB];    // gathered pieces
    };
    auto load_idx = [&](Regs& r, int64_t base) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoadsA; ++j) {
            const int64_t link = base + (tid + j * kThreads) / Cfg::kPiecesA;
            r.ia[j] = (int)__builtin_amdgcn_raw_buffer_load_b32(rPO, link < it.end ? (uint32_t)link * 4u : kOutside, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < kLoadsB; ++j) {
            const int64_t link = base + (tid + j * kThreads) / Cfg::kPiecesB;
            r.ib[j] = (int)__builtin_amdgcn_raw_buffer_load_b32(rPI, link < it.end ? (uint32_t)link * 4u : kOutside, 0, 0);
        }
    };
    auto load_rows = [&](Regs& r, int64_t base) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoadsA; ++j) {
            const int q = tid + j * kThreads;
            const int64_t link = base + q / Cfg::kPiecesA;
            const uint32_t off = (uint32_t)r.ia[j] * rowbytes_a + col_a + (q % Cfg::kPiecesA) * 16;
            r.va[j] = __builtin_amdgcn_raw_buffer_load_b128(rDY, link < it.end ? off : kOutside, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < kLoadsB; ++j) {
            const int q = tid + j * kThreads;
            const int64_t link = base + q / Cfg::kPiecesB;
            const uint32_t off = (uint32_t)r.ib[j] * rowbytes_b + col_b + (q % Cfg::kPiecesB) * 16;
            r.vb[j] = __builtin_amdgcn_raw_buffer_load_b128(rX, link < it.end ? off : kOutside, 0, 0);
        }
    };
    auto store_rows = [&](const Regs& r, unsigned char* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoadsA; ++j) {
            const int q = tid + j * kThreads;
            if (kS * Cfg::kPiecesA % kThreads == 0 || q < kS * Cfg::kPiecesA)
                *reinterpret_cast<u32x4*>(buf + (q / Cfg::kPiecesA) * kPA + (q % Cfg::kPiecesA) * 16) = r.va[j];
        }
#pragma unroll
        for (int j = 0; j < kLoadsB; ++j) {
            const int q = tid + j * kThreads;
            if (kS * Cfg::kPiecesB % kThreads == 0 || q < kS * Cfg::kPiecesB)
                *reinterpret_cast<u32x4*>(buf + kS * kPA + (q / Cfg::kPiecesB) * kPB + (q % Cfg::kPiecesB) * 16) = r.vb[j];
        }
    };

    f32x4 acc[kTA][kTB];
#pragma unroll
    for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
        for (int tb = 0; tb < kTB; ++tb) acc[ta][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this wavefront's 32 links of the step, its channel slices
    const int a_col = (wco * kTA * 16) * Cfg::kElt, b_col = (wci * kTB * 16) * Cfg::kElt;
    auto compute = [&](const unsigned char* buf) __attribute__((always_inline)) {
        const unsigned char* A = buf + (32 * wk) * kPA + a_col;
        const unsigned char* B = buf + kS * kPA + (32 * wk) * kPB + b_col;
        if constexpr (kIsF32) {
            // MFMA 16x16x4: lane (channel n16, link g) of both operands
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float av[kTA], bv[kTB];
#pragma unroll
                for (int ta = 0; ta < kTA; ++ta) av[ta] = *reinterpret_cast<const float*>(A + (4 * j + g) * kPA + (ta * 16 + n16) * 4);
#pragma unroll
                for (int tb = 0; tb < kTB; ++tb) bv[tb] = *reinterpret_cast<const float*>(B + (4 * j + g) * kPB + (tb * 16 + n16) * 4);
#pragma unroll
                for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                    for (int tb = 0; tb < kTB; ++tb)
                        acc[ta][tb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ta], bv[tb], acc[ta][tb], 0, 0, 0);
            }
        } else {
            // MFMA 16x16x32: lane (channel n16, links 8g .. 8g+7).  One transpose read: the 16 lanes of group g
            // point at 4 rows x 16 channels (lane i: row i/4, channels 4*(i%4)..+3) and lane i receives
            // channel i of those 4 rows.
            typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
            auto frag = [&](const unsigned char* base, int pitch) __attribute__((always_inline)) {
                const unsigned char* p = base + (8 * g + (n16 >> 2)) * pitch + (n16 & 3) * 8;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * pitch));
                const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                return __builtin_bit_cast(bf16x8, v);
            };
            bf16x8 av[kTA], bv[kTB];
#pragma unroll
            for (int ta = 0; ta < kTA; ++ta) av[ta] = frag(A + ta * 32, kPA);
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb) bv[tb] = frag(B + tb * 32, kPB);
#pragma unroll
            for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                for (int tb = 0; tb < kTB; ++tb)
                    acc[ta][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[ta], bv[tb], acc[ta][tb], 0, 0, 0);
        }
    };

    // step s: rows of step s+1 and row numbers of step s+2 are requested before step s is computed
    Regs r = {};
    load_idx(r, it.beg);
    load_rows(r, it.beg);
    load_idx(r, it.beg + kS);
    store_rows(r, smem);
    __syncthreads();
    int cur = 0;
    for (int64_t base = it.beg; base < it.end; base += kS) {
        load_rows(r, base + kS);
        load_idx(r, base + 2 * kS);
        compute(smem + cur * Cfg::kBufBytes);
        store_rows(r, smem + (cur ^ 1) * Cfg::kBufBytes);
        __syncthreads();
        cur ^= 1;
    }

    // acc[ta][tb][j] is element (co = .. + 4*g + j, ci = .. + n16).  The WK link slices are added in order.
    float* dst = a.part + (size_t)blockIdx.x * a.cout * a.cin;
    if constexpr (WK > 1) {
        float* red = reinterpret_cast<float*>(smem);
        for (int w = 0; w < WK; ++w) {
            if (wk == w) {
#pragma unroll
                for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                    for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int e = ((wco * kTA + ta) * 16 + g * 4 + j) * CIB + (wci * kTB + tb) * 16 + n16;
                            red[e] = (w == 0 ? 0.f : red[e]) + acc[ta][tb][j];
                        }
            }
            __syncthreads();
        }
        for (int e = tid * 4; e < COB * CIB; e += kThreads * 4) {
            const int co = e / CIB, ci = e % CIB;
            *reinterpret_cast<f32x4*>(dst + (size_t)(co0 + co) * a.cin + ci0 + ci) = *reinterpret_cast<const f32x4*>(red + e);
        }
    } else {
#pragma unroll
        for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    dst[(size_t)(co0 + (wco * kTA + ta) * 16 + g * 4 + j) * a.cin + ci0 + (wci * kTB + tb) * 16 + n16] =
                        acc[ta][tb][j];
    }
}

// Plain kernel for channel counts that are not multiples of 16: one thread per weight element.
template <typename T>
__global__ __launch_bounds__(256) void wgrad_plain_kernel(const int32_t* __restrict__ pair_in,
                                                          const int32_t* __restrict__ pair_out,
                                                          const int32_t* __restrict__ koff, const T* __restrict__ X,
                                                          const T* __restrict__ dY, int cin, int cout,
                                                          float* __restrict__ dw) {
    const int k = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= cin * cout) return;
    const int co = e / cin, ci = e % cin;
    float s = 0.f;
    for (int p = koff[k]; p < koff[k + 1]; ++p)
        s = fmaf(load_f32(dY + (size_t)pair_out[p] * cout + co), load_f32(X + (size_t)pair_in[p] * cin + ci), s);
    dw[(size_t)k * cin * cout + e] = s;
}

template <typename T, int COB, int CIB>
void launch_partial(const sp_kmap* m, int items, int chunk, const void* x, const void* dy, int cin, int cout,
                    float* part, hipStream_t s) {
    hipLaunchKernelGGL((wgrad_partial_kernel<T, COB, CIB>), dim3(items, cout / COB, cin / CIB), dim3(256), 0, s,
                       ptr<int32_t>(m->pair_in), ptr<int32_t>(m->pair_out), ptr<int32_t>(m->d_koff), m->kvol, chunk,
                       static_cast<const T*>(x), static_cast<const T*>(dy), cin, cout, part);
}

template <typename T, int COB, int CIB, int WCO, int WCI, int WK>
int launch_staged(const sp_kmap* m, const void* x, const void* dy, int cin, int cout, float* dw, hipStream_t s) {
    using Cfg = StagedCfg<T, COB, CIB, WCO, WCI, WK>;
    auto kern = wgrad_staged_kernel<T, COB, CIB, WCO, WCI, WK>;
    static bool attr_set = false;  // one-time opt-in to > 64 KB of dynamic LDS
    if (!attr_set) {
        SP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)Cfg::kLds));
        attr_set = true;
    }
    // chunk: about 2048 workgroups over the whole launch, at least 4 steps each, a whole number of steps
    const int64_t tiles = (int64_t)(cout / COB) * (cin / CIB);
    int64_t want = 2048 / tiles;
    want = want < m->kvol ? m->kvol : want;
    int64_t chunk = (m->total + want - 1) / want;
    chunk = chunk < 4 * Cfg::kS ? 4 * Cfg::kS : (chunk > 16384 ? 16384 : chunk);
    chunk = (chunk + Cfg::kS - 1) / Cfg::kS * Cfg::kS;
    int64_t items = 0;
    for (int k = 0; k < m->kvol; ++k) items += (m->counts[k] + chunk - 1) / chunk;
    const int per = cin * cout;
    Buf part = dev_alloc((size_t)(items ? items : 1) * per * 4);
    if (!part) return SP_ERR_ALLOC;
    if (items > 0) {
        StagedArgs a;
        a.pair_in = ptr<int32_t>(m->pair_in);
        a.pair_out = ptr<int32_t>(m->pair_out);
        a.koff = ptr<int32_t>(m->d_koff);
        a.x = x;
        a.dy = dy;
        a.part = ptr<float>(part);
        a.kvol = m->kvol;
        a.chunk = (int)chunk;
        a.cin = cin;
        a.cout = cout;
        a.x_bytes = (uint32_t)((uint64_t)m->n_in * cin * sizeof(T));
        a.dy_bytes = (uint32_t)((uint64_t)m->n_out * cout * sizeof(T));
        a.pair_bytes = (uint32_t)((uint64_t)m->total * 4);
        hipLaunchKernelGGL(kern, dim3((unsigned)items, cout / COB, cin / CIB), dim3(Cfg::kThreads), Cfg::kLds, s, a);
    }
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((per + 63) / 64, m->kvol), dim3(256), 0, s, ptr<float>(part),
                       ptr<int32_t>(m->d_koff), m->kvol, (int)chunk, per, dw);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// largest of 128, 64, 32, 16 dividing c (c is a multiple of 16)
int channel_block(int c) { return c % 128 == 0 ? 128 : (c % 64 == 0 ? 64 : (c % 32 == 0 ? 32 : 16)); }

template <typename T>
int wgrad_typed(const sp_kmap* m, const void* x, const void* dy, float* dw, int cin, int cout, hipStream_t s) {
    const int kvol = m->kvol;
    if (cin % 16 || cout % 16) {
        hipLaunchKernelGGL(wgrad_plain_kernel<T>, dim3((cin * cout + 255) / 256, kvol), dim3(256), 0, s,
                           ptr<int32_t>(m->pair_in), ptr<int32_t>(m->pair_out), ptr<int32_t>(m->d_koff),
                           static_cast<const T*>(x), static_cast<const T*>(dy), cin, cout, dw);
        SP_HIP(hipGetLastError());
        return SP_OK;
    }
    const uint64_t lim = 0x7fffffffull;
    const bool small = (uint64_t)m->n_in * cin * sizeof(T) < lim && (uint64_t)m->n_out * cout * sizeof(T) < lim &&
                       (uint64_t)m->total * 4 < lim;
    if (small) {
        int cob = channel_block(cout), cib = channel_block(cin);
        if (cob == 128 && cib < 64) cob = 64;  // 128-wide tiles only in the combinations instantiated below
        if (cib == 128 && cob < 64) cib = 64;
#define SP_STAGED(COB, CIB, WCO, WCI, WK) \
    if (cob == COB && cib == CIB) return launch_staged<T, COB, CIB, WCO, WCI, WK>(m, x, dy, cin, cout, dw, s)
        SP_STAGED(128, 128, 2, 2, 1);
        SP_STAGED(128, 64, 2, 1, 2);
        SP_STAGED(64, 128, 1, 2, 2);
        SP_STAGED(64, 64, 2, 1, 2);
        SP_STAGED(64, 32, 2, 1, 2);
        SP_STAGED(32, 64, 1, 2, 2);
        SP_STAGED(64, 16, 2, 1, 2);
        SP_STAGED(16, 64, 1, 2, 2);
        SP_STAGED(32, 32, 1, 1, 2);
        SP_STAGED(32, 16, 1, 1, 4);
        SP_STAGED(16, 32, 1, 1, 4);
        SP_STAGED(16, 16, 1, 1, 4);
#undef SP_STAGED
    }
    // buffers of 2 GiB and more: fragment-shaped global loads with 64-bit addressing
    // chunk: about 1024 work items over the whole map, between 64 and 4096 links each, a multiple of 16
    int64_t chunk = (m->total + 1023) / 1024;
    chunk = chunk < 64 ? 64 : (chunk > 4096 ? 4096 : chunk);
    chunk = (chunk + 15) / 16 * 16;
    int64_t items = 0;
    for (int k = 0; k < kvol; ++k) items += (m->counts[k] + chunk - 1) / chunk;
    const int per = cin * cout;
    Buf part = dev_alloc((size_t)(items ? items : 1) * per * 4);
    if (!part) return SP_ERR_ALLOC;
    if (items > 0) {
        const bool co32 = cout % 32 == 0, ci32 = cin % 32 == 0;
        if (co32 && ci32) launch_partial<T, 32, 32>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
        else launch_partial<T, 16, 16>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
    }
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((per + 63) / 64, kvol), dim3(256), 0, s, ptr<float>(part),
                       ptr<int32_t>(m->d_koff), kvol, (int)chunk, per, dw);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

}  // namespace

int conv_wgrad(const sp_kmap* m, const void* d_x, const void* d_dy, float* d_dw, int cin, int cout, sp_dtype dt,
               hipStream_t s) {
    return dt == SP_F32 ? wgrad_typed<float>(m, d_x, d_dy, d_dw, cin, cout, s)
                        : wgrad_typed<bf16_t>(m, d_x, d_dy, d_dw, cin, cout, s);
}

}  // namespace sp

extern "C" int sp_conv_bwd_weight(const sp_kmap_t* m, const void* d_x, const void* d_dy, float* d_dw, int32_t cin,
                                  int32_t cout, sp_dtype dt, void* stream) {
    using namespace sp;
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (cin < 1 || cout < 1 || cin > 4096 || cout > 4096) return fail(SP_ERR_INVALID_ARG, "bad channel count");
    if (dt != SP_F32 && dt != SP_BF16) return fail(SP_ERR_INVALID_ARG, "bad dtype");
    if ((!d_x && m->n_in > 0) || (!d_dy && m->n_out > 0) || !d_dw)
        return fail(SP_ERR_INVALID_ARG, "a feature/gradient pointer is NULL");
    return conv_wgrad(m, d_x, d_dy, d_dw, cin, cout, dt, (hipStream_t)stream);
}
