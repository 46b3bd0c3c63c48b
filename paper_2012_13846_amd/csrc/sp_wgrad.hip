// Weight gradient of Eq. 2: dW_k[co][ci] = sum over the links (i,o) of offset k of dY[o][co] * X[i][ci].
//
// Per offset this is a GEMM whose contraction runs over that offset's link list.  The lists of all offsets
// are cut into chunks; one workgroup reduces one chunk into a partial Cout x Cin block on the matrix cores
// (operands gathered from global memory straight into MFMA fragments: lane = channel, so each gathered row
// is read as one contiguous segment), and a second kernel adds the partials of each offset in a fixed order.
// No atomics: the result is reproducible run to run.
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
        const bool co64 = cout % 64 == 0, ci64 = cin % 64 == 0, co32 = cout % 32 == 0, ci32 = cin % 32 == 0;
        if (co64 && ci64) launch_partial<T, 64, 64>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
        else if (co64 && ci32) launch_partial<T, 64, 32>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
        else if (co32 && ci64) launch_partial<T, 32, 64>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
        else if (co32 && ci32) launch_partial<T, 32, 32>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
        else if (co32) launch_partial<T, 32, 16>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
        else if (ci32) launch_partial<T, 16, 32>(m, (int)items, (int)chunk, x, dy, cin, cout, ptr<float>(part), s);
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
