// Device-wide exclusive prefix sum of int32 (reduce, scan of block sums, apply).  Used to turn
// first-occurrence flags into row numbers and per-(tile, offset) pair counts into list offsets.
#include "sp_internal.h"

namespace sp {
namespace {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;

__device__ __forceinline__ int wave_inclusive_scan(int v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread over the block (blockDim.x a multiple of 64, <= 1024).
// Returns the exclusive prefix; *block_total receives the block's sum (same value in every thread).
__device__ __forceinline__ int block_exclusive_scan(int v, int* block_total) {
    __shared__ int wsum[16];
    __shared__ int wtot;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    int inc = wave_inclusive_scan(v);
    __syncthreads();  // protects wsum/wtot against a previous call's readers
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < nw; ++i) {
            int t = wsum[i];
            wsum[i] = run;
            run += t;
        }
        wtot = run;
    }
    __syncthreads();
    *block_total = wtot;
    return wsum[w] + inc - v;
}

__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(const int32_t* __restrict__ in, int64_t n,
                                                                   int32_t* __restrict__ partials) {
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int s = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j)
        if (base + j < n) s += in[base + j];
    int tot;
    (void)block_exclusive_scan(s, &tot);
    if (threadIdx.x == 0) partials[blockIdx.x] = tot;
}

// In-place exclusive scan of `partials` by one block, in chunks of blockDim.x with a running carry.
__global__ __launch_bounds__(1024) void scan_partials_kernel(int32_t* __restrict__ partials, int64_t nb,
                                                             int32_t* __restrict__ total) {
    int carry = 0;
    for (int64_t c = 0; c < nb; c += blockDim.x) {
        int64_t i = c + threadIdx.x;
        int v = i < nb ? partials[i] : 0;
        int tot;
        int ex = block_exclusive_scan(v, &tot);
        if (i < nb) partials[i] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0 && total) *total = carry;
}

__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(const int32_t* __restrict__ in,
                                                                  int32_t* __restrict__ out, int64_t n,
                                                                  const int32_t* __restrict__ partials,
                                                                  int32_t* __restrict__ total) {
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int v[kScanItems];
    int s = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = base + j < n ? in[base + j] : 0;
        s += v[j];
    }
    int tot;
    int ex = block_exclusive_scan(s, &tot) + (partials ? partials[blockIdx.x] : 0);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (base + j < n) out[base + j] = ex;
        ex += v[j];
    }
    if (!partials && total && threadIdx.x == 0) *total = tot;  // single-block case
}

__global__ void scan_zero_total_kernel(int32_t* total) { *total = 0; }

}  // namespace

int exclusive_scan_i32(const int32_t* d_in, int32_t* d_out, int64_t n, int32_t* d_total, hipStream_t s) {
    if (n <= 0) {
        if (d_total) hipLaunchKernelGGL(scan_zero_total_kernel, dim3(1), dim3(1), 0, s, d_total);
        return SP_OK;
    }
    const int64_t nb = (n + kScanTile - 1) / kScanTile;
    if (nb == 1) {
        hipLaunchKernelGGL(scan_apply_kernel, dim3(1), dim3(kScanThreads), 0, s, d_in, d_out, n, nullptr, d_total);
    } else {
        Buf partials = dev_alloc((size_t)nb * sizeof(int32_t));
        if (!partials) return SP_ERR_ALLOC;
        hipLaunchKernelGGL(scan_reduce_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, d_in, n,
                           ptr<int32_t>(partials));
        hipLaunchKernelGGL(scan_partials_kernel, dim3(1), dim3(1024), 0, s, ptr<int32_t>(partials), nb, d_total);
        hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, d_in, d_out, n,
                           ptr<int32_t>(partials), d_total);
        // `partials` returns to the pool here; any later user is ordered after these kernels on the stream.
    }
    SP_HIP(hipGetLastError());
    return SP_OK;
}

}  // namespace sp
