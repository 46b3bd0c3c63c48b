// Device-wide exclusive prefix sums of int32, one or two arrays per launch pair.  Used to turn per-(sub-tile,
// offset) link counts into list offsets.  Two kernels: per-block sums, then every block adds up the sums of
// the blocks before it (a few thousand at most) and scans its own tile; a single-block scan of the block
// sums is slotted in between only when there are too many blocks for that.
#include "sp_internal.h"

namespace sp {
namespace {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;
// Up to this many blocks every block adds up its predecessors' sums itself; beyond, one more launch scans them.
// (Not const: a test hook lowers it so that small inputs run the extra launch.)
int64_t g_self_base_max_blocks = 4096;

struct ScanJobDev {
    int32_t* data;
    int64_t n;
    int32_t* total;      // may be null
    int32_t* koff;       // may be null: koff[i] = exclusive prefix at element i*koff_stride, koff[koff_n] = total
    int64_t koff_stride;
    int32_t koff_n;
    int32_t* partials;
    int64_t nb;
    int32_t partials_scanned;
};
struct ScanArgs {
    ScanJobDev job[2];
    int njobs;
};

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

__device__ __forceinline__ const ScanJobDev& pick_job(const ScanArgs& a, int64_t* local_block) {
    int64_t b = blockIdx.x;
    if (a.njobs > 1 && b >= a.job[0].nb) {
        *local_block = b - a.job[0].nb;
        return a.job[1];
    }
    *local_block = b;
    return a.job[0];
}

__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(ScanArgs a) {
    int64_t lb;
    const ScanJobDev& j = pick_job(a, &lb);
    const int64_t base = lb * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i)
        if (base + i < j.n) s += j.data[base + i];
    int tot;
    (void)block_exclusive_scan(s, &tot);
    if (threadIdx.x == 0) j.partials[lb] = tot;
}

// In-place exclusive scan of `partials` by one block, in chunks of blockDim.x with a running carry.
__global__ __launch_bounds__(1024) void scan_partials_kernel(int32_t* __restrict__ partials, int64_t nb) {
    int carry = 0;
    for (int64_t c = 0; c < nb; c += blockDim.x) {
        int64_t i = c + threadIdx.x;
        int v = i < nb ? partials[i] : 0;
        int tot;
        int ex = block_exclusive_scan(v, &tot);
        if (i < nb) partials[i] = carry + ex;
        carry += tot;
    }
}

__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(ScanArgs a) {
    int64_t lb;
    const ScanJobDev& j = pick_job(a, &lb);
    // sum of the blocks before this one
    int before;
    if (j.partials_scanned) {
        before = j.partials[lb];
    } else {
        int s = 0;
        for (int64_t b = threadIdx.x; b < lb; b += kScanThreads) s += j.partials[b];
        int tot;
        (void)block_exclusive_scan(s, &tot);
        before = tot;
    }
    const int64_t base = lb * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int v[kScanItems];
    int s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        v[i] = base + i < j.n ? j.data[base + i] : 0;
        s += v[i];
    }
    int tot;
    int ex = block_exclusive_scan(s, &tot) + before;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < j.n) {
            j.data[base + i] = ex;
            if (j.koff && (base + i) % j.koff_stride == 0) j.koff[(base + i) / j.koff_stride] = ex;
        }
        ex += v[i];
    }
    if (lb == j.nb - 1 && threadIdx.x == 0) {
        if (j.total) *j.total = before + tot;
        if (j.koff) j.koff[j.koff_n] = before + tot;
    }
}

__global__ void scan_empty_kernel(ScanJobDev j) {
    if (threadIdx.x == 0 && j.total) *j.total = 0;
    if (j.koff && (int)threadIdx.x <= j.koff_n) j.koff[threadIdx.x] = 0;
}

}  // namespace

int exclusive_scan_jobs(const ScanJob* jobs, int njobs, hipStream_t s) {
    ScanArgs a{};
    a.njobs = 0;
    Buf partials[2];
    for (int i = 0; i < njobs && i < 2; ++i) {
        const ScanJob& in = jobs[i];
        ScanJobDev d{};
        d.data = in.data;
        d.n = in.n;
        d.total = in.total;
        d.koff = in.koff;
        d.koff_stride = in.koff_stride > 0 ? in.koff_stride : 1;
        d.koff_n = in.koff_n;
        if (in.n <= 0) {  // nothing to scan: only the outputs
            hipLaunchKernelGGL(scan_empty_kernel, dim3(1), dim3(128), 0, s, d);
            continue;
        }
        d.nb = (in.n + kScanTile - 1) / kScanTile;
        partials[a.njobs] = dev_alloc((size_t)d.nb * sizeof(int32_t), s);
        if (!partials[a.njobs]) return SP_ERR_ALLOC;
        d.partials = ptr<int32_t>(partials[a.njobs]);
        d.partials_scanned = d.nb > g_self_base_max_blocks ? 1 : 0;
        a.job[a.njobs++] = d;
    }
    if (a.njobs > 0) {
        const unsigned nblocks = (unsigned)(a.job[0].nb + (a.njobs > 1 ? a.job[1].nb : 0));
        hipLaunchKernelGGL(scan_reduce_kernel, dim3(nblocks), dim3(kScanThreads), 0, s, a);
        for (int i = 0; i < a.njobs; ++i)
            if (a.job[i].partials_scanned)
                hipLaunchKernelGGL(scan_partials_kernel, dim3(1), dim3(1024), 0, s, a.job[i].partials, a.job[i].nb);
        hipLaunchKernelGGL(scan_apply_kernel, dim3(nblocks), dim3(kScanThreads), 0, s, a);
    }
    SP_HIP(hipGetLastError());
    return SP_OK;  // `partials` return to the pool; later users are ordered behind these kernels on the stream
}

}  // namespace sp

// Test hook, not part of the ABI (not declared in sp_conv.h): sets the block count above which a scan takes
// the extra launch, returns the previous value.  Values < 1 only query.
extern "C" int64_t sp_debug_scan_self_base_max(int64_t blocks) {
    const int64_t old = sp::g_self_base_max_blocks;
    if (blocks >= 1) sp::g_self_base_max_blocks = blocks;
    return old;
}
