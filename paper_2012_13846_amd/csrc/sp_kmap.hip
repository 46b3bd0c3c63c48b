// Kernel maps (Sec. III-B step 2): for every kernel offset the (input row, output row) pairs it links,
// found by probing the input coordinate set's hash table, then compacted with wavefront ballots and
// prefix sums into (a) offset-major pair lists and (b) tile-major lists for the gather-GEMM kernels.
#include <algorithm>

#include "sp_hash.h"
#include "sp_internal.h"

namespace sp {
namespace {

constexpr int kThreads = kTileRows;  // one thread per row of a tile; 4 wavefronts = 4 sub-tiles

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* __restrict__ p, int64_t n, int32_t v) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// grid (tiles of n_out, K*K).  Thread (o, ax, ay) probes the K offsets (ax, ay, 0..K-1): the K searches of
// one thread are independent, so their memory latencies overlap, and the row's coordinates are read once.
// Writes nbr_out[k][o]; scatters nbr_in[k][i] = o when nbr_in is given; counts live links per 64-row
// half sub-tile (sub_counts[((tile*4 + wave)*kvol + k)*2 + half]) and per tile (blk_counts[k*ntiles + tile]).
// identity_k >= 0 (stride 1, odd K; input and output rows are the same set): the centre offset is the
// identity, and link (i, o) at offset k is link (o, i) at offset kvol-1-k, so only the offsets below the
// centre are searched and each hit is also written to the mirrored entry nbr_out[kvol-1-k][i] = o.  The
// entries above the centre that stay without a hit were set to -1 beforehand, and the counts come from a
// separate pass over the table (count_kernel): sub_counts is null here.
template <int K>
__global__ __launch_bounds__(kThreads) void probe_kernel(const int4* __restrict__ c_out, int64_t n_out,
                                                         const HashSlot* __restrict__ tab, uint32_t cap, int zshift, int step,
                                                         int identity_k, int32_t* __restrict__ nbr_out,
                                                         int32_t* __restrict__ nbr_in, int64_t n_in,
                                                         int32_t* __restrict__ sub_counts,
                                                         int32_t* __restrict__ blk_counts) {
    __shared__ int s_cnt[K][kSubTiles];
    constexpr int kvol = K * K * K;
    const int ay = blockIdx.y % K, ax = blockIdx.y / K;
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    constexpr int centre = (K & 1) ? (K - 1) / 2 : 0;
    const int k0 = (ax * K + ay) * K;
    int32_t v[K];
#pragma unroll
    for (int az = 0; az < K; ++az) v[az] = -1;
    if (o < n_out) {
        const int4 c = c_out[o];
        uint64_t key[K];
        bool ok[K];
#pragma unroll
        for (int az = 0; az < K; ++az)
            ok[az] = pack_key(c.x, c.y + (ax - centre) * step, c.z + (ay - centre) * step, c.w + (az - centre) * step,
                              &key[az]);
        // The K searches advance in lockstep: every turn issues the next slot's load of all searches still
        // running and only then looks at the answers, so their memory latencies overlap (run one after the
        // other, each search costs as many round trips as the longest probe sequence among the 64 lanes).
        uint32_t slot[K];
        bool run[K];
        bool any = false;
#pragma unroll
        for (int az = 0; az < K; ++az) {
            run[az] = false;
            slot[az] = 0;
            if (k0 + az == identity_k) {
                v[az] = (int32_t)o;
            } else if (ok[az] && (identity_k < 0 || k0 + az < identity_k)) {
                uint32_t bucket, pos;
                hash_home(key[az], cap, zshift, &bucket, &pos);
                slot[az] = bucket * 4 + pos;
                run[az] = true;
                any = true;
            }
        }
        for (uint32_t turn = 0; any && turn < cap; ++turn) {
            uint4 raw[K];
#pragma unroll
            for (int az = 0; az < K; ++az)
                if (run[az]) raw[az] = *reinterpret_cast<const uint4*>(&tab[slot[az]]);
            any = false;
#pragma unroll
            for (int az = 0; az < K; ++az) {
                if (!run[az]) continue;
                const unsigned long long cur = ((unsigned long long)raw[az].y << 32) | raw[az].x;
                if (cur == key[az]) {
                    v[az] = (int32_t)raw[az].w;
                    run[az] = false;
                } else if (cur == kEmptyKey) {
                    run[az] = false;
                } else {
                    slot[az] = (slot[az] + 1) & (cap - 1);
                    any = true;
                }
            }
        }
#pragma unroll
        for (int az = 0; az < K; ++az) {
            if (identity_k >= 0 && k0 + az > identity_k) continue;  // written by the mirrored offset's hits
            nbr_out[(int64_t)(k0 + az) * n_out + o] = v[az];
            if (nbr_in && v[az] >= 0) nbr_in[(int64_t)(k0 + az) * n_in + v[az]] = (int32_t)o;
            if (identity_k >= 0 && k0 + az < identity_k && v[az] >= 0)
                nbr_out[(int64_t)(kvol - 1 - (k0 + az)) * n_out + v[az]] = (int32_t)o;
        }
    }
    if (!sub_counts) return;  // uniform: the counts of a mirrored table are taken by count_kernel
    const int w = threadIdx.x >> 6;
#pragma unroll
    for (int az = 0; az < K; ++az) {
        const unsigned long long live = __ballot(v[az] >= 0);
        if ((threadIdx.x & 63) == 0) {
            const int lo = __popc((unsigned)live), hi = __popc((unsigned)(live >> 32));
            s_cnt[az][w] = lo + hi;
            int32_t* dst = sub_counts + (((int64_t)blockIdx.x * kSubTiles + w) * kvol + k0 + az) * kHalves;
            dst[0] = lo;
            dst[1] = hi;
        }
    }
    __syncthreads();
    if (threadIdx.x < K && blk_counts)
        blk_counts[(int64_t)(k0 + threadIdx.x) * gridDim.x + blockIdx.x] =
            s_cnt[threadIdx.x][0] + s_cnt[threadIdx.x][1] + s_cnt[threadIdx.x][2] + s_cnt[threadIdx.x][3];
}

// Same counting from an existing table (the scattered input-side table of a strided map).
__global__ __launch_bounds__(kThreads) void count_kernel(const int32_t* __restrict__ nbr, int64_t n_rows,
                                                         int32_t* __restrict__ sub_counts,
                                                         int32_t* __restrict__ blk_counts) {
    __shared__ int s_cnt[kSubTiles];
    const int k = blockIdx.y, kvol = gridDim.y;
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int32_t v = r < n_rows ? nbr[(int64_t)k * n_rows + r] : -1;
    const unsigned long long live = __ballot(v >= 0);
    if ((threadIdx.x & 63) == 0) {
        int32_t* dst = sub_counts + (((int64_t)blockIdx.x * kSubTiles + (threadIdx.x >> 6)) * kvol + k) * kHalves;
        dst[0] = __popc((unsigned)live);
        dst[1] = __popc((unsigned)(live >> 32));
        s_cnt[threadIdx.x >> 6] = __popcll(live);
    }
    if (!blk_counts) return;  // uniform
    __syncthreads();
    if (threadIdx.x == 0) blk_counts[(int64_t)k * gridDim.x + blockIdx.x] = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
}

// Compaction: every live (row, k) writes its entry at offset + (number of live lanes below it).
__global__ __launch_bounds__(kThreads) void emit_kernel(const int32_t* __restrict__ nbr, int64_t n_rows,
                                                        const int32_t* __restrict__ tl_off,
                                                        int32_t* __restrict__ tl_src, uint16_t* __restrict__ tl_row,
                                                        const int32_t* __restrict__ blk_off,
                                                        int32_t* __restrict__ pair_in, int32_t* __restrict__ pair_out) {
    __shared__ int s_cnt[kSubTiles];
    const int k = blockIdx.y, kvol = gridDim.y;
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int32_t v = r < n_rows ? nbr[(int64_t)k * n_rows + r] : -1;
    const unsigned long long live = __ballot(v >= 0);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int pos = __popcll(live & ((1ull << lane) - 1ull));  // among the wavefront's 64 rows
    if (v >= 0) {
        // the two 32-row halves of a sub-tile are adjacent in the list, so the position inside the sub-tile's
        // stretch is the plain 64-lane rank
        const int64_t e = (int64_t)tl_off[(((int64_t)blockIdx.x * kSubTiles + w) * kvol + k) * kHalves] + pos;
        tl_src[e] = v;
        tl_row[e] = (uint16_t)threadIdx.x;
    }
    if (pair_in) {  // uniform branch
        if (lane == 0) s_cnt[w] = __popcll(live);
        __syncthreads();
        int before = 0;
        for (int j = 0; j < w; ++j) before += s_cnt[j];
        if (v >= 0) {
            const int64_t p = (int64_t)blk_off[(int64_t)k * gridDim.x + blockIdx.x] + before + pos;
            pair_in[p] = v;
            pair_out[p] = (int32_t)r;
        }
    }
}

inline unsigned blocks256(int64_t n) { return (unsigned)((n + 255) / 256); }

// Position class of an input row inside its coarse cell: ((x/ts) mod s, (y/ts) mod s, (z/ts) mod s) as one number.
__device__ __forceinline__ int cell_class(const int4& c, int ts, int stride) {
    auto r = [&](int v) { const int q = v / ts % stride; return q < 0 ? q + stride : q; };  // coordinates are multiples of ts
    return (r(c.y) * stride + r(c.z)) * stride + r(c.w);
}

// Even kernel as wide as the stride (offsets 0 .. K-1 = the positions inside a coarse cell): every input row
// has exactly one link, to its own coarse cell (parent[i], from the coarse coordinates' merge), at the offset
// that is its position in the cell.  No searches.
__global__ __launch_bounds__(kThreads) void child_map_kernel(const int4* __restrict__ c_in, int64_t n_in, int ts,
                                                             int stride, const int32_t* __restrict__ parent,
                                                             int64_t n_out, int32_t* __restrict__ nbr_out,
                                                             int32_t* __restrict__ nbr_in) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n_in) return;
    const int k = cell_class(c_in[i], ts, stride);
    const int32_t o = parent[i];
    nbr_in[(int64_t)k * n_in + i] = o;
    nbr_out[(int64_t)k * n_out + o] = (int32_t)i;
}

// cnt[cls * ntiles + tile] = rows of the tile in class cls (tiles of 256 rows in row order)
__global__ __launch_bounds__(kThreads) void class_count_kernel(const int4* __restrict__ coords, int64_t n, int ts,
                                                               int stride, int nclass, int32_t* __restrict__ cnt) {
    __shared__ int s_cnt[32][kSubTiles];
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int cls = r < n ? cell_class(coords[r], ts, stride) : -1;
    const int w = threadIdx.x >> 6;
    for (int c = 0; c < nclass; ++c) {
        const unsigned long long m = __ballot(cls == c);
        if ((threadIdx.x & 63) == 0) s_cnt[c][w] = __popcll(m);
    }
    __syncthreads();
    if (threadIdx.x < nclass)
        cnt[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] =
            s_cnt[threadIdx.x][0] + s_cnt[threadIdx.x][1] + s_cnt[threadIdx.x][2] + s_cnt[threadIdx.x][3];
}

// perm[off[cls * ntiles + tile] + rank of the row among the tile's rows of its class] = row
__global__ __launch_bounds__(kThreads) void class_emit_kernel(const int4* __restrict__ coords, int64_t n, int ts,
                                                              int stride, int nclass, const int32_t* __restrict__ off,
                                                              int32_t* __restrict__ perm) {
    __shared__ int s_cnt[32][kSubTiles];
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int cls = r < n ? cell_class(coords[r], ts, stride) : -1;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int rank = 0;
    for (int c = 0; c < nclass; ++c) {
        const unsigned long long m = __ballot(cls == c);
        if (lane == 0) s_cnt[c][w] = __popcll(m);
        if (cls == c) rank = __popcll(m & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    if (cls >= 0) {
        for (int j = 0; j < w; ++j) rank += s_cnt[cls][j];
        perm[off[(int64_t)cls * gridDim.x + blockIdx.x] + rank] = (int32_t)r;
    }
}

// mask[tile][k / 32] bit k % 32 = offset k can link a row of one of the position classes present in
// perm[tile*256 .. +255].  Offset (ax, ay, az) links an input at class r to an output only if, per axis, the
// offset's displacement is congruent to r modulo the stride (output coordinates are multiples of the stride).
// One thread per tile; the classes' stretches of perm start at off[cls * ntiles].
__global__ __launch_bounds__(kThreads) void tile_mask_kernel(const int32_t* __restrict__ off, int64_t n, int64_t ntiles,
                                                             int K, int stride, uint32_t* __restrict__ mask) {
    __shared__ uint32_t s_cm[32][4];   // offsets possible for each class
    __shared__ int64_t s_beg[33];      // the classes' stretches of perm
    const int nclass = stride * stride * stride, centre = (K & 1) ? (K - 1) / 2 : 0;
    if (threadIdx.x < nclass) {
        const int c = threadIdx.x;
        const int r[3] = {c / (stride * stride), c / stride % stride, c % stride};
        uint32_t m[4] = {0u, 0u, 0u, 0u};
        for (int k = 0; k < K * K * K; ++k) {
            const int d[3] = {k / (K * K) - centre, k / K % K - centre, k % K - centre};
            bool ok = true;
            for (int ax = 0; ax < 3; ++ax) ok = ok && ((d[ax] % stride + stride) % stride == r[ax]);
            if (ok) m[k >> 5] |= 1u << (k & 31);
        }
        for (int i = 0; i < 4; ++i) s_cm[c][i] = m[i];
        s_beg[c] = off[(int64_t)c * ntiles];
        if (c == nclass - 1) s_beg[nclass] = n;
    }
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= ntiles) return;
    const int64_t lo = t * kTileRows, hi = lo + kTileRows < n ? lo + kTileRows : n;
    uint32_t m[4] = {0u, 0u, 0u, 0u};
    for (int c = 0; c < nclass; ++c)
        if (s_beg[c] < hi && s_beg[c + 1] > lo)
            for (int i = 0; i < 4; ++i) m[i] |= s_cm[c][i];
    for (int i = 0; i < 4; ++i) mask[t * 4 + i] = m[i];
}

// Rows of a strided map's input side sorted by position class, and the per-tile offset masks.
int build_classes(MapSide& side, const sp_coords* c, int stride, int K, hipStream_t s) {
    const int nclass = stride * stride * stride;
    const int64_t n = side.n_rows, ntiles = (n + kTileRows - 1) / kTileRows;
    if (nclass > 32 || n == 0) return SP_OK;  // larger strides: no class order, the kernels take all offsets
    Buf cnt = dev_alloc((size_t)(nclass * ntiles + 1) * 4, s);
    side.perm = dev_alloc((size_t)n * 4, s);
    side.tile_mask = dev_alloc((size_t)ntiles * 16, s);
    if (!cnt || !side.perm || !side.tile_mask) return SP_ERR_ALLOC;
    hipLaunchKernelGGL(class_count_kernel, dim3((unsigned)ntiles), dim3(kThreads), 0, s, ptr<int4>(c->coords), n, c->ts,
                       stride, nclass, ptr<int32_t>(cnt));
    ScanJob job;
    job.data = ptr<int32_t>(cnt);
    job.n = nclass * ntiles;
    SP_TRY(exclusive_scan_jobs(&job, 1, s));
    hipLaunchKernelGGL(class_emit_kernel, dim3((unsigned)ntiles), dim3(kThreads), 0, s, ptr<int4>(c->coords), n, c->ts,
                       stride, nclass, ptr<int32_t>(cnt), ptr<int32_t>(side.perm));
    hipLaunchKernelGGL(tile_mask_kernel, dim3(blocks256(ntiles)), dim3(kThreads), 0, s, ptr<int32_t>(cnt), n, ntiles, K,
                       stride, ptr<uint32_t>(side.tile_mask));
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// Generative transposed convolution.  Candidate (j, k) = input row j displaced by offset k times the output
// lattice step; rows (j*kvol + k) of cand, i.e. input row by input row, offsets in offset order.
__global__ __launch_bounds__(kThreads) void gen_candidates_kernel(const int4* __restrict__ c_in, int64_t n_in, int K,
                                                                  int step, int4* __restrict__ cand) {
    const int kvol = K * K * K;
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= n_in * kvol) return;
    const int64_t j = t / kvol;
    const int k = (int)(t % kvol);
    const int centre = (K & 1) ? (K - 1) / 2 : 0;
    int4 c = c_in[j];
    c.y += (k / (K * K) - centre) * step;
    c.z += (k / K % K - centre) * step;
    c.w += (k % K - centre) * step;
    cand[t] = c;
}

// where[j*kvol + k] = fine row of candidate (j, k).  As a stride-s convolution from the fine rows (inputs) to
// the coarse rows (outputs) every candidate is one link: nbr_out[k][j] = that fine row, nbr_in[k][fine] = j.
__global__ __launch_bounds__(kThreads) void gen_tables_kernel(const int32_t* __restrict__ where, int64_t n_coarse,
                                                              int64_t n_fine, int kvol, int32_t* __restrict__ nbr_out,
                                                              int32_t* __restrict__ nbr_in) {
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;   // = k * n_coarse + j: coalesced table writes
    if (t >= n_coarse * kvol) return;
    const int k = (int)(t / n_coarse);
    const int64_t j = t % n_coarse;
    const int32_t f = where[j * kvol + k];
    nbr_out[t] = f;
    nbr_in[(int64_t)k * n_fine + f] = (int32_t)j;
}

// Turns sub-tile counts (already in side.tl_off) into offsets and fills the tile lists.
// `total`: the number of links, or any upper bound of it (the lists are then allocated larger than needed).
int finish_side(MapSide& side, int kvol, int64_t total, const int32_t* d_blk_off, int32_t* d_pair_in,
                int32_t* d_pair_out, hipStream_t s) {
    const int64_t ntiles = (side.n_rows + kTileRows - 1) / kTileRows;
    side.tl_src = dev_alloc((size_t)(total ? total : 1) * 4, s);
    side.tl_row = dev_alloc((size_t)(total ? total : 1) * 2, s);
    if (!side.tl_src || !side.tl_row) return SP_ERR_ALLOC;
    if (ntiles > 0 && total > 0)
        hipLaunchKernelGGL(emit_kernel, dim3((unsigned)ntiles, kvol), dim3(kThreads), 0, s, ptr<int32_t>(side.nbr),
                           side.n_rows, ptr<int32_t>(side.tl_off), ptr<int32_t>(side.tl_src),
                           ptr<uint16_t>(side.tl_row), d_blk_off, d_pair_in, d_pair_out);
    SP_HIP(hipGetLastError());
    return SP_OK;
}


// Second half of a map build, shared by every way of filling the neighbour tables: on entry both tables are
// complete, so.tl_off holds the output side's link counts per (sub-tile, offset, half) and blk those per
// (offset, tile).  Scans them, reads the per-offset pair counts back, and compacts the tables into the pair
// lists and the tile lists of both sides (a symmetric map shares one table and one set of lists).
int finish_map(sp_kmap* m, bool symmetric, const Buf& blk, const Buf& small, hipStream_t s) {
    MapSide& so = m->out_side;
    MapSide& si = m->in_side;
    sp_coords* cin = m->c_in;
    const int kvol = m->kvol, stride = m->stride, kernel_size = m->K;
    const int64_t n_in = m->n_in, n_out = m->n_out;
    const int64_t nt_out = (n_out + kTileRows - 1) / kTileRows, nt_in = (n_in + kTileRows - 1) / kTileRows;
    int32_t* d_koff = ptr<int32_t>(small);
    // both scans in one launch pair: sub-tile-major list offsets, and offset-major pair-list offsets whose
    // values at the start of each offset (every nt_out-th element) are the per-offset prefix koff[]
    {
        const int64_t n_sub = nt_out * kvol * kSubTiles * kHalves;
        ScanJob jobs[2];
        jobs[0].data = ptr<int32_t>(so.tl_off);
        jobs[0].n = n_sub;
        jobs[0].total = ptr<int32_t>(so.tl_off) + n_sub;
        jobs[1].data = ptr<int32_t>(blk);
        jobs[1].n = nt_out * kvol;
        jobs[1].koff = d_koff;
        jobs[1].koff_stride = nt_out > 0 ? nt_out : 1;
        jobs[1].koff_n = kvol;
        SP_TRY(exclusive_scan_jobs(jobs, 2, s));
    }
    // The host needs the pair counts (for its own bookkeeping and the callers'), the device does not: unless
    // the lists would be huge, they are allocated for the most links there can be and the compaction is
    // enqueued behind the read-back, so the GPU does not idle while the host wakes up and launches.
    const int64_t most = std::min(n_out, n_in) * kvol;
    const bool early = most * 14 <= ((int64_t)512 << 20);
    int early_rc = SP_OK;
    auto emit_out_side = [&](int64_t total) {
        m->pair_in = dev_alloc((size_t)(total ? total : 1) * 4, s);
        m->pair_out = dev_alloc((size_t)(total ? total : 1) * 4, s);
        if (!m->pair_in || !m->pair_out) return (int)SP_ERR_ALLOC;
        return finish_side(so, kvol, total, ptr<int32_t>(blk), ptr<int32_t>(m->pair_in), ptr<int32_t>(m->pair_out), s);
    };
    // the input side of a map without the stride-1 symmetry: its own counts, list offsets, lists and classes
    auto emit_in_side = [&](int64_t total) {
        if (nt_in > 0)
            hipLaunchKernelGGL(count_kernel, dim3((unsigned)nt_in, kvol), dim3(kThreads), 0, s, ptr<int32_t>(si.nbr),
                               n_in, ptr<int32_t>(si.tl_off), (int32_t*)nullptr);
        const int64_t n_sub_in = nt_in * kvol * kSubTiles * kHalves;
        ScanJob job;
        job.data = ptr<int32_t>(si.tl_off);
        job.n = n_sub_in;
        job.total = ptr<int32_t>(si.tl_off) + n_sub_in;
        SP_TRY(exclusive_scan_jobs(&job, 1, s));
        SP_TRY(finish_side(si, kvol, total, nullptr, nullptr, nullptr, s));
        if (stride > 1) SP_TRY(build_classes(si, cin, stride, kernel_size, s));
        return (int)SP_OK;
    };
    std::vector<int32_t> h_koff(kvol + 1);
    SP_TRY(read_back(h_koff.data(), d_koff, (size_t)(kvol + 1) * 4, s, [&]() {
        if (!early) return;
        early_rc = emit_out_side(most);
        if (early_rc == SP_OK && !symmetric) early_rc = emit_in_side(most);
    }));
    SP_TRY(early_rc);
    m->koff.resize(kvol + 1);
    m->counts.resize(kvol);
    for (int k = 0; k <= kvol; ++k) m->koff[k] = h_koff[k];
    for (int k = 0; k < kvol; ++k) m->counts[k] = m->koff[k + 1] - m->koff[k];
    m->total = m->koff[kvol];
    m->d_koff = small;
    if (!early) SP_TRY(emit_out_side(m->total));
    if (symmetric) {
        si = so;  // same lists; the link (i, o) at offset k is the link (o, i) at offset kvol-1-k
        si.flip = true;
    } else if (!early) {
        SP_TRY(emit_in_side(m->total));
    }
    return SP_OK;
}

}  // namespace
}  // namespace sp

using namespace sp;

extern "C" {

int sp_kmap_build(const sp_coords_t* in, int32_t kernel_size, int32_t stride, int32_t dilation, void* stream,
                  sp_kmap_t** kmap, sp_coords_t** out_coords) {
    if (kmap) *kmap = nullptr;
    if (out_coords) *out_coords = nullptr;
    if (!in || !kmap) return fail(SP_ERR_INVALID_ARG, "coords handle or kmap out pointer is NULL");
    if (kernel_size < 1 || kernel_size > 5) return fail(SP_ERR_INVALID_ARG, "kernel_size %d not in 1..5", kernel_size);
    if (stride < 1 || dilation < 1) return fail(SP_ERR_INVALID_ARG, "stride and dilation must be >= 1");
    if (stride > 1 && dilation > 1) return fail(SP_ERR_UNSUPPORTED, "dilation > 1 together with stride > 1");
    if ((int64_t)in->ts * stride > 32768 || (int64_t)in->ts * dilation * kernel_size > 65536)
        return fail(SP_ERR_RANGE, "tensor stride * stride / dilation leaves the packable coordinate range");
    hipStream_t s = (hipStream_t)stream;
    const int kvol = kernel_size * kernel_size * kernel_size;
    if (in->n * (int64_t)kvol >= ((int64_t)1 << 31) - 4096)
        return fail(SP_ERR_INVALID_ARG, "n * kernel volume exceeds 32-bit list offsets");

    std::unique_ptr<sp_kmap, int (*)(sp_kmap*)> m(new sp_kmap, sp_kmap_destroy);
    m->K = kernel_size;
    m->kvol = kvol;
    m->stride = stride;
    m->dilation = dilation;
    sp_coords* cin = const_cast<sp_coords*>(in);
    cin->ref.fetch_add(1);
    m->c_in = cin;
    if (stride == 1) {
        cin->ref.fetch_add(1);
        m->c_out = cin;
    } else {
        sp_coords* co = nullptr;
        SP_TRY(coords_build_impl(ptr<int32_t>(in->coords), in->n, in->ts * stride, in->ts * stride, s, &co));
        m->c_out = co;
    }
    const int64_t n_in = in->n, n_out = m->c_out->n;
    m->n_in = n_in;
    m->n_out = n_out;
    const bool symmetric = (stride == 1) && (kernel_size & 1);
    const int64_t nt_out = (n_out + kTileRows - 1) / kTileRows, nt_in = (n_in + kTileRows - 1) / kTileRows;
    const int step = dilation * in->ts;

    MapSide& so = m->out_side;
    so.n_rows = n_out;
    so.n_src = n_in;
    so.nbr = dev_alloc((size_t)(n_out ? n_out : 1) * kvol * 4, s);
    so.tl_off = dev_alloc((size_t)(nt_out * kvol * kSubTiles * kHalves + 1) * 4, s);
    Buf blk = dev_alloc((size_t)(nt_out * kvol + 1) * 4, s);
    Buf small = dev_alloc((size_t)(kvol + 2) * 4, s);  // [0..kvol] koff, [kvol+1] scratch total
    if (!so.nbr || !so.tl_off || !blk || !small) return SP_ERR_ALLOC;
    MapSide& si = m->in_side;
    if (!symmetric) {
        si.n_rows = n_in;
        si.n_src = n_out;
        si.nbr = dev_alloc((size_t)(n_in ? n_in : 1) * kvol * 4, s);
        si.tl_off = dev_alloc((size_t)(nt_in * kvol * kSubTiles * kHalves + 1) * 4, s);
        if (!si.nbr || !si.tl_off) return SP_ERR_ALLOC;
        if (n_in > 0)
            hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks256(n_in * kvol)), dim3(256), 0, s, ptr<int32_t>(si.nbr),
                               n_in * kvol, -1);
    }
    const bool children = stride > 1 && kernel_size == stride && kernel_size % 2 == 0;
    if (nt_out > 0 && children) {
        hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks256(n_out * (int64_t)kvol)), dim3(256), 0, s, ptr<int32_t>(so.nbr),
                           n_out * (int64_t)kvol, -1);
        hipLaunchKernelGGL(child_map_kernel, dim3(blocks256(n_in)), dim3(kThreads), 0, s, ptr<int4>(in->coords), n_in,
                           in->ts, stride, ptr<int32_t>(m->c_out->inverse), n_out, ptr<int32_t>(so.nbr),
                           ptr<int32_t>(si.nbr));
        hipLaunchKernelGGL(count_kernel, dim3((unsigned)nt_out, kvol), dim3(kThreads), 0, s, ptr<int32_t>(so.nbr), n_out,
                           ptr<int32_t>(so.tl_off), ptr<int32_t>(blk));
    } else if (nt_out > 0) {
        const int identity_k = symmetric ? (kvol - 1) / 2 : -1;
        // mirrored table: only the (ax, ay) pairs that hold an offset up to the centre are launched, and the
        // entries above the centre start as "no link"
        const int pairs_xy = symmetric ? identity_k / kernel_size + 1 : kernel_size * kernel_size;
        const dim3 grid((unsigned)nt_out, (unsigned)pairs_xy);
        if (symmetric && kvol > 1)
            hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks256(n_out * (int64_t)(kvol - 1 - identity_k))), dim3(256), 0, s,
                               ptr<int32_t>(so.nbr) + (int64_t)(identity_k + 1) * n_out,
                               n_out * (int64_t)(kvol - 1 - identity_k), -1);
        int32_t* nbr_in_arg = symmetric ? (int32_t*)nullptr : ptr<int32_t>(si.nbr);
        int32_t* sub_arg = symmetric ? (int32_t*)nullptr : ptr<int32_t>(so.tl_off);
#define SP_LAUNCH_PROBE(KS)                                                                                     \
    hipLaunchKernelGGL(probe_kernel<KS>, grid, dim3(kThreads), 0, s, ptr<int4>(m->c_out->coords), n_out,          \
                       ptr<HashSlot>(in->tab.slots), in->tab.cap, in->tab.zshift, step, identity_k, ptr<int32_t>(so.nbr), nbr_in_arg, \
                       n_in, sub_arg, ptr<int32_t>(blk))
        switch (kernel_size) {
            case 1: SP_LAUNCH_PROBE(1); break;
            case 2: SP_LAUNCH_PROBE(2); break;
            case 3: SP_LAUNCH_PROBE(3); break;
            case 4: SP_LAUNCH_PROBE(4); break;
            default: SP_LAUNCH_PROBE(5); break;
        }
#undef SP_LAUNCH_PROBE
        if (symmetric)
            hipLaunchKernelGGL(count_kernel, dim3((unsigned)nt_out, kvol), dim3(kThreads), 0, s, ptr<int32_t>(so.nbr),
                               n_out, ptr<int32_t>(so.tl_off), ptr<int32_t>(blk));
    }
    SP_HIP(hipGetLastError());
    SP_TRY(finish_map(m.get(), symmetric, blk, small, s));
    if (out_coords) {
        m->c_out->ref.fetch_add(1);
        *out_coords = m->c_out;
    }
    *kmap = m.release();
    return SP_OK;
}

int sp_kmap_build_generative(const sp_coords_t* in, int32_t kernel_size, int32_t stride, void* stream, sp_kmap_t** kmap,
                             sp_coords_t** out_coords) {
    if (kmap) *kmap = nullptr;
    if (out_coords) *out_coords = nullptr;
    if (!in || !kmap) return fail(SP_ERR_INVALID_ARG, "coords handle or kmap out pointer is NULL");
    if (kernel_size < 1 || kernel_size > 5) return fail(SP_ERR_INVALID_ARG, "kernel_size %d not in 1..5", kernel_size);
    if (stride < 1) return fail(SP_ERR_INVALID_ARG, "stride must be >= 1");
    if (in->ts % stride != 0)
        return fail(SP_ERR_INVALID_ARG, "the tensor stride (%d) must be a multiple of the layer stride (%d)", in->ts, stride);
    hipStream_t s = (hipStream_t)stream;
    const int kvol = kernel_size * kernel_size * kernel_size;
    const int64_t n_coarse = in->n, n_cand = n_coarse * kvol;
    if (n_cand >= ((int64_t)1 << 30)) return fail(SP_ERR_INVALID_ARG, "n * kernel volume exceeds 2^30 candidates");
    const int ts_out = in->ts / stride;

    // candidates -> fine coordinates (first-occurrence order) and the candidate -> fine row table
    Buf cand = dev_alloc((size_t)(n_cand ? n_cand : 1) * 16, s);
    if (!cand) return SP_ERR_ALLOC;
    if (n_cand > 0)
        hipLaunchKernelGGL(gen_candidates_kernel, dim3(blocks256(n_cand)), dim3(kThreads), 0, s, ptr<int4>(in->coords),
                           n_coarse, kernel_size, ts_out, ptr<int4>(cand));
    SP_HIP(hipGetLastError());
    sp_coords* fine = nullptr;
    SP_TRY(coords_build_impl(ptr<int32_t>(cand), n_cand, 1, ts_out, s, &fine));

    // the stride-s convolution's map from the fine rows (inputs) to the coarse rows (outputs) ...
    std::unique_ptr<sp_kmap, int (*)(sp_kmap*)> m(new sp_kmap, sp_kmap_destroy);
    m->K = kernel_size;
    m->kvol = kvol;
    m->stride = stride;
    m->dilation = 1;
    m->c_in = fine;  // takes over the reference
    sp_coords* coarse = const_cast<sp_coords*>(in);
    coarse->ref.fetch_add(1);
    m->c_out = coarse;
    const int64_t n_fine = fine->n;
    m->n_in = n_fine;
    m->n_out = n_coarse;
    if (n_fine * (int64_t)kvol >= ((int64_t)1 << 31) - 4096)
        return fail(SP_ERR_INVALID_ARG, "n * kernel volume exceeds 32-bit list offsets");
    const int64_t nt_out = (n_coarse + kTileRows - 1) / kTileRows, nt_in = (n_fine + kTileRows - 1) / kTileRows;
    MapSide& so = m->out_side;
    MapSide& si = m->in_side;
    so.n_rows = n_coarse;
    so.n_src = n_fine;
    si.n_rows = n_fine;
    si.n_src = n_coarse;
    so.nbr = dev_alloc((size_t)(n_cand ? n_cand : 1) * 4, s);
    so.tl_off = dev_alloc((size_t)(nt_out * kvol * kSubTiles * kHalves + 1) * 4, s);
    si.nbr = dev_alloc((size_t)(n_fine ? n_fine : 1) * kvol * 4, s);
    si.tl_off = dev_alloc((size_t)(nt_in * kvol * kSubTiles * kHalves + 1) * 4, s);
    Buf blk = dev_alloc((size_t)(nt_out * kvol + 1) * 4, s);
    Buf small = dev_alloc((size_t)(kvol + 2) * 4, s);
    if (!so.nbr || !so.tl_off || !si.nbr || !si.tl_off || !blk || !small) return SP_ERR_ALLOC;
    if (n_cand > 0) {
        hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks256(n_fine * kvol)), dim3(256), 0, s, ptr<int32_t>(si.nbr),
                           n_fine * kvol, -1);
        hipLaunchKernelGGL(gen_tables_kernel, dim3(blocks256(n_cand)), dim3(kThreads), 0, s, ptr<int32_t>(fine->inverse),
                           n_coarse, n_fine, kvol, ptr<int32_t>(so.nbr), ptr<int32_t>(si.nbr));
        hipLaunchKernelGGL(count_kernel, dim3((unsigned)nt_out, kvol), dim3(kThreads), 0, s, ptr<int32_t>(so.nbr), n_coarse,
                           ptr<int32_t>(so.tl_off), ptr<int32_t>(blk));
    }
    SP_HIP(hipGetLastError());
    SP_TRY(finish_map(m.get(), false, blk, small, s));
    // ... handed out with the roles swapped: inputs = the given (coarse) rows, outputs = the created rows
    sp_kmap_t* t = nullptr;
    SP_TRY(sp_kmap_transpose(m.get(), &t));
    if (out_coords) {
        fine->ref.fetch_add(1);
        *out_coords = fine;
    }
    *kmap = t;
    return SP_OK;
}

int sp_kmap_transpose(const sp_kmap_t* f, sp_kmap_t** transposed) {
    if (transposed) *transposed = nullptr;
    if (!f || !transposed) return fail(SP_ERR_INVALID_ARG, "kmap handle or out pointer is NULL");
    sp_kmap* t = new sp_kmap;
    t->n_in = f->n_out;
    t->n_out = f->n_in;
    t->total = f->total;
    t->K = f->K;
    t->kvol = f->kvol;
    t->stride = f->stride;
    t->dilation = f->dilation;
    t->out_side = f->in_side;
    t->in_side = f->out_side;
    t->pair_in = f->pair_out;
    t->pair_out = f->pair_in;
    t->counts = f->counts;
    t->koff = f->koff;
    t->d_koff = f->d_koff;
    t->c_in = f->c_out;
    t->c_out = f->c_in;
    if (t->c_in) t->c_in->ref.fetch_add(1);
    if (t->c_out) t->c_out->ref.fetch_add(1);
    *transposed = t;
    return SP_OK;
}

int sp_kmap_info(const sp_kmap_t* m, int64_t* n_in, int64_t* n_out, int32_t* kvol, int64_t* total_pairs,
                 int64_t* h_counts) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (n_in) *n_in = m->n_in;
    if (n_out) *n_out = m->n_out;
    if (kvol) *kvol = m->kvol;
    if (total_pairs) *total_pairs = m->total;
    if (h_counts)
        for (int k = 0; k < m->kvol; ++k) h_counts[k] = m->counts[k];
    return SP_OK;
}

int sp_kmap_pairs(const sp_kmap_t* m, const int32_t** d_pair_in, const int32_t** d_pair_out) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (d_pair_in) *d_pair_in = ptr<int32_t>(m->pair_in);
    if (d_pair_out) *d_pair_out = ptr<int32_t>(m->pair_out);
    return SP_OK;
}

int sp_kmap_table(const sp_kmap_t* m, const int32_t** d_nbr_out, const int32_t** d_nbr_in, int32_t* out_reversed,
                  int32_t* in_reversed) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (d_nbr_out) *d_nbr_out = ptr<int32_t>(m->out_side.nbr);
    if (d_nbr_in) *d_nbr_in = ptr<int32_t>(m->in_side.nbr);
    if (out_reversed) *out_reversed = m->out_side.flip ? 1 : 0;
    if (in_reversed) *in_reversed = m->in_side.flip ? 1 : 0;
    return SP_OK;
}

int sp_kmap_destroy(sp_kmap_t* m) {
    if (!m) return SP_OK;
    sp_coords_destroy(m->c_in);
    sp_coords_destroy(m->c_out);
    delete m;
    return SP_OK;
}

}  // extern "C"
