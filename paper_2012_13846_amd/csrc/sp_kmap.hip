// Kernel maps (Sec. III-B step 2): for every kernel offset the (input row, output row) pairs it links,
// found by probing the input coordinate set's hash table, then compacted with wavefront ballots and
// prefix sums into (a) per-offset pair lists and (b) tile-major lists for the gather-GEMM kernels.
//
// No host round trip and no scan launches: the build is (1) one reset launch, (2) the searches, which fill the
// neighbour table(s), (3) per map side a count launch (links per 256-row tile and offset), a small prefix launch
// (one workgroup per offset scans its counts over the tiles) and an emit launch (every tile writes its stretch
// of the lists); the last tile delivers the per-offset totals
// to device memory and to a mail slot, which the host reads when it first asks (kmap_resolve).  Row counts that
// the host has not seen yet (the input set's N, the coarse set's N) are read from device memory by the kernels;
// grids and allocations use upper bounds.  (A single-pass count + look-back + emit kernel was measured slower:
// the look-back's device-coherent loads cost ~2 us a round trip and a tile near the end of a launch that starts
// all at once needs several of them per offset.)
#include <algorithm>

#include "sp_hash.h"
#include "sp_internal.h"

namespace sp {
namespace {

constexpr int kThreads = kTileRows;  // one thread per row of a tile; 4 wavefronts = 4 sub-tiles
constexpr int kMaxKvol = 125;

// A row count: the host's value, or (d != null) a count in device memory that the host has not seen yet.
struct Count {
    const int32_t* d;
    int64_t h;
};
__device__ __forceinline__ int64_t get(const Count& c) { return c.d ? (int64_t)*c.d : c.h; }

// table[k][r] <- -1 for k in [k_lo, kvol), r < n (n may live on the device); a second such region
struct NegRegion {
    int32_t* table;
    Count n;
    int k_lo, kvol;
};
__global__ __launch_bounds__(256) void reset_kernel(NegRegion a, NegRegion b) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (a.table) {
        const int64_t n = get(a.n);
        if (i < n * (a.kvol - a.k_lo)) a.table[(int64_t)a.k_lo * n + i] = -1;
    }
    if (b.table) {
        const int64_t n = get(b.n);
        if (i < n * (b.kvol - b.k_lo)) b.table[(int64_t)b.k_lo * n + i] = -1;
    }
}

// grid (tiles of n_out, K*K).  Thread (o, ax, ay) probes the K offsets (ax, ay, 0..K-1): the K searches of
// one thread are independent, so their memory latencies overlap, and the row's coordinates are read once.
// Writes nbr_out[k][o]; scatters nbr_in[k][i] = o when nbr_in is given.
// identity_k >= 0 (stride 1, odd K; input and output rows are the same set): the centre offset is the
// identity, and link (i, o) at offset k is link (o, i) at offset kvol-1-k, so only the offsets below the
// centre are searched and each hit is also written to the mirrored entry nbr_out[kvol-1-k][i] = o.  The
// entries above the centre that stay without a hit were set to -1 beforehand.
template <int K>
__global__ __launch_bounds__(kThreads) void probe_kernel(const int4* __restrict__ c_out, Count cn_out,
                                                         const HashSlot* __restrict__ tab, uint32_t cap, int zshift, int step,
                                                         int identity_k, int32_t* __restrict__ nbr_out,
                                                         int32_t* __restrict__ nbr_in, Count cn_in) {
    constexpr int kvol = K * K * K;
    const int64_t n_out = get(cn_out);
    const int ay = blockIdx.y % K, ax = blockIdx.y / K;
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (o >= n_out) return;
    const int64_t n_in = nbr_in ? get(cn_in) : 0;
    constexpr int centre = (K & 1) ? (K - 1) / 2 : 0;
    const int k0 = (ax * K + ay) * K;
    int32_t v[K];
#pragma unroll
    for (int az = 0; az < K; ++az) v[az] = -1;
    const int4 c = c_out[o];
    uint64_t key[K];
    bool ok[K];
#pragma unroll
    for (int az = 0; az < K; ++az)
        ok[az] = pack_key(c.x, c.y + (ax - centre) * step, c.z + (ay - centre) * step, c.w + (az - centre) * step, &key[az]);
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

// Position class of an input row inside its coarse cell: ((x/ts) mod s, (y/ts) mod s, (z/ts) mod s) as one number.
__device__ __forceinline__ int cell_class(const int4& c, int ts, int stride) {
    auto r = [&](int v) { const int q = v / ts % stride; return q < 0 ? q + stride : q; };  // coordinates are multiples of ts
    return (r(c.y) * stride + r(c.z)) * stride + r(c.w);
}

// Even kernel as wide as the stride (offsets 0 .. K-1 = the positions inside a coarse cell): every input row
// has exactly one link, to its own coarse cell (parent[i], from the coarse coordinates' merge), at the offset
// that is its position in the cell.  No searches.
__global__ __launch_bounds__(kThreads) void child_map_kernel(const int4* __restrict__ c_in, Count cn_in, int ts, int stride,
                                                             const int32_t* __restrict__ parent, Count cn_out,
                                                             int32_t* __restrict__ nbr_out, int32_t* __restrict__ nbr_in) {
    const int64_t n_in = get(cn_in), n_out = get(cn_out);
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n_in) return;
    const int k = cell_class(c_in[i], ts, stride);
    const int32_t o = parent[i];
    nbr_in[(int64_t)k * n_in + i] = o;
    nbr_out[(int64_t)k * n_out + o] = (int32_t)i;
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
                                                              Count cn_fine, int kvol, int32_t* __restrict__ nbr_out,
                                                              int32_t* __restrict__ nbr_in) {
    const int64_t n_fine = get(cn_fine);
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;   // = k * n_coarse + j: coalesced table writes
    if (t >= n_coarse * kvol) return;
    const int k = (int)(t / n_coarse);
    const int64_t j = t % n_coarse;
    const int32_t f = where[j * kvol + k];
    nbr_out[t] = f;
    nbr_in[(int64_t)k * n_fine + f] = (int32_t)j;
}

// ---------------------------------------------------------------------------------------------------------------
// One side of a map: neighbour table -> lists, in two launches.
//
// count_kernel: per tile (256 destination rows) the live entries per (sub-tile, offset, 32-row half) into cnt and
// the tile's links per offset into agg[tile][*].  On a strided map's input side the rows per position class ride
// along as extra sums (width = kvol + nclass).
// prefix_kernel: one workgroup per sum scans it over the tiles: excl[tile][*].
// emit_kernel: tile t writes
//   tl_off  list offsets of its 4 sub-tiles: index ((t*4 + sub)*kvol + k)*2 + half, sub-tile-major stretches
//   tl_src / tl_row  the tile lists (source row, destination row inside the tile), destination rows ascending
//   pair_in / pair_out (output side only)  offset k's pairs at k*pair_stride + (links of earlier tiles at k) + rank
//   cls_excl[t][*] (classes)  rows of each position class in earlier tiles, for class_emit_kernel
// The last tile writes koff (prefix of the per-offset totals) to device memory and the mail slot, and the class
// bases.
// ---------------------------------------------------------------------------------------------------------------
struct Sums {
    int32_t* agg;   // [tile][width]: the tile's own sums (count_kernel)
    int32_t* excl;  // [tile][width]: sums of all earlier tiles (prefix_kernel)
    int width;      // kvol (+ nclass)
};

struct CountArgs {
    const int32_t* nbr;
    Count n_rows;
    int kvol;
    int32_t* cnt;   // [tile][sub][k][half]
    Sums sums;
    const int4* coords;  // classes (input side of a strided map), else nclass = 0
    int ts, stride, nclass;
};

constexpr int kChunk = 9;  // offsets whose table entries a thread requests before it looks at any of them

// grid (tiles, chunks of kChunk offsets): a workgroup counts one chunk of offsets of one tile (one table entry per
// thread and offset, all requested before any is looked at); the chunk-0 workgroup also counts the classes.
__global__ __launch_bounds__(kThreads) void count_kernel(CountArgs a) {
    __shared__ int s_cnt[kSubTiles][kChunk][kHalves];
    __shared__ int s_cls[32][kSubTiles];
    const int kvol = a.kvol, width = a.sums.width;
    const int n_ent = kSubTiles * kvol * kHalves;
    const int64_t n = get(a.n_rows);
    const int64_t t = blockIdx.x;
    if (t * kTileRows >= n) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t r = t * kTileRows + tid;
    const int k0 = blockIdx.y * kChunk;
    int32_t v[kChunk];
#pragma unroll
    for (int j = 0; j < kChunk; ++j) v[j] = (r < n && k0 + j < kvol) ? a.nbr[(int64_t)(k0 + j) * n + r] : -1;
#pragma unroll
    for (int j = 0; j < kChunk; ++j) {
        const unsigned long long live = __ballot(v[j] >= 0);
        if (lane == 0) {
            s_cnt[w][j][0] = __popc((unsigned)live);
            s_cnt[w][j][1] = __popc((unsigned)(live >> 32));
        }
    }
    const bool classes = a.nclass && blockIdx.y == 0;
    if (classes) {
        const int cls = r < n ? cell_class(a.coords[r], a.ts, a.stride) : -1;
        for (int c = 0; c < a.nclass; ++c) {
            const unsigned long long m = __ballot(cls == c);
            if (lane == 0) s_cls[c][w] = __popcll(m);
        }
    }
    __syncthreads();
    if (tid < kSubTiles * kChunk * kHalves) {
        const int ww = tid / (kChunk * kHalves), j = tid / kHalves % kChunk, h = tid % kHalves;
        if (k0 + j < kvol) a.cnt[t * n_ent + (ww * kvol + k0 + j) * kHalves + h] = s_cnt[ww][j][h];
    }
    if (tid < kChunk && k0 + tid < kvol) {
        int sum = 0;
        for (int ww = 0; ww < kSubTiles; ++ww) sum += s_cnt[ww][tid][0] + s_cnt[ww][tid][1];
        a.sums.agg[t * width + k0 + tid] = sum;
    }
    if (classes && tid >= 64 && tid < 64 + a.nclass) {
        int sum = 0;
        for (int ww = 0; ww < kSubTiles; ++ww) sum += s_cls[tid - 64][ww];
        a.sums.agg[t * width + kvol + tid - 64] = sum;
    }
}

// Block i: excl[t][i] = sum of agg[t'][i] over t' < t, for all tiles (1024 tiles a round, running carry).
__global__ __launch_bounds__(1024) void prefix_kernel(Sums sm, Count n_rows) {
    __shared__ int s_wave[16];
    __shared__ int s_carry;
    const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t n = get(n_rows);
    const int64_t ntiles = (n + kTileRows - 1) / kTileRows;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int64_t t0 = 0; t0 < ntiles; t0 += 1024) {
        const int64_t t = t0 + tid;
        const int v = t < ntiles ? sm.agg[t * sm.width + i] : 0;
        int inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int u = __shfl_up(inc, d, 64);
            if (lane >= d) inc += u;
        }
        if (lane == 63) s_wave[w] = inc;
        __syncthreads();
        int before = s_carry;
        for (int ww = 0; ww < w; ++ww) before += s_wave[ww];
        if (t < ntiles) sm.excl[t * sm.width + i] = before + inc - v;
        __syncthreads();
        if (tid == 1023) s_carry = before + inc;
        __syncthreads();
    }
}

struct EmitArgs {
    const int32_t* nbr;
    Count n_rows;
    int kvol;
    const int32_t* cnt;  // count_kernel's counts (the workgroups that share a tile all read them: not tl_off itself)
    int32_t* tl_off;
    int32_t* tl_src;
    uint16_t* tl_row;
    int32_t* pair_in;   // null on the input side
    int32_t* pair_out;
    int64_t pair_stride;
    Sums sums;
    int nclass;
    int32_t* cls_excl;  // [tile][nclass]: rows of class c in earlier tiles
    int32_t* cls_base;  // [nclass + 1]: first position of class c in the class-sorted order (written by the last tile)
    // results
    int32_t* d_koff;    // [kvol + 1] (output side only)
    uint32_t* mail;     // null or the mail slot: n_in, n_out, error bits, koff[0..kvol]
    uint32_t mail_seq;
    Count n_in, n_out;  // for the mail
};

__global__ __launch_bounds__(kThreads) void emit_kernel(EmitArgs a) {
    __shared__ int s_cnt[kSubTiles * kMaxKvol * kHalves + 2];  // [sub][k][half]: counts, then list offsets
    __shared__ int s_own[kMaxKvol + 32], s_excl[kMaxKvol + 32];
    const int kvol = a.kvol, width = a.sums.width;
    const int64_t n = get(a.n_rows);
    const int64_t ntiles = (n + kTileRows - 1) / kTileRows;
    const int64_t t = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (t >= ntiles && !(t == 0 && ntiles == 0)) return;
    const bool empty = ntiles == 0;  // tile 0 of an empty side only delivers the (zero) results
    const int64_t r = t * kTileRows + tid;
    const int n_ent = kSubTiles * kvol * kHalves;

    // ---- this tile's counts, and the sums of everything before it
    if (!empty) {
        for (int e = tid; e < n_ent; e += kThreads) s_cnt[e] = a.cnt[t * n_ent + e];
        for (int i = tid; i < width; i += kThreads) {
            s_excl[i] = a.sums.excl[t * width + i];
            s_own[i] = a.sums.agg[t * width + i];
        }
    } else {
        for (int i = tid; i < width; i += kThreads) s_own[i] = s_excl[i] = 0;
    }
    __syncthreads();

    // ---- the last tile delivers the totals (gridDim.y workgroups share a tile: each emits a chunk of the offsets,
    // the first one also writes what belongs to the tile as a whole)
    const bool lead = blockIdx.y == 0;
    if (lead && t == (empty ? 0 : ntiles - 1) && tid == 0) {
        if (a.nclass) {
            int run = 0;
            for (int c = 0; c < a.nclass; ++c) {
                a.cls_base[c] = run;
                run += s_excl[kvol + c] + s_own[kvol + c];
            }
            a.cls_base[a.nclass] = run;
        }
        if (a.d_koff) {
            int run = 0;
            for (int k = 0; k < kvol; ++k) {
                a.d_koff[k] = run;
                if (a.mail) a.mail[3 + k] = (uint32_t)run;
                run += s_excl[k] + s_own[k];
            }
            a.d_koff[kvol] = run;
            if (a.mail) {
                a.mail[3 + kvol] = (uint32_t)run;
                a.mail[0] = (uint32_t)get(a.n_in);
                a.mail[1] = (uint32_t)get(a.n_out);
                a.mail[2] = 0u;
                __threadfence_system();
                __hip_atomic_store(a.mail + kMailSeqWord, a.mail_seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
    }
    if (empty) {
        if (lead && tid == 0) a.tl_off[0] = 0;
        return;
    }
    if (lead && a.nclass)
        for (int c = tid; c < a.nclass; c += kThreads) a.cls_excl[t * a.nclass + c] = s_excl[kvol + c];

    // ---- list offsets of the tile: links of all earlier tiles + exclusive scan over (sub, k, half).
    // Wavefront 0: lane l takes the entries [l*per, l*per + per).  s_cnt then holds offsets, with the end of the
    // tile's stretch in the entry after the last.
    if (w == 0) {
        int before = 0;
        for (int k = 0; k < kvol; ++k) before += s_excl[k];   // the same in every lane: links of all earlier tiles
        const int per = (n_ent + 63) / 64;
        int sum = 0;
        for (int j = 0; j < per; ++j) {
            const int e = lane * per + j;
            if (e < n_ent) sum += s_cnt[e];
        }
        int inc = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int u = __shfl_up(inc, d, 64);
            if (lane >= d) inc += u;
        }
        int run = before + inc - sum;
        for (int j = 0; j < per; ++j) {
            const int e = lane * per + j;
            if (e < n_ent) {
                const int c = s_cnt[e];
                s_cnt[e] = run;  // from here on: the entry's list offset
                if (lead) a.tl_off[t * n_ent + e] = run;
                run += c;
            }
        }
        if (lane == 63) {
            s_cnt[n_ent] = run;                                        // all lanes' entries precede: run = end of the tile
            if (lead && t == ntiles - 1) a.tl_off[ntiles * n_ent] = run;  // end of the last stretch = all links
        }
    }
    __syncthreads();

    // ---- emit: every live (row, k) writes its entry at offset + (number of live lanes below it)
    for (int k0 = blockIdx.y * kChunk; k0 < kvol; k0 += gridDim.y * kChunk) {
      int32_t vv[kChunk];
#pragma unroll
      for (int j = 0; j < kChunk; ++j) vv[j] = (r < n && k0 + j < kvol) ? a.nbr[(int64_t)(k0 + j) * n + r] : -1;
#pragma unroll
      for (int j = 0; j < kChunk; ++j) {
        const int k = k0 + j;
        const int32_t v = vv[j];
        const unsigned long long live = __ballot(v >= 0);
        const int pos = __popcll(live & ((1ull << lane) - 1ull));  // among the wavefront's 64 rows
        if (v >= 0) {
            // the two 32-row halves of a sub-tile are adjacent in the list, so the position inside the sub-tile's
            // stretch is the plain 64-lane rank
            const int64_t e = (int64_t)s_cnt[(w * kvol + k) * kHalves] + pos;
            a.tl_src[e] = v;
            a.tl_row[e] = (uint16_t)tid;
            if (a.pair_in) {
                // links of this tile at offset k in the sub-tiles before this one, from the sizes of their stretches
                int before = 0;
                for (int ww = 0; ww < w; ++ww)
                    before += s_cnt[(ww * kvol + k + 1) * kHalves] - s_cnt[(ww * kvol + k) * kHalves];
                const int64_t p = (int64_t)k * a.pair_stride + s_excl[k] + before + pos;
                a.pair_in[p] = v;
                a.pair_out[p] = (int32_t)r;
            }
        }
      }
    }
}

// Rows of a strided map's input side in position-class order, and per 256 entries of that order the offsets
// that can link them.  perm[cls_base[c] + (rows of class c in earlier tiles) + rank in the tile] = row.
// mask[tile][k / 32] bit k % 32 = offset k can link a row of one of the position classes present in
// perm[tile*256 .. +255]: offset (ax, ay, az) links an input at class r to an output only if, per axis, the
// offset's displacement is congruent to r modulo the stride (output coordinates are multiples of the stride).
__global__ __launch_bounds__(kThreads) void class_emit_kernel(const int4* __restrict__ coords, Count cn, int ts, int stride,
                                                              int nclass, int K, const int32_t* __restrict__ cls_excl,
                                                              const int32_t* __restrict__ cls_base,
                                                              int32_t* __restrict__ perm, uint32_t* __restrict__ mask) {
    __shared__ int s_cnt[32][kSubTiles];
    __shared__ uint32_t s_cm[32][4];  // offsets possible for each class
    const int64_t n = get(cn);
    const int64_t t = blockIdx.x;
    if (t * kTileRows >= n) return;
    const int64_t r = t * kTileRows + threadIdx.x;
    const int cls = r < n ? cell_class(coords[r], ts, stride) : -1;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int rank = 0;
    for (int c = 0; c < nclass; ++c) {
        const unsigned long long m = __ballot(cls == c);
        if (lane == 0) s_cnt[c][w] = __popcll(m);
        if (cls == c) rank = __popcll(m & ((1ull << lane) - 1ull));
    }
    const int centre = (K & 1) ? (K - 1) / 2 : 0;
    if ((int)threadIdx.x < nclass) {
        const int c = threadIdx.x;
        const int rr[3] = {c / (stride * stride), c / stride % stride, c % stride};
        uint32_t m[4] = {0u, 0u, 0u, 0u};
        for (int k = 0; k < K * K * K; ++k) {
            const int d[3] = {k / (K * K) - centre, k / K % K - centre, k % K - centre};
            bool ok = true;
            for (int ax = 0; ax < 3; ++ax) ok = ok && ((d[ax] % stride + stride) % stride == rr[ax]);
            if (ok) m[k >> 5] |= 1u << (k & 31);
        }
        for (int i = 0; i < 4; ++i) s_cm[c][i] = m[i];
    }
    __syncthreads();
    if (cls >= 0) {
        for (int j = 0; j < w; ++j) rank += s_cnt[cls][j];
        perm[cls_base[cls] + cls_excl[t * nclass + cls] + rank] = (int32_t)r;
    }
    if (threadIdx.x < 4) {  // the mask of tile t of the class-sorted order
        const int64_t lo = t * kTileRows, hi = lo + kTileRows < n ? lo + kTileRows : n;
        uint32_t m = 0u;
        for (int c = 0; c < nclass; ++c)
            if (cls_base[c] < hi && cls_base[c + 1] > lo) m |= s_cm[c][threadIdx.x];
        mask[t * 4 + threadIdx.x] = m;
    }
}

inline unsigned blocks256(int64_t n) { return (unsigned)((n + 255) / 256); }

// Everything a build needs besides the tables: the tile counts and sums of both sides, the class prefixes of a
// strided input side.
struct Work {
    Buf mem;
    int32_t *cnt_out = nullptr, *cnt_in = nullptr;
    Sums sums_out{}, sums_in{};
    int32_t *cls_excl = nullptr, *cls_base = nullptr;
};

int make_work(Work& wk, int64_t nt_out, int64_t nt_in, int kvol, int nclass, bool two_sides, hipStream_t s) {
    const int64_t no = nt_out ? nt_out : 1, ni = two_sides ? (nt_in ? nt_in : 1) : 0;
    const int w_out = kvol, w_in = kvol + nclass;
    const int64_t n_ent = (int64_t)kSubTiles * kvol * kHalves;
    const int64_t words = 2 * no * w_out + 2 * ni * w_in + ni * nclass + nclass + 2 + (no + ni) * n_ent;
    wk.mem = dev_alloc((size_t)words * 4, s);
    if (!wk.mem) return SP_ERR_ALLOC;
    int32_t* q = ptr<int32_t>(wk.mem);
    wk.sums_out = Sums{q, q + no * w_out, w_out};
    q += 2 * no * w_out;
    wk.sums_in = Sums{q, q + ni * w_in, w_in};
    q += 2 * ni * w_in;
    wk.cls_excl = q;
    wk.cls_base = q + ni * nclass;
    q += ni * nclass + nclass + 2;
    wk.cnt_out = q;
    wk.cnt_in = q + no * n_ent;
    return SP_OK;
}

// Second half of a map build, shared by every way of filling the neighbour tables: on entry both tables are
// complete (on the stream).  One launch per side turns them into lists; a strided input side also gets its
// position-class order.  n_in_ub / n_out_ub: upper bounds of the row counts, cn_in / cn_out: where the kernels
// find the true ones.
int finish_map(sp_kmap* m, bool symmetric, Work& wk, int64_t n_in_ub, int64_t n_out_ub, Count cn_in, Count cn_out,
               int nclass, hipStream_t s) {
    MapSide& so = m->out_side;
    MapSide& si = m->in_side;
    const int kvol = m->kvol;
    const int64_t nt_out = (n_out_ub + kTileRows - 1) / kTileRows, nt_in = (n_in_ub + kTileRows - 1) / kTileRows;
    const int64_t most = std::min(n_out_ub, n_in_ub) * kvol;  // links there can be
    m->pair_stride = std::min(n_out_ub, n_in_ub);
    m->pair_in = dev_alloc((size_t)(most ? most : 1) * 4, s);
    m->pair_out = dev_alloc((size_t)(most ? most : 1) * 4, s);
    m->d_koff = dev_alloc((size_t)(kvol + 1) * 4, s);
    so.tl_src = dev_alloc((size_t)(most ? most : 1) * 4, s);
    so.tl_row = dev_alloc((size_t)(most ? most : 1) * 2, s);
    if (!m->pair_in || !m->pair_out || !m->d_koff || !so.tl_src || !so.tl_row) return SP_ERR_ALLOC;
    const bool mailed = mail_acquire(&m->mail);
    EmitArgs a{};
    a.nbr = ptr<int32_t>(so.nbr);
    a.n_rows = cn_out;
    a.kvol = kvol;
    a.tl_off = ptr<int32_t>(so.tl_off);
    a.tl_src = ptr<int32_t>(so.tl_src);
    a.tl_row = ptr<uint16_t>(so.tl_row);
    a.pair_in = ptr<int32_t>(m->pair_in);
    a.pair_out = ptr<int32_t>(m->pair_out);
    a.pair_stride = m->pair_stride;
    a.cnt = wk.cnt_out;
    a.sums = wk.sums_out;
    a.d_koff = ptr<int32_t>(m->d_koff);
    a.mail = mailed ? m->mail.d : nullptr;
    a.mail_seq = m->mail.seq;
    a.n_in = cn_in;
    a.n_out = cn_out;
    {
        CountArgs c{};
        c.nbr = a.nbr;
        c.n_rows = cn_out;
        c.kvol = kvol;
        c.cnt = wk.cnt_out;
        c.sums = wk.sums_out;
        hipLaunchKernelGGL(count_kernel, dim3((unsigned)(nt_out ? nt_out : 1), (unsigned)((kvol + kChunk - 1) / kChunk)), dim3(kThreads), 0, s, c);
        hipLaunchKernelGGL(prefix_kernel, dim3((unsigned)c.sums.width), dim3(1024), 0, s, c.sums, cn_out);
    }
    const unsigned chunks = (unsigned)((kvol + kChunk - 1) / kChunk);
    hipLaunchKernelGGL(emit_kernel, dim3((unsigned)(nt_out ? nt_out : 1), chunks), dim3(kThreads), 0, s, a);
    m->mail.armed = mailed;
    m->mail.stream = s;
    if (symmetric) {
        si = so;  // same lists; the link (i, o) at offset k is the link (o, i) at offset kvol-1-k
        si.flip = true;
    } else {
        si.tl_src = dev_alloc((size_t)(most ? most : 1) * 4, s);
        si.tl_row = dev_alloc((size_t)(most ? most : 1) * 2, s);
        if (!si.tl_src || !si.tl_row) return SP_ERR_ALLOC;
        EmitArgs b{};
        b.nbr = ptr<int32_t>(si.nbr);
        b.n_rows = cn_in;
        b.kvol = kvol;
        b.tl_off = ptr<int32_t>(si.tl_off);
        b.tl_src = ptr<int32_t>(si.tl_src);
        b.tl_row = ptr<uint16_t>(si.tl_row);
        b.cnt = wk.cnt_in;
        b.sums = wk.sums_in;
        b.nclass = nclass;
        b.cls_excl = wk.cls_excl;
        b.cls_base = wk.cls_base;
        CountArgs c{};
        c.nbr = b.nbr;
        c.n_rows = cn_in;
        c.kvol = kvol;
        c.cnt = wk.cnt_in;
        c.sums = wk.sums_in;
        c.coords = ptr<int4>(m->c_in->coords);
        c.ts = m->c_in->ts;
        c.stride = m->stride;
        c.nclass = nclass;
        hipLaunchKernelGGL(count_kernel, dim3((unsigned)(nt_in ? nt_in : 1), chunks), dim3(kThreads), 0, s, c);
        hipLaunchKernelGGL(prefix_kernel, dim3((unsigned)c.sums.width), dim3(1024), 0, s, c.sums, cn_in);
        hipLaunchKernelGGL(emit_kernel, dim3((unsigned)(nt_in ? nt_in : 1), chunks), dim3(kThreads), 0, s, b);
        if (nclass && n_in_ub > 0) {
            si.perm = dev_alloc((size_t)n_in_ub * 4, s);
            si.tile_mask = dev_alloc((size_t)nt_in * 16, s);
            if (!si.perm || !si.tile_mask) return SP_ERR_ALLOC;
            hipLaunchKernelGGL(class_emit_kernel, dim3((unsigned)nt_in), dim3(kThreads), 0, s, ptr<int4>(m->c_in->coords), cn_in,
                               m->c_in->ts, m->stride, nclass, m->K, wk.cls_excl, wk.cls_base, ptr<int32_t>(si.perm),
                               ptr<uint32_t>(si.tile_mask));
        }
    }
    SP_HIP(hipGetLastError());
    if (!mailed) {  // no mail slot free: wait here
        std::vector<uint32_t> h(kvol + 1);
        SP_TRY(read_back(h.data(), ptr<int32_t>(m->d_koff), (size_t)(kvol + 1) * 4, s));
        SP_TRY(coords_resolve(m->c_in));
        SP_TRY(coords_resolve(m->c_out));
        m->set_sizes(m->c_in->n, m->c_out->n, h.data());
        m->status = SP_OK;
        m->resolved = true;
    }
    return SP_OK;
}

}  // namespace

int kmap_resolve(const sp_kmap_t* m) {
    std::lock_guard<std::mutex> lk(m->mu);
    if (!m->resolved) {
        SP_TRY(mail_wait(m->mail, m->stream));
        const uint32_t* h = m->mail.h;
        m->set_sizes((int64_t)h[0], (int64_t)h[1], h + 3);
        m->status = SP_OK;
        m->resolved = true;
        mail_release(&m->mail);
    }
    // an error found while the coordinate sets were built (a coordinate out of range) makes the map invalid too
    if (m->c_in) SP_TRY(coords_resolve(m->c_in));
    if (m->c_out && m->c_out != m->c_in) SP_TRY(coords_resolve(m->c_out));
    return SP_OK;
}

}  // namespace sp

// host copies of the sizes, once they have arrived: koff = kvol + 1 prefix values
void sp_kmap::set_sizes(int64_t ni, int64_t no, const uint32_t* koff_words) const {
    n_in = ni;
    n_out = no;
    koff.resize(kvol + 1);
    counts.resize(kvol);
    for (int k = 0; k <= kvol; ++k) koff[k] = koff_words[k];
    for (int k = 0; k < kvol; ++k) counts[k] = koff[k + 1] - koff[k];
    total = koff[kvol];
    out_side.n_rows = no;
    out_side.n_src = ni;
    in_side.n_rows = ni;
    in_side.n_src = no;
}

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
    // Sizes: the input set's row count may not have reached the host yet.  Then its source row count bounds it;
    // when that bound would make the tables and lists much larger than they can need to be (many duplicates in
    // a large input), waiting for the count is the cheaper choice.
    bool known;
    {
        std::lock_guard<std::mutex> lk(in->mu);
        known = in->resolved;
    }
    if (!known && in->n_raw * (int64_t)kvol * 18 > ((int64_t)1 << 30)) {
        SP_TRY(coords_resolve(in));
        known = true;
    }
    if (known) SP_TRY(coords_resolve(in));  // reports an error found while it was built
    const int64_t n_in_ub = known ? in->n : in->n_raw;
    if (n_in_ub * (int64_t)kvol >= ((int64_t)1 << 31) - 4096)
        return fail(SP_ERR_INVALID_ARG, "n * kernel volume exceeds 32-bit list offsets");
    const Count cn_in{known ? nullptr : ptr<int32_t>(in->meta) + kMetaN, known ? in->n : 0};

    std::unique_ptr<sp_kmap, int (*)(sp_kmap*)> m(new sp_kmap, sp_kmap_destroy);
    m->K = kernel_size;
    m->kvol = kvol;
    m->stride = stride;
    m->dilation = dilation;
    m->stream = s;
    sp_coords* cin = const_cast<sp_coords*>(in);
    cin->ref.fetch_add(1);
    m->c_in = cin;
    Count cn_out = cn_in;
    int64_t n_out_ub = n_in_ub;
    if (stride == 1) {
        cin->ref.fetch_add(1);
        m->c_out = cin;
    } else {
        sp_coords* co = nullptr;
        SP_TRY(coords_build_impl(ptr<int32_t>(in->coords), n_in_ub, cn_in.d, in->ts * stride, in->ts * stride, s, &co));
        cin->ref.fetch_add(1);
        co->src_of = cin;  // its inverse array has one entry per row of `in`
        m->c_out = co;
        cn_out = co->resolved ? Count{nullptr, co->n} : Count{ptr<int32_t>(co->meta) + kMetaN, 0};
        if (co->resolved) n_out_ub = co->n;
    }
    const bool symmetric = (stride == 1) && (kernel_size & 1);
    const int64_t nt_out = (n_out_ub + kTileRows - 1) / kTileRows, nt_in = (n_in_ub + kTileRows - 1) / kTileRows;
    const int step = dilation * in->ts;
    const int nclass = (stride > 1 && stride * stride * stride <= 32) ? stride * stride * stride : 0;

    MapSide& so = m->out_side;
    MapSide& si = m->in_side;
    so.nbr = dev_alloc((size_t)(n_out_ub ? n_out_ub : 1) * kvol * 4, s);
    so.tl_off = dev_alloc((size_t)(nt_out * kvol * kSubTiles * kHalves + 1) * 4, s);
    Work wk;
    SP_TRY(make_work(wk, nt_out, nt_in, kvol, nclass, !symmetric, s));
    if (!so.nbr || !so.tl_off) return SP_ERR_ALLOC;
    if (!symmetric) {
        si.nbr = dev_alloc((size_t)(n_in_ub ? n_in_ub : 1) * kvol * 4, s);
        si.tl_off = dev_alloc((size_t)(nt_in * kvol * kSubTiles * kHalves + 1) * 4, s);
        if (!si.nbr || !si.tl_off) return SP_ERR_ALLOC;
    }
    const bool children = stride > 1 && kernel_size == stride && kernel_size % 2 == 0;
    const int identity_k = symmetric ? (kvol - 1) / 2 : -1;
    // one reset launch: "no link" where the searches will not write, zeros in the bookkeeping words
    {
        NegRegion ra{nullptr, cn_out, 0, kvol}, rb{nullptr, cn_in, 0, kvol};
        int64_t cover = 0;
        if (symmetric && kvol > 1) {
            ra = NegRegion{ptr<int32_t>(so.nbr), cn_out, identity_k + 1, kvol};
            cover = std::max(cover, n_out_ub * (int64_t)(kvol - 1 - identity_k));
        }
        if (!symmetric) {
            rb = NegRegion{ptr<int32_t>(si.nbr), cn_in, 0, kvol};
            cover = std::max(cover, n_in_ub * (int64_t)kvol);
            if (children) {
                ra = NegRegion{ptr<int32_t>(so.nbr), cn_out, 0, kvol};
                cover = std::max(cover, n_out_ub * (int64_t)kvol);
            }
        }
        if (cover > 0) hipLaunchKernelGGL(reset_kernel, dim3(blocks256(cover)), dim3(256), 0, s, ra, rb);
    }
    if (nt_out > 0 && children) {
        hipLaunchKernelGGL(child_map_kernel, dim3(blocks256(n_in_ub)), dim3(kThreads), 0, s, ptr<int4>(in->coords), cn_in,
                           in->ts, stride, ptr<int32_t>(m->c_out->inverse), cn_out, ptr<int32_t>(so.nbr), ptr<int32_t>(si.nbr));
    } else if (nt_out > 0) {
        // mirrored table: only the (ax, ay) pairs that hold an offset up to the centre are launched
        const int pairs_xy = symmetric ? identity_k / kernel_size + 1 : kernel_size * kernel_size;
        const dim3 grid((unsigned)nt_out, (unsigned)pairs_xy);
        int32_t* nbr_in_arg = symmetric ? (int32_t*)nullptr : ptr<int32_t>(si.nbr);
#define SP_LAUNCH_PROBE(KS)                                                                                          \
    hipLaunchKernelGGL(probe_kernel<KS>, grid, dim3(kThreads), 0, s, ptr<int4>(m->c_out->coords), cn_out,              \
                       ptr<HashSlot>(in->tab.slots), in->tab.cap, in->tab.zshift, step, identity_k, ptr<int32_t>(so.nbr), \
                       nbr_in_arg, cn_in)
        switch (kernel_size) {
            case 1: SP_LAUNCH_PROBE(1); break;
            case 2: SP_LAUNCH_PROBE(2); break;
            case 3: SP_LAUNCH_PROBE(3); break;
            case 4: SP_LAUNCH_PROBE(4); break;
            default: SP_LAUNCH_PROBE(5); break;
        }
#undef SP_LAUNCH_PROBE
    }
    SP_HIP(hipGetLastError());
    SP_TRY(finish_map(m.get(), symmetric, wk, n_in_ub, n_out_ub, cn_in, cn_out, nclass, s));
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
    SP_TRY(coords_resolve(in));  // the candidate count sizes everything
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
    SP_TRY(coords_build_impl(ptr<int32_t>(cand), n_cand, nullptr, 1, ts_out, s, &fine));

    // the stride-s convolution's map from the fine rows (inputs) to the coarse rows (outputs) ...
    std::unique_ptr<sp_kmap, int (*)(sp_kmap*)> m(new sp_kmap, sp_kmap_destroy);
    m->K = kernel_size;
    m->kvol = kvol;
    m->stride = stride;
    m->dilation = 1;
    m->stream = s;
    m->c_in = fine;  // takes over the reference
    sp_coords* coarse = const_cast<sp_coords*>(in);
    coarse->ref.fetch_add(1);
    m->c_out = coarse;
    SP_TRY(coords_resolve(fine));  // the created rows' count: the lists are sized from it, not from the candidates
    const int64_t n_fine = fine->n;
    const Count cn_fine{nullptr, n_fine}, cn_coarse{nullptr, n_coarse};
    if (n_fine * (int64_t)kvol >= ((int64_t)1 << 31) - 4096)
        return fail(SP_ERR_INVALID_ARG, "n * kernel volume exceeds 32-bit list offsets");
    const int64_t nt_out = (n_coarse + kTileRows - 1) / kTileRows, nt_in = (n_fine + kTileRows - 1) / kTileRows;
    const int nclass = (stride > 1 && stride * stride * stride <= 32) ? stride * stride * stride : 0;
    MapSide& so = m->out_side;
    MapSide& si = m->in_side;
    so.nbr = dev_alloc((size_t)(n_cand ? n_cand : 1) * 4, s);
    so.tl_off = dev_alloc((size_t)(nt_out * kvol * kSubTiles * kHalves + 1) * 4, s);
    si.nbr = dev_alloc((size_t)(n_fine ? n_fine : 1) * kvol * 4, s);
    si.tl_off = dev_alloc((size_t)(nt_in * kvol * kSubTiles * kHalves + 1) * 4, s);
    Work wk;
    SP_TRY(make_work(wk, nt_out, nt_in, kvol, nclass, true, s));
    if (!so.nbr || !so.tl_off || !si.nbr || !si.tl_off) return SP_ERR_ALLOC;
    {
        NegRegion ra{nullptr, cn_coarse, 0, kvol}, rb{ptr<int32_t>(si.nbr), cn_fine, 0, kvol};
        const int64_t cover = n_fine * (int64_t)kvol;
        if (cover > 0) hipLaunchKernelGGL(reset_kernel, dim3(blocks256(cover)), dim3(256), 0, s, ra, rb);
    }
    if (n_cand > 0)
        hipLaunchKernelGGL(gen_tables_kernel, dim3(blocks256(n_cand)), dim3(kThreads), 0, s, ptr<int32_t>(fine->inverse),
                           n_coarse, cn_fine, kvol, ptr<int32_t>(so.nbr), ptr<int32_t>(si.nbr));
    SP_HIP(hipGetLastError());
    SP_TRY(finish_map(m.get(), false, wk, n_fine, n_coarse, cn_fine, cn_coarse, nclass, s));
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
    SP_TRY(kmap_resolve(f));
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
    t->pair_stride = f->pair_stride;
    t->counts = f->counts;
    t->koff = f->koff;
    t->d_koff = f->d_koff;
    t->c_in = f->c_out;
    t->c_out = f->c_in;
    t->stream = f->stream;
    t->resolved = true;
    t->status = SP_OK;
    if (t->c_in) t->c_in->ref.fetch_add(1);
    if (t->c_out) t->c_out->ref.fetch_add(1);
    *transposed = t;
    return SP_OK;
}

int sp_kmap_info(const sp_kmap_t* m, int64_t* n_in, int64_t* n_out, int32_t* kvol, int64_t* total_pairs,
                 int64_t* h_counts) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (kvol) *kvol = m->kvol;
    if (n_in || n_out || total_pairs || h_counts) SP_TRY(kmap_resolve(m));
    if (n_in) *n_in = m->n_in;
    if (n_out) *n_out = m->n_out;
    if (total_pairs) *total_pairs = m->total;
    if (h_counts)
        for (int k = 0; k < m->kvol; ++k) h_counts[k] = m->counts[k];
    return SP_OK;
}

int sp_kmap_pairs(const sp_kmap_t* m, const int32_t** d_pair_in, const int32_t** d_pair_out, int64_t* pair_stride) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    if (d_pair_in) *d_pair_in = ptr<int32_t>(m->pair_in);
    if (d_pair_out) *d_pair_out = ptr<int32_t>(m->pair_out);
    if (pair_stride) *pair_stride = m->pair_stride;
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
