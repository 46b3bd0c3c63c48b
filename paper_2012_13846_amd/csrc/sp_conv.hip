// Step 3 of the generalized sparse convolution (Eq. 2) and its input gradient, as one gather-GEMM kernel.
//
// One workgroup owns a tile of destination rows (output rows for the forward pass, input rows for the data
// gradient) and a slice of destination channels.  It keeps the tile's fp32 accumulator in LDS.  For every
// kernel offset it takes the tile's compacted link list (source row, destination row), gathers the source
// feature rows into LDS, multiplies 16-link blocks with the offset's weight matrix on the matrix cores and
// adds each result row into the accumulator row of its destination.  A destination row belongs to exactly
// one workgroup and appears at most once per offset, so nothing is atomic and the summation order is
// fixed (results are reproducible run to run).  The accumulator is written once, rounded once.
#include <mutex>
#include <type_traits>

#include "sp_internal.h"

namespace sp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
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
    int lds_per_wave;  // bytes of LDS of one wavefront in gather_wave_kernel
    int split_blocks;  // sub-tiles with at least this many 16-link blocks are shared by two wavefronts
    uint32_t f_bytes, w_bytes, src_bytes, row_bytes;  // sizes of f / w / tl_src / tl_row for buffer addressing (< 4 GiB)
    int wave_ok;       // host-side only: buffers small enough for 32-bit buffer addressing
    int w_transposed;  // host-side only: the stored weights are [k][cc][co] (data gradient) instead of [k][co][cc]
    void* scratch;     // host-side only: if set, device memory for the weight copy instead of a pool allocation
    size_t scratch_bytes;
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
    static constexpr int kRowBytes = CC * kElt + 32; // staged row + 32 B pad (measured: b128 fragment reads then run at the full LDS rate)
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
    const int q0 = (blockIdx.x % kPerTile) * (TR / 64);  // first 64-row sub-tile inside the 256-row tile
    constexpr int kNQ = TR / 64;
    const int co0 = blockIdx.y * COT;

    for (int i = tid; i < TR * Cfg::kAccStride; i += 256) acc[i] = 0.f;

    const T* __restrict__ F = static_cast<const T*>(a.f);
    const T* __restrict__ W = static_cast<const T*>(a.w);

    const int64_t wt0 = (int64_t)blockIdx.x * kNQ;       // first 64-row sub-tile of this workgroup
    for (int kk = 0; kk < a.kvol; ++kk) {
        // the lists are sub-tile-major: this workgroup's links of offset kk are kNQ separate segments
        int sb[kNQ], sl[kNQ], mtot = 0;
#pragma unroll
        for (int q = 0; q < kNQ; ++q) {
            sb[q] = a.tl_off[((wt0 + q) * a.kvol + kk) * kHalves];
            sl[q] = a.tl_off[((wt0 + q) * a.kvol + kk + 1) * kHalves] - sb[q];
            mtot += sl[q];
        }
        if (mtot == 0) continue;
        auto entry = [&](int p) {
            int q = 0;
#pragma unroll
            for (int j = 0; j < kNQ - 1; ++j)
                if (q == j && p >= sl[j]) { p -= sl[j]; ++q; }
            return sb[q] + p;
        };
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
        for (int c0 = 0; c0 < mtot; c0 += Cfg::kChunk) {
            const int m = min(Cfg::kChunk, mtot - c0);
            __syncthreads();  // everyone is done with the previous staging buffer and its accumulator updates
            for (int idx = tid; idx < m * Cfg::kPiecesPerRow; idx += 256) {
                const int p = idx / Cfg::kPiecesPerRow, piece = idx % Cfg::kPiecesPerRow;
                const int32_t src = a.tl_src[entry(c0 + p)];
                const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(F) +
                                                                ((size_t)src * CC * Cfg::kElt + piece * 16));
                *reinterpret_cast<uint4*>(abuf + (size_t)p * Cfg::kRowBytes + piece * 16) = v;
            }
            if (tid < m) s_row[tid] = (uint16_t)(a.tl_row[entry(c0 + tid)] - q0 * 64);
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

// ---------------------------------------------------------------------------------------------------------
// Narrow-channel variant: every wavefront owns 64 destination rows (one sub-tile) and all COT channels of a
// channel tile, and runs on its own: no workgroup barrier anywhere.  Its links of all offsets are one
// contiguous stretch of the sub-tile-major lists.
//
//  - The wavefront first cuts its links into blocks of up to 16 links of one offset and writes one packed
//    descriptor per block into LDS, so that block b+n is addressable without walking a cursor.
//  - Everything a block needs is requested well ahead of its use and kept in registers: link entries
//    (source row, destination row) 2*kDX = 6 blocks ahead, the gathered source rows kDX = 3 blocks ahead, the
//    weight matrix two blocks ahead (a matrix too large for two register copies: in halves, half a block ahead).
//  - Source rows are gathered with coalesced 16-byte loads (adjacent lanes = adjacent pieces of one row; a
//    fragment-shaped global load would cost one L1 tag lookup per lane) and pass through a small
//    wavefront-private LDS buffer to be re-read as MFMA fragments, one block ahead of the MFMAs using them.
//  - The offset's weight matrix is the MFMA A operand (rows = destination channels), read from a
//    fragment-major copy of the weights so that one wavefront load is 1 KB of consecutive bytes.  (In the
//    stored layout a lane's 16-byte piece is contiguous too, so the forward pass could skip the copy, but a
//    wavefront's load is then 16 stretches of 64 bytes: measured 81 us against 61 with the copy.)
//  - The gathered rows are the B operand (columns = links), so the product comes out transposed: a lane
//    holds 4 consecutive channels of ONE link and adds them with one 16-byte LDS read-modify-write to that
//    link's destination row in the wavefront's private fp32 accumulator.
// ---------------------------------------------------------------------------------------------------------
template <typename T, int CC, int COT>
struct WaveCfg {
    static constexpr bool kIsF32 = std::is_same<T, float>::value;
    static constexpr int kGroup = kIsF32 ? 16 : 32;       // contraction channels per 16-byte fragment group
    static constexpr int kGroups = CC / kGroup;
    static constexpr int kNCT = COT / 16;
    static constexpr int kStride = COT + 4;               // floats per accumulator row
    static constexpr int kAccBytes = 64 * kStride * 4;
    static constexpr int kRowBytes = CC * (int)sizeof(T); // one source row
    static constexpr int kPieces = kRowBytes / 16;        // 16-byte pieces per source row
    static constexpr int kXStride = kRowBytes + 32;       // staged row + pad (b128 fragment reads at the full LDS rate)
    static constexpr int kXBytes = 16 * kXStride;
    static constexpr int kXLoads = (16 * kPieces + 63) / 64;  // coalesced load instructions per 16-link block
    static int per_wave_bytes(int kvol) { return kAccBytes + kXBytes + ((kvol * 4 + 3) / 4) * 16; }
    // fragment-major weights: [kvol][co_total/COT][kNCT][kGroups][64 lanes][16 bytes]
    static constexpr size_t kWFragBytesPerOffsetTile = (size_t)kNCT * kGroups * 64 * 16;
};

__device__ __forceinline__ void wave_sync() {
    // LDS traffic of one wavefront is processed in order; this only stops the compiler from moving
    // the wavefront's own LDS accesses across the point.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <typename T, int CC, int COT>
__global__ __launch_bounds__(64) void gather_wave_kernel(GatherArgs a) {
    using Cfg = WaveCfg<T, CC, COT>;
    constexpr bool kIsF32 = Cfg::kIsF32;
    constexpr int kGroups = Cfg::kGroups, kNCT = Cfg::kNCT, kPieces = Cfg::kPieces, kXLoads = Cfg::kXLoads;
    using Frag = typename std::conditional<kIsF32, f32x4, bf16x8>::type;  // 16 bytes
    static_assert(CC % Cfg::kGroup == 0, "contraction channels must fill whole fragment groups");
    static_assert(kPieces % 4 == 0, "a source row must be a multiple of 64 bytes");
    // Blocks whose gathers are in flight, and blocks whose weights are.  A gather is two dependent trips to
    // memory behind the entry loads and mostly misses the L2; the weights are one trip that mostly hits.  Rows
    // cost few registers per block and weights many, so narrow rows are fetched deep and weights shallow.
    constexpr int kDX = 3;  // loads return in order: a deeper ring for the rows alone would still wait for the weights issued after it
    constexpr int kDW = 2;
    // A weight matrix of more than 32 fragment registers (e.g. fp32 64 x 64) does not fit a ring of two whole
    // matrices.  Then the two weight slots hold the two halves (channel tiles 0..kNCT/2-1 and the rest) of ONE
    // block's matrix: a half is re-requested for the next block as soon as this block's MFMAs on it are issued,
    // i.e. half a block ahead of its next use, which is enough for a matrix that lives in L2.
    constexpr bool kHalfW = kNCT * kGroups > 8;
    constexpr int kWT = kHalfW ? kNCT / 2 : kNCT;  // channel tiles per weight slot
    static_assert(!kHalfW || kNCT % 2 == 0, "halves");
    constexpr int kTurn = 6;  // bodies per loop turn: a multiple of kDX, kDW and the two result sets
    static_assert(kTurn % kDX == 0 && kTurn % kDW == 0 && kTurn % 2 == 0, "ring sizes must divide the turn");

    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    // grid.x = 2 * sub-tiles: the first half of the grid takes half 0 (or the whole sub-tile), the second half
    // of the grid half 1.  (Workgroups are dealt to the 8 XCDs round-robin: pairing (u,0),(u,1) on adjacent
    // indices would leave every other XCD with nothing but wavefronts that leave at once.)
    const int64_t nwt = (a.n_rows + 63) / 64;
    const int half = blockIdx.x >= nwt ? 1 : 0;     // which 32-row half it takes if the sub-tile is split
    const int64_t wt = (int64_t)blockIdx.x - (half ? nwt : 0);  // this wavefront's sub-tile
    unsigned char* base = smem;
    float* acc = reinterpret_cast<float*>(base);
    unsigned char* xbuf = base + Cfg::kAccBytes;
    int* s_blk = reinterpret_cast<int*>(xbuf + Cfg::kXBytes);
    const int n16 = lane & 15, g = lane >> 4;
    const int kvol = a.kvol;

    for (int i = lane; i < Cfg::kAccBytes / 16; i += 64) reinterpret_cast<f32x4*>(acc)[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- block descriptors: k | (links-1) << 7 | (blocks left in this offset - 1) << 11 | (first link - off0) << 13
    // Two wavefronts are launched per sub-tile.  When the launch is small (a.split_blocks set by the host)
    // and the sub-tile is long, each takes one 32-row half, which halves the longest dependent chain of the
    // launch; otherwise the first takes all 64 rows and the second leaves.
    const int32_t* __restrict__ offp = a.tl_off + wt * kvol * kHalves;
    const int off0 = offp[0];
    int nblk_whole = 0;
    for (int kb = 0; kb < kvol; kb += 64) {
        const int k = kb + lane;
        int nb = k < kvol ? (offp[(k + 1) * kHalves] - offp[k * kHalves] + 15) >> 4 : 0;
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) nb += __shfl_xor(nb, d, 64);
        nblk_whole += nb;
    }
    const bool split = nblk_whole >= a.split_blocks;
    if (!split && half == 1) return;
    const int row_base = split ? 32 * half : 0;
    const int row_count = split ? 32 : 64;
    int nblk = 0;
    for (int kb = 0; kb < kvol; kb += 64) {
        const int k = kb + lane;
        int o0 = 0, o1 = 0;
        if (k < kvol) {
            o0 = offp[k * kHalves + (split ? half : 0)];
            o1 = offp[k * kHalves + (split ? half + 1 : kHalves)];
        }
        const int cnt = o1 - o0, nb = (cnt + 15) >> 4;
        int inc = nb;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(inc, d, 64);
            if (lane >= d) inc += t;
        }
        const int ex = nblk + inc - nb;
        for (int i = 0; i < nb; ++i)
            s_blk[ex + i] = k | ((min(16, cnt - 16 * i) - 1) << 7) | ((nb - i - 1) << 11) | ((o0 - off0 + 16 * i) << 13);
        nblk += __shfl(inc, 63, 64);
    }
    wave_sync();

    // Buffer addressing: a 32-bit byte offset per lane against a descriptor in scalar registers costs one
    // integer multiply-add per load instead of 64-bit pointer arithmetic, and reads past the end return 0.
    constexpr int kRsrcFlags = 0x00020000;
    const __amdgpu_buffer_rsrc_t rF = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.f), 0, (int)a.f_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.w), 0, (int)a.w_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rSrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(a.tl_src), 0, (int)a.src_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rRow =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.tl_row), 0, (int)a.row_bytes, kRsrcFlags);
    const uint32_t w_tile_off = (uint32_t)(blockIdx.y * Cfg::kWFragBytesPerOffsetTile);
    const uint32_t w_offset_stride = (uint32_t)((a.co_total / COT) * Cfg::kWFragBytesPerOffsetTile);

    auto load_weights = [&](int k, Frag (&wf)[kWT][kGroups], int ct0) __attribute__((always_inline)) {
        const int wk = a.flip ? kvol - 1 - k : k;
        // the offset index is the same in every lane, but it came through LDS: tell the compiler
        const int soff = __builtin_amdgcn_readfirstlane((int)(w_tile_off + (uint32_t)wk * w_offset_stride));
#pragma unroll
        for (int ct = 0; ct < kWT; ++ct)
#pragma unroll
            for (int s = 0; s < kGroups; ++s)
                wf[ct][s] = __builtin_bit_cast(
                    Frag, __builtin_amdgcn_raw_buffer_load_b128(rW, lane * 16 + ((ct0 + ct) * kGroups + s) * 1024, soff, 0));
    };

    // The main loop is straight-line code with the same loads in every turn (blocks past the end are
    // clamped to the last one and their results dropped): the compiler can then count outstanding loads
    // exactly and wait only for the oldest, instead of draining the whole prefetch queue at every branch.
    struct Slot {
        int dc;                   // descriptor of the block whose gathered rows are in x
        int drow;                 // destination row of that block's link n16
        int de;                   // descriptor of the block whose entries are in esrc / erow
        int esrc[kXLoads];        // source row of the link this lane gathers a piece of, per load
        int erow;                 // destination row of link n16
        u32x4 x[kXLoads];         // gathered pieces, coalesced layout: piece (t*64 + lane) of the block
    };
    struct WSlot {
        Frag w[kWT][kGroups];     // a block's weight matrix (kHalfW: one half of it)
    };
    const int last = nblk - 1;
    // (Starting each wavefront at a block of its own, so that the wavefronts of a compute unit do not ask for
    // the same weight lines at the same moment, was measured and is slower: in step, they share the lines in L1.)
    auto load_entries = [&](Slot& sl, int b) __attribute__((always_inline)) {
        sl.de = s_blk[min(b, last)];
        const int cnt = ((sl.de >> 7) & 15) + 1, e0 = off0 + (sl.de >> 13);
#pragma unroll
        for (int t = 0; t < kXLoads; ++t)
            sl.esrc[t] = (int)__builtin_amdgcn_raw_buffer_load_b32(rSrc, (e0 + min((t * 64 + lane) / kPieces, cnt - 1)) * 4, 0, 0);
        sl.erow = (int)__builtin_amdgcn_raw_buffer_load_b16(rRow, (e0 + min(n16, cnt - 1)) * 2, 0, 0);
    };
    auto issue_gather = [&](Slot& sl) __attribute__((always_inline)) {
        sl.dc = sl.de;
        sl.drow = (sl.erow & 63) - row_base;
#pragma unroll
        for (int t = 0; t < kXLoads; ++t)
            sl.x[t] = __builtin_amdgcn_raw_buffer_load_b128(rF, sl.esrc[t] * Cfg::kRowBytes + ((t * 64 + lane) % kPieces) * 16, 0, 0);
    };
    auto issue_weights = [&](WSlot& ws, int b, int ct0 = 0) __attribute__((always_inline)) {
        load_weights(s_blk[min(b, last)] & 127, ws.w, ct0);
    };
    auto stage = [&](const Slot& sl) __attribute__((always_inline)) {  // gathered rows -> LDS, row-major, padded
#pragma unroll
        for (int t = 0; t < kXLoads; ++t) {
            const int idx = t * 64 + lane;
            *reinterpret_cast<u32x4*>(xbuf + (idx / kPieces) * Cfg::kXStride + (idx % kPieces) * 16) = sl.x[t];
        }
    };
    auto read_frags = [&](Frag (&xf)[kGroups]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < kGroups; ++s)
            xf[s] = *reinterpret_cast<const Frag*>(xbuf + n16 * Cfg::kXStride + s * 64 + g * 16);
    };

    if (nblk > 0) {
        Slot xs[kDX] = {};
        WSlot ws[kDW] = {};
#pragma unroll
        for (int j = 0; j < kDX; ++j) load_entries(xs[j], j);
#pragma unroll
        for (int j = 0; j < kDW; ++j) {
            if constexpr (kHalfW) issue_weights(ws[j], 0, j * kWT);  // both halves of block 0
            else issue_weights(ws[j], j);
        }
#pragma unroll
        for (int j = 0; j < kDX; ++j) issue_gather(xs[j]);
#pragma unroll
        for (int j = 0; j < kDX; ++j) load_entries(xs[j], kDX + j);
        Frag xf_c[kGroups];
        stage(xs[0]);
        wave_sync();
        read_frags(xf_c);
        wave_sync();

        // One block: sl holds block b, sn holds block b + 1.  A wavefront issues in order, so the block's
        // MFMAs only overlap with its other work if that work does not depend on them and is interleaved
        // with them: the accumulator update of block b-1, the staging of block b+1 and the loads for
        // later blocks are therefore issued between the MFMAs of block b.
        // Two result sets alternate, so a block's products stay where the MFMAs left them until the next
        // block's turn adds them to the accumulator.
        struct Result {
            f32x4 d[kNCT];  // d[ct][i] = channel ct*16 + 4*g + i of link n16 of the block
            float* dst;     // accumulator row of that link (+ 4*g)
            bool valid;     // this lane's link exists
        };
        Result res[2] = {};
        res[0].dst = res[1].dst = acc + g * 4;
        // the accumulator rows are read at the start of a turn and written back at its end, so the LDS
        // latency is paid once, under the turn's MFMAs
        auto flush_read = [&](const Result& r, f32x4 (&av)[kNCT]) __attribute__((always_inline)) {
#pragma unroll
            for (int ct = 0; ct < kNCT; ++ct) av[ct] = *reinterpret_cast<const f32x4*>(r.dst + ct * 16);
        };
        // (Letting lanes without a link update spare LDS bytes instead, one row for all or 16 bytes per lane, makes
        // a turn one basic block in which the compiler deals the update and the loads out between the MFMAs;
        // both were measured at 73-76 us against 62 with this branch.)
        auto flush_write = [&](const Result& r, const f32x4 (&av)[kNCT]) __attribute__((always_inline)) {
            if (r.valid) {
#pragma unroll
                for (int ct = 0; ct < kNCT; ++ct) *reinterpret_cast<f32x4*>(r.dst + ct * 16) = av[ct] + r.d[ct];
            }
        };
        auto mfmas = [&](Result& cur, const WSlot& wl, int ct0, const Frag (&xf)[kGroups]) __attribute__((always_inline)) {
#pragma unroll
            for (int s = 0; s < kGroups; ++s)
#pragma unroll
                for (int c = 0; c < kWT; ++c) {
                    const int ct = ct0 + c;
                    if constexpr (kIsF32) {
                        cur.d[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(wl.w[c][s][0], xf[s][0], cur.d[ct], 0, 0, 0);
                        cur.d[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(wl.w[c][s][1], xf[s][1], cur.d[ct], 0, 0, 0);
                        cur.d[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(wl.w[c][s][2], xf[s][2], cur.d[ct], 0, 0, 0);
                        cur.d[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(wl.w[c][s][3], xf[s][3], cur.d[ct], 0, 0, 0);
                    } else {
                        cur.d[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl.w[c][s], xf[s], cur.d[ct], 0, 0, 0);
                    }
                }
        };
        auto body = [&](int b, Slot& sl, const Slot& sn, WSlot& wl, WSlot& wl2, Result& cur, const Result& prev) __attribute__((always_inline)) {
            const int cnt = ((sl.dc >> 7) & 15) + 1;
            cur.valid = n16 < cnt;
            cur.dst = acc + sl.drow * Cfg::kStride + g * 4;
            stage(sn);  // the next block's rows (this block's fragments are already in registers)
            wave_sync();
            f32x4 av[kNCT];
            flush_read(prev, av);
            Frag xf_n[kGroups];
            read_frags(xf_n);

#pragma unroll
            for (int ct = 0; ct < kNCT; ++ct) cur.d[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (kHalfW) {
                mfmas(cur, wl, 0, xf_c);
                issue_weights(wl, b + 1, 0);        // first half of the next block's matrix
                mfmas(cur, wl2, kWT, xf_c);
                issue_gather(sl);
                load_entries(sl, b + 2 * kDX);
                issue_weights(wl2, b + 1, kWT);     // its second half
            } else {
                mfmas(cur, wl, 0, xf_c);
                issue_gather(sl);               // block b + kDX: its entries arrived kDX turns ago
                load_entries(sl, b + 2 * kDX);
                issue_weights(wl, b + kDW);
            }
            flush_write(prev, av);
#pragma unroll
            for (int s = 0; s < kGroups; ++s) xf_c[s] = xf_n[s];
            // scheduling hint: one MFMA, then a few of the other instructions, repeated
            if constexpr (kIsF32) {
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);  // VALU
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // DS write
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
            }
        };
        int done = 0;  // number of blocks computed; the last one's result is still to be added
        for (int b = 0; b < nblk; b += kTurn) {
            bool stop = false;
#pragma unroll
            for (int j = 0; j < kTurn; ++j) {
                if (!stop) {
                    body(b + j, xs[j % kDX], xs[(j + 1) % kDX], ws[kHalfW ? 0 : j % kDW], ws[1], res[j % 2], res[(j + 1) % 2]);
                    done = b + j + 1;
                    stop = b + j + 1 >= nblk;
                }
            }
        }
        f32x4 av[kNCT];
        if ((done + 1) % 2 == 0) { flush_read(res[0], av); flush_write(res[0], av); }  // the set of block done-1
        else { flush_read(res[1], av); flush_write(res[1], av); }
    }
    wave_sync();
    const int co0 = blockIdx.y * COT;
    constexpr int kQuads = COT / 4;
    for (int idx = lane; idx < row_count * kQuads; idx += 64) {
        const int r = idx / kQuads, c4 = (idx % kQuads) * 4;
        const int64_t row = wt * 64 + row_base + r;
        if (row >= a.n_rows) break;
        const f32x4 v = *reinterpret_cast<const f32x4*>(acc + r * Cfg::kStride + c4);
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

// Weights as stored (element (k, co, cc) at w[k*per + co*s_co + cc*s_cc]) -> fragment-major copy for
// gather_wave_kernel: [k][co tile][ct][s][lane = n16 + 16*g][16 bytes] holding channels
// co = tile*COT + ct*16 + n16, cc = s*kGroup + g*(kGroup/4) + 0..kGroup/4-1.
template <typename T, int CC, int COT>
__global__ __launch_bounds__(256) void weight_frag_kernel(const T* __restrict__ w, T* __restrict__ wf, int kvol,
                                                          int co_total, int s_co, int s_cc) {
    using Cfg = WaveCfg<T, CC, COT>;
    constexpr int kPer = Cfg::kGroup / 4;  // elements per 16-byte fragment
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)kvol * co_total * CC;
    if (idx >= total) return;
    int64_t r = idx;
    const int i = (int)(r % kPer); r /= kPer;
    const int lane = (int)(r % 64); r /= 64;
    const int s = (int)(r % Cfg::kGroups); r /= Cfg::kGroups;
    const int ct = (int)(r % Cfg::kNCT); r /= Cfg::kNCT;
    const int tile = (int)(r % (co_total / COT)); r /= (co_total / COT);
    const int k = (int)r;
    const int co = tile * COT + ct * 16 + (lane & 15);
    const int cc = s * Cfg::kGroup + (lane >> 4) * kPer + i;
    wf[idx] = w[(size_t)k * co_total * CC + (size_t)co * s_co + (size_t)cc * s_cc];
}

template <typename T, int CC, int COT>
int launch_wave(GatherArgs a, hipStream_t s) {
    using Cfg = WaveCfg<T, CC, COT>;
    auto kern = gather_wave_kernel<T, CC, COT>;
    a.lds_per_wave = Cfg::per_wave_bytes(a.kvol);
    a.w_bytes = (uint32_t)((size_t)a.kvol * a.co_total * CC * sizeof(T));
    const int lds = a.lds_per_wave;  // one wavefront per workgroup: they are independent, small groups place freely
    {
        static std::mutex mu;
        static int attr_lds = 0;  // largest dynamic LDS size opted into so far
        std::lock_guard<std::mutex> lk(mu);
        if (lds > attr_lds) {
            SP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
            attr_lds = lds;
        }
    }
    // fragment-major copy of the weights (also undoes the data gradient's transposition)
    const int64_t n = (int64_t)a.kvol * a.co_total * CC;
    Buf wf;
    T* d_wf = static_cast<T*>(a.scratch);
    if (d_wf) {
        if ((size_t)n * sizeof(T) > a.scratch_bytes)
            return fail(SP_ERR_UNSUPPORTED, "weights of %lld bytes exceed the %zu bytes of static scratch",
                        (long long)(n * sizeof(T)), a.scratch_bytes);
    } else {
        wf = dev_alloc((size_t)n * sizeof(T), s);
        if (!wf) return SP_ERR_ALLOC;
        d_wf = ptr<T>(wf);
    }
    const int s_co = a.w_transposed ? 1 : CC, s_cc = a.w_transposed ? a.co_total : 1;
    hipLaunchKernelGGL((weight_frag_kernel<T, CC, COT>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       static_cast<const T*>(a.w), d_wf, a.kvol, a.co_total, s_co, s_cc);
    a.w = d_wf;
    const int64_t nwt = (a.n_rows + 63) / 64;
    // A launch whose sub-tiles fit the GPU's LDS at once runs as long as its longest wavefront: then long
    // sub-tiles (48 blocks and more, against a typical 27-35; measured best of 32..64) are shared by two
    // wavefronts.  Larger launches
    // run in several rounds, where splitting would only add padding.
    const int64_t resident_tiles = 256 * (160 * 1024 / (int64_t)a.lds_per_wave);
    a.split_blocks = (nwt * (a.co_total / COT) * 5 / 4 <= resident_tiles) ? 48 : 0x7fffffff;
    // two wavefronts per sub-tile only where sub-tiles may be split (the second one leaves at once otherwise)
    dim3 grid((unsigned)((a.split_blocks == 0x7fffffff ? 1 : 2) * nwt), (unsigned)(a.co_total / COT));
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, s, a);
    SP_HIP(hipGetLastError());
    return SP_OK;  // wf goes back to the pool; later users are ordered behind this launch on the stream
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
        // one link's dot product first, then added: a single chain over all kvol * cc terms (6000 for a 5x5x5
        // kernel on 48 channels) measured 8e-6 against the fp64 definition, this 1e-6
        float dot = 0.f;
        for (int j = 0; j < cc; ++j) {
            if constexpr (std::is_same<T, float>::value)
                dot = fmaf(wp[(size_t)j * w_cc], fp[j], dot);
            else
                dot = fmaf(bf16_to_f32(wp[(size_t)j * w_cc]), bf16_to_f32(fp[j]), dot);
        }
        acc += dot;
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
int launch_gather(GatherArgs a, hipStream_t s) {
    using Cfg = GatherCfg<T, CC, COT, TR>;
    auto kern = gather_mma_kernel<T, CC, COT, TR>;
    {
        static std::mutex mu;
        static bool attr_set = false;  // one-time opt-in to > 64 KB of dynamic LDS
        std::lock_guard<std::mutex> lk(mu);
        if (!attr_set) {
            SP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)Cfg::kLds));
            attr_set = true;
        }
    }
    Buf wt;
    if (a.w_transposed) {  // stored matrix is [cout = cc][cin = co]; the kernel wants [co][cc]
        const int64_t n = (int64_t)a.kvol * CC * a.co_total;
        wt = dev_alloc((size_t)n * sizeof(T), s);
        if (!wt) return SP_ERR_ALLOC;
        hipLaunchKernelGGL(transpose_w_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           static_cast<const T*>(a.w), ptr<T>(wt), a.kvol, CC, a.co_total);
        a.w = wt->p;
    }
    const int64_t ntiles = (a.n_rows + kTileRows - 1) / kTileRows;
    dim3 grid((unsigned)(ntiles * (kTileRows / TR)), (unsigned)(a.co_total / COT));
    hipLaunchKernelGGL(kern, grid, dim3(256), Cfg::kLds, s, a);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// Narrow layers take the wavefront-private kernel, with the widest channel tile whose weight matrix fits in
// 32 fragment registers (CC/group * COT/16 fragments of 4 registers each).  Returns that tile, or 0 when the
// workgroup-cooperative kernel takes the layer.
int wave_tile(int cc, int co, bool is_f32, bool wave_ok) {
    const int groups = cc / (is_f32 ? 16 : 32);
    if (!wave_ok) return 0;
    if (groups * 4 <= 16 && co % 64 == 0) return 64;  // more than 8 fragments per lane: the matrix is held in two halves
    if (groups * 2 <= 8 && co % 32 == 0) return 32;
    if (groups <= 2 && (co == 16 || co == 48)) return 16;
    return 0;
}

template <typename T, int CC>
int dispatch_co(const GatherArgs& a, hipStream_t s) {
    constexpr int kGroups = CC / (std::is_same<T, float>::value ? 16 : 32);
    const int cot = wave_tile(CC, a.co_total, std::is_same<T, float>::value, a.wave_ok != 0);
    if constexpr (kGroups * 4 <= 16)
        if (cot == 64) return launch_wave<T, CC, 64>(a, s);
    if constexpr (kGroups * 2 <= 8)
        if (cot == 32) return launch_wave<T, CC, 32>(a, s);
    if constexpr (kGroups <= 2)
        if (cot == 16) return launch_wave<T, CC, 16>(a, s);
    // Wide layers: workgroup-cooperative kernel; rows per workgroup keep accumulator + staging within
    // ~64 KB so two workgroups share a CU
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

namespace {
// Which gather kernel a layer takes: 0 row-stationary (sp_conv_dense.hip), 1 wavefront-private link lists,
// 2 workgroup-cooperative link lists, 3 plain.
int select_gather(const MapSide& side, int kvol, int64_t total_links, int cc, int co, sp_dtype dt) {
    const size_t elt = dt == SP_F32 ? 4 : 2;
    // Row-stationary kernel: it multiplies all kvol offsets of every row, the link-list kernels only the links
    // that exist but pay per link for bookkeeping, weight re-reads and the accumulator update.  Measured, it is
    // the faster one from about 1 link in 20 row-offsets upwards on 128- and 256-channel inputs, from 1 in 4
    // on 64-channel inputs.
    // (A side with position classes skips the offsets its tiles cannot have: its cost follows the links.)
    const uint64_t lim = 0x7fffffffull;
    if (dense_shape_ok(cc, co, dt) &&
        (side.tile_mask || (double)total_links >= dense_min_fill(cc) * (double)side.n_rows * kvol) &&
        (uint64_t)side.n_src * cc * elt < lim && (uint64_t)side.n_rows * kvol * 4 < lim && (uint64_t)kvol * cc * co * elt < lim)
        return 0;
    if (mma_shape_ok(cc, co, dt)) {
        const bool wave_ok = (uint64_t)side.n_src * cc * elt < 0xffffffffull && (uint64_t)total_links * 4 < 0xffffffffull;
        return wave_tile(cc, co, dt == SP_F32, wave_ok) ? 1 : 2;
    }
    return 3;
}
}  // namespace

// side: which rows are destinations.  w_transposed = false: W[k][co][cc] as stored (forward);
// true: the stored W is [k][cc][co] (data gradient), transposed into pool memory first for the MFMA path.
int conv_gather(const MapSide& side, int kvol, int64_t total_links, const void* d_f, const void* d_w, bool w_transposed,
                void* d_g, int cc, int co, sp_dtype dt, hipStream_t s, void* scratch, size_t scratch_bytes) {
    if (side.n_rows == 0) return SP_OK;
    if (scratch && w_transposed) return fail(SP_ERR_UNSUPPORTED, "no allocation-free path for transposed weights");
    const size_t elt = dt == SP_F32 ? 4 : 2;
    const int kind = select_gather(side, kvol, total_links, cc, co, dt);
    if (kind == 0) {
        Buf wt;
        const void* w = d_w;
        if (w_transposed) {  // stored matrix is [cout = cc][cin = co]; the kernel wants [co][cc]
            const int64_t n = (int64_t)kvol * cc * co;
            wt = dev_alloc((size_t)n * elt, s);
            if (!wt) return SP_ERR_ALLOC;
            hipLaunchKernelGGL(transpose_w_kernel<bf16_t>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                               static_cast<const bf16_t*>(d_w), ptr<bf16_t>(wt), kvol, cc, co);
            w = wt->p;
        }
        return conv_gather_dense(side, kvol, d_f, w, d_g, cc, co, s);
    }
    if (kind == 1 || kind == 2) {
        GatherArgs a;
        a.tl_off = ptr<int32_t>(side.tl_off);
        a.tl_src = ptr<int32_t>(side.tl_src);
        a.tl_row = ptr<uint16_t>(side.tl_row);
        a.f = d_f;
        a.w = d_w;
        a.w_transposed = w_transposed ? 1 : 0;
        a.scratch = scratch;
        a.scratch_bytes = scratch_bytes;
        const uint64_t fb = (uint64_t)side.n_src * cc * elt, sb = (uint64_t)total_links * 4;
        a.wave_ok = fb < 0xffffffffull && sb < 0xffffffffull;
        a.f_bytes = (uint32_t)fb;
        a.src_bytes = (uint32_t)sb;
        a.row_bytes = (uint32_t)((uint64_t)total_links * 2);
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

// Scratch of the allocation-free entry point: the fragment-major weight copy that sp_conv_fwd takes from the
// pool.  One copy of the array exists on every GPU the library is loaded on, at its own address; host code
// must not use the array's name as a pointer, only the address hipGetSymbolAddress reports for the current
// device.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
int static_scratch(void** out) {
    int dev = 0;
    SP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SP_ERR_UNSUPPORTED, "device %d: more devices than expected", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        SP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(SP_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SP_OK;
}

// a: source features (rows_a), b: weights, c: destination (rows_c); a zero-sized buffer may be NULL
// a_is_in: a holds the map's input rows and c its output rows (forward), else the other way round
int check_conv_args(const sp_kmap_t* m, const void* a, bool a_is_in, const void* b, const void* c, int cin, int cout,
                    sp_dtype dt) {
    if (!m) return fail(SP_ERR_INVALID_ARG, "kmap handle is NULL");
    SP_TRY(kmap_resolve(m));  // the sizes of a map whose build has not reported yet
    const int64_t rows_a = a_is_in ? m->n_in : m->n_out, rows_c = a_is_in ? m->n_out : m->n_in;
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
    SP_TRY(check_conv_args(m, d_x, true, d_w, d_y, cin, cout, dt));
    return conv_gather(m->out_side, m->kvol, m->total, d_x, d_w, false, d_y, cin, cout, dt, (hipStream_t)stream);
}

int sp_conv_bwd_data(const sp_kmap_t* m, const void* d_dy, const void* d_w, void* d_dx, int32_t cin, int32_t cout,
                     sp_dtype dt, void* stream) {
    SP_TRY(check_conv_args(m, d_dy, false, d_w, d_dx, cin, cout, dt));
    return conv_gather(m->in_side, m->kvol, m->total, d_dy, d_w, true, d_dx, cout, cin, dt, (hipStream_t)stream);
}

const char* sp_conv_kernel_name(const sp_kmap_t* m, int32_t cin, int32_t cout, sp_dtype dt, int32_t direction) {
    static const char* const names[] = {"gather_dense_kernel", "gather_wave_kernel", "gather_mma_kernel",
                                        "gather_plain_kernel"};
    if (!m || cin < 1 || cout < 1 || (dt != SP_F32 && dt != SP_BF16) || kmap_resolve(m) != SP_OK) return "";
    return direction == 0 ? names[select_gather(m->out_side, m->kvol, m->total, cin, cout, dt)]
                          : names[select_gather(m->in_side, m->kvol, m->total, cout, cin, dt)];
}

int sp_conv_fwd_noalloc(const sp_kmap_t* m, const void* d_x, const void* d_w, void* d_y, int32_t cin, int32_t cout,
                        sp_dtype dt, void* stream) {
    SP_TRY(check_conv_args(m, d_x, true, d_w, d_y, cin, cout, dt));
    void* scratch = nullptr;
    SP_TRY(static_scratch(&scratch));
    return conv_gather(m->out_side, m->kvol, m->total, d_x, d_w, false, d_y, cin, cout, dt, (hipStream_t)stream,
                       scratch, kStaticScratchBytes);
}

}  // extern "C"
