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
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "sp_internal.h"

namespace sp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;

__device__ __forceinline__ float load_f32(const float* p) { return *p; }
__device__ __forceinline__ float load_f32(const bf16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

// Work decomposition.  Offset k's links are sorted by row on one side, so the j-th fraction of every
// offset's list covers about the same rows (and, on the other side, their spatial neighbours).  The lists are
// cut into S8 "strips" (the host uses 8, one per XCD): strip s is, for every offset in turn, the s-th 1/S8 of
// its list; the concatenation of these stretches is the strip's link sequence.  Workgroup i runs on XCD i % 8,
// so a strip's rows, touched by up to 27 offsets, are fetched by one XCD.  A strip's sequence is cut into nc
// chunks of C links, one workgroup each (times the channel tiles): equal work whatever the offsets'
// densities.  A chunk that spans several offsets produces one partial block per offset ("piece").
//
// Partial blocks are numbered strip by strip in sequence order: within a strip, the piece that starts at
// sequence position p has number ceil(p / C) + (offset stretches starting before p at a position that is
// not a multiple of C): every chunk start and every such stretch start begins exactly one piece.
struct PlanArgs {
    int kvol, S8, nc, C, tiles;
    int pair_stride;      // offset k's pairs start at k * pair_stride in the pair arrays
    int slots_per_strip;  // nc + kvol: more than the largest piece number of a strip
    int32_t koff[130];    // exclusive prefix of the offsets' link counts
};
// stretch of offset k in strip s: links [lo, lo + len), lo = koff[k] + floor(cnt * s / S8) in 32-bit steps
__device__ __forceinline__ void strip_stretch(const PlanArgs& pa, int k, int s, int* lo, int* len) {
    const uint32_t k0 = (uint32_t)k * (uint32_t)pa.pair_stride, cnt = (uint32_t)(pa.koff[k + 1] - pa.koff[k]), n = (uint32_t)pa.S8;
    const uint32_t q = cnt / n, r = cnt % n;  // r * s < 2^20
    const uint32_t b0 = q * (uint32_t)s + r * (uint32_t)s / n, b1 = q * (uint32_t)(s + 1) + r * (uint32_t)(s + 1) / n;
    *lo = (int)(k0 + b0);
    *len = (int)(b1 - b0);
}

// The plan of one strip, computed by every wavefront for itself (lane = offset; registers only): lo/len of the
// stretches of offsets lane and lane + 64, and for chunk `chunk` of the strip (positions [chunk*C, chunk*C + C)
// of the strip's sequence): the offset whose stretch holds the chunk's first position (kvol: the chunk lies past
// the strip's end), that stretch's start position, and the number of stretches before it that start off a chunk
// boundary.
struct StripPlan {
    int lo[2], len[2];      // this lane's offsets
    int k0, pos0, nb0;      // the chunk's start (the same in every lane)
};
__device__ __forceinline__ StripPlan strip_plan(const PlanArgs& pa, int s, int chunk, int lane) {
    StripPlan sp;
    const int cb = chunk * pa.C;
    sp.k0 = pa.kvol;
    sp.pos0 = 0;
    sp.nb0 = 0;
    int pos_base = 0, nb_base = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int k = h * 64 + lane;
        int lo = 0, len = 0;
        if (k < pa.kvol) strip_stretch(pa, k, s, &lo, &len);
        int inc = len;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(inc, d, 64);
            if (lane >= d) inc += t;
        }
        const int pos = pos_base + inc - len;
        const bool real = len > 0 && pos % pa.C != 0;
        const unsigned long long mask = __ballot(real);
        const int nb = nb_base + __popcll(mask & ((1ull << lane) - 1ull));
        sp.lo[h] = lo;
        sp.len[h] = len;
        const unsigned long long here = __ballot(len > 0 && pos <= cb && cb < pos + len);
        if (here) {  // exactly one lane
            const int src = __builtin_ctzll(here);
            sp.k0 = h * 64 + src;
            sp.pos0 = __shfl(pos, src, 64);
            sp.nb0 = __shfl(nb, src, 64);
        }
        pos_base += __shfl(inc, 63, 64);
        nb_base += __popcll(mask);
    }
    return sp;
}

// dW[k][e] = sum of offset k's partial blocks, strip by strip, in a fixed order: 16 interleaved running sums
// per element, each over every 16th block, then added in order 0..15.  grid (per/64, kvol); block = 16 lanes
// x 4 elements each x 16 block slices.
// P: type of the partial blocks and of the sums (double on the fp32 path, see wgrad_staged_kernel).
// first / count [S8][kvol]: number of offset k's first partial block in strip s and how many it has (written by
// the staged kernel).
template <typename P>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const P* __restrict__ part,
                                                           const int32_t* __restrict__ first,
                                                           const int32_t* __restrict__ count, int S8, int kvol, int per,
                                                           float* __restrict__ dw) {
    typedef P Px4 __attribute__((ext_vector_type(4)));
    constexpr int kMaxStrips = 64;
    __shared__ int s_first[kMaxStrips], s_count[kMaxStrips];
    __shared__ Px4 red[16][16];
    const int k = blockIdx.y;
    const int el = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int e = (blockIdx.x * 16 + el) * 4;
    for (int s = threadIdx.x; s < S8; s += 256) {
        s_first[s] = first[s * kvol + k];
        s_count[s] = count[s * kvol + k];
    }
    __syncthreads();
    Px4 sum = {0, 0, 0, 0};
    int n = 0;
    for (int s = 0; s < S8; ++s) {
        const int f = s_first[s], c = s_count[s];
        for (int j = (grp - n) & 15; j < c; j += 16)
            sum += *reinterpret_cast<const Px4*>(part + (size_t)(f + j) * per + e);
        n += c;
    }
    red[grp][el] = sum;
    __syncthreads();
    if (grp == 0) {
        Px4 t = red[0][el];
#pragma unroll
        for (int i = 1; i < 16; ++i) t += red[i][el];
        *reinterpret_cast<f32x4*>(dw + (size_t)k * per + e) = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
    }
}

// ---------------------------------------------------------------------------------------------------------
// Staged kernel.  Tile COB x CIB of dW per workgroup; WCO x WCI x WK wavefronts: the tile is cut WCO x WCI
// ways and each step's 32*WK links WK ways.  One workgroup per (chunk, channel tile).
// ---------------------------------------------------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T, int COB, int CIB, int WCO, int WCI, int WK>
struct StagedCfg {
    static constexpr int kElt = sizeof(T);
    static constexpr bool kIsF32 = sizeof(T) == 4;
    static constexpr int kWaves = WCO * WCI * WK, kThreads = 64 * kWaves;
    static constexpr int kS = 32 * WK;                     // links per step
    static constexpr int kTPR = kThreads / kS;             // threads that share the loading of one row
    static constexpr int kTA = COB / WCO / 16, kTB = CIB / WCI / 16;  // 16x16 tiles per wavefront
    // Row pad so that a fragment read (4 link rows x 16 lanes) hits disjoint banks: bf16 transpose reads take
    // 32 bytes per row, fp32 reads 64 * kT bytes per row (a lane reads its kT channels at once).
    static constexpr int pad_f32(int kt) { return kt >= 4 ? 0 : 64 * kt; }
    static constexpr int kPA = COB * kElt + (kIsF32 ? pad_f32(kTA) : 32);  // staged row pitch of dY rows
    static constexpr int kPB = CIB * kElt + (kIsF32 ? pad_f32(kTB) : 32);  // and of X rows
    static constexpr int kPiecesA = COB * kElt / 16, kPiecesB = CIB * kElt / 16;  // 16-byte pieces per row
    static constexpr int kLoadsA = (kPiecesA + kTPR - 1) / kTPR;  // per thread and step
    static constexpr int kLoadsB = (kPiecesB + kTPR - 1) / kTPR;
    static constexpr int kBufBytes = kS * (kPA + kPB);
    static constexpr int kPartElt = kIsF32 ? 8 : 4;        // partial blocks: double on the fp32 path, float for bf16
    static constexpr int kRedBytes = WK > 1 ? COB * CIB * kPartElt : 0;
    static constexpr int kLds = 2 * kBufBytes > kRedBytes ? 2 * kBufBytes : kRedBytes;
    static_assert(COB % (16 * WCO) == 0 && CIB % (16 * WCI) == 0, "tile split");
    static_assert(kThreads % kS == 0, "whole threads per row");
    static_assert(!kIsF32 || (kTA <= 4 && kTB <= 4), "an fp32 lane reads its channels with one LDS load");
};

struct StagedArgs {
    const int32_t* pair_in;
    const int32_t* pair_out;
    const void* x;
    const void* dy;
    void* part;   // partial blocks [slot][cout][cin], double (fp32 path) or float (bf16 path)
    int cin, cout;
    uint32_t x_bytes, dy_bytes, pair_bytes;  // buffer sizes (< 2 GiB each)
    PlanArgs plan;
    int32_t* first;   // [S8][kvol], for the reduction: written here by the workgroup in whose chunk a stretch starts
    int32_t* count;
};

template <typename T, int COB, int CIB, int WCO, int WCI, int WK, int kD>
__global__ __launch_bounds__(64 * WCO * WCI * WK) void wgrad_staged_kernel(StagedArgs a) {
    using Cfg = StagedCfg<T, COB, CIB, WCO, WCI, WK>;
    constexpr bool kIsF32 = Cfg::kIsF32;
    constexpr int kTA = Cfg::kTA, kTB = Cfg::kTB, kPA = Cfg::kPA, kPB = Cfg::kPB, kS = Cfg::kS, kTPR = Cfg::kTPR;
    constexpr int kLoadsA = Cfg::kLoadsA, kLoadsB = Cfg::kLoadsB, kThreads = Cfg::kThreads;
    extern __shared__ __align__(16) unsigned char smem[];

    // workgroup -> (strip, chunk, channel tile): XCD = id % 8 takes strips XCD, XCD + 8, ... in that order
    const PlanArgs& pa = a.plan;
    const int tile = blockIdx.x % pa.tiles, q0 = blockIdx.x / pa.tiles;
    const int q = q0 >> 3, strip = (q0 & 7) + 8 * (q / pa.nc), chunk = q % pa.nc;
    const int cb = chunk * pa.C, ce = cb + pa.C;  // this chunk's positions in the strip's link sequence
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wci = (wave / WK) % WCI, wco = wave / (WK * WCI);
    const int n16 = lane & 15, g = lane >> 4;
    const int co0 = (tile / (a.cin / CIB)) * COB, ci0 = (tile % (a.cin / CIB)) * CIB;

    // Buffer addressing: a lane whose link lies past the piece's end asks for an offset outside the buffer
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

    // Loading: thread = (row of the step, sub); it loads the 16-byte pieces sub, sub + kTPR, ... of that row of
    // dY and of X: one row number and one address per operand, the pieces differ by constant offsets; four
    // adjacent lanes read 64 consecutive bytes.
    const int ld_row = tid / kTPR, ld_sub = tid % kTPR;
    const uint32_t col_a = (uint32_t)co0 * Cfg::kElt + ld_sub * 16, col_b = (uint32_t)ci0 * Cfg::kElt + ld_sub * 16;
    const int st_a = ld_row * kPA + ld_sub * 16, st_b = kS * kPA + ld_row * kPB + ld_sub * 16;  // LDS offsets
    uint32_t beg4 = 0;  // byte offset of the piece's first link in the pair lists
    int len = 0;        // links of the piece

    struct Regs {
        int ia, ib;                        // gathered row numbers
        u32x4 va[kLoadsA], vb[kLoadsB];    // gathered pieces
    };
    struct RowAddr {
        uint32_t a, b;
    };
    // rel: position of the step's first link in the piece
    auto load_idx = [&](Regs& r, int rel) __attribute__((always_inline)) {
        const uint32_t off = rel + ld_row < len ? beg4 + (uint32_t)(rel + ld_row) * 4u : kOutside;
        r.ia = (int)__builtin_amdgcn_raw_buffer_load_b32(rPO, off, 0, 0);
        r.ib = (int)__builtin_amdgcn_raw_buffer_load_b32(rPI, off, 0, 0);
    };
    // Row loads in two halves, so that the next row numbers can be requested between them: a wavefront's
    // loads complete in order, and the wait for row numbers at the top of the next step must not also wait
    // for this step's rows.
    auto row_addrs = [&](const Regs& r, int rel, RowAddr& ra) __attribute__((always_inline)) {
        const bool live = rel + ld_row < len;
        ra.a = live ? (uint32_t)r.ia * rowbytes_a + col_a : kOutside;
        ra.b = live ? (uint32_t)r.ib * rowbytes_b + col_b : kOutside;
    };
    auto issue_rows = [&](Regs& r, const RowAddr& ra) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoadsA; ++j) {
            const bool mine = Cfg::kPiecesA % kTPR == 0 || ld_sub + j * kTPR < Cfg::kPiecesA;
            r.va[j] = __builtin_amdgcn_raw_buffer_load_b128(rDY, mine ? ra.a + j * kTPR * 16 : kOutside, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < kLoadsB; ++j) {
            const bool mine = Cfg::kPiecesB % kTPR == 0 || ld_sub + j * kTPR < Cfg::kPiecesB;
            r.vb[j] = __builtin_amdgcn_raw_buffer_load_b128(rX, mine ? ra.b + j * kTPR * 16 : kOutside, 0, 0);
        }
    };
    auto load_rows = [&](Regs& r, int rel) __attribute__((always_inline)) {
        RowAddr ra;
        row_addrs(r, rel, ra);
        issue_rows(r, ra);
    };
    auto store_rows = [&](const Regs& r, unsigned char* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoadsA; ++j)
            if (Cfg::kPiecesA % kTPR == 0 || ld_sub + j * kTPR < Cfg::kPiecesA)
                *reinterpret_cast<u32x4*>(buf + st_a + j * kTPR * 16) = r.va[j];
#pragma unroll
        for (int j = 0; j < kLoadsB; ++j)
            if (Cfg::kPiecesB % kTPR == 0 || ld_sub + j * kTPR < Cfg::kPiecesB)
                *reinterpret_cast<u32x4*>(buf + st_b + j * kTPR * 16) = r.vb[j];
    };

    // fp32 path: the matrix cores' accumulator only ever holds the sum of kFlushEvery * kD steps (64 links); it
    // is then added into a double-precision total, the partial blocks are doubles and so are the final sums.
    // Sums whose terms mostly share a sign within long stretches of rows and cancel between them (gradients
    // that are constant per cloud, as global pooling produces) otherwise lose more than the 1e-5 parity bound
    // to the rounding of the large intermediate sums.
    typedef double f64x4 __attribute__((ext_vector_type(4)));
    using Part = typename std::conditional<kIsF32, double, float>::type;
    f32x4 acc[kTA][kTB];
    f64x4 tot[kIsF32 ? kTA : 1][kIsF32 ? kTB : 1];
    constexpr int kFlushEvery = 2 / kD > 0 ? 2 / kD : 1;

    // This wavefront's 32 links of the step and its channel slices.  Channel of (16x16 tile t, index m in the
    // tile) within the slice: bf16 t*16 + m; fp32 m*kT + t, so that a lane's kT values are adjacent in LDS.
    const int frag_a = (32 * wk) * kPA + (wco * kTA * 16) * Cfg::kElt;
    const int frag_b = kS * kPA + (32 * wk) * kPB + (wci * kTB * 16) * Cfg::kElt;
    const int lane_a = kIsF32 ? g * kPA + n16 * kTA * 4 : (8 * g + (n16 >> 2)) * kPA + (n16 & 3) * 8;
    const int lane_b = kIsF32 ? g * kPB + n16 * kTB * 4 : (8 * g + (n16 >> 2)) * kPB + (n16 & 3) * 8;
    auto compute = [&](const unsigned char* buf) __attribute__((always_inline)) {
        const unsigned char* A = buf + frag_a + lane_a;
        const unsigned char* B = buf + frag_b + lane_b;
        if constexpr (kIsF32) {
            // MFMA 16x16x4: lane (index n16 in the tile, link g) of both operands; the fragments of the next 4
            // links are read while the current ones are multiplied
            typedef float fvA __attribute__((ext_vector_type(kTA == 3 ? 4 : kTA)));
            typedef float fvB __attribute__((ext_vector_type(kTB == 3 ? 4 : kTB)));
            float av[2][kTA], bv[2][kTB];
            auto read = [&](int j, float (&x)[kTA], float (&y)[kTB]) __attribute__((always_inline)) {
                if constexpr (kTA == 1) x[0] = *reinterpret_cast<const float*>(A + 4 * j * kPA);
                else {
                    const fvA v = *reinterpret_cast<const fvA*>(A + 4 * j * kPA);
#pragma unroll
                    for (int ta = 0; ta < kTA; ++ta) x[ta] = v[ta];
                }
                if constexpr (kTB == 1) y[0] = *reinterpret_cast<const float*>(B + 4 * j * kPB);
                else {
                    const fvB v = *reinterpret_cast<const fvB*>(B + 4 * j * kPB);
#pragma unroll
                    for (int tb = 0; tb < kTB; ++tb) y[tb] = v[tb];
                }
            };
            read(0, av[0], bv[0]);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j < 7) read(j + 1, av[(j + 1) & 1], bv[(j + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);  // keeps the reads ahead of the products that hide them
#pragma unroll
                for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                    for (int tb = 0; tb < kTB; ++tb)
                        acc[ta][tb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[j & 1][ta], bv[j & 1][tb], acc[ta][tb], 0, 0, 0);
            }
        } else {
            // MFMA 16x16x32: lane (channel n16, links 8g .. 8g+7).  One transpose read: the 16 lanes of group g
            // point at 4 rows x 16 channels (lane i: row i/4, channels 4*(i%4)..+3) and lane i receives
            // channel i of those 4 rows.
            typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
            auto frag = [&](const unsigned char* base, int pitch) __attribute__((always_inline)) {
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + 4 * pitch));
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

    // Ring of kD register sets: in step s the rows of step s+kD are requested with the row numbers that were
    // requested in step s-kD, and the row numbers of step s+2*kD are requested.  The step count is rounded up
    // to a multiple of kD (steps past the piece's end load zeros) to keep the loop body branch-free.
    Regs r[kD];
    // the strip's plan (a few hundred cycles of integer arithmetic per wavefront: cheaper than a launch that
    // writes it to memory and the loads that read it back)
    const StripPlan plan = strip_plan(pa, strip, chunk, lane);
    if (chunk == 0 && tile == 0 && wave == 0) {  // offsets without links in this strip: no partial blocks
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int k = h * 64 + lane;
            if (k < pa.kvol && plan.len[h] == 0) {
                a.first[strip * pa.kvol + k] = 0;
                a.count[strip * pa.kvol + k] = 0;
            }
        }
    }
    // the chunk's pieces: walk the strip's stretches, offset by offset
    int pos = plan.pos0, nb = plan.nb0;
    for (int k = plan.k0; k < pa.kvol && pos < ce; ++k) {
        const int lo = __shfl(k < 64 ? plan.lo[0] : plan.lo[1], k & 63, 64);
        const int slen = __shfl(k < 64 ? plan.len[0] : plan.len[1], k & 63, 64);
        if (slen == 0) continue;
        const int s0 = pos, p0 = max(s0, cb), p1 = min(s0 + slen, ce);
        const bool real = s0 % pa.C != 0;
        pos += slen;
        const int nb_here = nb + ((real && s0 < p0) ? 1 : 0);
        if (s0 >= cb && tile == 0 && tid == 0) {  // the stretch starts in this chunk: tell the reduction where its blocks are
            a.first[strip * pa.kvol + k] = strip * pa.slots_per_strip + (s0 + pa.C - 1) / pa.C + nb;
            a.count[strip * pa.kvol + k] = (s0 + slen + pa.C - 1) / pa.C - s0 / pa.C;
        }
        nb += real ? 1 : 0;
        if (p0 >= p1) continue;
        beg4 = (uint32_t)(lo + (p0 - s0)) * 4u;
        len = p1 - p0;
        const int slot = strip * pa.slots_per_strip + (p0 == cb ? chunk : chunk + 1) + nb_here;

#pragma unroll
        for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb) {
                acc[ta][tb] = f32x4{0.f, 0.f, 0.f, 0.f};
                if constexpr (kIsF32) tot[ta][tb] = f64x4{0., 0., 0., 0.};
            }
#pragma unroll
        for (int d = 0; d < kD; ++d) {
            r[d] = Regs{};
            load_idx(r[d], d * kS);
        }
#pragma unroll
        for (int d = 0; d < kD; ++d) {
            load_rows(r[d], d * kS);
            load_idx(r[d], (kD + d) * kS);
        }
        store_rows(r[0], smem);
        __syncthreads();
        int step = 0;
        for (int base = 0; base < len; base += kD * kS, step += kD) {
#pragma unroll
            for (int d = 0; d < kD; ++d) {
                const int b = base + d * kS;
                const int par = (step + d) & 1;  // step s computes from buffer s & 1 and fills the other
                const unsigned char* cur = smem + par * Cfg::kBufBytes;
                unsigned char* nxt = smem + (par ^ 1) * Cfg::kBufBytes;
                RowAddr ra;
                row_addrs(r[d], b + kD * kS, ra);
                __builtin_amdgcn_sched_barrier(0);
                load_idx(r[d], b + 2 * kD * kS);
                __builtin_amdgcn_sched_barrier(0);
                issue_rows(r[d], ra);
                __builtin_amdgcn_sched_barrier(0);  // the requests go out before the step's arithmetic, not after it
                compute(cur);
                __builtin_amdgcn_sched_barrier(0);
                store_rows(r[(d + 1) % kD], nxt);
                __syncthreads();
            }
            if constexpr (kIsF32) {
                // two-level sum: a long fp32 chain would lose more than the accuracy target
                if ((step / kD) % kFlushEvery == kFlushEvery - 1) {
#pragma unroll
                    for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                        for (int tb = 0; tb < kTB; ++tb) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) tot[ta][tb][j] += (double)acc[ta][tb][j];
                            acc[ta][tb] = f32x4{0.f, 0.f, 0.f, 0.f};
                        }
                }
            }
        }
        if constexpr (kIsF32) {
#pragma unroll
            for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
                    for (int j = 0; j < 4; ++j) tot[ta][tb][j] += (double)acc[ta][tb][j];
        }
        // value of this piece's element (ta, tb, j)
        auto piece_val = [&](int ta, int tb, int j) __attribute__((always_inline)) -> Part {
            if constexpr (kIsF32) return tot[ta][tb][j];
            else return acc[ta][tb][j];
        };

        // acc[ta][tb][j] is element (co: tile ta, index 4*g + j; ci: tile tb, index n16) of the wavefront's
        // slice.  The WK link slices are added in order.
        auto chan = [&](int t, int m, int kt) { return kIsF32 ? m * kt + t : t * 16 + m; };
        typedef Part Partx4 __attribute__((ext_vector_type(4)));
        Part* dst = static_cast<Part*>(a.part) + (size_t)slot * a.cout * a.cin;
        // Large tiles: the lane's position is made opaque here, or the store addresses below are computed before the
        // main loop, where the registers that hold them get spilled and reloaded between the gathers (a reload waits
        // for every load issued before it; 256 x 256) or cost two thirds of the wavefronts per SIMD (128 x 128).
        auto opaque = [](int v) __attribute__((always_inline)) {
            if constexpr (COB * CIB >= 128 * 128) asm volatile("" : "+v"(v));
            return v;
        };
        const int g_here = opaque(g), n16_here = opaque(n16);
        if constexpr (WK > 1) {
            Part* red = reinterpret_cast<Part*>(smem);
            for (int w = 0; w < WK; ++w) {
                if (wk == w) {
#pragma unroll
                    for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                        for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int e = (wco * kTA * 16 + chan(ta, g_here * 4 + j, kTA)) * CIB + wci * kTB * 16 + chan(tb, n16_here, kTB);
                                red[e] = (w == 0 ? (Part)0 : red[e]) + piece_val(ta, tb, j);
                            }
                }
                __syncthreads();
            }
            for (int e = tid * 4; e < COB * CIB; e += kThreads * 4) {
                const int co = e / CIB, ci = e % CIB;
                *reinterpret_cast<Partx4*>(dst + (size_t)(co0 + co) * a.cin + ci0 + ci) = *reinterpret_cast<const Partx4*>(red + e);
            }
        } else {
#pragma unroll
            for (int ta = 0; ta < kTA; ++ta)
#pragma unroll
                for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        dst[(size_t)(co0 + wco * kTA * 16 + chan(ta, g_here * 4 + j, kTA)) * a.cin + ci0 + wci * kTB * 16 +
                            chan(tb, n16_here, kTB)] = piece_val(ta, tb, j);
        }
        __syncthreads();  // the next piece reuses the staging buffers
    }
}

// Plain kernel for channel counts that are not multiples of 16: one thread per weight element.
template <typename T>
__global__ __launch_bounds__(256) void wgrad_plain_kernel(const int32_t* __restrict__ pair_in,
                                                          const int32_t* __restrict__ pair_out,
                                                          const int32_t* __restrict__ koff, int64_t pair_stride,
                                                          const T* __restrict__ X, const T* __restrict__ dY, int cin,
                                                          int cout, float* __restrict__ dw) {
    const int k = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= cin * cout) return;
    const int co = e / cin, ci = e % cin;
    float s = 0.f;
    const int64_t p0 = (int64_t)k * pair_stride;
    for (int64_t p = p0; p < p0 + (koff[k + 1] - koff[k]); ++p)
        s = fmaf(load_f32(dY + (size_t)pair_out[p] * cout + co), load_f32(X + (size_t)pair_in[p] * cin + ci), s);
    dw[(size_t)k * cin * cout + e] = s;
}

template <typename T, int COB, int CIB, int WCO, int WCI, int WK, int kD>
int launch_staged(const sp_kmap* m, const void* x, const void* dy, int cin, int cout, float* dw, hipStream_t s) {
    using Cfg = StagedCfg<T, COB, CIB, WCO, WCI, WK>;
    auto kern = wgrad_staged_kernel<T, COB, CIB, WCO, WCI, WK, kD>;
    static std::mutex mu;  // guards the two one-time queries below
    static bool attr_set = false;  // one-time opt-in to > 64 KB of dynamic LDS
    static int occ = 0;  // workgroups of this kernel that fit a CU: asked once
    {
        std::lock_guard<std::mutex> lk(mu);
        if (!attr_set) {
            SP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)Cfg::kLds));
            attr_set = true;
        }
        if (occ == 0) {
            int q = 1;
            SP_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&q, kern, Cfg::kThreads, Cfg::kLds));
            occ = q < 1 ? 1 : q;
        }
    }
    const int kvol = m->kvol, per = cin * cout;
    StagedArgs a;
    PlanArgs& pa = a.plan;
    pa.kvol = kvol;
    pa.pair_stride = (int)m->pair_stride;
    pa.tiles = (cout / COB) * (cin / CIB);
    for (int k = 0; k <= kvol; ++k) pa.koff[k] = (int32_t)m->koff[k];
    // Strips: one per XCD.  (More strips, sized so that a strip's rows fit an XCD's L2, were measured slower on
    // every workload, 4-19 %: each strip adds one partial block per offset, and the rows' L2 hits did not pay for
    // that traffic.  Fewer than one per XCD, with the chunks dealt to the XCDs in turn, were 1-12 % slower too.)
    pa.S8 = 8;
    // Chunks (one workgroup each): exactly as many as workgroups are resident together, so the launch is one
    // round of equal chunks whatever the size of the map.  A chunk costs a partial block (per * 4 or 8 bytes written
    // and read again) and a pipeline fill; shorter chunks in several rounds were measured slower throughout
    // (2048-link chunks: +10 % on 11.5 M links, +30 % on 5 M links of 64 -> 64 fp32).
    const int64_t strip_links = (m->total + pa.S8 - 1) / pa.S8 + kvol;  // upper bound of a strip's sequence
    const int64_t resident = std::max<int64_t>(pa.S8, (int64_t)256 * occ / pa.tiles);
    const int64_t nc = resident / pa.S8;  // chunks per strip
    int64_t C = (strip_links + nc - 1) / nc;
    C = (C + Cfg::kS - 1) / Cfg::kS * Cfg::kS;
    pa.nc = (int)nc;
    pa.C = (int)C;
    pa.slots_per_strip = (int)nc + kvol;
    const int64_t slots = (int64_t)pa.S8 * pa.slots_per_strip;
    Buf part = dev_alloc((size_t)slots * per * Cfg::kPartElt, s);
    Buf tabs = dev_alloc((size_t)2 * pa.S8 * kvol * 4, s);
    if (!part || !tabs) return SP_ERR_ALLOC;
    a.first = ptr<int32_t>(tabs);
    a.count = a.first + (size_t)pa.S8 * kvol;
    a.pair_in = ptr<int32_t>(m->pair_in);
    a.pair_out = ptr<int32_t>(m->pair_out);
    a.x = x;
    a.dy = dy;
    a.part = part->p;
    a.cin = cin;
    a.cout = cout;
    a.x_bytes = (uint32_t)((uint64_t)m->n_in * cin * sizeof(T));
    a.dy_bytes = (uint32_t)((uint64_t)m->n_out * cout * sizeof(T));
    a.pair_bytes = (uint32_t)((uint64_t)kvol * m->pair_stride * 4);
    const int64_t wgs = (int64_t)pa.S8 * nc * pa.tiles;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(Cfg::kThreads), Cfg::kLds, s, a);
    if constexpr (Cfg::kIsF32)
        hipLaunchKernelGGL(wgrad_reduce_kernel<double>, dim3(per / 64, kvol), dim3(256), 0, s, ptr<double>(part), a.first,
                           a.count, pa.S8, kvol, per, dw);
    else
        hipLaunchKernelGGL(wgrad_reduce_kernel<float>, dim3(per / 64, kvol), dim3(256), 0, s, ptr<float>(part), a.first,
                           a.count, pa.S8, kvol, per, dw);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// largest of 128, 64, 32, 16 dividing c (c is a multiple of 16)
int channel_block(int c) { return c % 128 == 0 ? 128 : (c % 64 == 0 ? 64 : (c % 32 == 0 ? 32 : 16)); }

template <typename T>
int wgrad_typed(const sp_kmap* m, const void* x, const void* dy, float* dw, int cin, int cout, hipStream_t s) {
    const int kvol = m->kvol;
    const uint64_t lim = 0x7fffffffull;  // the staged kernel addresses its buffers with 32-bit offsets
    const bool small = (uint64_t)m->n_in * cin * sizeof(T) < lim && (uint64_t)m->n_out * cout * sizeof(T) < lim &&
                       (uint64_t)kvol * m->pair_stride * 4 < lim;
    if (cin % 16 || cout % 16 || !small || m->total == 0 || kvol > 128) {
        hipLaunchKernelGGL(wgrad_plain_kernel<T>, dim3((cin * cout + 255) / 256, kvol), dim3(256), 0, s,
                           ptr<int32_t>(m->pair_in), ptr<int32_t>(m->pair_out), ptr<int32_t>(m->d_koff), m->pair_stride,
                           static_cast<const T*>(x), static_cast<const T*>(dy), cin, cout, dw);
        SP_HIP(hipGetLastError());
        return SP_OK;
    }
    int cob = channel_block(cout), cib = channel_block(cin);
    if (cob == 128 && cib < 64) cob = 64;  // 128-wide tiles only in the combinations instantiated below
    if (cib == 128 && cob < 64) cib = 64;
    // register stages of gathered rows: two for bf16 (a step's arithmetic is short next to the gather latency)
    constexpr int kD = sizeof(T) == 2 ? 2 : 1;
#define SP_STAGED(COB, CIB, WCO, WCI, WK) \
    if (cob == COB && cib == CIB) return launch_staged<T, COB, CIB, WCO, WCI, WK, kD>(m, x, dy, cin, cout, dw, s)
    if constexpr (sizeof(T) == 2) {  // bf16: the whole 256 x 256 matrix in one workgroup, every row gathered once
        if (cout % 256 == 0 && cin % 256 == 0) return launch_staged<T, 256, 256, 2, 4, 1, 1>(m, x, dy, cin, cout, dw, s);
    }
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
    return fail(SP_ERR_UNSUPPORTED, "no weight-gradient kernel for %d x %d channels", cout, cin);
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
    SP_TRY(kmap_resolve(m));  // sizes of a map whose build has not reported yet
    if (cin < 1 || cout < 1 || cin > 4096 || cout > 4096) return fail(SP_ERR_INVALID_ARG, "bad channel count");
    if (dt != SP_F32 && dt != SP_BF16) return fail(SP_ERR_INVALID_ARG, "bad dtype");
    if ((!d_x && m->n_in > 0) || (!d_dy && m->n_out > 0) || !d_dw)
        return fail(SP_ERR_INVALID_ARG, "a feature/gradient pointer is NULL");
    if ((((uintptr_t)d_x | (uintptr_t)d_dy | (uintptr_t)d_dw) & 15) != 0)
        return fail(SP_ERR_INVALID_ARG, "feature/gradient pointers must be 16-byte aligned");
    return conv_wgrad(m, d_x, d_dy, d_dw, cin, cout, dt, (hipStream_t)stream);
}
