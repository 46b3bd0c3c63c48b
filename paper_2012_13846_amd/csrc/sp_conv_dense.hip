// Step 3 of the generalized sparse convolution (Eq. 2) for wide bf16 layers on dense-ish maps: a
// destination-row-stationary kernel whose accumulators never leave the registers.
//
// A workgroup owns 256 destination rows and 128 destination channels.  For every kernel offset it reads the
// rows' neighbour table entries, gathers the neighbours' feature rows (zeros where an offset has no
// neighbour) and the offset's weight matrix through LDS in slices of 64 contraction channels, and
// multiplies on the bf16 matrix cores: acc[row][co] += X[nbr_k(row)][:] . W_k[co][:].  Rows without a
// neighbour multiply zeros, so the kernel pays for all kvol offsets of every row: it is chosen only when a
// good part of them is there (the host decides from the map's link count), where it wins because bf16 MFMA
// throughput is 16 times the fp32 one while this form needs no per-link bookkeeping, no scatter and no
// accumulator traffic.  Each destination row belongs to one workgroup and the offsets are added in index
// order: no atomics, reproducible, rounded once.
#include <mutex>

#include "sp_internal.h"

namespace sp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint16_t bf16_t;

__device__ __forceinline__ uint32_t bf16_bits(float f) {  // nearest-even rounding; NaN stays NaN
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// acc += A * B in place.  Written as an instruction because the compiler, given the builtin and this much
// register pressure, gives the products fresh registers and copies all 128 accumulators around at the loop's
// back edge; the tied operand keeps every accumulator in one AGPR quad for the whole kernel.
__device__ __forceinline__ void mfma_acc(f32x4& acc, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

struct DenseArgs {
    const int32_t* nbr;  // [kvol][n_rows] source row or -1
    const void* f;       // source features [n_src][CC] bf16
    const void* w;       // weights [kvol][co_total][CC] bf16
    void* g;             // destination features [n_rows][co_total] bf16
    int64_t n_rows;
    int kvol, co_total, flip;
    uint32_t f_bytes, w_bytes, nbr_bytes;
    const int32_t* perm;        // null, or the order in which the destination rows are taken (tile = 256 entries)
    const uint32_t* tile_mask;  // null, or per tile 4 words: the offsets that link any of its rows
};

// CC contraction channels, COT destination channels per workgroup (64, 128: 4 wavefronts; 256: 8), KS
// contraction channels per step (64 or 32).
template <int CC, int COT, int KS>
struct DenseCfg {
    static constexpr int kTR = 256;                  // destination rows per workgroup
    static constexpr int kKS = KS;
    static constexpr int kRowBytes = KS * 2;         // one staged slice row: 128 or 64 bytes
    static constexpr int kP = kRowBytes / 16;        // 16-byte pieces per staged row
    static constexpr int kKSteps = KS / 32;          // MFMA k-steps per slice
    static constexpr int kWaves = COT == 256 ? 8 : 4;  // 4 row quarters x (COT == 256: 2 channel halves)
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kXBytes = kTR * kRowBytes, kWBytes = COT * kRowBytes, kBuf = kXBytes + kWBytes;
    static constexpr int kSlices = CC / kKS;
    static constexpr int kRP = kThreads / kP;        // rows loaded per pass: kP lanes per row
    static constexpr int kXLoads = kTR / kRP;        // 16-byte pieces per thread and step
    static constexpr int kWLoads = COT / kRP;
    static constexpr int kWDepth = kWaves > 4 ? 1 : 2;  // register stages of the weight slices (the rows always have 2)
    // Weight fragments in flight per wavefront.  With 8 wavefronts and four slices per offset (CC = 256) a third one
    // makes the compiler spill, and a reload inside the loop waits for every gather in flight (loads return in
    // order), which undoes the rows' second register stage.
    static constexpr int kWF = (kWaves > 4 && CC == 256) ? 2 : 3;
    static constexpr int kOutPitch = COT * 2 + 16;   // output staging row (bf16)
    static constexpr int kLds = 2 * kBuf > kTR * kOutPitch ? 2 * kBuf : kTR * kOutPitch;
    static constexpr int kMI = 4;                    // 16-row groups per wavefront: 64 rows
    static constexpr int kNI = COT == 64 ? 4 : 8;    // 16-channel tiles per wavefront: 64 or 128 channels
    static_assert(CC % kKS == 0, "whole slices");
    static_assert(COT == 64 || COT == 128 || COT == 256, "channel slice");
    static_assert(KS == 64 || KS == 32, "slice width");
    static_assert(COT % kRP == 0 && kTR % kRP == 0, "whole loads per thread");
};

// Staged rows have no pad; the 16-byte piece p of row r sits in slot p ^ f(r), f(r) = (r >> 1) & 7 for 128-byte
// rows and (r >> 2) & 3 for 64-byte rows (rows that share a bank range get different slots).  With this swizzle
// the b128 fragment reads (16 rows x 4 k-groups per wavefront) run at the full LDS rate, like a 32-byte pad
// would, and the buffers stay small enough for 8 wavefronts' worth of tile.
template <int P>
__device__ __forceinline__ int swz(int row, int piece) {
    return (P == 8 ? (piece ^ ((row >> 1) & 7)) : (piece ^ ((row >> 2) & 3))) * 16;
}

template <int COT>
constexpr int kDenseThreads = COT == 256 ? 512 : 256;

template <int CC, int COT, int KS>
__global__ __launch_bounds__(kDenseThreads<COT>, (KS == 32 ? 2 : 1)) void gather_dense_kernel(DenseArgs a) {
    using Cfg = DenseCfg<CC, COT, KS>;
    constexpr int kMI = Cfg::kMI, kNI = Cfg::kNI, kSlices = Cfg::kSlices, kRP = Cfg::kRP, kP = Cfg::kP;
    constexpr int kRowBytes = Cfg::kRowBytes, kKSteps = Cfg::kKSteps;
    constexpr int kXLoads = Cfg::kXLoads, kWLoads = Cfg::kWLoads, kWDepth = Cfg::kWDepth;
    extern __shared__ __align__(16) unsigned char smem[];

    // Workgroups of one row tile (one per channel slice) get ids that differ by 8: same XCD (id % 8), launched
    // back to back, so the second one's gathers hit that XCD's L2.
    const int nslice = a.co_total / COT;
    const int id = blockIdx.x;
    const int64_t tile = (int64_t)(id / (8 * nslice)) * 8 + id % 8;
    const int co0 = ((id / 8) % nslice) * COT;
    const int64_t row0 = tile * Cfg::kTR;  // first entry of the tile (in perm order if there is one)
    if (row0 >= a.n_rows) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int rq = wave & 3, ch = wave >> 2;  // this wavefront: tile rows rq*64 .. +63, slice channels ch*128 .. (+127 | +63)

    constexpr int kRsrcFlags = 0x00020000;
    constexpr uint32_t kOutside = 0x80000000u;  // buffers are smaller than 2 GiB: this offset reads as zeros
    const __amdgpu_buffer_rsrc_t rF = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.f), 0, (int)a.f_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.w), 0, (int)a.w_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rN =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(a.nbr), 0, (int)a.nbr_bytes, kRsrcFlags);

    // Loading: kP adjacent lanes fetch the pieces of one slice row; thread t takes piece t % kP of the tile
    // rows t / kP + kRP j and of the weight rows (destination channels) t / kP + kRP j.
    const int piece = tid % kP, lrow = tid / kP;
    const int st_off = lrow * kRowBytes + swz<kP>(lrow, piece);  // + kRP j rows: kRP is a multiple of 16, the swizzle stays
    // Per offset and thread: the byte offsets of its kXLoads source rows (kOutside where the row has no
    // neighbour: such a load returns zeros) and of its first weight row.  A step's loads then differ from
    // these only by constants, which ride in the instruction's scalar offset.
    struct Where {
        uint32_t x[kXLoads], w;
    };
    // destination rows this thread gathers for: entry row0 + lrow + kRP j of the tile, -1 past the end
    int my_row[kXLoads];
#pragma unroll
    for (int j = 0; j < kXLoads; ++j) {
        const int64_t e = row0 + lrow + kRP * j;
        my_row[j] = e < a.n_rows ? (a.perm ? a.perm[e] : (int)e) : -1;
    }
    auto load_nbr = [&](int k, int (&raw)[kXLoads]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kXLoads; ++j) {
            const bool live = my_row[j] >= 0 && k < a.kvol;
            // past the table the load returns 0, which would name row 0: such entries are masked in locate()
            raw[j] = (int)__builtin_amdgcn_raw_buffer_load_b32(
                rN, live ? (uint32_t)(((int64_t)k * a.n_rows + my_row[j]) * 4) : kOutside, 0, 0);
        }
    };
    auto locate = [&](int k, const int (&raw)[kXLoads], Where& wh) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kXLoads; ++j) {
            const bool live = my_row[j] >= 0 && k < a.kvol && raw[j] >= 0;
            wh.x[j] = live ? (uint32_t)raw[j] * (CC * 2) + piece * 16 : kOutside;
        }
        const int wk = a.flip ? a.kvol - 1 - k : k;
        wh.w = k < a.kvol ? ((uint32_t)wk * a.co_total + co0 + lrow) * (CC * 2) + piece * 16 : kOutside;
    };
    auto load_x = [&](u32x4 (&x)[kXLoads], int j, int s, const Where& wh) __attribute__((always_inline)) {
        x[j] = __builtin_amdgcn_raw_buffer_load_b128(rF, wh.x[j], s * kRowBytes, 0);
    };
    auto load_w = [&](u32x4 (&w)[kWLoads], int j, int s, const Where& wh) __attribute__((always_inline)) {
        w[j] = __builtin_amdgcn_raw_buffer_load_b128(rW, wh.w, j * kRP * (CC * 2) + s * kRowBytes, 0);
    };
    auto store_x = [&](const u32x4 (&x)[kXLoads], int j, unsigned char* buf) __attribute__((always_inline)) {
        *reinterpret_cast<u32x4*>(buf + st_off + j * kRP * kRowBytes) = x[j];
    };
    auto store_w = [&](const u32x4 (&w)[kWLoads], int j, unsigned char* buf) __attribute__((always_inline)) {
        *reinterpret_cast<u32x4*>(buf + Cfg::kXBytes + st_off + j * kRP * kRowBytes) = w[j];
    };
    // acc[ni][mi][i]: destination channel co0 + ch*128 + ni*16 + 4*g + i, tile row rq*64 + mi*16 + n16
    // (weights are the MFMA A operand, the gathered rows the B operand: a lane ends up with 4 adjacent channels
    // of one row, which pack into one 8-byte store)
    f32x4 acc[kNI][kMI];
#pragma unroll
    for (int ni = 0; ni < kNI; ++ni)
#pragma unroll
        for (int mi = 0; mi < kMI; ++mi) acc[ni][mi] = f32x4{0.f, 0.f, 0.f, 0.f};
    // fragment of (row n16 of a 16-row group, k-group g) for the two k-steps; + 16-row groups as constants
    // (for 64-byte rows there is one k-step and the second entries are not used)
    const int frag_x[2] = {(rq * 64 + n16) * kRowBytes + swz<kP>(n16, g),
                           (rq * 64 + n16) * kRowBytes + swz<kP>(n16, (4 + g) % kP)};
    const int frag_w[2] = {Cfg::kXBytes + (ch * 128 + n16) * kRowBytes + swz<kP>(n16, g),
                           Cfg::kXBytes + (ch * 128 + n16) * kRowBytes + swz<kP>(n16, (4 + g) % kP)};
    // One step = kKSteps k-steps x kNI channel tiles = kGroups groups of kMI MFMAs.  A wavefront issues in order
    // and an MFMA runs for 16 cycles once issued, so everything else the step has to do is dealt out over the
    // groups and issued in the shadow of their MFMAs: the LDS fragment reads (kWF - 1 groups ahead of their
    // use: kWF rotating weight fragments; the second k-step's row fragments during the first k-step), the
    // global loads of later steps and the LDS stores of the next step's stage, kPerGroup of each per group.
    constexpr int kGroups = kKSteps * kNI;
    constexpr int kLoads = kXLoads + kWLoads;
    constexpr int kPerGroup = (kLoads + kGroups - 1) / kGroups;
    auto compute = [&](const unsigned char* buf, auto&& extra) __attribute__((always_inline)) {
        constexpr int kWF = Cfg::kWF;
        bf16x8 xf[kKSteps][kMI], wf[kWF];
        auto read_w = [&](int grp) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8*>(buf + frag_w[grp / kNI] + (grp % kNI) * 16 * kRowBytes);
        };
        auto read_x = [&](int ks, int mi) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8*>(buf + frag_x[ks] + mi * 16 * kRowBytes);
        };
#pragma unroll
        for (int mi = 0; mi < kMI; ++mi) xf[0][mi] = read_x(0, mi);
#pragma unroll
        for (int i = 0; i < kWF - 1; ++i) wf[i] = read_w(i);
#pragma unroll
        for (int grp = 0; grp < kGroups; ++grp) {
            if (grp + kWF - 1 < kGroups) wf[(grp + kWF - 1) % kWF] = read_w(grp + kWF - 1);
            if (kKSteps == 2 && grp >= 1 && grp <= kMI) xf[kKSteps - 1][grp - 1] = read_x(1, grp - 1);
#pragma unroll
            for (int e = 0; e < kPerGroup; ++e) extra(grp * kPerGroup + e);
            __builtin_amdgcn_sched_barrier(0);  // keeps this group's other work ahead of the MFMAs that hide it
#pragma unroll
            for (int mi = 0; mi < kMI; ++mi) mfma_acc(acc[grp % kNI][mi], wf[grp % kWF], xf[grp / kNI][mi]);
        }
    };

    // The loop runs over "turns" of kRS = 2, 4 or 8 steps.  Normally a turn is one offset and its steps are
    // the offset's slices; when an offset is a single slice, a turn is two offsets, one step each (the sum
    // over offsets and the sum over channels are one contraction, so a step is just more columns of it).
    // Step j of a turn works out of LDS buffer j % 2.  The gathered rows have two register stages (they mostly
    // miss L2, and one step of arithmetic is shorter than that latency): during a step the rows of the step two
    // ahead are requested and those of the next step are stored to the other buffer.  The weight slices (L2
    // hits) have kWDepth stages.  The neighbour entries are requested two turns ahead.
    constexpr int kSPO = kSlices;                   // slices per offset: 1, 2 or 4
    constexpr int kOPR = kSPO == 1 ? 2 : 1;         // offsets per turn
    constexpr int kRS = kSPO * kOPR;                // steps per turn
    static_assert(kRS % 2 == 0, "the register stage and LDS buffer of a step are its index in the turn % 2");
    // The offsets to visit, ascending: all of them, or those of the tile's mask.  next_offset() hands them out
    // one by one and then kvol (for which every load reads zeros) for ever.
    // (Four named words, not an array: an array here ends up in scratch memory, and each read of it then makes
    // the wavefront wait for every gather it has in flight.)
    auto mask_word = [&](int i) __attribute__((always_inline)) {
        const int n = a.kvol - 32 * i;
        uint32_t all = n >= 32 ? 0xffffffffu : (n > 0 ? (1u << n) - 1u : 0u);
        if (a.tile_mask) all &= a.tile_mask[tile * 4 + i];
        return (uint32_t)__builtin_amdgcn_readfirstlane(all);
    };
    uint32_t todo0 = mask_word(0), todo1 = mask_word(1), todo2 = mask_word(2), todo3 = mask_word(3);
    auto next_offset = [&]() __attribute__((always_inline)) {
        // every word is assigned on every call (a store under a condition would bring the memory form back)
        const bool u0 = todo0 != 0, u1 = !u0 && todo1 != 0, u2 = !u0 && !u1 && todo2 != 0,
                   u3 = !u0 && !u1 && !u2 && todo3 != 0;
        const int k = u0 ? __builtin_ctz(todo0)
                         : (u1 ? 32 + __builtin_ctz(todo1)
                               : (u2 ? 64 + __builtin_ctz(todo2) : (u3 ? 96 + __builtin_ctz(todo3) : a.kvol)));
        todo0 = u0 ? (todo0 & (todo0 - 1)) : todo0;
        todo1 = u1 ? (todo1 & (todo1 - 1)) : todo1;
        todo2 = u2 ? (todo2 & (todo2 - 1)) : todo2;
        todo3 = u3 ? (todo3 & (todo3 - 1)) : todo3;
        return k;
    };
    Where cur[kOPR], nxt[kOPR];  // the offsets of this turn and of the next
    int k_cur[kOPR];             // this turn's offsets (kvol: none left)
    int raw[kOPR][kXLoads];      // neighbour entries of the turn after that, in flight
    int k_raw[kOPR];
#pragma unroll
    for (int o = 0; o < kOPR; ++o) {
        k_cur[o] = next_offset();
        load_nbr(k_cur[o], raw[o]);
        locate(k_cur[o], raw[o], cur[o]);
    }
    int k_nxt[kOPR];
#pragma unroll
    for (int o = 0; o < kOPR; ++o) {
        k_nxt[o] = next_offset();
        load_nbr(k_nxt[o], raw[o]);
        locate(k_nxt[o], raw[o], nxt[o]);
    }
#pragma unroll
    for (int o = 0; o < kOPR; ++o) {
        k_raw[o] = next_offset();
        load_nbr(k_raw[o], raw[o]);
    }
    // step j of this turn (j < kRS) or of the next (j >= kRS): its offset's addresses and its slice
    auto where_of = [&](int j) -> const Where& { return j < kRS ? cur[j / kSPO] : nxt[(j - kRS) / kSPO]; };
    auto advance_turn = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int o = 0; o < kOPR; ++o) {
            cur[o] = nxt[o];
            k_cur[o] = k_nxt[o];
            k_nxt[o] = k_raw[o];
            locate(k_nxt[o], raw[o], nxt[o]);
            k_raw[o] = next_offset();
            load_nbr(k_raw[o], raw[o]);
        }
    };
    u32x4 sx[2][kXLoads], sw[kWDepth][kWLoads];
#pragma unroll
    for (int j = 0; j < kXLoads; ++j) load_x(sx[0], j, 0, where_of(0));
#pragma unroll
    for (int j = 0; j < kWLoads; ++j) load_w(sw[0], j, 0, where_of(0));
#pragma unroll
    for (int j = 0; j < kXLoads; ++j) load_x(sx[1], j, 1 % kSPO, where_of(1));
    if constexpr (kWDepth == 2) {
#pragma unroll
        for (int j = 0; j < kWLoads; ++j) load_w(sw[1], j, 1 % kSPO, where_of(1));
    }
#pragma unroll
    for (int j = 0; j < kXLoads; ++j) store_x(sx[0], j, smem);
#pragma unroll
    for (int j = 0; j < kWLoads; ++j) store_w(sw[0], j, smem);
    __syncthreads();
    while (k_cur[0] < a.kvol) {
#pragma unroll
        for (int s = 0; s < kRS; ++s) {
            compute(smem + (s % 2) * Cfg::kBuf, [&](int slot) __attribute__((always_inline)) {
                // slot = 0 .. kGroups * kPerGroup - 1.  Requests: weight slice of the step kWDepth ahead, then
                // the rows of the step 2 ahead
                if (slot < kWLoads) {
                    constexpr int d = kWDepth;
                    load_w(sw[(s + d) % kWDepth], slot, (s + d) % kSPO, where_of(s + d));
                } else if (slot < kLoads) {
                    load_x(sx[s % 2], slot - kWLoads, (s + 2) % kSPO, where_of(s + 2));
                }
                // stores of the next step's stage in the last slots: rows first (requested a step ago), weights last
                const int st = slot - (kGroups * kPerGroup - kLoads);
                unsigned char* other = smem + ((s + 1) % 2) * Cfg::kBuf;
                if (st >= 0 && st < kXLoads) store_x(sx[(s + 1) % 2], st, other);
                else if (st >= kXLoads) store_w(sw[(s + 1) % kWDepth], st - kXLoads, other);
            });
            __syncthreads();
        }
        advance_turn();
    }

    // the accumulators are read below by ordinary instructions: the MFMAs were written as opaque instructions,
    // so the wait states between the last of them and the first read are put in by hand (18 are required)
    asm volatile("s_nop 15\n s_nop 15" ::: "memory");
    // one rounding to bf16, stage the tile in LDS, write whole rows
    unsigned char* out = smem;  // all staging reads are behind the last barrier
#pragma unroll
    for (int ni = 0; ni < kNI; ++ni)
#pragma unroll
        for (int mi = 0; mi < kMI; ++mi) {
            const f32x4 v = acc[ni][mi];
            u32x2 p;
            p[0] = bf16_bits(v[0]) | (bf16_bits(v[1]) << 16);
            p[1] = bf16_bits(v[2]) | (bf16_bits(v[3]) << 16);
            *reinterpret_cast<u32x2*>(out + (rq * 64 + mi * 16 + n16) * Cfg::kOutPitch + (ch * 128 + ni * 16 + 4 * g) * 2) = p;
        }
    __syncthreads();
    constexpr int kRowPieces = COT * 2 / 16;
    for (int idx = tid; idx < Cfg::kTR * kRowPieces; idx += Cfg::kThreads) {
        const int r = idx / kRowPieces, pc = idx % kRowPieces;
        if (row0 + r >= a.n_rows) break;
        const int64_t row = a.perm ? a.perm[row0 + r] : row0 + r;
        *reinterpret_cast<u32x4*>(static_cast<unsigned char*>(a.g) + ((size_t)row * a.co_total + co0) * 2 + pc * 16) =
            *reinterpret_cast<const u32x4*>(out + r * Cfg::kOutPitch + pc * 16);
    }
}

template <int CC, int COT, int KS>
int launch_dense(const DenseArgs& a, hipStream_t s) {
    using Cfg = DenseCfg<CC, COT, KS>;
    auto kern = gather_dense_kernel<CC, COT, KS>;
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
    const int64_t ntiles = (a.n_rows + Cfg::kTR - 1) / Cfg::kTR;
    const int nslice = a.co_total / COT;
    const int64_t wgs = (ntiles + 7) / 8 * 8 * nslice;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(Cfg::kThreads), Cfg::kLds, s, a);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

}  // namespace

// Cin = 64: its steps hold little arithmetic next to the gather latency, so it only beats the link-list
// kernel on well-filled maps (see dense_min_fill).
bool dense_shape_ok(int cc, int co, sp_dtype dt) {
    return dt == SP_BF16 && (cc == 64 || cc == 128 || cc == 256) && co % 64 == 0;
}
// smallest links / (rows * kvol) from which the row-stationary kernel is the faster one (measured)
double dense_min_fill(int cc) { return cc == 64 ? 0.25 : 0.06; }

// d_w: [kvol][co][cc] (contraction index fastest).  Buffers must be smaller than 2 GiB.
int conv_gather_dense(const MapSide& side, int kvol, const void* d_f, const void* d_w, void* d_g, int cc, int co,
                      hipStream_t s) {
    DenseArgs a;
    a.nbr = ptr<int32_t>(side.nbr);
    a.f = d_f;
    a.w = d_w;
    a.g = d_g;
    a.n_rows = side.n_rows;
    a.kvol = kvol;
    a.co_total = co;
    a.flip = side.flip ? 1 : 0;
    a.f_bytes = (uint32_t)((uint64_t)side.n_src * cc * 2);
    a.w_bytes = (uint32_t)((uint64_t)kvol * co * cc * 2);
    a.nbr_bytes = (uint32_t)((uint64_t)kvol * side.n_rows * 4);
    a.perm = ptr<int32_t>(side.perm);
    a.tile_mask = ptr<uint32_t>(side.tile_mask);
    const int cot = co % 256 == 0 ? 256 : (co % 128 == 0 ? 128 : 64);
#define SP_DENSE(CC, COT, KS) \
    if (cc == CC && cot == COT) return launch_dense<CC, COT, KS>(a, s)
    // 8 wavefronts: 64-channel slices.  4 wavefronts: 32-channel slices, which halve the LDS buffers and the
    // staged registers so that two workgroups share a CU (measured 13-15 % faster than 64-channel slices)
    SP_DENSE(256, 256, 64);
    SP_DENSE(256, 128, 32);
    SP_DENSE(256, 64, 32);
    SP_DENSE(128, 256, 64);
    SP_DENSE(128, 128, 32);
    SP_DENSE(128, 64, 32);
    SP_DENSE(64, 256, 64);
    SP_DENSE(64, 128, 32);
    SP_DENSE(64, 64, 32);
#undef SP_DENSE
    return fail(SP_ERR_UNSUPPORTED, "no row-stationary kernel for %d -> %d channels", cc, co);
}

}  // namespace sp
