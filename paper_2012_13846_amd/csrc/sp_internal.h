// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <functional>
#include <memory>
#include <mutex>
#include <vector>

#include "sp_conv.h"

namespace sp {

// ---- errors -------------------------------------------------------------------------------------------
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);

#define SP_HIP(call)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess) return sp::fail(SP_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define SP_TRY(expr)              \
    do {                          \
        int rc_ = (expr);         \
        if (rc_ != SP_OK) return rc_; \
    } while (0)

// ---- device memory: size-class caching pool, or the caller's allocator (sp_set_allocator) ------------------
// A block remembers the stream it was allocated for; all work that touches it is enqueued on that stream
// (one handle = one stream is the documented contract).  When the last owner drops it, the pool keeps it
// with that stream: the next allocation for the same stream takes it at once, an allocation for another
// stream first makes its stream wait for the old one (see sp_runtime.hip).
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    hipStream_t stream = nullptr;
    sp_free_fn free_ = nullptr;  // set when the block came from the caller's allocator
    void* ctx = nullptr;
    ~DevBuf();
};
using Buf = std::shared_ptr<DevBuf>;
// nullptr (and error set) on failure; bytes == 0 gives a valid tiny block.  s: the stream the block is used on.
Buf dev_alloc(size_t bytes, hipStream_t s);
template <class T>
inline T* ptr(const Buf& b) { return b ? static_cast<T*>(b->p) : nullptr; }
int pool_trim();
int64_t pool_bytes();
int64_t pool_cross_stream();

// Pinned host staging area for small read-backs (one per process, guarded by a mutex inside).
// Blocks until `bytes` at d_src, as of everything enqueued on s so far, are in h_dst.  `then_enqueue`, if given,
// is called once the read-back itself is enqueued and before the host starts waiting: work that the caller
// wants on the stream but whose result the host does not need runs while the host wakes up.
int read_back(void* h_dst, const void* d_src, size_t bytes, hipStream_t s,
              const std::function<void()>& then_enqueue = nullptr);

// ---- mail slots (sp_runtime.hip): counts that a build's last kernel writes into pinned host memory ----------------
constexpr int kMailSlots = 2048;      // builds whose counts nobody has asked for yet
constexpr int kMailSlotWords = 256;   // 1 KB a slot: payload words, then the sequence word
constexpr int kMailSeqWord = kMailSlotWords - 1;
struct MailSlot {
    int index = -1;         // -1: none held
    uint32_t* h = nullptr;  // host view
    uint32_t* d = nullptr;  // device view of the same memory
    uint32_t seq = 0;       // the value the kernel writes to word kMailSeqWord when the payload is complete
    bool armed = false;     // the kernel that will write the slot has been enqueued (on `stream`)
    hipStream_t stream = nullptr;
};
bool mail_acquire(MailSlot* out);                  // false: none free (the caller then waits for its stream instead)
// Gives the slot back.  A slot whose kernel is enqueued but has not delivered yet (a handle destroyed before its
// counts were asked for) is parked and only reused once the delivery, or the end of its stream's work, is seen:
// a late write must not land in a slot that another build already owns.
void mail_release(MailSlot* slot);
int mail_wait(const MailSlot& slot, hipStream_t s);  // blocks until the slot's payload has arrived

// ---- hash table ---------------------------------------------------------------------------------------------
struct HashTab {
    Buf slots;         // HashSlot [cap] (sp_hash.h): 16 bytes {key, first source row, row number}
    uint32_t cap = 0;  // power of two, >= 2 * entries
    int zshift = 0;    // floor(log2(tensor stride)): see sp_hash.h
};

// ---- coords (sp_coords.hip) ---------------------------------------------------------------------------------------
// Builds a coordinate set from d_src rows; floor_step > 1 floors x,y,z to multiples of it first.  n_src_ub is an
// upper bound of the row count (sizes every allocation and grid); d_n_src, if not null, points at the true count
// in device memory (a count that the host has not seen yet), else the count is n_src_ub.  Does not wait.
int coords_build_impl(const int32_t* d_src, int64_t n_src_ub, const int32_t* d_n_src, int32_t floor_step,
                      int32_t tensor_stride, hipStream_t s, sp_coords_t** out);
// Waits (first call only) until the handle's row count has come back; reports device-detected errors.
int coords_resolve(const sp_coords_t* c);
int kmap_resolve(const sp_kmap_t* m);

constexpr int kTileRows = 256;   // rows per tile of the tile lists (= map-build block size)
constexpr int kSubTiles = 4;     // 64-row sub-tiles (one wavefront ballot each) per tile
constexpr int kHalves = 2;       // list offsets are kept per 32-row half of a sub-tile

}  // namespace sp

// Words of a coordinate set's device-side `meta` block (int32)
enum { kMetaN = 0, kMetaErr = 1, kMetaWords = 4 };

struct sp_coords {
    std::atomic<int> ref{1};
    int64_t n_raw = 0;   // source rows (an upper bound of them when the set was derived from an unresolved one)
    int32_t ts = 1;
    sp::Buf coords;   // int32 [n][4] (allocated for n_raw rows)
    sp::Buf inverse;  // int32 [n_raw]
    sp::Buf meta;     // int32 [kMetaWords]: the row count n, error bits, ...: what kernels of later builds read
    sp::HashTab tab;
    hipStream_t stream = nullptr;
    // the host's copy of n arrives through a mail slot and is read on first demand (coords_resolve)
    mutable std::mutex mu;
    mutable bool resolved = false;
    mutable int status = 0;       // SP_OK or the device-detected error, once resolved
    mutable int64_t n = -1;
    mutable sp::MailSlot mail;
    sp_coords* src_of = nullptr;  // set on a coarser set derived from another: the set whose rows were its source rows (reference held)
    ~sp_coords();
};

namespace sp {

// One direction of a kernel map, as the gather-GEMM kernel consumes it: `n_rows` destination rows in tiles
// of kTileRows; for (64-row sub-tile u, offset k, 32-row half h) the entries [off[(u*kvol+k)*2+h], off[(u*kvol+k)*2+h+1])
// of src/row list the live (source row, destination row within the tile) links, destination rows ascending.
struct MapSide {
    int64_t n_rows = 0, n_src = 0;
    Buf nbr;      // int32 [kvol][n_rows]: source row or -1
    Buf tl_off;   // int32 [nsub*kvol*2 + 1], nsub = 4*ntiles, index (sub*kvol + k)*2 + half (sub-tile-major)
    Buf tl_src;   // int32 [total]
    Buf tl_row;   // uint16 [total]
    bool flip = false;  // weight offset index = kvol-1-k (side derived by the stride-1 symmetry)
    // Input side of a strided map only: which offsets can link an input row depends on the row's position inside
    // its coarse cell (stride 2, K = 3: 1 to 8 of the 27).  `perm` lists the rows sorted by that position class
    // and `tile_mask` holds, per 256 entries of perm, the offsets that link at least one of them (4 words, bit k
    // of word k/32), so that a row-stationary kernel walking perm skips the other offsets of a tile.
    Buf perm;       // int32 [n_rows] or null
    Buf tile_mask;  // uint32 [ceil(n_rows/256)][4] or null
};

}  // namespace sp

struct sp_kmap {
    // Host copies of the sizes: valid once resolved (kmap_resolve); the kernels of the build read them from
    // device memory instead.
    mutable int64_t n_in = 0, n_out = 0, total = 0;
    int32_t K = 0, kvol = 0, stride = 1, dilation = 1;
    mutable sp::MapSide out_side;  // destinations = output rows, sources = input rows   (forward)
    mutable sp::MapSide in_side;   // destinations = input rows,  sources = output rows  (data gradient)
    sp::Buf pair_in, pair_out;  // int32 [kvol][pair_stride]: offset k's pairs are the first counts[k] entries of row k
    int64_t pair_stride = 0;
    mutable std::vector<int64_t> counts;   // [kvol]
    mutable std::vector<int64_t> koff;     // [kvol+1] exclusive prefix of counts
    sp::Buf d_koff;                // int32 [kvol+1], the same prefix on the device
    sp_coords* c_in = nullptr;     // references held
    sp_coords* c_out = nullptr;
    hipStream_t stream = nullptr;
    mutable std::mutex mu;
    mutable bool resolved = false;
    mutable int status = 0;
    mutable sp::MailSlot mail;     // payload: n_in, n_out, error bits, koff[0..kvol]
    void set_sizes(int64_t n_in_, int64_t n_out_, const uint32_t* koff_words) const;
    ~sp_kmap() { sp::mail_release(&mail); }
    // filled on first use (average pooling's backward pass): links per output row, int32 [n_out]
    mutable std::mutex cache_mu;
    mutable sp::Buf out_link_cnt;
};

namespace sp {
// conv launchers (sp_conv.hip / sp_wgrad.hip)
// scratch != null: the call must not allocate; the weight copy of the link-list kernel goes there (forward only)
int conv_gather(const MapSide& side, int kvol, int64_t total_links, const void* d_f, const void* d_w, bool w_transposed,
                void* d_g, int cc, int co, sp_dtype dt, hipStream_t s, void* scratch = nullptr, size_t scratch_bytes = 0);
// wide bf16 layers on maps where most offsets of a row have a neighbour (sp_conv_dense.hip); d_w is [kvol][co][cc]
bool dense_shape_ok(int cc, int co, sp_dtype dt);
double dense_min_fill(int cc);
int conv_gather_dense(const MapSide& side, int kvol, const void* d_f, const void* d_w, void* d_g, int cc, int co,
                      hipStream_t s);
int conv_wgrad(const sp_kmap* m, const void* d_x, const void* d_dy, float* d_dw, int cin, int cout, sp_dtype dt,
               hipStream_t s);
}  // namespace sp
