// Host runtime of the library: error strings, the caching device-memory pool, pinned read-back staging.
#include <cstring>
#include <map>
#include <mutex>
#include <string>

#include "sp_internal.h"

namespace sp {

static thread_local std::string g_err;

void set_error(const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
}

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

// ---- pool -----------------------------------------------------------------------------------------------
// Size-class caching pool.  A block carries the stream its last owner used it on.  An allocation for the
// same stream takes it at once (the stream orders the old and the new work).  An allocation for another
// stream may still take it, but first makes that stream wait for everything enqueued so far on the block's
// old stream (an event recorded there now is later than the block's last use), so library scratch and
// handle memory can be recycled between callers that drive the library from different streams.
namespace {
struct FreeBlock {
    void* p;
    hipStream_t stream;
};
struct Pool {
    std::mutex mu;
    std::multimap<size_t, FreeBlock> free_blocks;  // size class -> block
    std::map<void*, size_t> live;                  // block -> size class
    std::vector<hipEvent_t> events;                // spare events for cross-stream hand-overs
    int64_t held = 0;
    int64_t cross_stream = 0;                      // hand-overs between streams so far (diagnostics)

    // Size classes: multiples of 1/8 of the power of two below the request (<= 12.5 % slack), min 512 B.
    static size_t size_class(size_t b) {
        if (b < 512) return 512;
        size_t p = 512;
        while ((p << 1) <= b) p <<= 1;
        size_t g = p >> 3;
        return (b + g - 1) / g * g;
    }

    // Orders `to` behind everything enqueued on `from` so far.  false: could not (the caller skips the block).
    bool hand_over(hipStream_t from, hipStream_t to) {
        hipEvent_t ev = nullptr;
        if (!events.empty()) {
            ev = events.back();
            events.pop_back();
        } else if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        bool ok = hipEventRecord(ev, from) == hipSuccess && hipStreamWaitEvent(to, ev, 0) == hipSuccess;
        if (!ok) {
            // the old stream may be gone: wait for the whole device instead
            (void)hipGetLastError();
            ok = hipDeviceSynchronize() == hipSuccess;
        }
        events.push_back(ev);  // a recorded event may be re-recorded: the wait above keeps its own snapshot
        return ok;
    }

    void* alloc(size_t bytes, hipStream_t s) {
        size_t c = size_class(bytes);
        {
            std::lock_guard<std::mutex> lk(mu);
            auto range = free_blocks.equal_range(c);
            auto pick = free_blocks.end();
            for (auto it = range.first; it != range.second; ++it) {
                if (it->second.stream == s) {
                    pick = it;
                    break;
                }
                if (pick == free_blocks.end()) pick = it;
            }
            if (pick != free_blocks.end()) {
                const FreeBlock b = pick->second;
                if (b.stream == s || hand_over(b.stream, s)) {
                    if (b.stream != s) ++cross_stream;
                    free_blocks.erase(pick);
                    live[b.p] = c;
                    return b.p;
                }
            }
        }
        void* p = nullptr;
        hipError_t e = hipMalloc(&p, c);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            trim();  // give cached blocks back and retry once
            e = hipMalloc(&p, c);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                set_error("hipMalloc(%zu bytes) failed: %s", c, hipGetErrorString(e));
                return nullptr;
            }
        }
        std::lock_guard<std::mutex> lk(mu);
        live[p] = c;
        held += (int64_t)c;
        return p;
    }

    void release(void* p, hipStream_t s) {
        std::lock_guard<std::mutex> lk(mu);
        auto it = live.find(p);
        if (it == live.end()) return;
        free_blocks.emplace(it->second, FreeBlock{p, s});
        live.erase(it);
    }

    int trim() {
        std::multimap<size_t, FreeBlock> blocks;
        {
            std::lock_guard<std::mutex> lk(mu);
            blocks.swap(free_blocks);
        }
        if (blocks.empty()) return SP_OK;
        hipError_t e = hipDeviceSynchronize();
        int64_t freed = 0;
        for (auto& kv : blocks) {
            (void)hipFree(kv.second.p);
            freed += (int64_t)kv.first;
        }
        std::lock_guard<std::mutex> lk(mu);
        held -= freed;
        return e == hipSuccess ? SP_OK : fail(SP_ERR_HIP, "hipDeviceSynchronize: %s", hipGetErrorString(e));
    }
};

Pool& pool() {
    static Pool* p = new Pool;  // leaked on purpose: device memory goes with the process
    return *p;
}

// The caller's allocator, if one is installed (sp_set_allocator): then the pool above is not used.
struct External {
    std::mutex mu;
    sp_alloc_fn alloc = nullptr;
    sp_free_fn free_ = nullptr;
    void* ctx = nullptr;
};
External& external() {
    static External* e = new External;
    return *e;
}

struct Stage {
    std::mutex mu;
    void* h = nullptr;
    size_t bytes = 0;
};
Stage& stage() {
    static Stage* s = new Stage;
    return *s;
}
}  // namespace

DevBuf::~DevBuf() {
    if (!p) return;
    if (free_)
        free_(p, ctx);
    else
        pool().release(p, stream);
}

Buf dev_alloc(size_t bytes, hipStream_t s) {
    sp_alloc_fn ext_alloc;
    sp_free_fn ext_free;
    void* ext_ctx;
    {
        External& e = external();
        std::lock_guard<std::mutex> lk(e.mu);
        ext_alloc = e.alloc;
        ext_free = e.free_;
        ext_ctx = e.ctx;
    }
    auto b = std::make_shared<DevBuf>();
    b->bytes = bytes;
    b->stream = s;
    if (ext_alloc) {
        b->p = ext_alloc(bytes ? bytes : 1, (void*)s, ext_ctx);
        if (!b->p) {
            set_error("the installed allocator returned NULL for %zu bytes", bytes);
            return nullptr;
        }
        if (((uintptr_t)b->p & 255) != 0) {
            ext_free(b->p, ext_ctx);
            b->p = nullptr;
            set_error("the installed allocator returned memory that is not 256-byte aligned");
            return nullptr;
        }
        b->free_ = ext_free;  // the block goes back where it came from, whatever is installed by then
        b->ctx = ext_ctx;
        return b;
    }
    b->p = pool().alloc(bytes ? bytes : 1, s);
    if (!b->p) return nullptr;
    return b;
}

int pool_trim() { return pool().trim(); }
int64_t pool_bytes() {
    std::lock_guard<std::mutex> lk(pool().mu);
    return pool().held;
}
int64_t pool_cross_stream() {
    std::lock_guard<std::mutex> lk(pool().mu);
    return pool().cross_stream;
}

// ---- small read-backs through a mailbox in pinned host memory ------------------------------------------------
// The host needs a few numbers of every map build (row count, pairs per offset) before it can size the next
// launches.  A copy + stream synchronisation costs the copy kernel and the runtime's wake-up; instead the last
// kernel of the stream writes the numbers straight into coherent pinned host memory, then a sequence number,
// and the host polls that word.  Ordered behind everything earlier on the stream, like the copy was.
namespace {
constexpr size_t kMailWords = 1024;  // 4 KB of payload
struct Mailbox {
    std::mutex mu;
    uint32_t* h = nullptr;  // [kMailWords] payload, then the sequence word
    uint32_t* d = nullptr;  // the same memory as the device sees it
    uint32_t seq = 0;
    bool tried = false;
};
Mailbox& mailbox() {
    static Mailbox* m = new Mailbox;
    return *m;
}
__global__ __launch_bounds__(256) void mailbox_kernel(const uint32_t* __restrict__ src, int nwords, uint32_t* dst,
                                                      uint32_t seq) {
    for (int i = threadIdx.x; i < nwords; i += 256) dst[i] = src[i];
    __threadfence_system();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(dst + kMailWords, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}
}  // namespace


// ---- mail slots: small results that a build's last kernel writes straight into pinned host memory ----------------
// The builds do not wait for their row and pair counts: the kernel that computes them writes them into a slot of
// coherent pinned host memory (payload first, then a sequence word with system-scope release), and the host
// reads the slot only when somebody asks for the numbers (mail_wait polls the sequence word).
namespace {
struct MailPool {
    std::mutex mu;
    uint32_t* h = nullptr;  // kMailSlots slots of kMailSlotWords words, as the host sees them
    uint32_t* d = nullptr;  // the same memory as the device sees it
    std::vector<int> free_slots;
    struct Parked {
        int index;
        uint32_t seq;
        hipStream_t stream;
    };
    std::vector<Parked> parked;  // released before their kernel delivered
    uint32_t next_seq = 1;
    bool tried = false;
};
MailPool& mail_pool() {
    static MailPool* m = new MailPool;
    return *m;
}
}  // namespace

bool mail_acquire(MailSlot* out) {
    MailPool& mp = mail_pool();
    std::lock_guard<std::mutex> lk(mp.mu);
    if (!mp.tried) {
        mp.tried = true;
        void* h = nullptr;
        const size_t bytes = (size_t)kMailSlots * kMailSlotWords * 4;
        if (hipHostMalloc(&h, bytes, hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess) {
            void* d = nullptr;
            if (hipHostGetDevicePointer(&d, h, 0) == hipSuccess) {
                memset(h, 0, bytes);
                mp.h = static_cast<uint32_t*>(h);
                mp.d = static_cast<uint32_t*>(d);
                for (int i = kMailSlots - 1; i >= 0; --i) mp.free_slots.push_back(i);
            } else {
                (void)hipHostFree(h);
            }
        }
        (void)hipGetLastError();
    }
    if (!mp.h) return false;
    if (!mp.parked.empty() && mp.free_slots.size() < 64) {  // look whether parked slots have been delivered meanwhile
        size_t keep = 0;
        for (size_t j = 0; j < mp.parked.size(); ++j) {
            const MailPool::Parked& pk = mp.parked[j];
            const uint32_t got = __atomic_load_n(mp.h + (size_t)pk.index * kMailSlotWords + kMailSeqWord, __ATOMIC_ACQUIRE);
            bool done = got == pk.seq;
            if (!done) {
                done = hipStreamQuery(pk.stream) != hipErrorNotReady;  // nothing left that could still write it
                (void)hipGetLastError();
            }
            if (done) mp.free_slots.push_back(pk.index);
            else mp.parked[keep++] = pk;
        }
        mp.parked.resize(keep);
    }
    if (mp.free_slots.empty()) return false;
    const int i = mp.free_slots.back();
    mp.free_slots.pop_back();
    out->index = i;
    out->h = mp.h + (size_t)i * kMailSlotWords;
    out->d = mp.d + (size_t)i * kMailSlotWords;
    out->seq = mp.next_seq++;
    out->armed = false;
    out->stream = nullptr;
    if (mp.next_seq == 0) mp.next_seq = 1;
    return true;
}

void mail_release(MailSlot* slot) {
    if (slot->index < 0) return;
    MailPool& mp = mail_pool();
    std::lock_guard<std::mutex> lk(mp.mu);
    const bool delivered = __atomic_load_n(slot->h + kMailSeqWord, __ATOMIC_ACQUIRE) == slot->seq;
    if (slot->armed && !delivered) mp.parked.push_back({slot->index, slot->seq, slot->stream});
    else mp.free_slots.push_back(slot->index);
    slot->index = -1;
}

int mail_wait(const MailSlot& slot, hipStream_t s) {
    volatile uint32_t* flag = slot.h + kMailSeqWord;
    // poll; every ~50 us of silence ask the runtime whether the stream has failed or finished
    for (uint64_t spins = 0;; ++spins) {
        if (__atomic_load_n(flag, __ATOMIC_ACQUIRE) == slot.seq) return SP_OK;
        if ((spins & 0x3fff) == 0x3fff) {
            const hipError_t q = hipStreamQuery(s);
            if (q == hipSuccess) {  // everything enqueued has run: the stores are visible by now
                if (__atomic_load_n(flag, __ATOMIC_ACQUIRE) == slot.seq) return SP_OK;
                return fail(SP_ERR_HIP, "a build finished without delivering its counts");
            }
            if (q != hipErrorNotReady) return fail(SP_ERR_HIP, "hipStreamQuery: %s", hipGetErrorString(q));
        }
    }
}

int read_back(void* h_dst, const void* d_src, size_t bytes, hipStream_t s, const std::function<void()>& then_enqueue) {
    if (bytes == 0) {
        if (then_enqueue) then_enqueue();
        SP_HIP(hipStreamSynchronize(s));
        return SP_OK;
    }
    if (bytes % 4 == 0 && bytes <= kMailWords * 4) {
        Mailbox& mb = mailbox();
        std::lock_guard<std::mutex> lk(mb.mu);
        if (!mb.tried) {
            mb.tried = true;
            void* h = nullptr;
            if (hipHostMalloc(&h, (kMailWords + 16) * 4, hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess) {
                void* d = nullptr;
                if (hipHostGetDevicePointer(&d, h, 0) == hipSuccess) {
                    memset(h, 0, (kMailWords + 16) * 4);
                    mb.h = static_cast<uint32_t*>(h);
                    mb.d = static_cast<uint32_t*>(d);
                } else {
                    (void)hipHostFree(h);
                }
            }
            (void)hipGetLastError();  // a refusal only means the slower path below
        }
        if (mb.h) {
            const uint32_t seq = ++mb.seq;
            hipLaunchKernelGGL(mailbox_kernel, dim3(1), dim3(256), 0, s, static_cast<const uint32_t*>(d_src),
                               (int)(bytes / 4), mb.d, seq);
            SP_HIP(hipGetLastError());
            if (then_enqueue) then_enqueue();
            volatile uint32_t* flag = mb.h + kMailWords;
            // poll; every ~50 us of silence ask the runtime whether the stream has failed or finished
            for (uint64_t spins = 0;; ++spins) {
                if (__atomic_load_n(flag, __ATOMIC_ACQUIRE) == seq) break;
                if ((spins & 0x3fff) == 0x3fff) {
                    const hipError_t q = hipStreamQuery(s);
                    if (q == hipSuccess) {  // the kernel is done: its stores are visible by now
                        if (__atomic_load_n(flag, __ATOMIC_ACQUIRE) == seq) break;
                        return fail(SP_ERR_HIP, "read-back mailbox: kernel finished without delivering");
                    }
                    if (q != hipErrorNotReady) return fail(SP_ERR_HIP, "hipStreamQuery: %s", hipGetErrorString(q));
                }
            }
            memcpy(h_dst, mb.h, bytes);
            return SP_OK;
        }
    }
    Stage& st = stage();
    std::lock_guard<std::mutex> lk(st.mu);
    if (st.bytes < bytes) {
        if (st.h) (void)hipHostFree(st.h);
        st.h = nullptr;
        st.bytes = 0;
        size_t want = bytes < 65536 ? 65536 : bytes;
        hipError_t e = hipHostMalloc(&st.h, want, hipHostMallocDefault);
        if (e != hipSuccess) {
            st.h = nullptr;
            return fail(SP_ERR_ALLOC, "hipHostMalloc(%zu): %s", want, hipGetErrorString(e));
        }
        st.bytes = want;
    }
    SP_HIP(hipMemcpyAsync(st.h, d_src, bytes, hipMemcpyDeviceToHost, s));
    if (then_enqueue) then_enqueue();
    SP_HIP(hipStreamSynchronize(s));
    memcpy(h_dst, st.h, bytes);
    return SP_OK;
}

}  // namespace sp

namespace sp {
// iters x 8 independent MFMAs per wavefront, operands and accumulators in registers
template <bool kF32>
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* __restrict__ sink) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    f32x4 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float a = 1.0f + (float)(threadIdx.x & 3) * 0.25f, b = 0.5f;
    bf16x8 ah, bh;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        ah[j] = (__bf16)a;
        bh[j] = (__bf16)b;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // (a different first operand per chain: identical chains would be merged into one)
            if constexpr (kF32) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a + (float)j, b, acc[j], 0, 0, 0);
            else {
                bf16x8 aj = ah;
                aj[0] = (__bf16)(float)j;
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aj, bh, acc[j], 0, 0, 0);
            }
        }
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) t += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (t == 123.456f) sink[threadIdx.x] = t;  // never true: keeps the loop alive without a store in the way
}
}  // namespace sp

extern "C" {

const char* sp_last_error(void) { return sp::g_err.c_str(); }

int sp_set_allocator(sp_alloc_fn alloc, sp_free_fn free_, void* ctx) {
    if ((alloc == nullptr) != (free_ == nullptr))
        return sp::fail(SP_ERR_INVALID_ARG, "alloc and free must both be given or both be NULL");
    sp::External& e = sp::external();
    std::lock_guard<std::mutex> lk(e.mu);
    e.alloc = alloc;
    e.free_ = free_;
    e.ctx = ctx;
    return SP_OK;
}
int sp_measure_mfma_peak(sp_dtype dt, void* stream, double* tflops) {
    if (!tflops || (dt != SP_F32 && dt != SP_BF16)) return sp::fail(SP_ERR_INVALID_ARG, "sp_measure_mfma_peak: bad argument");
    hipStream_t s = static_cast<hipStream_t>(stream);
    sp::Buf sink = sp::dev_alloc(4096, s);
    if (!sink) return SP_ERR_ALLOC;
    const int iters = 4000, blocks = 256 * 4 * 2 / 4;  // 8 wavefronts per CU = 2 per SIMD, 4 per workgroup
    hipEvent_t e0, e1;
    SP_HIP(hipEventCreate(&e0));
    SP_HIP(hipEventCreate(&e1));
    for (int rep = 0; rep < 2; ++rep) {  // the first launch warms up
        SP_HIP(hipEventRecord(e0, s));
        if (dt == SP_F32) hipLaunchKernelGGL(sp::mfma_loop_kernel<true>, dim3(blocks), dim3(256), 0, s, iters, sp::ptr<float>(sink));
        else hipLaunchKernelGGL(sp::mfma_loop_kernel<false>, dim3(blocks), dim3(256), 0, s, iters, sp::ptr<float>(sink));
        SP_HIP(hipEventRecord(e1, s));
        SP_HIP(hipEventSynchronize(e1));
    }
    float ms = 0.f;
    SP_HIP(hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    const double flop_per_mfma = dt == SP_F32 ? 2.0 * 16 * 16 * 4 : 2.0 * 16 * 16 * 32;
    *tflops = (double)blocks * 4 * iters * 8 * flop_per_mfma / (ms * 1e-3) / 1e12;
    return SP_OK;
}

int64_t sp_pool_cross_stream(void) { return sp::pool_cross_stream(); }
int sp_pool_trim(void) { return sp::pool_trim(); }
int64_t sp_pool_bytes(void) { return sp::pool_bytes(); }
const char* sp_version(void) { return "sp_conv 0.1 (gfx950)"; }

}  // extern "C"
