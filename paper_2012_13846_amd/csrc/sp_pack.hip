// Stage-boundary packing of a sparse tensor (Sec. III-B, last paragraph: the coordinate matrix and the feature
// matrix are what crosses a stage boundary): (C, F) -> one contiguous device buffer with a small header, and back.
// One launch each way; pure streaming copies (HBM bound: every byte is read once and written once).
//
// Layout (little-endian, sections 256-byte aligned, padding zero):
//   0 "SPCF" | 4 u32 version 1 | 8 i64 n | 16 i32 channels | 20 i32 dtype | 24 i32 tensor stride | 28 0 |
//   32 i64 coords offset (256) | 40 i64 features offset | 48 i64 total bytes | 56..255 0 | coords | features
#include "sp_internal.h"

namespace sp {
namespace {

constexpr int kThreads = 256;
constexpr int64_t kHeader = 256, kAlign = 256;

inline int64_t up(int64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline int elt_of(sp_dtype dt) { return dt == SP_F32 ? 4 : 2; }

struct Layout {
    int64_t n, c_off, f_off, total, c_bytes, f_bytes;
};
Layout layout_of(int64_t n, int c, sp_dtype dt) {
    Layout l;
    l.n = n;
    l.c_off = kHeader;
    l.c_bytes = 16 * n;
    l.f_off = kHeader + up(l.c_bytes);
    l.f_bytes = n * c * elt_of(dt);
    l.total = l.f_off + up(l.f_bytes);
    return l;
}

// Copies `bytes` from src to dst + writes zeros up to `padded`; thread = one 16-byte piece of the padded range.
// vec: both pointers 16-byte aligned (then whole pieces move as one access).
__device__ __forceinline__ void copy_piece(unsigned char* __restrict__ dst, const unsigned char* __restrict__ src,
                                           int64_t piece, int64_t bytes, bool vec) {
    const int64_t b0 = piece * 16;
    if (b0 + 16 <= bytes && vec) {
        *reinterpret_cast<uint4*>(dst + b0) = *reinterpret_cast<const uint4*>(src + b0);
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) dst[b0 + i] = b0 + i < bytes ? src[b0 + i] : (unsigned char)0;
    }
}

__global__ __launch_bounds__(kThreads) void pack_kernel(const unsigned char* __restrict__ coords,
                                                        const unsigned char* __restrict__ feats, Layout l, int c, int dt,
                                                        int ts, int vec_f, unsigned char* __restrict__ buf) {
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t hp = kHeader / 16, cp = (l.f_off - l.c_off) / 16, fp = (l.total - l.f_off) / 16;
    if (t < hp) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (t == 0) {
            w[0] = 0x46435053u;  // "SPCF"
            w[1] = 1u;
            w[2] = (uint32_t)l.n;
            w[3] = (uint32_t)((uint64_t)l.n >> 32);
        } else if (t == 1) {
            w[0] = (uint32_t)c;
            w[1] = (uint32_t)dt;
            w[2] = (uint32_t)ts;
        } else if (t == 2) {
            w[0] = (uint32_t)l.c_off;
            w[1] = (uint32_t)((uint64_t)l.c_off >> 32);
            w[2] = (uint32_t)l.f_off;
            w[3] = (uint32_t)((uint64_t)l.f_off >> 32);
        } else if (t == 3) {
            w[0] = (uint32_t)l.total;
            w[1] = (uint32_t)((uint64_t)l.total >> 32);
        }
        *reinterpret_cast<uint4*>(buf + t * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    } else if (t < hp + cp) {
        copy_piece(buf + l.c_off, coords, t - hp, l.c_bytes, true);
    } else if (t < hp + cp + fp) {
        copy_piece(buf + l.f_off, feats, t - hp - cp, l.f_bytes, vec_f != 0);
    }
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(const unsigned char* __restrict__ buf, Layout l, int vec_f,
                                                          unsigned char* __restrict__ coords,
                                                          unsigned char* __restrict__ feats) {
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t cp = (l.c_bytes + 15) / 16, fp = (l.f_bytes + 15) / 16;
    if (t < cp) {
        *reinterpret_cast<uint4*>(coords + t * 16) = *reinterpret_cast<const uint4*>(buf + l.c_off + t * 16);
    } else if (t < cp + fp) {
        const int64_t b0 = (t - cp) * 16;
        if (b0 + 16 <= l.f_bytes && vec_f) {
            *reinterpret_cast<uint4*>(feats + b0) = *reinterpret_cast<const uint4*>(buf + l.f_off + b0);
        } else {
            for (int i = 0; i < 16 && b0 + i < l.f_bytes; ++i) feats[b0 + i] = buf[l.f_off + b0 + i];
        }
    }
}

int check(int64_t n, int c, sp_dtype dt) {
    if (n < 0 || n >= ((int64_t)1 << 31)) return fail(SP_ERR_INVALID_ARG, "bad row count");
    if (c < 1 || c > 65536) return fail(SP_ERR_INVALID_ARG, "bad channel count");
    if (dt != SP_F32 && dt != SP_BF16) return fail(SP_ERR_INVALID_ARG, "bad dtype");
    return SP_OK;
}

}  // namespace
}  // namespace sp

using namespace sp;

extern "C" {

int64_t sp_pack_bytes(int64_t n, int32_t c, sp_dtype dt) {
    if (check(n, c, dt) != SP_OK) return -1;
    return layout_of(n, c, dt).total;
}

int sp_pack(const int32_t* d_coords, const void* d_feats, int64_t n, int32_t c, sp_dtype dt, int32_t tensor_stride,
            void* d_buf, void* stream) {
    SP_TRY(check(n, c, dt));
    if (!d_buf || (n > 0 && (!d_coords || !d_feats))) return fail(SP_ERR_INVALID_ARG, "a pointer is NULL");
    if (((uintptr_t)d_buf & 255) != 0 || ((uintptr_t)d_coords & 15) != 0)
        return fail(SP_ERR_INVALID_ARG, "d_buf must be 256-byte aligned and d_coords 16-byte aligned");
    if (tensor_stride < 1) return fail(SP_ERR_INVALID_ARG, "tensor_stride < 1");
    const Layout l = layout_of(n, c, dt);
    const int64_t pieces = l.total / 16;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((pieces + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       (hipStream_t)stream, reinterpret_cast<const unsigned char*>(d_coords),
                       static_cast<const unsigned char*>(d_feats), l, c, (int)dt, tensor_stride,
                       ((uintptr_t)d_feats & 15) == 0 ? 1 : 0, static_cast<unsigned char*>(d_buf));
    SP_HIP(hipGetLastError());
    return SP_OK;
}

int sp_unpack_info(const void* d_buf, void* stream, int64_t* n, int32_t* c, sp_dtype* dt, int32_t* tensor_stride,
                   int64_t* total_bytes) {
    if (!d_buf) return fail(SP_ERR_INVALID_ARG, "d_buf is NULL");
    uint32_t h[16];
    SP_TRY(read_back(h, d_buf, sizeof h, (hipStream_t)stream));
    if (h[0] != 0x46435053u || h[1] != 1u) return fail(SP_ERR_INVALID_ARG, "not a packed sparse tensor (bad magic or version)");
    const int64_t nn = (int64_t)(((uint64_t)h[3] << 32) | h[2]);
    const int cc = (int)h[4], dd = (int)h[5], ts = (int)h[6];
    if (check(nn, cc, (sp_dtype)dd) != SP_OK || ts < 1) return fail(SP_ERR_INVALID_ARG, "packed header holds invalid sizes");
    const Layout l = layout_of(nn, cc, (sp_dtype)dd);
    const int64_t c_off = (int64_t)(((uint64_t)h[9] << 32) | h[8]), f_off = (int64_t)(((uint64_t)h[11] << 32) | h[10]);
    const int64_t total = (int64_t)(((uint64_t)h[13] << 32) | h[12]);
    if (c_off != l.c_off || f_off != l.f_off || total != l.total)
        return fail(SP_ERR_INVALID_ARG, "packed header's offsets do not match its sizes");
    if (n) *n = nn;
    if (c) *c = cc;
    if (dt) *dt = (sp_dtype)dd;
    if (tensor_stride) *tensor_stride = ts;
    if (total_bytes) *total_bytes = total;
    return SP_OK;
}

int sp_unpack(const void* d_buf, int64_t n, int32_t c, sp_dtype dt, int32_t* d_coords, void* d_feats, void* stream) {
    SP_TRY(check(n, c, dt));
    if (!d_buf || (n > 0 && (!d_coords || !d_feats))) return fail(SP_ERR_INVALID_ARG, "a pointer is NULL");
    if (((uintptr_t)d_buf & 255) != 0 || ((uintptr_t)d_coords & 15) != 0)
        return fail(SP_ERR_INVALID_ARG, "d_buf must be 256-byte aligned and d_coords 16-byte aligned");
    const Layout l = layout_of(n, c, dt);
    const int64_t pieces = (l.c_bytes + 15) / 16 + (l.f_bytes + 15) / 16;
    if (pieces == 0) return SP_OK;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((pieces + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       (hipStream_t)stream, static_cast<const unsigned char*>(d_buf), l,
                       ((uintptr_t)d_feats & 15) == 0 ? 1 : 0, reinterpret_cast<unsigned char*>(d_coords),
                       static_cast<unsigned char*>(d_feats));
    SP_HIP(hipGetLastError());
    return SP_OK;
}

}  // extern "C"
