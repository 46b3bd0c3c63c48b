/*
 * sp_conv.h - C ABI of the MI355X (gfx950) generalized sparse convolution library.
 *
 * The library implements the three steps of the generalized sparse convolution
 * (Sec. III-B: 1 output coordinates, 2 input/output mapping per kernel weight,
 * 3 the sum of Eq. 2) and the gradients of Eq. 2 w.r.t. inputs and weights
 * (Sec. II-A), all as HIP kernels.  There is no CPU fallback.
 *
 * Conventions
 *   - A sparse tensor is (C, F) (Sec. III-B): C is int32 [N][4], rows (b, x, y, z),
 *     batch index first; F is [N][channels], row j of F belongs to row j of C.
 *     Both row-major, in device memory.
 *   - Kernel weights are W[K^3][N_out][N_in] (Sec. III-B: K^D matrices of size
 *     N_out x N_in), row-major, device memory.
 *   - Kernel offset number k = (ax*K + ay)*K + az (z fastest); an odd K uses offsets
 *     a - (K-1)/2 (centred, as V^1(3) = {-1,0,1}), an even K uses offsets a in 0..K-1.
 *     Offsets are multiplied by dilation * (input tensor stride).
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work of a call is enqueued on it.  The build calls return without waiting:
 *     row and pair counts reach the host through pinned memory and the first call
 *     that needs one on the host (the size queries, the convolutions, transpose)
 *     waits for it then, and only for that build's last kernel, not for the stream.
 *   - Every function returns SP_OK (0) or a negative sp_status; sp_last_error()
 *     gives a message for the calling thread's last failure.  Argument checks are
 *     done on the host before anything is launched.
 *   - Handles own their device memory (taken from a caching pool inside the
 *     library) until destroyed.  Pointers returned by *_data/_pairs/_table/_tiles are
 *     borrowed and die with the handle.  Feature / weight / gradient buffers are
 *     owned by the caller and must stay alive until the stream passed the call.
 *   - All calls that touch one handle must use the same stream (or be ordered by
 *     the caller).  Different handles may be driven from different streams and
 *     host threads at the same time.  Coordinates must satisfy 0 <= b < 65536 and
 *     -32768 <= x,y,z < 32768, else SP_ERR_RANGE.
 */
#ifndef SP_CONV_H
#define SP_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SP_OK = 0,
    SP_ERR_INVALID_ARG = -1, /* null pointer, negative size, bad kernel/stride/dilation/channels */
    SP_ERR_RANGE = -2,       /* a coordinate cannot be packed into the 64-bit key */
    SP_ERR_ALLOC = -3,       /* device or host allocation failed */
    SP_ERR_HIP = -4,         /* a HIP runtime call failed */
    SP_ERR_UNSUPPORTED = -5, /* valid request this build does not implement (dilation > 1 with stride > 1) */
    SP_ERR_TABLE_FULL = -6   /* hash table overflow (cannot happen at the load factor used; checked anyway) */
} sp_status;

typedef enum { SP_F32 = 0, SP_BF16 = 1 } sp_dtype; /* storage type of features/weights; accumulation is fp32 */

typedef struct sp_coords sp_coords_t; /* distinct coordinates + their hash table + tensor stride   */
typedef struct sp_kmap sp_kmap_t;     /* kernel map of one (coords, kernel, stride, dilation)      */

/* ---- step 0: the sparse tensor's coordinate set (Sec. III-B, sparse tensor definition) --------------
 * Hashes d_raw [n_raw][4] into an open-addressing table, merges duplicate rows and numbers the
 * distinct rows in first-occurrence order (unique row r = r-th distinct coordinate met walking the
 * rows in order).  tensor_stride (>= 1) is recorded, coordinates are expected on that lattice.
 * Returns without waiting for the stream: d_raw must stay valid until the stream has passed the call.  A
 * coordinate outside the packable range is found on the device and reported (SP_ERR_RANGE) by the first later
 * call that needs this set's row count on the host (sp_coords_size, or any call on a map built from it).
 * n_raw may be 0.  *out receives a new handle (caller destroys). */
int sp_coords_build(const int32_t* d_raw, int64_t n_raw, int32_t tensor_stride, void* stream, sp_coords_t** out);

/* N and the tensor stride.  Asking for N waits (the first time) until the build's numbering kernel has delivered
 * it, and returns the build's device-detected error if there was one.  Either out pointer may be NULL. */
int sp_coords_size(const sp_coords_t* c, int64_t* n, int32_t* tensor_stride);

/* d_coords: int32 [N][4]; d_inverse: int32 [n_raw], inverse[j] = distinct row that raw row j merged into.
 * (The buffers are allocated for the source row count; only the first N rows of d_coords are meaningful.)
 * No waiting, except that n_raw of a coarser set made by sp_kmap_build waits for its source set's N. */
int sp_coords_data(const sp_coords_t* c, const int32_t** d_coords, const int32_t** d_inverse, int64_t* n_raw);

/* Drops one reference; the memory is returned to the pool when the last reference goes. */
int sp_coords_destroy(sp_coords_t* c);

/* ---- steps 1 + 2: output coordinates and the kernel map (Sec. III-B steps 1, 2) -----------------------
 * kernel_size in 1..5, stride >= 1, dilation >= 1 (dilation > 1 needs stride == 1).
 * Step 1: stride 1 keeps the coordinates (out_coords = a new reference to `in`); stride s > 1 floors
 *   x,y,z to multiples of S = tensor_stride*s (true floor), merges duplicates in first-occurrence
 *   order, and the new tensor stride is S.
 * Step 2: M_k = {(i,o) : c_in[i] = c_out[o] + offset_k * dilation * tensor_stride, same batch index},
 *   found by probing the input set's hash table.
 * Returns without waiting: where `in`'s N has not reached the host yet the kernels read it from device memory
 * and buffers are sized from `in`'s source row count (if that bound is wasteful - above 1 GiB of tables and
 * lists - the call waits for N first).
 * *kmap and *out_coords receive new handles (caller destroys both; out_coords may be NULL if unwanted). */
int sp_kmap_build(const sp_coords_t* in, int32_t kernel_size, int32_t stride, int32_t dilation, void* stream,
                  sp_kmap_t** kmap, sp_coords_t** out_coords);

/* The map of the transposed (upsampling) convolution that undoes `fwd`'s coordinate change: the same
 * pairs with the roles of input and output swapped, same offset numbering.  Its outputs are fwd's input
 * coordinates (the cached finer level).  (The paper defines no transposed convolution; this is the
 * coordinate-hierarchy-reusing reading.)  No device work; shares fwd's buffers.  Caller destroys. */
int sp_kmap_transpose(const sp_kmap_t* fwd, sp_kmap_t** transposed);

/* Host-side facts; everything but kvol waits (the first time) until the build has delivered its counts.
 * h_counts, if not NULL, receives kvol pair counts |M_k|. */
int sp_kmap_info(const sp_kmap_t* m, int64_t* n_in, int64_t* n_out, int32_t* kvol, int64_t* total_pairs,
                 int64_t* h_counts);

/* Pair lists, one row of *pair_stride entries per offset: list k is entries [k * pair_stride, k * pair_stride +
 * counts[k]) of both arrays (the rest of a row is unused); entry p links input row d_pair_in[p] to output row
 * d_pair_out[p].  (A row has room for the most pairs an offset can have, so that the build can place a
 * pair before the totals of the other offsets are known.)  Order inside a list: ascending output row. */
int sp_kmap_pairs(const sp_kmap_t* m, const int32_t** d_pair_in, const int32_t** d_pair_out, int64_t* pair_stride);

/* Neighbour tables, offset-major: d_nbr_out [kvol][n_out] = input row linked to (o,k) or -1;
 * d_nbr_in [kvol][n_in] = output row linked to (i,k) or -1.  A stride-1 map with an odd kernel stores one
 * table for both (the link (i,o) at offset k is the link (o,i) at offset kvol-1-k): then *in_reversed (or,
 * for its transpose, *out_reversed) is 1 and block k of that table holds offset kvol-1-k. */
int sp_kmap_table(const sp_kmap_t* m, const int32_t** d_nbr_out, const int32_t** d_nbr_in, int32_t* out_reversed,
                  int32_t* in_reversed);

int sp_kmap_destroy(sp_kmap_t* m);

/* Generative transposed (upsampling) convolution: creates the finer coordinates instead of looking them up in
 * a cached level.  (The paper defines no transposed convolution; this completes the reading taken by
 * sp_kmap_transpose for the case where no finer level exists.)  `in` has tensor stride ts_in, a multiple of
 * `stride`; ts_out = ts_in / stride; the output set is { u + offset_k * ts_out : u in `in`, all K^3 offsets },
 * duplicates merged, rows numbered in first-occurrence order over the candidates taken input row by input row
 * and, inside a row, in offset order.  The returned map has the roles of sp_kmap_transpose's result: its
 * inputs are the rows of `in`, its outputs the created rows, M_k = {(j, o) : c_out[o] = c_in[j] + offset_k *
 * ts_out}; every offset has exactly n_in pairs.  sp_conv_fwd on it is the transposed convolution
 * (W[k][cout][cin], cin = channels on `in`); sp_kmap_transpose of it is the stride-`stride` convolution back.
 * *out_coords' inverse array (sp_coords_data) has K^3 * n_in entries: entry j*K^3 + k is the output row of
 * candidate (j, k).  Synchronises `stream`.  Caller destroys both handles. */
int sp_kmap_build_generative(const sp_coords_t* in, int32_t kernel_size, int32_t stride, void* stream,
                             sp_kmap_t** kmap, sp_coords_t** out_coords);

/* ---- step 3 and its gradients (Eq. 2; Sec. II-A for the backward pass) --------------------------------
 * cin / cout are N_in / N_out of W[kvol][cout][cin].  dt is the storage type of x, w, y, dy, dx
 * (SP_BF16: 16-bit bfloat16, results rounded to nearest even once); accumulation is always fp32.
 * Outputs are overwritten (rows / offsets without pairs become zero).  No host synchronisation.
 * All feature / weight / gradient pointers must be 16-byte aligned (SP_ERR_INVALID_ARG otherwise).
 * Matrix-core kernels exist for: forward / data gradient with a contraction width (cin for the forward pass,
 * cout for the data gradient) of 16 (fp32 only), 32, 64, 128 or 256 and the other width a multiple of 16;
 * weight gradient with both widths multiples of 16.  Every other channel count runs on a plain
 * one-thread-per-output kernel (correct, slow).
 *
 *   sp_conv_fwd:        y[o,:]  = sum_k sum_{(i,o) in M_k} W_k   x[i,:]      x [n_in][cin]   -> y  [n_out][cout]
 *   sp_conv_bwd_data:   dx[i,:] = sum_k sum_{(i,o) in M_k} W_k^T dy[o,:]     dy [n_out][cout] -> dx [n_in][cin]
 *   sp_conv_bwd_weight: dw_k    = sum_{(i,o) in M_k} dy[o,:] x[i,:]^T        -> dw fp32 [kvol][cout][cin]
 * For a transposed map the same formulas hold with that map's own n_in (coarse) / n_out (fine). */
int sp_conv_fwd(const sp_kmap_t* m, const void* d_x, const void* d_w, void* d_y, int32_t cin, int32_t cout,
                sp_dtype dt, void* stream);
int sp_conv_bwd_data(const sp_kmap_t* m, const void* d_dy, const void* d_w, void* d_dx, int32_t cin, int32_t cout,
                     sp_dtype dt, void* stream);
int sp_conv_bwd_weight(const sp_kmap_t* m, const void* d_x, const void* d_dy, float* d_dw, int32_t cin,
                       int32_t cout, sp_dtype dt, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): sp_conv_fwd with the same arguments, results and kernel choice, except that the
 * call allocates nothing (no hipMalloc / hipFree, no pool request).  Where sp_conv_fwd takes scratch from the
 * pool (the fragment-major copy of the weights that the link-list kernel reads), this call uses a 4 MiB
 * array in static device memory, which every GPU the library runs on holds until the process ends.
 * Weights larger than that on a shape that needs the copy give SP_ERR_UNSUPPORTED (kvol * cin * cout *
 * element size <= 4 MiB always fits).  All calls on one GPU share that array: calls that overlap in time on
 * one GPU (different streams) race; calls on one stream are ordered and safe.  The array's contents are
 * rewritten by every call, nothing in it needs to start at zero. */
int sp_conv_fwd_noalloc(const sp_kmap_t* m, const void* d_x, const void* d_w, void* d_y, int32_t cin, int32_t cout,
                        sp_dtype dt, void* stream);

/* ---- pooling over a kernel map (Sec. III, caption of the partition-overview figure: pooling layers sit
 * between the SparseConv blocks; the paper gives no formula) -------------------------------------------------
 * Eq. 2 with the weighted sum replaced by a reduction over the same neighbour set: for every output row o and
 * channel, over the inputs i linked to o by any offset of the map,
 *   SP_POOL_MAX: the maximum;  SP_POOL_SUM: the sum;  SP_POOL_AVG: the sum / number of linked inputs (the
 *   inputs present, not the kernel volume).  An output without links becomes 0.
 * x [n_in][c] -> y [n_out][c], storage type dt, accumulation fp32, rounded once.  d_arg (MAX only; may be NULL
 * if no backward pass follows): uint8 [n_out][c], the offset number of the link that gave the maximum, 255
 * where the row has no link; among equal maxima the lowest offset number wins.
 * Backward: dx [n_in][c] from dy [n_out][c]: SUM passes dy to every linked input, AVG dy / links, MAX passes
 * dy to the input recorded in d_arg.  No atomics, fixed summation order.  No host synchronisation. */
typedef enum { SP_POOL_MAX = 0, SP_POOL_AVG = 1, SP_POOL_SUM = 2 } sp_pool_mode;
int sp_pool_fwd(const sp_kmap_t* m, const void* d_x, void* d_y, uint8_t* d_arg, int32_t c, sp_pool_mode mode,
                sp_dtype dt, void* stream);
int sp_pool_bwd(const sp_kmap_t* m, const void* d_dy, const uint8_t* d_arg, void* d_dx, int32_t c, sp_pool_mode mode,
                sp_dtype dt, void* stream);

/* ---- the layers between sparse convolutions ----------------------------------------------------------------
 * (Sec. III, caption of the partition-overview figure: batch normalisation, activation and pooling layers sit
 * between the SparseConv blocks; Sec. IV-A: a 40-category classifier.)  The paper gives no formulas; these are
 * the standard definitions.  Features are [n][c] row-major of storage type dt; parameters, statistics and
 * everything per cloud are fp32.  Reductions are two-level with a fixed order (reproducible); no host
 * synchronisation.
 *
 * sp_bn_relu_fwd: training-mode batch normalisation over the n rows, per channel, biased variance:
 *   y = gamma * (x - mean) * rstd + beta, rstd = 1/sqrt(var + eps), then max(y, 0) if relu != 0.
 *   d_mean / d_rstd [c] are outputs (the backward pass needs them).
 * sp_bn_relu_bwd: with dyh = dy (masked where y <= 0 if relu), xhat = (x - mean) * rstd:
 *   dbeta = sum dyh, dgamma = sum dyh * xhat, dx = gamma * rstd / n * (n * dyh - dbeta - xhat * dgamma).
 *   d_y (the forward output) is only read when relu != 0. */
int sp_bn_relu_fwd(const void* d_x, int64_t n, int32_t c, const float* d_gamma, const float* d_beta, float eps,
                   int32_t relu, void* d_y, float* d_mean, float* d_rstd, sp_dtype dt, void* stream);
int sp_bn_relu_bwd(const void* d_x, const void* d_y, const void* d_dy, int64_t n, int32_t c, const float* d_gamma,
                   const float* d_mean, const float* d_rstd, int32_t relu, void* d_dx, float* d_dgamma,
                   float* d_dbeta, sp_dtype dt, void* stream);

/* Global average pooling per cloud: d_out [n_clouds][c] = mean of the rows whose batch index (column 0 of
 * d_coords [n][4]) is that cloud, zero for an empty cloud; d_counts [n_clouds] = rows per cloud (as float).
 * Rows with a batch index outside [0, n_clouds) are ignored.  Backward: dx[r] = dout[b(r)] / count[b(r)]. */
int sp_pool_avg_fwd(const int32_t* d_coords, const void* d_x, int64_t n, int32_t c, int32_t n_clouds, float* d_out,
                    float* d_counts, sp_dtype dt, void* stream);
int sp_pool_avg_bwd(const int32_t* d_coords, const float* d_dout, const float* d_counts, int64_t n, int32_t c,
                    int32_t n_clouds, void* d_dx, sp_dtype dt, void* stream);

/* Linear layer on the pooled features: out [n_clouds][m] = in [n_clouds][c] * w[m][c]^T + bias[m] (bias may be
 * NULL); backward gives din, dw [m][c], dbias [m]. */
int sp_linear_fwd(const float* d_in, const float* d_w, const float* d_bias, int32_t n_clouds, int32_t c, int32_t m,
                  float* d_out, void* stream);
int sp_linear_bwd(const float* d_in, const float* d_w, const float* d_dout, int32_t n_clouds, int32_t c, int32_t m,
                  float* d_din, float* d_dw, float* d_dbias, void* stream);

/* Mean over the clouds of -log softmax(logits)[label]: d_loss [1], d_dlogits [n_clouds][m] (gradient of the
 * mean loss).  labels int32 [n_clouds] in [0, m). */
int sp_softmax_ce(const float* d_logits, const int32_t* d_labels, int32_t n_clouds, int32_t m, float* d_loss,
                  float* d_dlogits, void* stream);

/* ---- stage-boundary packing of a sparse tensor (Sec. III-B, last paragraph: the coordinate matrix and the
 * feature matrix are what is exchanged between pipeline stages) ---------------------------------------------
 * (C, F) -> one contiguous device buffer that any transport can send as a single message, and back.  Layout,
 * little-endian, every section 256-byte aligned, padding zero:
 *   0 "SPCF" | 4 u32 version (1) | 8 i64 n | 16 i32 channels | 20 i32 dtype | 24 i32 tensor stride | 28 0 |
 *   32 i64 coordinates offset (256) | 40 i64 features offset | 48 i64 total bytes | 56..255 0 |
 *   coordinates int32 [n][4] | features [n][channels]
 * sp_pack_bytes: size of the buffer (-1 for invalid sizes).  sp_pack: one kernel launch, no synchronisation;
 * d_buf (caller-owned, >= sp_pack_bytes, 256-byte aligned) is fully written, header included.
 * sp_unpack_info: reads the header back to the host (synchronises `stream`) and validates it.
 * sp_unpack: one kernel launch; d_coords int32 [n][4] and d_feats [n][c] are caller-owned; n, c, dt are the
 * header's values as sp_unpack_info returned them. */
int64_t sp_pack_bytes(int64_t n, int32_t c, sp_dtype dt);
int sp_pack(const int32_t* d_coords, const void* d_feats, int64_t n, int32_t c, sp_dtype dt, int32_t tensor_stride,
            void* d_buf, void* stream);
int sp_unpack_info(const void* d_buf, void* stream, int64_t* n, int32_t* c, sp_dtype* dt, int32_t* tensor_stride,
                   int64_t* total_bytes);
int sp_unpack(const void* d_buf, int64_t n, int32_t c, sp_dtype dt, int32_t* d_coords, void* d_feats, void* stream);

/* ---- housekeeping -------------------------------------------------------------------------------------- */
const char* sp_last_error(void);  /* message of the calling thread's last failure ("" if none) */

/* Device memory.  By default handles and per-call scratch come from a caching pool inside the library
 * (hipMalloc on a miss; a freed block is reused at once by the stream that used it last, and by another
 * stream only after that stream has been made to wait for the first).  sp_set_allocator installs the caller's
 * allocator instead (for instance a framework's caching allocator, so that one allocator owns all device
 * memory): alloc(bytes, stream, ctx) returns device memory, at least 256-byte aligned, that may be used by
 * work enqueued on `stream` from now on, or NULL on failure (reported as SP_ERR_ALLOC); free_(ptr, ctx) is
 * called when the library drops the block, possibly while the last kernels using it are still in flight on
 * the stream it was allocated for (the semantics of stream-ordered caching allocators).  Both callbacks may
 * be called from any thread that calls the library.  Blocks taken from an allocator go back to that same
 * allocator even if another one has been installed since.  NULL, NULL restores the pool. */
typedef void* (*sp_alloc_fn)(size_t bytes, void* stream, void* ctx);
typedef void (*sp_free_fn)(void* ptr, void* ctx);
int sp_set_allocator(sp_alloc_fn alloc, sp_free_fn free_, void* ctx);

int sp_pool_trim(void);           /* synchronises the device and frees all cached (unused) device memory */
int64_t sp_pool_bytes(void);      /* device bytes currently held by the pool (in use + cached) */
int64_t sp_pool_cross_stream(void); /* blocks handed from one stream to another so far (diagnostics) */
const char* sp_version(void);
/* Name of the gather kernel that sp_conv_fwd (direction 0) or sp_conv_bwd_data (direction 1) launches for this
 * map and these channel counts ("" for invalid arguments).  For benchmarks and profiles that must name the
 * kernel they time; the choice itself is the library's and may change between versions. */
const char* sp_conv_kernel_name(const sp_kmap_t* m, int32_t cin, int32_t cout, sp_dtype dt, int32_t direction);
/* Measured matrix-core roof of this GPU, for benchmarks that quote a fraction of it: runs a loop of independent
 * register-resident MFMAs (SP_F32: v_mfma_f32_16x16x4_f32; SP_BF16: v_mfma_f32_16x16x32_bf16) on every SIMD for about a
 * millisecond on `stream`, waits for it, and writes the rate in TFLOP/s to *tflops (host pointer).  No operands
 * come from memory.  Allocates 4 KB from the pool. */
int sp_measure_mfma_peak(sp_dtype dt, void* stream, double* tflops);

#ifdef __cplusplus
}
#endif
#endif /* SP_CONV_H */
