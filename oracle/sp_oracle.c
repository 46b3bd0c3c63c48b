/*
 * CPU oracle for the generalized sparse convolution (Sec. III-B).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the
 * HIP library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.
 *
 * What it computes, and where the paper defines it:
 *   - sparse tensor (C, F): C is an int matrix of rows (b, x, y, z), batch index
 *     first; row j of F belongs to row j of C              (Sec. III-B, sparse tensor)
 *   - step 1: output coordinates from input coordinates, layer stride and the
 *     input tensor stride                                  (Sec. III-B, step 1)
 *   - step 2: for every kernel weight W_i the list of (input row, output row)
 *     pairs it links                                       (Sec. III-B, step 2)
 *   - step 3: x_out[u] = sum over offsets i with u+i in C_in of W_i x_in[u+i],
 *     for u in C_out                                       (Eq. 2)
 *   - backward: gradients w.r.t. inputs and weights follow by differentiating
 *     Eq. 2 (it is bilinear in x_in and W)                 (Sec. II-A)
 *
 * No hashing anywhere: coordinates are looked up by sorting + binary search.
 * Floating point accumulates in double, in the order the definition states
 * (over kernel offsets, then over that offset's pairs).  No blocking, fusion
 * or threading.
 *
 * Readings where the paper is silent (listed in the design document too):
 *   - offsets of an odd kernel size K are {-(K-1)/2..(K-1)/2}^3 (the paper's
 *     V^1(3) = {-1,0,1}); of an even K they are {0..K-1}^3;
 *   - offset number k = (ax*K + ay)*K + az, z fastest, each axis low to high;
 *   - offsets are scaled by `step` = dilation * input tensor stride;
 *   - strided output coordinates are floor(c / S) * S per spatial axis (true
 *     floor), S = tensor stride * layer stride, duplicates merged;
 *   - merged rows keep first-occurrence order: unique row r is the r-th distinct
 *     coordinate met when walking the input rows in order.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- lexicographic order on (b,x,y,z) rows ------------------------------ */
static int cmp_row(const int32_t *a, const int32_t *b)
{
    for (int d = 0; d < 4; ++d) {
        if (a[d] < b[d]) return -1;
        if (a[d] > b[d]) return 1;
    }
    return 0;
}

typedef struct { int32_t c[4]; int64_t idx; } keyed_t;

static int cmp_keyed(const void *pa, const void *pb)
{
    const keyed_t *a = (const keyed_t *)pa, *b = (const keyed_t *)pb;
    int r = cmp_row(a->c, b->c);
    if (r) return r;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

static int32_t floor_to_multiple(int32_t v, int32_t s)
{
    /* floor(v / s) * s with a true floor (C's / truncates toward zero) */
    int32_t q = v / s;
    if ((v % s != 0) && ((v < 0) != (s < 0))) --q;
    return q * s;
}

/*
 * Merge duplicate coordinates (Sec. III-B sparse tensor; step 1 when floor_step > 1).
 *   raw        [n][4] rows (b,x,y,z)
 *   floor_step if > 1, x,y,z are first floored to a multiple of floor_step
 *   uniq       [n][4] out: distinct rows in first-occurrence order (first N rows valid)
 *   inverse    [n]    out: inverse[j] = unique row that raw row j merged into
 * Returns N, or -1 on allocation failure.
 */
int64_t sp_oracle_unique(const int32_t *raw, int64_t n, int32_t floor_step,
                         int32_t *uniq, int32_t *inverse)
{
    if (n == 0) return 0;
    keyed_t *s = (keyed_t *)malloc((size_t)n * sizeof(keyed_t));
    int64_t *rep = (int64_t *)malloc((size_t)n * sizeof(int64_t));   /* first raw row of j's group */
    int64_t *rank = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!s || !rep || !rank) { free(s); free(rep); free(rank); return -1; }
    for (int64_t j = 0; j < n; ++j) {
        s[j].c[0] = raw[4 * j];
        for (int d = 1; d < 4; ++d)
            s[j].c[d] = floor_step > 1 ? floor_to_multiple(raw[4 * j + d], floor_step) : raw[4 * j + d];
        s[j].idx = j;
    }
    qsort(s, (size_t)n, sizeof(keyed_t), cmp_keyed);
    /* equal coordinates are now adjacent, lowest raw index first */
    for (int64_t a = 0; a < n;) {
        int64_t b = a;
        while (b < n && cmp_row(s[a].c, s[b].c) == 0) { rep[s[b].idx] = s[a].idx; ++b; }
        a = b;
    }
    int64_t N = 0;
    for (int64_t j = 0; j < n; ++j) {
        if (rep[j] == j) {
            rank[j] = N;
            uniq[4 * N] = raw[4 * j];
            for (int d = 1; d < 4; ++d)
                uniq[4 * N + d] = floor_step > 1 ? floor_to_multiple(raw[4 * j + d], floor_step) : raw[4 * j + d];
            ++N;
        }
    }
    for (int64_t j = 0; j < n; ++j) inverse[j] = (int32_t)rank[rep[j]];
    free(s); free(rep); free(rank);
    return N;
}

/* kernel offset number k -> (ix,iy,iz), z fastest (see header) */
static void offset_of(int32_t k, int32_t K, int32_t off[3])
{
    int32_t az = k % K, ay = (k / K) % K, ax = k / (K * K);
    int32_t centre = (K % 2 == 1) ? (K - 1) / 2 : 0;
    off[0] = ax - centre; off[1] = ay - centre; off[2] = az - centre;
}

typedef struct { int32_t in, out; } pair_t;

static int cmp_pair(const void *pa, const void *pb)
{
    const pair_t *a = (const pair_t *)pa, *b = (const pair_t *)pb;
    if (a->in != b->in) return (a->in > b->in) - (a->in < b->in);
    return (a->out > b->out) - (a->out < b->out);
}

/*
 * Kernel map (Sec. III-B step 2; N^D(u, C_in) below Eq. 2):
 *   M_k = { (i, o) : c_in[i] = c_out[o] + offset_k * step, same batch index }.
 *   c_in  [n_in][4], distinct rows;  c_out [n_out][4], distinct rows
 *   K     kernel size per axis; step = dilation * input tensor stride
 *   pair_in / pair_out: out, lists of all k concatenated in k order, each sorted
 *                       by (in, out); may both be NULL to only count
 *   counts [K^3] out
 * Returns the total number of pairs, or -1 on allocation failure.
 */
int64_t sp_oracle_kmap(const int32_t *c_in, int64_t n_in, const int32_t *c_out, int64_t n_out,
                       int32_t K, int32_t step, int32_t *pair_in, int32_t *pair_out, int64_t *counts)
{
    int32_t kvol = K * K * K;
    int64_t total = 0;
    keyed_t *s = (keyed_t *)malloc((size_t)(n_in > 0 ? n_in : 1) * sizeof(keyed_t));
    pair_t *buf = (pair_t *)malloc((size_t)(n_out > 0 ? n_out : 1) * sizeof(pair_t));
    if (!s || !buf) { free(s); free(buf); return -1; }
    for (int64_t j = 0; j < n_in; ++j) { memcpy(s[j].c, c_in + 4 * j, 16); s[j].idx = j; }
    qsort(s, (size_t)n_in, sizeof(keyed_t), cmp_keyed);
    for (int32_t k = 0; k < kvol; ++k) {
        int32_t off[3];
        offset_of(k, K, off);
        int64_t cnt = 0;
        for (int64_t o = 0; o < n_out; ++o) {
            int32_t t[4];
            t[0] = c_out[4 * o];
            for (int d = 0; d < 3; ++d) t[d + 1] = c_out[4 * o + 1 + d] + off[d] * step;
            int64_t lo = 0, hi = n_in;          /* first sorted row >= t */
            while (lo < hi) {
                int64_t mid = lo + (hi - lo) / 2;
                if (cmp_row(s[mid].c, t) < 0) lo = mid + 1; else hi = mid;
            }
            if (lo < n_in && cmp_row(s[lo].c, t) == 0) {
                buf[cnt].in = (int32_t)s[lo].idx; buf[cnt].out = (int32_t)o; ++cnt;
            }
        }
        qsort(buf, (size_t)cnt, sizeof(pair_t), cmp_pair);
        if (pair_in && pair_out)
            for (int64_t p = 0; p < cnt; ++p) { pair_in[total + p] = buf[p].in; pair_out[total + p] = buf[p].out; }
        counts[k] = cnt;
        total += cnt;
    }
    free(s); free(buf);
    return total;
}

/*
 * Forward (Eq. 2 / step 3): Y[o,:] = sum_k sum_{(i,o) in M_k} W_k X[i,:].
 *   X [n_in][cin] float (values as stored: fp32, or bf16-representable fp32)
 *   W [kvol][cout][cin]  (K^D x N_out x N_in, Sec. III-B)
 *   Y [n_out][cout] double, overwritten
 */
void sp_oracle_conv_fwd(const int32_t *pair_in, const int32_t *pair_out, const int64_t *counts, int32_t kvol,
                        const float *X, const float *W, double *Y, int64_t n_out, int32_t cin, int32_t cout)
{
    memset(Y, 0, (size_t)n_out * (size_t)cout * sizeof(double));
    int64_t base = 0;
    for (int32_t k = 0; k < kvol; ++k) {
        const float *Wk = W + (size_t)k * cout * cin;
        for (int64_t p = base; p < base + counts[k]; ++p) {
            const float *x = X + (size_t)pair_in[p] * cin;
            double *y = Y + (size_t)pair_out[p] * cout;
            for (int32_t co = 0; co < cout; ++co) {
                double acc = 0.0;
                for (int32_t ci = 0; ci < cin; ++ci) acc += (double)Wk[(size_t)co * cin + ci] * (double)x[ci];
                y[co] += acc;
            }
        }
        base += counts[k];
    }
}

/*
 * Gradient w.r.t. the input features (derivative of Eq. 2 in x_in):
 *   dX[i,:] = sum_k sum_{(i,o) in M_k} W_k^T dY[o,:].   dX [n_in][cin] double, overwritten.
 */
void sp_oracle_conv_bwd_data(const int32_t *pair_in, const int32_t *pair_out, const int64_t *counts, int32_t kvol,
                             const float *dY, const float *W, double *dX, int64_t n_in, int32_t cin, int32_t cout)
{
    memset(dX, 0, (size_t)n_in * (size_t)cin * sizeof(double));
    int64_t base = 0;
    for (int32_t k = 0; k < kvol; ++k) {
        const float *Wk = W + (size_t)k * cout * cin;
        for (int64_t p = base; p < base + counts[k]; ++p) {
            const float *dy = dY + (size_t)pair_out[p] * cout;
            double *dx = dX + (size_t)pair_in[p] * cin;
            for (int32_t ci = 0; ci < cin; ++ci) {
                double acc = 0.0;
                for (int32_t co = 0; co < cout; ++co) acc += (double)Wk[(size_t)co * cin + ci] * (double)dy[co];
                dx[ci] += acc;
            }
        }
        base += counts[k];
    }
}

/*
 * Gradient w.r.t. the weights (derivative of Eq. 2 in W_i):
 *   dW_k[co][ci] = sum_{(i,o) in M_k} dY[o][co] * X[i][ci].   dW [kvol][cout][cin] double, overwritten.
 */
void sp_oracle_conv_bwd_weight(const int32_t *pair_in, const int32_t *pair_out, const int64_t *counts, int32_t kvol,
                               const float *X, const float *dY, double *dW, int32_t cin, int32_t cout)
{
    memset(dW, 0, (size_t)kvol * (size_t)cout * (size_t)cin * sizeof(double));
    int64_t base = 0;
    for (int32_t k = 0; k < kvol; ++k) {
        double *dWk = dW + (size_t)k * cout * cin;
        for (int64_t p = base; p < base + counts[k]; ++p) {
            const float *x = X + (size_t)pair_in[p] * cin;
            const float *dy = dY + (size_t)pair_out[p] * cout;
            for (int32_t co = 0; co < cout; ++co)
                for (int32_t ci = 0; ci < cin; ++ci)
                    dWk[(size_t)co * cin + ci] += (double)dy[co] * (double)x[ci];
        }
        base += counts[k];
    }
}
