/*
 * CPU oracle for sparse convolution on voxelized point clouds.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * tests, the smoke check and the benchmark's cpu_baseline leg compare the GPU
 * library against.  It shares no code with the GPU path and the product never
 * calls it.
 *
 * What it computes, and where the paper defines it:
 *   - kernel-offset set Delta^3(K) and the sparse convolution sum      (Sec. 2, Eq. 1)
 *   - output coordinates for stride s                                   (Sec. 2.1.1, Alg. 3)
 *   - kernel maps M = {(j, k, n)} with p_j = s*q_k + delta_n            (Sec. 2.1.2, Alg. 1)
 *
 * How: coordinates are indexed by sorting (b,x,y,z) tuples lexicographically
 * and looked up by binary search (no hashing, no key packing).  Features are
 * the direct evaluation of Eq. 1: one output row at a time, one kernel offset
 * at a time, accumulated in double.  OpenMP, when enabled, splits output rows
 * across threads and changes no arithmetic.
 *
 * Conventions (the paper leaves these open; they are this build's readings):
 *   - coords are int32 [N,4] = (batch, x, y, z); the batch index is never
 *     offset or strided, and points with different batch never interact.
 *   - Delta^3(K) = {-r .. K-1-r}^3 with r = floor((K-1)/2): {-1,0,1}^3 for
 *     K=3 (as printed in Sec. 2), {0,1}^3 for K=2 (even K is not defined in
 *     the paper).
 *   - weight index n = ((dx+r)*K + (dy+r))*K + (dz+r), x slowest.
 *   - Alg. 3's boundary check: with a boundary b (three positive ints) a candidate u is kept
 *     when 0 <= u < s*b on every axis, i.e. outputs live on the grid [0, b) (the listing prints
 *     the upper test only; its coordinates are never negative).  Without b nothing is cut.
 *   - Unique() returns the outputs in ascending lexicographic (b,x,y,z) order.
 *   - transposed convolution (not in the paper): same pair set as the forward
 *     strided convolution between the fine and the coarse set, roles swapped:
 *     y_j = sum over (k,n) with p_j = s*q_k + delta_n of x_k * W_n.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t c[4];
    int64_t idx;
} orc_pt;

static int orc_cmp_coord(const int32_t *a, const int32_t *b) {
    for (int d = 0; d < 4; ++d) {
        if (a[d] < b[d]) return -1;
        if (a[d] > b[d]) return 1;
    }
    return 0;
}

static int orc_cmp_pt(const void *a, const void *b) {
    return orc_cmp_coord(((const orc_pt *)a)->c, ((const orc_pt *)b)->c);
}

/* Sorted index over a coordinate list.  Returns NULL on allocation failure. */
static orc_pt *orc_index_build(const int32_t *coords, int64_t n) {
    orc_pt *pts = (orc_pt *)malloc((size_t)(n > 0 ? n : 1) * sizeof(orc_pt));
    if (!pts) return NULL;
    for (int64_t i = 0; i < n; ++i) {
        memcpy(pts[i].c, coords + 4 * i, 4 * sizeof(int32_t));
        pts[i].idx = i;
    }
    qsort(pts, (size_t)n, sizeof(orc_pt), orc_cmp_pt);
    return pts;
}

/* Row index of coordinate r in the indexed list, or -1. */
static int64_t orc_index_find(const orc_pt *pts, int64_t n, const int32_t r[4]) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        int c = orc_cmp_coord(pts[mid].c, r);
        if (c == 0) return pts[mid].idx;
        if (c < 0) lo = mid + 1; else hi = mid;
    }
    return -1;
}

static int orc_has_duplicates(const orc_pt *pts, int64_t n) {
    for (int64_t i = 1; i < n; ++i)
        if (orc_cmp_coord(pts[i - 1].c, pts[i].c) == 0) return 1;
    return 0;
}

/* Kernel offset delta_n of Delta^3(K) (Sec. 2), n = ((dx+r)K + (dy+r))K + (dz+r). */
void orc_offset(int K, int n, int32_t d[3]) {
    int r = (K - 1) / 2;
    d[0] = n / (K * K) - r;
    d[1] = (n / K) % K - r;
    d[2] = n % K - r;
}

/*
 * Output coordinates (Alg. 3).  s == 1: P_out = P_in in the same order.
 * s > 1: every u = p - delta whose x,y,z are all divisible by s yields the
 * candidate u/s; the result is the sorted set of distinct candidates.
 * Writes at most cap rows to out (out may be NULL when cap == 0) and returns
 * the number of outputs, or -1 on allocation failure.
 */
int64_t orc_out_coords(const int32_t *in, int64_t n_in, int K, int s, const int32_t *boundary, int32_t *out,
                       int64_t cap) {
    if (s == 1) {
        int64_t w = n_in < cap ? n_in : cap;
        if (w > 0) memcpy(out, in, (size_t)w * 4 * sizeof(int32_t));
        return n_in;
    }
    int K3 = K * K * K;
    orc_pt *cand = (orc_pt *)malloc((size_t)(n_in * K3 + 1) * sizeof(orc_pt));
    if (!cand) return -1;
    int64_t nc = 0;
    for (int64_t i = 0; i < n_in; ++i) {
        const int32_t *p = in + 4 * i;
        for (int n = 0; n < K3; ++n) {
            int32_t d[3], u[3];
            orc_offset(K, n, d);
            int ok = 1;
            for (int a = 0; a < 3; ++a) {
                u[a] = p[1 + a] - d[a];
                if (u[a] % s != 0) ok = 0;
                if (boundary && (u[a] < 0 || (int64_t)u[a] >= (int64_t)s * boundary[a])) ok = 0;
            }
            if (!ok) continue;
            cand[nc].c[0] = p[0];
            for (int a = 0; a < 3; ++a) cand[nc].c[1 + a] = u[a] / s;
            cand[nc].idx = 0;
            ++nc;
        }
    }
    qsort(cand, (size_t)nc, sizeof(orc_pt), orc_cmp_pt);
    int64_t n_out = 0;
    for (int64_t i = 0; i < nc; ++i) {
        if (i > 0 && orc_cmp_coord(cand[i - 1].c, cand[i].c) == 0) continue;
        if (n_out < cap) memcpy(out + 4 * n_out, cand[i].c, 4 * sizeof(int32_t));
        ++n_out;
    }
    free(cand);
    return n_out;
}

/*
 * Map search (Alg. 1): for every output k (in order) and every offset n (in
 * order), r = s*q_k + delta_n; if r is an input point j, emit (j, k, n).
 * Writes at most cap triples (3 int32 each) and returns M; -1 on allocation
 * failure, -2 if the input coordinates are not distinct.
 */
int64_t orc_kmap(const int32_t *in, int64_t n_in, const int32_t *out, int64_t n_out, int K, int s,
                 int32_t *triples, int64_t cap) {
    orc_pt *idx = orc_index_build(in, n_in);
    if (!idx) return -1;
    if (orc_has_duplicates(idx, n_in)) { free(idx); return -2; }
    int K3 = K * K * K;
    int64_t m = 0;
    for (int64_t k = 0; k < n_out; ++k) {
        const int32_t *q = out + 4 * k;
        for (int n = 0; n < K3; ++n) {
            int32_t d[3], r[4];
            orc_offset(K, n, d);
            r[0] = q[0];
            for (int a = 0; a < 3; ++a) r[1 + a] = s * q[1 + a] + d[a];
            int64_t j = orc_index_find(idx, n_in, r);
            if (j < 0) continue;
            if (m < cap) {
                triples[3 * m + 0] = (int32_t)j;
                triples[3 * m + 1] = (int32_t)k;
                triples[3 * m + 2] = (int32_t)n;
            }
            ++m;
        }
    }
    free(idx);
    return m;
}

/*
 * Sparse convolution (Eq. 1), forward:
 *   y_k = sum_n sum_j 1[p_j = s*q_k + delta_n] x_j W_n
 * X [n_in, c_in], W [K^3, c_in, c_out], Y [n_out, c_out], all double, row-major.
 * threads <= 0 keeps the OpenMP default.  Returns 0, -1 (allocation), -2 (duplicates).
 */
int orc_conv(const int32_t *in, int64_t n_in, const int32_t *out, int64_t n_out, int K, int s,
             const double *X, int c_in, const double *W, int c_out, double *Y, int threads) {
    orc_pt *idx = orc_index_build(in, n_in);
    if (!idx) return -1;
    if (orc_has_duplicates(idx, n_in)) { free(idx); return -2; }
    int K3 = K * K * K;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel for schedule(dynamic, 256)
#endif
    for (int64_t k = 0; k < n_out; ++k) {
        const int32_t *q = out + 4 * k;
        double *y = Y + (size_t)k * c_out;
        for (int co = 0; co < c_out; ++co) y[co] = 0.0;
        for (int n = 0; n < K3; ++n) {
            int32_t d[3], r[4];
            orc_offset(K, n, d);
            r[0] = q[0];
            for (int a = 0; a < 3; ++a) r[1 + a] = s * q[1 + a] + d[a];
            int64_t j = orc_index_find(idx, n_in, r);
            if (j < 0) continue;
            const double *x = X + (size_t)j * c_in;
            const double *w = W + (size_t)n * c_in * c_out;
            for (int ci = 0; ci < c_in; ++ci)
                for (int co = 0; co < c_out; ++co)
                    y[co] += x[ci] * w[(size_t)ci * c_out + co];
        }
    }
    free(idx);
    (void)threads;
    return 0;
}

/*
 * Transposed sparse convolution: fine points p_j are the outputs, coarse
 * points q_k the inputs, and the pair set is that of the forward (K, s)
 * convolution fine -> coarse:
 *   y_j = sum_n sum_k 1[p_j = s*q_k + delta_n] x_k W_n
 * For each fine point and offset, u = p_j - delta_n must be divisible by s and
 * u/s must be a coarse point.
 * X [n_coarse, c_in], W [K^3, c_in, c_out], Y [n_fine, c_out].
 */
int orc_conv_transposed(const int32_t *fine, int64_t n_fine, const int32_t *coarse, int64_t n_coarse,
                        int K, int s, const double *X, int c_in, const double *W, int c_out,
                        double *Y, int threads) {
    orc_pt *idx = orc_index_build(coarse, n_coarse);
    if (!idx) return -1;
    if (orc_has_duplicates(idx, n_coarse)) { free(idx); return -2; }
    int K3 = K * K * K;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel for schedule(dynamic, 256)
#endif
    for (int64_t j = 0; j < n_fine; ++j) {
        const int32_t *p = fine + 4 * j;
        double *y = Y + (size_t)j * c_out;
        for (int co = 0; co < c_out; ++co) y[co] = 0.0;
        for (int n = 0; n < K3; ++n) {
            int32_t d[3], q[4];
            orc_offset(K, n, d);
            int ok = 1;
            q[0] = p[0];
            for (int a = 0; a < 3; ++a) {
                int32_t u = p[1 + a] - d[a];
                if (u % s != 0) ok = 0;
                q[1 + a] = u / s;
            }
            if (!ok) continue;
            int64_t k = orc_index_find(idx, n_coarse, q);
            if (k < 0) continue;
            const double *x = X + (size_t)k * c_in;
            const double *w = W + (size_t)n * c_in * c_out;
            for (int ci = 0; ci < c_in; ++ci)
                for (int co = 0; co < c_out; ++co)
                    y[co] += x[ci] * w[(size_t)ci * c_out + co];
        }
    }
    free(idx);
    (void)threads;
    return 0;
}

/* Number of threads the OpenMP loops will use (1 without OpenMP). */
int orc_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
