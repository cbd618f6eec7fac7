/*
 * CPU oracle for convolution on native points (PointCNN++), in binary64.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition of what
 * the GPU library computes.  It shares no code with the GPU path and is used
 * by the tests, by the smoke check and by the benchmark's cpu_baseline leg;
 * nothing in the product path may call it.
 *
 * What it follows:
 *   - triplet set T: Sec. 3.2 "Definition" (centres at the original output
 *     points, neighbourhood search in continuous space, local voxelisation
 *     centred on the output point at the kernel's resolution) with the fixed
 *     radius search of Sec. 4.1;
 *   - forward:        Eq. (1), Sec. 3.1.1   out[o] = sum_{(o,i,k)} W[k] x[i]
 *   - backward input: first gradient equation of Sec. 3.3.3
 *                     dx[i] = sum_{(o,i,k)} W[k]^T dy[o]
 *   - backward weight: Eq. (5), Sec. 3.3.3  dW[k] = sum_{(o,i,k)} dy[o] (x) x[i]
 *
 * Readings where the paper is silent (shared with the GPU library by
 * convention, not by code):
 *   - neighbourhood = closed Euclidean ball: |d|^2 <= r^2, d = in - out;
 *   - the test is evaluated in binary64 on the binary32 inputs, as
 *     (dx*dx + dy*dy) + dz*dz <= (double)r*(double)r, no fused multiply-add;
 *   - the local grid has t x t x t cells tiling the cube [-r, r]^3 centred on
 *     the output point; cell along one axis = floor((d + r) * (t / (2 r))),
 *     clamped to [0, t-1], so a point on an interior face goes to the upper
 *     cell and d = +r falls in cell t-1;
 *   - k = (cx * t + cy) * t + cz, offset taken as input minus output
 *     (cross-correlation, no flip);
 *   - coincident points and the self pair are ordinary triplets;
 *   - T is listed in ascending (k, o, i) order; seg_offsets[k] is the start of
 *     cell k's run, seg_offsets[K] = |T|;
 *   - no normalisation, bias or activation.
 *
 * Parity status: the ball predicate, the sign of the offset, the x-slowest
 * linearisation and Eq. (1)/(4)/(5) are pinned by the CPU tests (dense conv3d
 * on a lattice, neighbour counts against a k-d tree, sparse-matrix products,
 * adjoint identities, hand-derived cells).  The tie rule at cell faces and the
 * (k, o, i) listing order are conventions with no external truth:
 * "parity unpinned" for those two choices.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (see build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Cell of offset d along one axis of the local grid (Sec. 3.2, item 3). */
static inline int axis_cell(double d, double R, double inv, int t)
{
    double u = (d + R) * inv;
    double f = floor(u);
    int c = (int)f;
    if (f < 0.0) c = 0;
    if (c > t - 1) c = t - 1;
    return c;
}

/*
 * Brute-force O(n_out * n_in) triplet construction.
 * Returns |T|.  When tri_o/tri_i/tri_k are NULL only the count is returned.
 * When |T| > capacity nothing is written and |T| is still returned.
 */
int64_t oracle_build_triplets(const float *in_xyz, int64_t n_in,
                              const float *out_xyz, int64_t n_out,
                              float radius, int t,
                              int32_t *tri_o, int32_t *tri_i, int32_t *tri_k,
                              int64_t capacity, int64_t *seg_offsets)
{
    const double R = (double)radius;
    const double r2 = R * R;
    const double inv = (double)t / (2.0 * R);
    const int K = t * t * t;

    int64_t *row = (int64_t *)calloc((size_t)n_out + 1, sizeof(int64_t));
    if (!row) return -1;

    /* pass 1: neighbours per output */
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t o = 0; o < n_out; ++o) {
        const double ox = (double)out_xyz[3 * o], oy = (double)out_xyz[3 * o + 1], oz = (double)out_xyz[3 * o + 2];
        int64_t c = 0;
        for (int64_t i = 0; i < n_in; ++i) {
            double dx = (double)in_xyz[3 * i] - ox;
            double dy = (double)in_xyz[3 * i + 1] - oy;
            double dz = (double)in_xyz[3 * i + 2] - oz;
            double d2 = (dx * dx + dy * dy) + dz * dz;
            c += (d2 <= r2);
        }
        row[o + 1] = c;
    }
    for (int64_t o = 0; o < n_out; ++o) row[o + 1] += row[o];
    const int64_t total = row[n_out];
    if (!tri_o || !tri_i || !tri_k || total > capacity) {
        free(row);
        return total;
    }

    /* pass 2: list (o, i, k) with o ascending, i ascending inside each o */
    int32_t *lo = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
    int32_t *li = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
    int32_t *lk = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
    if (!lo || !li || !lk) { free(row); free(lo); free(li); free(lk); return -1; }
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t o = 0; o < n_out; ++o) {
        const double ox = (double)out_xyz[3 * o], oy = (double)out_xyz[3 * o + 1], oz = (double)out_xyz[3 * o + 2];
        int64_t p = row[o];
        for (int64_t i = 0; i < n_in; ++i) {
            double dx = (double)in_xyz[3 * i] - ox;
            double dy = (double)in_xyz[3 * i + 1] - oy;
            double dz = (double)in_xyz[3 * i + 2] - oz;
            double d2 = (dx * dx + dy * dy) + dz * dz;
            if (d2 <= r2) {
                int cx = axis_cell(dx, R, inv, t);
                int cy = axis_cell(dy, R, inv, t);
                int cz = axis_cell(dz, R, inv, t);
                lo[p] = (int32_t)o;
                li[p] = (int32_t)i;
                lk[p] = (cx * t + cy) * t + cz;
                ++p;
            }
        }
    }

    /* stable counting sort on k: (o, i) order is kept inside each k, giving (k, o, i) */
    int64_t *start = (int64_t *)calloc((size_t)K + 1, sizeof(int64_t));
    for (int64_t p = 0; p < total; ++p) start[lk[p] + 1]++;
    for (int k = 0; k < K; ++k) start[k + 1] += start[k];
    if (seg_offsets) memcpy(seg_offsets, start, ((size_t)K + 1) * sizeof(int64_t));
    for (int64_t p = 0; p < total; ++p) {
        int64_t q = start[lk[p]]++;
        tri_o[q] = lo[p];
        tri_i[q] = li[p];
        tri_k[q] = lk[p];
    }
    free(start); free(lo); free(li); free(lk); free(row);
    return total;
}

/* Eq. (1): out[o, co] = sum over triplets of sum_ci W[k, co, ci] * x[i, ci].  out is overwritten. */
void oracle_mvmr_fwd(const double *x, const double *w, double *out,
                     int64_t n_in, int64_t n_out, int c_in, int c_out, int K,
                     const int32_t *tri_o, const int32_t *tri_i, const int32_t *tri_k,
                     int64_t n_triplets)
{
    (void)n_in; (void)K;
    memset(out, 0, (size_t)n_out * (size_t)c_out * sizeof(double));
    /* output channels are independent: one thread per channel, triplets in list order */
#pragma omp parallel for schedule(static)
    for (int co = 0; co < c_out; ++co) {
        for (int64_t p = 0; p < n_triplets; ++p) {
            const double *wr = w + ((size_t)tri_k[p] * c_out + co) * c_in;
            const double *xr = x + (size_t)tri_i[p] * c_in;
            double s = 0.0;
            for (int ci = 0; ci < c_in; ++ci) s += wr[ci] * xr[ci];
            out[(size_t)tri_o[p] * c_out + co] += s;
        }
    }
}

/* Sec. 3.3.3, gradient w.r.t. the input features: dx[i, ci] = sum W[k, co, ci] * dy[o, co]. */
void oracle_mvmr_bwd_input(const double *dy, const double *w, double *dx,
                           int64_t n_in, int64_t n_out, int c_in, int c_out, int K,
                           const int32_t *tri_o, const int32_t *tri_i, const int32_t *tri_k,
                           int64_t n_triplets)
{
    (void)n_out; (void)K;
    memset(dx, 0, (size_t)n_in * (size_t)c_in * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int ci = 0; ci < c_in; ++ci) {
        for (int64_t p = 0; p < n_triplets; ++p) {
            const double *wk = w + (size_t)tri_k[p] * c_out * c_in;
            const double *g = dy + (size_t)tri_o[p] * c_out;
            double s = 0.0;
            for (int co = 0; co < c_out; ++co) s += wk[(size_t)co * c_in + ci] * g[co];
            dx[(size_t)tri_i[p] * c_in + ci] += s;
        }
    }
}

/* Eq. (5): dW[k, co, ci] = sum over triplets with cell k of dy[o, co] * x[i, ci]. */
void oracle_mvmr_bwd_weight(const double *x, const double *dy, double *dw,
                            int64_t n_in, int64_t n_out, int c_in, int c_out, int K,
                            const int32_t *tri_o, const int32_t *tri_i, const int32_t *tri_k,
                            int64_t n_triplets)
{
    (void)n_in; (void)n_out;
    memset(dw, 0, (size_t)K * (size_t)c_out * (size_t)c_in * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int co = 0; co < c_out; ++co) {
        for (int64_t p = 0; p < n_triplets; ++p) {
            double g = dy[(size_t)tri_o[p] * c_out + co];
            const double *xr = x + (size_t)tri_i[p] * c_in;
            double *d = dw + ((size_t)tri_k[p] * c_out + co) * c_in;
            for (int ci = 0; ci < c_in; ++ci) d[ci] += g * xr[ci];
        }
    }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
