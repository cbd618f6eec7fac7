/*
 * CPU oracle, second part: the variants around the main path -- TEST INFRASTRUCTURE ONLY (see pcpp_oracle.c).
 *
 *   - batches of clouds held as one concatenated array plus offsets (the jagged representation of Sec. 4.1,
 *     implementation details): a triplet pairs points of the same cloud only;
 *   - the "degraded" operator of Sec. 3.2 ("Voxel Convolution as a Special Case"; "Ours (degraded)" in Sec. 4.2):
 *     the three degradations that turn convolution on native points into convolution on sparse voxels --
 *     centres snapped to the voxels of a global voxelisation of pitch v, neighbours searched in voxel space
 *     (Chebyshev distance), kernel resolution tied to the voxels of the receptive field;
 *   - voxel-grid down-sampling that keeps original coordinates (Sec. 4.1): one point per occupied voxel.
 *
 * Readings where the paper is silent:
 *   - voxel of a point along one axis = floor((double)p / (double)v), in binary64;
 *   - voxel mode, t odd, h = (t - 1) / 2: input i is a neighbour of output o iff its voxel differs from o's by at
 *     most h along every axis; cell c_a = (vox_in_a - vox_out_a) + h, k = (c_x * t + c_y) * t + c_z (x slowest,
 *     offset input minus output, as in the native operator).  Only the voxels enter: where inside its voxel a
 *     point lies makes no difference (that is degradation 1), several input points of one voxel all land in the
 *     same cell;
 *   - down-sampling keeps the point with the lowest index of every occupied voxel and lists the kept indices in
 *     ascending order.
 * Parity status: the voxel mode is pinned against a dense conv3d on the occupancy lattice and against a
 * dictionary-based sparse convolution written independently in the tests; with one batch and the ball mode this
 * file must reproduce pcpp_oracle.c's list exactly (tested); the subsampling is pinned against numpy.unique.
 * The choice of floor(p / v) (rather than a multiplication by 1 / v) at voxel faces is a convention:
 * "parity unpinned" for points that lie exactly on a face in one formula and not in the other.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MODE_BALL  0
#define ORACLE_MODE_VOXEL 1

static inline int axis_cell_ball(double d, double R, double inv, int t)
{
    double f = floor((d + R) * inv);
    int c = (int)f;
    if (f < 0.0) c = 0;
    if (c > t - 1) c = t - 1;
    return c;
}

/* cell of the pair (output o, input i), or -1 when i is not a neighbour of o */
static int pair_cell(const float *pi, const float *po, double size, int t, int mode)
{
    if (mode == ORACLE_MODE_BALL) {
        const double R = size, inv = (double)t / (2.0 * R);
        double dx = (double)pi[0] - (double)po[0];
        double dy = (double)pi[1] - (double)po[1];
        double dz = (double)pi[2] - (double)po[2];
        double d2 = (dx * dx + dy * dy) + dz * dz;
        if (!(d2 <= R * R)) return -1;
        return (axis_cell_ball(dx, R, inv, t) * t + axis_cell_ball(dy, R, inv, t)) * t + axis_cell_ball(dz, R, inv, t);
    }
    const int h = (t - 1) / 2;
    int c[3];
    for (int a = 0; a < 3; ++a) {
        const double vi = floor((double)pi[a] / size), vo = floor((double)po[a] / size);
        const double dv = vi - vo;
        if (dv < -(double)h || dv > (double)h) return -1;
        c[a] = (int)dv + h;
    }
    return (c[0] * t + c[1]) * t + c[2];
}

/*
 * Brute-force triplet construction over a batch of clouds.  Cloud b owns inputs [in_off[b], in_off[b+1]) and
 * outputs [out_off[b], out_off[b+1]) of the concatenated arrays.  size = radius (ball mode) or voxel pitch (voxel
 * mode).  List in (k, o, i) order, indices into the concatenated arrays.  Returns |T|; writes nothing when the
 * arrays are NULL or |T| > capacity.  Returns -2 for voxel mode with an even t.
 */
int64_t oracle_build_triplets_general(const float *in_xyz, const float *out_xyz,
                                      const int64_t *in_off, const int64_t *out_off, int n_batches,
                                      float size, int t, int mode,
                                      int32_t *tri_o, int32_t *tri_i, int32_t *tri_k,
                                      int64_t capacity, int64_t *seg_offsets)
{
    const int K = t * t * t;
    if (mode == ORACLE_MODE_VOXEL && t % 2 == 0) return -2;
    int64_t total = 0;
    for (int pass = 0; pass < 2; ++pass) {
        int64_t p = 0;
        /* (o, i) ascending; the stable counting sort below then yields (k, o, i) */
        int32_t *lo = NULL, *li = NULL, *lk = NULL;
        if (pass == 1) {
            if (!tri_o || !tri_i || !tri_k || total > capacity) return total;
            lo = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * 4);
            li = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * 4);
            lk = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * 4);
            if (!lo || !li || !lk) { free(lo); free(li); free(lk); return -1; }
        }
        for (int b = 0; b < n_batches; ++b)
            for (int64_t o = out_off[b]; o < out_off[b + 1]; ++o)
                for (int64_t i = in_off[b]; i < in_off[b + 1]; ++i) {
                    const int k = pair_cell(in_xyz + 3 * i, out_xyz + 3 * o, (double)size, t, mode);
                    if (k < 0) continue;
                    if (pass == 1) { lo[p] = (int32_t)o; li[p] = (int32_t)i; lk[p] = k; }
                    ++p;
                }
        if (pass == 0) { total = p; continue; }
        int64_t *start = (int64_t *)calloc((size_t)K + 1, sizeof(int64_t));
        for (int64_t q = 0; q < total; ++q) start[lk[q] + 1]++;
        for (int k = 0; k < K; ++k) start[k + 1] += start[k];
        if (seg_offsets) memcpy(seg_offsets, start, ((size_t)K + 1) * sizeof(int64_t));
        for (int64_t q = 0; q < total; ++q) {
            const int64_t d = start[lk[q]]++;
            tri_o[d] = lo[q]; tri_i[d] = li[q]; tri_k[d] = lk[q];
        }
        free(start); free(lo); free(li); free(lk);
    }
    return total;
}

/*
 * Voxel-grid down-sampling with original coordinates kept (Sec. 4.1): for every occupied voxel of pitch v the
 * lowest point index; kept[] ascending.  O(n^2) on purpose: a point is kept iff no earlier point shares its voxel.
 * Returns the number of kept points (kept may be NULL).
 */
int64_t oracle_voxel_subsample(const float *xyz, int64_t n, float pitch, int32_t *kept)
{
    int64_t m = 0;
    for (int64_t p = 0; p < n; ++p) {
        const double v = (double)pitch;
        const double ax = floor((double)xyz[3 * p] / v), ay = floor((double)xyz[3 * p + 1] / v), az = floor((double)xyz[3 * p + 2] / v);
        int first = 1;
        for (int64_t q = 0; q < p && first; ++q)
            if (floor((double)xyz[3 * q] / v) == ax && floor((double)xyz[3 * q + 1] / v) == ay && floor((double)xyz[3 * q + 2] / v) == az)
                first = 0;
        if (first) { if (kept) kept[m] = (int32_t)p; ++m; }
    }
    return m;
}
