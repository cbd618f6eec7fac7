// Triplet construction on the GPU: hashed uniform grid, fixed-radius query with local
// voxelisation (Sec. 3.2 "Definition"; fixed radius search of Sec. 4.1), and the reordering of
// Sec. 3.3.2 done as a counting sort on the composite key (k, centre): the query's count pass is
// the histogram, a prefix sum gives every (k, centre) run its place, the fill pass writes each
// triplet straight to its final position with ties ordered by the other index.
//
// This file is compiled with -ffp-contract=off: the inclusion test and the cell index are a fixed
// sequence of binary64 operations (see pcpp.h) and must not be fused.
#include <math.h>

#include "pcpp_internal.h"

namespace pcpp {

namespace {

constexpr unsigned long long EMPTY_KEY = ~0ull;
constexpr int CELL_BIAS = 1 << 20;
constexpr double CELL_CLAMP = (double)((1 << 20) - 2);   // +-1 stencil steps stay inside 21 bits
constexpr int SEARCH_THREADS = 1024;                      // 16 waves share a tile of 64 centres: 4 centres each
constexpr int SEARCH_WAVES = SEARCH_THREADS / 64;
constexpr int LIST_CAP_MAX = 512;                         // neighbours of one centre kept in LDS (per wave)

__device__ inline uint32_t hash_key(unsigned long long k)
{
    k ^= k >> 33; k *= 0xff51afd7ed558ccdULL;
    k ^= k >> 33; k *= 0xc4ceb9fe1a85ec53ULL;
    k ^= k >> 33;
    return (uint32_t)k;
}

__device__ inline int grid_coord(float p, double inv_g)
{
    double u = floor((double)p * inv_g);
    u = fmin(fmax(u, -CELL_CLAMP), CELL_CLAMP);      // NaN falls to a bound; no out-of-range key
    return (int)u;
}

__device__ inline unsigned long long pack_key(int cx, int cy, int cz)
{
    return ((unsigned long long)(uint32_t)(cx + CELL_BIAS) << 42) |
           ((unsigned long long)(uint32_t)(cy + CELL_BIAS) << 21) |
           (unsigned long long)(uint32_t)(cz + CELL_BIAS);
}

// Which cloud of a batch a point belongs to: the largest b with off[b] <= idx (off has n_batches + 1 entries).
__device__ inline int find_batch(const int32_t *__restrict__ off, int n_batches, int idx)
{
    int lo = 0, hi = n_batches - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (off[mid] <= idx) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Voxel of a coordinate in a global voxelisation of pitch v (voxel mode): floor(p / v) in binary64.
__device__ inline double voxel_of(float p, double v) { return floor(__ddiv_rn((double)p, v)); }

__device__ inline int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

// How points map to cells of the hashed grid.  Ball mode: cells of pitch 1 / inv_g (a hair above the radius).
// Voxel mode: cells of hp = max(h, 1) voxels per axis, so that voxels at most h apart lie in adjacent cells.
// With batches the cloud's number is mixed into the key: equal keys of different clouds are possible but harmless,
// because a centre only accepts candidates of its own cloud (their index range) and never probes two cells whose
// keys the mixing could make equal (it is a bijection within one cloud).
struct GridMap {
    double inv_g;
    double vox;       // voxel pitch, voxel mode only
    int hp;
    int voxel_mode;
};

__device__ inline void grid_cell3(float fx, float fy, float fz, const GridMap &m, int &gx, int &gy, int &gz)
{
    if (m.voxel_mode) {
        const double lim = CELL_CLAMP * (double)m.hp;
        gx = floor_div((int)fmin(fmax(voxel_of(fx, m.vox), -lim), lim), m.hp);
        gy = floor_div((int)fmin(fmax(voxel_of(fy, m.vox), -lim), lim), m.hp);
        gz = floor_div((int)fmin(fmax(voxel_of(fz, m.vox), -lim), lim), m.hp);
    } else {
        gx = grid_coord(fx, m.inv_g);
        gy = grid_coord(fy, m.inv_g);
        gz = grid_coord(fz, m.inv_g);
    }
}

__device__ inline unsigned long long mix_batch(unsigned long long key, int batch)
{
    key ^= (unsigned long long)(batch + 1) * 0x9E3779B97F4A7C15ull;
    return key == EMPTY_KEY ? key - 1ull : key;
}

// ---- hashed grid over the candidate set ------------------------------------------------------

// empty table: no keys, zero populations (slots + 1 entries, the input of the prefix sum), zero cursors;
// the first call of a build also zeroes the status words of all its prefix sums
__global__ __launch_bounds__(256) void grid_clear(unsigned long long *__restrict__ keys, uint32_t *__restrict__ cnt,
                                                  uint32_t *__restrict__ cursor, int64_t slots,
                                                  unsigned long long *__restrict__ scan_status, int64_t scan_words)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i <= slots; i += stride) {
        cnt[i] = 0u;
        if (i < slots) { keys[i] = EMPTY_KEY; cursor[i] = 0u; }
    }
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < scan_words; i += stride) scan_status[i] = 0ull;
}

__global__ __launch_bounds__(256) void grid_insert(const float *__restrict__ xyz, int64_t n, GridMap gm,
                                                   const int32_t *__restrict__ batch_off, int n_batches,
                                                   unsigned long long *__restrict__ keys,
                                                   uint32_t *__restrict__ slot_cnt, uint32_t mask,
                                                   uint32_t *__restrict__ point_slot)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    int gx, gy, gz;
    grid_cell3(xyz[3 * p], xyz[3 * p + 1], xyz[3 * p + 2], gm, gx, gy, gz);
    unsigned long long key = pack_key(gx, gy, gz);
    if (batch_off) key = mix_batch(key, find_batch(batch_off, n_batches, (int)p));
    uint32_t slot = hash_key(key) & mask;
    // the table has at least twice as many slots as points, so an empty slot is always reached
    for (;;) {
        unsigned long long prev = atomicCAS(&keys[slot], EMPTY_KEY, key);
        if (prev == EMPTY_KEY || prev == key) break;
        slot = (slot + 1) & mask;
    }
    atomicAdd(&slot_cnt[slot], 1u);
    point_slot[p] = slot;
}

__global__ __launch_bounds__(256) void grid_scatter(const float *__restrict__ xyz, int64_t n,
                                                    const uint32_t *__restrict__ point_slot,
                                                    const uint32_t *__restrict__ slot_start,
                                                    uint32_t *__restrict__ cursor, float4 *__restrict__ pts,
                                                    const uint32_t *__restrict__ err)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n || *err) return;                       // err: the slot offsets come from a prefix sum that gave up
    const uint32_t slot = point_slot[p];
    const uint32_t pos = slot_start[slot] + atomicAdd(&cursor[slot], 1u);
    pts[pos] = make_float4(xyz[3 * p], xyz[3 * p + 1], xyz[3 * p + 2], __int_as_float((int)p));
}

struct GridView {
    const unsigned long long *keys;
    const uint32_t *slot_start;   // [slots + 1]
    const float4 *pts;            // candidates grouped by grid cell; .w carries the original index
    uint32_t mask;
    GridMap map;
};

// Ball mode (Sec. 3.2 "Definition"): R, r2, inv_cell.  Voxel mode (the degraded operator of Sec. 3.2, "Voxel
// Convolution as a Special Case"): neighbours are the points whose voxel differs from the centre's by at most
// h = (t - 1) / 2 along every axis, the cell is the voxel offset (input minus output) plus h.
// Batches: c_off / d_off are the offsets of the clouds in the centre set and in the candidate set.
struct QueryParams {
    double R;         // (double)radius, or the voxel pitch
    double r2;        // R * R
    double inv_cell;  // t / (2 R)
    int t;
    int voxel_mode, h;
    const int32_t *c_off, *d_off;
    int n_batches;
};

__device__ inline uint32_t wave_incl_scan_u32(uint32_t v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t u = __shfl_up(v, d, 64);
        if (lane >= d) v += u;
    }
    return v;
}

// Candidates of one centre, held across the lanes of a wave: lane j < 27 owns stencil cell j.
// Every method must be called by all 64 lanes of the wave (it uses cross-lane reads).
// EXT: the voxel operator and batches of clouds are compiled in (the plain search kernels, which are bound by
// instruction issue, do without their tests).
template <bool SWAP, bool EXT>
struct Candidates {
    double cx, cy, cz;       // centre coordinate (ball mode) or its voxel (voxel mode)
    uint32_t my_start;       // lane j: first candidate of stencil cell j
    uint32_t my_excl;        // lane j: candidates in cells before j
    uint32_t total;
    int d_lo, d_hi;          // candidates of the centre's own cloud: indices [d_lo, d_hi)

    __device__ inline void open(const float *__restrict__ centres, int64_t a, const GridView &g, const QueryParams &q,
                                int lane)
    {
        const float fx = centres[3 * a], fy = centres[3 * a + 1], fz = centres[3 * a + 2];
        if (EXT && q.voxel_mode) { cx = voxel_of(fx, q.R); cy = voxel_of(fy, q.R); cz = voxel_of(fz, q.R); }
        else { cx = (double)fx; cy = (double)fy; cz = (double)fz; }
        int batch = 0;
        d_lo = 0; d_hi = 0x7fffffff;
        if (EXT && q.c_off) {
            batch = find_batch(q.c_off, q.n_batches, (int)a);
            d_lo = q.d_off[batch]; d_hi = q.d_off[batch + 1];
        }
        uint32_t cnt = 0;
        my_start = 0;
        if (lane < 27) {
            int gx, gy, gz;
            if constexpr (EXT) {
                grid_cell3(fx, fy, fz, g.map, gx, gy, gz);
            } else {
                gx = grid_coord(fx, g.map.inv_g); gy = grid_coord(fy, g.map.inv_g); gz = grid_coord(fz, g.map.inv_g);
            }
            gx += lane / 9 - 1; gy += (lane / 3) % 3 - 1; gz += lane % 3 - 1;
            unsigned long long key = pack_key(gx, gy, gz);
            if (EXT && q.c_off) key = mix_batch(key, batch);
            uint32_t slot = hash_key(key) & g.mask;
            for (;;) {
                const unsigned long long kk = g.keys[slot];
                if (kk == key) {
                    my_start = g.slot_start[slot];
                    cnt = g.slot_start[slot + 1] - my_start;
                    break;
                }
                if (kk == EMPTY_KEY) break;
                slot = (slot + 1) & g.mask;
            }
        }
        const uint32_t incl = wave_incl_scan_u32(cnt, lane);
        my_excl = incl - cnt;
        total = __shfl(incl, 63, 64);
    }

    // Candidate number idx (idx may differ per lane).  Returns whether it is a neighbour;
    // b = its original index, k = its kernel cell.  With MIRROR, k2 = the cell of the opposite offset, i.e.
    // the cell this pair falls in when the roles of the two points are swapped.
    __device__ inline bool fetch(uint32_t idx, const GridView &g, const QueryParams &q, int &b, int &k) const
    {
        int k2;
        return fetch2<false>(idx, g, q, b, k, k2);
    }

    // Ball mode, the pieces of the test.  d = input - output, in binary64, no contraction.
    __device__ inline void offset_of(const float4 &p, double &dx, double &dy, double &dz) const
    {
        dx = SWAP ? __dsub_rn(cx, (double)p.x) : __dsub_rn((double)p.x, cx);
        dy = SWAP ? __dsub_rn(cy, (double)p.y) : __dsub_rn((double)p.y, cy);
        dz = SWAP ? __dsub_rn(cz, (double)p.z) : __dsub_rn((double)p.z, cz);
    }
    __device__ static inline bool inside(double dx, double dy, double dz, const QueryParams &q)
    {
        return __dadd_rn(__dadd_rn(__dmul_rn(dx, dx), __dmul_rn(dy, dy)), __dmul_rn(dz, dz)) <= q.r2;
    }
    // kernel cell of the offset, and with MIRROR of the exactly negated offset (what the swapped subtraction gives)
    template <bool MIRROR>
    __device__ static inline void cells_of(double dx, double dy, double dz, const QueryParams &q, int &k, int &k2)
    {
        const int tm1 = q.t - 1;
        const double ux = floor(__dmul_rn(__dadd_rn(dx, q.R), q.inv_cell));
        const double uy = floor(__dmul_rn(__dadd_rn(dy, q.R), q.inv_cell));
        const double uz = floor(__dmul_rn(__dadd_rn(dz, q.R), q.inv_cell));
        int kx = ux < 0.0 ? 0 : (int)fmin(ux, (double)tm1);
        int ky = uy < 0.0 ? 0 : (int)fmin(uy, (double)tm1);
        int kz = uz < 0.0 ? 0 : (int)fmin(uz, (double)tm1);
        k = (kx * q.t + ky) * q.t + kz;
        if constexpr (MIRROR) {
            const double vx = floor(__dmul_rn(__dadd_rn(-dx, q.R), q.inv_cell));
            const double vy = floor(__dmul_rn(__dadd_rn(-dy, q.R), q.inv_cell));
            const double vz = floor(__dmul_rn(__dadd_rn(-dz, q.R), q.inv_cell));
            const int mx = vx < 0.0 ? 0 : (int)fmin(vx, (double)tm1);
            const int my = vy < 0.0 ? 0 : (int)fmin(vy, (double)tm1);
            const int mz = vz < 0.0 ? 0 : (int)fmin(vz, (double)tm1);
            k2 = (mx * q.t + my) * q.t + mz;
        }
    }

    template <bool MIRROR>
    __device__ inline bool fetch2(uint32_t idx, const GridView &g, const QueryParams &q, int &b, int &k, int &k2) const
    {
        const bool in_range = idx < total;
        const uint32_t id = in_range ? idx : 0u;
        int j = 0;
#pragma unroll
        for (int step = 16; step >= 1; step >>= 1) {
            const int c = j + step;
            const int cc = c <= 26 ? c : 26;
            const uint32_t e = __shfl(my_excl, cc, 64);
            if (c <= 26 && e <= id) j = c;
        }
        const uint32_t s = __shfl(my_start, j, 64);
        const uint32_t e = __shfl(my_excl, j, 64);
        bool hit = false;
        b = 0; k = 0; k2 = 0;
        if (in_range) {
            const float4 p = g.pts[s + (id - e)];
            b = __float_as_int(p.w);
            if (EXT && q.voxel_mode) {
                // voxel offset, input minus output; exact small integers in binary64
                const double vx = voxel_of(p.x, q.R), vy = voxel_of(p.y, q.R), vz = voxel_of(p.z, q.R);
                const double ox = SWAP ? cx - vx : vx - cx, oy = SWAP ? cy - vy : vy - cy, oz = SWAP ? cz - vz : vz - cz;
                const double hh = (double)q.h;
                hit = fabs(ox) <= hh && fabs(oy) <= hh && fabs(oz) <= hh && b >= d_lo && b < d_hi;
                if (hit) {
                    const int ix = (int)ox, iy = (int)oy, iz = (int)oz;
                    k = ((ix + q.h) * q.t + iy + q.h) * q.t + iz + q.h;
                    if constexpr (MIRROR) k2 = ((q.h - ix) * q.t + q.h - iy) * q.t + q.h - iz;
                }
                return hit;
            }
            double dx, dy, dz;
            offset_of(p, dx, dy, dz);
            hit = inside(dx, dy, dz, q) && (!EXT || (b >= d_lo && b < d_hi));
            cells_of<MIRROR>(dx, dy, dz, q, k, k2);
        }
        return hit;
    }
};

constexpr uint32_t SMALL_LIST = 160;      // up to this many neighbours the all-pairs rank is cheaper than bucketing
constexpr uint32_t KEEP_MAX = 256;        // longest neighbour list the count pass keeps per centre
constexpr uint32_t BUCKET_FROM = 64;      // ... and from here on bucketing through LDS adds is cheaper, when keys pack
constexpr int HIT_INDEX_BITS = 24;         // a stored hit = cell << 24 | candidate index
constexpr uint32_t HIT_INDEX_MASK = (1u << HIT_INDEX_BITS) - 1u;

// ---- pass 1: neighbours per (cell k, centre) --------------------------------------------------
// One block per tile of TILE centres, one wave per centre at a time.  Outputs of one side:
//   tile_cnt   [n_tiles][K][TILE]   (may be NULL: totals only)
//   tile_k_cnt [K * n_tiles]        k-major, input of the prefix sum
//   hits       [n_centres][hit_stride] (may be NULL): every centre's first neighbours, cell << 24 | index
// With BOTH (a cloud queried against itself) the same pass also fills the tables of the side with the roles
// swapped: the pair (centre c, candidate b) is the pair (centre c, other point b) of that side too, in the cell
// of the opposite offset.
struct CountOut {
    uint32_t *tile_cnt, *tile_k_cnt, *hits;
    uint32_t *n_hits;        // (may be NULL) [n_centres]: every centre's number of neighbours, with `hits`
};
// Lists that an earlier count pass over the same centres kept (indexed by centre, not by slot; same stride): a centre
// whose list is complete is counted from it without a search.  cand_xyz: the candidates' coordinates by index.
struct Reuse {
    const uint32_t *hits, *n_hits;
    const float *cand_xyz;
};

template <bool SWAP, bool BOTH, bool EXT>
__global__ __launch_bounds__(SEARCH_THREADS, 8) void query_count(const float *__restrict__ centres, int64_t n_centres,
                                                              const int32_t *__restrict__ perm,
                                                              GridView g, QueryParams q, int K, int64_t n_tiles,
                                                              CountOut side, CountOut mirror, uint32_t hit_stride,
                                                              const uint32_t *__restrict__ err, Reuse reuse)
{
    extern __shared__ uint32_t tbl[];          // [K][TILE], with BOTH followed by the mirror side's [K][TILE]
    __shared__ uint32_t stage[(BOTH ? 2 : 1) * SEARCH_WAVES * KEEP_MAX];   // hit lists on their way to memory
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = blockIdx.x;
    uint32_t *tbl2 = tbl + K * TILE;
    uint32_t *mine = stage + wave * KEEP_MAX, *mine2 = stage + (SEARCH_WAVES + wave) * KEEP_MAX;
    if (*err) return;                              // block-uniform: the grid's offsets are not to be trusted
    for (int idx = threadIdx.x; idx < (BOTH ? 2 : 1) * K * TILE; idx += SEARCH_THREADS) tbl[idx] = 0u;
    __syncthreads();
    const bool keep = side.hits != nullptr;
    // With lists to reuse, a centre costs two memory round trips (its list, the coordinates of the listed points) once
    // its own index, list length and coordinates are known: those of the wave's four centres are fetched together up
    // front (lane j: index and length of the j-th, lane 3 j + axis: a coordinate).
    constexpr int PER_WAVE = TILE / SEARCH_WAVES;
    int pre_ac = 0;
    uint32_t pre_n = ~0u;
    float pre_xyz = 0.f;
    if (!EXT && reuse.hits) {
        const int64_t a_j = tile * TILE + wave + (int64_t)(lane < PER_WAVE ? lane : 0) * SEARCH_WAVES;
        if (lane < PER_WAVE && a_j < n_centres) pre_ac = perm ? perm[a_j] : (int)a_j;
        if (lane < PER_WAVE && a_j < n_centres) pre_n = reuse.n_hits[pre_ac];
        const int of = lane / 3 < PER_WAVE ? lane / 3 : 0;
        const int ac_of = __shfl(pre_ac, of, 64);
        const int64_t a_of = tile * TILE + wave + (int64_t)of * SEARCH_WAVES;
        if (lane < 3 * PER_WAVE && a_of < n_centres) pre_xyz = centres[3 * (int64_t)ac_of + lane % 3];
    }
    int nth = 0;
    for (int al = wave; al < TILE; al += SEARCH_WAVES, ++nth) {
        const int64_t a = tile * TILE + al;        // slot; the tables and lists are indexed by it
        if (a >= n_centres) break;                 // wave-uniform
        const bool pre = !EXT && reuse.hits;
        const int64_t ac = pre ? (int64_t)__shfl(pre_ac, nth, 64) : (perm ? (int64_t)perm[a] : a);     // the centre's index
        Candidates<SWAP, EXT> c;
        uint32_t filled = 0;
        // what is done for every neighbour: its cell's counter(s), and its place in the list that is kept
        auto account = [&](bool hit, int b, int k, int k2) {
            if (hit) {
                atomicAdd(&tbl[k * TILE + al], 1u);
                if constexpr (BOTH) atomicAdd(&tbl2[k2 * TILE + al], 1u);
            }
            if (keep) {                            // the centre's first hit_stride neighbours, in arrival order
                const unsigned long long m = __ballot(hit);
                const uint32_t slot = filled + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
                if (hit && slot < hit_stride) {
                    mine[slot] = ((uint32_t)k << HIT_INDEX_BITS) | (uint32_t)b;
                    if constexpr (BOTH) mine2[slot] = ((uint32_t)k2 << HIT_INDEX_BITS) | (uint32_t)b;
                }
                filled += (uint32_t)__popcll(m);
            }
        };
        bool searched = true;
        if constexpr (!EXT) {
            const uint32_t n_known = pre ? (uint32_t)__shfl((int)pre_n, nth, 64) : ~0u;      // wave-uniform
            if (n_known <= hit_stride) {
                // the whole neighbourhood is in the earlier pass's list, in the order in which a search finds it
                searched = false;
                c.cx = (double)__shfl(pre_xyz, 3 * nth, 64);
                c.cy = (double)__shfl(pre_xyz, 3 * nth + 1, 64);
                c.cz = (double)__shfl(pre_xyz, 3 * nth + 2, 64);
                for (uint32_t e0 = 0; e0 < n_known; e0 += 64) {
                    const uint32_t e = e0 + (uint32_t)lane;
                    const bool on = e < n_known;
                    int b = 0, k = 0, k2 = 0;
                    if (on) {
                        const uint32_t key = reuse.hits[(size_t)ac * hit_stride + e];
                        b = (int)(key & HIT_INDEX_MASK);
                        k = (int)(key >> HIT_INDEX_BITS);
                        if constexpr (BOTH) {      // the mirrored cell needs the offset again
                            const float *pp = reuse.cand_xyz + 3 * (size_t)b;
                            const float4 p = float4{pp[0], pp[1], pp[2], 0.f};
                            double dx, dy, dz;
                            c.offset_of(p, dx, dy, dz);
                            Candidates<SWAP, EXT>::template cells_of<true>(dx, dy, dz, q, k, k2);
                        }
                    }
                    account(on, b, k, k2);
                }
            }
        }
        if (searched) {
            c.open(centres, ac, g, q, lane);
            for (uint32_t base = 0; base < c.total; base += 64) {
                int b, k, k2;
                const bool hit = c.template fetch2<BOTH>(base + lane, g, q, b, k, k2);
                account(hit, b, k, k2);
            }
        }
        if (side.n_hits && lane == 0) side.n_hits[a] = filled;
        if (keep) {                                // one contiguous write per centre
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const uint32_t n = filled < hit_stride ? filled : hit_stride;
            for (uint32_t e = lane; e < n; e += 64) {
                side.hits[(size_t)a * hit_stride + e] = mine[e];
                if constexpr (BOTH) mirror.hits[(size_t)a * hit_stride + e] = mine2[e];
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
    __syncthreads();
#pragma unroll
    for (int sd = 0; sd < (BOTH ? 2 : 1); ++sd) {
        const CountOut &o = sd == 0 ? side : mirror;
        const uint32_t *t = sd == 0 ? tbl : tbl2;
        if (o.tile_cnt) {
            uint32_t *dst = o.tile_cnt + (size_t)tile * K * TILE;
            for (int idx = threadIdx.x; idx < K * TILE; idx += SEARCH_THREADS) dst[idx] = t[idx];
        }
        for (int k = wave; k < K; k += SEARCH_WAVES) {
            uint32_t v = t[k * TILE + lane];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
            if (lane == 0) o.tile_k_cnt[(size_t)k * n_tiles + tile] = v;
        }
    }
}

// ---- pass 2: write every triplet to its place in (k, centre, other) order ----------------------
//   tile_cnt  [n_tiles][K][TILE]  counts from pass 1
//   tile_ptr  [K * n_tiles + 1]   exclusive prefix sum of tile_k_cnt
//   perm                          centre index of each slot (NULL: slots are centre indices); tables, lists and
//                                 the centre's position in the order use the slot, coordinates and out_c the index
// One wave per centre at a time.  The centre's neighbours are compacted into per-cell buckets of an
// LDS list with wave ballots and prefix popcounts (the bucket sizes are the counts of pass 1), then
// each neighbour's rank inside its bucket (number of smaller candidate indices) gives its final slot,
// so ties between equal (k, centre) are ordered by the other index without any global sort.
constexpr int KGROUPS = (MAX_K + 63) / 64;

// Where the fill pass writes.  out_c / out_b / out_k: centre index, candidate index, cell of each triplet (any may
// be NULL).  With tail_index >= 0 the candidate indices go to the tail_index-th |T|-sized array behind `tail`
// instead (each align_up(|T| * 4) bytes, |T| read from the prefix sum's last entry), with GATHER_LAST set on the
// last triplet of every run.  Nothing is written at or beyond position out_cap, and nothing at all when |T|
// exceeds it (the pass is queued before the host has compared the count with what the caller provided).
struct FillOut {
    int32_t *out_c, *out_b, *out_k;
    char *tail;
    int tail_index;
    uint32_t out_cap;
};

struct Emit {
    int32_t *out_c, *out_b, *out_k;
    const uint32_t *cnt_tile;
    uint32_t cap;
    bool flag_last;
    __device__ inline void operator()(uint32_t run0, uint32_t rank, int al, int k, int32_t centre, uint32_t b) const
    {
        const uint32_t pos = run0 + rank;
        if (pos >= cap) return;
        if (out_c) out_c[pos] = centre;
        if (out_b) out_b[pos] = (int32_t)((flag_last && rank + 1u == cnt_tile[k * TILE + al]) ? (b | GATHER_LAST) : b);
        if (out_k) out_k[pos] = k;
    }
};

template <bool SWAP, bool EXT>
__global__ __launch_bounds__(SEARCH_THREADS, 8) void query_fill(const float *__restrict__ centres, int64_t n_centres,
                                                             const int32_t *__restrict__ perm,
                                                             GridView g, QueryParams q, int K, int64_t n_tiles,
                                                             const uint32_t *__restrict__ tile_cnt,
                                                             const uint32_t *__restrict__ tile_ptr,
                                                             FillOut fo,
                                                             uint32_t *__restrict__ run_start_out, int list_cap,
                                                             const uint32_t *__restrict__ hits, uint32_t hit_stride,
                                                             int64_t *__restrict__ seg_out,
                                                             int pack_ok, const uint32_t *__restrict__ err)
{
    extern __shared__ uint32_t tbl[];          // [K][TILE]: start of each (k, centre) run, then [SEARCH_WAVES][K] bucket words
    __shared__ uint32_t list_all[SEARCH_WAVES][LIST_CAP_MAX];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = blockIdx.x;
    if (*err) return;                          // block-uniform: a prefix sum of this build gave up
    const uint32_t total = tile_ptr[(size_t)K * n_tiles];
    Emit emit;
    emit.out_c = fo.out_c; emit.out_b = fo.out_b; emit.out_k = fo.out_k;
    emit.cnt_tile = tile_cnt + (size_t)tile * K * TILE;
    emit.cap = total <= fo.out_cap ? fo.out_cap : 0u;
    emit.flag_last = false;
    if (fo.tail_index >= 0) {
        emit.out_b = reinterpret_cast<int32_t *>(fo.tail + (size_t)fo.tail_index * (((size_t)total * 4 + 255) / 256 * 256));
        emit.flag_last = true;
    }
    // start of every cell's segment (Sec. 3.3.2): the offset of its first tile; entry K is |T|
    if (seg_out && tile == 0)
        for (int k = threadIdx.x; k <= K; k += SEARCH_THREADS) seg_out[k] = (int64_t)tile_ptr[(size_t)k * n_tiles];
    const uint32_t *cnt_tile = tile_cnt + (size_t)tile * K * TILE;
    for (int idx = threadIdx.x; idx < K * TILE; idx += SEARCH_THREADS) tbl[idx] = cnt_tile[idx];
    __syncthreads();
    for (int k = wave; k < K; k += SEARCH_WAVES) {
        const uint32_t v = tbl[k * TILE + lane];
        const uint32_t inc = wave_incl_scan_u32(v, lane);
        tbl[k * TILE + lane] = tile_ptr[(size_t)k * n_tiles + tile] + inc - v;
    }
    __syncthreads();
    if (run_start_out) {
        uint32_t *dst = run_start_out + (size_t)tile * K * TILE;
        for (int idx = threadIdx.x; idx < K * TILE; idx += SEARCH_THREADS) dst[idx] = tbl[idx];
    }
    uint32_t *list = list_all[wave];
    const unsigned long long lane_lt = (1ull << lane) - 1ull;
    // A centre whose neighbours the count pass left in `hits` needs no second search.
    constexpr int PER_WAVE = TILE / SEARCH_WAVES;
    const uint32_t reuse_max = hits ? (hit_stride < KEEP_MAX ? hit_stride : KEEP_MAX) : 0u;
    Candidates<SWAP, EXT> cand[1];
    uint32_t n_of[PER_WAVE];
#pragma unroll
    for (int u = 0; u < PER_WAVE; ++u) {
        const int al = wave + u * SEARCH_WAVES;
        const int64_t a = tile * TILE + al;
        uint32_t nn = 0;
        if (a < n_centres)
            for (int k = lane; k < K; k += 64) nn += cnt_tile[k * TILE + al];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) nn += __shfl_xor(nn, d, 64);
        n_of[u] = nn;
    }
    // Two centres at a time, one per half wave, while both of their kept lists fit 32 lanes (most do: the all-pairs
    // ranking then costs one pass for the two).  Centres done here are marked by a zero count.
    if (reuse_max >= 32 && list_cap >= 64) {
        const int half = lane >> 5, l = lane & 31;
#pragma unroll
        for (int u = 0; u + 1 < PER_WAVE; u += 2) {
            const uint32_t n0 = n_of[u], n1 = n_of[u + 1];
            if (n0 == 0 || n1 == 0 || n0 > 32 || n1 > 32) continue;       // wave-uniform
            const int al = wave + (u + half) * SEARCH_WAVES;
            const int64_t a = tile * TILE + al;                         // both exist: their counts are not zero
            const uint32_t n = half ? n1 : n0, nmax = n0 > n1 ? n0 : n1;
            const uint32_t key = l < (int)n ? hits[(size_t)a * hit_stride + l] : 0xffffffffu;   // padding ranks nobody
            list[lane] = key;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const uint32_t kbase = key & ~HIT_INDEX_MASK, rel = key & HIT_INDEX_MASK;
            const uint32_t *other = list + 32 * half;
            uint32_t rank = 0;
            for (uint32_t e2 = 0; e2 < nmax; e2 += 8) {                 // reads past nmax see padding or real keys of
                uint32_t v[8];                                          // this half only up to n: entries >= n are padding
#pragma unroll
                for (int w = 0; w < 8; ++w) v[w] = other[e2 + w];
#pragma unroll
                for (int w = 0; w < 8; ++w) rank += (v[w] - kbase) < rel ? 1u : 0u;
            }
            if (l < (int)n) {
                const int k = (int)(key >> HIT_INDEX_BITS);
                emit(tbl[k * TILE + al], rank, al, k, (int32_t)(perm ? (int64_t)perm[a] : a), rel);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            n_of[u] = n_of[u + 1] = 0;
        }
    }
#pragma unroll
    for (int u = 0; u < PER_WAVE; ++u) {
        const int al = wave + u * SEARCH_WAVES;
        const int64_t a = tile * TILE + al;    // slot
        if (a >= n_centres) break;             // wave-uniform
        if (n_of[u] == 0) continue;            // wave-uniform
        const int32_t ac = (int32_t)(perm ? (int64_t)perm[a] : a);   // the centre's own index
        if (pack_ok && n_of[u] > BUCKET_FROM && n_of[u] <= (uint32_t)list_cap) {
            // Longer lists, when cell and candidate index fit one word (cell << 24 | index).  The keys -- read back from the count pass
            // when it kept them, found again otherwise -- are dropped into per-cell buckets of the list through one
            // LDS word per cell (bucket start << 16 | fill count, advanced with an LDS add; the order inside a
            // bucket is whatever the adds made it), and each key's rank among the smaller keys of its own bucket
            // is its final slot: a key is compared with its cell's neighbours only.
            const uint32_t n = n_of[u];
            uint32_t *wk = tbl + K * TILE + wave * K;
            uint32_t run = 0;
            for (int k0 = 0; k0 < K; k0 += 64) {
                const int k = k0 + lane;
                const uint32_t c1 = k < K ? cnt_tile[k * TILE + al] : 0u;
                const uint32_t inc = wave_incl_scan_u32(c1, lane);
                if (k < K) wk[k] = (run + inc - c1) << 16;
                run += (uint32_t)__shfl((int)inc, 63, 64);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (n <= reuse_max) {
                const uint32_t *mine = hits + (size_t)a * hit_stride;
                for (uint32_t e = lane; e < n; e += 64) {
                    const uint32_t key = mine[e];
                    const uint32_t old = atomicAdd(&wk[key >> HIT_INDEX_BITS], 1u);
                    list[(old >> 16) + (old & 0xffffu)] = key;
                }
            } else {
                Candidates<SWAP, EXT> &c = cand[0];
                c.open(centres, ac, g, q, lane);
                for (uint32_t base = 0; base < c.total; base += 64) {
                    int b, k;
                    if (c.fetch(base + lane, g, q, b, k)) {
                        const uint32_t old = atomicAdd(&wk[k], 1u);
                        list[(old >> 16) + (old & 0xffffu)] = ((uint32_t)k << HIT_INDEX_BITS) | (uint32_t)b;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (uint32_t e0 = 0; e0 < n; e0 += 64) {
                const uint32_t e = e0 + lane;
                const bool have = e < n;
                const uint32_t key = have ? list[e] : 0u;
                const int k = (int)(key >> HIT_INDEX_BITS);
                const uint32_t w = have ? wk[k] : 0u;
                const uint32_t b0 = w >> 16, nk = w & 0xffffu;
                uint32_t rank = 0;
                for (uint32_t j = 0; __ballot(j < nk) != 0ull; ++j) {
                    const uint32_t v = j < nk ? list[b0 + j] : 0xffffffffu;
                    rank += v < key ? 1u : 0u;
                }
                if (have) emit(tbl[k * TILE + al], rank, al, k, ac, key & HIT_INDEX_MASK);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            continue;
        }
        if (n_of[u] <= reuse_max && n_of[u] <= (uint32_t)list_cap) {
            // rank the stored (cell, index) keys by comparing all pairs
            const uint32_t n = n_of[u];
            const uint32_t *mine = hits + (size_t)a * hit_stride;
            for (uint32_t e = lane; e < n; e += 64) list[e] = mine[e];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (uint32_t e = lane; e < n; e += 64) {
                const uint32_t key = list[e];
                const uint32_t kbase = key & ~HIT_INDEX_MASK, rel = key & HIT_INDEX_MASK;
                uint32_t rank = 0, e2 = 0;
                for (; e2 + 8 <= n; e2 += 8) {
                    uint32_t v[8];
#pragma unroll
                    for (int w = 0; w < 8; ++w) v[w] = list[e2 + w];
#pragma unroll
                    for (int w = 0; w < 8; ++w) rank += (v[w] - kbase) < rel ? 1u : 0u;
                }
                for (; e2 < n; ++e2) rank += (list[e2] - kbase) < rel ? 1u : 0u;
                const int k = (int)(key >> HIT_INDEX_BITS);
                emit(tbl[k * TILE + al], rank, al, k, ac, rel);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            continue;
        }
        // bucket of cell k = [bbase, bbase + bcnt) in the list; lane (k % 64) of group (k / 64) holds it
        uint32_t bcnt[KGROUPS], bbase[KGROUPS], bcur[KGROUPS];
        uint32_t n = 0;
#pragma unroll
        for (int gi = 0; gi < KGROUPS; ++gi) {
            bcnt[gi] = 0; bbase[gi] = n; bcur[gi] = 0;
            if (gi * 64 < K) {                 // wave-uniform
                const int k = gi * 64 + lane;
                bcnt[gi] = k < K ? cnt_tile[k * TILE + al] : 0u;
                const uint32_t inc = wave_incl_scan_u32(bcnt[gi], lane);
                bbase[gi] = n + inc - bcnt[gi];
                n += __shfl(inc, 63, 64);
            }
        }
        if (n == 0) continue;                  // wave-uniform
        Candidates<SWAP, EXT> &c = cand[0];
        c.open(centres, ac, g, q, lane);
        if (n <= SMALL_LIST && n <= (uint32_t)list_cap) {
            // few neighbours: one flat list of (cell, index) keys in arrival order, rank by comparing all pairs
            unsigned long long *keys = reinterpret_cast<unsigned long long *>(list);
            uint32_t filled = 0;
            for (uint32_t base = 0; base < c.total; base += 64) {
                int b, k;
                const bool hit = c.fetch(base + lane, g, q, b, k);
                const unsigned long long m = __ballot(hit);
                if (hit) keys[filled + (uint32_t)__popcll(m & lane_lt)] = ((unsigned long long)(uint32_t)k << 32) | (uint32_t)b;
                filled += (uint32_t)__popcll(m);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (uint32_t e = lane; e < n; e += 64) {
                const unsigned long long key = keys[e];
                const unsigned long long kbase = key & 0xffffffff00000000ull;
                const unsigned long long rel = key - kbase;
                uint32_t rank = 0, e2 = 0;
                for (; e2 + 8 <= n; e2 += 8) {
                    unsigned long long v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = keys[e2 + u];
#pragma unroll
                    for (int u = 0; u < 8; ++u) rank += ((v[u] - kbase) < rel) ? 1u : 0u;
                }
                for (; e2 < n; ++e2) rank += ((keys[e2] - kbase) < rel) ? 1u : 0u;
                const int k = (int)(key >> 32);
                emit(tbl[k * TILE + al], rank, al, k, ac, (uint32_t)key);
            }
        } else if (n <= (uint32_t)list_cap) {
            for (uint32_t base = 0; base < c.total; base += 64) {
                int b, k;
                const bool hit = c.fetch(base + lane, g, q, b, k);
                unsigned long long rem = __ballot(hit);
                while (rem) {                  // one round per distinct cell among this batch's hits
                    const int kk = __shfl(k, __ffsll((long long)rem) - 1, 64);
                    const unsigned long long mk = __ballot(hit && k == kk);
                    uint32_t slot0 = 0;
#pragma unroll
                    for (int gi = 0; gi < KGROUPS; ++gi)
                        if ((kk >> 6) == gi) {
                            slot0 = __shfl(bbase[gi] + bcur[gi], kk & 63, 64);
                            if (lane == (kk & 63)) bcur[gi] += (uint32_t)__popcll(mk);
                        }
                    if (hit && k == kk) list[slot0 + (uint32_t)__popcll(mk & lane_lt)] = (uint32_t)b;
                    rem &= ~mk;
                }
            }
            // the list was written by other lanes of this wave: LDS operations of one wave complete in
            // order, the fence keeps the compiler from moving the reads above the writes
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int gi = 0; gi < KGROUPS; ++gi) {
                unsigned long long occ = __ballot(bcnt[gi] != 0);
                while (occ) {                  // buckets of this group, ascending cell
                    const int kl = __ffsll((long long)occ) - 1;
                    occ &= occ - 1;
                    const int k = gi * 64 + kl;
                    const uint32_t nk = __shfl(bcnt[gi], kl, 64), b0 = __shfl(bbase[gi], kl, 64);
                    const uint32_t run0 = tbl[k * TILE + al];
                    for (uint32_t e0 = 0; e0 < nk; e0 += 64) {
                        const uint32_t e = e0 + lane;
                        const uint32_t mine = e < nk ? list[b0 + e] : 0xffffffffu;
                        uint32_t rank = 0, e2 = 0;
                        for (; e2 + 8 <= nk; e2 += 8) {
                            uint32_t v[8];
#pragma unroll
                            for (int u = 0; u < 8; ++u) v[u] = list[b0 + e2 + u];
#pragma unroll
                            for (int u = 0; u < 8; ++u) rank += v[u] < mine ? 1u : 0u;
                        }
                        for (; e2 < nk; ++e2) rank += list[b0 + e2] < mine ? 1u : 0u;
                        if (e < nk) emit(run0, rank, al, k, ac, mine);
                    }
                }
            }
        } else {
            // more neighbours than the list holds: rank each one by scanning the candidates again
            for (uint32_t base = 0; base < c.total; base += 64) {
                int b, k;
                const bool hit = c.fetch(base + lane, g, q, b, k);
                uint32_t rank = 0;
                for (uint32_t idx2 = 0; idx2 < c.total; ++idx2) {
                    int b2, k2;
                    const bool hit2 = c.fetch(idx2, g, q, b2, k2);
                    rank += (hit2 && k2 == k && b2 < b) ? 1u : 0u;
                }
                if (hit) emit(tbl[k * TILE + al], rank, al, k, ac, (uint32_t)b);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- voxel-grid down-sampling that keeps original coordinates (Sec. 4.1) ----------------------------------------
// One point per occupied voxel of pitch v: the one with the lowest index.  The voxels go through the same kind of
// hash table as the search grid; every slot keeps the lowest index inserted into it.

__global__ __launch_bounds__(256) void sub_clear(unsigned long long *__restrict__ keys, int *__restrict__ lowest,
                                                 int64_t slots, unsigned long long *__restrict__ zero_from,
                                                 int64_t zero_words)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < slots; i += stride) {
        keys[i] = EMPTY_KEY;
        lowest[i] = 0x7fffffff;
    }
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < zero_words; i += stride) zero_from[i] = 0ull;
}

__global__ __launch_bounds__(256) void sub_insert(const float *__restrict__ xyz, int64_t n, double v,
                                                  unsigned long long *__restrict__ keys, int *__restrict__ lowest,
                                                  uint32_t mask, uint32_t *__restrict__ point_slot)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    int c[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) c[a] = (int)fmin(fmax(voxel_of(xyz[3 * p + a], v), -CELL_CLAMP), CELL_CLAMP);
    const unsigned long long key = pack_key(c[0], c[1], c[2]);
    uint32_t slot = hash_key(key) & mask;
    for (;;) {
        unsigned long long prev = atomicCAS(&keys[slot], EMPTY_KEY, key);
        if (prev == EMPTY_KEY || prev == key) break;
        slot = (slot + 1) & mask;
    }
    atomicMin(&lowest[slot], (int)p);
    point_slot[p] = slot;
}

__global__ __launch_bounds__(256) void sub_flag(int64_t n, const int *__restrict__ lowest,
                                                const uint32_t *__restrict__ point_slot, uint32_t *__restrict__ flag)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) flag[p] = lowest[point_slot[p]] == (int)p ? 1u : 0u;
}

// pos = exclusive prefix sum of the flags, computed in place over them: a point is kept iff pos[p + 1] > pos[p]
__global__ __launch_bounds__(256) void sub_scatter(int64_t n, const uint32_t *__restrict__ pos, int32_t *__restrict__ kept,
                                                   const uint32_t *__restrict__ err)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n || *err) return;
    if (pos[p + 1] != pos[p]) kept[pos[p]] = (int32_t)p;
}

// ---- host side ------------------------------------------------------------------------------

struct GridScratch {
    size_t keys_off, cnt_off, cursor_off, point_slot_off, pts_off, end;
    int64_t slots;
};

int64_t grid_slots(int64_t n)
{
    int64_t s = 64;
    while (s < 2 * n) s <<= 1;
    return s;
}

struct SubScratch {
    size_t err_off, total_off, scan_off, keys_off, lowest_off, slot_off, flag_off, end;
    int64_t slots;
};

SubScratch sub_scratch(int64_t n)
{
    SubScratch s;
    s.slots = grid_slots(n);
    size_t off = 0;
    s.err_off = off;    off += 256;
    s.total_off = off;  off += 256;
    s.scan_off = off;   off += scan_scratch_bytes(n > 0 ? n : 1);
    s.keys_off = off;   off += align_up((size_t)s.slots * 8);
    s.lowest_off = off; off += align_up((size_t)s.slots * 4);
    s.slot_off = off;   off += align_up((size_t)(n > 0 ? n : 1) * 4);
    s.flag_off = off;   off += align_up((size_t)(n + 1) * 4);
    s.end = off;
    return s;
}

GridScratch grid_scratch(size_t base, int64_t n)
{
    GridScratch s;
    s.slots = grid_slots(n);
    size_t off = base;
    s.keys_off = off;        off += align_up((size_t)s.slots * 8);
    s.cnt_off = off;         off += align_up((size_t)(s.slots + 1) * 4);
    s.cursor_off = off;      off += align_up((size_t)s.slots * 4);
    s.point_slot_off = off;  off += align_up((size_t)(n > 0 ? n : 1) * 4);
    s.pts_off = off;         off += align_up((size_t)(n > 0 ? n : 1) * 16);
    s.end = off;
    return s;
}

// prefix sums of one build, each with status words of its own: the two grids, the public (k, o, i) list, the
// two sides of a spatial plan (or the input-gradient side of a plain one), and the passes of two spatial sorts
constexpr int SCAN_GRID_IN = 0, SCAN_GRID_OUT = 1, SCAN_PUBLIC = 2, SCAN_FWD_SIDE = 3, SCAN_BWD_SIDE = 4,
              SCAN_SORT_OUT = 5, SCAN_SORT_IN = SCAN_SORT_OUT + SPATIAL_ORDER_SCANS,
              N_SCANS = SCAN_SORT_IN + SPATIAL_ORDER_SCANS;

struct BuildScratch {
    GridScratch grid_in, grid_out;
    size_t err_off;                  // one word: raised by a prefix sum whose wait ran out
    size_t total_off;                // |T| as the prefix sum leaves it, when the caller's landing word is pageable
    size_t scan_off;                 // status words of the prefix sums: N_SCANS regions of scan_stride bytes
    size_t scan_stride;
    size_t fwd_ptr_off, fwd_cnt_off; // per-(k, tile) sums / offsets and per-(k, centre) counts of the pass in flight
    size_t bwd_ptr_off, bwd_cnt_off;
    size_t sort_off;                 // scratch of the spatial sorts
    size_t end;                      // without hit lists
    // Optional, after `end`: the first hit_stride neighbours of every centre as found by the count pass, so
    // that the fill pass need not search again (needs the triplet capacity to size the lists).
    uint32_t fwd_stride = 0, bwd_stride = 0;
    size_t fwd_hits_off = 0, bwd_hits_off = 0, end_with_hits = 0;
    // Optional, after that: a second set of lists of the outputs and their lengths.  A plan in spatial order counts
    // the same neighbourhoods twice, once in index order for the public list and once in slot order; with these the
    // second count reads the first one's lists instead of searching again.
    size_t pub_hits_off = 0, n_hits_off = 0, end_with_reuse = 0;
};

// list length per centre: twice the mean neighbour count, within [32, KEEP_MAX]
uint32_t hit_stride_for(int64_t capacity, int64_t n_centres)
{
    if (n_centres <= 0 || capacity <= 0) return 0;
    int64_t s = (2 * ceil_div(capacity, n_centres) + 15) / 16 * 16;
    if (s < 32) s = 32;
    if (s > (int64_t)KEEP_MAX) s = KEEP_MAX;
    return (uint32_t)s;
}

BuildScratch build_scratch(int64_t n_in, int64_t n_out, int K, int64_t capacity = -1)
{
    BuildScratch b;
    b.grid_in = grid_scratch(0, n_in);
    b.grid_out = grid_scratch(b.grid_in.end, n_out);
    size_t off = b.grid_out.end;
    const int64_t nt_o = ceil_div(n_out, TILE), nt_i = ceil_div(n_in, TILE);
    int64_t scan_n = b.grid_in.slots > b.grid_out.slots ? b.grid_in.slots : b.grid_out.slots;
    if ((int64_t)K * nt_o > scan_n) scan_n = (int64_t)K * nt_o;
    if ((int64_t)K * nt_i > scan_n) scan_n = (int64_t)K * nt_i;
    const int64_t n_max = n_in > n_out ? n_in : n_out;
    if (spatial_order_scan_items(n_max) > scan_n) scan_n = spatial_order_scan_items(n_max);
    b.err_off = off;     off += 256;
    b.total_off = off;   off += 256;
    b.scan_stride = scan_scratch_bytes(scan_n);
    b.scan_off = off;    off += N_SCANS * b.scan_stride;
    b.fwd_ptr_off = off; off += align_up((size_t)(K * nt_o + 1) * 4);
    b.fwd_cnt_off = off; off += align_up((size_t)(nt_o > 0 ? nt_o : 1) * K * TILE * 4);
    b.bwd_ptr_off = off; off += align_up((size_t)(K * nt_i + 1) * 4);
    b.bwd_cnt_off = off; off += align_up((size_t)(nt_i > 0 ? nt_i : 1) * K * TILE * 4);
    b.sort_off = off;    off += spatial_order_scratch_bytes(n_max);
    b.end = off;
    b.end_with_hits = off;
    // stored hits carry the candidate index in HIT_INDEX_BITS bits
    if (capacity > 0 && n_in < (1 << HIT_INDEX_BITS) && n_out < (1 << HIT_INDEX_BITS)) {
        b.fwd_stride = hit_stride_for(capacity, n_out);
        b.bwd_stride = hit_stride_for(capacity, n_in);
        b.fwd_hits_off = off; off += align_up((size_t)n_out * b.fwd_stride * 4);
        b.bwd_hits_off = off; off += align_up((size_t)n_in * b.bwd_stride * 4);
        b.end_with_hits = off;
        b.n_hits_off = off;   off += align_up((size_t)n_out * 4);
        b.pub_hits_off = off; off += align_up((size_t)n_out * b.fwd_stride * 4);
    }
    b.end_with_reuse = off;
    return b;
}

// scan_scratch: the status words of this grid's prefix sum.  clear_words > 0: the first grid of a build, whose
// clearing kernel also zeroes the error word and the status words of all the build's prefix sums (they follow
// the error word in the workspace).
int build_grid(const float *xyz, int64_t n, const GridMap &gm, const int32_t *batch_off, int n_batches, char *ws,
               const GridScratch &gs, void *scan_scratch, unsigned long long *clear_from, int64_t clear_words,
               uint32_t *err, GridView *view, hipStream_t stream)
{
    auto *keys = reinterpret_cast<unsigned long long *>(ws + gs.keys_off);
    auto *cnt = reinterpret_cast<uint32_t *>(ws + gs.cnt_off);
    auto *cursor = reinterpret_cast<uint32_t *>(ws + gs.cursor_off);
    auto *point_slot = reinterpret_cast<uint32_t *>(ws + gs.point_slot_off);
    auto *pts = reinterpret_cast<float4 *>(ws + gs.pts_off);
    int rc;
    {
        int64_t blocks = ceil_div(gs.slots + 1, 256);
        if (blocks > 4096) blocks = 4096;
        grid_clear<<<(unsigned)blocks, 256, 0, stream>>>(keys, cnt, cursor, gs.slots, clear_from, clear_words);
        PCPP_HIP_CHECK(hipGetLastError());
    }
    if (n > 0) {
        const unsigned blocks = (unsigned)ceil_div(n, 256);
        grid_insert<<<blocks, 256, 0, stream>>>(xyz, n, gm, batch_off, n_batches, keys, cnt, (uint32_t)(gs.slots - 1),
                                                point_slot);
        PCPP_HIP_CHECK(hipGetLastError());
    }
    if ((rc = scan_exclusive_u32(cnt, cnt, gs.slots, scan_scratch, nullptr, err, stream)) != PCPP_OK) return rc;
    if (n > 0) {
        const unsigned blocks = (unsigned)ceil_div(n, 256);
        grid_scatter<<<blocks, 256, 0, stream>>>(xyz, n, point_slot, cnt, cursor, pts, err);
        PCPP_HIP_CHECK(hipGetLastError());
    }
    view->keys = keys;
    view->slot_start = cnt;
    view->pts = pts;
    view->mask = (uint32_t)(gs.slots - 1);
    view->map = gm;
    return PCPP_OK;
}

// The event that tells the host that |T| has landed; created and destroyed inside one call.
struct CallEvent {
    hipEvent_t ev = nullptr;
    ~CallEvent() { if (ev) (void)hipEventDestroy(ev); }
};

}  // namespace

PlanLayout plan_layout(int64_t n_in, int64_t n_out, int K, int64_t n_triplets, int flags)
{
    PlanLayout p;
    const bool spatial = (flags & PCPP_PLAN_SPATIAL) != 0;
    size_t off = 256;   // header (reserved)
    auto side = [&](SideLayout &s, int64_t n_centres, bool with_gather) {
        s.n_centres = n_centres;
        s.n_tiles = ceil_div(n_centres, TILE);
        s.perm_off = off;
        if (spatial) off += align_up((size_t)(n_centres > 0 ? n_centres : 1) * 4);
        s.tile_ptr_off = off;  off += align_up((size_t)(K * s.n_tiles + 1) * 4);
        s.run_start_off = off; off += align_up((size_t)(s.n_tiles > 0 ? s.n_tiles : 1) * K * TILE * 4);
        if (with_gather) s.gather_index = p.n_tail++;
    };
    if (flags & PCPP_PLAN_FWD) side(p.fwd, n_out, spatial);
    if (flags & PCPP_PLAN_BWD_INPUT) side(p.bwd, n_in, true);
    p.tail_off = off;
    const size_t each = align_up((size_t)(n_triplets > 0 ? n_triplets : 1) * 4);
    if (p.fwd.gather_index >= 0) p.fwd.gather_off = off + (size_t)p.fwd.gather_index * each;
    if (p.bwd.gather_index >= 0) p.bwd.gather_off = off + (size_t)p.bwd.gather_index * each;
    p.bytes = off + (size_t)p.n_tail * each;
    return p;
}

}  // namespace pcpp

using namespace pcpp;

extern "C" {

size_t pcpp_build_triplets_workspace_bytes(int64_t n_in, int64_t n_out, int t)
{
    if (n_in < 0 || n_out < 0 || t < 1 || t > PCPP_MAX_T) return 0;
    return build_scratch(n_in, n_out, t * t * t).end;
}

size_t pcpp_build_triplets_workspace_bytes_for(int64_t n_in, int64_t n_out, int t, int64_t capacity)
{
    if (n_in < 0 || n_out < 0 || t < 1 || t > PCPP_MAX_T || capacity < 0) return 0;
    return build_scratch(n_in, n_out, t * t * t, capacity).end_with_reuse;
}

size_t pcpp_plan_bytes(int64_t n_in, int64_t n_out, int t, int64_t n_triplets, int plan_flags)
{
    if (n_in < 0 || n_out < 0 || t < 1 || t > PCPP_MAX_T || n_triplets < 0) return 0;
    return plan_layout(n_in, n_out, t * t * t, n_triplets, plan_flags & PLAN_FLAG_MASK).bytes;
}

int pcpp_build_triplets(const float *in_xyz, int64_t n_in, const float *out_xyz, int64_t n_out,
                        float radius, int t,
                        int32_t *tri_o, int32_t *tri_i, int32_t *tri_k, int64_t capacity,
                        int64_t *seg_offsets, int64_t *n_triplets,
                        void *plan, size_t plan_bytes, int plan_flags,
                        void *workspace, size_t workspace_bytes, void *stream_)
{
    return pcpp_build_triplets_batched(in_xyz, n_in, out_xyz, n_out, nullptr, nullptr, 1, radius, t, tri_o, tri_i, tri_k,
                                       capacity, seg_offsets, n_triplets, plan, plan_bytes, plan_flags, workspace,
                                       workspace_bytes, stream_);
}

int pcpp_build_triplets_batched(const float *in_xyz, int64_t n_in, const float *out_xyz, int64_t n_out,
                                const int32_t *in_batch_offsets, const int32_t *out_batch_offsets, int n_batches,
                                float radius, int t,
                                int32_t *tri_o, int32_t *tri_i, int32_t *tri_k, int64_t capacity,
                                int64_t *seg_offsets, int64_t *n_triplets,
                                void *plan, size_t plan_bytes, int plan_flags,
                                void *workspace, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (n_batches < 1 || n_batches > 65536 || ((in_batch_offsets == nullptr) != (out_batch_offsets == nullptr)) ||
        (n_batches > 1 && !in_batch_offsets)) {
        set_error("pcpp_build_triplets_batched: n_batches must be in 1..65536 and both offset arrays given (or neither, "
                  "for one cloud)");
        return PCPP_ERR_INVALID_ARG;
    }
    if (n_in < 0 || n_out < 0 || (n_in > 0 && !in_xyz) || (n_out > 0 && !out_xyz) || !n_triplets) {
        set_error("pcpp_build_triplets: null pointer or negative size");
        return PCPP_ERR_INVALID_ARG;
    }
    if (n_in >= INT32_MAX || n_out >= INT32_MAX) {
        set_error("pcpp_build_triplets: point counts must be below 2^31");
        return PCPP_ERR_UNSUPPORTED;
    }
    if (!(radius > 0.0f) || !isfinite(radius)) {
        set_error("pcpp_build_triplets: radius must be finite and positive");
        return PCPP_ERR_INVALID_ARG;
    }
    if (t < 1 || t > PCPP_MAX_T) {
        set_error("pcpp_build_triplets: t must be in 1..%d", PCPP_MAX_T);
        return PCPP_ERR_INVALID_ARG;
    }
    const int n_null = (tri_o == nullptr) + (tri_i == nullptr) + (tri_k == nullptr);
    if (n_null != 0 && n_null != 3) {
        set_error("pcpp_build_triplets: tri_o, tri_i, tri_k must be all NULL or all non-NULL");
        return PCPP_ERR_INVALID_ARG;
    }
    const bool count_only = n_null == 3;
    if (!count_only && (capacity < 0 || !seg_offsets)) {
        set_error("pcpp_build_triplets: seg_offsets is NULL or capacity negative");
        return PCPP_ERR_INVALID_ARG;
    }
    const int test_flags = plan_flags & (PCPP_BUILD_TEST_SHORT_LISTS | PCPP_BUILD_TEST_WIDE_KEYS);
    if (plan_flags & ~(PLAN_FLAG_MASK | PCPP_BUILD_TEST_SHORT_LISTS | PCPP_BUILD_TEST_WIDE_KEYS | PCPP_BUILD_VOXEL)) {
        set_error("pcpp_build_triplets: unknown bits in plan_flags");
        return PCPP_ERR_INVALID_ARG;
    }
    const bool voxel = (plan_flags & PCPP_BUILD_VOXEL) != 0;
    const bool ext = voxel || in_batch_offsets != nullptr;     // the search kernels with the variants compiled in
    if (voxel && t % 2 == 0) {
        set_error("pcpp_build_triplets: the voxel operator needs an odd t (a centre voxel)");
        return PCPP_ERR_INVALID_ARG;
    }
    plan_flags &= PLAN_FLAG_MASK;
    if (plan && !(plan_flags & PCPP_PLAN_FWD)) {
        set_error("pcpp_build_triplets: plan_flags must include PCPP_PLAN_FWD");
        return PCPP_ERR_INVALID_ARG;
    }
    const int K = t * t * t;
    const BuildScratch bs = build_scratch(n_in, n_out, K, count_only ? -1 : capacity);
    if (!workspace || workspace_bytes < bs.end || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
        set_error("pcpp_build_triplets: workspace missing, misaligned or smaller than %zu bytes", bs.end);
        return PCPP_ERR_WORKSPACE;
    }
    if (plan && (reinterpret_cast<uintptr_t>(plan) & 255)) {
        set_error("pcpp_build_triplets: plan must be 256-byte aligned");
        return PCPP_ERR_WORKSPACE;
    }
    *n_triplets = 0;
    char *ws = static_cast<char *>(workspace);
    const bool wide_keys = (test_flags & PCPP_BUILD_TEST_WIDE_KEYS) != 0;
    const bool keep_hits = bs.fwd_stride != 0 && workspace_bytes >= bs.end_with_hits && !wide_keys;
    uint32_t *f_hits = keep_hits ? reinterpret_cast<uint32_t *>(ws + bs.fwd_hits_off) : nullptr;
    uint32_t *b_hits = keep_hits ? reinterpret_cast<uint32_t *>(ws + bs.bwd_hits_off) : nullptr;
    const Reuse no_reuse{nullptr, nullptr, nullptr};
    uint32_t *err = reinterpret_cast<uint32_t *>(ws + bs.err_off);
    auto scan_scratch = [&](int which) -> void * { return ws + bs.scan_off + (size_t)which * bs.scan_stride; };
    const int list_cap = (test_flags & PCPP_BUILD_TEST_SHORT_LISTS) ? 40 : LIST_CAP_MAX;

    // Where |T| lands.  Pinned host memory is written by the device itself (the prefix sum's last block), so the
    // host can pick the count up while the second pass is already running; pageable memory gets it through a
    // blocking copy before that pass is queued.
    unsigned long long *total_dev = reinterpret_cast<unsigned long long *>(ws + bs.total_off);
    bool pinned = false;
    {
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, n_triplets) == hipSuccess && attr.type == hipMemoryTypeHost &&
            attr.devicePointer) {
            total_dev = static_cast<unsigned long long *>(attr.devicePointer);
            pinned = true;
        } else {
            (void)hipGetLastError();                 // an unregistered pointer is reported as an error; it is not one
        }
    }

    // grid pitch a hair above r so that, with the binary64 cell computation, any accepted pair lies
    // in adjacent grid cells (27-cell stencil is conservative)
    const double R = (double)radius;
    GridMap gm;
    gm.inv_g = 1.0 / (R * (1.0 + 1.0 / 1048576.0));
    gm.vox = R;
    gm.hp = (t - 1) / 2 > 1 ? (t - 1) / 2 : 1;
    gm.voxel_mode = voxel ? 1 : 0;
    QueryParams q;
    q.R = R;
    q.r2 = R * R;
    q.inv_cell = (double)t / (2.0 * R);
    q.t = t;
    q.voxel_mode = voxel ? 1 : 0;
    q.h = (t - 1) / 2;
    q.c_off = out_batch_offsets;         // forward orientation: centres = outputs, candidates = inputs
    q.d_off = in_batch_offsets;
    q.n_batches = n_batches;
    QueryParams qs = q;                  // roles swapped: centres = inputs, candidates = outputs
    qs.c_off = in_batch_offsets;
    qs.d_off = out_batch_offsets;

    int rc;
    GridView grid_in;
    // the clearing kernel of the first grid zeroes the error word, the total and all status words (contiguous)
    if ((rc = build_grid(in_xyz, n_in, gm, in_batch_offsets, n_batches, ws, bs.grid_in, scan_scratch(SCAN_GRID_IN),
                         reinterpret_cast<unsigned long long *>(ws + bs.err_off),
                         (int64_t)((512 + N_SCANS * bs.scan_stride) / sizeof(unsigned long long)), err, &grid_in,
                         stream)) != PCPP_OK)
        return rc;

    const int64_t nt_o = ceil_div(n_out, TILE), nt_i = ceil_div(n_in, TILE);
    const size_t lds = (size_t)K * TILE * sizeof(uint32_t);
    // the second pass also keeps one bucket word per (wave, cell); a key packs cell and candidate index into 32 bits
    const size_t lds_fill = lds + (size_t)SEARCH_WAVES * K * sizeof(uint32_t);
    const int pack_ok = !wide_keys && K <= 256 && n_in < (1 << HIT_INDEX_BITS) && n_out < (1 << HIT_INDEX_BITS);
    if (lds > (size_t)32 * 1024) {
        // large t: the per-tile table plus the neighbour lists exceed the default dynamic LDS limit
        if ((rc = raise_lds_limit(ext ? reinterpret_cast<const void *>(&query_count<false, false, true>)
                                      : reinterpret_cast<const void *>(&query_count<false, false, false>), lds)) != PCPP_OK) return rc;
        if ((rc = raise_lds_limit(ext ? reinterpret_cast<const void *>(&query_count<true, false, true>)
                                      : reinterpret_cast<const void *>(&query_count<true, false, false>), lds)) != PCPP_OK) return rc;
    }
    if (lds_fill > (size_t)32 * 1024) {
        if ((rc = raise_lds_limit(ext ? reinterpret_cast<const void *>(&query_fill<false, true>)
                                      : reinterpret_cast<const void *>(&query_fill<false, false>), lds_fill)) != PCPP_OK) return rc;
        if ((rc = raise_lds_limit(ext ? reinterpret_cast<const void *>(&query_fill<true, true>)
                                      : reinterpret_cast<const void *>(&query_fill<true, false>), lds_fill)) != PCPP_OK) return rc;
    }
    const bool want_plan = plan && !count_only;
    const bool want_bwd = want_plan && (plan_flags & PCPP_PLAN_BWD_INPUT);
    const bool spatial = want_plan && (plan_flags & PCPP_PLAN_SPATIAL);
    const bool self = out_xyz == in_xyz && n_out == n_in && in_batch_offsets == out_batch_offsets;

    // A cloud queried against itself: one pass counts both sides of the plan (while two [K][64] tables fit the
    // LDS that one block may allocate, beside the lists).
    bool one_pass = want_bwd && self && 2 * lds <= (size_t)72 * 1024;
    if (one_pass && 2 * lds > (size_t)32 * 1024) {
        int dev = 0, per_block = 0;
        PCPP_HIP_CHECK(hipGetDevice(&dev));
        PCPP_HIP_CHECK(hipDeviceGetAttribute(&per_block, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
        if (2 * lds + (size_t)2 * SEARCH_WAVES * KEEP_MAX * sizeof(uint32_t) + 1024 > (size_t)per_block) one_pass = false;
        else if ((rc = raise_lds_limit(ext ? reinterpret_cast<const void *>(&query_count<false, true, true>)
                                           : reinterpret_cast<const void *>(&query_count<false, true, false>), 2 * lds)) != PCPP_OK)
            return rc;
    }

    // the offsets of everything but the |T|-sized arrays do not depend on |T|
    const PlanLayout pl = want_plan ? plan_layout(n_in, n_out, K, 0, plan_flags) : PlanLayout{};
    if (want_plan && plan_bytes < pl.bytes) {
        set_error("pcpp_build_triplets: plan buffer has %zu bytes, needs at least %zu", plan_bytes, pl.bytes);
        return PCPP_ERR_WORKSPACE;
    }
    char *pb = static_cast<char *>(plan);
    uint32_t *f_ptr = reinterpret_cast<uint32_t *>(ws + bs.fwd_ptr_off);
    uint32_t *f_cnt = reinterpret_cast<uint32_t *>(ws + bs.fwd_cnt_off);
    uint32_t *b_cnt = reinterpret_cast<uint32_t *>(ws + bs.bwd_cnt_off);
    uint32_t *b_sum = reinterpret_cast<uint32_t *>(ws + bs.bwd_ptr_off);   // per-(k, tile) sums of the swapped side
    const CountOut none{nullptr, nullptr, nullptr};
    // the plan's own tables, when the first pass already runs in the plan's order (a plain plan)
    const bool fwd_direct = want_plan && !spatial;
    uint32_t *f_off = fwd_direct ? reinterpret_cast<uint32_t *>(pb + pl.fwd.tile_ptr_off) : f_ptr;

    // ---- the public list: centres = outputs in index order, candidates = inputs ------------------------------
    // With a plan in spatial order the same neighbourhoods are counted again in slot order: given the room, this pass
    // leaves its lists where that one can read them while it writes its own.
    const bool reuse_lists = keep_hits && spatial && !ext && !count_only && workspace_bytes >= bs.end_with_reuse;
    uint32_t *pub_hits = reuse_lists ? reinterpret_cast<uint32_t *>(ws + bs.pub_hits_off) : f_hits;
    uint32_t *pub_n = reuse_lists ? reinterpret_cast<uint32_t *>(ws + bs.n_hits_off) : nullptr;
    const Reuse from_public{reuse_lists ? pub_hits : nullptr, pub_n, in_xyz};
    if (nt_o > 0) {
        const CountOut fwd_out{count_only ? nullptr : f_cnt, f_ptr, pub_hits, pub_n};
        if (one_pass && !spatial)
            {
                if (ext) query_count<false, true, true><<<(unsigned)nt_o, SEARCH_THREADS, 2 * lds, stream>>>(
                out_xyz, n_out, nullptr, grid_in, q, K, nt_o, fwd_out, CountOut{b_cnt, b_sum, b_hits}, bs.fwd_stride, err, no_reuse);
                else query_count<false, true, false><<<(unsigned)nt_o, SEARCH_THREADS, 2 * lds, stream>>>(
                out_xyz, n_out, nullptr, grid_in, q, K, nt_o, fwd_out, CountOut{b_cnt, b_sum, b_hits}, bs.fwd_stride, err, no_reuse);
            }
        else
            {
                if (ext) query_count<false, false, true><<<(unsigned)nt_o, SEARCH_THREADS, lds, stream>>>(
                out_xyz, n_out, nullptr, grid_in, q, K, nt_o, fwd_out, none, bs.fwd_stride, err, no_reuse);
                else query_count<false, false, false><<<(unsigned)nt_o, SEARCH_THREADS, lds, stream>>>(
                out_xyz, n_out, nullptr, grid_in, q, K, nt_o, fwd_out, none, bs.fwd_stride, err, no_reuse);
            }
        PCPP_HIP_CHECK(hipGetLastError());
    }
    if ((rc = scan_exclusive_u32(f_ptr, f_off, (int64_t)K * nt_o, scan_scratch(SCAN_PUBLIC), total_dev, err, stream)) != PCPP_OK)
        return rc;
    CallEvent landed;
    unsigned long long total = 0;
    bool have_total = false;
    auto wait_total = [&]() -> int {
        if (!have_total) {
            if (pinned) {
                PCPP_HIP_CHECK(hipEventSynchronize(landed.ev));
                total = *reinterpret_cast<volatile unsigned long long *>(n_triplets);
            } else {
                PCPP_HIP_CHECK(hipMemcpyAsync(&total, total_dev, sizeof(total), hipMemcpyDeviceToHost, stream));
                PCPP_HIP_CHECK(hipStreamSynchronize(stream));
            }
            have_total = true;
        }
        if (total == ~0ull) {
            *n_triplets = 0;
            set_error("pcpp_build_triplets: a wait inside a device-wide prefix sum ran out");
            return PCPP_ERR_HIP;
        }
        *n_triplets = (int64_t)total;
        if (total >= (unsigned long long)INT32_MAX) {
            set_error("pcpp_build_triplets: %llu triplets; the library indexes at most 2^31-1", total);
            return PCPP_ERR_UNSUPPORTED;
        }
        return PCPP_OK;
    };
    if (pinned) {
        PCPP_HIP_CHECK(hipEventCreateWithFlags(&landed.ev, hipEventDisableTiming));
        PCPP_HIP_CHECK(hipEventRecord(landed.ev, stream));
    } else if ((rc = wait_total()) != PCPP_OK) {
        return rc;
    }
    if (count_only) return wait_total();

    const uint32_t tri_cap = (uint32_t)(capacity < (int64_t)INT32_MAX ? capacity : (int64_t)INT32_MAX);
    // how many triplets the |T|-sized arrays of the plan have room for
    uint32_t tail_cap = 0;
    if (want_plan && pl.n_tail > 0) {
        const size_t room = (plan_bytes - pl.tail_off) / (size_t)pl.n_tail / 256 * 256 / 4;
        tail_cap = (uint32_t)(room < (size_t)tri_cap ? room : (size_t)tri_cap);
    }
    if (nt_o > 0) {
        uint32_t *f_runs = fwd_direct ? reinterpret_cast<uint32_t *>(pb + pl.fwd.run_start_off) : nullptr;
        {
                if (ext) query_fill<false, true><<<(unsigned)nt_o, SEARCH_THREADS, lds_fill, stream>>>(
            out_xyz, n_out, nullptr, grid_in, q, K, nt_o, f_cnt, f_off, FillOut{tri_o, tri_i, tri_k, nullptr, -1, tri_cap},
            f_runs, list_cap, pub_hits, bs.fwd_stride, seg_offsets, pack_ok, err);
                else query_fill<false, false><<<(unsigned)nt_o, SEARCH_THREADS, lds_fill, stream>>>(
            out_xyz, n_out, nullptr, grid_in, q, K, nt_o, f_cnt, f_off, FillOut{tri_o, tri_i, tri_k, nullptr, -1, tri_cap},
            f_runs, list_cap, pub_hits, bs.fwd_stride, seg_offsets, pack_ok, err);
            }
        PCPP_HIP_CHECK(hipGetLastError());
    } else {
        // no outputs: every run starts at 0
        if ((rc = fill_u64(reinterpret_cast<unsigned long long *>(seg_offsets), 0ull, K + 1, stream)) != PCPP_OK) return rc;
    }

    // ---- the plan's sides ---------------------------------------------------------------------------------------
    GridView grid_out = grid_in;
    if (want_bwd && !self) {
        if ((rc = build_grid(out_xyz, n_out, gm, out_batch_offsets, n_batches, ws, bs.grid_out, scan_scratch(SCAN_GRID_OUT),
                             nullptr, 0, err, &grid_out, stream)) != PCPP_OK)
            return rc;
    }
    const int32_t *perm_o = nullptr, *perm_i = nullptr;
    if (spatial) {
        // cells of half the radius: a tile of 64 centres then spans a few radii at the densities the layers see
        const double pitch = 0.5 * R;
        int32_t *po = reinterpret_cast<int32_t *>(pb + pl.fwd.perm_off);
        if ((rc = spatial_order(out_xyz, n_out, pitch, po, ws + bs.sort_off, scan_scratch(SCAN_SORT_OUT), bs.scan_stride,
                                err, stream)) != PCPP_OK)
            return rc;
        perm_o = po;
        if (want_bwd) {
            int32_t *pi = reinterpret_cast<int32_t *>(pb + pl.bwd.perm_off);
            if (self) {
                PCPP_HIP_CHECK(hipMemcpyAsync(pi, po, (size_t)n_in * 4, hipMemcpyDeviceToDevice, stream));
            } else if ((rc = spatial_order(in_xyz, n_in, pitch, pi, ws + bs.sort_off, scan_scratch(SCAN_SORT_IN),
                                           bs.scan_stride, err, stream)) != PCPP_OK) {
                return rc;
            }
            perm_i = pi;
        }
        // forward side in the spatial order: same search, centres taken through the permutation
        uint32_t *sf_ptr = reinterpret_cast<uint32_t *>(pb + pl.fwd.tile_ptr_off);
        if (nt_o > 0) {
            const CountOut fwd_out{f_cnt, f_ptr, f_hits};
            if (one_pass)
                {
                if (ext) query_count<false, true, true><<<(unsigned)nt_o, SEARCH_THREADS, 2 * lds, stream>>>(
                    out_xyz, n_out, perm_o, grid_in, q, K, nt_o, fwd_out, CountOut{b_cnt, b_sum, b_hits}, bs.fwd_stride, err, from_public);
                else query_count<false, true, false><<<(unsigned)nt_o, SEARCH_THREADS, 2 * lds, stream>>>(
                    out_xyz, n_out, perm_o, grid_in, q, K, nt_o, fwd_out, CountOut{b_cnt, b_sum, b_hits}, bs.fwd_stride, err, from_public);
            }
            else
                {
                if (ext) query_count<false, false, true><<<(unsigned)nt_o, SEARCH_THREADS, lds, stream>>>(
                    out_xyz, n_out, perm_o, grid_in, q, K, nt_o, fwd_out, none, bs.fwd_stride, err, from_public);
                else query_count<false, false, false><<<(unsigned)nt_o, SEARCH_THREADS, lds, stream>>>(
                    out_xyz, n_out, perm_o, grid_in, q, K, nt_o, fwd_out, none, bs.fwd_stride, err, from_public);
            }
            PCPP_HIP_CHECK(hipGetLastError());
        }
        if ((rc = scan_exclusive_u32(f_ptr, sf_ptr, (int64_t)K * nt_o, scan_scratch(SCAN_FWD_SIDE), nullptr, err, stream)) != PCPP_OK)
            return rc;
        if (nt_o > 0) {
            {
                if (ext) query_fill<false, true><<<(unsigned)nt_o, SEARCH_THREADS, lds_fill, stream>>>(
                out_xyz, n_out, perm_o, grid_in, q, K, nt_o, f_cnt, sf_ptr,
                FillOut{nullptr, nullptr, nullptr, pb + pl.tail_off, pl.fwd.gather_index, tail_cap},
                reinterpret_cast<uint32_t *>(pb + pl.fwd.run_start_off), list_cap, f_hits, bs.fwd_stride, nullptr, pack_ok, err);
                else query_fill<false, false><<<(unsigned)nt_o, SEARCH_THREADS, lds_fill, stream>>>(
                out_xyz, n_out, perm_o, grid_in, q, K, nt_o, f_cnt, sf_ptr,
                FillOut{nullptr, nullptr, nullptr, pb + pl.tail_off, pl.fwd.gather_index, tail_cap},
                reinterpret_cast<uint32_t *>(pb + pl.fwd.run_start_off), list_cap, f_hits, bs.fwd_stride, nullptr, pack_ok, err);
            }
            PCPP_HIP_CHECK(hipGetLastError());
        }
    }
    if (want_bwd) {
        // input-gradient side: centres = inputs, candidates = outputs; same predicate with the roles
        // swapped, so the set is identical and only the grouping changes to (k, i, o)
        uint32_t *b_ptr = reinterpret_cast<uint32_t *>(pb + pl.bwd.tile_ptr_off);
        uint32_t *b_runs = reinterpret_cast<uint32_t *>(pb + pl.bwd.run_start_off);
        if (nt_i > 0 && !one_pass) {
            {
                if (ext) query_count<true, false, true><<<(unsigned)nt_i, SEARCH_THREADS, lds, stream>>>(
                in_xyz, n_in, perm_i, grid_out, qs, K, nt_i, CountOut{b_cnt, b_sum, b_hits}, none, bs.bwd_stride, err, no_reuse);
                else query_count<true, false, false><<<(unsigned)nt_i, SEARCH_THREADS, lds, stream>>>(
                in_xyz, n_in, perm_i, grid_out, qs, K, nt_i, CountOut{b_cnt, b_sum, b_hits}, none, bs.bwd_stride, err, no_reuse);
            }
            PCPP_HIP_CHECK(hipGetLastError());
        }
        if ((rc = scan_exclusive_u32(b_sum, b_ptr, (int64_t)K * nt_i, scan_scratch(SCAN_BWD_SIDE), nullptr, err, stream)) != PCPP_OK)
            return rc;
        if (nt_i > 0) {
            {
                if (ext) query_fill<true, true><<<(unsigned)nt_i, SEARCH_THREADS, lds_fill, stream>>>(
                in_xyz, n_in, perm_i, grid_out, qs, K, nt_i, b_cnt, b_ptr,
                FillOut{nullptr, nullptr, nullptr, pb + pl.tail_off, pl.bwd.gather_index, tail_cap}, b_runs, list_cap,
                b_hits, bs.bwd_stride, nullptr, pack_ok, err);
                else query_fill<true, false><<<(unsigned)nt_i, SEARCH_THREADS, lds_fill, stream>>>(
                in_xyz, n_in, perm_i, grid_out, qs, K, nt_i, b_cnt, b_ptr,
                FillOut{nullptr, nullptr, nullptr, pb + pl.tail_off, pl.bwd.gather_index, tail_cap}, b_runs, list_cap,
                b_hits, bs.bwd_stride, nullptr, pack_ok, err);
            }
            PCPP_HIP_CHECK(hipGetLastError());
        }
    }
    // everything is queued; now compare the count with what the caller provided
    if ((rc = wait_total()) != PCPP_OK) return rc;
    if ((int64_t)total > capacity) {
        set_error("pcpp_build_triplets: %llu triplets but capacity is %lld", total, (long long)capacity);
        return PCPP_ERR_CAPACITY;
    }
    if (plan) {
        const size_t need = plan_layout(n_in, n_out, K, (int64_t)total, plan_flags).bytes;
        if (plan_bytes < need) {
            set_error("pcpp_build_triplets: plan buffer has %zu bytes, needs %zu", plan_bytes, need);
            return PCPP_ERR_WORKSPACE;
        }
    }
    return PCPP_OK;
}

size_t pcpp_voxel_subsample_workspace_bytes(int64_t n)
{
    if (n < 0 || n >= INT32_MAX) return 0;
    return sub_scratch(n).end;
}

int pcpp_voxel_subsample(const float *xyz, int64_t n, float pitch, int32_t *kept, int64_t *n_kept, void *workspace,
                         size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (n < 0 || (n > 0 && (!xyz || !kept)) || !n_kept) {
        set_error("pcpp_voxel_subsample: null pointer or negative size");
        return PCPP_ERR_INVALID_ARG;
    }
    if (n >= INT32_MAX) {
        set_error("pcpp_voxel_subsample: point count must be below 2^31");
        return PCPP_ERR_UNSUPPORTED;
    }
    if (!(pitch > 0.0f) || !isfinite(pitch)) {
        set_error("pcpp_voxel_subsample: pitch must be finite and positive");
        return PCPP_ERR_INVALID_ARG;
    }
    const SubScratch ss = sub_scratch(n);
    if (!workspace || workspace_bytes < ss.end || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
        set_error("pcpp_voxel_subsample: workspace missing, misaligned or smaller than %zu bytes", ss.end);
        return PCPP_ERR_WORKSPACE;
    }
    *n_kept = 0;
    if (n == 0) return PCPP_OK;
    char *ws = static_cast<char *>(workspace);
    auto *keys = reinterpret_cast<unsigned long long *>(ws + ss.keys_off);
    int *lowest = reinterpret_cast<int *>(ws + ss.lowest_off);
    auto *point_slot = reinterpret_cast<uint32_t *>(ws + ss.slot_off);
    auto *flag = reinterpret_cast<uint32_t *>(ws + ss.flag_off);
    auto *err = reinterpret_cast<uint32_t *>(ws + ss.err_off);
    unsigned long long *total_dev = reinterpret_cast<unsigned long long *>(ws + ss.total_off);
    bool pinned = false;
    {
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, n_kept) == hipSuccess && attr.type == hipMemoryTypeHost && attr.devicePointer) {
            total_dev = static_cast<unsigned long long *>(attr.devicePointer);
            pinned = true;
        } else {
            (void)hipGetLastError();
        }
    }
    int64_t blocks = ceil_div(ss.slots, 256);
    if (blocks > 4096) blocks = 4096;
    // the error word, the landing word and the prefix sum's status words are contiguous at the start of the workspace
    sub_clear<<<(unsigned)blocks, 256, 0, stream>>>(keys, lowest, ss.slots, reinterpret_cast<unsigned long long *>(ws),
                                                    (int64_t)(ss.keys_off / sizeof(unsigned long long)));
    const unsigned pb = (unsigned)ceil_div(n, 256);
    sub_insert<<<pb, 256, 0, stream>>>(xyz, n, (double)pitch, keys, lowest, (uint32_t)(ss.slots - 1), point_slot);
    sub_flag<<<pb, 256, 0, stream>>>(n, lowest, point_slot, flag);
    PCPP_HIP_CHECK(hipGetLastError());
    int rc;
    if ((rc = scan_exclusive_u32(flag, flag, n, ws + ss.scan_off, total_dev, err, stream)) != PCPP_OK) return rc;
    sub_scatter<<<pb, 256, 0, stream>>>(n, flag, kept, err);
    PCPP_HIP_CHECK(hipGetLastError());
    unsigned long long total = 0;
    if (pinned) {
        PCPP_HIP_CHECK(hipStreamSynchronize(stream));
        total = *reinterpret_cast<volatile unsigned long long *>(n_kept);
    } else {
        PCPP_HIP_CHECK(hipMemcpyAsync(&total, total_dev, sizeof(total), hipMemcpyDeviceToHost, stream));
        PCPP_HIP_CHECK(hipStreamSynchronize(stream));
    }
    if (total == ~0ull) {
        *n_kept = 0;
        set_error("pcpp_voxel_subsample: a wait inside a device-wide prefix sum ran out");
        return PCPP_ERR_HIP;
    }
    *n_kept = (int64_t)total;
    return PCPP_OK;
}

}  // extern "C"
