// Exclusion lists of FastPoint (arXiv 2507.23480) as a data structure of their own, for gfx950:
// the list-building loops of Algorithm 2 (Section 4.1 step 2) -- for every level l and every point i the points
// j with dist2(P_i, P_j) < R_l^2, one distance per pair serving all levels -- plus the extra list
// at the ball-query radius of Section 4.2, and the ball query that is a lookup in such a list.
//
// The paper builds the lists from all N^2 pairs.  Here a uniform grid with cells at least as
// wide as the largest radius of the cloud limits the pairs that are examined to the 27 cells
// around a point; the lists that come out are those of the all-pairs loop, in its order
// (ascending j).
//
//   grid_*        bounding box, cell size and dimensions per cloud, points counted and scattered
//                 into cell order (x, y, z and the original index as one 16-byte record)
//   excl_count    one wave per point: the 9 runs of 3 x-adjacent cells are contiguous in cell
//                 order; 64 candidates per pass, one distance each, compared with every level;
//                 lane l keeps the size of the level-l list
//   scan_*        sizes -> row offsets (64-bit, in place)
//   excl_fill     one wave per point: the hits at the largest radius are collected in LDS, sorted
//                 by index (bitonic network, one wave, no barriers), then walked in order; each
//                 level keeps the members below its own radius (ballot compaction keeps the
//                 order).  A point with more hits than the LDS buffer holds is left to
//   excl_fill_heavy: ascending index is the order of a bitmap -- the wave marks the hits of the
//                 27 cells in a bitmap over a slab of 32768 or 65536 indices (LDS), reads it back 64
//                 words a pass and walks the indices of the set bits; no sort.
//   bq_lists      first k members of a row, padded with the first
//
// Squared distances are evaluated as ((dx*dx)+(dy*dy))+(dz*dz), every operation rounded on its
// own; the file is compiled with -ffp-contract=off and without packed fp32 instructions.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

#pragma clang fp contract(off)

namespace fastpoint {
namespace {

constexpr int kWaves = 4;              // waves (= points) per workgroup of the list kernels
constexpr int kSortCap = 2048;         // hits at the largest radius that one wave sorts in LDS
constexpr int kHeavyWaves = 4;         // waves (= points) per workgroup of the kernel for longer rows
constexpr int kSlabWordsMax = 2048;    // 32-bit words of one wave's index bitmap: a slab of up to 65536 indices
constexpr int kScanBlock = 2048;       // elements per workgroup of the offset scan (256 threads x 8)
constexpr int kCellTile = 16384;       // cells per workgroup of the scan over a grid's cells (1024 threads x 16)
constexpr float kCellSlack = 1.001f;   // cell width = largest radius x this (absorbs the rounding of
                                       // the cell coordinate, at most 1024 cells per axis)

__device__ __forceinline__ float dist2(float ax, float ay, float az, float bx, float by, float bz)
{
    float dx = ax - bx;
    float dy = ay - by;
    float dz = az - bz;
    float t = dx * dx;
    t = t + dy * dy;
    t = t + dz * dz;
    return t;
}

__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                          __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
__device__ __forceinline__ uint32_t rdlane(uint32_t v, int l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, l);
}
__device__ __forceinline__ float rdlane_f(float v, int l)
{
    return __uint_as_float(rdlane(__float_as_uint(v), l));
}
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// order-preserving map of binary32 to uint32 (for atomicMin / atomicMax on coordinates)
__device__ __forceinline__ uint32_t f2ord(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ord2f(uint32_t o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}

__device__ __forceinline__ int cell_coord(float x, float lo, float inv_h, int dim)
{
    int c = (int)((x - lo) * inv_h);
    c = c < 0 ? 0 : c;
    return c > dim - 1 ? dim - 1 : c;
}

// ----------------------------------------------------------------------------- grid
__global__ void grid_init_kernel(ExclGrid* gp, int B, int32_t* cell_cnt, int64_t ncnt)
{
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (t < B) {
        gp[t].lo[0] = gp[t].lo[1] = gp[t].lo[2] = 0xFFFFFFFFu;
        gp[t].hi[0] = gp[t].hi[1] = gp[t].hi[2] = 0u;
    }
    for (; t < ncnt; t += stride) cell_cnt[t] = 0;
}

__global__ __launch_bounds__(256) void grid_bounds_kernel(const float* __restrict__ xyz, int N, ExclGrid* gp)
{
    __shared__ uint32_t slo[4][3], shi[4][3];
    const int b = (int)blockIdx.y;
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    uint32_t lo[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, hi[3] = {0u, 0u, 0u};
    for (int i = (int)(blockIdx.x * 256 + threadIdx.x); i < N; i += (int)gridDim.x * 256) {
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            const float v = cloud[(int64_t)i * 3 + a];
            if (v == v) {                           // NaN coordinates (gathers of bad indices) do not count
                const uint32_t o = f2ord(v);
                lo[a] = min(lo[a], o);
                hi[a] = max(hi[a], o);
            }
        }
    }
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        for (int s = 32; s > 0; s >>= 1) {
            lo[a] = min(lo[a], (uint32_t)__shfl_xor((int)lo[a], s, 64));
            hi[a] = max(hi[a], (uint32_t)__shfl_xor((int)hi[a], s, 64));
        }
        if ((threadIdx.x & 63) == 0) {
            slo[threadIdx.x >> 6][a] = lo[a];
            shi[threadIdx.x >> 6][a] = hi[a];
        }
    }
    __syncthreads();
    if (threadIdx.x < 3) {              // one atomic pair per axis and workgroup
        const int a = (int)threadIdx.x;
        atomicMin(&gp[b].lo[a], min(min(slo[0][a], slo[1][a]), min(slo[2][a], slo[3][a])));
        atomicMax(&gp[b].hi[a], max(max(shi[0][a], shi[1][a]), max(shi[2][a], shi[3][a])));
    }
}

// One thread per cloud: the largest radius, the cell width and the grid dimensions.
__global__ void grid_setup_kernel(ExclGrid* gp, int B, const float* __restrict__ thr2, int L, int maxcells,
                                  float r2_all)
{
    const int b = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (b >= B) return;
    ExclGrid g = gp[b];
    float rmax2 = 0.0f;
    int lmax = 0;
    for (int l = 0; l < L; ++l) {
        const float t = thr2 ? thr2[(int64_t)b * L + l] : r2_all;      // no table: one radius for all clouds
        if (t > rmax2) {            // NaN and values <= 0 never win
            rmax2 = t;
            lmax = l;
        }
    }
    float ext[3];
    for (int a = 0; a < 3; ++a) {
        g.origin[a] = ord2f(g.lo[a]);
        ext[a] = ord2f(g.hi[a]) - g.origin[a];
        if (!(ext[a] >= 0.0f)) ext[a] = 0.0f;
    }
    float h = sqrtf(rmax2) * kCellSlack;
    const float emax = fmaxf(ext[0], fmaxf(ext[1], ext[2]));
    if (!(h > emax * (1.0f / 1024.0f))) h = emax * (1.0f / 1024.0f);      // at most 1024 cells per axis
    if (!(h > 0.0f)) h = 1.0f;                                             // all points coincide, radius 0
    int dim[3];
    for (int it = 0; it < 200; ++it) {
        int64_t cells = 1;
        for (int a = 0; a < 3; ++a) {
            const float q = ext[a] / h;
            dim[a] = q < 1023.0f ? (int)q + 1 : 1024;
            cells *= dim[a];
        }
        if (cells <= maxcells) break;
        h = h * 1.26f;
    }
    if ((int64_t)dim[0] * dim[1] * dim[2] > maxcells) dim[0] = dim[1] = dim[2] = 1;   // h overflowed
    g.inv_h = 1.0f / h;
    if (!(g.inv_h > 0.0f && g.inv_h < 3.0e38f)) {         // h = +inf or denormal: one cell
        g.inv_h = 0.0f;
        dim[0] = dim[1] = dim[2] = 1;
    }
    g.dim[0] = dim[0];
    g.dim[1] = dim[1];
    g.dim[2] = dim[2];
    g.ncells = dim[0] * dim[1] * dim[2];
    g.rmax2 = rmax2;
    g.lmax = lmax;
    g.curve_bits = 0;
    gp[b] = g;
}

// Position of cell (cx, cy, cz) of a 2^b x 2^b x 2^b grid along a Hilbert curve: consecutive
// positions are cells that share a face, so a run of consecutive cells is a compact piece of space
// wherever it starts (a curve by bit interleaving jumps across the grid at every power of two).
// Skilling's transform of the coordinates (AIP Conf. Proc. 707, 2004): from the top bit down,
// exchange or invert the low bits according to the bits above, Gray-code the result, and read the
// three words bit by bit.
__device__ __forceinline__ int hilbert_index(int cx, int cy, int cz, int b)
{
    uint32_t X[3] = {(uint32_t)cx, (uint32_t)cy, (uint32_t)cz};
    const uint32_t top = 1u << (b - 1);
    for (uint32_t q = top; q > 1; q >>= 1) {
        const uint32_t low = q - 1;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            if (X[i] & q) {
                X[0] ^= low;
            } else {
                const uint32_t t = (X[0] ^ X[i]) & low;
                X[0] ^= t;
                X[i] ^= t;
            }
        }
    }
    X[1] ^= X[0];
    X[2] ^= X[1];
    uint32_t t = 0;
    for (uint32_t q = top; q > 1; q >>= 1)
        if (X[2] & q) t ^= q - 1;
    X[0] ^= t;
    X[1] ^= t;
    X[2] ^= t;
    uint32_t id = 0;
    for (int k = b - 1; k >= 0; --k)
        id = (id << 3) | (((X[0] >> k) & 1u) << 2) | (((X[1] >> k) & 1u) << 1) | ((X[2] >> k) & 1u);
    return (int)id;
}

__device__ __forceinline__ int cell_of(const ExclGrid& g, float x, float y, float z, int& cx, int& cy, int& cz)
{
    cx = cell_coord(x, g.origin[0], g.inv_h, g.dim[0]);
    cy = cell_coord(y, g.origin[1], g.inv_h, g.dim[1]);
    cz = cell_coord(z, g.origin[2], g.inv_h, g.dim[2]);
    if (g.curve_bits > 0) return hilbert_index(cx, cy, cz, g.curve_bits);
    return (cz * g.dim[1] + cy) * g.dim[0] + cx;
}

// One thread per cloud: a cubic grid of 2^bits cells per axis over the bounding box.
__global__ void sort_setup_kernel(ExclGrid* gp, int B, int bits)
{
    const int b = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (b >= B) return;
    ExclGrid g = gp[b];
    float emax = 0.0f;
    for (int a = 0; a < 3; ++a) {
        g.origin[a] = ord2f(g.lo[a]);
        const float e = ord2f(g.hi[a]) - g.origin[a];
        if (e > emax) emax = e;
    }
    const int dim = 1 << bits;
    g.inv_h = emax > 0.0f ? (float)dim / emax : 0.0f;
    if (!(g.inv_h < 3.0e38f)) g.inv_h = 0.0f;        // extent too small to divide: one cell
    g.dim[0] = g.dim[1] = g.dim[2] = dim;
    g.ncells = dim * dim * dim;
    g.rmax2 = 0.0f;
    g.lmax = 0;
    g.curve_bits = bits;
    gp[b] = g;
}

// Adds 1 to counter[cell] for every lane with `todo` and returns the value the counter had for
// this lane (as if the lanes had added one after the other).  Lanes of a wave that share a cell
// send one atomic together: clouds in scan order put most of a wave into one or two cells, and
// thousands of single atomics on one address would queue up.  After a few distinct cells the
// remaining lanes add on their own.
__device__ __forceinline__ int grouped_add(int32_t* counter, int cell, bool todo, int lane)
{
    int pos = 0;
    for (int it = 0; it < 6; ++it) {
        const uint64_t act = __builtin_amdgcn_ballot_w64(todo);
        if (act == 0) return pos;
        const int leader = __builtin_ctzll(act);
        const int c0 = (int)rdlane((uint32_t)cell, leader);
        const bool mine = todo && cell == c0;
        const uint64_t same = __builtin_amdgcn_ballot_w64(mine);
        int base = 0;
        if (lane == leader) base = atomicAdd(&counter[c0], (int)__builtin_popcountll(same));
        base = (int)rdlane((uint32_t)base, leader);
        if (mine) {
            pos = base + lanes_below(same);
            todo = false;
        }
    }
    if (todo) pos = atomicAdd(&counter[cell], 1);
    return pos;
}

__global__ __launch_bounds__(256) void grid_count_kernel(const float* __restrict__ xyz, int N,
                                                         const ExclGrid* __restrict__ gp, int32_t* cell_cnt,
                                                         int maxcells)
{
    const int b = (int)blockIdx.y;
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    const bool valid = i < N;
    const ExclGrid g = gp[b];
    const float* p = xyz + ((int64_t)b * N + (valid ? i : 0)) * 3;
    int cx, cy, cz;
    const int c = cell_of(g, p[0], p[1], p[2], cx, cy, cz);
    grouped_add(cell_cnt + (int64_t)b * maxcells, c, valid, (int)threadIdx.x & 63);
}

// One workgroup per cloud: cell_start = exclusive scan of the cell counts; the counts become
// the scatter cursors.
// Exclusive scan of the cell counts of every cloud (cell starts, and the cursors of the scatter), in
// tiles of kCellTile cells: a first launch adds up every tile, the second gives every tile the sum
// of the tiles in front of it and scans inside.  A thread takes 16 consecutive cells (four 16-byte
// reads and writes where the arrays are aligned for them).
constexpr int kCellPer = 16;
static_assert(kCellTile == 1024 * kCellPer, "a tile is what one workgroup takes in one turn");

__device__ __forceinline__ void load_cells(const int32_t* cnt, int c0, int ncells, bool wide, int (&v)[kCellPer])
{
    if (c0 + kCellPer <= ncells && wide) {
#pragma unroll
        for (int q = 0; q < kCellPer / 4; ++q) {
            const int4 t = reinterpret_cast<const int4*>(cnt + c0)[q];
            v[4 * q] = t.x;
            v[4 * q + 1] = t.y;
            v[4 * q + 2] = t.z;
            v[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int u = 0; u < kCellPer; ++u) v[u] = c0 + u < ncells ? cnt[c0 + u] : 0;
    }
}

// sum over the workgroup (1024 threads); every thread gets it
__device__ __forceinline__ int block_sum_1024(int v, int32_t* wsum16)
{
    const int tid = (int)threadIdx.x, lane = tid & 63, w = tid >> 6;
    for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, 64);
    if (lane == 0) wsum16[w] = v;
    __syncthreads();
    int total = 0;
    for (int k = 0; k < 16; ++k) total += wsum16[k];
    __syncthreads();
    return total;
}

__global__ __launch_bounds__(1024) void grid_tile_sum_kernel(const ExclGrid* __restrict__ gp,
                                                             const int32_t* __restrict__ cell_cnt,
                                                             int32_t* __restrict__ tile_sum, int maxcells, int tiles)
{
    __shared__ int32_t wsum[16];
    const int b = (int)blockIdx.y, t = (int)blockIdx.x;
    const int ncells = gp[b].ncells;
    const int32_t* cnt = cell_cnt + (int64_t)b * maxcells;
    const bool wide = (reinterpret_cast<uintptr_t>(cnt) & 15u) == 0;
    int v[kCellPer];
    load_cells(cnt, t * kCellTile + (int)threadIdx.x * kCellPer, ncells, wide, v);
    int tsum = 0;
#pragma unroll
    for (int u = 0; u < kCellPer; ++u) tsum += v[u];
    const int total = block_sum_1024(tsum, wsum);
    if (threadIdx.x == 0) tile_sum[(int64_t)b * tiles + t] = total;
}

__global__ __launch_bounds__(1024) void grid_scan_kernel(const ExclGrid* __restrict__ gp, int32_t* cell_cnt,
                                                         int32_t* cell_start, const int32_t* __restrict__ tile_sum,
                                                         int maxcells, int tiles)
{
    __shared__ int32_t wsum[16];
    const int b = (int)blockIdx.y, t = (int)blockIdx.x;
    const int ncells = gp[b].ncells;
    const int base = t * kCellTile;
    if (base >= ncells) return;                          // uniform over the workgroup
    int32_t* cnt = cell_cnt + (int64_t)b * maxcells;
    int32_t* st = cell_start + (int64_t)b * (maxcells + 1);
    const bool cnt_wide = (reinterpret_cast<uintptr_t>(cnt) & 15u) == 0;
    const bool st_wide = (reinterpret_cast<uintptr_t>(st) & 15u) == 0;
    const int tid = (int)threadIdx.x, lane = tid & 63, w = tid >> 6;
    // what lies in front of this tile
    int front = 0;
    for (int k = tid; k < t; k += 1024) front += tile_sum[(int64_t)b * tiles + k];
    const int carry = block_sum_1024(front, wsum);
    const int c0 = base + tid * kCellPer;
    const bool full = c0 + kCellPer <= ncells;
    int v[kCellPer];
    load_cells(cnt, c0, ncells, cnt_wide, v);
    int tsum = 0;
#pragma unroll
    for (int u = 0; u < kCellPer; ++u) tsum += v[u];
    int incl = tsum;
    for (int s = 1; s < 64; s <<= 1) {
        const int up = __shfl_up(incl, s, 64);
        if (lane >= s) incl += up;
    }
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    int woff = 0;
    for (int k = 0; k < 16; ++k) woff += (k < w) ? wsum[k] : 0;
    int total = 0;
    for (int k = 0; k < 16; ++k) total += wsum[k];
    int run = carry + woff + incl - tsum;
#pragma unroll
    for (int u = 0; u < kCellPer; ++u) {                 // v becomes the exclusive prefix: start and scatter cursor
        const int mine = v[u];
        v[u] = run;
        run += mine;
    }
    if (full && cnt_wide) {
#pragma unroll
        for (int q = 0; q < kCellPer / 4; ++q)
            reinterpret_cast<int4*>(cnt + c0)[q] = make_int4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    } else {
#pragma unroll
        for (int u = 0; u < kCellPer; ++u)
            if (c0 + u < ncells) cnt[c0 + u] = v[u];
    }
    if (full && st_wide) {
#pragma unroll
        for (int q = 0; q < kCellPer / 4; ++q)
            reinterpret_cast<int4*>(st + c0)[q] = make_int4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    } else {
#pragma unroll
        for (int u = 0; u < kCellPer; ++u)
            if (c0 + u < ncells) st[c0 + u] = v[u];
    }
    if (tid == 0 && base + kCellTile >= ncells) st[ncells] = carry + total;      // the cloud's last tile
}

// the two launches of the scan; a grid of one tile per cloud has no tiles in front of any and
// takes the second only
static void launch_cell_scan(const ExclGrid* gp, int32_t* cnt, int32_t* st, int32_t* tile_sum, int B, int maxcells,
                             hipStream_t stream)
{
    const int tiles = (maxcells + kCellTile - 1) / kCellTile;
    const dim3 grid((unsigned)tiles, (unsigned)B);
    if (tiles > 1)
        hipLaunchKernelGGL(grid_tile_sum_kernel, grid, dim3(1024), 0, stream, gp, (const int32_t*)cnt, tile_sum,
                           maxcells, tiles);
    hipLaunchKernelGGL(grid_scan_kernel, grid, dim3(1024), 0, stream, gp, cnt, st, (const int32_t*)tile_sum, maxcells,
                       tiles);
}

__global__ __launch_bounds__(256) void grid_scatter_kernel(const float* __restrict__ xyz, int N,
                                                           const ExclGrid* __restrict__ gp, int32_t* cell_cur,
                                                           float4* __restrict__ sorted, int maxcells)
{
    const int b = (int)blockIdx.y;
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    const bool valid = i < N;
    const ExclGrid g = gp[b];
    const float* p = xyz + ((int64_t)b * N + (valid ? i : 0)) * 3;
    const float x = p[0], y = p[1], z = p[2];
    int cx, cy, cz;
    const int c = cell_of(g, x, y, z, cx, cy, cz);
    const int pos = grouped_add(cell_cur + (int64_t)b * maxcells, c, valid, (int)threadIdx.x & 63);
    if (valid) sorted[(int64_t)b * N + pos] = make_float4(x, y, z, __int_as_float(i));
}

// ------------------------------------------------------------------ walking the 27 cells
// Calls f(record, valid) for every point of the 27 cells around (cx, cy, cz), 64 per pass;
// all lanes take part in every call; f returns false (the same in all lanes) to end the walk.  The 9 runs of x-adjacent cells are contiguous in cell
// order: lanes 0..8 fetch the bounds of one run each, and the runs are then walked as one
// sequence, so a pass is full except for the last and the loads of successive passes do not
// wait for one another.
template <typename F>
__device__ __forceinline__ void for_neighbours(const ExclGrid& g, const int32_t* __restrict__ st,
                                               const float4* __restrict__ sorted, int cx, int cy, int cz,
                                               int lane, F f)
{
    const int x0 = cx > 0 ? cx - 1 : 0;
    const int x1 = cx < g.dim[0] - 1 ? cx + 1 : g.dim[0] - 1;
    int mybegin = 0, mylen = 0;
    if (lane < 9) {
        const int z = cz + lane / 3 - 1, y = cy + lane % 3 - 1;
        if (z >= 0 && z < g.dim[2] && y >= 0 && y < g.dim[1]) {
            const int c0 = (z * g.dim[1] + y) * g.dim[0] + x0;
            mybegin = st[c0];
            mylen = st[c0 + (x1 - x0) + 1] - mybegin;
        }
    }
    int begin[9], pre[10];
    pre[0] = 0;
#pragma unroll
    for (int r = 0; r < 9; ++r) {
        begin[r] = (int)rdlane((uint32_t)mybegin, r);
        pre[r + 1] = pre[r] + (int)rdlane((uint32_t)mylen, r);
    }
    const int total = pre[9];
    for (int t0 = 0; t0 < total; t0 += 64) {
        const int t = t0 + lane;
        const bool valid = t < total;
        int at = begin[0] + t;
#pragma unroll
        for (int r = 1; r < 9; ++r) at = t >= pre[r] ? begin[r] + (t - pre[r]) : at;
        const float4 rec = sorted[valid ? at : 0];
        if (!f(rec, valid)) break;
    }
}

// The same walk run by run (a last pass per run that may be partly empty; no search for the run a
// position falls into): cheaper per pass, for points with many passes.  The record of the next
// pass is requested before the current one is used.
template <typename F>
__device__ __forceinline__ void for_neighbour_runs(const ExclGrid& g, const int32_t* __restrict__ st,
                                                   const float4* __restrict__ sorted, int cx, int cy, int cz,
                                                   int lane, F f)
{
    const int x0 = cx > 0 ? cx - 1 : 0;
    const int x1 = cx < g.dim[0] - 1 ? cx + 1 : g.dim[0] - 1;
    int mybegin = 0, mylen = 0;
    if (lane < 9) {
        const int z = cz + lane / 3 - 1, y = cy + lane % 3 - 1;
        if (z >= 0 && z < g.dim[2] && y >= 0 && y < g.dim[1]) {
            const int c0 = (z * g.dim[1] + y) * g.dim[0] + x0;
            mybegin = st[c0];
            mylen = st[c0 + (x1 - x0) + 1] - mybegin;
        }
    }
    for (int r = 0; r < 9; ++r) {
        const int begin = (int)rdlane((uint32_t)mybegin, r);
        const int len = (int)rdlane((uint32_t)mylen, r);
        if (len <= 0) continue;
        const float4* __restrict__ run = sorted + begin;
        float4 cur = run[lane < len ? lane : 0];
        for (int t0 = 0; t0 < len; t0 += 64) {
            const int tn = t0 + 64 + lane;
            const float4 nxt = run[tn < len ? tn : 0];
            f(cur, t0 + lane < len);
            cur = nxt;
        }
    }
}

// Pass 1: lane l of the point's wave ends up with the size of the level-l list.
__global__ __launch_bounds__(kWaves * 64) void excl_count_kernel(
    const float* __restrict__ xyz, int B, int N, const float* __restrict__ thr2, int L,
    int64_t* __restrict__ offsets, const ExclGrid* __restrict__ gp, const int32_t* __restrict__ cell_start,
    const float4* __restrict__ sorted, int maxcells)
{
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int i = uni((int)blockIdx.x * kWaves + ((int)threadIdx.x >> 6));
    if (i >= N) return;
    const ExclGrid g = gp[b];
    const float* p = xyz + ((int64_t)b * N + i) * 3;
    const float px = p[0], py = p[1], pz = p[2];
    int cx, cy, cz;
    cell_of(g, px, py, pz, cx, cy, cz);
    const float mythr = lane < L ? thr2[(int64_t)b * L + lane] : 0.0f;
    int mycnt = 0;
    const float rmax2 = g.rmax2;
    for_neighbour_runs(g, cell_start + (int64_t)b * (maxcells + 1), sorted + (int64_t)b * N, cx, cy, cz, lane,
                       [&](const float4& r, bool valid) {
                           const float d = dist2(px, py, pz, r.x, r.y, r.z);
                           if (__builtin_amdgcn_ballot_w64(valid && d < rmax2) == 0) return;
                           for (int l = 0; l < L; ++l) {
                               const float t = rdlane_f(mythr, l);
                               const int pc = __builtin_popcountll(__builtin_amdgcn_ballot_w64(valid && d < t));
                               mycnt += lane == l ? pc : 0;
                           }
                       });
    if (lane < L) offsets[1 + ((int64_t)lane * B + b) * N + i] = mycnt;
}

// ----------------------------------------------------------- sizes -> offsets (in place)
__global__ __launch_bounds__(256) void scan_blocks_kernel(int64_t* __restrict__ v, int64_t count,
                                                          int64_t* __restrict__ totals)
{
    __shared__ int64_t wsum[4];
    const int tid = (int)threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + tid * 8;
    int64_t e[8];
    int64_t tsum = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        e[u] = base + u < count ? v[base + u] : 0;
        tsum += e[u];
    }
    int64_t incl = tsum;
    for (int s = 1; s < 64; s <<= 1) {
        const int64_t up = __shfl_up(incl, s, 64);
        if (lane >= s) incl += up;
    }
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    int64_t woff = 0;
    for (int k = 0; k < 4; ++k) woff += (k < w) ? wsum[k] : 0;
    int64_t run = woff + incl - tsum;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        run += e[u];
        if (base + u < count) v[base + u] = run;            // inclusive within the block
    }
    if (tid == 255) totals[blockIdx.x] = run;
}

__global__ __launch_bounds__(1024) void scan_totals_kernel(int64_t* __restrict__ totals, int64_t nblk)
{
    __shared__ int64_t wsum[16];
    __shared__ int64_t carry_s;
    const int tid = (int)threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < nblk; base += 1024) {
        const int64_t mine = base + tid < nblk ? totals[base + tid] : 0;
        int64_t incl = mine;
        for (int s = 1; s < 64; s <<= 1) {
            const int64_t up = __shfl_up(incl, s, 64);
            if (lane >= s) incl += up;
        }
        if (lane == 63) wsum[w] = incl;
        __syncthreads();
        int64_t woff = 0, total = 0;
        for (int k = 0; k < 16; ++k) {
            woff += (k < w) ? wsum[k] : 0;
            total += wsum[k];
        }
        const int64_t carry = carry_s;
        if (base + tid < nblk) totals[base + tid] = carry + woff + incl - mine;    // exclusive
        __syncthreads();
        if (tid == 0) carry_s = carry + total;
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void scan_add_kernel(int64_t* __restrict__ v, int64_t count,
                                                       const int64_t* __restrict__ totals)
{
    const int64_t add = totals[blockIdx.x];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock;
    for (int u = (int)threadIdx.x; u < kScanBlock; u += 256)
        if (base + u < count) v[base + u] += add;
}

__global__ void zero_first_kernel(int64_t* p) { *p = 0; }

// ------------------------------------------------------------------------- pass 2
// Which of the two fill kernels builds a row with `hits` members at the largest radius.  The
// bitmap kernel takes the 27 cells once per slab of indices but orders nothing, the other takes
// them once and sorts.  Measured on 120000 points in four slabs: the bitmap kernel is the cheaper
// one from about 128 hits per slab of the cloud; the sort buffer's capacity is the limit in any case.
__device__ __forceinline__ bool is_long_row(int64_t hits, int N, int slab_words)
{
    const int64_t slabs = ((int64_t)N + slab_words * 32 - 1) / (slab_words * 32);
    const int64_t limit = 128 * slabs < kSortCap ? 128 * slabs : kSortCap;
    return hits > limit;
}

// Level cursors: lane l holds how many members of the level-l row are written already.
struct Emit {
    int64_t mybase;      // lane l: start of the level-l row
    int mycur;           // lane l: members written
    float mythr;
    int L;
    int32_t* entries;
    int64_t capacity;
    // j (valid lanes, ascending over the lanes) at squared distance d
    __device__ __forceinline__ void operator()(int j, float d, bool valid, int lane)
    {
        for (int l = 0; l < L; ++l) {
            const float t = rdlane_f(mythr, l);
            const bool hit = valid && d < t;
            const uint64_t mk = __builtin_amdgcn_ballot_w64(hit);
            if (mk == 0) continue;
            const uint32_t blo = rdlane((uint32_t)mybase, l), bhi = rdlane((uint32_t)(mybase >> 32), l);
            const int64_t at = (int64_t)(((uint64_t)bhi << 32) | blo) + (int)rdlane((uint32_t)mycur, l) +
                               lanes_below(mk);
            if (hit && at < capacity) entries[at] = j;
            mycur += lane == l ? __builtin_popcountll(mk) : 0;
        }
    }
};

// ascending bitonic sort of buf[0 .. n2) (n2 a power of two >= 64) by one wave
__device__ __forceinline__ void wave_sort(uint32_t* buf, int n2, int lane)
{
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = lane; t < (n2 >> 1); t += 64) {
                // t-th compare-exchange of this step: lower partner index
                const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const int hi = lo | j;
                const uint32_t a = buf[lo], b = buf[hi];
                const bool up = (lo & k) == 0;
                if ((a > b) == up) {
                    buf[lo] = b;
                    buf[hi] = a;
                }
            }
            // one wave: its LDS operations execute in program order; keep the compiler from
            // moving the next step's reads above these writes
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// Orders buf[0 .. H) (distinct values) ascending: by counting across the lanes when there are
// at most 64, else by the bitonic network.  One wave.
__device__ __forceinline__ void wave_order(uint32_t* buf, int H, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (H <= 64) {
        const uint32_t mine = lane < H ? buf[lane] : 0xFFFFFFFFu;
        int rank = 0;
        for (int t = 0; t < H; ++t) rank += rdlane(mine, t) < mine ? 1 : 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (lane < H) buf[rank] = mine;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        int n2 = 128;
        while (n2 < H) n2 <<= 1;
        for (int t = H + lane; t < n2; t += 64) buf[t] = 0xFFFFFFFFu;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        wave_sort(buf, n2, lane);
    }
}

__global__ __launch_bounds__(kWaves * 64) void excl_fill_kernel(
    const float* __restrict__ xyz, int B, int N, const float* __restrict__ thr2, int L,
    const int64_t* __restrict__ offsets, int32_t* __restrict__ entries, int64_t capacity,
    const ExclGrid* __restrict__ gp, const int32_t* __restrict__ cell_start, const float4* __restrict__ sorted,
    int maxcells, int slab_words)
{
    __shared__ uint32_t sortbuf[kWaves][kSortCap];
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int w = uni((int)threadIdx.x >> 6);
    const int i = uni((int)blockIdx.x * kWaves + w);
    if (i >= N) return;
    const ExclGrid g = gp[b];
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const float px = cloud[(int64_t)i * 3 + 0], py = cloud[(int64_t)i * 3 + 1], pz = cloud[(int64_t)i * 3 + 2];
    Emit em;
    em.L = L;
    em.entries = entries;
    em.capacity = capacity;
    em.mythr = lane < L ? thr2[(int64_t)b * L + lane] : 0.0f;
    em.mybase = lane < L ? offsets[((int64_t)lane * B + b) * N + i] : 0;
    em.mycur = 0;
    const int64_t rmaxrow = ((int64_t)g.lmax * B + b) * N + i;
    const int64_t hits64 = offsets[rmaxrow + 1] - offsets[rmaxrow];
    if (hits64 <= 0) return;                 // rows of smaller radii are empty as well
    if (!is_long_row(hits64, N, slab_words)) {
        const int H = (int)hits64;
        uint32_t* buf = sortbuf[w];
        int cx, cy, cz;
        cell_of(g, px, py, pz, cx, cy, cz);
        int got = 0;
        const float rmax2 = g.rmax2;
        for_neighbours(g, cell_start + (int64_t)b * (maxcells + 1), sorted + (int64_t)b * N, cx, cy, cz, lane,
                       [&](const float4& r, bool valid) {
                           const bool hit = valid && dist2(px, py, pz, r.x, r.y, r.z) < rmax2;
                           const uint64_t mk = __builtin_amdgcn_ballot_w64(hit);
                           const int at = got + lanes_below(mk);
                           if (hit && at < kSortCap) buf[at] = (uint32_t)__float_as_int(r.w);
                           got += __builtin_popcountll(mk);
                           return true;
                       });
        wave_order(buf, H, lane);
        for (int t0 = 0; t0 < H; t0 += 64) {
            const bool valid = t0 + lane < H;
            const int j = valid ? (int)buf[t0 + lane] : i;
            const float d = dist2(px, py, pz, cloud[(int64_t)j * 3 + 0], cloud[(int64_t)j * 3 + 1],
                                  cloud[(int64_t)j * 3 + 2]);
            em(j, d, valid, lane);
        }
    }
    // longer rows: excl_fill_heavy_kernel
}

// one wave: its LDS operations execute in program order; keeps the compiler from moving reads
// above the writes they depend on
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Pass 2 for the rows that excl_fill_kernel leaves out (is_long_row).  One wave per point.  The hits of the 27 cells are marked in a bitmap over a
// slab of slab_words * 32 consecutive indices; the bitmap is then read 64 words a pass (one per
// lane), and the set bits of a pass are handed out 64 at a time in ascending order: lane t finds
// the word that holds the t-th of them through the prefix sums of the words' bit counts, and
// the bit inside the word.  The words are cleared as they are read.  A cloud with more points
// than a slab takes the cells once per slab.
__global__ __launch_bounds__(kHeavyWaves * 64) void excl_fill_heavy_kernel(
    const float* __restrict__ xyz, int B, int N, const float* __restrict__ thr2, int L,
    const int64_t* __restrict__ offsets, int32_t* __restrict__ entries, int64_t capacity,
    const ExclGrid* __restrict__ gp, const int32_t* __restrict__ cell_start, const float4* __restrict__ sorted,
    int maxcells, int slab_words)
{
    extern __shared__ uint32_t bitmap[];            // kHeavyWaves x slab_words
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int w = uni((int)threadIdx.x >> 6);
    const int i = uni((int)blockIdx.x * kHeavyWaves + w);
    if (i >= N) return;
    const ExclGrid g = gp[b];
    const int64_t rmaxrow = ((int64_t)g.lmax * B + b) * N + i;
    if (!is_long_row(offsets[rmaxrow + 1] - offsets[rmaxrow], N, slab_words)) return;
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const float px = cloud[(int64_t)i * 3 + 0], py = cloud[(int64_t)i * 3 + 1], pz = cloud[(int64_t)i * 3 + 2];
    Emit em;
    em.L = L;
    em.entries = entries;
    em.capacity = capacity;
    em.mythr = lane < L ? thr2[(int64_t)b * L + lane] : 0.0f;
    em.mybase = lane < L ? offsets[((int64_t)lane * B + b) * N + i] : 0;
    em.mycur = 0;
    uint32_t* bm = bitmap + w * slab_words;
    for (int t = lane; t < slab_words; t += 64) bm[t] = 0u;
    wave_lds_sync();
    int cx, cy, cz;
    cell_of(g, px, py, pz, cx, cy, cz);
    const float rmax2 = g.rmax2;
    const int slab = slab_words * 32;
    for (int base = 0; base < N; base += slab) {
        const int span = N - base < slab ? N - base : slab;
        for_neighbour_runs(g, cell_start + (int64_t)b * (maxcells + 1), sorted + (int64_t)b * N, cx, cy, cz, lane,
                           [&](const float4& r, bool valid) {
                               const uint32_t rel = (uint32_t)__float_as_int(r.w) - (uint32_t)base;
                               const bool hit = valid && rel < (uint32_t)span &&
                                                dist2(px, py, pz, r.x, r.y, r.z) < rmax2;
                               if (hit) atomicOr(&bm[rel >> 5], 1u << (rel & 31u));
                           });
        wave_lds_sync();
        const int words = (span + 31) >> 5;
        for (int w0 = 0; w0 < words; w0 += 64) {
            const int wi = w0 + lane;
            uint32_t word = wi < words ? bm[wi] : 0u;
            if (__builtin_amdgcn_ballot_w64(word != 0u) == 0) continue;
            if (word != 0u) bm[wi] = 0u;
            const int cnt = __builtin_popcount(word);
            int incl = cnt;                                  // inclusive prefix sum over the lanes
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int o = __shfl_up(incl, (unsigned)d, 64);
                incl += lane >= d ? o : 0;
            }
            const int total = (int)rdlane((uint32_t)incl, 63);          // <= 64 * 32
            const int excl = incl - cnt;                                // set bits in the lanes below
            for (int t0 = 0; t0 < total; t0 += 64) {
                // lane t takes the (t0 + t)-th set bit of the pass: the word of the last lane whose
                // bits start at or before it (the prefix is non-decreasing over the lanes) ...
                const int want = t0 + lane;
                const bool valid = want < total;
                int src = 0;
#pragma unroll
                for (int step = 32; step > 0; step >>= 1) {
                    const int below = __shfl(excl, src + step, 64);     // src + step <= 63
                    src += below <= want ? step : 0;
                }
                uint32_t sw = (uint32_t)__shfl((int)word, src, 64);
                int nth = want - __shfl(excl, src, 64);
                // ... and in it the nth set bit: descend by halves
                int bit = 0;
#pragma unroll
                for (int width = 16; width > 0; width >>= 1) {
                    const int c = __builtin_popcount(sw & ((1u << width) - 1u));
                    const bool up = nth >= c;
                    nth -= up ? c : 0;
                    bit += up ? width : 0;
                    sw = up ? sw >> width : sw;
                }
                const int j = valid ? (int)((uint32_t)base + ((uint32_t)(w0 + src) << 5) + (uint32_t)bit) : i;
                const float d = dist2(px, py, pz, cloud[(int64_t)j * 3 + 0], cloud[(int64_t)j * 3 + 1],
                                      cloud[(int64_t)j * 3 + 2]);
                em(j, d, valid, lane);
            }
        }
    }
}

// Ball query over the uniform grid: the result of the brute-force scan (first k hits by
// ascending index, strict < on squared binary32 distances, unused slots repeat the first hit)
// from the 27 cells around the centre.  One wave per centre walks the cells and keeps the k lowest
// indices among the hits (in keep, ascending): once it has k of them the largest is a bound, and
// only hits with an index below it are collected; when the collection fills, and at the end, the
// k lowest of kept and collected values are taken one at a time (a point is in the ball once, so
// the values differ).  A ball of any size is answered from its 27 cells.
constexpr int kGridBatch = 256;        // hits collected between two selections of the k lowest

__global__ __launch_bounds__(kWaves * 64) void bq_grid_kernel(
    const float* __restrict__ xyz, int N, const int32_t* __restrict__ center_idx, int M, float r2, int k,
    int32_t* __restrict__ out_idx, int32_t* __restrict__ out_cnt, const ExclGrid* __restrict__ gp,
    const int32_t* __restrict__ cell_start, const float4* __restrict__ sorted, int maxcells)
{
    __shared__ int32_t keepbuf[kWaves][256];
    __shared__ int32_t hitbuf[kWaves][kGridBatch];
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int w = uni((int)threadIdx.x >> 6);
    const int q = uni((int)blockIdx.x * kWaves + w);
    if (q >= M) return;
    const int c = uni(center_idx[(int64_t)b * M + q]);
    int32_t* row = out_idx + ((int64_t)b * M + q) * k;
    if (c < 0 || c >= N) {
        for (int t = lane; t < k; t += 64) row[t] = -1;
        if (lane == 0 && out_cnt) out_cnt[(int64_t)b * M + q] = 0;
        return;
    }
    const ExclGrid g = gp[b];
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const float px = cloud[(int64_t)c * 3 + 0], py = cloud[(int64_t)c * 3 + 1], pz = cloud[(int64_t)c * 3 + 2];
    int32_t* keep = keepbuf[w];
    int32_t* hits = hitbuf[w];
    int cx, cy, cz;
    cell_of(g, px, py, pz, cx, cy, cz);
    int kept = 0, fresh = 0;
    int32_t bound = 0x7FFFFFFF;
    auto take_lowest = [&]() {
        // the same wave reads back what it wrote: the LDS keeps a wave's operations in order
        int32_t v[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] = lane + 64 * i < kept ? keep[lane + 64 * i] : 0x7FFFFFFF;
            v[4 + i] = lane + 64 * i < fresh ? hits[lane + 64 * i] : 0x7FFFFFFF;
        }
        const int want = kept + fresh < k ? kept + fresh : k;
        int32_t mn = 0x7FFFFFFF;
        for (int t = 0; t < want; ++t) {
            mn = v[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) mn = min(mn, v[i]);
#pragma unroll
            for (int sft = 32; sft > 0; sft >>= 1) mn = min(mn, __shfl_xor(mn, sft, 64));
            mn = uni(mn);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = v[i] == mn ? 0x7FFFFFFF : v[i];
            if (lane == 0) keep[t] = mn;
        }
        kept = want;
        fresh = 0;
        bound = kept == k ? mn : 0x7FFFFFFF;
    };
    for_neighbours(g, cell_start + (int64_t)b * (maxcells + 1), sorted + (int64_t)b * N, cx, cy, cz, lane,
                   [&](const float4& r, bool valid) {
                       const int32_t j = __float_as_int(r.w);
                       const bool hit = valid && dist2(px, py, pz, r.x, r.y, r.z) < r2 && j < bound;
                       const uint64_t mk = __builtin_amdgcn_ballot_w64(hit);
                       if (mk != 0) {
                           if (hit) hits[fresh + lanes_below(mk)] = j;
                           fresh += __builtin_popcountll(mk);
                           if (fresh > kGridBatch - 64) take_lowest();
                       }
                       return true;
                   });
    if (fresh > 0) take_lowest();
    const int first = kept > 0 ? keep[0] : -1;
    for (int t = lane; t < k; t += 64) row[t] = t < kept ? keep[t] : first;
    if (lane == 0 && out_cnt) out_cnt[(int64_t)b * M + q] = kept;
}

// k nearest samples through a grid over the SAMPLES (records carry the sample's position in the
// list): one thread per point visits the samples of the 27 cells around it and keeps the K
// nearest, ordered by (distance, position).  Every sample outside those cells is farther than the
// cell width, which exceeds the search radius: when the K-th nearest found is closer than the
// radius the result is exact.  The other points go to the cloud's list of deferred points, which
// the brute-force kernels search afterwards.
template <int K>
__global__ __launch_bounds__(256) void knn_grid_kernel(const float* __restrict__ xyz, int N, int k, float r2,
                                                       int32_t* __restrict__ out_pos, float* __restrict__ out_d2,
                                                       const ExclGrid* __restrict__ gp,
                                                       const int32_t* __restrict__ cell_start,
                                                       const float4* __restrict__ sorted, int n, int maxcells,
                                                       int32_t* __restrict__ count, int32_t* __restrict__ list)
{
    const int b = (int)blockIdx.y;
    const int j = (int)(blockIdx.x * 256 + threadIdx.x);
    if (j >= N) return;
    const ExclGrid g = gp[b];
    const float* p = xyz + ((int64_t)b * N + j) * 3;
    const float px = p[0], py = p[1], pz = p[2];
    int cx, cy, cz;
    cell_of(g, px, py, pz, cx, cy, cz);
    float bd[K];
    int32_t bq[K];
#pragma unroll
    for (int i = 0; i < K; ++i) {
        bd[i] = __builtin_inff();
        bq[i] = -1;
    }
    const int32_t* __restrict__ st = cell_start + (int64_t)b * (maxcells + 1);
    const float4* __restrict__ rec = sorted + (int64_t)b * n;
    const int x0 = cx > 0 ? cx - 1 : 0;
    const int x1 = cx < g.dim[0] - 1 ? cx + 1 : g.dim[0] - 1;
    for (int dz = -1; dz <= 1; ++dz) {
        const int z = cz + dz;
        if (z < 0 || z >= g.dim[2]) continue;
        for (int dy = -1; dy <= 1; ++dy) {
            const int y = cy + dy;
            if (y < 0 || y >= g.dim[1]) continue;
            const int c0 = (z * g.dim[1] + y) * g.dim[0] + x0;
            const int end = st[c0 + (x1 - x0) + 1];
            for (int t = st[c0]; t < end; ++t) {
                const float4 s = rec[t];
                const float dd = dist2(px, py, pz, s.x, s.y, s.z);
                const int32_t qq = __float_as_int(s.w);
                if (!(dd < bd[K - 1] || (dd == bd[K - 1] && qq < bq[K - 1]))) continue;    // NaN: never
#pragma unroll
                for (int i = K - 1; i >= 1; --i) {
                    const bool before = dd < bd[i - 1] || (dd == bd[i - 1] && qq < bq[i - 1]);
                    const bool here = dd < bd[i] || (dd == bd[i] && qq < bq[i]);
                    bd[i] = before ? bd[i - 1] : (here ? dd : bd[i]);
                    bq[i] = before ? bq[i - 1] : (here ? qq : bq[i]);
                }
                const bool first = dd < bd[0] || (dd == bd[0] && qq < bq[0]);
                bd[0] = first ? dd : bd[0];
                bq[0] = first ? qq : bq[0];
            }
        }
    }
    float kth = __builtin_inff();
    int32_t kq = -1;
#pragma unroll
    for (int i = 0; i < K; ++i)
        if (i == k - 1) {
            kth = bd[i];
            kq = bq[i];
        }
    if (kq >= 0 && kth < r2) {
        int32_t* pos = out_pos + ((int64_t)b * N + j) * k;
        float* d2 = out_d2 + ((int64_t)b * N + j) * k;
#pragma unroll
        for (int i = 0; i < K; ++i)
            if (i < k) {
                pos[i] = bq[i];
                d2[i] = bd[i];
            }
    } else {
        const int at = atomicAdd(&count[b], 1);
        list[(int64_t)b * N + at] = j;
    }
}

__global__ void zero_ints_kernel(int32_t* p, int n)
{
    const int t = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (t < n) p[t] = 0;
}

// Ball query by lookup: one wave per centre.
__global__ __launch_bounds__(256) void bq_lists_kernel(const int64_t* __restrict__ offsets,
                                                       const int32_t* __restrict__ entries, int B, int N, int level,
                                                       const int32_t* __restrict__ center_idx, int M, int k,
                                                       int32_t* __restrict__ out_idx, int32_t* __restrict__ out_cnt)
{
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int q = uni((int)blockIdx.x * 4 + ((int)threadIdx.x >> 6));
    if (q >= M) return;
    const int c = uni(center_idx[(int64_t)b * M + q]);
    int32_t* row = out_idx + ((int64_t)b * M + q) * k;
    int cnt = 0;
    int64_t begin = 0;
    if (c >= 0 && c < N) {
        const int64_t r = ((int64_t)level * B + b) * N + c;
        begin = offsets[r];
        const int64_t len = offsets[r + 1] - begin;
        cnt = len < k ? (int)len : k;
    }
    const int first = cnt > 0 ? entries[begin] : -1;
    for (int t = lane; t < k; t += 64) row[t] = t < cnt ? entries[begin + t] : first;
    if (lane == 0 && out_cnt) out_cnt[(int64_t)b * M + q] = cnt;
}

}  // namespace

ExclLayout excl_layout(int B, int N, int L)
{
    ExclLayout lay;
    int64_t mc = N;
    if (mc < 64) mc = 64;
    if (mc > ((int64_t)1 << 21)) mc = (int64_t)1 << 21;
    lay.maxcells = (int)mc;
    auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
    int64_t at = 0;
    lay.grid_off = at;
    at += up((int64_t)B * (int64_t)sizeof(ExclGrid));
    lay.cnt_off = at;
    at += up((int64_t)B * mc * 4);
    lay.start_off = at;
    at += up((int64_t)B * (mc + 1) * 4);
    lay.sorted_off = at;
    at += up((int64_t)B * N * 16);
    lay.totals_off = at;
    const int64_t rows = (int64_t)L * B * N;
    at += up(((rows + kScanBlock - 1) / kScanBlock + 1) * 8);
    lay.tiles_off = at;              // sums of the cell counts per tile of kCellTile cells (the scan over the cells)
    at += up((int64_t)B * ((mc + kCellTile - 1) / kCellTile) * 4);
    lay.bytes = at;
    return lay;
}

static int sort_bits(int maxcells)
{
    int bits = 1;
    while (bits < 7 && ((int64_t)1 << (3 * (bits + 1))) <= maxcells) ++bits;
    return bits;
}

int64_t spatial_sort_bytes(int B, int N) { return excl_layout(B, N, 1).bytes; }

const float4* spatial_sorted(int B, int N, const void* workspace)
{
    return reinterpret_cast<const float4*>(reinterpret_cast<const unsigned char*>(workspace) +
                                           excl_layout(B, N, 1).sorted_off);
}

hipError_t launch_spatial_sort(const float* xyz, int B, int N, void* workspace, hipStream_t stream)
{
    const ExclLayout lay = excl_layout(B, N, 1);
    unsigned char* base = reinterpret_cast<unsigned char*>(workspace);
    ExclGrid* gp = reinterpret_cast<ExclGrid*>(base + lay.grid_off);
    int32_t* cnt = reinterpret_cast<int32_t*>(base + lay.cnt_off);
    int32_t* st = reinterpret_cast<int32_t*>(base + lay.start_off);
    float4* sorted = reinterpret_cast<float4*>(base + lay.sorted_off);
    const int64_t ncnt = (int64_t)B * lay.maxcells;
    int initblocks = (int)((ncnt + 255) / 256);
    if (initblocks > 2048) initblocks = 2048;
    hipLaunchKernelGGL(grid_init_kernel, dim3(initblocks), dim3(256), 0, stream, gp, B, cnt, ncnt);
    int bblocks = (N + 2047) / 2048;
    if (bblocks > 64) bblocks = 64;
    hipLaunchKernelGGL(grid_bounds_kernel, dim3(bblocks, B), dim3(256), 0, stream, xyz, N, gp);
    hipLaunchKernelGGL(sort_setup_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, gp, B, sort_bits(lay.maxcells));
    const dim3 pgrid((unsigned)((N + 255) / 256), (unsigned)B);
    hipLaunchKernelGGL(grid_count_kernel, pgrid, dim3(256), 0, stream, xyz, N, gp, cnt, lay.maxcells);
    launch_cell_scan(gp, cnt, st, reinterpret_cast<int32_t*>(base + lay.tiles_off), B, lay.maxcells, stream);
    hipLaunchKernelGGL(grid_scatter_kernel, pgrid, dim3(256), 0, stream, xyz, N, gp, cnt, sorted, lay.maxcells);
    return hipGetLastError();
}

hipError_t launch_excl_count(const float* xyz, int B, int N, const float* thr2, int L, int64_t* offsets,
                             void* workspace, hipStream_t stream)
{
    const ExclLayout lay = excl_layout(B, N, L);
    unsigned char* base = reinterpret_cast<unsigned char*>(workspace);
    ExclGrid* gp = reinterpret_cast<ExclGrid*>(base + lay.grid_off);
    int32_t* cnt = reinterpret_cast<int32_t*>(base + lay.cnt_off);
    int32_t* st = reinterpret_cast<int32_t*>(base + lay.start_off);
    float4* sorted = reinterpret_cast<float4*>(base + lay.sorted_off);
    int64_t* totals = reinterpret_cast<int64_t*>(base + lay.totals_off);
    const int64_t ncnt = (int64_t)B * lay.maxcells;
    int initblocks = (int)((ncnt + 255) / 256);
    if (initblocks > 2048) initblocks = 2048;
    hipLaunchKernelGGL(grid_init_kernel, dim3(initblocks), dim3(256), 0, stream, gp, B, cnt, ncnt);
    int bblocks = (N + 2047) / 2048;
    if (bblocks > 64) bblocks = 64;
    hipLaunchKernelGGL(grid_bounds_kernel, dim3(bblocks, B), dim3(256), 0, stream, xyz, N, gp);
    hipLaunchKernelGGL(grid_setup_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, gp, B, thr2, L, lay.maxcells,
                       0.0f);
    const dim3 pgrid((unsigned)((N + 255) / 256), (unsigned)B);
    hipLaunchKernelGGL(grid_count_kernel, pgrid, dim3(256), 0, stream, xyz, N, gp, cnt, lay.maxcells);
    launch_cell_scan(gp, cnt, st, reinterpret_cast<int32_t*>(base + lay.tiles_off), B, lay.maxcells, stream);
    hipLaunchKernelGGL(grid_scatter_kernel, pgrid, dim3(256), 0, stream, xyz, N, gp, cnt, sorted, lay.maxcells);
    const dim3 wgrid((unsigned)((N + kWaves - 1) / kWaves), (unsigned)B);
    hipLaunchKernelGGL(excl_count_kernel, wgrid, dim3(kWaves * 64), 0, stream, xyz, B, N, thr2, L, offsets, gp, st,
                       sorted, lay.maxcells);
    const int64_t rows = (int64_t)L * B * N;
    const int64_t nblk = (rows + kScanBlock - 1) / kScanBlock;
    hipLaunchKernelGGL(zero_first_kernel, dim3(1), dim3(1), 0, stream, offsets);
    hipLaunchKernelGGL(scan_blocks_kernel, dim3((unsigned)nblk), dim3(256), 0, stream, offsets + 1, rows, totals);
    hipLaunchKernelGGL(scan_totals_kernel, dim3(1), dim3(1024), 0, stream, totals, nblk);
    hipLaunchKernelGGL(scan_add_kernel, dim3((unsigned)nblk), dim3(256), 0, stream, offsets + 1, rows, totals);
    return hipGetLastError();
}

hipError_t launch_excl_fill(const float* xyz, int B, int N, const float* thr2, int L, const int64_t* offsets,
                            int32_t* entries, int64_t capacity, void* workspace, hipStream_t stream)
{
    const ExclLayout lay = excl_layout(B, N, L);
    unsigned char* base = reinterpret_cast<unsigned char*>(workspace);
    const ExclGrid* gp = reinterpret_cast<const ExclGrid*>(base + lay.grid_off);
    const int32_t* st = reinterpret_cast<const int32_t*>(base + lay.start_off);
    const float4* sorted = reinterpret_cast<const float4*>(base + lay.sorted_off);
    const dim3 wgrid((unsigned)((N + kWaves - 1) / kWaves), (unsigned)B);
    // index slab of the bitmap kernel: a smaller bitmap lets more waves run on a compute unit, a
    // larger one takes the cells fewer times (measured on 120000 points: 32768 indices, four
    // walks, ahead of 65536 and two)
    const int slab_words = N <= 4 * 32768 ? kSlabWordsMax / 2 : kSlabWordsMax;
    hipLaunchKernelGGL(excl_fill_kernel, wgrid, dim3(kWaves * 64), 0, stream, xyz, B, N, thr2, L, offsets, entries,
                       capacity, gp, st, sorted, lay.maxcells, slab_words);
    // the rows that kernel leaves out (its waves return at once for all others)
    const dim3 hgrid((unsigned)((N + kHeavyWaves - 1) / kHeavyWaves), (unsigned)B);
    hipLaunchKernelGGL(excl_fill_heavy_kernel, hgrid, dim3(kHeavyWaves * 64),
                       (size_t)kHeavyWaves * slab_words * sizeof(uint32_t), stream, xyz, B, N, thr2, L, offsets,
                       entries, capacity, gp, st, sorted, lay.maxcells, slab_words);
    return hipGetLastError();
}

// Grid over the samples (their coordinates gathered to sample_xyz [B][n][3]) and the search of
// every point in it; the deferred points are left in `list` / `count` for the caller.
hipError_t launch_knn_grid(const float* xyz, int B, int N, const float* sample_xyz, int n, int k, float r2,
                           int32_t* out_pos, float* out_d2, int32_t* count, int32_t* list, void* grid_ws,
                           hipStream_t stream)
{
    const ExclLayout lay = excl_layout(B, n, 1);
    unsigned char* base = reinterpret_cast<unsigned char*>(grid_ws);
    ExclGrid* gp = reinterpret_cast<ExclGrid*>(base + lay.grid_off);
    int32_t* cnt = reinterpret_cast<int32_t*>(base + lay.cnt_off);
    int32_t* st = reinterpret_cast<int32_t*>(base + lay.start_off);
    float4* sorted = reinterpret_cast<float4*>(base + lay.sorted_off);
    const int64_t ncnt = (int64_t)B * lay.maxcells;
    int initblocks = (int)((ncnt + 255) / 256);
    if (initblocks > 2048) initblocks = 2048;
    hipLaunchKernelGGL(zero_ints_kernel, dim3((B + 255) / 256), dim3(256), 0, stream, count, B);
    hipLaunchKernelGGL(grid_init_kernel, dim3(initblocks), dim3(256), 0, stream, gp, B, cnt, ncnt);
    int bblocks = (n + 2047) / 2048;
    if (bblocks > 64) bblocks = 64;
    hipLaunchKernelGGL(grid_bounds_kernel, dim3(bblocks, B), dim3(256), 0, stream, sample_xyz, n, gp);
    hipLaunchKernelGGL(grid_setup_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, gp, B,
                       static_cast<const float*>(nullptr), 1, lay.maxcells, r2);
    const dim3 sgrid((unsigned)((n + 255) / 256), (unsigned)B);
    hipLaunchKernelGGL(grid_count_kernel, sgrid, dim3(256), 0, stream, sample_xyz, n, gp, cnt, lay.maxcells);
    launch_cell_scan(gp, cnt, st, reinterpret_cast<int32_t*>(base + lay.tiles_off), B, lay.maxcells, stream);
    hipLaunchKernelGGL(grid_scatter_kernel, sgrid, dim3(256), 0, stream, sample_xyz, n, gp, cnt, sorted, lay.maxcells);
    const dim3 pgrid((unsigned)((N + 255) / 256), (unsigned)B);
    if (k == 1)
        hipLaunchKernelGGL(knn_grid_kernel<1>, pgrid, dim3(256), 0, stream, xyz, N, k, r2, out_pos, out_d2, gp, st,
                           sorted, n, lay.maxcells, count, list);
    else if (k <= 3)
        hipLaunchKernelGGL(knn_grid_kernel<3>, pgrid, dim3(256), 0, stream, xyz, N, k, r2, out_pos, out_d2, gp, st,
                           sorted, n, lay.maxcells, count, list);
    else
        hipLaunchKernelGGL(knn_grid_kernel<8>, pgrid, dim3(256), 0, stream, xyz, N, k, r2, out_pos, out_d2, gp, st,
                           sorted, n, lay.maxcells, count, list);
    return hipGetLastError();
}

hipError_t launch_bq_grid(const float* xyz, int B, int N, const int32_t* center_idx, int M, float r2, int k,
                          int32_t* out_idx, int32_t* out_cnt, void* workspace, hipStream_t stream)
{
    if (M == 0) return hipSuccess;
    const ExclLayout lay = excl_layout(B, N, 1);
    unsigned char* base = reinterpret_cast<unsigned char*>(workspace);
    ExclGrid* gp = reinterpret_cast<ExclGrid*>(base + lay.grid_off);
    int32_t* cnt = reinterpret_cast<int32_t*>(base + lay.cnt_off);
    int32_t* st = reinterpret_cast<int32_t*>(base + lay.start_off);
    float4* sorted = reinterpret_cast<float4*>(base + lay.sorted_off);
    const int64_t ncnt = (int64_t)B * lay.maxcells;
    int initblocks = (int)((ncnt + 255) / 256);
    if (initblocks > 2048) initblocks = 2048;
    hipLaunchKernelGGL(grid_init_kernel, dim3(initblocks), dim3(256), 0, stream, gp, B, cnt, ncnt);
    int bblocks = (N + 2047) / 2048;
    if (bblocks > 64) bblocks = 64;
    hipLaunchKernelGGL(grid_bounds_kernel, dim3(bblocks, B), dim3(256), 0, stream, xyz, N, gp);
    hipLaunchKernelGGL(grid_setup_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, gp, B,
                       static_cast<const float*>(nullptr), 1, lay.maxcells, r2);
    const dim3 pgrid((unsigned)((N + 255) / 256), (unsigned)B);
    hipLaunchKernelGGL(grid_count_kernel, pgrid, dim3(256), 0, stream, xyz, N, gp, cnt, lay.maxcells);
    launch_cell_scan(gp, cnt, st, reinterpret_cast<int32_t*>(base + lay.tiles_off), B, lay.maxcells, stream);
    hipLaunchKernelGGL(grid_scatter_kernel, pgrid, dim3(256), 0, stream, xyz, N, gp, cnt, sorted, lay.maxcells);
    hipLaunchKernelGGL(bq_grid_kernel, dim3((unsigned)((M + kWaves - 1) / kWaves), (unsigned)B), dim3(kWaves * 64), 0,
                       stream, xyz, N, center_idx, M, r2, k, out_idx, out_cnt, gp, st, sorted, lay.maxcells);
    return hipGetLastError();
}

hipError_t launch_bq_lists(const int64_t* offsets, const int32_t* entries, int B, int N, int level,
                           const int32_t* center_idx, int M, int k, int32_t* out_idx, int32_t* out_cnt,
                           hipStream_t stream)
{
    if (M == 0) return hipSuccess;
    hipLaunchKernelGGL(bq_lists_kernel, dim3((unsigned)((M + 3) / 4), (unsigned)B), dim3(256), 0, stream, offsets,
                       entries, B, N, level, center_idx, M, k, out_idx, out_cnt);
    return hipGetLastError();
}

}  // namespace fastpoint
