// k nearest samples of every point (the k-NN of the up-sampling step, Section 3.1 of
// FastPoint, arXiv 2507.23480) for gfx950, by brute force and in the redundancy-free form of
// Section 4.2.
//
// Result for point j: the k samples with the smallest squared binary32 distance, nearest first,
// the lower sample position first among equal distances.  Every kernel feeds the samples to a
// point in ascending position and replaces an entry only on a strictly smaller distance, which
// is that order.
//
//   * brute force: a workgroup owns 512 points (two per thread, in registers); the samples are
//     gathered 256 at a time into LDS and read back at a wave-uniform address (one broadcast
//     read feeds 128 distance evaluations of a wave);
//   * redundancy-free: the sampler recorded, for every sample, which points are closer than
//     the cache radius (the exclusion list at an extra radius of Section 4.2).  Read per
//     point this is the list of samples near it: only those distances are evaluated.  When a point has at least k samples inside the radius they are its k nearest
//     (every other sample is farther than all of them); the remaining points are collected in a
//     list and searched by brute force afterwards (a wave per point while the list is short).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

#pragma clang fp contract(off)

namespace fastpoint {
namespace {

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

__device__ __forceinline__ float rdlane_f(float v, int l)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), l));
}

__device__ __forceinline__ uint64_t rdlane_u64(uint64_t v, int l)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

// The K nearest samples seen so far, ascending.  insert() must be called with ascending
// positions: an equal distance never displaces an earlier entry.
template <int K>
struct Nearest {
    float d[K];
    int32_t q[K];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int i = 0; i < K; ++i) {
            d[i] = __builtin_inff();
            q[i] = -1;
        }
    }
    __device__ __forceinline__ void insert(float dd, int32_t qq)
    {
#pragma unroll
        for (int i = K - 1; i >= 1; --i) {
            const bool before = dd < d[i - 1];      // belongs ahead of entry i-1, which moves down
            const bool here = dd < d[i];
            d[i] = before ? d[i - 1] : (here ? dd : d[i]);
            q[i] = before ? q[i - 1] : (here ? qq : q[i]);
        }
        const bool first = dd < d[0];
        d[0] = first ? dd : d[0];
        q[0] = first ? qq : q[0];
    }
    // the same for samples that arrive in any order: among equal distances the lower position
    // goes first (a sample must be offered once only)
    __device__ __forceinline__ void insert_any(float dd, int32_t qq)
    {
#pragma unroll
        for (int i = K - 1; i >= 1; --i) {
            const bool before = dd < d[i - 1] || (dd == d[i - 1] && (uint32_t)qq < (uint32_t)q[i - 1]);
            const bool here = dd < d[i] || (dd == d[i] && (uint32_t)qq < (uint32_t)q[i]);
            d[i] = before ? d[i - 1] : (here ? dd : d[i]);
            q[i] = before ? q[i - 1] : (here ? qq : q[i]);
        }
        const bool first = dd < d[0] || (dd == d[0] && (uint32_t)qq < (uint32_t)q[0]);
        d[0] = first ? dd : d[0];
        q[0] = first ? qq : q[0];
    }
    __device__ __forceinline__ void pop()            // drops the nearest entry
    {
#pragma unroll
        for (int i = 0; i + 1 < K; ++i) {
            d[i] = d[i + 1];
            q[i] = q[i + 1];
        }
        d[K - 1] = __builtin_inff();
        q[K - 1] = -1;
    }
    __device__ __forceinline__ void store(int k, int32_t* pos, float* d2) const
    {
#pragma unroll
        for (int i = 0; i < K; ++i)
            if (i < k) {
                pos[i] = q[i];
                d2[i] = d[i];
            }
    }
};

// one sample against the two points of a thread; `s` comes from a wave-uniform LDS address
// (a broadcast read)
template <int K, bool EARLY>
__device__ __forceinline__ void visit_sample(Nearest<K> (&nb)[2], const float (&px)[2], const float (&py)[2],
                                             const float (&pz)[2], const float4 s, int q)
{
    if constexpr (!EARLY) {
        // the first samples: most of them enter some lane's list
        const float d0 = dist2(px[0], py[0], pz[0], s.x, s.y, s.z);
        const float d1 = dist2(px[1], py[1], pz[1], s.x, s.y, s.z);
        if (__builtin_amdgcn_ballot_w64(d0 < nb[0].d[K - 1] || d1 < nb[1].d[K - 1]) != 0) {
            nb[0].insert(d0, q);
            nb[1].insert(d1, q);
        }
        return;
    }
    // After the first samples a wave rarely has a lane whose list changes, and that is mostly known
    // after two of dist2's three terms: its sum (dx dx + dy dy) + dz dz only grows term by term (every
    // term is >= 0, rounding is monotone), so a sample whose first two terms already reach the K-th
    // distance kept by every lane cannot enter a list.  The third term is added in dist2's order, so
    // a distance that is formed has the same bits.
    const float ax = px[0] - s.x, ay = py[0] - s.y;
    const float bx = px[1] - s.x, by = py[1] - s.y;
    float d0 = ax * ax;
    d0 = d0 + ay * ay;
    float d1 = bx * bx;
    d1 = d1 + by * by;
    if (__builtin_amdgcn_ballot_w64(d0 < nb[0].d[K - 1] || d1 < nb[1].d[K - 1]) != 0) {
        const float az = pz[0] - s.z, bz = pz[1] - s.z;
        d0 = d0 + az * az;
        d1 = d1 + bz * bz;
        if (__builtin_amdgcn_ballot_w64(d0 < nb[0].d[K - 1] || d1 < nb[1].d[K - 1]) != 0) {
            nb[0].insert(d0, q);
            nb[1].insert(d1, q);
        }
    }
}

constexpr int kTile = 256;          // samples staged in LDS per pass
constexpr int kFullTests = 1024;    // samples at the head of the list whose distances are formed in full at once
constexpr int kPointsPerWg = 512;   // two points per thread
constexpr int kWaveListMax = 4096;  // deferred points per cloud up to which each gets a whole wave

// Brute force over all n samples.  LIST = false: the workgroup takes points
// [blockIdx.x*512, +512) of cloud blockIdx.y.  LIST = true: it takes that range of the cloud's
// list of deferred points (list[b][0 .. count[b])) and leaves at once when the range is empty.
template <int K, bool LIST>
__global__ __launch_bounds__(256) void knn_brute_kernel(const float* __restrict__ xyz, int N,
                                                        const int32_t* __restrict__ sample_idx, int n, int k,
                                                        int32_t* __restrict__ out_pos,
                                                        float* __restrict__ out_d2,
                                                        const int32_t* __restrict__ list,
                                                        const int32_t* __restrict__ count,
                                                        int32_t* __restrict__ out_deferred)
{
    __shared__ float4 smp[kTile];
    const int b = (int)blockIdx.y;
    const int tid = (int)threadIdx.x;
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int32_t* __restrict__ sidx = sample_idx + (int64_t)b * n;
    int total = N;
    if (LIST) {
        total = count[b];
        if (blockIdx.x == 0 && tid == 0 && out_deferred) out_deferred[b] = total;
        if (total <= kWaveListMax) return;           // short lists are searched a wave per point
    }
    const int e0 = (int)blockIdx.x * kPointsPerWg;
    if (e0 >= total) return;                         // same for the whole workgroup

    int j[2];
    float px[2], py[2], pz[2];
    Nearest<K> nb[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int e = e0 + u * 256 + tid;
        j[u] = -1;
        if (e < total) j[u] = LIST ? list[(int64_t)b * N + e] : e;
        // a slot without a point compares false against everything
        px[u] = py[u] = pz[u] = __builtin_nanf("");
        if (j[u] >= 0 && j[u] < N) {
            px[u] = cloud[(int64_t)j[u] * 3 + 0];
            py[u] = cloud[(int64_t)j[u] * 3 + 1];
            pz[u] = cloud[(int64_t)j[u] * 3 + 2];
        }
        nb[u].clear();
    }

    for (int q0 = 0; q0 < n; q0 += kTile) {
        __syncthreads();
        {
            const int q = q0 + tid;
            float4 s;
            s.x = s.y = s.z = s.w = __builtin_nanf("");      // no such sample: never nearer
            if (q < n) {
                const int si = sidx[q];
                if (si >= 0 && si < N) {
                    s.x = cloud[(int64_t)si * 3 + 0];
                    s.y = cloud[(int64_t)si * 3 + 1];
                    s.z = cloud[(int64_t)si * 3 + 2];
                }
            }
            smp[tid] = s;
        }
        __syncthreads();
        const int cnt = n - q0 < kTile ? n - q0 : kTile;
        if (q0 < kFullTests) {                          // (uniform)
            if (cnt == kTile) {
#pragma unroll 4
                for (int t = 0; t < kTile; ++t) visit_sample<K, false>(nb, px, py, pz, smp[t], q0 + t);
            } else {
#pragma unroll 1
                for (int t = 0; t < cnt; ++t) visit_sample<K, false>(nb, px, py, pz, smp[t], q0 + t);
            }
        } else if (cnt == kTile) {
#pragma unroll 4
            for (int t = 0; t < kTile; ++t) visit_sample<K, true>(nb, px, py, pz, smp[t], q0 + t);
        } else {
#pragma unroll 1
            for (int t = 0; t < cnt; ++t) visit_sample<K, true>(nb, px, py, pz, smp[t], q0 + t);
        }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (j[u] >= 0 && j[u] < N) {
            const int64_t o = ((int64_t)b * N + j[u]) * k;
            nb[u].store(k, out_pos + o, out_d2 + o);
        }
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v = min(v, (uint32_t)__shfl_xor((int)v, s, 64));
    return v;
}

// Brute force for a short list of deferred points: one wave per point, the samples dealt out to
// the lanes (lane l takes positions l, l+64, ...), then the 64 sorted lists are merged by taking
// k times the smallest head (lower position among equal distances).  A point searched by one
// thread would walk all n samples alone, which takes far longer than the cached search it
// follows.
template <int K>
__global__ __launch_bounds__(256) void knn_list_wave_kernel(const float* __restrict__ xyz, int N,
                                                            const int32_t* __restrict__ sample_idx, int n, int k,
                                                            int32_t* __restrict__ out_pos,
                                                            float* __restrict__ out_d2,
                                                            const int32_t* __restrict__ list,
                                                            const int32_t* __restrict__ count)
{
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int total = count[b];
    const int e = (int)blockIdx.x * 4 + wave;
    if (total > kWaveListMax || e >= total) return;  // wave-uniform; the kernel has no barrier
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int32_t* __restrict__ sidx = sample_idx + (int64_t)b * n;
    const int j = __builtin_amdgcn_readfirstlane(list[(int64_t)b * N + e]);
    const float px = cloud[(int64_t)j * 3 + 0], py = cloud[(int64_t)j * 3 + 1], pz = cloud[(int64_t)j * 3 + 2];
    Nearest<K> nb;
    nb.clear();
    for (int q = lane; q < n; q += 64) {
        const int si = sidx[q];
        float d = __builtin_nanf("");                // no such sample: never nearer
        if (si >= 0 && si < N)
            d = dist2(px, py, pz, cloud[(int64_t)si * 3 + 0], cloud[(int64_t)si * 3 + 1],
                      cloud[(int64_t)si * 3 + 2]);
        nb.insert(d, q);
    }
    const int64_t o = ((int64_t)b * N + j) * k;
    for (int t = 0; t < k; ++t) {
        // distances are >= +0 or +inf: the unsigned order of the bit patterns is their order
        const uint32_t head = __float_as_uint(nb.d[0]);
        const uint32_t dmin = wave_min_u32(head);
        const uint32_t qmin = wave_min_u32(head == dmin ? (uint32_t)nb.q[0] : 0xFFFFFFFFu);
        if (head == dmin && (uint32_t)nb.q[0] == qmin) nb.pop();
        if (lane == 0) {
            out_pos[o + t] = (int32_t)qmin;          // 0xFFFFFFFF = -1: fewer than k valid samples
            out_d2[o + t] = __uint_as_float(dmin);
        }
    }
}

// flags[b] = 1 when the cache was recorded for exactly this sample list of cloud b;
// also empties the cloud's list of deferred points.
__global__ __launch_bounds__(256) void knn_check_kernel(const int32_t* __restrict__ sample_idx, int B, int N,
                                                        int n, const unsigned char* __restrict__ cache,
                                                        int32_t* __restrict__ flags,
                                                        int32_t* __restrict__ count, int64_t rows_cap)
{
    const int b = (int)blockIdx.x;
    const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
    // (a record whose blocks are positions of the sampler's cell order is not searched here: every
    // point of such a cloud goes to the brute-force pass)
    bool ok = h->magic == kBqMagic && h->valid == 1 && h->order == 0 && h->B == B && h->N == N && h->n == n;
    // a list that overflowed has lost entries: a point could miss a sample that is near it
    // (nor can one be used that does not fit the rows of the workspace)
    if (ok) {
        const int64_t chunks = (int64_t) reinterpret_cast<const uint32_t*>(cache + h->cursor_offset)[b];
        const int64_t most = h->cap / kBqChunk;
        ok = reinterpret_cast<const uint32_t*>(cache + h->ovf_offset)[b] == 0 &&
             (chunks < most ? chunks : most) * kBqChunk <= rows_cap;
    }
    int bad = 0;
    if (ok) {
        const int32_t* cidx = reinterpret_cast<const int32_t*>(cache + h->idx_offset);
        for (int q = (int)threadIdx.x; q < n; q += 256)
            bad |= cidx[(int64_t)b * n + q] != sample_idx[(int64_t)b * n + q];
    }
    const int anybad = __syncthreads_or(bad);
    if (threadIdx.x == 0) {
        flags[b] = (ok && !anybad) ? 1 : 0;
        count[b] = 0;
    }
}

// Redundancy-free search.  A wave owns one block of 64 points (lane l holds point 64*w + l).
// The entries of the cache, regrouped by point block, name the samples whose ball holds at least
// one of the 64 points, with the 64 tests: the wave takes its block's entries 64 at a time (one per
// lane, with the sample's coordinates), broadcasts them one after the other, and the lanes whose
// bit is set evaluate their distance to that sample.  The entries come in no particular order, so
// equal distances are ordered by sample position explicitly.
template <int K>
__global__ __launch_bounds__(256) void knn_cached_kernel(const float* __restrict__ xyz, int N,
                                                         const int32_t* __restrict__ sample_idx, int n, int k,
                                                         int32_t* __restrict__ out_pos,
                                                         float* __restrict__ out_d2,
                                                         const int32_t* __restrict__ flags,
                                                         int32_t* __restrict__ count,
                                                         int32_t* __restrict__ list,
                                                         const uint32_t* __restrict__ blk_off,
                                                         const BqEntry* __restrict__ blk_rows, int64_t cap)
{
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int blocks = (N + 63) >> 6;
    const int w = (int)blockIdx.x * 4 + wave;
    if (w >= blocks) return;                         // wave-uniform; the kernel has no barrier
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int32_t* __restrict__ sidx = sample_idx + (int64_t)b * n;

    const int j = (w << 6) | lane;
    float px = __builtin_nanf(""), py = px, pz = px;
    if (j < N) {
        px = cloud[(int64_t)j * 3 + 0];
        py = cloud[(int64_t)j * 3 + 1];
        pz = cloud[(int64_t)j * 3 + 2];
    }
    int hits = 0;
    Nearest<K> nb;
    nb.clear();

    const bool usable = __builtin_amdgcn_readfirstlane(flags[b]) != 0;
    if (usable) {
        const uint32_t* off = blk_off + (int64_t)b * ((int64_t)blocks + 1) + w;
        const uint32_t o0 = off[0];
        const int E = __builtin_amdgcn_readfirstlane((int)(off[1] - o0));
        const BqEntry* __restrict__ ent = blk_rows + (int64_t)b * cap + o0;
        for (int e0 = 0; e0 < E; e0 += 64) {
            const int cntw = E - e0 < 64 ? E - e0 : 64;
            BqEntry g;
            g.other = 0u;
            g.lo = g.hi = 0u;
            float sx = __builtin_nanf(""), sy = sx, sz = sx;
            if (lane < cntw) {
                g = ent[e0 + lane];
                const int si = g.other < (uint32_t)n ? sidx[g.other] : -1;
                if (si >= 0 && si < N) {
                    sx = cloud[(int64_t)si * 3 + 0];
                    sy = cloud[(int64_t)si * 3 + 1];
                    sz = cloud[(int64_t)si * 3 + 2];
                }
            }
            const uint64_t mine = ((uint64_t)g.hi << 32) | g.lo;
            for (int l = 0; l < cntw; ++l) {
                const float ax = rdlane_f(sx, l), ay = rdlane_f(sy, l), az = rdlane_f(sz, l);
                const uint64_t wd = rdlane_u64(mine, l);
                const int qq = __builtin_amdgcn_readlane((int)g.other, l);
                const bool hit = (wd >> lane) & 1ull;
                hits += hit ? 1 : 0;
                if (hit) nb.insert_any(dist2(px, py, pz, ax, ay, az), qq);
            }
        }
    }

    const bool in = j < N;
    const bool done = in && usable && hits >= k;
    if (done) {
        const int64_t o = ((int64_t)b * N + j) * k;
        nb.store(k, out_pos + o, out_d2 + o);
    }
    // fewer than k samples inside the radius: the point goes to the brute-force list
    const bool defer = in && !done;
    const uint64_t dm = __builtin_amdgcn_ballot_w64(defer);
    if (dm != 0) {
        int base = 0;
        if (lane == __builtin_ctzll(dm)) base = atomicAdd(count + b, __builtin_popcountll(dm));
        base = __builtin_amdgcn_readlane(base, __builtin_ctzll(dm));
        if (defer) list[(int64_t)b * N + base + lanes_below(dm)] = j;
    }
}

template <int K>
hipError_t launch_knn_k(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                        int32_t* out_pos, float* out_d2, const void* bq_cache, int32_t* flags,
                        int32_t* count, int32_t* list, int32_t* blk_cnt, uint32_t* blk_off, BqEntry* blk_rows,
                        int64_t blk_rows_cap, int32_t* out_deferred, hipStream_t stream)
{
    const dim3 grid_pts((unsigned)((N + kPointsPerWg - 1) / kPointsPerWg), (unsigned)B);
    if (!bq_cache) {
        hipLaunchKernelGGL((knn_brute_kernel<K, false>), grid_pts, dim3(256), 0, stream, xyz, N, sample_idx, n,
                           k, out_pos, out_d2, (const int32_t*)nullptr, (const int32_t*)nullptr,
                           (int32_t*)nullptr);
        return hipGetLastError();
    }
    const unsigned char* cache = reinterpret_cast<const unsigned char*>(bq_cache);
    hipLaunchKernelGGL(knn_check_kernel, dim3((unsigned)B), dim3(256), 0, stream, sample_idx, B, N, n, cache,
                       flags, count, blk_rows_cap);
    // the recorded tests by point block (a cache recorded for another shape leaves rows that are
    // never read: its flags are 0)
    if (launch_bq_group_by_block(bq_cache, B, N, blk_cnt, blk_off, blk_rows, blk_rows_cap, stream) != hipSuccess)
        return hipErrorInvalidValue;
    const int blocks = (N + 63) >> 6;
    const dim3 grid_words((unsigned)((blocks + 3) / 4), (unsigned)B);
    hipLaunchKernelGGL((knn_cached_kernel<K>), grid_words, dim3(256), 0, stream, xyz, N, sample_idx, n, k,
                       out_pos, out_d2, (const int32_t*)flags, count, list, (const uint32_t*)blk_off,
                       (const BqEntry*)blk_rows, blk_rows_cap);
    hipLaunchKernelGGL((knn_list_wave_kernel<K>), dim3(kWaveListMax / 4, (unsigned)B), dim3(256), 0, stream, xyz,
                       N, sample_idx, n, k, out_pos, out_d2, (const int32_t*)list, (const int32_t*)count);
    hipLaunchKernelGGL((knn_brute_kernel<K, true>), grid_pts, dim3(256), 0, stream, xyz, N, sample_idx, n, k,
                       out_pos, out_d2, (const int32_t*)list, (const int32_t*)count, out_deferred);
    return hipGetLastError();
}

}  // namespace

// The brute-force search of the points listed in list[b][0 .. count[b]) (left there by a first
// pass that could not settle them): a wave per point while the list is short, the tiled kernel for
// the rest.
template <int K>
hipError_t launch_knn_deferred_k(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                                 int32_t* out_pos, float* out_d2, int32_t* count, int32_t* list,
                                 int32_t* out_deferred, hipStream_t stream)
{
    const dim3 grid_pts((unsigned)((N + kPointsPerWg - 1) / kPointsPerWg), (unsigned)B);
    hipLaunchKernelGGL((knn_list_wave_kernel<K>), dim3(kWaveListMax / 4, (unsigned)B), dim3(256), 0, stream, xyz,
                       N, sample_idx, n, k, out_pos, out_d2, (const int32_t*)list, (const int32_t*)count);
    hipLaunchKernelGGL((knn_brute_kernel<K, true>), grid_pts, dim3(256), 0, stream, xyz, N, sample_idx, n, k,
                       out_pos, out_d2, (const int32_t*)list, (const int32_t*)count, out_deferred);
    return hipGetLastError();
}

hipError_t launch_knn_deferred(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                               int32_t* out_pos, float* out_d2, int32_t* count, int32_t* list,
                               int32_t* out_deferred, hipStream_t stream)
{
    if (k == 1)
        return launch_knn_deferred_k<1>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, count, list, out_deferred,
                                        stream);
    if (k <= 3)
        return launch_knn_deferred_k<3>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, count, list, out_deferred,
                                        stream);
    if (k <= 8)
        return launch_knn_deferred_k<8>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, count, list, out_deferred,
                                        stream);
    return hipErrorInvalidValue;
}

hipError_t launch_knn(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                      int32_t* out_pos, float* out_d2, const void* bq_cache, int32_t* flags,
                      int32_t* count, int32_t* list, int32_t* blk_cnt, uint32_t* blk_off, BqEntry* blk_rows,
                      int64_t blk_rows_cap, int32_t* out_deferred, hipStream_t stream)
{
    if (k == 1)
        return launch_knn_k<1>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, bq_cache, flags, count, list,
                               blk_cnt, blk_off, blk_rows, blk_rows_cap, out_deferred, stream);
    if (k <= 3)
        return launch_knn_k<3>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, bq_cache, flags, count, list,
                               blk_cnt, blk_off, blk_rows, blk_rows_cap, out_deferred, stream);
    if (k <= 8)
        return launch_knn_k<8>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, bq_cache, flags, count, list,
                               blk_cnt, blk_off, blk_rows, blk_rows_cap, out_deferred, stream);
    return hipErrorInvalidValue;
}

}  // namespace fastpoint
