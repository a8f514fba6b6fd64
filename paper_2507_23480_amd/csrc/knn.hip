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
//   * redundancy-free: the sampler recorded, for every sample, the bitmap of the points closer
//     than the cache radius (the exclusion list at an extra radius of Section 4.2).  Read
//     column-wise this is the list of samples near each point: only those distances are
//     evaluated.  When a point has at least k samples inside the radius they are its k nearest
//     (every other sample is farther than all of them); the remaining points are collected in a
//     list and searched by brute force in a second launch.
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
template <int K>
__device__ __forceinline__ void visit_sample(Nearest<K> (&nb)[2], const float (&px)[2], const float (&py)[2],
                                             const float (&pz)[2], const float4 s, int q)
{
    const float d0 = dist2(px[0], py[0], pz[0], s.x, s.y, s.z);
    const float d1 = dist2(px[1], py[1], pz[1], s.x, s.y, s.z);
    // after the first few samples a wave rarely has a lane whose list changes
    if (__builtin_amdgcn_ballot_w64(d0 < nb[0].d[K - 1] || d1 < nb[1].d[K - 1]) != 0) {
        nb[0].insert(d0, q);
        nb[1].insert(d1, q);
    }
}

constexpr int kTile = 256;          // samples staged in LDS per pass
constexpr int kPointsPerWg = 512;   // two points per thread

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
        if (cnt == kTile) {
#pragma unroll 4
            for (int t = 0; t < kTile; ++t) visit_sample<K>(nb, px, py, pz, smp[t], q0 + t);
        } else {
#pragma unroll 1
            for (int t = 0; t < cnt; ++t) visit_sample<K>(nb, px, py, pz, smp[t], q0 + t);
        }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (j[u] >= 0 && j[u] < N) {
            const int64_t o = ((int64_t)b * N + j[u]) * k;
            nb[u].store(k, out_pos + o, out_d2 + o);
        }
}

// flags[b] = 1 when the cache was recorded for exactly this sample list of cloud b;
// also empties the cloud's list of deferred points.
__global__ __launch_bounds__(256) void knn_check_kernel(const int32_t* __restrict__ sample_idx, int B, int N,
                                                        int n, const unsigned char* __restrict__ cache,
                                                        int32_t* __restrict__ flags,
                                                        int32_t* __restrict__ count)
{
    const int b = (int)blockIdx.x;
    const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
    const bool ok = h->magic == kBqMagic && h->valid == 1 && h->B == B && h->N == N && h->n == n;
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

constexpr int kWordsPerWave = 4;    // 64-bit bitmap words (64 points each) one wave owns

// Redundancy-free search.  A wave owns 4 consecutive bitmap words = 256 points (lane l holds
// bit l of each word); a workgroup's 4 waves cover 128 contiguous bytes of every row.  The rows
// (one per sample) are read 64 at a time, one row per lane; rows whose 4 words are all zero --
// nearly all of them -- cost nothing more.
template <int K>
__global__ __launch_bounds__(256) void knn_cached_kernel(const float* __restrict__ xyz, int N,
                                                         const int32_t* __restrict__ sample_idx, int n, int k,
                                                         int32_t* __restrict__ out_pos,
                                                         float* __restrict__ out_d2,
                                                         const unsigned char* __restrict__ cache,
                                                         const int32_t* __restrict__ flags,
                                                         int32_t* __restrict__ count,
                                                         int32_t* __restrict__ list)
{
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int nwords = (N + 63) >> 6;
    const int wbase = ((int)blockIdx.x * 4 + wave) * kWordsPerWave;
    if (wbase >= nwords) return;                     // wave-uniform; the kernel has no barrier
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int32_t* __restrict__ sidx = sample_idx + (int64_t)b * n;

    int j[kWordsPerWave];
    float px[kWordsPerWave], py[kWordsPerWave], pz[kWordsPerWave];
    int hits[kWordsPerWave];
    Nearest<K> nb[kWordsPerWave];
#pragma unroll
    for (int u = 0; u < kWordsPerWave; ++u) {
        j[u] = ((wbase + u) << 6) | lane;
        px[u] = py[u] = pz[u] = __builtin_nanf("");
        if (j[u] < N) {
            px[u] = cloud[(int64_t)j[u] * 3 + 0];
            py[u] = cloud[(int64_t)j[u] * 3 + 1];
            pz[u] = cloud[(int64_t)j[u] * 3 + 2];
        }
        hits[u] = 0;
        nb[u].clear();
    }

    const bool usable = __builtin_amdgcn_readfirstlane(flags[b]) != 0;
    if (usable) {
        const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
        const int64_t row_words = h->row_words;
        const uint64_t* __restrict__ bits =
            reinterpret_cast<const uint64_t*>(cache + h->bits_offset) + (int64_t)b * n * row_words + wbase;
        // words past ceil(N/64) belong to the row's padding and are not defined
        uint64_t keep[kWordsPerWave];
#pragma unroll
        for (int u = 0; u < kWordsPerWave; ++u) keep[u] = (wbase + u < nwords) ? ~0ull : 0ull;

        uint64_t cur[kWordsPerWave], nxt[kWordsPerWave];
#pragma unroll
        for (int u = 0; u < kWordsPerWave; ++u) cur[u] = 0;
        if (lane < n) {
            const ulonglong2* r = reinterpret_cast<const ulonglong2*>(bits + (int64_t)lane * row_words);
            const ulonglong2 a = r[0], c = r[1];
            cur[0] = a.x;
            cur[1] = a.y;
            cur[2] = c.x;
            cur[3] = c.y;
        }
        for (int q0 = 0; q0 < n; q0 += 64) {
            // the next 64 rows are requested before this block is examined
#pragma unroll
            for (int u = 0; u < kWordsPerWave; ++u) nxt[u] = 0;
            if (q0 + 64 + lane < n) {
                const ulonglong2* r =
                    reinterpret_cast<const ulonglong2*>(bits + (int64_t)(q0 + 64 + lane) * row_words);
                const ulonglong2 a = r[0], c = r[1];
                nxt[0] = a.x;
                nxt[1] = a.y;
                nxt[2] = c.x;
                nxt[3] = c.y;
            }
#pragma unroll
            for (int u = 0; u < kWordsPerWave; ++u) cur[u] &= keep[u];
            const bool nz = (cur[0] | cur[1] | cur[2] | cur[3]) != 0;
            uint64_t rows = __builtin_amdgcn_ballot_w64(nz);
            if (rows != 0) {
                float sx = __builtin_nanf(""), sy = sx, sz = sx;
                if (nz) {
                    const int si = sidx[q0 + lane];
                    if (si >= 0 && si < N) {
                        sx = cloud[(int64_t)si * 3 + 0];
                        sy = cloud[(int64_t)si * 3 + 1];
                        sz = cloud[(int64_t)si * 3 + 2];
                    }
                }
                while (rows != 0) {                  // ascending sample position
                    const int l = __builtin_ctzll(rows);
                    rows &= rows - 1;
                    const float ax = rdlane_f(sx, l), ay = rdlane_f(sy, l), az = rdlane_f(sz, l);
#pragma unroll
                    for (int u = 0; u < kWordsPerWave; ++u) {
                        const uint64_t wu = rdlane_u64(cur[u], l);
                        if (wu != 0) {
                            const bool hit = (wu >> lane) & 1ull;
                            const float d = hit ? dist2(px[u], py[u], pz[u], ax, ay, az) : __builtin_inff();
                            hits[u] += hit ? 1 : 0;
                            nb[u].insert(d, q0 + l);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kWordsPerWave; ++u) cur[u] = nxt[u];
        }
    }

#pragma unroll
    for (int u = 0; u < kWordsPerWave; ++u) {
        const bool in = j[u] < N;
        const bool done = in && usable && hits[u] >= k;
        if (done) {
            const int64_t o = ((int64_t)b * N + j[u]) * k;
            nb[u].store(k, out_pos + o, out_d2 + o);
        }
        // fewer than k samples inside the radius: the point goes to the brute-force list
        const bool defer = in && !done;
        const uint64_t dm = __builtin_amdgcn_ballot_w64(defer);
        if (dm != 0) {
            int base = 0;
            if (lane == __builtin_ctzll(dm)) base = atomicAdd(count + b, __builtin_popcountll(dm));
            base = __builtin_amdgcn_readlane(base, __builtin_ctzll(dm));
            if (defer) list[(int64_t)b * N + base + lanes_below(dm)] = j[u];
        }
    }
}

template <int K>
hipError_t launch_knn_k(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                        int32_t* out_pos, float* out_d2, const void* bq_cache, int32_t* flags,
                        int32_t* count, int32_t* list, int32_t* out_deferred, hipStream_t stream)
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
                       flags, count);
    const int nwords = (N + 63) >> 6;
    const dim3 grid_words((unsigned)((nwords + 4 * kWordsPerWave - 1) / (4 * kWordsPerWave)), (unsigned)B);
    hipLaunchKernelGGL((knn_cached_kernel<K>), grid_words, dim3(256), 0, stream, xyz, N, sample_idx, n, k,
                       out_pos, out_d2, cache, (const int32_t*)flags, count, list);
    hipLaunchKernelGGL((knn_brute_kernel<K, true>), grid_pts, dim3(256), 0, stream, xyz, N, sample_idx, n, k,
                       out_pos, out_d2, (const int32_t*)list, (const int32_t*)count, out_deferred);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_knn(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                      int32_t* out_pos, float* out_d2, const void* bq_cache, int32_t* flags,
                      int32_t* count, int32_t* list, int32_t* out_deferred, hipStream_t stream)
{
    if (k == 1)
        return launch_knn_k<1>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, bq_cache, flags, count, list,
                               out_deferred, stream);
    if (k <= 3)
        return launch_knn_k<3>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, bq_cache, flags, count, list,
                               out_deferred, stream);
    if (k <= 8)
        return launch_knn_k<8>(xyz, B, N, sample_idx, n, k, out_pos, out_d2, bq_cache, flags, count, list,
                               out_deferred, stream);
    return hipErrorInvalidValue;
}

}  // namespace fastpoint
