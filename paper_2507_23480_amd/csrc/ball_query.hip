// Ball query (Section 3.1 step 2 of FastPoint, arXiv 2507.23480), gather and the
// coverage metric for gfx950.
//
// Two ball-query kernels produce identical output (first k hits by ascending
// index, strict < on squared binary32 distances, padded with the first hit):
//   * brute force, one centre per lane: the points are streamed in index order through
//     scalar loads, so each lane scans "its" ball sequentially and the first-k rule and the
//     early exit fall out of the loop order; the index range is split over the waves of a
//     workgroup (more waves in flight) and the per-range hit lists are merged in LDS;
//   * cache reader, one centre per lane: reads the words the sampler recorded for that
//     sample (Section 4.2: the radius test was already done while the sample was folded
//     into the distance array) and keeps the first k set bits; a centre without usable
//     words is tested against all points by the same wave.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

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

constexpr int kChunk = 16;      // points tested per pass of the brute-force inner loop

// Last step of both ball-query kernels.  Each of the S waves of a workgroup has listed, per
// centre, the first hits of its part of the index range (hits [S][64][kp], counts [S][64], in
// LDS); the parts are concatenated in index order, cut at k and padded with the first hit.
// Wave w writes the rows of centres w, w+S, ...
template <int S>
__device__ __forceinline__ void merge_ranges(const int32_t* hits, const int32_t* counts, int kp, int k, int b,
                                             int q0, int M, int w, int lane, int32_t* __restrict__ out_idx,
                                             int32_t* __restrict__ out_cnt)
{
    for (int cc = w; cc < 64; cc += S) {
        const int qq = q0 + cc;
        if (qq >= M) break;
        int off[S + 1];
        off[0] = 0;
#pragma unroll
        for (int sgm = 0; sgm < S; ++sgm) off[sgm + 1] = off[sgm] + counts[sgm * 64 + cc];
        const int total = off[S] < k ? off[S] : k;
        int first = -1;
#pragma unroll
        for (int sgm = S - 1; sgm >= 0; --sgm)
            if (off[sgm + 1] > off[sgm]) first = hits[((int64_t)sgm * 64 + cc) * kp];
        int32_t* row = out_idx + ((int64_t)b * M + qq) * k;
        for (int t = lane; t < k; t += 64) {
            int v = first;
            if (t < total) {
#pragma unroll
                for (int sgm = 0; sgm < S; ++sgm)
                    if (t >= off[sgm] && t < off[sgm + 1]) v = hits[((int64_t)sgm * 64 + cc) * kp + (t - off[sgm])];
            }
            row[t] = v;
        }
        if (lane == 0 && out_cnt) out_cnt[(int64_t)b * M + qq] = total;
    }
}

// Brute-force ball query.  A workgroup of S waves owns 64 centres (one per lane); wave w scans
// the w-th of S equal index ranges of the cloud, so S times as many waves are in flight as
// there are groups of 64 centres and the scalar point loads of one wave hide behind the
// arithmetic of the others.  Each wave keeps the first k hits of its range per centre in LDS;
// the ranges are then concatenated in index order and cut at k.
//   LDS: hits [S][64][k+1] int32, counts [S][64] int32  (dynamic, S*64*(k+2)*4 bytes)
template <int S>
__global__ __launch_bounds__(S * 64) void bq_brute_kernel(const float* __restrict__ xyz, int N,
                                                          const int32_t* __restrict__ center_idx, int M,
                                                          float r2, int k, int32_t* __restrict__ out_idx,
                                                          int32_t* __restrict__ out_cnt)
{
    extern __shared__ int32_t lds[];
    const int kp = k + 1;                                   // padded row: conflict-free columns
    int32_t* hits = lds;                                    // [S][64][kp]
    int32_t* counts = lds + S * 64 * kp;                    // [S][64]
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);    // wave-uniform: scalar loads
    const int q0 = (int)blockIdx.x * 64;
    const int q = q0 + lane;
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int c = q < M ? center_idx[(int64_t)b * M + q] : -1;
    const bool okc = c >= 0 && c < N;
    // a centre that does not exist compares false against every point
    const float cx = okc ? cloud[(int64_t)c * 3 + 0] : __builtin_nanf("");
    const float cy = okc ? cloud[(int64_t)c * 3 + 1] : 0.0f;
    const float cz = okc ? cloud[(int64_t)c * 3 + 2] : 0.0f;

    int seg_len = (N + S - 1) / S;
    seg_len = (seg_len + kChunk - 1) / kChunk * kChunk;
    const int j_begin = w * seg_len < N ? w * seg_len : N;
    const int j_end = (w + 1) * seg_len < N ? (w + 1) * seg_len : N;
    int32_t* myrow = hits + ((int64_t)w * 64 + lane) * kp;
    int cnt = 0;

    const int nfull = j_begin + (j_end - j_begin) / kChunk * kChunk;
    int j0 = j_begin;
    for (; j0 < nfull; j0 += kChunk) {
        if (__builtin_amdgcn_ballot_w64(okc && cnt < k) == 0) break;
        uint64_t m[kChunk];
        uint64_t any = 0;
        const float* __restrict__ pb = cloud + (int64_t)j0 * 3;   // uniform address: scalar loads
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const float t = dist2(cx, cy, cz, pb[3 * u + 0], pb[3 * u + 1], pb[3 * u + 2]);
            m[u] = __builtin_amdgcn_ballot_w64(t < r2);
            any |= m[u];
        }
        if (any != 0) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                if (((m[u] >> lane) & 1ull) && cnt < k) {
                    myrow[cnt] = j0 + u;
                    ++cnt;
                }
            }
        }
    }
    if (j0 >= nfull) {
        for (int j = nfull; j < j_end; ++j) {
            const float* pj = cloud + (int64_t)j * 3;
            const float t = dist2(cx, cy, cz, pj[0], pj[1], pj[2]);
            if (t < r2 && cnt < k) {
                myrow[cnt] = j;
                ++cnt;
            }
        }
    }
    counts[w * 64 + lane] = cnt;
    __syncthreads();
    merge_ranges<S>(hits, counts, kp, k, b, q0, M, w, lane, out_idx, out_cnt);
}

constexpr int kCachedUnroll = 8;     // cache words requested together by the cache reader

// Cache reader.  A workgroup of S waves owns 64 consecutive centres of a cloud, one per lane;
// wave w takes the w-th of S equal ranges of point blocks.  Word [block][q] of the cache holds
// the radius tests of sample q against the 64 points of that block, and the words of consecutive
// samples are contiguous: every load of a wave brings one block for all its 64 centres.  A lane
// walks the set bits of its words in index order and keeps the first k of its range; the ranges
// are merged as in the brute-force kernel.  Centres without a usable column (not the cached
// sample of that position, or another radius) are tested against the points of the range instead.
//   LDS: hits [S][64][k+1] int32, counts [S][64] int32  (dynamic)
template <int S>
__global__ __launch_bounds__(S * 64) void bq_cached_kernel(const float* __restrict__ xyz, int B, int N,
                                                           const int32_t* __restrict__ center_idx, int M,
                                                           float r2, int k, int32_t* __restrict__ out_idx,
                                                           int32_t* __restrict__ out_cnt,
                                                           const unsigned char* __restrict__ cache)
{
    extern __shared__ int32_t lds[];
    const int kp = k + 1;                                   // padded row: conflict-free columns
    int32_t* hits = lds;                                    // [S][64][kp]
    int32_t* counts = lds + S * 64 * kp;                    // [S][64]
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int q0 = (int)blockIdx.x * 64;
    const int q = q0 + lane;
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int c = q < M ? center_idx[(int64_t)b * M + q] : -1;
    const bool okc = c >= 0 && c < N;
    int32_t* myrow = hits + ((int64_t)w * 64 + lane) * kp;
    int cnt = 0;

    // this wave's range of point blocks
    const int blocks = (N + 63) >> 6;
    const int per = (blocks + S - 1) / S;
    const int blk_begin = w * per < blocks ? w * per : blocks;
    const int blk_end = (w + 1) * per < blocks ? (w + 1) * per : blocks;

    const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
    bool usable = h->magic == kBqMagic && h->valid == 1 && h->B == B && h->N == N &&
                  h->r2_bits == __float_as_uint(r2) && okc && q < h->n;
    if (usable) {
        const int32_t* cidx = reinterpret_cast<const int32_t*>(cache + h->idx_offset);
        usable = cidx[(int64_t)b * h->n + q] == c;
    }
    if (__builtin_amdgcn_ballot_w64(usable) != 0) {
        const int64_t col_words = h->col_words;
        const uint64_t* __restrict__ col = reinterpret_cast<const uint64_t*>(cache + h->bits_offset) +
                                           (int64_t)b * blocks * col_words + (usable ? q : 0);
        for (int w0 = blk_begin; w0 < blk_end; w0 += kCachedUnroll) {
            if (__builtin_amdgcn_ballot_w64(usable && cnt < k) == 0) break;
            uint64_t wd[kCachedUnroll];
#pragma unroll
            for (int u = 0; u < kCachedUnroll; ++u)
                wd[u] = (usable && w0 + u < blk_end) ? col[(int64_t)(w0 + u) * col_words] : 0ull;
#pragma unroll
            for (int u = 0; u < kCachedUnroll; ++u) {
                uint64_t x = wd[u];
                while (x != 0 && cnt < k) {
                    myrow[cnt] = ((w0 + u) << 6) + __builtin_ctzll(x);
                    ++cnt;
                    x &= x - 1;
                }
            }
        }
    }
    if (__builtin_amdgcn_ballot_w64(okc && !usable) != 0) {
        const bool mine = okc && !usable;
        const float cx = mine ? cloud[(int64_t)c * 3 + 0] : __builtin_nanf("");
        const float cy = mine ? cloud[(int64_t)c * 3 + 1] : 0.0f;
        const float cz = mine ? cloud[(int64_t)c * 3 + 2] : 0.0f;
        const int j_end = blk_end * 64 < N ? blk_end * 64 : N;
        for (int j = blk_begin * 64; j < j_end; ++j) {
            if (__builtin_amdgcn_ballot_w64(mine && cnt < k) == 0) break;
            const float* pj = cloud + (int64_t)j * 3;        // uniform address: scalar loads
            if (dist2(cx, cy, cz, pj[0], pj[1], pj[2]) < r2 && cnt < k) {
                myrow[cnt] = j;
                ++cnt;
            }
        }
    }
    counts[w * 64 + lane] = cnt;
    __syncthreads();
    merge_ranges<S>(hits, counts, kp, k, b, q0, M, w, lane, out_idx, out_cnt);
}

__global__ void gather_kernel(const float* __restrict__ xyz, int B, int N,
                              const int32_t* __restrict__ idx, int M, float* __restrict__ out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)B * M) return;
    const int b = (int)(t / M);
    const int j = idx[t];
    float x, y, z;
    if (j >= 0 && j < N) {
        const float* p = xyz + ((int64_t)b * N + j) * 3;
        x = p[0];
        y = p[1];
        z = p[2];
    } else {
        x = y = z = __builtin_nanf("");
    }
    out[t * 3 + 0] = x;
    out[t * 3 + 1] = y;
    out[t * 3 + 2] = z;
}

__global__ void zero_floats_kernel(float* p, int n)
{
    const int t = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (t < n) p[t] = 0.0f;
}

// out[b] = max_j min_q dist2(P[j], S[q]); distances are >= +0 so the unsigned
// order of the bit patterns is the order of the values
__global__ __launch_bounds__(256) void coverage_kernel(const float* __restrict__ xyz, int N,
                                                       const float* __restrict__ sxyz, int n,
                                                       float* __restrict__ out)
{
    const int b = (int)blockIdx.y;
    const int j = (int)blockIdx.x * 256 + (int)threadIdx.x;
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const float* __restrict__ samp = sxyz + (int64_t)b * n * 3;
    float best = 0.0f;
    if (j < N) {
        const float px = cloud[(int64_t)j * 3 + 0], py = cloud[(int64_t)j * 3 + 1],
                    pz = cloud[(int64_t)j * 3 + 2];
        best = __builtin_inff();
        for (int q = 0; q < n; ++q) {
            const float* s = samp + (int64_t)q * 3;            // uniform address: scalar loads
            best = __builtin_fminf(best, dist2(s[0], s[1], s[2], px, py, pz));
        }
    }
    __shared__ uint32_t red[256];
    red[threadIdx.x] = __float_as_uint(best);
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] = max(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) atomicMax(reinterpret_cast<unsigned int*>(out) + b, red[0]);
}

// eight independent chains of a multiplication and an addition per thread (see fp_probe_fp32_rate)
__global__ __launch_bounds__(256) void probe_fp32_kernel(float* __restrict__ out, int iterations, float m, float c)
{
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = (float)(threadIdx.x + k) * 1.0e-3f;
    for (int i = 0; i < iterations; ++i) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float t = v[k] * m;
            v[k] = t + c;
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) s = s + v[k];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_probe_fp32(int blocks, int iterations, float* out, hipStream_t stream)
{
    // the factors are run-time values, so that the chains cannot be folded
    hipLaunchKernelGGL(probe_fp32_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, out, iterations,
                       0.9999f, 1.0e-4f);
    return hipGetLastError();
}

hipError_t launch_ball_query(const float* xyz, int B, int N, const int32_t* center_idx, int M,
                             float r2, int k, int32_t* out_idx, int32_t* out_cnt,
                             const void* bq_cache, hipStream_t stream)
{
    if (M == 0) return hipSuccess;
    const dim3 grid((unsigned)((M + 63) / 64), (unsigned)B);
    const size_t per_wave = (size_t)64 * (k + 2) * sizeof(int32_t);
    if (bq_cache) {
        // enough waves to fill the device, as far as the hit lists leave room in 48 KB of LDS
        const unsigned char* cache = reinterpret_cast<const unsigned char*>(bq_cache);
        const int64_t groups = (int64_t)grid.x * grid.y;
        const int64_t blocks = ((int64_t)N + 63) / 64;
        int want = groups >= 4096 ? 1 : groups >= 2048 ? 2 : groups >= 1024 ? 4 : 8;
        while (want > 1 && ((size_t)want * per_wave > 48 * 1024 || blocks < (int64_t)want * 4)) want >>= 1;
        if (want == 8)
            hipLaunchKernelGGL(bq_cached_kernel<8>, grid, dim3(512), 8 * per_wave, stream, xyz, B, N, center_idx, M,
                               r2, k, out_idx, out_cnt, cache);
        else if (want == 4)
            hipLaunchKernelGGL(bq_cached_kernel<4>, grid, dim3(256), 4 * per_wave, stream, xyz, B, N, center_idx, M,
                               r2, k, out_idx, out_cnt, cache);
        else if (want == 2)
            hipLaunchKernelGGL(bq_cached_kernel<2>, grid, dim3(128), 2 * per_wave, stream, xyz, B, N, center_idx, M,
                               r2, k, out_idx, out_cnt, cache);
        else if (per_wave <= 64 * 1024)
            hipLaunchKernelGGL(bq_cached_kernel<1>, grid, dim3(64), per_wave, stream, xyz, B, N, center_idx, M, r2,
                               k, out_idx, out_cnt, cache);
        else
            return hipErrorInvalidValue;
    } else {
        // As many waves per group of 64 centres as the hit lists leave room for in LDS: 48 KB, so
        // that several workgroups share a compute unit -- or, when the grid would leave most
        // compute units empty anyway, 144 of the 160 KB, which shortens each wave's scan.
        const int64_t groups = (int64_t)grid.x * grid.y;
        const size_t budget = groups <= 512 ? (size_t)144 * 1024 : (size_t)48 * 1024;
        // more than 64 KB has to be asked for, once per device
        static std::atomic<uint64_t> lds_raised{0};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return hipErrorInvalidValue;
        if (((lds_raised.load() >> dev) & 1u) == 0) {
            const int most = 160 * 1024;
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&bq_brute_kernel<8>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, most) != hipSuccess ||
                hipFuncSetAttribute(reinterpret_cast<const void*>(&bq_brute_kernel<4>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, most) != hipSuccess ||
                hipFuncSetAttribute(reinterpret_cast<const void*>(&bq_brute_kernel<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, most) != hipSuccess)
                return hipErrorInvalidValue;
            lds_raised.fetch_or((uint64_t)1 << dev);
        }
        if (8 * per_wave <= budget)
            hipLaunchKernelGGL(bq_brute_kernel<8>, grid, dim3(512), 8 * per_wave, stream, xyz, N, center_idx, M,
                               r2, k, out_idx, out_cnt);
        else if (4 * per_wave <= budget)
            hipLaunchKernelGGL(bq_brute_kernel<4>, grid, dim3(256), 4 * per_wave, stream, xyz, N, center_idx, M,
                               r2, k, out_idx, out_cnt);
        else if (2 * per_wave <= budget)
            hipLaunchKernelGGL(bq_brute_kernel<2>, grid, dim3(128), 2 * per_wave, stream, xyz, N, center_idx, M,
                               r2, k, out_idx, out_cnt);
        else if (per_wave <= 64 * 1024)
            hipLaunchKernelGGL(bq_brute_kernel<1>, grid, dim3(64), per_wave, stream, xyz, N, center_idx, M, r2,
                               k, out_idx, out_cnt);
        else
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gather(const float* xyz, int B, int N, const int32_t* idx, int M, float* out,
                         hipStream_t stream)
{
    const int64_t total = (int64_t)B * M;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(gather_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, xyz, B,
                       N, idx, M, out);
    return hipGetLastError();
}

hipError_t launch_coverage(const float* xyz, int B, int N, const float* sxyz, int n, float* out,
                           hipStream_t stream)
{
    hipLaunchKernelGGL(zero_floats_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, stream, out, B);
    hipLaunchKernelGGL(coverage_kernel, dim3((unsigned)((N + 255) / 256), (unsigned)B), dim3(256), 0,
                       stream, xyz, N, sxyz, n, out);
    return hipGetLastError();
}

}  // namespace fastpoint
