// Ball query (Section 3.1 step 2 of FastPoint, arXiv 2507.23480), gather and the
// coverage metric for gfx950.
//
// Two ball-query kernels produce identical output (first k hits by ascending
// index, strict < on squared binary32 distances, padded with the first hit):
//   * brute force, one centre per lane: the points are streamed in index order through
//     scalar loads, so each lane scans "its" ball sequentially and the first-k rule and the
//     early exit fall out of the loop order; the index range is split over the waves of a
//     workgroup (more waves in flight) and the per-range hit lists are merged in LDS;
//   * cache reader, one centre per wave: reads the bitmap row the sampler
//     recorded for that sample (Section 4.2: the radius test was already done
//     while the sample was folded into the distance array) and expands the
//     first k set bits; a centre without a usable row is tested against all
//     points by the same wave with a ballot per 64 points.
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

constexpr int kChunk = 16;      // points tested per pass of the brute-force inner loop

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

    // concatenate the S ranges of every centre in index order, cut at k, pad with the first hit
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

// emit the set bits of one 64-bit hit word (indices base..base+63) into the row
__device__ __forceinline__ void emit_word(uint64_t wd, int base, int lane, int k, int32_t* row,
                                          int& cnt, int& first)
{
    if (cnt == 0) first = base + __builtin_ctzll(wd);
    const bool bit = (wd >> lane) & 1ull;
    const int rank = cnt + lanes_below(wd);
    if (bit && rank < k) row[rank] = base + lane;
    cnt += __builtin_popcountll(wd);
}

__global__ __launch_bounds__(256) void bq_cached_kernel(const float* __restrict__ xyz, int B, int N,
                                                        const int32_t* __restrict__ center_idx, int M,
                                                        float r2, int k, int32_t* __restrict__ out_idx,
                                                        int32_t* __restrict__ out_cnt,
                                                        const unsigned char* __restrict__ cache)
{
    const int lane = (int)threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    if (wave >= (int64_t)B * M) return;
    const int b = (int)(wave / M), q = (int)(wave % M);
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int c = center_idx[(int64_t)b * M + q];
    int32_t* row = out_idx + ((int64_t)b * M + q) * k;
    int cnt = 0;
    int first = -1;
    if (c >= 0 && c < N) {
        const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
        bool usable = h->magic == kBqMagic && h->B == B && h->N == N && q < h->n &&
                      h->r2_bits == __float_as_uint(r2);
        if (usable) {
            const int32_t* cidx = reinterpret_cast<const int32_t*>(cache + h->idx_offset);
            usable = cidx[(int64_t)b * h->n + q] == c;
        }
        if (usable) {
            const uint64_t* bits = reinterpret_cast<const uint64_t*>(cache + h->bits_offset) +
                                   ((int64_t)b * h->n + q) * h->row_words;
            const int nwords = (N + 63) >> 6;
            for (int w0 = 0; w0 < nwords && cnt < k; w0 += 64) {
                const uint64_t word = (w0 + lane < nwords) ? bits[w0 + lane] : 0ull;
                uint64_t nz = __builtin_amdgcn_ballot_w64(word != 0);
                while (nz != 0 && cnt < k) {
                    const int l = __builtin_ctzll(nz);
                    nz &= nz - 1;
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)word, l);
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(word >> 32), l);
                    emit_word(((uint64_t)hi << 32) | lo, (w0 + l) << 6, lane, k, row, cnt, first);
                }
            }
        } else {
            const float cx = cloud[(int64_t)c * 3 + 0];
            const float cy = cloud[(int64_t)c * 3 + 1];
            const float cz = cloud[(int64_t)c * 3 + 2];
            for (int j0 = 0; j0 < N && cnt < k; j0 += 64) {
                const int j = j0 + lane;
                bool hit = false;
                if (j < N) {
                    const float* pj = cloud + (int64_t)j * 3;
                    hit = dist2(cx, cy, cz, pj[0], pj[1], pj[2]) < r2;
                }
                const uint64_t wd = __builtin_amdgcn_ballot_w64(hit);
                if (wd != 0) emit_word(wd, j0, lane, k, row, cnt, first);
            }
        }
        cnt = cnt < k ? cnt : k;
    }
    for (int t = cnt + lane; t < k; t += 64) row[t] = first;
    if (lane == 0 && out_cnt) out_cnt[(int64_t)b * M + q] = cnt;
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

__global__ void bq_header_kernel(BqHeader* dst, BqHeader h) { *dst = h; }

}  // namespace

hipError_t launch_ball_query(const float* xyz, int B, int N, const int32_t* center_idx, int M,
                             float r2, int k, int32_t* out_idx, int32_t* out_cnt,
                             const void* bq_cache, hipStream_t stream)
{
    if (M == 0) return hipSuccess;
    if (bq_cache) {
        const int64_t waves = (int64_t)B * M;
        const int64_t blocks = (waves + 3) / 4;
        hipLaunchKernelGGL(bq_cached_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, xyz, B, N,
                           center_idx, M, r2, k, out_idx, out_cnt,
                           reinterpret_cast<const unsigned char*>(bq_cache));
    } else {
        // as many waves per group of 64 centres as the hit lists leave room for in 48 KB of LDS
        const dim3 grid((unsigned)((M + 63) / 64), (unsigned)B);
        const size_t per_wave = (size_t)64 * (k + 2) * sizeof(int32_t);
        if (8 * per_wave <= 48 * 1024)
            hipLaunchKernelGGL(bq_brute_kernel<8>, grid, dim3(512), 8 * per_wave, stream, xyz, N, center_idx, M,
                               r2, k, out_idx, out_cnt);
        else if (4 * per_wave <= 48 * 1024)
            hipLaunchKernelGGL(bq_brute_kernel<4>, grid, dim3(256), 4 * per_wave, stream, xyz, N, center_idx, M,
                               r2, k, out_idx, out_cnt);
        else if (2 * per_wave <= 48 * 1024)
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

hipError_t launch_bq_header(void* cache, const BqHeader& h, hipStream_t stream)
{
    hipLaunchKernelGGL(bq_header_kernel, dim3(1), dim3(1), 0, stream, reinterpret_cast<BqHeader*>(cache), h);
    return hipGetLastError();
}

}  // namespace fastpoint
