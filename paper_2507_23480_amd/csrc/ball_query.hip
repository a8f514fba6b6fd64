// Ball query (Section 3.1 step 2 of FastPoint, arXiv 2507.23480), gather and the
// coverage metric for gfx950.
//
// Two ball-query kernels produce identical output (first k hits by ascending
// index, strict < on squared binary32 distances, padded with the first hit):
//   * brute force, one centre per lane: the points are streamed in index order through
//     scalar loads, so each lane scans "its" ball sequentially and the first-k rule and the
//     early exit fall out of the loop order; the index range is split over the waves of a
//     workgroup (more waves in flight) and the per-range hit lists are merged in LDS;
//   * cache reader, one wave per centre: reads the entries the sampler recorded for that
//     sample (Section 4.2: the radius test was already done while the sample was folded
//     into the distance array), one per point block its ball reaches, and keeps the first k
//     set bits in block order; a centre the record does not cover is tested against all
//     points by the same wave.
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
typedef float Quad __attribute__((ext_vector_type(4), aligned(4)));   // four coordinates, wherever they lie

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
        // The test t < r2 of dist2's t = (dx dx + dy dy) + dz dz, decided after the second term where it
        // can be: the partial sums only grow (every term is >= 0 and rounding is monotone), so a point
        // whose dx dx + dy dy is not below r2 for any of the wave's 64 centres is done after six
        // operations instead of nine -- nearly every point of a large cloud.  The sums are those of
        // dist2, term by term, so a decision that is reached is the same.  (Deciding after dx dx already
        // was slower: with 64 unrelated centres in a wave half of the points pass that test for one of
        // them, and a branch per point costs more than the three operations it saves.)
        float t2[kChunk];
        uint64_t m2[kChunk];
        uint64_t any = 0;
        const float* __restrict__ pb = cloud + (int64_t)j0 * 3;   // uniform address: scalar loads
        // the chunk's 48 coordinates as twelve 16-byte scalar loads: every one of them holds an x or a
        // y, so none of them moves into the branch below (where a wave would wait for it)
        Quad qd[3 * kChunk / 4];
#pragma unroll
        for (int v = 0; v < 3 * kChunk / 4; ++v) qd[v] = reinterpret_cast<const Quad*>(pb)[v];
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const float dx = cx - qd[(3 * u) / 4][(3 * u) % 4];
            const float dy = cy - qd[(3 * u + 1) / 4][(3 * u + 1) % 4];
            float t = dx * dx;
            t = t + dy * dy;
            t2[u] = t;
            m2[u] = __builtin_amdgcn_ballot_w64(t < r2);
            any |= m2[u];
        }
        if (any != 0) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                if (m2[u] != 0) {                                 // uniform
                    const float dz = cz - qd[(3 * u + 2) / 4][(3 * u + 2) % 4];
                    const float t3 = t2[u] + dz * dz;
                    if (t3 < r2 && cnt < k) {
                        myrow[cnt] = j0 + u;
                        ++cnt;
                    }
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

// ------------------------------------------------------------------ the recorded radius tests
// Grouping of a cache's entries (kernels.h) by a key -- the sample (rows the ball query reads) or
// the point block (rows the k-NN search reads): count per key, exclusive scan, scatter.  The
// entries of a row end up in no particular order; readers order them.
// Places of cloud b's list that may hold an entry: the chunks handed out -- none when the record
// is incomplete or would not fit the rows it is grouped into.  Place e holds an entry when
// bq_place_used() says so.
__device__ __forceinline__ int64_t bq_places(const BqHeader* h, const unsigned char* cache, int b, int64_t rows_cap)
{
    if (reinterpret_cast<const uint32_t*>(cache + h->ovf_offset)[b] != 0) return 0;
    const int64_t chunks = (int64_t) reinterpret_cast<const uint32_t*>(cache + h->cursor_offset)[b];
    const int64_t most = h->cap / kBqChunk;
    const int64_t places = (chunks < most ? chunks : most) * kBqChunk;
    return places <= rows_cap ? places : 0;
}
__device__ __forceinline__ bool bq_place_used(const BqHeader* h, const unsigned char* cache, int b, int64_t e)
{
    const uint32_t* fill = reinterpret_cast<const uint32_t*>(cache + h->fill_offset) + (int64_t)b * (h->cap / kBqChunk);
    return (uint32_t)(e % kBqChunk) < fill[e / kBqChunk];
}

// The three steps for the threads `tid` of `nthreads` that share cloud b (a whole grid row, or one
// workgroup).
template <bool BY_BLOCK>
__device__ __forceinline__ void group_count(const BqHeader* h, const unsigned char* cache, int b, int32_t* cnt,
                                            int keys, int64_t rows_cap, int64_t tid, int64_t nthreads)
{
    const int64_t E = bq_places(h, cache, b, rows_cap);
    const BqRaw* __restrict__ raw = reinterpret_cast<const BqRaw*>(cache + h->raw_offset) + (int64_t)b * h->cap;
    for (int64_t e = tid; e < E; e += nthreads) {
        if (!bq_place_used(h, cache, b, e)) continue;
        const uint32_t key = BY_BLOCK ? raw[e].blk : raw[e].q;
        if (key < (uint32_t)keys) atomicAdd(cnt + (int64_t)b * keys + key, 1);
    }
}

template <bool BY_BLOCK>
__device__ __forceinline__ void group_scatter(const BqHeader* h, const unsigned char* cache, int b, int32_t* cnt,
                                              const uint32_t* off, int keys, BqEntry* rows, int64_t rows_cap,
                                              int64_t tid, int64_t nthreads)
{
    const int64_t E = bq_places(h, cache, b, rows_cap);
    const BqRaw* __restrict__ raw = reinterpret_cast<const BqRaw*>(cache + h->raw_offset) + (int64_t)b * h->cap;
    BqEntry* __restrict__ out = rows + (int64_t)b * rows_cap;
    for (int64_t e = tid; e < E; e += nthreads) {
        if (!bq_place_used(h, cache, b, e)) continue;
        const BqRaw r = raw[e];
        const uint32_t key = BY_BLOCK ? r.blk : r.q;
        if (key >= (uint32_t)keys) continue;
        const uint32_t first = __hip_atomic_load(off + (int64_t)b * ((int64_t)keys + 1) + key, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t at = first + (uint32_t)atomicAdd(cnt + (int64_t)b * keys + key, 1);
        BqEntry g;
        g.other = BY_BLOCK ? r.q : r.blk;
        g.lo = (uint32_t)r.mask;
        g.hi = (uint32_t)(r.mask >> 32);
        out[at] = g;
    }
}

// off[b][0 .. keys] = exclusive prefix sums of cnt[b][0 .. keys); cnt is set back to zero (the
// scatter pass counts up again).  By the 1024 threads of one workgroup (all of them call): the keys
// are taken 4096 at a time, four consecutive ones per thread (so that the threads of a wave read
// consecutive memory), scanned inside the wave by shuffles and across the 16 waves through LDS.
__device__ __forceinline__ void group_scan(int b, int32_t* cnt, uint32_t* off, int keys, uint32_t* wsum)
{
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    int32_t* c = cnt + (int64_t)b * keys;
    uint32_t* o = off + (int64_t)b * ((int64_t)keys + 1);
    uint32_t carry = 0;
    for (int base = 0; base < keys; base += 4096) {
        const int k0 = base + tid * 4;
        uint32_t v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            v[i] = k0 + i < keys ? (uint32_t)__hip_atomic_load(c + k0 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        const uint32_t mine = v[0] + v[1] + v[2] + v[3];
        uint32_t incl = mine;
#pragma unroll
        for (int sft = 1; sft < 64; sft <<= 1) {
            const uint32_t up = (uint32_t)__shfl_up((int)incl, sft, 64);
            if (lane >= sft) incl += up;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const uint32_t t = wsum[w];
            before += w < wave ? t : 0u;
            total += t;
        }
        uint32_t run = carry + before + incl - mine;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (k0 + i < keys) {
                o[k0 + i] = run;
                __hip_atomic_store(c + k0 + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            run += v[i];
        }
        carry += total;
        __syncthreads();                 // wsum is written again in the next turn
    }
    if (tid == 0) o[keys] = carry;
}

template <bool BY_BLOCK>
__global__ __launch_bounds__(256) void bq_group_count_kernel(const unsigned char* __restrict__ cache,
                                                             int32_t* __restrict__ cnt, int keys, int64_t rows_cap)
{
    const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
    if (h->magic != kBqMagic || (int)blockIdx.y >= h->B) return;
    group_count<BY_BLOCK>(h, cache, (int)blockIdx.y, cnt, keys, rows_cap, (int64_t)blockIdx.x * 256 + threadIdx.x,
                          (int64_t)gridDim.x * 256);
}

__global__ __launch_bounds__(1024) void bq_group_scan_kernel(int32_t* __restrict__ cnt, uint32_t* __restrict__ off,
                                                             int keys)
{
    __shared__ uint32_t wsum[16];
    group_scan((int)blockIdx.x, cnt, off, keys, wsum);
}

template <bool BY_BLOCK>
__global__ __launch_bounds__(256) void bq_group_scatter_kernel(const unsigned char* __restrict__ cache,
                                                               int32_t* __restrict__ cnt,
                                                               const uint32_t* __restrict__ off, int keys,
                                                               BqEntry* __restrict__ rows, int64_t rows_cap)
{
    const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
    if (h->magic != kBqMagic || (int)blockIdx.y >= h->B) return;
    group_scatter<BY_BLOCK>(h, cache, (int)blockIdx.y, cnt, off, keys, rows, rows_cap,
                            (int64_t)blockIdx.x * 256 + threadIdx.x, (int64_t)gridDim.x * 256);
}

// Small clouds: the three steps by one workgroup per cloud in one launch (the counts are zeroed
// here as well).  Counts and offsets go through device-scope atomics, so that what one thread
// wrote before a barrier is what another reads after it.
template <bool BY_BLOCK>
__global__ __launch_bounds__(1024) void bq_group_small_kernel(const unsigned char* __restrict__ cache,
                                                              int32_t* __restrict__ cnt, uint32_t* __restrict__ off,
                                                              int keys, BqEntry* __restrict__ rows, int64_t rows_cap)
{
    __shared__ uint32_t wsum[16];
    const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
    const int b = (int)blockIdx.x;
    const bool ok = h->magic == kBqMagic && b < h->B;
    for (int t = (int)threadIdx.x; t < keys; t += 1024)
        __hip_atomic_store(cnt + (int64_t)b * keys + t, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ok) group_count<BY_BLOCK>(h, cache, b, cnt, keys, rows_cap, threadIdx.x, 1024);
    __syncthreads();
    group_scan(b, cnt, off, keys, wsum);
    __syncthreads();
    if (ok) group_scatter<BY_BLOCK>(h, cache, b, cnt, off, keys, rows, rows_cap, threadIdx.x, 1024);
}

__global__ void zero_ints_kernel(int32_t* p, int64_t n)
{
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (int64_t)gridDim.x * blockDim.x)
        p[t] = 0;
}

__device__ __forceinline__ uint32_t rdlane_u32(uint32_t v, int l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, l);
}

// Ball query from the recorded radius tests (Section 4.2): no distance is evaluated.  One wave per
// centre.  The centre's row holds one entry per point block its ball reaches; the entries are put
// in block order (a rank by counting when there are at most 64, else the smallest block not yet
// taken is looked for k times at most), their set bits are the hits in index order, and the first k
// are written.  A centre the record does not cover (not the recorded sample of that position,
// another radius, a cloud whose list overflowed) is tested against all points by its wave, 64
// points per step in index order.
// hits of a ball that the reader of a cell-ordered record looks at together, and the entries whose
// index reads it issues before using the first
constexpr int kCellBatch = 256;
constexpr int kCellLoads = 8;

__global__ __launch_bounds__(256) void bq_cached_kernel(const float* __restrict__ xyz, int B, int N,
                                                        const int32_t* __restrict__ center_idx, int M,
                                                        float r2, int k, int32_t* __restrict__ out_idx,
                                                        int32_t* __restrict__ out_cnt,
                                                        const unsigned char* __restrict__ cache)
{
    __shared__ uint32_t s_blk[4][64];
    __shared__ uint64_t s_mask[4][64];
    __shared__ int32_t s_out[4][256];
    __shared__ int32_t s_hit[4][kCellBatch];
    const int b = (int)blockIdx.y;
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int q = (int)blockIdx.x * 4 + wave;
    if (q >= M) return;                                     // wave-uniform; the kernel has no barrier
    const float* __restrict__ cloud = xyz + (int64_t)b * N * 3;
    const int c = __builtin_amdgcn_readfirstlane(center_idx[(int64_t)b * M + q]);
    int32_t* __restrict__ row = out_idx + ((int64_t)b * M + q) * k;
    if (c < 0 || c >= N) {                                  // no such centre
        for (int t = lane; t < k; t += 64) row[t] = -1;
        if (lane == 0 && out_cnt) out_cnt[(int64_t)b * M + q] = 0;
        return;
    }
    uint32_t* blk_s = s_blk[wave];
    uint64_t* mask_s = s_mask[wave];
    int32_t* out_s = s_out[wave];

    const BqHeader* h = reinterpret_cast<const BqHeader*>(cache);
    bool usable = h->magic == kBqMagic && h->valid == 1 && h->B == B && h->N == N &&
                  h->r2_bits == __float_as_uint(r2) && q < h->n;
    if (usable) {
        const int32_t* cidx = reinterpret_cast<const int32_t*>(cache + h->idx_offset);
        usable = cidx[(int64_t)b * h->n + q] == c && reinterpret_cast<const uint32_t*>(cache + h->ovf_offset)[b] == 0;
    }
    usable = __builtin_amdgcn_readfirstlane(usable ? 1 : 0) != 0;
    int nh = 0;                                             // hits kept so far (uniform)
    bool done = false;
    if (usable) {
        const uint32_t* off = reinterpret_cast<const uint32_t*>(cache + h->rowoff_offset) +
                              (int64_t)b * ((int64_t)h->n + 1) + q;
        const uint32_t o0 = off[0];
        const int E = __builtin_amdgcn_readfirstlane((int)(off[1] - o0));
        const BqEntry* __restrict__ ent = reinterpret_cast<const BqEntry*>(cache + h->rows_offset) +
                                          (int64_t)b * h->cap + o0;
        done = true;
        if (h->order == 1) {
            // A record of the cell-ordered sampler: a block is 64 consecutive positions of that order
            // and map[] gives the index of the point at a position, so the hits do not come out in
            // index order.  The wave keeps the k lowest indices seen so far (in out_s, ascending); once
            // it has k of them the largest is a bound, and only hits with an index below it are
            // collected (in hit_s).  When hit_s fills, and at the end, the k lowest of kept and
            // collected values are taken one at a time (a point is in the ball once, so the values
            // differ).  Entry by entry the 64 lanes read the indices of the block's 64 positions (one
            // line of memory); the reads of kCellLoads entries are issued together.
            const int32_t* __restrict__ map = reinterpret_cast<const int32_t*>(cache + h->map_offset) + (int64_t)b * N;
            int32_t* hit_s = s_hit[wave];
            int kept = 0, fresh = 0;
            int32_t bound = 0x7FFFFFFF;
            auto take_lowest = [&]() {
                // the same wave reads back what it wrote: the LDS keeps a wave's operations in order
                int32_t v[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[i] = lane + 64 * i < kept ? out_s[lane + 64 * i] : 0x7FFFFFFF;
                    v[4 + i] = lane + 64 * i < fresh ? hit_s[lane + 64 * i] : 0x7FFFFFFF;
                }
                const int want = kept + fresh < k ? kept + fresh : k;
                int32_t mn = 0x7FFFFFFF;
                for (int t = 0; t < want; ++t) {
                    mn = v[0];
#pragma unroll
                    for (int i = 1; i < 8; ++i) mn = min(mn, v[i]);
#pragma unroll
                    for (int sft = 32; sft > 0; sft >>= 1) mn = min(mn, __shfl_xor(mn, sft, 64));
                    mn = __builtin_amdgcn_readfirstlane(mn);
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = v[i] == mn ? 0x7FFFFFFF : v[i];
                    if (lane == 0) out_s[t] = mn;
                }
                kept = want;
                fresh = 0;
                bound = kept == k ? mn : 0x7FFFFFFF;
            };
            for (int e0 = 0; e0 < E; e0 += 64) {
                BqEntry g;
                g.other = 0u;
                g.lo = g.hi = 0u;
                if (e0 + lane < E) g = ent[e0 + lane];
                const int ne = E - e0 < 64 ? E - e0 : 64;
                for (int e = 0; e < ne; e += kCellLoads) {
                    int32_t at[kCellLoads];
#pragma unroll
                    for (int u = 0; u < kCellLoads; ++u) {
                        const int eu = e + u < ne ? e + u : ne - 1;         // wave-uniform
                        const int64_t pos = ((int64_t)rdlane_u32(g.other, eu) << 6) + lane;
                        at[u] = pos < N ? map[pos] : 0x7FFFFFFF;
                    }
#pragma unroll
                    for (int u = 0; u < kCellLoads; ++u) {
                        if (e + u < ne) {                                   // wave-uniform
                            const uint64_t em = ((uint64_t)rdlane_u32(g.hi, e + u) << 32) | rdlane_u32(g.lo, e + u);
                            const bool hit = ((em >> lane) & 1ull) != 0 && at[u] < bound;
                            const uint64_t bm = __builtin_amdgcn_ballot_w64(hit);
                            if (bm != 0) {
                                if (hit) hit_s[fresh + lanes_below(bm)] = at[u];
                                fresh += __builtin_popcountll(bm);
                                if (fresh > kCellBatch - 64) take_lowest();
                            }
                        }
                    }
                }
            }
            if (fresh > 0) take_lowest();
            nh = kept;
        } else if (E <= 64) {
            BqEntry me;
            me.other = 0xFFFFFFFFu;
            me.lo = me.hi = 0u;
            if (lane < E) me = ent[lane];
            int rank = 0;
            for (int j = 0; j < E; ++j) rank += rdlane_u32(me.other, j) < me.other ? 1 : 0;
            if (lane < E) {
                blk_s[rank] = me.other;
                mask_s[rank] = ((uint64_t)me.hi << 32) | me.lo;
            }
            // the same wave reads back what it wrote: the LDS keeps a wave's operations in order
            const uint32_t bk = lane < E ? blk_s[lane] : 0u;
            uint64_t m = lane < E ? mask_s[lane] : 0ull;
            const int pc = __builtin_popcountll(m);
            int incl = pc;
#pragma unroll
            for (int sft = 1; sft < 64; sft <<= 1) {
                const int up = __shfl_up(incl, sft, 64);
                if (lane >= sft) incl += up;
            }
            const int total = __builtin_amdgcn_readlane(incl, 63);
            int pos = incl - pc;
            while (m != 0 && pos < k) {
                out_s[pos] = (int32_t)((bk << 6) + (uint32_t)__builtin_ctzll(m));
                ++pos;
                m &= m - 1;
            }
            nh = total < k ? total : k;
        } else {
            int64_t last = -1;
            while (nh < k) {
                uint32_t best = 0xFFFFFFFFu;
                uint64_t bm = 0;
                for (int e0 = 0; e0 < E; e0 += 64) {
                    if (e0 + lane < E) {
                        const BqEntry g = ent[e0 + lane];
                        if ((int64_t)g.other > last && g.other < best) {
                            best = g.other;
                            bm = ((uint64_t)g.hi << 32) | g.lo;
                        }
                    }
                }
                uint32_t wmin = best;
#pragma unroll
                for (int sft = 32; sft > 0; sft >>= 1) wmin = min(wmin, (uint32_t)__shfl_xor((int)wmin, sft, 64));
                wmin = (uint32_t)__builtin_amdgcn_readfirstlane((int)wmin);
                if (wmin == 0xFFFFFFFFu) break;             // every block is taken
                const int src = __builtin_ctzll(__builtin_amdgcn_ballot_w64(best == wmin));   // blocks are distinct
                const uint64_t m = ((uint64_t)rdlane_u32((uint32_t)(bm >> 32), src) << 32) |
                                   rdlane_u32((uint32_t)bm, src);
                const bool hit = (m >> lane) & 1ull;
                const int pos = nh + lanes_below(m);
                if (hit && pos < k) out_s[pos] = (int32_t)((wmin << 6) + (uint32_t)lane);
                nh += __builtin_popcountll(m);
                last = (int64_t)wmin;
            }
            nh = nh < k ? nh : k;
        }
    }
    if (!done) {
        const float cx = cloud[(int64_t)c * 3 + 0], cy = cloud[(int64_t)c * 3 + 1], cz = cloud[(int64_t)c * 3 + 2];
        nh = 0;
        for (int j0 = 0; j0 < N && nh < k; j0 += 64) {
            const int j = j0 + lane;
            bool hit = false;
            if (j < N) {
                const float* pj = cloud + (int64_t)j * 3;
                hit = dist2(cx, cy, cz, pj[0], pj[1], pj[2]) < r2;
            }
            const uint64_t m = __builtin_amdgcn_ballot_w64(hit);
            const int pos = nh + lanes_below(m);
            if (hit && pos < k) out_s[pos] = j;
            nh += __builtin_popcountll(m);
        }
        nh = nh < k ? nh : k;
    }
    const int first = nh > 0 ? out_s[0] : -1;
    for (int t = lane; t < k; t += 64) row[t] = t < nh ? out_s[t] : first;
    if (lane == 0 && out_cnt) out_cnt[(int64_t)b * M + q] = nh;
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
        if (k > 254) return hipErrorInvalidValue;
        const unsigned char* cache = reinterpret_cast<const unsigned char*>(bq_cache);
        hipLaunchKernelGGL(bq_cached_kernel, dim3((unsigned)((M + 3) / 4), (unsigned)B), dim3(256), 0, stream, xyz,
                           B, N, center_idx, M, r2, k, out_idx, out_cnt, cache);
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

namespace {
// up to this size the grouping is one launch with one workgroup per cloud
constexpr int64_t kGroupSmallEntries = 160 * 1024;
constexpr int kGroupSmallKeys = 16 * 1024;

template <bool BY_BLOCK>
hipError_t group_entries(const unsigned char* cache, int B, int32_t* cnt, uint32_t* off, BqEntry* rows,
                         int64_t rows_cap, int keys, hipStream_t stream)
{
    if (rows_cap <= kGroupSmallEntries && keys <= kGroupSmallKeys) {
        hipLaunchKernelGGL((bq_group_small_kernel<BY_BLOCK>), dim3((unsigned)B), dim3(1024), 0, stream, cache, cnt,
                           off, keys, rows, rows_cap);
        return hipGetLastError();
    }
    int64_t gx = (rows_cap + 2047) / 2048;                // eight entries per thread when the list is full
    if (gx > 8192) gx = 8192;
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, (unsigned)B);
    {
        const int64_t words = (int64_t)B * keys;
        int zb = (int)((words + 255) / 256);
        if (zb > 1024) zb = 1024;
        hipLaunchKernelGGL(zero_ints_kernel, dim3((unsigned)zb), dim3(256), 0, stream, cnt, words);
    }
    hipLaunchKernelGGL((bq_group_count_kernel<BY_BLOCK>), grid, dim3(256), 0, stream, cache, cnt, keys, rows_cap);
    hipLaunchKernelGGL(bq_group_scan_kernel, dim3((unsigned)B), dim3(1024), 0, stream, cnt, off, keys);
    hipLaunchKernelGGL((bq_group_scatter_kernel<BY_BLOCK>), grid, dim3(256), 0, stream, cache, cnt,
                       (const uint32_t*)off, keys, rows, rows_cap);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_bq_group_by_sample(void* bq_cache, int B, int N, int n, int64_t cap, hipStream_t stream)
{
    unsigned char* cache = reinterpret_cast<unsigned char*>(bq_cache);
    const BqHeader lay = bq_layout(B, N, n, 1.0f, cap);
    return group_entries<false>(cache, B, reinterpret_cast<int32_t*>(cache + lay.rowcnt_offset),
                                reinterpret_cast<uint32_t*>(cache + lay.rowoff_offset),
                                reinterpret_cast<BqEntry*>(cache + lay.rows_offset), lay.cap, n, stream);
}

hipError_t launch_bq_group_by_block(const void* bq_cache, int B, int N, int32_t* cnt, uint32_t* off,
                                    BqEntry* rows, int64_t rows_cap, hipStream_t stream)
{
    const int blocks = (int)(((int64_t)N + 63) / 64);
    return group_entries<true>(reinterpret_cast<const unsigned char*>(bq_cache), B, cnt, off, rows, rows_cap,
                               blocks, stream);
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
