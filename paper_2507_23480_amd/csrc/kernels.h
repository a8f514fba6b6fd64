// Internal declarations shared by the HIP translation units of the library.
#ifndef FASTPOINT_KERNELS_H_
#define FASTPOINT_KERNELS_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastpoint.h"

namespace fastpoint {

constexpr int kMaxGroup = 256;          // most workgroups one cloud is spread over
constexpr int kLlSlotWords = 8;         // 64-bit words per workgroup slot of the pick exchange
constexpr int kCandPerRound = 64;       // candidates per round of exact FPS (one per lane of the control wave)
constexpr int kCandMax = 128;           // candidates per round of the threshold phase (two per lane)
constexpr int kCandWin = 256;           // candidates per round of the threshold phase, cell-ordered variant
constexpr int kCandWords = 5;           // exchanged 64-bit words per candidate (x, y, z, index, distance)
constexpr uint32_t kBqMagic = 0x46504232u;

// Ball-query cache (device memory): the radius tests of Section 4.2 that found a point, and only
// those.  While a sample is folded into the running distances every wave of the sampler compares
// its points with the ball-query radius as well; a 64-bit word of such tests (one block of 64
// consecutive points against one sample) that is not zero becomes one entry of a flat list per
// cloud.  After the sampler a small pass puts the entries in sample order (rows in compressed-row
// form), which is what the ball query reads; the k-NN search regroups them by point block.
constexpr int kBqChunk = 64;        // entries a wave of the sampler reserves at a time
constexpr uint32_t kBqNoChunk = 0xFFFFFFFFu;
struct BqRaw {              // as appended by the sampler
    uint64_t mask;          // bit l: point 64 * blk + l lies inside the ball of sample q
    uint32_t blk;           // point block
    uint32_t q;             // sample position
};
struct BqEntry {            // after grouping: the key (sample or block) is the row
    uint32_t other;         // point block (rows by sample) or sample position (rows by block)
    uint32_t lo, hi;        // the 64 tests
};
struct BqHeader {
    uint32_t magic;
    int32_t B, N, n;
    int32_t blocks;         // point blocks per cloud, ceil(N / 64)
    int32_t valid;          // 1 once the header is complete
    uint32_t r2_bits;       // radius^2 (binary32 bits) the tests were recorded with
    int32_t order;          // 0: a block is 64 consecutive indices; 1: 64 consecutive positions of the
                            // sampler's cell order, map[] gives the index at a position
    int64_t cap;            // entries a cloud's lists hold, a multiple of kBqChunk
    int64_t idx_offset;     // byte offset of the int32 [B][n] copy of the sample indices
    int64_t cursor_offset;  // uint32 [B]: chunks of kBqChunk entries handed out to the sampler's waves
    int64_t ovf_offset;     // uint32 [B]: not 0 when a wave found no chunk left (entries were dropped)
    int64_t rowcnt_offset;  // int32 [B][n]: entries of each sample
    int64_t fill_offset;    // uint32 [B][cap / kBqChunk]: entries in use in each chunk
    int64_t rowoff_offset;  // uint32 [B][n + 1]: first entry of each sample's row
    int64_t raw_offset;     // BqRaw [B][cap]
    int64_t rows_offset;    // BqEntry [B][cap], in sample order
    int64_t map_offset;     // int32 [B][N]: index of the point at each position (order 1 only)
    int64_t bytes;
};

__host__ __device__ inline int64_t bq_align(int64_t v) { return (v + 255) / 256 * 256; }
// entries per cloud the lists are sized for unless the caller says otherwise: two per point and
// sixteen per sample
__host__ __device__ inline int64_t bq_capacity(int32_t N, int32_t n) { return 2 * (int64_t)N + 16 * (int64_t)n; }
__host__ __device__ inline BqHeader bq_layout(int32_t B, int32_t N, int32_t n, float r2, int64_t cap, int32_t order = 0)
{
    BqHeader h;
    h.magic = kBqMagic;
    h.B = B;
    h.N = N;
    h.n = n;
    h.blocks = (int32_t)(((int64_t)N + 63) / 64);
    h.valid = 1;
    union { float f; uint32_t u; } cv;
    cv.f = r2;
    h.r2_bits = cv.u;
    h.order = order;
    h.cap = cap / kBqChunk * kBqChunk;
    h.idx_offset = 256;
    // cursor, overflow flags, row counts and chunk fills are one range, zeroed before the sampler runs
    h.cursor_offset = h.idx_offset + bq_align((int64_t)B * n * 4);
    h.ovf_offset = h.cursor_offset + bq_align((int64_t)B * 4);
    h.rowcnt_offset = h.ovf_offset + bq_align((int64_t)B * 4);
    h.fill_offset = h.rowcnt_offset + bq_align((int64_t)B * n * 4);
    h.rowoff_offset = h.fill_offset + bq_align((int64_t)B * (h.cap / kBqChunk) * 4);
    h.raw_offset = h.rowoff_offset + bq_align((int64_t)B * ((int64_t)n + 1) * 4);
    h.rows_offset = h.raw_offset + bq_align((int64_t)B * h.cap * (int64_t)sizeof(BqRaw));
    h.map_offset = h.rows_offset + bq_align((int64_t)B * h.cap * (int64_t)sizeof(BqEntry));
    h.bytes = h.map_offset + bq_align((int64_t)B * N * 4);
    return h;
}

struct SamplerArgs {
    const float* xyz;
    const int32_t* start_idx;
    int32_t* out_idx;
    float* out_mdc;
    fp_mdps_info* info;
    int32_t B, N, n, G;
    int32_t m;                      // exact FPS iterations before the threshold phase (n-1: all)
    int32_t nseg, fit_window, use_override;
    double exponent, bias2;
    float thr_override[FP_MAX_SEG];
    float level_scale[FP_MAX_SEG];
    unsigned char* bq_base;         // ball-query cache (NULL: nothing is recorded) ...
    int32_t* bq_idx;                // ... its copy of the sample indices [B][n]
    int32_t* bq_map;                // ... cell-ordered sampler: [B][N] index of the point at each position
    BqRaw* bq_raw;                  // ... entries [B][bq_cap], in chunks of kBqChunk
    uint32_t* bq_cursor;            // ... chunks handed out per cloud [B]
    uint32_t* bq_ovf;               // ... overflow flag per cloud [B]
    uint32_t* bq_fill;              // ... entries in use per chunk [B][bq_cap / kBqChunk]
    int64_t bq_cap;
    float bq_r2;
    int32_t bq_blocks;
    uint64_t* ll_pk;                // [groups][2][G][kLlSlotWords]
    uint64_t* ll_cd;                // [groups][2][G][kCandMax][kCandWords]
    uint64_t* ll_ct;                // [groups][2][G] candidate counts of a scan
#ifdef FASTPOINT_PHASE_CLOCKS
    long long* dbg;                 // tuning builds: [G][16] clock sums of every workgroup of the last cloud
#endif
    uint64_t* ll_rel;               // cell-ordered variant: [groups][2][kCandWin][16] relation words of a window round
    int64_t wait_ticks;
    const float* mlp;               // weights of the MLP curve estimator, or NULL (power function)
    const float4* sorted;           // cell-ordered variant: [B][N] records (x, y, z, index bits), else NULL
    uint64_t walk_inv;              // scattered scan order on cell-ordered records: 1/A mod N (place t of index j = j/A mod N)
};

struct Plan {
    int G, T, P;        // workgroups per cloud, threads per workgroup, points per thread
    int groups;         // clouds resident at once
};

// mode 0: exact FPS only; 1: MDPS, threshold rounds of kCandPerRound candidates; 2: MDPS, rounds of
// kCandMax candidates.  NULL for a combination that is not built.
const void* sampler_kernel_for(int threads, int points_per_thread, bool bq, bool perm, int mode);
// zeroes two ranges of 64-bit words (either may be empty)
hipError_t launch_zero_words(uint64_t* p, int64_t nwords, uint64_t* p2, int64_t nwords2, uint64_t* p3,
                             int64_t nwords3, hipStream_t stream);
// Scattered scan order of the threshold phase: writes the records (x, y, z, index bits) of every
// cloud in the order of the walk j_t = (t stride) mod N into out[B][N]; stride coprime to N.
hipError_t launch_scan_walk(const float* xyz, int B, int N, int64_t stride, float4* out, hipStream_t stream);
// puts the entries the sampler appended to a cache of `cap` entries per cloud into sample order
// (rows in compressed-row form)
hipError_t launch_bq_group_by_sample(void* bq_cache, int B, int N, int n, int64_t cap, hipStream_t stream);
// the same entries by point block, in caller memory: cnt int32 [B][blocks], off uint32 [B][blocks + 1],
// rows BqEntry [B][rows_cap]; clouds with more entries than rows_cap are left out (the caller does
// not read their rows); `cnt` ends up holding the row sizes
hipError_t launch_bq_group_by_block(const void* bq_cache, int B, int N, int32_t* cnt, uint32_t* off,
                                    BqEntry* rows, int64_t rows_cap, hipStream_t stream);

hipError_t launch_probe_fp32(int blocks, int iterations, float* out, hipStream_t stream);
hipError_t launch_ball_query(const float* xyz, int B, int N, const int32_t* center_idx, int M,
                             float r2, int k, int32_t* out_idx, int32_t* out_cnt,
                             const void* bq_cache, hipStream_t stream);
hipError_t launch_gather(const float* xyz, int B, int N, const int32_t* idx, int M, float* out,
                         hipStream_t stream);
hipError_t launch_coverage(const float* xyz, int B, int N, const float* sxyz, int n, float* out,
                           hipStream_t stream);
hipError_t launch_knn(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                      int32_t* out_pos, float* out_d2, const void* bq_cache, int32_t* flags,
                      int32_t* count, int32_t* list, int32_t* blk_cnt, uint32_t* blk_off, BqEntry* blk_rows,
                      int64_t blk_rows_cap, int32_t* out_deferred, hipStream_t stream);

// Uniform grid of one cloud for the exclusion-list kernels (device memory, in the workspace).
struct ExclGrid {
    uint32_t lo[3], hi[3];   // bounding box as order-preserving integers (filled by atomics)
    float origin[3];         // lower corner
    float inv_h;             // 1 / cell width
    int32_t dim[3];          // cells per axis
    int32_t ncells;
    float rmax2;             // largest squared radius of the cloud
    int32_t lmax;            // its level
    int32_t curve_bits;      // 0: cells numbered x-fastest; b > 0: 2^b cells per axis, numbered along
                             // a Hilbert curve
};

// Where the parts of an exclusion-list workspace lie (byte offsets).
struct ExclLayout {
    int maxcells;            // cells a cloud's grid may have
    int64_t grid_off, cnt_off, start_off, sorted_off, totals_off, tiles_off, bytes;
};

ExclLayout excl_layout(int B, int N, int L);
// Sorts every cloud into the order of a 2^b x 2^b x 2^b grid over its bounding box, cells
// numbered along a Hilbert curve; leaves records (x, y, z, index bits) at spatial_sorted().
hipError_t launch_spatial_sort(const float* xyz, int B, int N, void* workspace, hipStream_t stream);
int64_t spatial_sort_bytes(int B, int N);
const float4* spatial_sorted(int B, int N, const void* workspace);
hipError_t launch_excl_count(const float* xyz, int B, int N, const float* thr2, int L, int64_t* offsets,
                             void* workspace, hipStream_t stream);
hipError_t launch_excl_fill(const float* xyz, int B, int N, const float* thr2, int L, const int64_t* offsets,
                            int32_t* entries, int64_t capacity, void* workspace, hipStream_t stream);
hipError_t launch_knn_deferred(const float* xyz, int B, int N, const int32_t* sample_idx, int n, int k,
                               int32_t* out_pos, float* out_d2, int32_t* count, int32_t* list,
                               int32_t* out_deferred, hipStream_t stream);
hipError_t launch_knn_grid(const float* xyz, int B, int N, const float* sample_xyz, int n, int k, float r2,
                           int32_t* out_pos, float* out_d2, int32_t* count, int32_t* list, void* grid_ws,
                           hipStream_t stream);
hipError_t launch_bq_grid(const float* xyz, int B, int N, const int32_t* center_idx, int M, float r2, int k,
                          int32_t* out_idx, int32_t* out_cnt, void* workspace, hipStream_t stream);
hipError_t launch_bq_lists(const int64_t* offsets, const int32_t* entries, int B, int N, int level,
                           const int32_t* center_idx, int M, int k, int32_t* out_idx, int32_t* out_cnt,
                           hipStream_t stream);

}  // namespace fastpoint
#endif
