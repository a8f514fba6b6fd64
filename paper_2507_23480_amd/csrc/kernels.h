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
constexpr int kCandWords = 5;           // exchanged 64-bit words per candidate (x, y, z, index, distance)
constexpr uint32_t kBqMagic = 0x46504251u;

// Header at the start of a ball-query cache (device memory).  The radius tests are kept as a
// bit matrix per cloud, one 64-bit word per (block of 64 points, sample): word [w][q] holds, in
// bit l, whether point 64*w + l lies inside the ball of sample q.  Words of one point block are
// contiguous over the samples, so a wave of the sampler writes the words of up to 64 picks with
// one store, a ball-query wave reads the words of 64 consecutive centres with one load, and a
// k-NN wave streams the samples of its point block.
struct BqHeader {
    uint32_t magic;
    int32_t B, N, n;
    int32_t blocks;         // point blocks per cloud, ceil(N / 64)
    int32_t reserved;
    int64_t col_words;      // 64-bit words per point block (n rounded up to a multiple of 8)
    uint32_t r2_bits;       // radius^2 (binary32 bits) the tests were recorded with
    int32_t valid;          // 1 once the header is complete
    int64_t idx_offset;     // byte offset of the int32 [B][n] copy of the sample indices
    int64_t bits_offset;    // byte offset of the uint64 [B][blocks][col_words] words
};

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
    uint64_t* bq_bits;
    int32_t* bq_idx;
    float bq_r2;
    int32_t bq_blocks;
    int64_t bq_col_words;
    uint64_t* ll_pk;                // [groups][2][G][kLlSlotWords]
    uint64_t* ll_cd;                // [groups][2][G][kCandMax][kCandWords]
    int64_t wait_ticks;
    const float* mlp;               // weights of the MLP curve estimator, or NULL (power function)
    const float4* sorted;           // cell-ordered variant: [B][N] records (x, y, z, index bits), else NULL
};

struct Plan {
    int G, T, P;        // workgroups per cloud, threads per workgroup, points per thread
    int groups;         // clouds resident at once
};

// mode 0: exact FPS only; 1: MDPS, threshold rounds of kCandPerRound candidates; 2: MDPS, rounds of
// kCandMax candidates.  NULL for a combination that is not built.
const void* sampler_kernel_for(int threads, int points_per_thread, bool bq, bool perm, int mode);
hipError_t launch_zero_words(uint64_t* p, int64_t nwords, hipStream_t stream);

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
                      int32_t* count, int32_t* list, int32_t* out_deferred, hipStream_t stream);

// Uniform grid of one cloud for the exclusion-list kernels (device memory, in the workspace).
struct ExclGrid {
    uint32_t lo[3], hi[3];   // bounding box as order-preserving integers (filled by atomics)
    float origin[3];         // lower corner
    float inv_h;             // 1 / cell width
    int32_t dim[3];          // cells per axis
    int32_t ncells;
    float rmax2;             // largest squared radius of the cloud
    int32_t lmax;            // its level
    int32_t morton_bits;     // 0: cells numbered x-fastest; b > 0: 2^b cells per axis, numbered by
                             // interleaving the bits of the three coordinates
};

// Where the parts of an exclusion-list workspace lie (byte offsets).
struct ExclLayout {
    int maxcells;            // cells a cloud's grid may have
    int64_t grid_off, cnt_off, start_off, sorted_off, totals_off, bytes;
};

ExclLayout excl_layout(int B, int N, int L);
// Sorts every cloud into the order of a 2^b x 2^b x 2^b grid over its bounding box, cells
// numbered along a Z-order curve; leaves records (x, y, z, index bits) at spatial_sorted().
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
