/*
 * fastpoint.h -- C ABI of the MI355X (gfx950) library for farthest point
 * sampling, minimum-distance-prediction sampling (MDPS) and ball query
 * (FastPoint, arXiv 2507.23480).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller (contiguous,
 *     row-major), unless a parameter says "host".  The library never frees or
 *     keeps them and allocates no device memory itself: scratch comes from the
 *     caller's workspace (fp_workspace_bytes) and the optional ball-query cache
 *     (fp_bq_cache_bytes).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.
 *   - Arguments are validated on the host before anything is enqueued; a
 *     negative status means nothing was launched.
 *   - Arithmetic: squared Euclidean distance in IEEE binary32 evaluated as
 *     ((dx*dx)+(dy*dy))+(dz*dz), each operation rounded separately (no FMA);
 *     argmax and "any available point" resolve to the lowest index.  Index
 *     results are therefore reproducible bit for bit.
 *   - Inputs must be finite with |coordinate| < 1e18.
 *   - Calls that share a workspace or a cache must not overlap in time.
 *   - No global state: apart from the test and measurement hooks at the end of this
 *     header nothing persists between calls, and calls with distinct workspaces may run
 *     concurrently (other streams, other host threads).
 */
#ifndef FASTPOINT_H_
#define FASTPOINT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t fp_status;
enum {
    FP_OK = 0,
    FP_ERR_NULL = -1,      /* a required pointer is NULL                         */
    FP_ERR_SHAPE = -2,     /* B, N, n, M or k out of range / cloud too large     */
    FP_ERR_PARAM = -3,     /* radius or an MDPS parameter out of range           */
    FP_ERR_WORKSPACE = -4, /* workspace or cache missing, misaligned or too small */
    FP_ERR_DEVICE = -5,    /* a HIP runtime call failed                          */
    FP_ERR_CAPACITY = -6   /* beyond what the library's static scratch buffer holds */
};

#define FP_MAX_SEG 16
#define FP_KNN_MAX_K 8

/* MDPS hyper-parameters (Section 4.1; Appendix A.3 for the estimator). Host struct. */
typedef struct fp_mdps_params {
    float   p;            /* ratio of exact FPS iterations run first (paper: 0.1), 0 < p < 1   */
    int32_t nseg;         /* segments of the distance curve (paper default 6), 1..FP_MAX_SEG   */
    double  exponent;     /* e of the power-function estimator C(x) = a / x^e, in squared-
                             distance space, x = sample position; fitted offline per workload */
    float   bias;         /* factor on the predicted DISTANCE (bias^2 on the squared value), > 0 */
    int32_t fit_window;   /* trailing prefix points that determine a (1..64)                   */
    int32_t m_min;        /* lower limit of the prefix length                                  */
    int32_t use_override; /* nonzero: skip the estimator, use thr_override                     */
    float   thr_override[FP_MAX_SEG]; /* squared thresholds R_l^2, l = 1..nseg, non-increasing */
    float   level_scale[FP_MAX_SEG];  /* offline per-segment correction multiplying the predicted
                                         SQUARED value of segment l (> 0; 1 = pure power function) */
    const float* mlp_weights; /* NULL: power-function estimator.  Else a DEVICE pointer to the
                                 FP_MLP_WEIGHTS binary32 weights of the MLP estimator of Appendix
                                 A.3, a perceptron 32-128-128-64 with ReLU after the two hidden
                                 layers, input-major: W1[32][128] b1[128] W2[128][128] b2[128]
                                 W3[128][64] b3[64].  Input k = ln(curve[i_k] / curve[m]) with
                                 i_k = max(1, floor(m (k+1) / 32)); output j = ln(curve(x_j) /
                                 curve[m]) at x_j = m + (n-1-m)(j+1)/64, interpolated linearly
                                 between the x_j; binary64 arithmetic in a fixed order, so the
                                 thresholds are reproducible bit for bit.  exponent and fit_window
                                 are then unused; bias and level_scale still apply. */
    int32_t scan_order;   /* which available point the threshold phase takes next (Section 4.1
                             step 3 leaves it open: any available point).  0: the lowest index.
                             1: the first available point of the walk j_t = (t A) mod N,
                             t = 0, 1, ..., where A is the smallest integer >= max(1, floor(
                             0.6180339887498949 N)) that is coprime to N -- successive points of
                             the walk lie far apart in index, so a cloud stored in scanner order
                             is visited like a shuffled one and more picks of a round survive.
                             The exact-FPS parts are not affected.  With order 1 fp_mdps_sample
                             needs the larger workspace of fp_mdps_scattered_workspace_bytes and
                             does not record (bq_cache must be NULL; FP_ERR_PARAM otherwise);
                             fp_mdps_sample_pruned takes either order. */
    int32_t reserved0;    /* 0 */
} fp_mdps_params;

#define FP_MLP_WEIGHTS (32 * 128 + 128 + 128 * 128 + 128 + 128 * 64 + 64)

/* Per-cloud record written by the sampler kernels (device memory, [B], optional). */
typedef struct fp_mdps_info {
    int32_t m;                          /* exact FPS iterations run first                         */
    int32_t et_index;                   /* first sample position filled by the remainder FPS
                                           (early termination, Section 4.1 step 4); n if none     */
    int32_t level_start[FP_MAX_SEG];    /* sample position at which level l+1 became current, or -1 */
    int32_t level_exhausted[FP_MAX_SEG];/* 1 if level l+1 ran out of available points             */
    float   thr2[FP_MAX_SEG];           /* squared thresholds used                                */
    int32_t rounds;                     /* candidate rounds of the threshold phase                */
    int32_t status;                     /* 0 ok; 1 start index out of range; 2 a bounded wait
                                           between workgroups expired (output invalid)            */
    int32_t phase_ticks[4];             /* time the cloud spent in the four phases of Section 4.1,
                                           in 10 ns ticks of the device's constant clock: exact FPS
                                           iterations run first (all of them for fp_fps_exact),
                                           estimator and thresholds, threshold-guided sampling,
                                           exact FPS after early termination                      */
} fp_mdps_info;

/* Bytes of workspace fp_fps_exact / fp_mdps_sample need for B clouds of N points
 * (0 is returned for shapes the library rejects). Alignment: 256 bytes. */
size_t fp_workspace_bytes(int32_t B, int32_t N);

/* Bytes of the ball-query cache for B clouds of N points and n samples each.
 * The cache stores the radius tests that found a point -- the extra exclusion list at the
 * ball-query radius of Section 4.2 -- as entries (sample, block of 64 points, 64 test bits),
 * only for blocks a ball reaches, first as the sampler produces them and then in sample order.
 * entries_per_cloud is the caller's choice, <= 0 for the default of 2 N + 16 n (two lists of
 * 16 and 12 bytes per entry, plus 4 bytes per point: 90 MB for 10^6 points and 65 536 samples).  A ball holding h
 * points needs at most h entries, and about h / 10 when neighbours in space are neighbours in
 * the index order (scanner-ordered clouds); the sampler's wavefronts reserve entries 64 at a
 * time, which can leave up to N + 128 of them unused.  A cloud whose balls reach more blocks than the
 * cache holds is recorded incompletely and says so: readers then treat its centres like centres
 * that were never recorded (brute force), so results do not change.  Alignment: 256 bytes.
 * fp_bq_cache_entries: the entries per cloud that a buffer of `bytes` bytes holds (0: too small). */
size_t fp_bq_cache_bytes(int32_t B, int32_t N, int32_t n, int64_t entries_per_cloud);
int64_t fp_bq_cache_entries(size_t bytes, int32_t B, int32_t N, int32_t n);

/*
 * Exact farthest point sampling, Algorithm 1 (Section 3.3).
 *   xyz        [B][N][3] float32
 *   start_idx  [B] int32 seed index per cloud, or NULL for 0
 *   out_idx    [B][n] int32; out_idx[b][0] = seed
 *   out_mdc    [B][n] float32 or NULL: squared min-distance of each pick at pick
 *              time (the minimum distance curve of Section 4; +inf for the seed)
 *   info       [B] or NULL (only m, et_index = n and status are meaningful)
 *   bq_cache   NULL, or a buffer of bq_cache_bytes bytes (fp_bq_cache_bytes) that receives
 *              the radius tests of the (sample, point) pairs, those that found a point, as
 *              a by-product of the distance updates (Section 4.2); bq_radius is then
 *              required > 0
 * A seed index outside [0,N) makes that cloud's out_idx all -1 (info.status 1).
 */
fp_status fp_fps_exact(const float* xyz, int32_t B, int32_t N, int32_t n,
                       const int32_t* start_idx, int32_t* out_idx, float* out_mdc,
                       fp_mdps_info* info, void* bq_cache, size_t bq_cache_bytes, float bq_radius,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * fp_fps_exact for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same kernels and the same result as
 * fp_fps_exact without a cache and without an info record, but the words the workgroups of a
 * cloud exchange live in a device array that is part of the library (2 658 304 bytes, held by
 * every GPU the library runs on until the process ends) instead of a caller's workspace.  The
 * call allocates nothing, on the device or through any library; the first call on a device
 * looks that device's copy of the array up (no allocation either), so make one call before a
 * capture starts.  The caller still passes inputs and outputs (device memory, as above).
 *   Limit: N <= FP_STATIC_MAX_POINTS points per cloud (what the array's exchange slots serve);
 *   a larger N returns FP_ERR_CAPACITY and nothing is enqueued.
 *   All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (other
 *   streams, other threads) race and give wrong results; calls in stream order are fine, the
 *   words are cleared by a kernel at the start of every call.
 */
#define FP_STATIC_MAX_POINTS 2097152
fp_status fp_fps_exact_static(const float* xyz, int32_t B, int32_t N, int32_t n,
                              const int32_t* start_idx, int32_t* out_idx, float* out_mdc,
                              void* stream);

/*
 * Exact farthest point sampling with pruned distance updates -- the same result as
 * fp_fps_exact, bit for bit, reached with fewer distance evaluations (the role QuickFPS plays
 * for the exact iterations in Section 5.3 and Appendix B.3: an exact sampler that skips the
 * updates that cannot change anything).  The cloud is first put into the order of a uniform
 * grid traversed along a Hilbert curve, so that the points a wavefront holds lie in a small
 * box; a new sample is folded into a wavefront's distances only if it is closer to that box
 * than the largest distance the wavefront still holds.  Arguments as fp_fps_exact without the
 * ball-query cache; the workspace is larger (it also receives the reordered cloud).
 */
size_t fp_fps_pruned_workspace_bytes(int32_t B, int32_t N);
fp_status fp_fps_exact_pruned(const float* xyz, int32_t B, int32_t N, int32_t n,
                              const int32_t* start_idx, int32_t* out_idx, float* out_mdc,
                              fp_mdps_info* info, void* workspace, size_t workspace_bytes,
                              void* stream);

/*
 * Minimum Distance Prediction Sampling, Algorithm 2 (Section 4.1, Appendix A.1):
 * m = max(floor(p*n), m_min) exact FPS iterations that record the distance
 * curve, thresholds R_l from the estimated curve at the segment ends,
 * threshold-guided picks (next available point in prm->scan_order; level advances on quota or
 * on exhaustion), and exact FPS for whatever remains once the last level is
 * exhausted.  If m >= n-1 the call is exact FPS.  Arguments as fp_fps_exact;
 * prm is a HOST pointer.
 * With prm->scan_order = 1 (see fp_mdps_params) the workspace must hold
 * fp_mdps_scattered_workspace_bytes(B, N) bytes: it also receives a copy of the cloud in the
 * order of the walk (16 bytes per point), which is what the kernel then works on.
 */
size_t fp_mdps_scattered_workspace_bytes(int32_t B, int32_t N);
fp_status fp_mdps_sample(const float* xyz, int32_t B, int32_t N, int32_t n,
                         const int32_t* start_idx, const fp_mdps_params* prm,
                         int32_t* out_idx, fp_mdps_info* info,
                         void* bq_cache, size_t bq_cache_bytes, float bq_radius,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Minimum Distance Prediction Sampling with pruned distance updates -- the same result as
 * fp_mdps_sample, bit for bit: Algorithm 2 on the cell-ordered copy of the cloud that
 * fp_fps_exact_pruned works on, so that the exact iterations (prefix and remainder) and the
 * threshold-guided picks are folded only into the wavefronts they can affect.  The points are
 * no longer held in index order, so the next available points in the scan order (by index, or by
 * place in the walk of prm->scan_order = 1) are found through a sliding window of that key: a
 * round takes all available points of the window, up to 256, and settles which of them the
 * rule of Section 4.1 step 3 would accept one after the other from the pairwise "closer than
 * R_l" relation between them.  Arguments as fp_mdps_sample; workspace of
 * fp_fps_pruned_workspace_bytes(B, N) bytes.  With a bq_cache the radius tests are recorded as
 * by fp_mdps_sample (a sample is then also folded into every wavefront its ball can reach); the
 * blocks of such a record are 64 consecutive positions of the cell order and the record carries the
 * index at every position: fp_ball_query reads it like any other record (same result), fp_knn
 * does not use it (it searches all points by brute force, same result).
 */
fp_status fp_mdps_sample_pruned(const float* xyz, int32_t B, int32_t N, int32_t n,
                                const int32_t* start_idx, const fp_mdps_params* prm,
                                int32_t* out_idx, fp_mdps_info* info,
                                void* bq_cache, size_t bq_cache_bytes, float bq_radius,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Ball query (Section 3.1 step 2): for centre q of cloud b (a point of that
 * cloud, center_idx[b][q]) the indices j with dist^2(centre, P[j]) < radius^2
 * (strict, binary32), ascending, first k kept; unused slots repeat the first
 * hit; out_cnt = min(hits, k).  1 <= k <= 254.
 *   center_idx [B][M] int32, out_idx [B][M][k] int32, out_cnt [B][M] int32 or NULL
 *   bq_cache   NULL = brute force over all N points.  Otherwise a cache filled
 *              by fp_fps_exact / fp_mdps_sample / fp_mdps_sample_pruned on the same xyz: centres that
 *              are the cached samples (same position q, same radius) are read
 *              from the cache with no distance evaluation (redundancy-free ball
 *              query, Section 4.2); any other centre, and every centre of a cloud
 *              whose record is incomplete, falls back to the brute-force test
 *              inside the same kernel.  Results are identical.
 * A centre index outside [0,N) yields a row of -1 and count 0.  M = 0 is accepted (the
 * centre and output pointers may then be NULL).
 */
fp_status fp_ball_query(const float* xyz, int32_t B, int32_t N,
                        const int32_t* center_idx, int32_t M, float radius, int32_t k,
                        int32_t* out_idx, int32_t* out_cnt,
                        const void* bq_cache, void* stream);

/*
 * Ball query through a uniform grid: the result of fp_ball_query without a cache, byte for
 * byte, for any centre set, from the 27 grid cells around a centre instead of all N points
 * (cells as wide as the radius; of the hits the k lowest indices are kept, in ascending order,
 * which is what the scan over all points finds first).  The grid is built in the workspace by
 * every call.
 */
size_t fp_ball_query_grid_workspace_bytes(int32_t B, int32_t N);
fp_status fp_ball_query_grid(const float* xyz, int32_t B, int32_t N, const int32_t* center_idx,
                             int32_t M, float radius, int32_t k, int32_t* out_idx, int32_t* out_cnt,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace fp_knn needs when it is given a cache of cache_entries entries per cloud
 * (fp_bq_cache_entries; 0 for shapes the library rejects).  With a smaller workspace, down to
 * cache_entries = 0, fp_knn still works: clouds whose record does not fit are searched by brute
 * force.  Alignment: 256 bytes. */
size_t fp_knn_workspace_bytes(int32_t B, int32_t N, int64_t cache_entries);

/*
 * k nearest samples of every point -- the k-NN of the up-sampling (feature propagation)
 * step, Section 3.1: for point j of cloud b the k samples with the smallest squared
 * binary32 distance, nearest first; among equal distances the lower position q first.
 *   sample_idx [B][n] int32 indices into the cloud (a sampler's output), 1 <= k <= min(n, 8)
 *   out_pos    [B][N][k] int32 positions q into sample_idx
 *   out_d2     [B][N][k] float32 squared distances, ascending
 *   bq_cache   NULL = every point is compared with all n samples.  Otherwise a cache
 *              filled by fp_fps_exact / fp_mdps_sample on the same xyz whose samples are
 *              sample_idx (redundancy-free k-NN, Section 4.2): the search space of a point
 *              is the samples whose recorded ball contains it, which are its k nearest
 *              whenever there are at least k of them; points with fewer, and clouds whose
 *              sample list differs from the cached one or whose record is incomplete, are
 *              searched by brute force in a second pass.  Results are identical to the
 *              brute-force search.
 *   out_deferred [B] int32 or NULL: with a cache, the number of points per cloud that took
 *              the brute-force pass
 *   workspace  required with a cache (fp_knn_workspace_bytes), else ignored
 * A sample index outside [0,N) is never a neighbour; slots no sample fills hold
 * position -1 and distance +inf.
 */
fp_status fp_knn(const float* xyz, int32_t B, int32_t N, const int32_t* sample_idx, int32_t n,
                 int32_t k, int32_t* out_pos, float* out_d2, const void* bq_cache,
                 int32_t* out_deferred, void* workspace, size_t workspace_bytes, void* stream);

#define FP_EXCL_MAX_LEVELS 17   /* FP_MAX_SEG thresholds and the ball-query radius */

/* Bytes of workspace fp_excl_count / fp_excl_fill need (0 for shapes the library rejects).
 * Alignment: 256 bytes. */
size_t fp_excl_workspace_bytes(int32_t B, int32_t N, int32_t L);

/*
 * Exclusion lists as a data structure, the list-building loops of Algorithm 2 (Section 4.1 step 2) with
 * the extra list at the ball-query radius of Section 4.2: for level l, cloud b and point i,
 * row r = (l*B + b)*N + i holds the points j of the cloud with dist^2(P_i, P_j) < thr2[b][l]
 * (strict, binary32) in ascending j -- the order in which the paper's loop over j appends
 * them; i itself is a member whenever thr2[b][l] > 0.  One distance per examined pair serves
 * all levels; a uniform grid limits the pairs examined to the 27 cells around a point.
 * Two passes, as for any compressed-row structure:
 *   fp_excl_count  builds the grid in the workspace and writes offsets [L*B*N + 1] int64:
 *                  row r occupies entries[offsets[r] .. offsets[r+1]); offsets[L*B*N] is the
 *                  number of members in total, which the caller reads back to size `entries`
 *   fp_excl_fill   writes the members.  Same xyz, thr2, L and workspace as the count call,
 *                  with nothing else using the workspace in between.  Members whose position
 *                  is >= capacity are not written (no error is raised on the device).
 *   thr2  [B][L] float32 squared radii, DEVICE memory (e.g. the thr2 fields of fp_mdps_info,
 *         or radius*radius of a ball query), any order, 1 <= L <= FP_EXCL_MAX_LEVELS;
 *         a value <= 0 or NaN gives empty rows
 */
fp_status fp_excl_count(const float* xyz, int32_t B, int32_t N, const float* thr2, int32_t L,
                        int64_t* offsets, void* workspace, size_t workspace_bytes, void* stream);
fp_status fp_excl_fill(const float* xyz, int32_t B, int32_t N, const float* thr2, int32_t L,
                       const int64_t* offsets, int32_t* entries, int64_t capacity,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Ball query by lookup in exclusion lists (Section 4.2: the neighbours of a centre are its
 * list at the query radius): the first k members of row (level*B + b)*N + center_idx[b][q],
 * unused slots repeating the first member, out_cnt = min(members, k).  With the level's
 * radius equal to the query radius this is fp_ball_query's result for any centre set.
 * An empty row or a centre index outside [0,N) gives -1 in every slot and count 0.
 *   out_idx [B][M][k] int32, out_cnt [B][M] int32 or NULL, 1 <= k
 */
fp_status fp_ball_query_lists(const int64_t* offsets, const int32_t* entries, int32_t B, int32_t N,
                              int32_t level, int32_t L, const int32_t* center_idx, int32_t M, int32_t k,
                              int32_t* out_idx, int32_t* out_cnt, void* stream);

/*
 * k nearest samples through a uniform grid over the samples: the result of fp_knn, bit for
 * bit.  A point looks at the samples of the 27 cells around it (cells as wide as `radius`);
 * when its k-th nearest among them is closer than `radius` no sample elsewhere can be nearer,
 * and the point is done.  The remaining points (out_deferred[b] of them) are searched by brute
 * force.  A radius of two to three times the samples' coverage radius settles almost every
 * point in the grid.  Arguments as fp_knn without a cache.
 */
size_t fp_knn_grid_workspace_bytes(int32_t B, int32_t N, int32_t n);
fp_status fp_knn_grid(const float* xyz, int32_t B, int32_t N, const int32_t* sample_idx, int32_t n,
                      int32_t k, float radius, int32_t* out_pos, float* out_d2, int32_t* out_deferred,
                      void* workspace, size_t workspace_bytes, void* stream);

/* out_xyz[b][q] = xyz[b][idx[b][q]] -- input of the next stage of a hierarchy
 * (Section 3.1).  Indices outside [0,N) give NaN coordinates. */
fp_status fp_gather_xyz(const float* xyz, int32_t B, int32_t N,
                        const int32_t* idx, int32_t M, float* out_xyz, void* stream);

/* Sampling-quality helper: out_cov2[b] = max_j min_q dist^2(P[j], S[q]) in
 * binary32, the squared coverage radius of the sample set.
 *   sample_xyz [B][n][3] (e.g. from fp_gather_xyz), out_cov2 [B] float32 */
fp_status fp_coverage(const float* xyz, int32_t B, int32_t N,
                      const float* sample_xyz, int32_t n, float* out_cov2, void* stream);

/* Measurement aid: the plain binary32 rate this build can reach.  Every thread of
 * `blocks` workgroups of 256 runs `iterations` times over eight independent chains of one
 * multiplication and one addition, each rounded on its own like the distance update (the library
 * is compiled without contraction and without packed binary32 instructions), and stores its sum in
 * out[blocks * 256] (float32).  The operations performed are blocks * 256 * iterations * 16; the
 * caller times the call.  Price a kernel's operations against this rate to see how much of the
 * reachable arithmetic throughput it uses. */
fp_status fp_probe_fp32_rate(int32_t blocks, int32_t iterations, float* out, void* stream);

/* How the sampler splits one cloud: workgroups per cloud, threads per workgroup that
 * hold points (a workgroup has one more wave, which holds none), points per thread.
 * Returns FP_ERR_SHAPE if the cloud does not fit. */
fp_status fp_plan(int32_t B, int32_t N, int32_t* wg_per_cloud, int32_t* threads,
                  int32_t* points_per_thread);

/*
 * ---- Test and measurement hooks -------------------------------------------------------
 * The three setters below are the library's ONLY process-wide mutable state.  Every other
 * entry point keeps its state in its arguments (workspace, cache, outputs) and is re-entrant
 * with distinct workspaces.  The hooks exist for tests and profiling runs, take effect for
 * calls made after they return, are not synchronised with calls in flight on other threads,
 * and are left at their defaults by production callers.
 */

/* Force the number of workgroups per cloud (0 = automatic, the default).  Lets a test run a
 * small cloud through the multi-workgroup exchange. */
void fp_set_wg_per_cloud(int32_t wg_per_cloud);

/* Multi-workgroup launches are cooperative by default (the runtime guarantees that all
 * workgroups are resident, which the waits between them rely on).  0 switches to a plain
 * launch, for tools that cannot trace cooperative launches: the grid never exceeds one
 * workgroup per compute unit, so it is resident on an otherwise idle device, and a wait that
 * cannot be met still ends through the wait limit. */
void fp_set_cooperative_launch(int32_t on);

/* Upper limit, in microseconds, of any wait of one workgroup on another
 * (default 2 000 000).  A wait that expires ends the kernel with info.status 2.  With 0 a
 * wait gives up as soon as two polls in a row find nothing (a hook for tests of that path). */
void fp_set_wait_limit_us(int64_t microseconds);

const char* fp_status_string(fp_status s);

#ifdef __cplusplus
}
#endif
#endif /* FASTPOINT_H_ */
