// Host side of the C ABI declared in include/fastpoint.h: argument checks,
// launch planning and kernel launches.  No device memory is allocated here.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "kernels.h"

namespace fastpoint {
namespace {

std::atomic<int> g_force_wg_per_cloud{0};
std::atomic<int64_t> g_wait_limit_us{2000000};
std::atomic<int> g_cooperative{1};

struct DeviceInfo {
    bool ok = false;
    int cus = 0;
    int64_t wall_khz = 100000;
    void* scratch = nullptr;      // this device's copy of the static scratch array (fp_fps_exact_static)
};

// exchange words between the workgroups of a cloud: what a sampler workspace holds
constexpr int64_t kLlPkWords = (int64_t)2 * kMaxGroup * kLlSlotWords;             // all groups together
constexpr int64_t kLlCdWords = (int64_t)2 * kMaxGroup * kCandMax * kCandWords;
constexpr int64_t kLlCtWords = (int64_t)2 * kMaxGroup;
constexpr int64_t kLlWords = kLlPkWords + kLlCdWords + kLlCtWords;
constexpr size_t kScratchBytes = (size_t)(kLlWords * 8);                          // 2 658 304 bytes

// Scratch of fp_fps_exact_static: the same exchange words, but in device memory that belongs to
// the library's code object instead of a caller's workspace, so that the call allocates nothing.
// Every GPU the library runs on holds its own copy at its own address until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
DeviceInfo g_dev[kMaxDevices];
std::mutex g_dev_mutex;

bool device_info(DeviceInfo* out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (!g_dev[dev].ok) {
        int cus = 0, khz = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return false;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0)
            khz = 100000;
        g_dev[dev].cus = cus;
        g_dev[dev].wall_khz = khz;
        g_dev[dev].ok = cus > 0;
    }
    *out = g_dev[dev];
    return out->ok;
}

// capacities (threads, points per thread) the sampler kernel is built for
struct Shape {
    int T, P;
};
// T threads hold points (two waves per SIMD, so that their plain fp32 operations issue
// together); the launch adds one control wave
constexpr Shape kShapes[] = {{512, 2}, {512, 4}, {512, 8}, {512, 16}};
constexpr int kNumShapes = (int)(sizeof(kShapes) / sizeof(kShapes[0]));
constexpr int kCtrlThreads = 64;
constexpr int kTargetPointsPerWg = 1024;

bool shape_for(int64_t points_per_wg, Shape* s)
{
    for (int i = 0; i < kNumShapes; ++i)
        if ((int64_t)kShapes[i].T * kShapes[i].P >= points_per_wg) {
            *s = kShapes[i];
            return true;
        }
    return false;
}

constexpr int kMaxPointsPerWg = 512 * 16;

// Splits B clouds of N points over at most `cus` resident workgroups: G workgroups per
// cloud, `groups` clouds resident at once (further clouds are taken in turn).
bool make_plan(int B, int N, int cus, Plan* plan)
{
    if (B < 1 || N < 1 || cus < 1) return false;
    int gcap = cus < kMaxGroup ? cus : kMaxGroup;              // most workgroups one cloud can get
    int gneed = (int)(((int64_t)N + kMaxPointsPerWg - 1) / kMaxPointsPerWg);
    if (gneed > gcap) return false;                            // cloud too large to stay resident
    int G = (int)(((int64_t)N + kTargetPointsPerWg - 1) / kTargetPointsPerWg);
    if (G > gcap) G = gcap;
    // keep every cloud resident when that still leaves each workgroup within its capacity
    if ((int64_t)B * G > cus) {
        int share = cus / (B < cus ? B : cus);
        if (share < 1) share = 1;
        G = share > gneed ? share : gneed;
        if (G > gcap) G = gcap;
    }
    const int forced = g_force_wg_per_cloud.load();
    if (forced > 0) G = forced < gneed ? gneed : (forced > gcap ? gcap : forced);
    if (G < 1) G = 1;
    Shape s;
    if (!shape_for(((int64_t)N + G - 1) / G, &s)) return false;
    plan->G = G;
    plan->T = s.T;
    plan->P = s.P;
    int groups = cus / G;
    if (groups > B) groups = B;
    if (groups < 1) groups = 1;
    plan->groups = groups;
    return true;
}

inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

int64_t bq_blocks(int N) { return ((int64_t)N + 63) / 64; }

// The address of the current device's copy of `scratch`, looked up once per device (with that
// device current) and kept; NULL if the runtime cannot give it.
void* static_scratch()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (!g_dev[dev].scratch) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        if ((reinterpret_cast<uintptr_t>(ptr) & 255u) != 0) return nullptr;
        g_dev[dev].scratch = ptr;
    }
    return g_dev[dev].scratch;
}

// Stride of the scattered scan order: the smallest integer >= max(1, floor(0.6180339887498949 N))
// that has no common factor with N, so that t -> (t A) mod N visits every index once.
int64_t scan_walk_stride(int32_t N)
{
    int64_t A = (int64_t)floor(0.6180339887498949 * (double)N);
    if (A < 1) A = 1;
    for (;; ++A) {
        int64_t x = A, y = N;
        while (y != 0) {
            const int64_t r = x % y;
            x = y;
            y = r;
        }
        if (x == 1) return A;
    }
}

// x with (A x) mod N == 1, for A coprime to N (extended Euclid); 0 for N == 1
int64_t inverse_mod(int64_t A, int64_t N)
{
    int64_t r0 = N, r1 = A % N, t0 = 0, t1 = 1;
    while (r1 != 0) {
        const int64_t q = r0 / r1;
        const int64_t r2 = r0 - q * r1, t2 = t0 - q * t1;
        r0 = r1;
        r1 = r2;
        t0 = t1;
        t1 = t2;
    }
    return ((t0 % N) + N) % N;
}

// Cell-ordered variant: words through which the workgroups of a cloud hand each other the relations
// between the candidates of a window round, [resident clouds][2][kCandWin][16]; a cloud spread over
// several workgroups leaves room for at most kMaxGroup / 2 resident clouds.
constexpr int64_t kRelWordsPerCloud = (int64_t)2 * kCandWin * 16;
int64_t rel_exchange_bytes(int32_t B)
{
    const int64_t clouds = B < kMaxGroup / 2 ? B : kMaxGroup / 2;
#ifdef FASTPOINT_PHASE_CLOCKS
    return clouds * kRelWordsPerCloud * 8 + kMaxGroup * 16 * 8;
#else
    return clouds * kRelWordsPerCloud * 8;
#endif
}

int64_t scan_walk_bytes(int32_t B, int32_t N) { return align_up((int64_t)B * N * (int64_t)sizeof(float4), 256); }

fp_status run_sampler(const float* xyz, int32_t B, int32_t N, int32_t n, const int32_t* start_idx,
                      const fp_mdps_params* prm, int32_t* out_idx, float* out_mdc, fp_mdps_info* info,
                      void* bq_cache, size_t bq_cache_bytes, float bq_radius, void* workspace,
                      size_t workspace_bytes, void* stream_v, bool pruned = false)
{
    if (!xyz || !out_idx) return FP_ERR_NULL;
    if (B < 1 || N < 1 || n < 1 || n > N) return FP_ERR_SHAPE;
    if ((int64_t)B * N > (int64_t)1 << 40) return FP_ERR_SHAPE;
    DeviceInfo di;
    if (!device_info(&di)) return FP_ERR_DEVICE;
    Plan plan;
    if (!make_plan(B, N, di.cus < 256 ? di.cus : 256, &plan)) return FP_ERR_SHAPE;
    if (bq_cache) {
        if (!(bq_radius > 0.0f) || !isfinite(bq_radius)) return FP_ERR_PARAM;
        if ((reinterpret_cast<uintptr_t>(bq_cache) & 255u) != 0) return FP_ERR_WORKSPACE;
    }
    const bool walk = prm != nullptr && prm->scan_order == 1;
    if (prm && (prm->scan_order < 0 || prm->scan_order > 1)) return FP_ERR_PARAM;
    if (bq_cache && ((walk && !pruned) || (pruned && !prm))) return FP_ERR_PARAM;
    if (walk && !pruned && fp_mdps_scattered_workspace_bytes(B, N) == 0) return FP_ERR_SHAPE;
    if (!workspace ||
        workspace_bytes < (pruned ? fp_fps_pruned_workspace_bytes(B, N)
                                  : (walk ? fp_mdps_scattered_workspace_bytes(B, N) : fp_workspace_bytes(B, N))) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return FP_ERR_WORKSPACE;

    SamplerArgs a;
    memset(&a, 0, sizeof(a));
    a.xyz = xyz;
    a.start_idx = start_idx;
    a.out_idx = out_idx;
    a.out_mdc = out_mdc;
    a.info = info;
    a.B = B;
    a.N = N;
    a.n = n;
    a.G = plan.G;
    a.m = n - 1;
    a.nseg = 1;
    if (prm) {
        if (!(prm->p > 0.0f) || !(prm->p < 1.0f)) return FP_ERR_PARAM;
        if (prm->nseg < 1 || prm->nseg > FP_MAX_SEG) return FP_ERR_PARAM;
        if (prm->m_min < 1) return FP_ERR_PARAM;
        if (prm->use_override) {
            for (int l = 0; l < prm->nseg; ++l) {
                if (!(prm->thr_override[l] > 0.0f)) return FP_ERR_PARAM;
                if (l > 0 && prm->thr_override[l] > prm->thr_override[l - 1]) return FP_ERR_PARAM;
                a.thr_override[l] = prm->thr_override[l];
            }
        } else {
            if (!(prm->bias > 0.0f) || !isfinite(prm->bias) || !isfinite(prm->exponent))
                return FP_ERR_PARAM;
            if (prm->fit_window < 1 || prm->fit_window > 64) return FP_ERR_PARAM;
            for (int l = 0; l < prm->nseg; ++l) {
                if (!(prm->level_scale[l] > 0.0f) || !isfinite(prm->level_scale[l])) return FP_ERR_PARAM;
                a.level_scale[l] = prm->level_scale[l];
            }
        }
        int64_t m = (int64_t)floor((double)prm->p * (double)n);
        if (m < prm->m_min) m = prm->m_min;
        if (m > n - 1) m = n - 1;
        a.m = (int32_t)m;
        a.nseg = prm->nseg;
        a.fit_window = prm->fit_window;
        a.use_override = prm->use_override ? 1 : 0;
        a.exponent = prm->exponent;
        a.bias2 = (double)prm->bias * (double)prm->bias;
        a.mlp = prm->use_override ? nullptr : prm->mlp_weights;
    }
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    a.ll_pk = reinterpret_cast<uint64_t*>(workspace);
    a.ll_cd = a.ll_pk + kLlPkWords;
    a.ll_ct = a.ll_cd + kLlCdWords;
    a.wait_ticks = g_wait_limit_us.load() * di.wall_khz / 1000;

    if (pruned) {
        // the cloud in cell order, behind the exchange words
        void* sort_ws = reinterpret_cast<unsigned char*>(workspace) + fp_workspace_bytes(B, N);
        if (launch_spatial_sort(xyz, B, N, sort_ws, stream) != hipSuccess) return FP_ERR_DEVICE;
        a.sorted = spatial_sorted(B, N, sort_ws);
        if (walk) a.walk_inv = (uint64_t)inverse_mod(scan_walk_stride(N), N);
        a.ll_rel = reinterpret_cast<uint64_t*>(reinterpret_cast<unsigned char*>(sort_ws) + spatial_sort_bytes(B, N));
#ifdef FASTPOINT_PHASE_CLOCKS
        a.dbg = reinterpret_cast<long long*>(reinterpret_cast<unsigned char*>(workspace) +
                                             fp_fps_pruned_workspace_bytes(B, N) - kMaxGroup * 16 * 8);
#endif
    }
    if (walk && !pruned && a.m < n - 1) {
        // the cloud in the order of the walk, behind the exchange words (not needed when the prefix
        // covers everything: the call is exact FPS then)
        float4* rec = reinterpret_cast<float4*>(reinterpret_cast<unsigned char*>(workspace) + fp_workspace_bytes(B, N));
        if (launch_scan_walk(xyz, B, N, scan_walk_stride(N), rec, stream) != hipSuccess) return FP_ERR_DEVICE;
        a.sorted = rec;
    }
    const bool reordered = pruned || a.sorted != nullptr;
    const bool bq = bq_cache != nullptr;
    uint64_t* bq_zero = nullptr;
    int64_t bq_zero_words = 0;
    if (bq) {
        // layout (kernels.h): header (written by the sampler kernel), copy of the sample indices,
        // per-cloud cursors and per-sample counts (zeroed here), row offsets, the two entry lists
        const int64_t cap = fp_bq_cache_entries(bq_cache_bytes, B, N, n);
        if (cap < kBqChunk) return FP_ERR_WORKSPACE;
        const BqHeader lay = bq_layout(B, N, n, bq_radius * bq_radius, cap);
        unsigned char* base = reinterpret_cast<unsigned char*>(bq_cache);
        a.bq_base = base;
        a.bq_idx = reinterpret_cast<int32_t*>(base + lay.idx_offset);
        a.bq_cursor = reinterpret_cast<uint32_t*>(base + lay.cursor_offset);
        a.bq_ovf = reinterpret_cast<uint32_t*>(base + lay.ovf_offset);
        a.bq_fill = reinterpret_cast<uint32_t*>(base + lay.fill_offset);
        a.bq_raw = reinterpret_cast<BqRaw*>(base + lay.raw_offset);
        a.bq_map = reinterpret_cast<int32_t*>(base + lay.map_offset);
        a.bq_cap = lay.cap;
        a.bq_r2 = bq_radius * bq_radius;
        a.bq_blocks = (int32_t)bq_blocks(N);
        bq_zero = reinterpret_cast<uint64_t*>(base + lay.cursor_offset);
        bq_zero_words = (lay.rowoff_offset - lay.cursor_offset) / 8;      // cursors, flags, counts, chunk fills
    }

    // MDPS threshold rounds with two candidates per control-wave lane: measured faster except
    // where one workgroup both holds the cloud and records the radius tests
    const int mode = prm == nullptr ? 0
                     : (walk && pruned ? 4 : (walk && a.sorted != nullptr ? 3 : ((pruned || !bq || plan.G > 1) ? 2 : 1)));
    const void* fn = sampler_kernel_for(plan.T, plan.P, bq, reordered, mode);
    if (!fn) return FP_ERR_SHAPE;
    const unsigned grid = (unsigned)(plan.groups * plan.G);
    void* kargs[] = {&a};
    hipError_t err;
    // words that have to start at zero when the workgroups of a cloud wait on each other: the exchange
    // words (stamps start at 1 in every launch) and the chunk counters of a ball-query cache.  (A
    // cloud held by one workgroup has its counters zeroed by that workgroup.)
    if (plan.G > 1) {
        // ... and, cell-ordered MDPS, the relation words
        const int64_t rel_words = pruned && prm ? (int64_t)plan.groups * kRelWordsPerCloud : 0;
        if (launch_zero_words(a.ll_pk, kLlWords, bq_zero, bq_zero_words, a.ll_rel, rel_words, stream) != hipSuccess)
            return FP_ERR_DEVICE;
    }
    if (plan.G > 1 && g_cooperative.load())    // the whole grid has to be resident
        err = hipLaunchCooperativeKernel(fn, dim3(grid), dim3((unsigned)(plan.T + kCtrlThreads)), kargs, 0, stream);
    else
        err = hipLaunchKernel(fn, dim3(grid), dim3((unsigned)(plan.T + kCtrlThreads)), kargs, 0, stream);
    if (err == hipSuccess && bq) err = launch_bq_group_by_sample(bq_cache, B, N, n, a.bq_cap, stream);
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

}  // namespace
}  // namespace fastpoint

using namespace fastpoint;

extern "C" {

size_t fp_workspace_bytes(int32_t B, int32_t N)
{
    if (B < 1 || N < 1) return 0;
    return (size_t)(kLlWords * 8);
}

size_t fp_bq_cache_bytes(int32_t B, int32_t N, int32_t n, int64_t entries_per_cloud)
{
    if (B < 1 || N < 1 || n < 1 || n > N || B > 65535 || (int64_t)B * n > ((int64_t)1 << 31)) return 0;
    int64_t cap = entries_per_cloud > 0 ? entries_per_cloud : bq_capacity(N, n);
    cap = (cap + kBqChunk - 1) / kBqChunk * kBqChunk;   // whole chunks
    if (cap > ((int64_t)1 << 31)) return 0;             // entries are addressed with 32 bits
    return (size_t)bq_layout(B, N, n, 1.0f, cap).bytes;
}

int64_t fp_bq_cache_entries(size_t bytes, int32_t B, int32_t N, int32_t n)
{
    if (B < 1 || N < 1 || n < 1 || n > N || B > 65535 || (int64_t)B * n > ((int64_t)1 << 31)) return 0;
    const int64_t fixed = bq_layout(B, N, n, 1.0f, 0).bytes;
    if ((int64_t)bytes <= fixed) return 0;
    // an upper estimate (every part is rounded up to 256 bytes), then down to what fits
    int64_t cap = ((int64_t)bytes - fixed) / ((int64_t)B * (int64_t)(sizeof(BqRaw) + sizeof(BqEntry))) + kBqChunk;
    if (cap > ((int64_t)1 << 31)) cap = (int64_t)1 << 31;
    cap = cap / kBqChunk * kBqChunk;
    while (cap > 0 && bq_layout(B, N, n, 1.0f, cap).bytes > (int64_t)bytes) cap -= kBqChunk;
    return cap;
}

fp_status fp_fps_exact(const float* xyz, int32_t B, int32_t N, int32_t n, const int32_t* start_idx,
                       int32_t* out_idx, float* out_mdc, fp_mdps_info* info, void* bq_cache,
                       size_t bq_cache_bytes, float bq_radius, void* workspace, size_t workspace_bytes,
                       void* stream)
{
    return run_sampler(xyz, B, N, n, start_idx, nullptr, out_idx, out_mdc, info, bq_cache, bq_cache_bytes,
                       bq_radius, workspace, workspace_bytes, stream);
}

fp_status fp_fps_exact_static(const float* xyz, int32_t B, int32_t N, int32_t n, const int32_t* start_idx,
                              int32_t* out_idx, float* out_mdc, void* stream)
{
    if (!xyz || !out_idx) return FP_ERR_NULL;
    if (B < 1 || N < 1 || n < 1 || n > N) return FP_ERR_SHAPE;
    if (N > FP_STATIC_MAX_POINTS) return FP_ERR_CAPACITY;
    void* ws = static_scratch();
    if (!ws) return FP_ERR_DEVICE;
    return run_sampler(xyz, B, N, n, start_idx, nullptr, out_idx, out_mdc, nullptr, nullptr, 0, 0.0f, ws,
                       kScratchBytes, stream);
}

size_t fp_mdps_scattered_workspace_bytes(int32_t B, int32_t N)
{
    if (B < 1 || N < 1 || (int64_t)B * N > ((int64_t)1 << 33)) return 0;
    return fp_workspace_bytes(B, N) + (size_t)scan_walk_bytes(B, N);
}

size_t fp_fps_pruned_workspace_bytes(int32_t B, int32_t N)
{
    if (B < 1 || N < 1 || B > 65535 || (int64_t)B * N > ((int64_t)1 << 33)) return 0;
    return fp_workspace_bytes(B, N) + (size_t)spatial_sort_bytes(B, N) + (size_t)rel_exchange_bytes(B);
}

fp_status fp_fps_exact_pruned(const float* xyz, int32_t B, int32_t N, int32_t n, const int32_t* start_idx,
                              int32_t* out_idx, float* out_mdc, fp_mdps_info* info, void* workspace,
                              size_t workspace_bytes, void* stream)
{
    if (B > 65535 || (int64_t)B * N > ((int64_t)1 << 33)) return FP_ERR_SHAPE;
    return run_sampler(xyz, B, N, n, start_idx, nullptr, out_idx, out_mdc, info, nullptr, 0, 0.0f, workspace,
                       workspace_bytes, stream, true);
}

fp_status fp_mdps_sample_pruned(const float* xyz, int32_t B, int32_t N, int32_t n, const int32_t* start_idx,
                                const fp_mdps_params* prm, int32_t* out_idx, fp_mdps_info* info,
                                void* bq_cache, size_t bq_cache_bytes, float bq_radius, void* workspace,
                                size_t workspace_bytes, void* stream)
{
    if (!prm) return FP_ERR_NULL;
    if (B > 65535 || (int64_t)B * N > ((int64_t)1 << 33)) return FP_ERR_SHAPE;
    return run_sampler(xyz, B, N, n, start_idx, prm, out_idx, nullptr, info, bq_cache, bq_cache_bytes, bq_radius,
                       workspace, workspace_bytes, stream, true);
}

fp_status fp_mdps_sample(const float* xyz, int32_t B, int32_t N, int32_t n, const int32_t* start_idx,
                         const fp_mdps_params* prm, int32_t* out_idx, fp_mdps_info* info,
                         void* bq_cache, size_t bq_cache_bytes, float bq_radius, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    if (!prm) return FP_ERR_NULL;
    return run_sampler(xyz, B, N, n, start_idx, prm, out_idx, nullptr, info, bq_cache, bq_cache_bytes,
                       bq_radius, workspace, workspace_bytes, stream);
}

fp_status fp_ball_query(const float* xyz, int32_t B, int32_t N, const int32_t* center_idx, int32_t M,
                        float radius, int32_t k, int32_t* out_idx, int32_t* out_cnt,
                        const void* bq_cache, void* stream)
{
    if (B < 1 || N < 1 || M < 0 || k < 1 || k > 254 || B > 65535) return FP_ERR_SHAPE;
    if (!(radius > 0.0f) || !isfinite(radius)) return FP_ERR_PARAM;
    if (!xyz) return FP_ERR_NULL;
    if (M == 0) return FP_OK;                 // no centres: nothing to write, the arrays may be empty
    if (!center_idx || !out_idx) return FP_ERR_NULL;
    if (bq_cache && (reinterpret_cast<uintptr_t>(bq_cache) & 255u) != 0) return FP_ERR_WORKSPACE;
    const float r2 = radius * radius;
    hipError_t err = launch_ball_query(xyz, B, N, center_idx, M, r2, k, out_idx, out_cnt, bq_cache,
                                       reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

size_t fp_ball_query_grid_workspace_bytes(int32_t B, int32_t N)
{
    if (B < 1 || N < 1 || B > 65535 || (int64_t)B * N > ((int64_t)1 << 33)) return 0;
    return (size_t)spatial_sort_bytes(B, N);
}

fp_status fp_ball_query_grid(const float* xyz, int32_t B, int32_t N, const int32_t* center_idx, int32_t M,
                             float radius, int32_t k, int32_t* out_idx, int32_t* out_cnt, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    if (B < 1 || N < 1 || M < 0 || k < 1 || k > 254 || B > 65535) return FP_ERR_SHAPE;
    if ((int64_t)B * N > ((int64_t)1 << 33)) return FP_ERR_SHAPE;
    if (!(radius > 0.0f) || !isfinite(radius)) return FP_ERR_PARAM;
    if (!xyz) return FP_ERR_NULL;
    if (M == 0) return FP_OK;
    if (!center_idx || !out_idx) return FP_ERR_NULL;
    if (!workspace || workspace_bytes < fp_ball_query_grid_workspace_bytes(B, N) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return FP_ERR_WORKSPACE;
    hipError_t err = launch_bq_grid(xyz, B, N, center_idx, M, radius * radius, k, out_idx, out_cnt, workspace,
                                    reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

// parts of a k-NN workspace (byte offsets): per cloud a flag, a counter and a list of up to N
// deferred points; with a cache also the entries of the cache regrouped by point block
struct KnnLayout {
    int64_t flags, count, list, blk_cnt, blk_off, blk_rows, bytes;
};
static KnnLayout knn_layout(int32_t B, int32_t N, int64_t cache_entries)
{
    KnnLayout l;
    l.flags = 0;
    l.count = align_up((int64_t)B * 4, 256);
    l.list = l.count + align_up((int64_t)B * 4, 256);
    l.blk_cnt = l.list + align_up((int64_t)B * N * 4, 256);
    l.blk_off = l.blk_cnt + align_up((int64_t)B * bq_blocks(N) * 4, 256);
    l.blk_rows = l.blk_off + align_up((int64_t)B * (bq_blocks(N) + 1) * 4, 256);
    l.bytes = l.blk_rows + align_up((int64_t)B * cache_entries * (int64_t)sizeof(BqEntry), 256);
    return l;
}

size_t fp_knn_workspace_bytes(int32_t B, int32_t N, int64_t cache_entries)
{
    if (B < 1 || N < 1 || cache_entries < 0 || cache_entries > ((int64_t)1 << 31) || B > 65535) return 0;
    return (size_t)knn_layout(B, N, cache_entries).bytes;
}

fp_status fp_knn(const float* xyz, int32_t B, int32_t N, const int32_t* sample_idx, int32_t n, int32_t k,
                 int32_t* out_pos, float* out_d2, const void* bq_cache, int32_t* out_deferred,
                 void* workspace, size_t workspace_bytes, void* stream)
{
    if (!xyz || !sample_idx || !out_pos || !out_d2) return FP_ERR_NULL;
    if (B < 1 || N < 1 || n < 1 || n > N || k < 1 || k > FP_KNN_MAX_K || k > n || B > 65535) return FP_ERR_SHAPE;
    if ((int64_t)B * N > (int64_t)1 << 40) return FP_ERR_SHAPE;
    int32_t *flags = nullptr, *count = nullptr, *list = nullptr, *blk_cnt = nullptr;
    uint32_t* blk_off = nullptr;
    BqEntry* blk_rows = nullptr;
    int64_t blk_rows_cap = 0;
    if (bq_cache) {
        if ((reinterpret_cast<uintptr_t>(bq_cache) & 255u) != 0) return FP_ERR_WORKSPACE;
        if (!workspace || workspace_bytes < fp_knn_workspace_bytes(B, N, 0) ||
            (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
            return FP_ERR_WORKSPACE;
        const KnnLayout l = knn_layout(B, N, 0);
        // whatever lies behind the fixed parts holds the cache's entries regrouped by point block; a
        // cloud with more entries than fit there is searched by brute force
        blk_rows_cap = ((int64_t)workspace_bytes - l.blk_rows) / ((int64_t)B * (int64_t)sizeof(BqEntry));
        unsigned char* base = reinterpret_cast<unsigned char*>(workspace);
        flags = reinterpret_cast<int32_t*>(base + l.flags);
        count = reinterpret_cast<int32_t*>(base + l.count);
        list = reinterpret_cast<int32_t*>(base + l.list);
        blk_cnt = reinterpret_cast<int32_t*>(base + l.blk_cnt);
        blk_off = reinterpret_cast<uint32_t*>(base + l.blk_off);
        blk_rows = reinterpret_cast<BqEntry*>(base + l.blk_rows);
    }
    hipError_t err = launch_knn(xyz, B, N, sample_idx, n, k, out_pos, out_d2, bq_cache, flags, count, list,
                                blk_cnt, blk_off, blk_rows, blk_rows_cap, bq_cache ? out_deferred : nullptr,
                                reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

static bool excl_shape_ok(int32_t B, int32_t N, int32_t L)
{
    if (B < 1 || N < 1 || L < 1 || L > FP_EXCL_MAX_LEVELS || B > 65535) return false;
    return (int64_t)L * B * N <= ((int64_t)1 << 40) && (int64_t)B * N <= ((int64_t)1 << 33);
}

size_t fp_excl_workspace_bytes(int32_t B, int32_t N, int32_t L)
{
    if (!excl_shape_ok(B, N, L)) return 0;
    return (size_t)excl_layout(B, N, L).bytes;
}

fp_status fp_excl_count(const float* xyz, int32_t B, int32_t N, const float* thr2, int32_t L,
                        int64_t* offsets, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!xyz || !thr2 || !offsets) return FP_ERR_NULL;
    if (!excl_shape_ok(B, N, L)) return FP_ERR_SHAPE;
    if (!workspace || workspace_bytes < fp_excl_workspace_bytes(B, N, L) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return FP_ERR_WORKSPACE;
    hipError_t err = launch_excl_count(xyz, B, N, thr2, L, offsets, workspace,
                                       reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

fp_status fp_excl_fill(const float* xyz, int32_t B, int32_t N, const float* thr2, int32_t L,
                       const int64_t* offsets, int32_t* entries, int64_t capacity, void* workspace,
                       size_t workspace_bytes, void* stream)
{
    if (!xyz || !thr2 || !offsets || (!entries && capacity > 0)) return FP_ERR_NULL;
    if (!excl_shape_ok(B, N, L) || capacity < 0) return FP_ERR_SHAPE;
    if (!workspace || workspace_bytes < fp_excl_workspace_bytes(B, N, L) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return FP_ERR_WORKSPACE;
    hipError_t err = launch_excl_fill(xyz, B, N, thr2, L, offsets, entries, capacity, workspace,
                                      reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

fp_status fp_ball_query_lists(const int64_t* offsets, const int32_t* entries, int32_t B, int32_t N,
                              int32_t level, int32_t L, const int32_t* center_idx, int32_t M, int32_t k,
                              int32_t* out_idx, int32_t* out_cnt, void* stream)
{
    if (!excl_shape_ok(B, N, L) || level < 0 || level >= L || M < 0 || k < 1) return FP_ERR_SHAPE;
    if (!offsets || !entries) return FP_ERR_NULL;
    if (M == 0) return FP_OK;
    if (!center_idx || !out_idx) return FP_ERR_NULL;
    hipError_t err = launch_bq_lists(offsets, entries, B, N, level, center_idx, M, k, out_idx, out_cnt,
                                     reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

size_t fp_knn_grid_workspace_bytes(int32_t B, int32_t N, int32_t n)
{
    if (B < 1 || N < 1 || n < 1 || B > 65535 || (int64_t)B * N > ((int64_t)1 << 33)) return 0;
    // the deferred-point bookkeeping of fp_knn, the samples' coordinates, the grid over them
    return fp_knn_workspace_bytes(B, N, 0) + (size_t)align_up((int64_t)B * n * 12, 256) +
           (size_t)spatial_sort_bytes(B, n);
}

fp_status fp_knn_grid(const float* xyz, int32_t B, int32_t N, const int32_t* sample_idx, int32_t n, int32_t k,
                      float radius, int32_t* out_pos, float* out_d2, int32_t* out_deferred, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    if (!xyz || !sample_idx || !out_pos || !out_d2) return FP_ERR_NULL;
    if (B < 1 || N < 1 || n < 1 || k < 1 || k > FP_KNN_MAX_K || k > n || B > 65535) return FP_ERR_SHAPE;
    if ((int64_t)B * N > ((int64_t)1 << 33)) return FP_ERR_SHAPE;
    if (!(radius > 0.0f) || !isfinite(radius)) return FP_ERR_PARAM;
    if (!workspace || workspace_bytes < fp_knn_grid_workspace_bytes(B, N, n) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return FP_ERR_WORKSPACE;
    unsigned char* base = reinterpret_cast<unsigned char*>(workspace);
    int32_t* count = reinterpret_cast<int32_t*>(base + align_up((int64_t)B * 4, 256));
    int32_t* list = reinterpret_cast<int32_t*>(base + 2 * align_up((int64_t)B * 4, 256));
    float* sample_xyz = reinterpret_cast<float*>(base + fp_knn_workspace_bytes(B, N, 0));
    void* grid_ws = base + fp_knn_workspace_bytes(B, N, 0) + align_up((int64_t)B * n * 12, 256);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (launch_gather(xyz, B, N, sample_idx, n, sample_xyz, st) != hipSuccess) return FP_ERR_DEVICE;
    if (launch_knn_grid(xyz, B, N, sample_xyz, n, k, radius * radius, out_pos, out_d2, count, list, grid_ws, st) !=
        hipSuccess)
        return FP_ERR_DEVICE;
    hipError_t err = launch_knn_deferred(xyz, B, N, sample_idx, n, k, out_pos, out_d2, count, list, out_deferred, st);
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

fp_status fp_gather_xyz(const float* xyz, int32_t B, int32_t N, const int32_t* idx, int32_t M,
                        float* out_xyz, void* stream)
{
    if (B < 1 || N < 1 || M < 0) return FP_ERR_SHAPE;
    if (!xyz) return FP_ERR_NULL;
    if (M == 0) return FP_OK;
    if (!idx || !out_xyz) return FP_ERR_NULL;
    hipError_t err = launch_gather(xyz, B, N, idx, M, out_xyz, reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

fp_status fp_coverage(const float* xyz, int32_t B, int32_t N, const float* sample_xyz, int32_t n,
                      float* out_cov2, void* stream)
{
    if (!xyz || !sample_xyz || !out_cov2) return FP_ERR_NULL;
    if (B < 1 || N < 1 || n < 1 || B > 65535) return FP_ERR_SHAPE;
    hipError_t err = launch_coverage(xyz, B, N, sample_xyz, n, out_cov2,
                                     reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? FP_OK : FP_ERR_DEVICE;
}

fp_status fp_probe_fp32_rate(int32_t blocks, int32_t iterations, float* out, void* stream)
{
    if (!out) return FP_ERR_NULL;
    if (blocks < 1 || blocks > (1 << 20) || iterations < 1) return FP_ERR_SHAPE;
    return launch_probe_fp32(blocks, iterations, out, reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? FP_OK
               : FP_ERR_DEVICE;
}

fp_status fp_plan(int32_t B, int32_t N, int32_t* wg_per_cloud, int32_t* threads,
                  int32_t* points_per_thread)
{
    DeviceInfo di;
    int cus = 256;
    if (device_info(&di)) cus = di.cus < 256 ? di.cus : 256;
    Plan plan;
    if (!make_plan(B, N, cus, &plan)) return FP_ERR_SHAPE;
    if (wg_per_cloud) *wg_per_cloud = plan.G;
    if (threads) *threads = plan.T;
    if (points_per_thread) *points_per_thread = plan.P;
    return FP_OK;
}

void fp_set_wg_per_cloud(int32_t wg_per_cloud) { g_force_wg_per_cloud.store(wg_per_cloud > 0 ? wg_per_cloud : 0); }

void fp_set_cooperative_launch(int32_t on) { g_cooperative.store(on ? 1 : 0); }

void fp_set_wait_limit_us(int64_t microseconds) { g_wait_limit_us.store(microseconds > 0 ? microseconds : 0); }

const char* fp_status_string(fp_status s)
{
    switch (s) {
        case FP_OK: return "ok";
        case FP_ERR_NULL: return "a required pointer is NULL";
        case FP_ERR_SHAPE: return "shape out of range";
        case FP_ERR_PARAM: return "parameter out of range";
        case FP_ERR_WORKSPACE: return "workspace or cache missing, misaligned or too small";
        case FP_ERR_DEVICE: return "HIP runtime error";
        case FP_ERR_CAPACITY: return "beyond the capacity of the library's static scratch buffer";
        default: return "unknown status";
    }
}

}  // extern "C"
