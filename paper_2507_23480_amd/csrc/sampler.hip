// Persistent sampler kernel for gfx950: exact farthest point sampling
// (Algorithm 1) and minimum-distance-prediction sampling (Algorithm 2) of
// FastPoint, arXiv 2507.23480, with the ball-query radius test recorded as a
// by-product of the distance updates (Section 4.2).
//
// One cloud is owned by a group of G workgroups that stay resident for the
// whole call.  Every thread keeps P points (x, y, z and the running minimum
// squared distance) in registers; wave `gw` of the cloud owns the 64*P
// consecutive indices [gw*64*P, (gw+1)*64*P), slot p of lane l being index
// (gw*P + p)*64 + l, so that one 64-lane compare mask of a slot is one 64-bit
// word of index-ordered bits.
//
// Per exact-FPS iteration: fold the last sample into the P distances, per-lane
// arg-max, DPP max/min reduction inside the wave, one LDS record per wave, one
// workgroup barrier, and -- when G > 1 -- an exchange between the workgroups of
// the cloud through self-validating 64-bit words (payload in the low half, a
// sequence stamp in the high half, relaxed agent-scope atomics, no fences).
//
// A workgroup has T threads that hold points plus one more wave, the control wave, that holds
// none: it resolves the picks of a round one after the other (a chain of dependent steps) and
// publishes each in LDS as soon as it is known, while the point waves fold the published picks
// into their distances.  The fold, which is throughput bound, thereby hides behind the
// resolution, which is latency bound.
//
// The threshold phase of Algorithm 2 uses the equivalent running-distance form:
// point j is available at level l iff dists[j] >= R_l^2.  Each round takes the
// first 64 available indices, resolves them in index order against the picks
// accepted earlier in the round (exactly what picking them one at a time would
// do), and folds all accepted picks into the distances in one sweep.
//
// Which available point the threshold phase takes next is left open by Section 4.1 step 3; two
// deterministic orders are built: the lowest index, and the first point of a scattered walk over the
// indices (j_t = (t A) mod N).  Three layouts of a cloud in the registers serve them: the cloud as
// given (index order), a copy in the order of the walk (positions are places in the walk), and a
// copy in the order of a Hilbert curve over a grid (cell order) -- there a wave's points lie in a
// small box, a pick is folded only into the waves it can affect, and a round's candidates are all
// available points of a window of indices (or places in the walk), settled together from the pairwise
// relations "comes before" and "lies closer than R_l" instead of one after the other.
//
// All floating point here must round every operation separately: the file is
// compiled with -ffp-contract=off and without packed fp32 instructions.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

#pragma clang fp contract(off)

namespace fastpoint {
namespace {

constexpr int kCand = kCandPerRound;    // candidates of an exact-FPS round (one per lane of the control wave)
constexpr float kPadCoord = 3.0e38f;    // coordinates of slots beyond N: every distance becomes +inf
constexpr uint32_t kNoIdx = 0xFFFFFFFFu;
constexpr int kStage = 512;             // ring of picks not yet written to global memory (a round adds up to kCandWin)
constexpr int kFlush = 128;             // ... written out once this many are waiting
constexpr int kCtrlThreads = 64;        // the control wave, after the T point threads
constexpr int kRkStride = 512 + kCtrlThreads;   // threads of a workgroup

// ---------------------------------------------------------------- wave helpers
// Values that are equal in all lanes but come out of LDS or cross-lane operations: telling the
// compiler so keeps the control flow that depends on them on the scalar unit.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint32_t uni(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ float unif(float v)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane((int)__float_as_uint(v)));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v)
{
    // every lane has a valid source for the controls used here, so bound_ctrl is irrelevant;
    // this form lets the compiler fuse the move into the following min/max
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, true);
}
// after these four steps every lane holds the reduction over its row of 16 lanes
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v)
{
    v = max(v, dpp<0xB1>(v));    // quad_perm [1,0,3,2]
    v = max(v, dpp<0x4E>(v));    // quad_perm [2,3,0,1]
    v = max(v, dpp<0x141>(v));   // row_half_mirror
    v = max(v, dpp<0x140>(v));   // row_mirror
    return v;
}
__device__ __forceinline__ uint32_t row_min_u32(uint32_t v)
{
    v = min(v, dpp<0xB1>(v));
    v = min(v, dpp<0x4E>(v));
    v = min(v, dpp<0x141>(v));
    v = min(v, dpp<0x140>(v));
    return v;
}
__device__ __forceinline__ uint32_t rdlane(uint32_t v, int l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, l);
}
__device__ __forceinline__ float rdlane_f(float v, int l)
{
    return __uint_as_float(rdlane(__float_as_uint(v), l));
}
// puts a wave-uniform value into lane `lane` of v
__device__ __forceinline__ void set_lane(uint32_t& v, int my_lane, int lane, uint32_t uniform_value)
{
    v = my_lane == lane ? uniform_value : v;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = row_max_u32(v);
    return max(max(rdlane(v, 0), rdlane(v, 16)), max(rdlane(v, 32), rdlane(v, 48)));     // scalar unit
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
    v = row_min_u32(v);
    return min(min(rdlane(v, 0), rdlane(v, 16)), min(rdlane(v, 32), rdlane(v, 48)));
}
// maximum over the wave as a scalar-unit value: the loop that uses it branches on it
__device__ __forceinline__ uint32_t smax(uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("s_max_u32 %0, %1, %2" : "=s"(r) : "s"(a), "s"(b) : "scc");
    return r;
}
__device__ __forceinline__ uint32_t wave_max_scalar(uint32_t v)
{
    v = row_max_u32(v);
    return smax(smax(rdlane(v, 0), rdlane(v, 16)), smax(rdlane(v, 32), rdlane(v, 48)));
}
// inclusive prefix sum over the lanes of a wave: inside a row of 16 lanes by shifts of 1, 2, 4, 8
// (a lane whose source lies outside its row adds 0), then the totals of the rows in front
__device__ __forceinline__ int wave_incl_sum(int v, int lane)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);    // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);    // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);    // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);    // row_shr:8
    const int r0 = (int)rdlane((uint32_t)v, 15), r1 = (int)rdlane((uint32_t)v, 31), r2 = (int)rdlane((uint32_t)v, 47);
    const int row = lane >> 4;
    return v + (row > 0 ? r0 : 0) + (row > 1 ? r1 : 0) + (row > 2 ? r2 : 0);
}
__device__ __forceinline__ int first_lane(uint64_t mask) { return __builtin_ctzll(mask); }
__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                          __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// squared distance, ((dx*dx)+(dy*dy))+(dz*dz), each operation rounded on its own
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

// ------------------------------------------------- words exchanged between workgroups
__device__ __forceinline__ void ll_store(uint64_t* p, uint32_t val, uint32_t stamp)
{
    __hip_atomic_store(p, ((uint64_t)stamp << 32) | (uint64_t)val, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ll_load(const uint64_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Waits until the NW words at p carry `stamp`; false if the wait limit expired.
template <int NWORDS>
__device__ __forceinline__ bool ll_wait(const uint64_t* p, uint32_t stamp, uint32_t (&val)[NWORDS],
                                        int64_t wait_ticks)
{
    int64_t t0 = 0;
    for (uint32_t spin = 0;; ++spin) {
        uint64_t v[NWORDS];
#pragma unroll
        for (int k = 0; k < NWORDS; ++k) v[k] = ll_load(p + k);
        bool ok = true;
#pragma unroll
        for (int k = 0; k < NWORDS; ++k) ok = ok && ((uint32_t)(v[k] >> 32) == stamp);
        if (ok) {
#pragma unroll
            for (int k = 0; k < NWORDS; ++k) val[k] = (uint32_t)v[k];
            return true;
        }
        if ((spin & 63u) == 63u || wait_ticks <= 0) {
            int64_t now = (int64_t)wall_clock64();
            if (t0 == 0) t0 = now;
            else if (now - t0 > wait_ticks) return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

// Slots in LDS through which the control wave hands the picks of a round to the point waves,
// in acceptance order.  A slot is one 64-bit word: low half = round tag << 9 | lane of the pick
// in the candidate list (kLiveEnd: the round has no further pick), high half = the pick's
// squared distance bits.  It is written by all lanes of the control wave with the same value (one
// 64-bit store); readers take the pick's coordinates from the candidate list.  The LDS executes
// the operations of one wave in issue order; the fences only restrain the compiler.
constexpr uint32_t kLiveMask = 0x1FFu;     // a round has up to 256 candidates
constexpr uint32_t kLiveEnd = kLiveMask;
constexpr int kLiveShift = 9;

__device__ __forceinline__ void lds_publish(uint64_t* p, uint32_t stamp, uint32_t dbits)
{
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __hip_atomic_store(p, ((uint64_t)dbits << 32) | stamp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}
// The control wave's position in the slot array and its round tag, both kept in vector registers
// (they are operands of vector instructions in every step of a loop whose length in
// instructions is what matters).
struct LiveCursor {
    uint32_t off, tag;
    __device__ __forceinline__ LiveCursor(uint32_t round_tag) : off(0), tag(round_tag)
    {
        asm volatile("" : "+v"(off), "+v"(tag));
    }
    __device__ __forceinline__ void publish(uint64_t* slots, uint32_t lane_or_end, uint32_t dbits)
    {
        lds_publish(reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(slots) + off), tag | lane_or_end, dbits);
        off += 8;
    }
};
// The low half of a slot (tag and candidate lane).  A 32-bit read on purpose: the unused high half of
// a 64-bit read would occupy a register that the next instructions reuse, and the wait for that
// would put the read of the slot and the read of the pick's coordinates one after the other.
__device__ __forceinline__ uint32_t lds_observe(const uint64_t* p)
{
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    const uint32_t v = __hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_WORKGROUP);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    return v;
}

struct Rec {          // one arg-max candidate: squared distance bits, index, coordinates
    uint32_t d, idx;
    float x, y, z;
    uint32_t fail;
    uint32_t pad0, pad1;
};

// A candidate or accepted pick: coordinates, index, squared distance bits.  The coordinates and
// the index are one aligned 16-byte quarter of the 32-byte record, so a lane that reads its own
// record takes them with one 128-bit LDS read (32-bit reads 32 bytes apart collide eight ways).
struct alignas(16) Cand {
    float x, y, z;
    uint32_t idx;
    uint32_t d;
    uint32_t pad0, pad1, pad2;
};

template <int T>
struct Shared {
    static constexpr int NW = T / 64;
    Rec wrec[2][NW];
    Rec win[2];
    float ring[64];
    float thr_meas[FP_MAX_SEG];
    float thr[FP_MAX_SEG];
    double terms[64];
    double powb[FP_MAX_SEG];
    int32_t level_start[FP_MAX_SEG];
    int32_t level_exhausted[FP_MAX_SEG];
    int32_t wcnt[NW];
    Cand cand[kCandWin];
    long long phase_t[5];      // constant 100 MHz clock at the phase boundaries of the cloud in hand (thread 0)
    Cand pend[kCand];
    int32_t bl[FP_MAX_SEG];    // segment boundaries b_l (curve positions that become thresholds)
    int32_t qend[FP_MAX_SEG + 1];   // qend[l] = ceil(n l / nseg): the quota rule raises the level to l + 1 there
    int32_t mlp_pos[32];       // MLP estimator: curve positions i_k of its 32 inputs (-1: not in use)
    float mlp_val[32];         // ... the curve there
    double mlp_a[128], mlp_b[128];   // ... activations of successive layers
    int32_t gpre[kMaxGroup + 1];
    uint16_t own[kCandWin];   // scan_candidates: the workgroup that lists the cloud's r-th candidate
    int32_t gtot[8];          // scan_candidates: totals of the (up to four) waves that add up the workgroups' counts
    int32_t ctrl[4];      // [0] accepted picks of the round, [1] points passing in the cloud,
                          // [2] failure, [3] distance bits of the last accepted pick
    // picks of the round being resolved, in acceptance order
    uint64_t live[kCandWin + 2];
    // scattered scan order: conf[2 c], conf[2 c + 1] = which candidates 0..63 / 64..127 of the round
    // lie closer than R_l to candidate c (bit j of the word: candidate j or 64 + j); acc[s] =
    // coordinates and index bits of the round's s-th accepted pick; progress = round number << 16 |
    // kRoundOver once the round has no further pick | picks in acc so far
    uint64_t conf[2 * kCandMax];
    float4 acc[kCandMax];
    // cell order: rel[j] = for candidate j of a window round, which candidates come before it in the
    // order of the sampling rule (words 0..3) and which of those lie closer to it than R_l (words 4..7);
    // took = the accepted candidates of the round, one bit each.  A row is nine words long, the last
    // unused: lane l of the control wave reads word w of candidate l (+ 64 q), and with rows of 64 bytes
    // the 64 lanes would meet in two pairs of LDS banks; with 72 bytes they spread over all of them.
    uint64_t rel[kCandWin][9];
    uint64_t took[kCandWin / 64];
    uint16_t place[kCandWin];  // ... and of each accepted one its place among the round's picks
    uint32_t progress;
#ifdef FASTPOINT_PHASE_CLOCKS
    long long chain_cycles;   // shader clocks the control wave spent in the exact-FPS chain loop
    long long chain_picks;
    long long scan_clk[8];    // wall-clock ticks of thread 0 in the parts of scan_candidates (threshold scans)
#endif
    uint32_t st_idx[kStage];   // picks waiting to be written out (ring, by sample position)
    float st_mdc[kStage];
};

// Everything one thread needs to know about where it sits.
struct Where {
    bool ctrl;            // the control wave (holds no points)
    int tid, lane, w;     // thread, lane, wave in workgroup
    int g, G, grp;        // workgroup in cloud, workgroups per cloud, group slot in the grid
    int gw;               // wave in cloud
    int c;                // cloud
    uint64_t* rows;       // recording kernels: this wave's [P][64] radius-test words in LDS
    uint32_t* rk;         // cell order with the scattered scan order: this thread's [P] places in the walk
                          // j_t = (t A) mod N, in LDS kRkStride words apart (looked at once per scan:
                          // in registers they would push other values out to scratch memory)
};

// P floats that stay in registers; element [p] with a wave-uniform p compiles to
// relative VGPR addressing, not to scratch memory
template <int P>
struct RegVec {
    typedef float type __attribute__((ext_vector_type(P)));
};

template <int P>
struct RegVecU {
    typedef uint32_t type __attribute__((ext_vector_type(P)));
};

template <int P, bool BQ>
struct Points {
    typename RegVec<P>::type x, y, z, d;
    typename RegVecU<P>::type oi;       // cell-ordered variant: the point's index in the caller's cloud
    float lox, loy, loz, hix, hiy, hiz; // cell-ordered variant: box of the wave's points (wave-uniform)
    uint32_t ub;                        // ... and an upper bound of their running distances (bits)
    // recording kernels: where this wave's next entry of the cloud's list goes.  [bq_cur, bq_lim) is
    // what is left of the chunk the wave is filling; bq_nxt holds (in lane 0) the number of the chunk
    // it has reserved for afterwards, asked for when the current one was taken, so that the answer
    // has long arrived when it is needed.
    uint32_t bq_cur, bq_lim, bq_nxt;
    bool bq_dead;                       // no chunk was left: nothing more is recorded for this cloud
};

// Cell-ordered variant: squared distance of a pick to the box of a wave's points, evaluated like
// dist2 with the nearest box coordinate per axis.  Rounding is monotone, so dist2 of every point
// of the wave is at least this value: a pick for which it is at least `ub` cannot lower any of the
// wave's distances, and folding it would change nothing.
template <int P, bool BQ>
struct Points;
template <int P, bool BQ>
__device__ __forceinline__ float box_dist2(const Points<P, BQ>& pt, float cx, float cy, float cz);

template <int P, bool BQ>
__device__ __forceinline__ float box_dist2(const Points<P, BQ>& pt, float cx, float cy, float cz)
{
    const float dx = fmaxf(fmaxf(pt.lox - cx, cx - pt.hix), 0.0f);
    const float dy = fmaxf(fmaxf(pt.loy - cy, cy - pt.hiy), 0.0f);
    const float dz = fmaxf(fmaxf(pt.loz - cz, cz - pt.hiz), 0.0f);
    float t = dx * dx;
    t = t + dy * dy;
    t = t + dz * dz;
    return t;
}

// Radius-test results of up to 64 picks that a wave has folded but not written to the cache
// yet: word [p][s] (one per slot p) of the s-th of those picks, in the wave's own part of LDS.
// A hit mask is wave-uniform, so it is stored by all lanes at one address (one instruction, no
// lane select); when the picks are written out lane s reads the words of pick s.  The LDS
// executes a wave's operations in issue order, so the wave needs no barrier between the two.
template <int P, bool BQ>
struct RowWords {
    uint64_t* row;
    __device__ __forceinline__ void clear(const Where& wh)
    {
        row = wh.rows;
        if constexpr (BQ) {
#pragma unroll
            for (int p = 0; p < P; ++p) row[p * 64 + wh.lane] = 0;
        }
    }
};

// The distance update of Alg. 1 for this thread's points; with BQ also the radius test of Section 4.2: the
// 64-bit hit mask of every slot goes to lane `s` of `rw`.  Most balls miss most waves of a large cloud:
// there is one test per group of slots on the vector unit (the minimum of the group's distances against
// the radius), and the per-slot masks are formed only when some point of the group hits.  How they
// are formed depends on how often that happens.  DENSE (a cloud held by few waves: nearly every ball
// reaches every wave): from the distances of the update, kept until the test.  Otherwise the
// distances are worked out once more in the rare branch: kept alive from the update they cost eight
// registers, and the compiler then moves every running distance of the thread from one register to
// another once per pick.  (The pick's coordinates pass through an empty asm statement there, so that
// the second evaluation is not merged with the first.)
template <int P, bool BQ, bool DENSE, int P0, bool REC>
__device__ __forceinline__ void fold_groups(Points<P, BQ>& pt, float cx, float cy, float cz, float bq_r2,
                                            int s, RowWords<P, BQ>& rw)
{
    constexpr int GRP = P < 8 ? P : 8;      // slots whose radius tests are examined together
    if constexpr (P0 < P) {
        uint32_t tb[GRP];                   // squared distances as bit patterns (>= +0: unsigned order)
        uint32_t tmin = 0xFFFFFFFFu;
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
            const int p = P0 + u;
            tb[u] = __float_as_uint(dist2(cx, cy, cz, pt.x[p], pt.y[p], pt.z[p]));
            pt.d[p] = __uint_as_float(min(__float_as_uint(pt.d[p]), tb[u]));
            if (BQ && REC) tmin = min(tmin, tb[u]);
        }
        if (BQ && REC) {
            const uint32_t r2b = __float_as_uint(bq_r2);
            if (__builtin_amdgcn_ballot_w64(tmin < r2b) != 0) {
                if constexpr (DENSE) {
#pragma unroll
                    for (int u = 0; u < GRP; ++u)
                        rw.row[(P0 + u) * 64 + s] = __builtin_amdgcn_ballot_w64(tb[u] < r2b);
                } else {
                    float hx = cx, hy = cy, hz = cz;
                    asm volatile("" : "+v"(hx), "+v"(hy), "+v"(hz));
#pragma unroll
                    for (int u = 0; u < GRP; ++u) {
                        const int p = P0 + u;
                        const uint32_t again = __float_as_uint(dist2(hx, hy, hz, pt.x[p], pt.y[p], pt.z[p]));
                        rw.row[p * 64 + s] = __builtin_amdgcn_ballot_w64(again < r2b);
                    }
                }
            }
        }
        fold_groups<P, BQ, DENSE, P0 + GRP, REC>(pt, cx, cy, cz, bq_r2, s, rw);
    }
}

// REC false: a pick of a recording kernel whose ball is known to miss every point of the wave
// (cell-ordered variant: the ball does not reach the wave's box) -- the update alone.
template <int P, bool BQ, bool DENSE = true, bool REC = true>
__device__ __forceinline__ void fold(Points<P, BQ>& pt, float cx, float cy, float cz,
                                     const SamplerArgs& a, const Where& wh, int s, RowWords<P, BQ>& rw)
{
    fold_groups<P, BQ, DENSE, 0, REC>(pt, cx, cy, cz, a.bq_r2, s, rw);
}

// Hands the words of `count` picks (sample positions base, base+1, ...; count <= 64; or, with
// my_offset >= 0, base + my_offset for the pick of this lane) to the cache.
// Lane s looks at the words of pick s; only a word that is not zero -- the ball holds one of the
// block's 64 points -- becomes an entry (sample, block, word) of the cloud's list.  A wave fills
// chunks of kBqChunk entries that it reserves from the cloud's chunk counter: the places inside a
// chunk come from ballots and bit counts, and the atomic addition that reserves the next chunk is
// issued when a chunk is taken and read when that chunk is full, so no wave ever waits for memory
// here (except for its very first entry of a cloud).  After every call lane 0 notes how much of the
// chunk is in use.  When no chunk is left the cloud's overflow flag is raised and the wave records
// nothing more: readers then treat the cloud as not recorded.
// (Kept in one piece: split into helpers for the chunk bookkeeping the index-ordered recorder of the
// million-point workload ran 3 % slower.)
template <int P, bool BQ>
__device__ __forceinline__ void flush_rows(const RowWords<P, BQ>& rw, const SamplerArgs& a, const Where& wh,
                                           Points<P, BQ>& pt, int base, int count, int my_offset = -1)
{
    if constexpr (BQ) {
        if (pt.bq_dead) return;
        const bool mine = wh.lane < count;
        uint64_t m[P];
        int total = 0;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int blk = wh.gw * P + p;              // slots wholly beyond N have no block
            const uint64_t w = rw.row[p * 64 + wh.lane];
            m[p] = __builtin_amdgcn_ballot_w64(mine && blk < a.bq_blocks && w != 0);
            total += __builtin_popcountll(m[p]);
        }
        if (total == 0) return;                         // uniform
        const uint32_t nchunks = (uint32_t)(a.bq_cap / kBqChunk);
        uint32_t* cursor = a.bq_cursor + wh.c;
        uint32_t* fill = a.bq_fill + (int64_t)wh.c * nchunks;
        BqRaw* __restrict__ list = a.bq_raw + (int64_t)wh.c * a.bq_cap;
        int done = 0;                                   // entries of this call that are placed (uniform)
        while (done < total) {
            if (pt.bq_cur == pt.bq_lim) {               // the chunk is full (or there is none yet)
                uint32_t ch;
                if (uni(pt.bq_nxt) == kBqNoChunk && pt.bq_lim == 0) {
                    // the wave's first entry of this cloud: two chunks at once
                    uint32_t c0 = 0;
                    if (wh.lane == 0) c0 = __hip_atomic_fetch_add(cursor, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ch = uni(c0);
                    pt.bq_nxt = ch + 1;
                } else {
                    ch = uni(pt.bq_nxt);
                    uint32_t c1 = 0;
                    if (wh.lane == 0) c1 = __hip_atomic_fetch_add(cursor, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    pt.bq_nxt = c1;                     // not looked at before the next chunk is needed
                }
                if (ch >= nchunks) {                    // the list is full
                    if (wh.lane == 0) a.bq_ovf[wh.c] = 1u;
                    pt.bq_dead = true;
                    return;
                }
                pt.bq_cur = ch * (uint32_t)kBqChunk;
                pt.bq_lim = pt.bq_cur + (uint32_t)kBqChunk;
            }
            const int room = (int)(pt.bq_lim - pt.bq_cur);
            const int take = total - done < room ? total - done : room;
            int before = 0;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (m[p] != 0) {
                    const int i = before + lanes_below(m[p]) - done;       // place among this turn's entries
                    if (((m[p] >> wh.lane) & 1ull) != 0 && i >= 0 && i < take) {
                        BqRaw e;
                        e.mask = rw.row[p * 64 + wh.lane];
                        e.blk = (uint32_t)(wh.gw * P + p);
                        e.q = (uint32_t)(base + (my_offset >= 0 ? my_offset : wh.lane));
                        list[pt.bq_cur + (uint32_t)i] = e;
                    }
                    before += __builtin_popcountll(m[p]);
                }
            }
            pt.bq_cur += (uint32_t)take;
            done += take;
            if (wh.lane == 0) fill[(pt.bq_lim - 1u) / (uint32_t)kBqChunk] = pt.bq_cur - (pt.bq_lim - (uint32_t)kBqChunk);
        }
    }
}

// Arg-max over the workgroup's points (lowest index among equals).  On return
// every thread of the workgroup holds the record of the workgroup's best point
// (G == 1) -- or wave 0 holds it (G > 1).
template <int T, int P, bool BQ, bool PERM>
__device__ __forceinline__ Rec wave_best(const Points<P, BQ>& pt, const Where& wh)
{
    uint32_t bits = __float_as_uint(pt.d[0]);          // distances are >= +0: unsigned order
    int bp = 0;
#pragma unroll
    for (int p = 1; p < P; ++p) {
        const uint32_t v = __float_as_uint(pt.d[p]);
        if (v > bits) {
            bits = v;
            bp = p;
        }
    }
    if constexpr (PERM) {
        // positions are in cell order: the lowest index of the caller's cloud among equal maxima
        uint32_t boi = pt.oi[0];
        bits = __float_as_uint(pt.d[0]);
        bp = 0;
#pragma unroll
        for (int p = 1; p < P; ++p) {
            const uint32_t v = __float_as_uint(pt.d[p]);
            if (v > bits || (v == bits && pt.oi[p] < boi)) {
                bits = v;
                boi = pt.oi[p];
                bp = p;
            }
        }
        const uint32_t wmax_p = wave_max_u32(bits);
        const uint32_t widx_p = wave_min_u32(bits == wmax_p ? boi : kNoIdx);
        const int wl_p = first_lane(__builtin_amdgcn_ballot_w64(bits == wmax_p && boi == widx_p));
        const int slot_p = (int)rdlane((uint32_t)bp, wl_p);
        Rec r;
        r.d = wmax_p;
        r.idx = widx_p;
        r.x = rdlane_f(pt.x[slot_p], wl_p);
        r.y = rdlane_f(pt.y[slot_p], wl_p);
        r.z = rdlane_f(pt.z[slot_p], wl_p);
        r.fail = 0;
        r.pad0 = r.pad1 = 0;
        return r;
    }
    const uint32_t wmax = wave_max_u32(bits);
    const uint32_t myj = (uint32_t)(((wh.gw * P + bp) << 6) | wh.lane);
    const uint32_t widx = wave_min_u32(bits == wmax ? myj : kNoIdx);
    const int slot = (int)(widx >> 6) - wh.gw * P;      // uniform
    const int wl = (int)(widx & 63u);
    const int slot_u = __builtin_amdgcn_readfirstlane(slot);
    const float sx = pt.x[slot_u], sy = pt.y[slot_u], sz = pt.z[slot_u];
    Rec r;
    r.d = wmax;
    r.idx = widx;
    r.x = rdlane_f(sx, wl);
    r.y = rdlane_f(sy, wl);
    r.z = rdlane_f(sz, wl);
    r.fail = 0;
    r.pad0 = r.pad1 = 0;
    return r;
}

// reduce `nrec` records held by lanes 0..nrec-1 of a wave (nrec <= 64)
__device__ __forceinline__ Rec reduce_recs(Rec r, bool valid)
{
    const uint32_t d = valid ? r.d : 0u;
    const uint32_t idx = valid ? r.idx : kNoIdx;
    const uint32_t dmax = wave_max_u32(d);
    const uint32_t imin = wave_min_u32((valid && d == dmax) ? idx : kNoIdx);
    const uint64_t who = __builtin_amdgcn_ballot_w64(valid && idx == imin);
    const int src = first_lane(who);
    Rec o;
    o.d = dmax;
    o.idx = imin;
    o.x = rdlane_f(r.x, src);
    o.y = rdlane_f(r.y, src);
    o.z = rdlane_f(r.z, src);
    o.fail = __builtin_amdgcn_ballot_w64(valid && r.fail != 0) != 0 ? 1u : 0u;
    o.pad0 = o.pad1 = 0;
    return o;
}

// One arg-max over the whole cloud.  `it` counts the reductions done so far in
// this kernel (LDS double buffering), `seq` the exchanges between workgroups.
template <int T, int P, bool BQ, bool PERM>
__device__ __forceinline__ Rec cloud_argmax(const Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                            const SamplerArgs& a, uint32_t& it, uint32_t& seq)
{
    constexpr int NW = T / 64;
    const int buf = (int)(it & 1u);
    ++it;
    Rec mine = wave_best<T, P, BQ, PERM>(pt, wh);
    if (wh.lane == 0 && !wh.ctrl) sh.wrec[buf][wh.w] = mine;
    __syncthreads();
    if (wh.G == 1) {
        Rec r = sh.wrec[buf][wh.lane < NW ? wh.lane : 0];
        return reduce_recs(r, wh.lane < NW);
    }
    ++seq;
    if (wh.w == 0) {
        Rec r = sh.wrec[buf][wh.lane < NW ? wh.lane : 0];
        Rec wg = reduce_recs(r, wh.lane < NW);
        const int par = (int)(seq & 1u);
        uint64_t* base = a.ll_pk + ((int64_t)(wh.grp * 2 + par) * wh.G) * kLlSlotWords;
        uint32_t v = wg.d;
        v = wh.lane == 1 ? wg.idx : v;
        v = wh.lane == 2 ? __float_as_uint(wg.x) : v;
        v = wh.lane == 3 ? __float_as_uint(wg.y) : v;
        v = wh.lane == 4 ? __float_as_uint(wg.z) : v;
        if (wh.lane < 5) ll_store(base + (int64_t)wh.g * kLlSlotWords + wh.lane, v, seq);
        Rec best;
        best.d = 0;
        best.idx = kNoIdx;
        best.x = best.y = best.z = 0.0f;
        best.fail = 0;
        best.pad0 = best.pad1 = 0;
        bool have = false;
        for (int t = wh.lane; t < wh.G; t += 64) {
            uint32_t val[5];
            bool ok = ll_wait<5>(base + (int64_t)t * kLlSlotWords, seq, val, a.wait_ticks);
            if (!ok) {
                best.fail = 1;
            } else if (!have || val[0] > best.d || (val[0] == best.d && val[1] < best.idx)) {
                best.d = val[0];
                best.idx = val[1];
                best.x = __uint_as_float(val[2]);
                best.y = __uint_as_float(val[3]);
                best.z = __uint_as_float(val[4]);
            }
            have = true;
        }
        Rec all = reduce_recs(best, have);
        if (wh.lane == 0) sh.win[buf] = all;
    }
    __syncthreads();
    return sh.win[buf];
}

// Picks are staged in LDS and written to global memory in blocks: a global store inside the
// iteration loop would make every iteration wait for the previous store to complete.
template <int T>
__device__ __forceinline__ void stage_pick(Shared<T>& sh, int pos, uint32_t idx, float d)
{
    sh.st_idx[pos & (kStage - 1)] = idx;
    sh.st_mdc[pos & (kStage - 1)] = d;
}

// Writes the staged picks [flushed, upto) when enough are waiting (or `force`).  Called by all
// threads of the workgroup at a point where they are converged.
template <int T, bool BQ>
__device__ __forceinline__ void flush_picks(const SamplerArgs& a, Shared<T>& sh, const Where& wh,
                                            int& flushed, int upto, bool force)
{
    if (upto - flushed < kFlush && !force) return;
    __syncthreads();
    if (wh.g == 0) {
        for (int t = flushed + wh.tid; t < upto; t += T + kCtrlThreads) {
            const uint32_t v = sh.st_idx[t & (kStage - 1)];
            a.out_idx[(int64_t)wh.c * a.n + t] = (int32_t)v;
            if (BQ) a.bq_idx[(int64_t)wh.c * a.n + t] = (int32_t)v;
            if (a.out_mdc) a.out_mdc[(int64_t)wh.c * a.n + t] = sh.st_mdc[t & (kStage - 1)];
        }
    }
    flushed = upto;
}

// x^e for an integer x >= 1 in binary64 using only + - * / (each correctly rounded
// by IEEE 754), in a fixed order: ln x from the atanh series after scaling x into
// [sqrt(1/2), sqrt(2)), then exp by its Taylor series after removing a multiple of ln 2.
// A CPU reference that performs the same operations in the same order gets the same bits.
__device__ __noinline__ double pow_int_base(int64_t x, double e)
{
    const double LN2 = 0.6931471805599453;
    int k = 63 - __builtin_clzll((unsigned long long)x);
    double f = (double)x * __longlong_as_double((long long)(1023 - k) << 52);   // exact, in [1,2)
    if (f > 1.4142135623730951) {
        f = f * 0.5;
        k = k + 1;
    }
    const double s = (f - 1.0) / (f + 1.0);
    const double s2 = s * s;
    double sum = 0.0;
    // unrolled: the quotients 1/(2t+1) are then constants (rounded correctly when the compiler folds
    // them, the bits the division gives at run time), and thirteen divisions go away
#pragma unroll
    for (int t = 12; t >= 0; --t) sum = sum * s2 + 1.0 / (double)(2 * t + 1);
    const double lnx = ((double)k * LN2) + ((2.0 * s) * sum);
    const double y = e * lnx;
    const double q = floor(y / LN2 + 0.5);
    const double r = y - q * LN2;
    double acc = 1.0;
#pragma unroll 1
    for (int t = 20; t >= 1; --t) acc = 1.0 + acc * (r / (double)t);
    return acc * __longlong_as_double((long long)(1023 + (int)q) << 52);
}

// Cell-ordered variant: which of the first `count` entries of `list` (one entry per lane) this
// wave has to fold -- those that can lower one of its distances and, in a recording kernel, those
// whose ball can reach into the wave's box.  `ball` gets the latter: only they need the radius test.
template <int P, bool BQ>
__device__ __forceinline__ uint64_t near_mask(const Points<P, BQ>& pt, const Cand* list, int count, int lane,
                                              float bq_r2, uint64_t& ball)
{
    const Cand c = list[lane < count ? lane : 0];
    const uint32_t bd = __float_as_uint(box_dist2<P, BQ>(pt, c.x, c.y, c.z));
    ball = BQ ? __builtin_amdgcn_ballot_w64(lane < count && bd < __float_as_uint(bq_r2)) : 0ull;
    return __builtin_amdgcn_ballot_w64(lane < count && bd < pt.ub) | ball;
}
template <int P, bool BQ>
__device__ __forceinline__ void refresh_bound(Points<P, BQ>& pt)
{
    uint32_t m = __float_as_uint(pt.d[0]);
#pragma unroll
    for (int p = 1; p < P; ++p) m = max(m, __float_as_uint(pt.d[p]));
    pt.ub = wave_max_u32(m);
}

// ln v for a normal positive binary64 v and exp y, with + - * / only in a fixed order (the steps
// pow_int_base is made of): a CPU reference performing the same operations gets the same bits.
__device__ __noinline__ double ln_fixed(double v)
{
    const double LN2 = 0.6931471805599453;
    const long long bits = __double_as_longlong(v);
    int k = (int)((bits >> 52) & 0x7FF) - 1023;
    double f = __longlong_as_double((bits & 0x000FFFFFFFFFFFFFll) | (1023ll << 52));   // in [1,2)
    if (f > 1.4142135623730951) {
        f = f * 0.5;
        k = k + 1;
    }
    const double s = (f - 1.0) / (f + 1.0);
    const double s2 = s * s;
    double sum = 0.0;
    // unrolled: the quotients 1/(2t+1) are then constants (rounded correctly when the compiler folds
    // them, the bits the division gives at run time), and thirteen divisions go away
#pragma unroll
    for (int t = 12; t >= 0; --t) sum = sum * s2 + 1.0 / (double)(2 * t + 1);
    return ((double)k * LN2) + ((2.0 * s) * sum);
}
__device__ __noinline__ double exp_fixed(double y)
{
    const double LN2 = 0.6931471805599453;
    if (!(y >= -700.0)) y = -700.0;
    if (y > 700.0) y = 700.0;
    const double q = floor(y / LN2 + 0.5);
    const double r = y - q * LN2;
    double acc = 1.0;
#pragma unroll 1
    for (int t = 20; t >= 1; --t) acc = 1.0 + acc * (r / (double)t);
    return acc * __longlong_as_double((long long)(1023 + (int)q) << 52);
}

// One layer of the MLP estimator: neuron `o` (of NOUT) starts from its bias and adds the products
// with the NIN inputs in ascending order; weights input-major, so the threads of a wave read
// adjacent words.
template <int NIN, int NOUT, bool RELU>
__device__ __forceinline__ void mlp_layer(const float* __restrict__ w, const float* __restrict__ bias,
                                          const double* in, double* out, int o)
{
    if (o >= NOUT) return;
    double acc = (double)bias[o];
#pragma unroll 4
    for (int k = 0; k < NIN; ++k) acc = acc + (double)w[k * NOUT + o] * in[k];
    out[o] = (RELU && !(acc > 0.0)) ? 0.0 : acc;
}

// Folds the picks waiting in sh.pend (sample positions base, base+1, ...) into the distances.
template <int T, int P, bool BQ, bool PERM>
__device__ __forceinline__ void fold_pending(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                             const SamplerArgs& a, int npend, int base)
{
    if (npend <= 0 || wh.ctrl) return;
    RowWords<P, BQ> rw;
    if constexpr (PERM) {
        uint64_t ball;
        uint64_t plain = near_mask<P, BQ>(pt, sh.pend, npend, wh.lane, a.bq_r2, ball) & ~ball;
        rw.row = wh.rows;
        while (plain != 0) {
            const int s = first_lane(plain);
            plain &= plain - 1;
            const Cand cur = sh.pend[s];
            fold<P, BQ, true, false>(pt, cur.x, cur.y, cur.z, a, wh, s, rw);
        }
        if (ball != 0) {                                // uniform
            rw.clear(wh);
            while (ball != 0) {
                const int s = first_lane(ball);
                ball &= ball - 1;
                const Cand cur = sh.pend[s];
                fold<P, BQ>(pt, cur.x, cur.y, cur.z, a, wh, s, rw);
            }
            flush_rows<P, BQ>(rw, a, wh, pt, base, npend);
        }
        return;
    }
    rw.clear(wh);
    Cand nxt = sh.pend[0];
    for (int s = 0; s < npend; ++s) {                   // npend <= kCand
        const Cand cur = nxt;
        if (s + 1 < npend) nxt = sh.pend[s + 1];       // fetched while the current pick is folded
        fold<P, BQ>(pt, cur.x, cur.y, cur.z, a, wh, s, rw);
    }
    flush_rows<P, BQ>(rw, a, wh, pt, base, npend);
}

// The point waves' side of a round that the control wave resolves: folds the picks (sample
// positions base, base+1, ...) as they are published, until the slot that closes the round.
// The next slot is requested before the current pick is folded.  Cell-ordered variant: the
// candidates of the round (`total` of them) are tested against the wave's box once, all
// together; a published pick that is not near is passed over.
template <int T, int P, bool BQ, bool PERM, int NQ>
__device__ __forceinline__ void follow_picks(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                             const SamplerArgs& a, int base, uint32_t tag, int total)
{
    int s = 0;
    RowWords<P, BQ> rw;
    uint64_t near[NQ], ball[NQ];                    // one bit per candidate (word q: candidates 64 q ...)
    uint64_t anyball = 0;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        near[q] = ball[q] = ~0ull;
        if constexpr (PERM) near[q] = near_mask<P, BQ>(pt, sh.cand + 64 * q, total - 64 * q, wh.lane, a.bq_r2, ball[q]);
        anyball |= ball[q];
    }
    // a cell-ordered wave records only when the ball of some candidate reaches its box
    const bool records = BQ && anyball != 0;
    rw.row = wh.rows;
    if (records) rw.clear(wh);
    uint32_t slot = lds_observe(&sh.live[0]);
    // Lane s of `rw` holds the words of a pick, so a recording wave takes a round of more than 64
    // candidates in parts of up to 64 picks and hands a part's words over before the next; that
    // hand-over is kept out of the loop over the picks (whatever is written there would be carried,
    // and copied, through every iteration).
    constexpr int kParts = BQ ? NQ : 1;
    bool ended = false;
    int handed = 0;                                 // picks whose words the record has
#pragma unroll 1
    for (int part = 0; part < kParts && !ended; ++part) {
        const int stop = kParts > 1 ? 64 * (part + 1) : 0x7FFFFFFF;
        if (part >= 1 && records) rw.clear(wh);
        for (;;) {
            // wait for slot s of this round (requested before the previous pick was folded); nothing
            // but the slot changes in the inner loop, so the distances and row words stay where they
            // are across it
            slot = uni(slot);
            while ((slot & ~kLiveMask) != tag) {    // not written yet in this round
                __builtin_amdgcn_s_sleep(1);
                slot = uni(lds_observe(&sh.live[s]));
            }
            if ((slot & kLiveMask) == kLiveEnd) {
                ended = true;
                break;
            }
            if (s == stop) break;                   // the slot stays in hand for the next part
            const uint32_t cl = slot & kLiveMask;
            slot = lds_observe(&sh.live[s + 1]);
            uint64_t nword = near[0], bword = ball[0];
#pragma unroll
            for (int q = 1; q < NQ; ++q) {
                nword = (cl >> 6) == (uint32_t)q ? near[q] : nword;
                bword = (cl >> 6) == (uint32_t)q ? ball[q] : bword;
            }
            if (!PERM || ((nword >> (cl & 63u)) & 1ull) != 0) {
                const Cand c = sh.cand[cl];
                // narrow rounds are those of clouds held by one or a few workgroups
                if (!(PERM && BQ) || ((bword >> (cl & 63u)) & 1ull) != 0)
                    fold<P, BQ, NQ == 1>(pt, c.x, c.y, c.z, a, wh, kParts > 1 ? (s & 63) : s, rw);
                else
                    fold<P, BQ, NQ == 1, false>(pt, c.x, c.y, c.z, a, wh, 0, rw);
            }
            ++s;
        }
        // the words of this part's picks (the one place where they are handed over: the code is long)
        if (records) flush_rows<P, BQ>(rw, a, wh, pt, base + handed, s - handed);
        handed = s;
    }
}

// segment boundary b_l (curve index whose value becomes R_l), l = 1..nseg
__device__ __forceinline__ int boundary_index(int n, int nseg, int l)
{
    int64_t b = ((int64_t)n * l) / nseg;
    b = b < 1 ? 1 : b;
    b = b > n - 1 ? n - 1 : b;
    return (int)b;
}

// Optional phase timing for tuning (-DFASTPOINT_PHASE_CLOCKS): wall-clock ticks spent in
// fold / scan / resolve / plain picks, reported in info.thr2[8..11] (microseconds).
#ifdef FASTPOINT_PHASE_CLOCKS
#define PHASE_BEGIN() const long long phase_t0__ = wall_clock64()
#define PHASE_END(st, k) (st).clk[k] += wall_clock64() - phase_t0__
#else
#define PHASE_BEGIN() do { } while (0)
#define PHASE_END(st, k) do { } while (0)
#endif

// Progress of one cloud; every field is uniform over all workgroups of the cloud.
struct CloudState {
    int i;          // next sample position to fill
    int npend;      // picks in sh.pend that are not folded into the distances yet
    int flushed;    // sample positions [0, flushed) are in global memory
    int rounds;     // candidate scans so far
    int resolved;   // rounds the control wave has resolved; the next round's slots carry resolved + 1
    float dlast;    // squared distance of the last exact-FPS pick at pick time; < 0: unknown
    float om;       // an exact-FPS round takes the points above dlast * (1 - om) as candidates
    int my_bl;      // thread l < nseg: segment boundary b_(l+1); else -1
#ifdef FASTPOINT_PHASE_CLOCKS
    long long clk[12];
#endif
};

// Curve capture of the prefix (the prefix loop of Alg. 2), by the lanes of one wave.
template <int T>
__device__ __forceinline__ void capture_curve(Shared<T>& sh, const Where& wh, const CloudState& st, int pos,
                                              float d)
{
    if (wh.tid == 0) sh.ring[pos & 63] = d;
    if (st.my_bl == pos) sh.thr_meas[wh.tid] = d;
    if (wh.tid < 32 && sh.mlp_pos[wh.tid] == pos) sh.mlp_val[wh.tid] = d;
}

// One plain iteration of Alg. 1 (distance update, arg-max) on distances that are already up to date:
// arg-max over the cloud, lowest index among equals.  Always makes progress; the batched
// rounds below fall back to it.  Returns false if a wait between workgroups expired.
template <int T, int P, bool BQ, bool PERM>
__device__ __forceinline__ bool plain_pick(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                           const SamplerArgs& a, uint32_t& it, uint32_t& seq,
                                           CloudState& st, bool capture)
{
    const Rec r = cloud_argmax<T, P, BQ, PERM>(pt, sh, wh, a, it, seq);
    if (uni(r.fail)) return false;
    const float dpick = __uint_as_float(uni(r.d));
    if (wh.tid == 0) {
        stage_pick<T>(sh, st.i, r.idx, dpick);
        Cand c;
        c.idx = r.idx;
        c.x = r.x;
        c.y = r.y;
        c.z = r.z;
        c.d = r.d;
        sh.pend[0] = c;
    }
    if (capture && wh.w == 0) capture_curve<T>(sh, wh, st, st.i, dpick);
    __syncthreads();
    st.npend = 1;
    st.dlast = dpick;
    ++st.i;
    return true;
}

// Whether slot p of this thread passes a scan: distance d > thr (STRICT) or d >= thr, and (WIN,
// cell-ordered variant) the point's own index -- RK: its place in the walk of the scattered scan
// order -- lies in [win_lo, win_lo + win_len).
template <int P, bool BQ, bool STRICT, bool WIN, bool RK>
__device__ __forceinline__ bool passes(const Points<P, BQ>& pt, const uint32_t* rk, int p, float thr,
                                       uint32_t win_lo, uint32_t win_len)
{
    const bool av = STRICT ? (pt.d[p] > thr) : (pt.d[p] >= thr);
    if constexpr (WIN) return av && (uint32_t)((RK ? rk[p * kRkStride] : pt.oi[p]) - win_lo) < win_len;
    return av;
}

// Collects the cloud's first CAP points (in the order the workgroups hold them: ascending index,
// or cell order in the cell-ordered variant) that pass -- see passes() -- into sh.cand of every
// workgroup (RK: with the point's place in the walk instead of its distance).  Returns the number
// collected (at most CAP), -1 if a wait expired; `alltot` receives the number of points that pass
// in the whole cloud.  With several workgroups each hands on at most PUB of its own: when the
// number returned is below both CAP and `alltot`, some workgroup held more than that.
template <int T, int P, bool BQ, bool PERM, bool STRICT, int CAP, bool WIN = false, bool RK = false,
          int PUB = CAP>
__device__ __forceinline__ int scan_candidates(const Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                               const SamplerArgs& a, uint32_t& seq, float thr, int& alltot,
                                               uint32_t win_lo = 0, uint32_t win_len = 0)
{
    constexpr int NW = T / 64;
    // Cell-ordered kernels (they sit at the register limit): lane and thread number as values the
    // compiler knows nothing about, so that the addresses below are formed here instead of being
    // carried through the kernel (see settle_relations).  The others have the registers, and there
    // the known values save instructions.
    int lane = wh.lane, tid = wh.tid;
    if constexpr (PERM) asm volatile("" : "+v"(lane), "+v"(tid));
    // 1. how many of this wave's points pass
#ifdef FASTPOINT_PHASE_CLOCKS
    long long sc_t = wall_clock64();
#define SCAN_MARK(k) do { if (!STRICT && tid == 0) { const long long now__ = wall_clock64(); sh.scan_clk[k] += now__ - sc_t; sc_t = now__; } } while (0)
#else
#define SCAN_MARK(k) do { } while (0)
#endif
    int cntw = 0;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const bool av = passes<P, BQ, STRICT, WIN, RK>(pt, wh.rk, p, thr, win_lo, win_len);
        cntw += __builtin_popcountll(__builtin_amdgcn_ballot_w64(av));
    }
    if (lane == 0 && !wh.ctrl) sh.wcnt[wh.w] = cntw;     // the control wave has none (cntw == 0)
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        const int v = sh.wcnt[k];
        off += (k < wh.w) ? v : 0;
        tot += v;
    }
    off = uni(off);
    tot = uni(tot);
    // 2. the workgroup's first CAP of them, in index order
    if (cntw > 0 && off < CAP) {
        int base = off;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const bool av = passes<P, BQ, STRICT, WIN, RK>(pt, wh.rk, p, thr, win_lo, win_len);
            const uint64_t mk = __builtin_amdgcn_ballot_w64(av);
            if (mk != 0 && base < CAP) {
                const int rank = base + lanes_below(mk);
                if (av && rank < CAP) {
                    Cand cd;
                    cd.idx = PERM ? pt.oi[p] : (uint32_t)(((wh.gw * P + p) << 6) | lane);
                    cd.x = pt.x[p];
                    cd.y = pt.y[p];
                    cd.z = pt.z[p];
                    // (a threshold round does not look at a candidate's distance: RK puts the place in the walk there)
                    cd.d = RK ? wh.rk[p * kRkStride] : __float_as_uint(pt.d[p]);
                    sh.cand[rank] = cd;
                }
                base += __builtin_popcountll(mk);
            }
        }
    }
    __syncthreads();
    SCAN_MARK(0);
    int total = tot < CAP ? tot : CAP;
    alltot = tot;
    if (wh.G == 1) return total;

    // 3. exchange: every workgroup publishes its list, all take the first CAP of the cloud
    //    in workgroup (= index) order
    //    (lists CAP entries apart: a word is only taken with this round's stamp, so rounds of
    //    different CAP may lay the same buffer out differently)
    ++seq;
    const int par = (int)(seq & 1u);
    uint64_t* cd = a.ll_cd + ((int64_t)(wh.grp * 2 + par) * wh.G) * (kCandMax * kCandWords);
    static_assert(PUB <= CAP && PUB <= kCandMax, "a workgroup's list in the exchange buffer holds kCandMax entries");
    static_assert(CAP <= kCandWin, "sh.own holds one entry per candidate of a round");
    const int publish = tot < PUB ? tot : PUB;     // (PUB < CAP: a workgroup hands on at most PUB of its own)
    for (int e = tid; e < publish * kCandWords; e += T + kCtrlThreads) {
        const int r = e / kCandWords, k = e - r * kCandWords;
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&sh.cand[r]);
        ll_store(cd + ((int64_t)wh.g * PUB + r) * kCandWords + k, src[k], seq);
    }
    // (the counts of the cloud's workgroups lie side by side: a wave that waits for 64 of them touches
    // eight lines of memory, not 64)
    uint64_t* ct = a.ll_ct + (int64_t)(wh.grp * 2 + par) * wh.G;
    if (tid == 0) ll_store(ct + wh.g, (uint32_t)tot, seq);
    __syncthreads();          // sh.cand is about to be overwritten
    SCAN_MARK(1);
    // Thread t waits for the count of workgroup t, so that all waits are in flight together.  The
    // prefix sums over the workgroups (gpre[t]: entries listed by the workgroups in front of t, a
    // workgroup lists at most PUB) are formed by the waves that hold the counts: inside a wave by lane
    // shifts, across the (at most four) waves through their totals in LDS.  Up to 64 workgroups wave 0
    // does it alone, which saves a barrier.
    int v = 0;
    bool bad = false;
    if (tid < wh.G) {
        uint32_t val[1];
        if (ll_wait<1>(ct + tid, seq, val, a.wait_ticks)) v = (int)val[0];
        else bad = true;
    }
    const int c = v < PUB ? v : PUB;
    const int nwv = (wh.G + 63) >> 6;                  // waves that hold counts (uniform)
    static_assert(kMaxGroup <= 256, "the totals of four waves");
    int incl = 0, uincl = 0;
    if (wh.w < nwv) {                                  // wave-uniform
        incl = wave_incl_sum(c, lane);
        uincl = wave_incl_sum(v, lane);
        if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) sh.ctrl[2] = 1;
    }
    if (nwv > 1) {
        if (wh.w < nwv && lane == 63) {
            sh.gtot[wh.w] = incl;
            sh.gtot[4 + wh.w] = uincl;
        }
        __syncthreads();
        SCAN_MARK(2);
    }
    if (wh.w < nwv) {
        int base = 0, ubase = 0;
        if (nwv > 1) {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                if (k < wh.w) {
                    base += sh.gtot[k];
                    ubase += sh.gtot[4 + k];
                }
            }
        }
        if (tid < wh.G) {
            // which workgroup lists the cloud's r-th candidate, for the first CAP of them
            const int first = base + incl - c;
            sh.gpre[tid] = first;
            for (int r = first; r < first + c && r < CAP; ++r) sh.own[r] = (uint16_t)tid;
        }
        if (tid == wh.G - 1) {
            sh.gpre[wh.G] = base + incl;
            sh.ctrl[1] = ubase + uincl;
        }
    }
    __syncthreads();
    SCAN_MARK(3);
    alltot = uni(sh.ctrl[1]);
    const int listed = uni(sh.gpre[wh.G]);
    total = listed < CAP ? listed : CAP;
    if (uni(sh.ctrl[2]) == 0) {
        // a thread fetches up to NE words of the list: all of them are requested before the first is
        // looked at (a word that has not arrived yet is then waited for on its own)
        constexpr int NE = (CAP * kCandWords + T + kCtrlThreads - 1) / (T + kCtrlThreads);
        const uint64_t* src[NE];
        uint64_t got[NE];
#pragma unroll
        for (int u = 0; u < NE; ++u) {
            const int e = tid + u * (T + kCtrlThreads);
            src[u] = nullptr;
            if (e < total * kCandWords) {
                const int r = e / kCandWords, k = e - r * kCandWords;
                const int lo = (int)sh.own[r];  // workgroup whose range holds rank r
                src[u] = cd + ((int64_t)lo * PUB + (r - sh.gpre[lo])) * kCandWords + k;
            }
        }
#pragma unroll
        for (int u = 0; u < NE; ++u) got[u] = src[u] ? ll_load(src[u]) : 0;
#pragma unroll
        for (int u = 0; u < NE; ++u) {
            if (src[u]) {
                const int e = tid + u * (T + kCtrlThreads);
                uint32_t val[1];
                val[0] = (uint32_t)got[u];
                if ((uint32_t)(got[u] >> 32) != seq && !ll_wait<1>(src[u], seq, val, a.wait_ticks)) sh.ctrl[2] = 1;
                reinterpret_cast<uint32_t*>(&sh.cand[e / kCandWords])[e % kCandWords] = val[0];
            }
        }
    }
    __syncthreads();
    SCAN_MARK(4);
    return uni(sh.ctrl[2]) != 0 ? -1 : total;
}

// Threshold phase of Alg. 2 (list clearing and findAnyOne for up to kCandMax picks at once): the candidates are
// taken in index order; one stays available iff no pick accepted before it in this round lies
// closer than R_l.  Run by the control wave of every workgroup (all do the same work), lane l
// holding candidates l and 64 + l; each accepted pick is published at once for the point waves
// to fold.
template <int T, bool WIDE>
__device__ __forceinline__ void resolve_threshold(Shared<T>& sh, const Where& wh, const CloudState& st,
                                                  int total, int limit, float r2, uint32_t tag)
{
    total = uni(total);
    limit = uni(limit);
    const bool has0 = wh.lane < total;
    const bool has1 = WIDE && wh.lane + 64 < total;
    const bool two = WIDE && total > 64;           // uniform
    const Cand me0 = sh.cand[has0 ? wh.lane : 0];
    Cand me1 = me0;
    if constexpr (WIDE) me1 = sh.cand[has1 ? wh.lane + 64 : 0];
    uint64_t alive0 = __builtin_amdgcn_ballot_w64(has0);
    uint64_t alive1 = 0;
    if constexpr (WIDE) alive1 = __builtin_amdgcn_ballot_w64(has1);
    int nacc = 0;
    LiveCursor cur(tag);
    __builtin_amdgcn_s_setprio(3);
    asm volatile("" ::"v"(me0.x), "v"(me0.y), "v"(me0.z));
    if constexpr (WIDE) asm volatile("" ::"v"(me1.x), "v"(me1.y), "v"(me1.z));
    while (alive0 != 0 && nacc < limit) {          // candidates 0..63 come first in index order
        const int cl = first_lane(alive0);
        const float ax = rdlane_f(me0.x, cl), ay = rdlane_f(me0.y, cl), az = rdlane_f(me0.z, cl);
        cur.publish(sh.live, (uint32_t)cl, 0u);
        const float t0 = dist2(ax, ay, az, me0.x, me0.y, me0.z);
        const uint64_t kill = __builtin_amdgcn_ballot_w64(t0 < r2);     // includes the pick itself
        alive0 &= ~kill;
        alive0 &= ~(1ull << cl);
        if constexpr (WIDE) {
            if (two) {
                const float t1 = dist2(ax, ay, az, me1.x, me1.y, me1.z);
                alive1 &= ~__builtin_amdgcn_ballot_w64(t1 < r2);
            }
        }
        nacc = uni(nacc + 1);
    }
    if constexpr (WIDE) {
        while (alive1 != 0 && nacc < limit) {
            const int cl = first_lane(alive1);
            const float ax = rdlane_f(me1.x, cl), ay = rdlane_f(me1.y, cl), az = rdlane_f(me1.z, cl);
            cur.publish(sh.live, (uint32_t)(64 + cl), 0u);
            const float t1 = dist2(ax, ay, az, me1.x, me1.y, me1.z);
            alive1 &= ~__builtin_amdgcn_ballot_w64(t1 < r2);
            alive1 &= ~(1ull << cl);
            nacc = uni(nacc + 1);
        }
    }
    cur.publish(sh.live, kLiveEnd, 0u);
    __builtin_amdgcn_s_setprio(0);
    if constexpr (WIDE) {
        for (int t = wh.lane; t < nacc; t += 64) {
            const uint32_t cl = (uint32_t)sh.live[t] & kLiveMask;
            stage_pick<T>(sh, st.i + t, sh.cand[cl].idx, 0.0f);
        }
    } else if (wh.lane < nacc) {
        const uint32_t cl = (uint32_t)sh.live[wh.lane] & kLiveMask;
        stage_pick<T>(sh, st.i + wh.lane, sh.cand[cl].idx, 0.0f);
    }
    if (wh.lane == 0) sh.ctrl[0] = nacc;
}

// ---- Threshold rounds of the scattered scan order.  Whether a candidate of the round stays
// available depends only on a yes/no relation between candidates -- "lies closer than R_l" -- so the
// relation is worked out first, by all waves of the workgroup side by side, and the picks are then
// resolved from its bits alone.  (With the scan in index order few candidates of a round survive and
// this costs more than it saves; with the scattered order most of them do.)
//
// build_conflicts: wave w takes candidates w, w + NW + 1, ...; candidate c is read by all lanes
// (one broadcast), lane j tests it against candidates j and 64 + j, and the two ballots are row c
// of the relation.  dist2 gives the same bits with its points exchanged, so row c is also what
// the fold of pick c will find for the other candidates.  Called by all threads; the rows are
// complete after the next barrier.
constexpr uint32_t kRoundOver = 0x8000u;

template <int T>
__device__ __forceinline__ void build_conflicts(Shared<T>& sh, const Where& wh, int total, float r2)
{
    constexpr int NWALL = T / 64 + 1;              // the control wave takes its share
    total = uni(total);
    const bool has0 = wh.lane < total;
    const bool has1 = wh.lane + 64 < total;
    const bool two = total > 64;                   // uniform
    const Cand me0 = sh.cand[has0 ? wh.lane : 0];
    const Cand me1 = sh.cand[has1 ? wh.lane + 64 : 0];
    for (int c = wh.w; c < total; c += NWALL) {
        const Cand pk = sh.cand[c];
        const float t0 = dist2(pk.x, pk.y, pk.z, me0.x, me0.y, me0.z);
        const uint64_t k0 = __builtin_amdgcn_ballot_w64(has0 && t0 < r2);
        uint64_t k1 = 0;
        if (two) {
            const float t1 = dist2(pk.x, pk.y, pk.z, me1.x, me1.y, me1.z);
            k1 = __builtin_amdgcn_ballot_w64(has1 && t1 < r2);
        }
        if (wh.lane == 0) {
            sh.conf[2 * c] = k0;
            sh.conf[2 * c + 1] = k1;
        }
    }
}

__device__ __forceinline__ uint64_t rdlane64(uint64_t v, int l)
{
    return ((uint64_t)rdlane((uint32_t)(v >> 32), l) << 32) | (uint64_t)rdlane((uint32_t)v, l);
}

__device__ __forceinline__ void progress_publish(uint32_t* p, uint32_t v)
{
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}
__device__ __forceinline__ uint32_t progress_observe(const uint32_t* p)
{
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    const uint32_t v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    return v;
}

// resolve_conflicts: the candidates are taken in the order of the list; one stays available iff no
// pick accepted before it in this round lies closer than R_l.  Run by the control wave of every
// workgroup (all do the same work): lane l keeps rows l and 64 + l of the relation in registers, the
// set of candidates still available is two scalar 64-bit words, and a step is "lowest set bit,
// fetch its row from the lane that holds it, clear the row's bits" -- no arithmetic on the chain.
// The lane that holds an accepted candidate appends its coordinates to sh.acc, then the count in
// sh.progress goes up: the point waves fold whatever the count covers.
template <int T>
__device__ __forceinline__ void resolve_conflicts(Shared<T>& sh, const Where& wh, const CloudState& st,
                                                  int total, int limit, uint32_t round_no)
{
    total = uni(total);
    limit = uni(limit);
    const bool two = total > 64;                   // uniform
    const bool has0 = wh.lane < total;
    const bool has1 = wh.lane + 64 < total;
    const Cand me0 = sh.cand[has0 ? wh.lane : 0];
    const Cand me1 = sh.cand[has1 ? wh.lane + 64 : 0];
    const uint64_t r00 = sh.conf[2 * wh.lane], r01 = sh.conf[2 * wh.lane + 1];
    const uint64_t r11 = sh.conf[2 * (64 + wh.lane) + 1];
    // (rows of lanes at or beyond `total` are left-overs of earlier rounds: never selected)
    uint64_t alive0 = total >= 64 ? ~0ull : ((1ull << total) - 1ull);
    uint64_t alive1 = !two ? 0ull : (total >= 128 ? ~0ull : ((1ull << (total - 64)) - 1ull));
    int nacc = 0;
    const uint32_t word = round_no << 16;
    __builtin_amdgcn_s_setprio(3);
    asm volatile("" ::"v"(r00), "v"(r01), "v"(r11), "v"(me0.x), "v"(me1.x));   // arrived before the loop starts
    while (alive0 != 0 && nacc < limit) {          // candidates 0..63 come first
        const int cl = first_lane(alive0);
        if (wh.lane == cl) sh.acc[nacc] = make_float4(me0.x, me0.y, me0.z, __uint_as_float(me0.idx));
        nacc = uni(nacc + 1);
        progress_publish(&sh.progress, word | (uint32_t)nacc);
        alive0 &= ~rdlane64(r00, cl);              // includes the pick itself (0 < R_l^2) ...
        alive0 &= ~(1ull << cl);                   // ... whatever the threshold
        if (two) alive1 &= ~rdlane64(r01, cl);
    }
    while (alive1 != 0 && nacc < limit) {
        const int cl = first_lane(alive1);
        if (wh.lane == cl) sh.acc[nacc] = make_float4(me1.x, me1.y, me1.z, __uint_as_float(me1.idx));
        nacc = uni(nacc + 1);
        progress_publish(&sh.progress, word | (uint32_t)nacc);
        alive1 &= ~rdlane64(r11, cl);
        alive1 &= ~(1ull << cl);
    }
    progress_publish(&sh.progress, word | kRoundOver | (uint32_t)nacc);
    __builtin_amdgcn_s_setprio(0);
    for (int t = wh.lane; t < nacc; t += 64) stage_pick<T>(sh, st.i + t, __float_as_uint(sh.acc[t].w), 0.0f);
    if (wh.lane == 0) sh.ctrl[0] = nacc;
}

// The point waves' side of such a round: folds the picks of sh.acc up to the published count, looks
// at the count again, and so on until the round is over.  No wait per pick: the control wave is far
// ahead after the first few picks.
template <int T, int P, bool BQ>
__device__ __forceinline__ void follow_stream(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                              const SamplerArgs& a, uint32_t round_no)
{
    static_assert(!BQ, "the scattered scan order does not record");
    RowWords<P, BQ> rw;
    rw.clear(wh);
    int done = 0;
    for (;;) {
        uint32_t pr = uni(progress_observe(&sh.progress));
        while ((pr >> 16) != round_no || (int)(pr & 0xFFu) == done) {     // not of this round, or nothing new
            if ((pr >> 16) == round_no && (pr & kRoundOver) != 0) return;
            __builtin_amdgcn_s_sleep(1);
            pr = uni(progress_observe(&sh.progress));
        }
        const int cnt = (int)(pr & 0xFFu);
        for (int s = done; s < cnt; ++s) {
            const float4 c = sh.acc[s];
            fold<P, BQ>(pt, c.x, c.y, c.z, a, wh, 0, rw);
        }
        done = cnt;
        if ((pr & kRoundOver) != 0) return;
    }
}

// ---- Threshold rounds of the cell-ordered variant.  The candidates of a round are ALL available
// points of a window of keys (the point's index, or with the scattered scan order its place in the
// walk), up to kCandWin of them, in no particular order.  Taking them one after the other in key
// order, one is accepted iff no candidate accepted before it lies closer than R_l.  That is settled
// without walking through them:
//
// build_relations (all waves): for candidate j, which candidates have a lower key (`before`) and
// which of those lie closer than R_l (`blockers`), as bit sets over the candidate list.  Lane l
// holds candidates l, 64 + l, ...; a wave takes one j at a time, reads it with one broadcast, and
// each test over the list is a ballot.  dist2 gives the same bits with its points
// exchanged, so a blocker bit is also what the fold of that pick will find for candidate j.
//
// settle_relations (control wave): a candidate all of whose blockers are rejected is accepted, one
// with an accepted blocker is rejected; repeated until none is undecided.  The undecided candidate
// with the lowest key is decided in every sweep (its blockers all are), so the sweeps end, and
// they are as many as the longest chain of candidates each waiting for the one before -- a
// handful when neighbours in key order are not neighbours in space.  The place of an accepted
// candidate in the output is the number of accepted candidates before it; those from place `limit`
// on are dropped (the level's quota ends the round there).
constexpr int kWinWords = kCandWin / 64;

constexpr int kRelWords = 4 * kWinWords;           // 32-bit words of a candidate's two bit sets

template <int T, bool BYD>
__device__ __forceinline__ void build_relations(Shared<T>& sh, const Where& wh, const SamplerArgs& a,
                                                uint32_t seq, int total, float r2)
{
    constexpr int NWALL = T / 64 + 1;              // the control wave takes its share
    total = uni(total);
    const int nq = (total + 63) >> 6;              // uniform
    // lane and thread number as values the compiler knows nothing about, so that the addresses below
    // are formed here instead of being carried through the kernel (see settle_relations)
    int lane = wh.lane, tid = wh.tid;
    asm volatile("" : "+v"(lane), "+v"(tid));
    Cand me[kWinWords];
#pragma unroll
    for (int q = 0; q < kWinWords; ++q) {
        const int c = lane + 64 * q;
        me[q] = sh.cand[c < total ? c : 0];
    }
    // With several workgroups every one of them works out the sets of the candidates g, g + G, ...
    // only and hands them to the others through stamped words (as the candidates themselves came).
    const int first = wh.G == 1 ? wh.w : wh.g + wh.G * wh.w;
    const int step = wh.G == 1 ? NWALL : wh.G * NWALL;
    uint64_t* buf = wh.G == 1 ? nullptr : a.ll_rel + (int64_t)(wh.grp * 2 + (int)(seq & 1u)) * (kCandWin * kRelWords);
    for (int j = first; j < total; j += step) {
        const Cand pj = sh.cand[j];
        const uint32_t kj = BYD ? pj.d : pj.idx;
        uint32_t pay = 0;                           // lane l: word l of (before, blockers)
#pragma unroll
        for (int q = 0; q < kWinWords; ++q) {
            uint64_t before = 0, blockers = 0;
            if (q < nq) {
                const bool earlier = lane + 64 * q < total && (BYD ? me[q].d : me[q].idx) < kj;
                const float t = dist2(pj.x, pj.y, pj.z, me[q].x, me[q].y, me[q].z);
                before = __builtin_amdgcn_ballot_w64(earlier);
                blockers = __builtin_amdgcn_ballot_w64(earlier && t < r2);
            }
            set_lane(pay, lane, 2 * q, (uint32_t)before);
            set_lane(pay, lane, 2 * q + 1, (uint32_t)(before >> 32));
            set_lane(pay, lane, 2 * kWinWords + 2 * q, (uint32_t)blockers);
            set_lane(pay, lane, 2 * kWinWords + 2 * q + 1, (uint32_t)(blockers >> 32));
        }
        if (lane < kRelWords) {
            if (wh.G == 1) reinterpret_cast<uint32_t*>(&sh.rel[j][0])[lane] = pay;
            else ll_store(buf + (int64_t)j * kRelWords + lane, pay, seq);
        }
    }
    if (wh.G == 1) return;
    constexpr int NE = (kCandWin * kRelWords + T + kCtrlThreads - 1) / (T + kCtrlThreads);
    uint64_t got[NE];
#pragma unroll
    for (int u = 0; u < NE; ++u) {
        const int e = tid + u * (T + kCtrlThreads);
        got[u] = e < total * kRelWords ? ll_load(buf + e) : 0;
    }
#pragma unroll
    for (int u = 0; u < NE; ++u) {
        const int e = tid + u * (T + kCtrlThreads);
        if (e < total * kRelWords) {
            uint32_t val[1];
            val[0] = (uint32_t)got[u];
            if ((uint32_t)(got[u] >> 32) != seq && !ll_wait<1>(buf + e, seq, val, a.wait_ticks)) sh.ctrl[2] = 1;
            reinterpret_cast<uint32_t*>(&sh.rel[e / kRelWords][0])[e % kRelWords] = val[0];
        }
    }
}

template <int T>
__device__ __forceinline__ void settle_relations(Shared<T>& sh, const Where& wh, const CloudState& st,
                                                 int total, int limit)
{
    total = uni(total);
    limit = uni(limit);
    // The lane number as a value the compiler knows nothing about: the LDS addresses below are then
    // formed here.  Formed once per kernel they stay alive through all of it, end up in scratch memory,
    // and every use in this function waits for a reload.
    int lane = wh.lane;
    asm volatile("" : "+v"(lane));
    const int nq = (total + 63) >> 6;              // uniform
    uint64_t blockers[kWinWords][kWinWords];
    uint64_t und[kWinWords], acc[kWinWords], rej[kWinWords];
#pragma unroll
    for (int q = 0; q < kWinWords; ++q) {
        const int c = lane + 64 * q;
        const bool has = c < total;
        und[q] = __builtin_amdgcn_ballot_w64(has);
        acc[q] = 0;
        rej[q] = 0;
#pragma unroll
        for (int w = 0; w < kWinWords; ++w) blockers[q][w] = has ? sh.rel[c][kWinWords + w] : 0;
    }
    for (int sweep = 0; sweep <= total; ++sweep) {  // ends much earlier: see above
        uint64_t left = 0;
#pragma unroll
        for (int q = 0; q < kWinWords; ++q) {
            if (q < nq && und[q] != 0) {
                uint64_t open = 0, hit = 0;
#pragma unroll
                for (int w = 0; w < kWinWords; ++w) {
                    open |= blockers[q][w] & ~rej[w];
                    hit |= blockers[q][w] & acc[w];
                }
                const bool mine = ((und[q] >> lane) & 1ull) != 0;
                const uint64_t na = __builtin_amdgcn_ballot_w64(mine && open == 0);
                const uint64_t nr = __builtin_amdgcn_ballot_w64(mine && hit != 0);
                acc[q] |= na;
                rej[q] |= nr;
                und[q] &= ~(na | nr);
                left |= und[q];
            }
        }
        if (left == 0) break;
    }
    int count = 0;
#pragma unroll
    for (int q = 0; q < kWinWords; ++q) count += __builtin_popcountll(acc[q]);
    const int nacc = count < limit ? count : limit;
#pragma unroll
    for (int q = 0; q < kWinWords; ++q) {
        const int c = lane + 64 * q;
        const bool mine = ((acc[q] >> lane) & 1ull) != 0;
        int place = 0;
#pragma unroll
        for (int w = 0; w < kWinWords; ++w)
            if (q < nq && w < nq) place += __builtin_popcountll((mine ? sh.rel[c][w] : 0ull) & acc[w]);
        const bool keep = mine && place < limit;
        if (keep) {
            stage_pick<T>(sh, st.i + place, sh.cand[c].idx, 0.0f);
            sh.place[c] = (uint16_t)place;
        }
        const uint64_t took = __builtin_amdgcn_ballot_w64(keep);
        if (lane == 0) sh.took[q] = took;
    }
    if (lane == 0) sh.ctrl[0] = nacc;
}

// The point waves' side: which candidates are near the wave's box (while the control wave settles
// the round), then -- after the barrier -- the fold of the accepted ones among them.
struct NearWords {
    uint64_t w[kWinWords];      // candidates to fold
    uint64_t b[kWinWords];      // of those, the ones whose ball reaches the wave's box (recording kernels)
};
template <int T, int P, bool BQ>
__device__ __forceinline__ NearWords near_candidates(const Points<P, BQ>& pt, const Shared<T>& sh,
                                                     const Where& wh, int total, float bq_r2)
{
    NearWords nw;
#pragma unroll
    for (int q = 0; q < kWinWords; ++q)
        nw.w[q] = near_mask<P, BQ>(pt, sh.cand + 64 * q, total - 64 * q, wh.lane, bq_r2, nw.b[q]);
    return nw;
}
template <int T, int P, bool BQ>
__device__ __forceinline__ void fold_accepted(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                              const SamplerArgs& a, const NearWords& nw, int base)
{
    RowWords<P, BQ> rw;
    rw.row = wh.rows;
    uint64_t m[kWinWords], mb[kWinWords];
    uint64_t left = 0;
#ifdef FASTPOINT_PHASE_CLOCKS
    long long fa_t = wall_clock64();
#define FOLD_MARK(k) do { if (wh.tid == 0) { const long long now__ = wall_clock64(); sh.scan_clk[k] += now__ - fa_t; fa_t = now__; } } while (0)
#else
#define FOLD_MARK(k) do { } while (0)
#endif
#pragma unroll
    for (int q = 0; q < kWinWords; ++q) {
        const uint64_t t = nw.w[q] & sh.took[q];
        mb[q] = BQ ? t & nw.b[q] : 0ull;
        m[q] = t & ~mb[q];
        left |= mb[q];
    }
    // the accepted candidates that need no radius test
#pragma unroll
    for (int q = 0; q < kWinWords; ++q) {
        while (m[q] != 0) {
            const Cand c = sh.cand[64 * q + first_lane(m[q])];
            m[q] &= m[q] - 1;
            fold<P, BQ, true, false>(pt, c.x, c.y, c.z, a, wh, 0, rw);
        }
    }
    FOLD_MARK(5);
    if constexpr (BQ) {
        // a recording wave takes the others up to 64 at a time: lane t of the row buffer holds the words
        // of the t-th of them and the place of that pick among the round's picks.  (Appending a pick's
        // words to the list one by one as they are formed saves the row buffer but costs more wherever
        // balls hold many blocks: measured.)
#pragma unroll 1
        while (left != 0) {
            rw.clear(wh);
            int s = 0;
            int my_place = 0;
            left = 0;
#pragma unroll
            for (int q = 0; q < kWinWords; ++q) {
                while (mb[q] != 0 && s < 64) {
                    const int cl = 64 * q + first_lane(mb[q]);
                    const Cand c = sh.cand[cl];
                    mb[q] &= mb[q] - 1;
                    if (wh.lane == s) my_place = (int)sh.place[cl];
                    fold<P, BQ>(pt, c.x, c.y, c.z, a, wh, s, rw);
                    ++s;
                }
                left |= mb[q];
            }
            FOLD_MARK(6);
            flush_rows<P, BQ>(rw, a, wh, pt, base, s, my_place);
            FOLD_MARK(7);
        }
    }
}

// Exact FPS for several picks at once.  The candidates are ALL points whose distance exceeds
// tau, so every other point is at most tau and can only decrease.  Repeatedly: the candidate with
// the largest up-to-date distance (lowest index among equals) is the true arg-max of Alg. 1
// as long as that distance exceeds tau; accepting it lowers the other candidates'
// distances exactly as the fold will.  Stops when no candidate exceeds tau any more.  Run by the
// control wave; picks are published one by one like those of the threshold phase.
// The candidates are in ascending index order, so the lowest lane among equal distances is the
// lowest index.  One step is a chain of dependent instructions of a single wave: its length in
// instructions is what a pick costs.
// One run of the chain: up to `limit` picks (CHECK) or as many as exceed tau (a candidate is
// accepted at most once, so that needs no count).  Returns the number accepted.
template <bool CHECK, bool PERM>
__device__ __forceinline__ int chain_loop(uint64_t* live, LiveCursor& cur, const Cand& me, uint32_t& cd,
                                          uint32_t tau_bits, int limit, uint32_t& dl)
{
    int nacc = 0;
    uint32_t dmax = wave_max_scalar(cd);
    while (dmax > tau_bits) {
        if (CHECK && nacc >= limit) break;
        const uint64_t eq = __builtin_amdgcn_ballot_w64(cd == dmax);
        int cl = first_lane(eq);
        if (PERM && __builtin_expect(__builtin_popcountll(eq) > 1, 0)) {
            // cell order: among equal distances the lowest index of the caller's cloud, not the lowest lane
            const uint32_t imin = wave_min_u32(cd == dmax ? me.idx : kNoIdx);
            cl = first_lane(__builtin_amdgcn_ballot_w64(cd == dmax && me.idx == imin));
        }
        const float ax = rdlane_f(me.x, cl), ay = rdlane_f(me.y, cl), az = rdlane_f(me.z, cl);
        cur.publish(live, (uint32_t)cl, dmax);
        dl = dmax;
        // lanes without a candidate hold 0 and stay there
        cd = min(cd, __float_as_uint(dist2(ax, ay, az, me.x, me.y, me.z)));
        nacc = uni(nacc + 1);
        dmax = wave_max_scalar(cd);
    }
    return nacc;
}

// The same run with two candidates per lane (lane l holds candidates l and 64 + l of the round's
// list, which is in ascending index order -- or, cell-ordered variant, in any order with ties
// settled by the points' own indices).  A step costs a third more instructions; a round takes
// twice the candidates, which halves the scans and their exchanges between workgroups.
template <bool CHECK, bool PERM>
__device__ __forceinline__ int chain_loop_wide(uint64_t* live, LiveCursor& cur, const Cand& me0, const Cand& me1,
                                               uint32_t& cd0, uint32_t& cd1, uint32_t tau_bits, int limit,
                                               uint32_t& dl)
{
    int nacc = 0;
    uint32_t dmax = wave_max_scalar(max(cd0, cd1));
    while (dmax > tau_bits) {
        if (CHECK && nacc >= limit) break;
        uint64_t e0 = __builtin_amdgcn_ballot_w64(cd0 == dmax);
        uint64_t e1 = __builtin_amdgcn_ballot_w64(cd1 == dmax);
        if (PERM && __builtin_expect(__builtin_popcountll(e0) + __builtin_popcountll(e1) > 1, 0)) {
            // cell order: among equal distances the lowest index of the caller's cloud
            const uint32_t i0 = cd0 == dmax ? me0.idx : kNoIdx;
            const uint32_t i1 = cd1 == dmax ? me1.idx : kNoIdx;
            const uint32_t imin = wave_min_u32(min(i0, i1));
            e0 = __builtin_amdgcn_ballot_w64(i0 == imin);
            e1 = __builtin_amdgcn_ballot_w64(i1 == imin);
        }
        float ax, ay, az;
        uint32_t slot;
        if (e0 != 0) {                                  // the lower half of the list comes first
            const int cl = first_lane(e0);
            ax = rdlane_f(me0.x, cl);
            ay = rdlane_f(me0.y, cl);
            az = rdlane_f(me0.z, cl);
            slot = (uint32_t)cl;
        } else {
            const int cl = first_lane(e1);
            ax = rdlane_f(me1.x, cl);
            ay = rdlane_f(me1.y, cl);
            az = rdlane_f(me1.z, cl);
            slot = 64u + (uint32_t)cl;
        }
        cur.publish(live, slot, dmax);
        dl = dmax;
        // lanes without a candidate hold 0 and stay there
        cd0 = min(cd0, __float_as_uint(dist2(ax, ay, az, me0.x, me0.y, me0.z)));
        cd1 = min(cd1, __float_as_uint(dist2(ax, ay, az, me1.x, me1.y, me1.z)));
        nacc = uni(nacc + 1);
        dmax = wave_max_scalar(max(cd0, cd1));
    }
    return nacc;
}

template <int T, bool PERM, int NQ>
__device__ __forceinline__ void resolve_chain(Shared<T>& sh, const Where& wh, const CloudState& st,
                                              int total, int limit, float tau, bool capture, int nseg,
                                              uint32_t tag)
{
    total = uni(total);
    limit = uni(limit);
    Cand me[NQ];
    uint32_t cd[NQ];                                   // bit patterns; distances are >= +0
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const bool has = wh.lane + 64 * q < total;
        me[q] = sh.cand[has ? wh.lane + 64 * q : 0];
        cd[q] = has ? me[q].d : 0u;
    }
    const uint32_t tau_bits = uni(__float_as_uint(tau));    // tau >= 0
    uint32_t dl = __float_as_uint(st.dlast);
    LiveCursor cur(tag);
    __builtin_amdgcn_s_setprio(3);
#ifdef FASTPOINT_PHASE_CLOCKS
    const long long chain_t0 = clock64();
#endif
    // the candidates have arrived from LDS before the loop starts, not inside it
#pragma unroll
    for (int q = 0; q < NQ; ++q) asm volatile("" ::"v"(me[q].x), "v"(me[q].y), "v"(me[q].z), "v"(cd[q]));
    int nacc;
    static_assert(NQ <= 2, "the chain is written for one or two candidates per lane");
    if constexpr (NQ > 1) {
        nacc = limit >= total
                   ? chain_loop_wide<false, PERM>(sh.live, cur, me[0], me[1], cd[0], cd[1], tau_bits, limit, dl)
                   : chain_loop_wide<true, PERM>(sh.live, cur, me[0], me[1], cd[0], cd[1], tau_bits, limit, dl);
    } else {
        nacc = limit >= total ? chain_loop<false, PERM>(sh.live, cur, me[0], cd[0], tau_bits, limit, dl)
                              : chain_loop<true, PERM>(sh.live, cur, me[0], cd[0], tau_bits, limit, dl);
    }
    cur.publish(sh.live, kLiveEnd, 0u);
    __builtin_amdgcn_s_setprio(0);
#ifdef FASTPOINT_PHASE_CLOCKS
    if (wh.lane == 0) {
        sh.chain_cycles += clock64() - chain_t0;
        sh.chain_picks += nacc;
    }
#endif
    for (int t = wh.lane; t < nacc; t += 64) {             // a second turn only after a wide round
        const int pos = st.i + t;
        const uint64_t word = sh.live[t];
        const float d = __uint_as_float((uint32_t)(word >> 32));
        stage_pick<T>(sh, pos, sh.cand[(uint32_t)word & kLiveMask].idx, d);
        if (capture) {                  // prefix loop of Alg. 2: keep the curve
            sh.ring[pos & 63] = d;
            for (int l = 0; l < nseg; ++l)
                if (sh.bl[l] == pos) sh.thr_meas[l] = d;
            if (sh.mlp_pos[0] >= 0)
                for (int k = 0; k < 32; ++k)
                    if (sh.mlp_pos[k] == pos) sh.mlp_val[k] = d;
        }
    }
    if (wh.lane == 0) {
        sh.ctrl[0] = nacc;
        sh.ctrl[3] = (int)dl;
    }
}

// ---- exact FPS for sample positions [st.i, upto) (the loop of Alg. 1), in batched rounds with
// plain iterations as the fallback.  Returns false if a wait between workgroups expired.
template <int T, int P, bool BQ, bool PERM, int kFpsQ>
__device__ __forceinline__ bool fps_rounds_of(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                              const SamplerArgs& a, uint32_t& it, uint32_t& seq,
                                              CloudState& st, int upto, bool capture)
{
    constexpr int kCandFps = 64 * kFpsQ;            // candidates of a round: one, two or four per lane of the control wave
    while (st.i < upto) {
        flush_picks<T, BQ>(a, sh, wh, st.flushed, st.i, false);
        {
            PHASE_BEGIN();
            fold_pending<T, P, BQ, PERM>(pt, sh, wh, a, st.npend, st.i - st.npend);
            PHASE_END(st, 0);
        }
        st.npend = 0;
        if constexpr (PERM) refresh_bound<P, BQ>(pt);
        bool good = false;
        int total = 0, alltot = 0;
        float tau = 0.0f;
        if (st.dlast > 0.0f && st.dlast < __builtin_inff()) {
            for (int tries = 0; tries < 4 && !good; ++tries) {
                tau = st.dlast - st.om * st.dlast;
                PHASE_BEGIN();
                total = scan_candidates<T, P, BQ, PERM, true, kCandFps, false, false,
                                        (kCandFps < kCandMax ? kCandFps : kCandMax)>(pt, sh, wh, a, seq, tau, alltot);
                PHASE_END(st, 1);
                if (total < 0) return false;
                ++st.rounds;
                if (alltot > 0 && alltot == total) good = true;      // all of them are in the list
                else if (alltot == 0) st.om = st.om * 2.0f < 0.99f ? st.om * 2.0f : 0.99f;
                else st.om = st.om * 0.5f;
            }
        }
        if (!good) {
            PHASE_BEGIN();
            const bool picked = plain_pick<T, P, BQ, PERM>(pt, sh, wh, a, it, seq, st, capture);
            PHASE_END(st, 3);
            if (!picked) return false;
            continue;
        }
        {
            PHASE_BEGIN();
            const uint32_t tag = (uint32_t)(st.resolved + 1) << kLiveShift;
            if (wh.ctrl) resolve_chain<T, PERM, kFpsQ>(sh, wh, st, total, upto - st.i, tau, capture, a.nseg, tag);
            else follow_picks<T, P, BQ, PERM, kFpsQ>(pt, sh, wh, a, st.i, tag, total);
            __syncthreads();
            PHASE_END(st, 2);
        }
        ++st.resolved;
        st.npend = 0;                               // folded while they were resolved
        st.dlast = __uint_as_float(uni((uint32_t)sh.ctrl[3]));
        st.i += uni(sh.ctrl[0]);
        if (alltot < 40 * (kCandFps / kCand)) st.om = st.om * 1.15f < 0.99f ? st.om * 1.15f : 0.99f;
        else if (alltot > 58 * (kCandFps / kCand)) st.om = st.om * 0.87f;
    }
    return true;
}

// Rounds of 64, 128 or 256 candidates.  With four or more points per thread folding a pick takes the
// point waves longer than finding it takes the control wave, so the longer chain step of a round
// with two candidates per lane is hidden and the halved number of scans is a gain.  With two
// points per thread the chain is what a pick costs, and the wide round pays only where a scan is
// expensive: when the cloud is spread over many workgroups (measured: 24 yes, 4 and 1 no).
// ONE_WG: the kernel is only ever launched with one workgroup per cloud.
template <int T, int P, bool BQ, bool PERM, bool ONE_WG>
__device__ __forceinline__ bool fps_rounds(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                           const SamplerArgs& a, uint32_t& it, uint32_t& seq,
                                           CloudState& st, int upto, bool capture)
{
    // (Four candidates per lane, rounds of 256, were measured with eight points per thread, where a
    // fold takes 260 ns: the million-point cloud then needs 436 scans instead of 814, but a chain step
    // grows to 355 ns and becomes what a pick costs -- 23.2 ms either way; and a chain loop written
    // for any number of candidates per lane was a tenth slower with two than the one written for two.)
    if constexpr (P >= 4) {
        return fps_rounds_of<T, P, BQ, PERM, 2>(pt, sh, wh, a, it, seq, st, upto, capture);
    } else {
        if constexpr (!PERM && !ONE_WG) // (the cell-ordered variant gained nothing there and pays for the code)
            if (wh.G >= 8) return fps_rounds_of<T, P, BQ, PERM, 2>(pt, sh, wh, a, it, seq, st, upto, capture);
        return fps_rounds_of<T, P, BQ, PERM, 1>(pt, sh, wh, a, it, seq, st, upto, capture);
    }
}

// ------------------------------------------------------------------ one cloud
// MODE 0: exact FPS only (the code of Alg. 2 is left out of the kernel); 1: MDPS with threshold rounds
// of kCand candidates; 2: MDPS with threshold rounds of kCandMax candidates; 3: MDPS with the
// scattered scan order -- the records of a.sorted are in the order of the walk, so the first
// kCandMax available positions are the candidates, already in the order the rule takes them; 4: the
// same sampling rule on records in cell order (pruned distance updates): every point knows its
// place t in the walk, and the windows of the cell-ordered variant run over t instead of the index.
template <int T, int P, bool BQ, bool PERM, int MODE>
__device__ __forceinline__ void run_cloud(const SamplerArgs& a, Shared<T>& sh, const Where& wh,
                                          uint32_t& it, uint32_t& seq)
{
    constexpr bool WIDE = MODE >= 2;
    constexpr bool WALK = MODE == 3;                // positions are the scan order itself
    constexpr bool RANKED = MODE == 4;              // cell order, threshold phase by place in the walk
    constexpr bool WINDOWS = PERM && !WALK;         // cell order: the lowest indices (places) through a window
    static_assert(MODE < 3 || PERM, "the scattered scan order works on reordered records");
    static_assert(MODE != 3 || !BQ, "records in walk order are not recorded");
    const int n = a.n, N = a.N;
    const bool writer = (wh.g == 0 && wh.tid == 0);
    const float* cloud = a.xyz + (int64_t)wh.c * N * 3;

    const int start = uni(a.start_idx ? a.start_idx[wh.c] : 0);
    if (start < 0 || start >= N) {          // uniform over the group
        if (wh.g == 0) {
            for (int k = wh.tid; k < n; k += T + kCtrlThreads) {
                a.out_idx[(int64_t)wh.c * n + k] = -1;
                if (BQ) a.bq_idx[(int64_t)wh.c * n + k] = -1;      // no centre matches this cloud's record
            }
            if (wh.tid == 0 && a.info) {
                fp_mdps_info inf = {};
                inf.status = 1;
                a.info[wh.c] = inf;
            }
        }
        return;
    }

    Points<P, BQ> pt;
    if constexpr (PERM) {
        // positions follow the cell order of a.sorted; a record carries the point's own index
        const float4* __restrict__ rec = a.sorted + (int64_t)wh.c * N;
        float lo[3] = {__builtin_inff(), __builtin_inff(), __builtin_inff()};
        float hi[3] = {-__builtin_inff(), -__builtin_inff(), -__builtin_inff()};
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int j = ((wh.gw * P + p) << 6) | wh.lane;
            if (j < N) {
                const float4 r = rec[j];
                pt.x[p] = r.x;
                pt.y[p] = r.y;
                pt.z[p] = r.z;
                pt.oi[p] = __float_as_uint(r.w);
                if constexpr (BQ) a.bq_map[(int64_t)wh.c * N + j] = (int32_t)pt.oi[p];
                if constexpr (RANKED) wh.rk[p * kRkStride] = (uint32_t)(((uint64_t)pt.oi[p] * a.walk_inv) % (uint64_t)N);
                pt.d[p] = __builtin_inff();
                lo[0] = fminf(lo[0], r.x);
                lo[1] = fminf(lo[1], r.y);
                lo[2] = fminf(lo[2], r.z);
                hi[0] = fmaxf(hi[0], r.x);
                hi[1] = fmaxf(hi[1], r.y);
                hi[2] = fmaxf(hi[2], r.z);
            } else {
                pt.x[p] = kPadCoord;
                pt.y[p] = kPadCoord;
                pt.z[p] = kPadCoord;
                pt.oi[p] = kNoIdx;
                if constexpr (RANKED) wh.rk[p * kRkStride] = kNoIdx;
                pt.d[p] = 0.0f;
            }
        }
#pragma unroll
        for (int k = 0; k < 3; ++k)
            for (int sft = 32; sft > 0; sft >>= 1) {
                lo[k] = fminf(lo[k], __shfl_xor(lo[k], sft, 64));
                hi[k] = fmaxf(hi[k], __shfl_xor(hi[k], sft, 64));
            }
        pt.lox = unif(lo[0]);
        pt.loy = unif(lo[1]);
        pt.loz = unif(lo[2]);
        pt.hix = unif(hi[0]);
        pt.hiy = unif(hi[1]);
        pt.hiz = unif(hi[2]);
        pt.ub = 0x7F800000u;
    } else {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int j = ((wh.gw * P + p) << 6) | wh.lane;
            if (j < N) {
                pt.x[p] = cloud[(int64_t)j * 3 + 0];
                pt.y[p] = cloud[(int64_t)j * 3 + 1];
                pt.z[p] = cloud[(int64_t)j * 3 + 2];
                pt.d[p] = __builtin_inff();
            } else {
                pt.x[p] = kPadCoord;
                pt.y[p] = kPadCoord;
                pt.z[p] = kPadCoord;
                pt.d[p] = 0.0f;
            }
        }
    }
    pt.bq_cur = pt.bq_lim = 0;
    pt.bq_nxt = kBqNoChunk;
    pt.bq_dead = false;
    if constexpr (BQ) {
        // a cloud held by one workgroup: its counters in the cache are zeroed here (the barrier below
        // comes before the first entry); with several workgroups a launch in front has done it
        if (wh.G == 1) {
            const int nchunks = (int)(a.bq_cap / kBqChunk);
            for (int t = wh.tid; t < nchunks; t += T + kCtrlThreads) a.bq_fill[(int64_t)wh.c * nchunks + t] = 0u;
            if (wh.tid == 0) {
                a.bq_cursor[wh.c] = 0u;
                a.bq_ovf[wh.c] = 0u;
            }
        }
    }
    if (wh.tid < kCandWin + 2) sh.live[wh.tid] = 0;    // round tags start at 1 in every cloud
    if (wh.tid == 0) sh.progress = 0;
    if (wh.tid < 32) {
        int64_t ik = ((int64_t)a.m * (wh.tid + 1)) / 32;
        sh.mlp_pos[wh.tid] = a.mlp ? (int)(ik < 1 ? 1 : ik) : -1;
        sh.mlp_val[wh.tid] = 0.0f;
    }
    if (wh.tid < FP_MAX_SEG) {
        sh.level_start[wh.tid] = -1;
        sh.level_exhausted[wh.tid] = 0;
        sh.thr[wh.tid] = 0.0f;
        sh.thr_meas[wh.tid] = 0.0f;
        sh.bl[wh.tid] = wh.tid < a.nseg ? boundary_index(n, a.nseg, wh.tid + 1) : -1;
    }
    CloudState st;
    st.i = 1;
    st.npend = 1;
    st.flushed = 0;
    st.rounds = 0;
    st.resolved = 0;
    st.dlast = -1.0f;
    st.om = 0.25f;
    st.my_bl = wh.tid < a.nseg ? boundary_index(n, a.nseg, wh.tid + 1) : -1;
#ifdef FASTPOINT_PHASE_CLOCKS
    for (int k = 0; k < 12; ++k) st.clk[k] = 0;
    const long long cloud_t0__ = wall_clock64();
#endif
    if (wh.tid == 0) {
        sh.ctrl[2] = 0;
#ifdef FASTPOINT_PHASE_CLOCKS
        sh.chain_cycles = 0;
        sh.chain_picks = 0;
        for (int k = 0; k < 8; ++k) sh.scan_clk[k] = 0;
#endif
        Cand c0;                       // first step of Alg. 1: the seed is sample 0, not folded yet
        c0.idx = (uint32_t)start;
        c0.x = cloud[(int64_t)start * 3 + 0];
        c0.y = cloud[(int64_t)start * 3 + 1];
        c0.z = cloud[(int64_t)start * 3 + 2];
        c0.d = 0;
        sh.pend[0] = c0;
        stage_pick<T>(sh, 0, (uint32_t)start, __builtin_inff());
    }
    __syncthreads();

    const int m = a.m;                 // exact FPS picks before the threshold phase
    const bool pure_fps = MODE == 0 || (m >= n - 1);
    int et_index = n;
    if (wh.tid == 0) {
        const long long t = wall_clock64();
        for (int k = 0; k < 5; ++k) sh.phase_t[k] = t;
    }

    bool ok = fps_rounds<T, P, BQ, PERM, MODE == 1>(pt, sh, wh, a, it, seq, st, pure_fps ? n : m + 1, !pure_fps);

    if (wh.tid == 0) {
        const long long t = wall_clock64();
        for (int k = 1; k < 5; ++k) sh.phase_t[k] = t;
    }
    if constexpr (MODE != 0) if (ok && !pure_fps) {
        // ---- thresholds from the estimated curve (Eq. 1 with a/x^e; estimator call and list radii of Alg. 2)
        __syncthreads();
        if (a.use_override) {
            if (wh.tid < a.nseg) sh.thr[wh.tid] = a.thr_override[wh.tid];
        } else if (a.mlp) {
            // ---- MLP estimator (Appendix A.3): 32 log-ratios of the prefix curve in, 64 log-ratios
            //      of the rest of the curve out; every workgroup of the cloud computes the same
            const float* __restrict__ W1 = a.mlp;
            const float* __restrict__ b1 = W1 + 32 * 128;
            const float* __restrict__ W2 = b1 + 128;
            const float* __restrict__ b2 = W2 + 128 * 128;
            const float* __restrict__ W3 = b2 + 128;
            const float* __restrict__ b3 = W3 + 128 * 64;
            const double last = (double)sh.ring[m & 63];
            if (wh.tid < 32) {
                const double ratio = (double)sh.mlp_val[wh.tid] / last;
                sh.mlp_a[wh.tid] = (ratio >= 1.0 && ratio <= 1e300) ? ln_fixed(ratio) : 0.0;
            }
            __syncthreads();
            mlp_layer<32, 128, true>(W1, b1, sh.mlp_a, sh.mlp_b, wh.tid);
            __syncthreads();
            mlp_layer<128, 128, true>(W2, b2, sh.mlp_b, sh.mlp_a, wh.tid);
            __syncthreads();
            mlp_layer<128, 64, false>(W3, b3, sh.mlp_a, sh.mlp_b, wh.tid);
            __syncthreads();
            if (wh.tid < a.nseg) {
                // the estimated curve at this level's boundary: the outputs interpolated linearly
                const int l = wh.tid;
                const int64_t b = boundary_index(n, a.nseg, l + 1);
                float r;
                if (b <= m) {
                    r = sh.thr_meas[l];
                } else {
                    const double u = ((double)(b - m) * 64.0) / (double)(n - 1 - m);
                    int j0 = (int)floor(u);
                    if (j0 > 64) j0 = 64;
                    const double frac = u - (double)j0;
                    const double v0 = j0 == 0 ? 0.0 : sh.mlp_b[j0 - 1];
                    const double v1 = j0 >= 64 ? sh.mlp_b[63] : sh.mlp_b[j0];
                    const double y = v0 + frac * (v1 - v0);
                    r = (float)((a.bias2 * (double)a.level_scale[l]) * (last * exp_fixed(y)));
                }
                if (!(r >= 1.17549435e-38f)) r = 1.17549435e-38f;
                sh.thr[l] = r;
            }
            __syncthreads();
            if (wh.tid == 0)
                for (int l = 1; l < a.nseg; ++l)
                    if (sh.thr[l] > sh.thr[l - 1]) sh.thr[l] = sh.thr[l - 1];
        } else {
            const int W = a.fit_window < m ? a.fit_window : m;
            if (wh.tid < W) {
                const int ii = m - W + 1 + wh.tid;
                sh.terms[wh.tid] = (double)sh.ring[ii & 63] * pow_int_base(ii, a.exponent);
            } else if (wh.tid >= 64 && wh.tid < 64 + a.nseg) {
                const int l = wh.tid - 64;
                sh.powb[l] = pow_int_base(boundary_index(n, a.nseg, l + 1), a.exponent);
            }
            __syncthreads();
            if (wh.tid == 0) {
                double acc = 0.0;
                for (int t = 0; t < W; ++t) acc += sh.terms[t];
                acc = acc / (double)W;
                float prev = 0.0f;
                for (int l = 0; l < a.nseg; ++l) {
                    float r;
                    if (boundary_index(n, a.nseg, l + 1) <= m) r = sh.thr_meas[l];
                    else r = (float)(((a.bias2 * (double)a.level_scale[l]) * acc) / sh.powb[l]);
                    if (!(r >= 1.17549435e-38f)) r = 1.17549435e-38f;
                    if (l >= 1 && r > prev) r = prev;
                    sh.thr[l] = r;
                    prev = r;
                }
            }
        }
        __syncthreads();
        int seg = 0;
        if (wh.tid == 0) {
            const long long t = wall_clock64();
            for (int k = 2; k < 5; ++k) sh.phase_t[k] = t;
        }
#ifdef FASTPOINT_PHASE_CLOCKS
        const long long thrphase_t0 = wall_clock64();
#endif

        // ---- threshold sampling (main loop of Alg. 2), running-distance form
        // candidates per round: one or (WIDE) two per lane of the control wave
        constexpr int kCandThr = WINDOWS ? kCandWin : (WIDE ? kCandMax : kCand);
        [[maybe_unused]] constexpr int kWinAim = kCandWin * 3 / 4;      // candidates a window is sized for (7/8: more repeated scans on the LiDAR clouds than rounds saved)
        // The quota rule (the level floor of Alg. 2) puts sample position i on level 1 + floor(i nseg / n), i.e. on a
        // level above l as soon as i >= ceil(n l / nseg): the positions are tabulated once, a round
        // then compares with the one that ends its level.
        if (wh.tid <= a.nseg) sh.qend[wh.tid] = (int32_t)(((int64_t)n * wh.tid + a.nseg - 1) / a.nseg);
        __syncthreads();
        int level_end = 0;                 // qend[seg]: first position the quota rule puts above level seg
        // Cell-ordered variant: the points are not held in index order, so "the first available
        // points by index" are found through a window of indices [win_lo, win_lo + win_len): within
        // a level the picks have ascending indices and a point once unavailable stays so, hence
        // every index below win_lo is settled; a round takes ALL available points of the window
        // (the window is shortened and the scan repeated if they are more than a round holds) and
        // puts them in index order -- the same candidates, in the same order, as the scan in index
        // order would give, up to where the window ends.
        uint32_t win_lo = 0, win_len = (uint32_t)N;
        while (st.i < n) {
            flush_picks<T, BQ>(a, sh, wh, st.flushed, st.i, false);
            if (st.i >= level_end) {
                while (st.i >= level_end) {
                    ++seg;
                    level_end = uni(sh.qend[seg]);
                }
                if (wh.tid == 0 && sh.level_start[seg - 1] < 0) sh.level_start[seg - 1] = st.i;
                win_lo = 0;                // a smaller radius: points settled so far may be available again
            }
            fold_pending<T, P, BQ, PERM>(pt, sh, wh, a, st.npend, st.i - st.npend);   // picks since the last sweep
            st.npend = 0;
            if constexpr (WINDOWS) refresh_bound<P, BQ>(pt);      // (else the last bound stays: never too low)
            const float r2 = unif(sh.thr[seg - 1]);
            // samples of this level end where the quota rule would raise the level
            const int limit = (level_end < n ? level_end : n) - st.i;
            ++st.rounds;
            int alltot = 0;
#ifdef FASTPOINT_PHASE_CLOCKS
            const long long thr_t0 = wall_clock64();
#endif
            int total = scan_candidates<T, P, BQ, PERM, false, kCandThr, WINDOWS, RANKED,
                                        (kCandThr < kCandMax ? kCandThr : kCandMax)>(pt, sh, wh, a, seq, r2, alltot,
                                                                                     win_lo, win_len);
#ifdef FASTPOINT_PHASE_CLOCKS
            const long long thr_t1 = wall_clock64();
            st.clk[4] += thr_t1 - thr_t0;
#endif
            if (total < 0) {
                ok = false;
                break;
            }
            [[maybe_unused]] bool window_is_last = false;
            if constexpr (WINDOWS) {
                window_is_last = (uint64_t)win_lo + win_len >= (uint64_t)N;
                if (alltot > total) {       // more than a round (or a workgroup's list) holds: a shorter window
                    uint64_t len = (uint64_t)win_len * (uint64_t)kWinAim / (uint64_t)alltot;
                    if (len > win_len / 2) len = win_len / 2;
                    win_len = len < 1 ? 1u : (uint32_t)len;
                    continue;
                }
                if (total == 0 && !window_is_last) {        // nothing available in the window: so little is left
                    win_lo += win_len;                       // that all the indices beyond it come next
                    win_len = (uint32_t)N;
                    continue;
                }
            }
            if (total == 0) {              // level exhausted: Alg. 2 moves to the next level
                if (wh.tid == 0) sh.level_exhausted[seg - 1] = 1;
                ++seg;
                if (seg > a.nseg) break;   // early termination
                level_end = uni(sh.qend[seg]);
                if (wh.tid == 0 && sh.level_start[seg - 1] < 0) sh.level_start[seg - 1] = st.i;
                win_lo = 0;
                continue;
            }
#ifdef FASTPOINT_PHASE_CLOCKS
            const long long thr_t2 = wall_clock64();
#endif
            if constexpr (WINDOWS) {
                build_relations<T, RANKED>(sh, wh, a, seq, total, r2);
                __syncthreads();
                if (uni(sh.ctrl[2]) != 0) {     // a wait between workgroups expired
                    ok = false;
                    break;
                }
#ifdef FASTPOINT_PHASE_CLOCKS
                const long long thr_t3 = wall_clock64();
                st.clk[9] += thr_t3 - thr_t2;
#endif
                NearWords nw = {};
                if (wh.ctrl) settle_relations<T>(sh, wh, st, total, limit);
                else nw = near_candidates<T, P, BQ>(pt, sh, wh, total, a.bq_r2);
                __syncthreads();
#ifdef FASTPOINT_PHASE_CLOCKS
                const long long thr_t4 = wall_clock64();
                st.clk[10] += thr_t4 - thr_t3;
#endif
                if (!wh.ctrl) fold_accepted<T, P, BQ>(pt, sh, wh, a, nw, st.i);
#ifdef FASTPOINT_PHASE_CLOCKS
                st.clk[11] += wall_clock64() - thr_t4;
#endif
            } else if constexpr (WALK) {
                const uint32_t round_no = ((uint32_t)(st.resolved + 1) & 0x7FFFu) + 1u;   // never 0
                build_conflicts<T>(sh, wh, total, r2);
                __syncthreads();
                if (wh.ctrl) resolve_conflicts<T>(sh, wh, st, total, limit, round_no);
                else follow_stream<T, P, BQ>(pt, sh, wh, a, round_no);
            } else {
                const uint32_t tag = (uint32_t)(st.resolved + 1) << kLiveShift;
                if (wh.ctrl) resolve_threshold<T, WIDE>(sh, wh, st, total, limit, r2, tag);
                else follow_picks<T, P, BQ, PERM, (WIDE ? 2 : 1)>(pt, sh, wh, a, st.i, tag, total);
            }
            __syncthreads();
            ++st.resolved;
            st.npend = 0;                           // folded while they were resolved
            st.i += uni(sh.ctrl[0]);
#ifdef FASTPOINT_PHASE_CLOCKS
            st.clk[5] += wall_clock64() - thr_t1;
#endif
            bool exhausted = alltot < kCandThr;
            if constexpr (WINDOWS) {
                // the quota did not cut the round short (checked below): the window is worked off;
                // the next one is as long as should hold three quarters of a round's candidates
                exhausted = window_is_last;
                win_lo = window_is_last ? 0u : win_lo + win_len;
                uint64_t len = (uint64_t)win_len * (uint64_t)kWinAim / (uint64_t)(alltot > 0 ? alltot : 1);
                if (len > (uint64_t)win_len * 2) len = (uint64_t)win_len * 2;     // availability is uneven along the indices
                win_len = len < 1 ? 1u : (len > (uint64_t)N ? (uint32_t)N : (uint32_t)len);
            }
            if (exhausted && st.i < level_end && st.i < n) {
                // Every available point of the cloud was a candidate and the quota did not cut the
                // round short: each one has been accepted or lies within R_l of an accepted one, so
                // the level is exhausted (Alg. 2 moves to the next one) -- no scan is needed to find that out.
                if (wh.tid == 0) sh.level_exhausted[seg - 1] = 1;
                ++seg;
                if (seg > a.nseg) break;   // early termination
                level_end = uni(sh.qend[seg]);
                if (wh.tid == 0 && sh.level_start[seg - 1] < 0) sh.level_start[seg - 1] = st.i;
            }
        }

#ifdef FASTPOINT_PHASE_CLOCKS
        st.clk[6] = wall_clock64() - thrphase_t0;
#endif
        if (wh.tid == 0) {
            const long long t = wall_clock64();
            sh.phase_t[3] = t;
            sh.phase_t[4] = t;
        }
        if (ok && st.i < n) {
            // ---- early termination (closing part of Alg. 2): dists is already the true running
            //      minimum, so the remainder is exact FPS on the same registers
            et_index = st.i;
            st.dlast = -1.0f;
            ok = fps_rounds<T, P, BQ, PERM, MODE == 1>(pt, sh, wh, a, it, seq, st, n, false);
        }
    }
    // the rows of the picks that were never folded (at least the last sample) are still missing
    if (ok && BQ) fold_pending<T, P, BQ, PERM>(pt, sh, wh, a, st.npend, st.i - st.npend);

    if (ok) flush_picks<T, BQ>(a, sh, wh, st.flushed, n, true);
    __syncthreads();
    if (writer && a.info) {
        fp_mdps_info inf = {};
        inf.m = pure_fps ? n - 1 : m;
        inf.et_index = et_index;
        for (int l = 0; l < FP_MAX_SEG; ++l) {
            inf.level_start[l] = sh.level_start[l];
            inf.level_exhausted[l] = sh.level_exhausted[l];
            inf.thr2[l] = sh.thr[l];
        }
        inf.rounds = st.rounds;
        if constexpr (MODE != 0) {
            if (!pure_fps) sh.phase_t[4] = wall_clock64();          // end of the remainder FPS
        }
        for (int k = 0; k < 4; ++k) inf.phase_ticks[k] = (int32_t)(sh.phase_t[k + 1] - sh.phase_t[k]);
#ifdef FASTPOINT_PHASE_CLOCKS
        if (a.nseg <= 8)
        {
            for (int k = 0; k < 4; ++k) inf.thr2[8 + k] = (float)st.clk[k] * 0.01f;   // 100 MHz ticks
            st.clk[7] = wall_clock64() - cloud_t0__;
            for (int k = 4; k < 8; ++k) inf.level_start[4 + k] = (int)st.clk[k];      // 10 ns ticks
            for (int k = 8; k < 12; ++k) inf.level_exhausted[k] = (int)st.clk[k];
            for (int k = 0; k < 4; ++k) inf.level_exhausted[12 + k] = (int)sh.scan_clk[k];
            inf.thr2[14] = (float)sh.scan_clk[4];
            inf.thr2[12] = (float)sh.chain_cycles;
            inf.thr2[13] = (float)sh.chain_picks;
        }
#endif
        inf.status = ok ? 0 : 2;
        a.info[wh.c] = inf;
    }
#ifdef FASTPOINT_PHASE_CLOCKS
    if (a.dbg && wh.tid == 0) {
        for (int k = 0; k < 8; ++k) a.dbg[wh.g * 16 + k] = sh.scan_clk[k];
        for (int k = 8; k < 12; ++k) a.dbg[wh.g * 16 + k] = st.clk[k];
        a.dbg[wh.g * 16 + 12] = st.clk[4];
        a.dbg[wh.g * 16 + 13] = st.clk[5];
    }
#endif
    if (!ok && wh.g == 0)
        for (int k = wh.tid; k < n; k += T + kCtrlThreads) {
            a.out_idx[(int64_t)wh.c * n + k] = -1;
            if (BQ) a.bq_idx[(int64_t)wh.c * n + k] = -1;          // no centre matches this cloud's record
        }
    __syncthreads();
}

template <int T, int P, bool BQ, bool PERM, int MODE>
__global__ __launch_bounds__(T + kCtrlThreads) void sampler_kernel(SamplerArgs a)
{
    __shared__ Shared<T> sh;
    __shared__ uint64_t bq_rows[BQ ? (T / 64) * P * 64 : 1];     // radius-test words not written out yet
    Where wh;
    wh.tid = (int)threadIdx.x;
    wh.lane = wh.tid & 63;
    wh.w = uni(wh.tid >> 6);
    wh.ctrl = wh.w == T / 64;
    wh.rows = bq_rows + (BQ && !wh.ctrl ? wh.w * P * 64 : 0);    // the control wave folds nothing
    static_assert(T + kCtrlThreads == kRkStride, "stride of the places in the walk");
    __shared__ uint32_t rk_words[MODE == 4 ? kRkStride * P : 1];
    wh.rk = rk_words + (MODE == 4 ? wh.tid : 0);
    wh.G = a.G;
    wh.grp = (int)blockIdx.x / a.G;
    wh.g = (int)blockIdx.x % a.G;
    // the control wave's slots lie beyond every point of the cloud: they are padding
    wh.gw = wh.ctrl ? a.G * (T / 64) : wh.g * (T / 64) + wh.w;
    const int ngroups = (int)gridDim.x / a.G;
    if constexpr (BQ) {
        // the header of the ball-query cache (256 bytes in front of the copy of the sample indices):
        // written here rather than by a launch of its own, which would lie in front of every
        // recording sampler on the stream
        if (blockIdx.x == 0 && threadIdx.x == 0)
            *reinterpret_cast<BqHeader*>(a.bq_base) = bq_layout(a.B, a.N, a.n, a.bq_r2, a.bq_cap, PERM ? 1 : 0);
    }
    uint32_t it = 0, seq = 0;
    for (int c = wh.grp; c < a.B; c += ngroups) {
        wh.c = c;
        run_cloud<T, P, BQ, PERM, MODE>(a, sh, wh, it, seq);
    }
}

// zeroes up to three ranges of words before a launch: the exchange words (stamps start at 1 in
// every launch), the counters of a ball-query cache, the relation words of the cell-ordered sampler
__global__ void zero_words_kernel(uint64_t* p, int64_t nwords, uint64_t* p2, int64_t nwords2, uint64_t* p3,
                                  int64_t nwords3)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = i; t < nwords; t += stride) p[t] = 0;
    for (int64_t t = i; t < nwords2; t += stride) p2[t] = 0;
    for (int64_t t = i; t < nwords3; t += stride) p3[t] = 0;
}

template <int T, int P, bool BQ, bool PERM>
const void* pick_mode(int mode)
{
    switch (mode) {
        case 0: return reinterpret_cast<const void*>(&sampler_kernel<T, P, BQ, PERM, 0>);
        case 1: return reinterpret_cast<const void*>(&sampler_kernel<T, P, BQ, PERM, 1>);
        case 2: return reinterpret_cast<const void*>(&sampler_kernel<T, P, BQ, PERM, 2>);
        default: return nullptr;
    }
}

template <int T, int P>
const void* pick_bq(bool bq, bool perm, int mode)
{
    if (perm) {                     // reordered records: threshold rounds always wide; MDPS in cell order records
        if (mode == 1) return nullptr;
        if (bq) {
            if (mode == 2) return reinterpret_cast<const void*>(&sampler_kernel<T, P, true, true, 2>);
            if (mode == 4) return reinterpret_cast<const void*>(&sampler_kernel<T, P, true, true, 4>);
            return nullptr;
        }
        if (mode == 3) return reinterpret_cast<const void*>(&sampler_kernel<T, P, false, true, 3>);
        if (mode == 4) return reinterpret_cast<const void*>(&sampler_kernel<T, P, false, true, 4>);
        return mode == 0 ? reinterpret_cast<const void*>(&sampler_kernel<T, P, false, true, 0>)
                         : reinterpret_cast<const void*>(&sampler_kernel<T, P, false, true, 2>);
    }
    if (mode >= 3) return nullptr;
    if (bq) return pick_mode<T, P, true, false>(mode);
    // without recording the wide rounds were faster on every shape
    return mode == 1 ? nullptr : pick_mode<T, P, false, false>(mode);
}

}  // namespace

const void* sampler_kernel_for(int threads, int points_per_thread, bool bq, bool perm, int mode)
{
    if (threads == 512) {
        switch (points_per_thread) {
            case 2: return pick_bq<512, 2>(bq, perm, mode);
            case 4: return pick_bq<512, 4>(bq, perm, mode);
            case 8: return pick_bq<512, 8>(bq, perm, mode);
            case 16: return pick_bq<512, 16>(bq, perm, mode);
            default: return nullptr;
        }
    }
    return nullptr;
}

// Records (x, y, z, index bits) of every cloud in the order of the walk j_t = (t A) mod N.
__global__ void scan_walk_kernel(const float* __restrict__ xyz, int64_t total, int N, uint64_t stride,
                                 float4* __restrict__ out)
{
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += step) {
        const int64_t b = e / N;
        const uint64_t t = (uint64_t)(e - b * N);
        const uint32_t j = (uint32_t)((t * stride) % (uint64_t)N);         // t, A < 2^31: no overflow
        const float* src = xyz + (b * N + (int64_t)j) * 3;
        out[e] = make_float4(src[0], src[1], src[2], __uint_as_float(j));
    }
}

hipError_t launch_scan_walk(const float* xyz, int B, int N, int64_t stride, float4* out, hipStream_t stream)
{
    const int64_t total = (int64_t)B * N;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(scan_walk_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, xyz, total, N,
                       (uint64_t)stride, out);
    return hipGetLastError();
}

hipError_t launch_zero_words(uint64_t* p, int64_t nwords, uint64_t* p2, int64_t nwords2, uint64_t* p3,
                             int64_t nwords3, hipStream_t stream)
{
    int64_t most = nwords > nwords2 ? nwords : nwords2;
    most = most > nwords3 ? most : nwords3;
    if (most <= 0) return hipSuccess;
    int blocks = (int)((most + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(zero_words_kernel, dim3(blocks), dim3(256), 0, stream, p, nwords > 0 ? nwords : 0, p2,
                       nwords2 > 0 ? nwords2 : 0, p3, nwords3 > 0 ? nwords3 : 0);
    return hipGetLastError();
}

}  // namespace fastpoint
