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
constexpr int kStage = 256;             // ring of picks not yet written to global memory
constexpr int kFlush = 128;             // ... written out once this many are waiting
constexpr int kCtrlThreads = 64;        // the control wave, after the T point threads

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
// in acceptance order.  A slot is one 64-bit word: low half = round tag << 8 | lane of the pick
// in the candidate list (kLiveEnd: the round has no further pick), high half = the pick's
// squared distance bits.  It is written by all lanes of the control wave with the same value (one
// 64-bit store); readers take the pick's coordinates from the candidate list.  The LDS executes
// the operations of one wave in issue order; the fences only restrain the compiler.
constexpr uint32_t kLiveEnd = 0xFFu;

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
    Cand cand[kCandMax];
    long long phase_t[5];      // constant 100 MHz clock at the phase boundaries of the cloud in hand (thread 0)
    int32_t rank[kCandMax];    // cell-ordered variant: position of a candidate among those of its round, by index
    Cand pend[kCand];
    int32_t bl[FP_MAX_SEG];    // segment boundaries b_l (curve positions that become thresholds)
    int32_t qend[FP_MAX_SEG + 1];   // qend[l] = ceil(n l / nseg): the quota rule raises the level to l + 1 there
    int32_t mlp_pos[32];       // MLP estimator: curve positions i_k of its 32 inputs (-1: not in use)
    float mlp_val[32];         // ... the curve there
    double mlp_a[128], mlp_b[128];   // ... activations of successive layers
    int32_t gpre[kMaxGroup + 1];
    int32_t ctrl[4];      // [0] accepted picks of the round, [1] points passing in the cloud,
                          // [2] failure, [3] distance bits of the last accepted pick
    // picks of the round being resolved, in acceptance order
    uint64_t live[kCandMax + 2];
#ifdef FASTPOINT_PHASE_CLOCKS
    long long chain_cycles;   // shader clocks the control wave spent in the exact-FPS chain loop
    long long chain_picks;
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
template <int P, bool BQ, bool DENSE, int P0>
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
            if (BQ) tmin = min(tmin, tb[u]);
        }
        if (BQ) {
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
        fold_groups<P, BQ, DENSE, P0 + GRP>(pt, cx, cy, cz, bq_r2, s, rw);
    }
}

template <int P, bool BQ, bool DENSE = true>
__device__ __forceinline__ void fold(Points<P, BQ>& pt, float cx, float cy, float cz,
                                     const SamplerArgs& a, const Where& wh, int s, RowWords<P, BQ>& rw)
{
    fold_groups<P, BQ, DENSE, 0>(pt, cx, cy, cz, a.bq_r2, s, rw);
}

// Hands the words of `count` picks (sample positions base, base+1, ...; count <= 64) to the cache.
// Lane s looks at the words of pick s; only a word that is not zero -- the ball holds one of the
// block's 64 points -- becomes an entry (sample, block, word) of the cloud's list.  A wave fills
// chunks of kBqChunk entries that it reserves from the cloud's chunk counter: the places inside a
// chunk come from ballots and bit counts, and the atomic addition that reserves the next chunk is
// issued when a chunk is taken and read when that chunk is full, so no wave ever waits for memory
// here (except for its very first entry of a cloud).  After every call lane 0 notes how much of the
// chunk is in use.  When no chunk is left the cloud's overflow flag is raised and the wave records
// nothing more: readers then treat the cloud as not recorded.
template <int P, bool BQ>
__device__ __forceinline__ void flush_rows(const RowWords<P, BQ>& rw, const SamplerArgs& a, const Where& wh,
                                           Points<P, BQ>& pt, int base, int count)
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
                        e.q = (uint32_t)(base + wh.lane);
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

// Cell-ordered variant: which of the first `count` entries of `list` can lower a distance of
// this wave (one entry per lane), and the wave's bound brought up to date.
template <int P, bool BQ>
__device__ __forceinline__ uint64_t near_mask(const Points<P, BQ>& pt, const Cand* list, int count, int lane)
{
    const Cand c = list[lane < count ? lane : 0];
    const float bd = box_dist2<P, BQ>(pt, c.x, c.y, c.z);
    return __builtin_amdgcn_ballot_w64(lane < count && __float_as_uint(bd) < pt.ub);
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
    rw.clear(wh);
    if constexpr (PERM) {
        uint64_t near = near_mask<P, BQ>(pt, sh.pend, npend, wh.lane);
        while (near != 0) {
            const int s = first_lane(near);
            near &= near - 1;
            const Cand cur = sh.pend[s];
            fold<P, BQ>(pt, cur.x, cur.y, cur.z, a, wh, s, rw);
        }
        return;
    }
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
template <int T, int P, bool BQ, bool PERM, bool WIDE>
__device__ __forceinline__ void follow_picks(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                             const SamplerArgs& a, int base, uint32_t tag, int total)
{
    int s = 0;
    RowWords<P, BQ> rw;
    rw.clear(wh);
    uint64_t near = ~0ull, near_hi = ~0ull;         // one bit per candidate (near_hi: candidates 64..127)
    if constexpr (PERM) {
        near = near_mask<P, BQ>(pt, sh.cand, total < 64 ? total : 64, wh.lane);
        if constexpr (WIDE) near_hi = near_mask<P, BQ>(pt, sh.cand + 64, total - 64, wh.lane);
    }
    uint32_t slot = lds_observe(&sh.live[0]);
    // Lane s of `rw` holds the words of a pick, so a recording wave takes a wide round in two halves
    // of up to 64 picks and hands the first half's words over in between; that hand-over is kept
    // out of the loop over the picks (whatever is written there would be carried, and copied,
    // through every iteration).
    constexpr int kHalves = (WIDE && BQ) ? 2 : 1;
    bool ended = false;
#pragma unroll 1
    for (int half = 0; half < kHalves && !ended; ++half) {
        const int stop = kHalves == 2 ? 64 * (half + 1) : 0x7FFFFFFF;
        if (half == 1) {
            flush_rows<P, BQ>(rw, a, wh, pt, base, 64);
            rw.clear(wh);
        }
        for (;;) {
            // wait for slot s of this round (requested before the previous pick was folded); nothing
            // but the slot changes in the inner loop, so the distances and row words stay where they
            // are across it
            slot = uni(slot);
            while ((slot & ~0xFFu) != tag) {        // not written yet in this round
                __builtin_amdgcn_s_sleep(1);
                slot = uni(lds_observe(&sh.live[s]));
            }
            if ((slot & 0xFFu) == kLiveEnd) {
                ended = true;
                break;
            }
            if (s == stop) break;                   // the slot stays in hand for the second half
            const uint32_t cl = slot & 0xFFu;
            slot = lds_observe(&sh.live[s + 1]);
            const uint64_t nbit = (WIDE && cl >= 64u) ? (near_hi >> (cl - 64u)) : (near >> cl);
            if (!PERM || (nbit & 1ull) != 0) {
                const Cand c = sh.cand[cl];
                // narrow rounds are those of clouds held by one or a few workgroups
                fold<P, BQ, !WIDE>(pt, c.x, c.y, c.z, a, wh, WIDE ? (s & 63) : s, rw);
            }
            ++s;
        }
    }
    if (WIDE)   // the picks not written yet: all of them up to 64, else those from the 65th on
        flush_rows<P, BQ>(rw, a, wh, pt, s > 64 ? base + 64 : base, s > 64 ? s - 64 : s);
    else
        flush_rows<P, BQ>(rw, a, wh, pt, base, s);  // a round has at most kCand picks
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
    long long clk[8];
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
// cell-ordered variant) the point's own index lies in [win_lo, win_lo + win_len).
template <int P, bool BQ, bool STRICT, bool WIN>
__device__ __forceinline__ bool passes(const Points<P, BQ>& pt, int p, float thr, uint32_t win_lo, uint32_t win_len)
{
    const bool av = STRICT ? (pt.d[p] > thr) : (pt.d[p] >= thr);
    if constexpr (WIN) return av && (uint32_t)(pt.oi[p] - win_lo) < win_len;
    return av;
}

// Collects the cloud's first CAP points (in the order the workgroups hold them: ascending index,
// or cell order in the cell-ordered variant) that pass -- see passes() -- into sh.cand of every
// workgroup.  Returns the number collected (at most CAP), -1 if a wait expired; `alltot`
// receives the number of points that pass in the whole cloud.
template <int T, int P, bool BQ, bool PERM, bool STRICT, int CAP, bool WIN = false>
__device__ __forceinline__ int scan_candidates(const Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                               const SamplerArgs& a, uint32_t& seq, float thr, int& alltot,
                                               uint32_t win_lo = 0, uint32_t win_len = 0)
{
    constexpr int NW = T / 64;
    // 1. how many of this wave's points pass
    int cntw = 0;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const bool av = passes<P, BQ, STRICT, WIN>(pt, p, thr, win_lo, win_len);
        cntw += __builtin_popcountll(__builtin_amdgcn_ballot_w64(av));
    }
    if (wh.lane == 0 && !wh.ctrl) sh.wcnt[wh.w] = cntw;     // the control wave has none (cntw == 0)
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
            const bool av = passes<P, BQ, STRICT, WIN>(pt, p, thr, win_lo, win_len);
            const uint64_t mk = __builtin_amdgcn_ballot_w64(av);
            if (mk != 0 && base < CAP) {
                const int rank = base + lanes_below(mk);
                if (av && rank < CAP) {
                    Cand cd;
                    cd.idx = PERM ? pt.oi[p] : (uint32_t)(((wh.gw * P + p) << 6) | wh.lane);
                    cd.x = pt.x[p];
                    cd.y = pt.y[p];
                    cd.z = pt.z[p];
                    cd.d = __float_as_uint(pt.d[p]);
                    sh.cand[rank] = cd;
                }
                base += __builtin_popcountll(mk);
            }
        }
    }
    __syncthreads();
    int total = tot < CAP ? tot : CAP;
    alltot = tot;
    if (wh.G == 1) return total;

    // 3. exchange: every workgroup publishes its list, all take the first CAP of the cloud
    //    in workgroup (= index) order
    //    (lists CAP entries apart: a word is only taken with this round's stamp, so rounds of
    //    different CAP may lay the same buffer out differently)
    ++seq;
    const int par = (int)(seq & 1u);
    uint64_t* pk = a.ll_pk + ((int64_t)(wh.grp * 2 + par) * wh.G) * kLlSlotWords;
    uint64_t* cd = a.ll_cd + ((int64_t)(wh.grp * 2 + par) * wh.G) * (kCandMax * kCandWords);
    for (int e = wh.tid; e < total * kCandWords; e += T + kCtrlThreads) {
        const int r = e / kCandWords, k = e - r * kCandWords;
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&sh.cand[r]);
        ll_store(cd + ((int64_t)wh.g * CAP + r) * kCandWords + k, src[k], seq);
    }
    if (wh.tid == 0) ll_store(pk + (int64_t)wh.g * kLlSlotWords + 5, (uint32_t)tot, seq);
    __syncthreads();          // sh.cand is about to be overwritten
    // More than 64 workgroups: thread t waits for the count of workgroup t, so that all waits
    // are in flight together, and hands it over in LDS.  Up to 64: the lanes of wave 0 wait
    // themselves (one count each), which saves the barrier.
    const bool spread = wh.G > 64;
    if (spread) {
        if (wh.tid < wh.G) {
            uint32_t val[1];
            const bool got = ll_wait<1>(pk + (int64_t)wh.tid * kLlSlotWords + 5, seq, val, a.wait_ticks);
            sh.gpre[wh.tid + 1] = got ? (int)val[0] : -1;
        }
        __syncthreads();
    }
    if (wh.w == 0) {
        // lane t adds up the counts of workgroups [t*per, (t+1)*per)
        const int per = (wh.G + 63) / 64;
        int sum = 0, usum = 0;
        bool bad = false;
        for (int k = 0; k < per; ++k) {
            const int t = wh.lane * per + k;
            if (t < wh.G) {
                int v;
                if (spread) {
                    v = sh.gpre[t + 1];
                } else {
                    uint32_t val[1];
                    v = ll_wait<1>(pk + (int64_t)t * kLlSlotWords + 5, seq, val, a.wait_ticks) ? (int)val[0] : -1;
                }
                if (v < 0) {
                    bad = true;
                } else {
                    usum += v;
                    sum += v < CAP ? v : CAP;
                }
                sh.gpre[t + 1] = sum;      // inclusive inside the lane, fixed below
            }
        }
        int incl = sum;
        for (int s = 1; s < 64; s <<= 1) {
            const int up = __shfl_up(incl, s, 64);
            if (wh.lane >= s) incl += up;
        }
        const int excl = incl - sum;
        for (int k = 0; k < per; ++k) {
            const int t = wh.lane * per + k;
            if (t < wh.G) sh.gpre[t + 1] += excl;
        }
        for (int s = 32; s > 0; s >>= 1) usum += __shfl_xor(usum, s, 64);
        const bool anybad = __builtin_amdgcn_ballot_w64(bad) != 0;
        if (wh.lane == 0) {
            sh.gpre[0] = 0;
            sh.ctrl[1] = usum;
            if (anybad) sh.ctrl[2] = 1;
        }
    }
    __syncthreads();
    alltot = uni(sh.ctrl[1]);
    const int listed = uni(sh.gpre[wh.G]);
    total = listed < CAP ? listed : CAP;
    if (uni(sh.ctrl[2]) == 0) {
        for (int e = wh.tid; e < total * kCandWords; e += T + kCtrlThreads) {
            const int r = e / kCandWords, k = e - r * kCandWords;
            int lo = 0, hi = wh.G;             // workgroup whose range holds rank r
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (sh.gpre[mid] <= r) lo = mid;
                else hi = mid;
            }
            uint32_t val[1];
            val[0] = 0;
            const bool got = ll_wait<1>(cd + ((int64_t)lo * CAP + (r - sh.gpre[lo])) * kCandWords + k, seq,
                                        val, a.wait_ticks);
            if (!got) sh.ctrl[2] = 1;
            reinterpret_cast<uint32_t*>(&sh.cand[r])[k] = val[0];
        }
    }
    __syncthreads();
    return uni(sh.ctrl[2]) != 0 ? -1 : total;
}

// Cell-ordered variant: the candidates of a threshold round arrive in cell order, the rule of
// the threshold phase takes them by index.  rank = number of candidates with a lower index (the
// indices differ); the point waves count a share of the comparisons each.  Called by all threads.
template <int T>
__device__ __forceinline__ void sort_candidates(Shared<T>& sh, const Where& wh, int total)
{
    constexpr int NW = T / 64;
    total = uni(total);
    if (total < 2) return;
    if (wh.tid < kCandMax) sh.rank[wh.tid] = 0;
    __syncthreads();
    if (!wh.ctrl) {
        const int chunk = (total + NW - 1) / NW;
        const int j0 = wh.w * chunk;
        const int j1 = j0 + chunk < total ? j0 + chunk : total;
        const bool h0 = wh.lane < total, h1 = wh.lane + 64 < total;
        const uint32_t k0 = sh.cand[h0 ? wh.lane : 0].idx;
        const uint32_t k1 = sh.cand[h1 ? wh.lane + 64 : 0].idx;
        int r0 = 0, r1 = 0;
        for (int j = j0; j < j1; ++j) {
            const uint32_t key = sh.cand[j].idx;
            r0 += key < k0 ? 1 : 0;
            r1 += key < k1 ? 1 : 0;
        }
        if (h0 && r0 != 0) atomicAdd(&sh.rank[wh.lane], r0);
        if (h1 && r1 != 0) atomicAdd(&sh.rank[wh.lane + 64], r1);
    }
    __syncthreads();
    Cand me = {};
    int r = 0;
    if (wh.tid < total) {
        me = sh.cand[wh.tid];
        r = sh.rank[wh.tid];
    }
    __syncthreads();
    if (wh.tid < total) sh.cand[r] = me;
    __syncthreads();
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
            const uint32_t cl = (uint32_t)sh.live[t] & 0xFFu;
            stage_pick<T>(sh, st.i + t, sh.cand[cl].idx, 0.0f);
        }
    } else if (wh.lane < nacc) {
        const uint32_t cl = (uint32_t)sh.live[wh.lane] & 0xFFu;
        stage_pick<T>(sh, st.i + wh.lane, sh.cand[cl].idx, 0.0f);
    }
    if (wh.lane == 0) sh.ctrl[0] = nacc;
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

template <int T, bool PERM, bool WIDE>
__device__ __forceinline__ void resolve_chain(Shared<T>& sh, const Where& wh, const CloudState& st,
                                              int total, int limit, float tau, bool capture, int nseg,
                                              uint32_t tag)
{
    total = uni(total);
    limit = uni(limit);
    const bool has = wh.lane < total;
    const Cand me = sh.cand[has ? wh.lane : 0];
    uint32_t cd = has ? me.d : 0u;                     // bit pattern; distances are >= +0
    const bool has1 = WIDE && wh.lane + 64 < total;
    Cand me1 = me;
    if constexpr (WIDE) me1 = sh.cand[has1 ? wh.lane + 64 : 0];
    uint32_t cd1 = has1 ? me1.d : 0u;
    const uint32_t tau_bits = uni(__float_as_uint(tau));    // tau >= 0
    uint32_t dl = __float_as_uint(st.dlast);
    LiveCursor cur(tag);
    __builtin_amdgcn_s_setprio(3);
#ifdef FASTPOINT_PHASE_CLOCKS
    const long long chain_t0 = clock64();
#endif
    // the candidates have arrived from LDS before the loop starts, not inside it
    asm volatile("" ::"v"(me.x), "v"(me.y), "v"(me.z), "v"(cd));
    int nacc;
    if constexpr (WIDE) {
        asm volatile("" ::"v"(me1.x), "v"(me1.y), "v"(me1.z), "v"(cd1));
        nacc = limit >= total
                   ? chain_loop_wide<false, PERM>(sh.live, cur, me, me1, cd, cd1, tau_bits, limit, dl)
                   : chain_loop_wide<true, PERM>(sh.live, cur, me, me1, cd, cd1, tau_bits, limit, dl);
    } else {
        nacc = limit >= total ? chain_loop<false, PERM>(sh.live, cur, me, cd, tau_bits, limit, dl)
                              : chain_loop<true, PERM>(sh.live, cur, me, cd, tau_bits, limit, dl);
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
        stage_pick<T>(sh, pos, sh.cand[(uint32_t)word & 0xFFu].idx, d);
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
template <int T, int P, bool BQ, bool PERM, bool kWideFps>
__device__ __forceinline__ bool fps_rounds_of(Points<P, BQ>& pt, Shared<T>& sh, const Where& wh,
                                              const SamplerArgs& a, uint32_t& it, uint32_t& seq,
                                              CloudState& st, int upto, bool capture)
{
    constexpr int kCandFps = kWideFps ? kCandMax : kCand;
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
                total = scan_candidates<T, P, BQ, PERM, true, kCandFps>(pt, sh, wh, a, seq, tau, alltot);
                PHASE_END(st, 1);
                if (total < 0) return false;
                ++st.rounds;
                if (alltot > 0 && alltot <= kCandFps) good = true;
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
            const uint32_t tag = (uint32_t)(st.resolved + 1) << 8;
            if (wh.ctrl) resolve_chain<T, PERM, kWideFps>(sh, wh, st, total, upto - st.i, tau, capture, a.nseg, tag);
            else follow_picks<T, P, BQ, PERM, kWideFps>(pt, sh, wh, a, st.i, tag, total);
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

// Rounds of 64 or of 128 candidates.  With four or more points per thread folding a pick takes the
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
    if constexpr (P >= 4) {
        return fps_rounds_of<T, P, BQ, PERM, true>(pt, sh, wh, a, it, seq, st, upto, capture);
    } else {
        if constexpr (!PERM && !ONE_WG) // (the cell-ordered variant gained nothing there and pays for the code)
            if (wh.G >= 8) return fps_rounds_of<T, P, BQ, PERM, true>(pt, sh, wh, a, it, seq, st, upto, capture);
        return fps_rounds_of<T, P, BQ, PERM, false>(pt, sh, wh, a, it, seq, st, upto, capture);
    }
}

// ------------------------------------------------------------------ one cloud
// MODE 0: exact FPS only (the code of Alg. 2 is left out of the kernel); 1: MDPS with threshold rounds
// of kCand candidates; 2: MDPS with threshold rounds of kCandMax candidates.
template <int T, int P, bool BQ, bool PERM, int MODE>
__device__ __forceinline__ void run_cloud(const SamplerArgs& a, Shared<T>& sh, const Where& wh,
                                          uint32_t& it, uint32_t& seq)
{
    constexpr bool WIDE = MODE == 2;
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
    if (wh.tid < kCandMax + 2) sh.live[wh.tid] = 0;    // round tags start at 1 in every cloud
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
    for (int k = 0; k < 8; ++k) st.clk[k] = 0;
    const long long cloud_t0__ = wall_clock64();
#endif
    if (wh.tid == 0) {
        sh.ctrl[2] = 0;
#ifdef FASTPOINT_PHASE_CLOCKS
        sh.chain_cycles = 0;
        sh.chain_picks = 0;
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
        constexpr int kCandThr = WIDE ? kCandMax : kCand;
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
            if constexpr (PERM) refresh_bound<P, BQ>(pt);
            const float r2 = unif(sh.thr[seg - 1]);
            // samples of this level end where the quota rule would raise the level
            const int limit = (level_end < n ? level_end : n) - st.i;
            ++st.rounds;
            int alltot = 0;
#ifdef FASTPOINT_PHASE_CLOCKS
            const long long thr_t0 = wall_clock64();
#endif
            int total = scan_candidates<T, P, BQ, PERM, false, kCandThr, PERM>(pt, sh, wh, a, seq, r2, alltot,
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
            if constexpr (PERM) {
                window_is_last = (uint64_t)win_lo + win_len >= (uint64_t)N;
                if (total >= 0 && alltot > kCandThr) {      // more than a round holds: a shorter window
                    const uint64_t len = (uint64_t)win_len * (uint64_t)(kCandThr * 7 / 8) / (uint64_t)alltot;
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
            if constexpr (PERM) sort_candidates<T>(sh, wh, total);
            const uint32_t tag = (uint32_t)(st.resolved + 1) << 8;
            if (wh.ctrl) resolve_threshold<T, WIDE>(sh, wh, st, total, limit, r2, tag);
            else follow_picks<T, P, BQ, PERM, WIDE>(pt, sh, wh, a, st.i, tag, total);
            __syncthreads();
            ++st.resolved;
            st.npend = 0;                           // folded while they were resolved
            st.i += uni(sh.ctrl[0]);
#ifdef FASTPOINT_PHASE_CLOCKS
            st.clk[5] += wall_clock64() - thr_t1;
#endif
            bool exhausted = alltot < kCandThr;
            if constexpr (PERM) {
                // the quota did not cut the round short (checked below): the window is worked off;
                // the next one is as long as should hold seven eighths of a round's candidates
                exhausted = window_is_last;
                win_lo = window_is_last ? 0u : win_lo + win_len;
                uint64_t len = (uint64_t)win_len * (uint64_t)(kCandThr * 7 / 8) / (uint64_t)(alltot > 0 ? alltot : 1);
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
            inf.thr2[12] = (float)sh.chain_cycles;
            inf.thr2[13] = (float)sh.chain_picks;
        }
#endif
        inf.status = ok ? 0 : 2;
        a.info[wh.c] = inf;
    }
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
            *reinterpret_cast<BqHeader*>(a.bq_base) = bq_layout(a.B, a.N, a.n, a.bq_r2, a.bq_cap);
    }
    uint32_t it = 0, seq = 0;
    for (int c = wh.grp; c < a.B; c += ngroups) {
        wh.c = c;
        run_cloud<T, P, BQ, PERM, MODE>(a, sh, wh, it, seq);
    }
}

// zeroes two ranges of words before a launch: the exchange words (stamps start at 1 in every
// launch) and the counters of a ball-query cache
__global__ void zero_words_kernel(uint64_t* p, int64_t nwords, uint64_t* p2, int64_t nwords2)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = i; t < nwords; t += stride) p[t] = 0;
    for (int64_t t = i; t < nwords2; t += stride) p2[t] = 0;
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
    if (perm) {                     // cell-ordered: no recording, threshold rounds always wide
        if (bq || mode == 1) return nullptr;
        return mode == 0 ? reinterpret_cast<const void*>(&sampler_kernel<T, P, false, true, 0>)
                         : reinterpret_cast<const void*>(&sampler_kernel<T, P, false, true, 2>);
    }
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

hipError_t launch_zero_words(uint64_t* p, int64_t nwords, uint64_t* p2, int64_t nwords2, hipStream_t stream)
{
    const int64_t most = nwords > nwords2 ? nwords : nwords2;
    if (most <= 0) return hipSuccess;
    int blocks = (int)((most + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(zero_words_kernel, dim3(blocks), dim3(256), 0, stream, p, nwords > 0 ? nwords : 0, p2,
                       nwords2 > 0 ? nwords2 : 0);
    return hipGetLastError();
}

}  // namespace fastpoint
