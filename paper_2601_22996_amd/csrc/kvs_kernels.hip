/*
 * kvs_kernels.hip -- gfx950 kernels and C ABI of the schedule-evaluation
 * library (declared in include/kvsched.h).
 *
 * Citations: "Competitive Non-Clairvoyant KV-Cache Scheduling for LLM
 * Inference" (Feng, Yang, Zhang): Section 2.1 (model, occupancy, flow time),
 * Procedure 1 (SPS), appendix "Lower Bounds for SimS" (SimS), Lemmas "Peak
 * Memory Usage of SPS" / "Feasible Parallelism of SPS", Algorithms 1 (GSA)
 * and 2 (GBA).
 *
 * Design in one paragraph.  Sweep points whose initial slices are
 * base * 2^m share one ladder of slices base * 2^g.  One workgroup takes one
 * instance and one such group of points.  A job's class on the ladder does
 * not depend on m; a point with shift m merges the levels 0..m into its
 * first phase and uses the levels above m unchanged.  So every level phase is
 * evaluated once per (subroutine, parallelism) variant and shared by all the
 * points, and only the merged first phases are evaluated per shift.  Jobs are
 * brought into phase order in LDS: when every job has exactly one phase, a
 * copy of the instance is cut into the phases by stable partitions inside LDS
 * (the jobs are read from memory once); otherwise each phase is compacted
 * from memory.  Inside
 * a phase nothing is stepped round by round: the occupancy of round t is
 *     occ(t) = A(t) + t * C(t),
 *     C(t) = number of active runs,  A(t) = sum over them of (s + 1 - start),
 * both prefix sums over time of per-round event sums (a run adds
 * (s + 1 - start, 1) in its first round and takes it away in the round after
 * its last).  The rounds of a phase are cut into slabs; a wavefront takes a
 * slab, sums the runs already active when it begins, scatters the events
 * that fall inside into its own LDS window, scans it and keeps the maximum.
 * Slabs need nothing from each other, so no barrier is taken while phases
 * are evaluated.  All values are exact integers: the result equals the
 * stepped definition bit for bit.
 */
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "kvsched.h"
#include "kvsched_test.h"
#include "kvs_internal.h"
#include "kvs_math.h"
#include "kvs_phase.h"
#include "kvs_wave.h"

namespace {

constexpr int kLevelsGeo = 32;         /* ladder levels base * 2^g that 2^30-bounded lengths can reach */
constexpr int kLevelsMax = KVS_MAX_LEVELS; /* levels of an explicit ladder                              */
constexpr int kMaxM = 8;               /* distinct shifts m per launch                                  */
constexpr int kMaxV = 4;               /* distinct (subroutine, parallelism) variants per launch        */
constexpr uint32_t kLenMax = 1u << 30; /* largest length the 32-bit arithmetic is sized for             */

/* what is wrong with an instance's job data; any of these and none of its points is evaluated */
constexpr uint32_t FLAG_EINVAL = 1u; /* o < 1, s < 0, o_est < 1, or no slice of an explicit ladder covers a job */
constexpr uint32_t FLAG_ERANGE = 2u; /* a length above 2^30                                                       */
constexpr uint32_t FLAG_EJOB = 4u;   /* s + o > M: the job does not fit the budget on its own (Section 2.1)        */
constexpr uint8_t FEASIBLE_PENDING = 0xFD; /* internal: left for the two-word-entry kernel */

constexpr int MODE_GBA = 0, MODE_GSA = 1, MODE_SINGLE = 2;

/*
 * The instantiations of the evaluation kernel, by how the jobs get into phase order in LDS.
 *   NESTED  every job has one phase (Algorithm 2 on true lengths): a copy of the instance
 *           is cut into the phases by stable partitions inside LDS;
 *   ALIVE   every job is tried in every phase until it completes (Algorithm 1, and a lone
 *           invocation of the subroutine): the unfinished jobs stay in LDS in input order,
 *           phases are evaluated from that list and the completed jobs are taken out of it;
 *   GATHER  classes by estimates: the instance stays in LDS beside the phase buffer and the
 *           phases are gathered from it, as many at a time as the buffer holds;
 *   STREAM  the same, gathered from memory (instances too large for two copies in LDS
 *           beside a second workgroup);
 *   WIDE    two-word entries, every phase compacted from memory: whatever the others
 *           leave behind because a value is too wide for their one-word entries.
 * The first four read the jobs from memory once (STREAM: once per batch of phases).
 */
constexpr int KIND_NESTED = 0, KIND_ALIVE = 1, KIND_GATHER = 2, KIND_STREAM = 3, KIND_WIDE = 4;

struct JobsDev {
    const int32_t *o;
    const int32_t *s;
    const int32_t *e;
    int32_t n_inst;
    int32_t n_jobs;
    uint32_t s_scalar;
    uint32_t vec4; /* rows are 16-byte aligned and n_jobs is a multiple of 4: 128-bit loads allowed */
    uint32_t wide_all; /* two-word kernel: every instance is its to do, not only the marked ones   */
    uint64_t M;
};

/* One launch: the points of a sweep that share a ladder. */
struct GroupArg {
    uint32_t base;                   /* slice of level 0; level g has base << g                  */
    uint32_t v_k[kMaxV];             /* forced parallelism per variant, 0 = automatic            */
    uint16_t pt_q[KVS_MAX_POINTS];   /* output row of each point                                 */
    uint8_t pt_m[KVS_MAX_POINTS];    /* index into m[]                                           */
    uint8_t pt_v[KVS_MAX_POINTS];    /* index into the variants                                  */
    uint8_t m[kMaxM];                /* shifts: the point's initial slice is base << m           */
    uint8_t v_sched[kMaxV];
    uint8_t lg_base, mode, n_m, n_v, n_pts;
    uint8_t n_lv;                    /* > 0: the slices are ladder[0 .. n_lv), not base << g     */
    uint32_t ladder[kLevelsMax];
};

struct OutsDev {
    int64_t *peak;
    uint8_t *feasible;
    int64_t *flow;
    int64_t *job_steps;
    int32_t *n_completed;
};

/* What one job means on the ladder. */
struct JobView {
    uint32_t o, s;
    uint32_t ga; /* level at which it first takes part           */
    uint32_t gb; /* level at which it takes part for the last time */
    uint32_t go; /* level of o: it completes in phases that reach it */
    uint32_t bad; /* FLAG_* bits, 0 for a job that can be scheduled */
};

/* A job as it sits in memory. */
struct RawJob {
    int32_t o, s, e;
};

__device__ __forceinline__ RawJob load_job(const JobsDev &J, size_t idx, bool want_e)
{
    RawJob r;
    r.o = J.o[idx];
    r.s = J.s ? J.s[idx] : (int32_t)J.s_scalar;
    r.e = want_e ? J.e[idx] : 1;
    return r;
}

/* Level of a length on the launch's ladder: the smallest g whose slice is >= x.
 * Geometric ladders (base << g) answer with a leading-zero count; explicit
 * ones are searched (lad holds the n_lv slices in LDS, non-decreasing); a
 * length above the last slice has no level and is reported through ok. */
template <bool EXPLICIT>
__device__ __forceinline__ uint32_t level_of(uint32_t x, const GroupArg &G, const uint32_t *lad,
                                             bool &ok)
{
    if (!EXPLICIT)
        return kvs_class_index(x, G.base, G.lg_base);
    static_assert(kLevelsMax == 64, "kvs_ladder_level searches 64 slices");
    uint32_t p = kvs_ladder_level(x, lad, G.n_lv);
    if (p >= G.n_lv) {
        ok = false;
        p = G.n_lv - 1u;
    }
    return p;
}

template <bool EXPLICIT>
__device__ __forceinline__ JobView view_job(const RawJob &r, const JobsDev &J, const GroupArg &G,
                                            const uint32_t *lad, int mode, bool with_estimates)
{
    JobView v;
    const int32_t o = r.o;
    const int32_t s = r.s;
    bool covered = true; /* some slice of an explicit ladder reaches the length */
    v.bad = 0;
    if (o < 1 || s < 0)
        v.bad = FLAG_EINVAL;
    else if ((uint32_t)o > kLenMax || (uint32_t)s > kLenMax)
        v.bad = FLAG_ERANGE;
    else if ((uint64_t)(uint32_t)s + (uint64_t)(uint32_t)o > J.M)
        v.bad = FLAG_EJOB;
    v.o = (o < 1) ? 1u : ((uint32_t)o > kLenMax ? kLenMax : (uint32_t)o);
    v.s = (s < 0) ? 0u : ((uint32_t)s > kLenMax ? kLenMax : (uint32_t)s);
    v.go = level_of<EXPLICIT>(v.o, G, lad, covered);
    if (mode != MODE_GBA) { /* GSA, or one invocation of the subroutine: everybody from the start */
        v.ga = 0;
        v.gb = v.go;
    } else if (with_estimates) {
        const int32_t e = r.e;
        if (e < 1)
            v.bad |= FLAG_EINVAL;
        else if ((uint32_t)e > kLenMax)
            v.bad |= FLAG_ERANGE;
        uint64_t cap = (J.M > v.s) ? (J.M - v.s) : 1u; /* M - s, at least 1 */
        if (cap > kLenMax)
            cap = kLenMax;
        uint32_t eu = (e < 1) ? 1u : (uint32_t)e;
        if (eu > (uint32_t)cap)
            eu = (uint32_t)cap;
        v.ga = level_of<EXPLICIT>(eu, G, lad, covered);
        v.gb = v.ga > v.go ? v.ga : v.go;
    } else {
        v.ga = v.go;
        v.gb = v.go;
    }
    if (!covered)
        v.bad |= FLAG_EINVAL;
    return v;
}

/* One instance at the points of one launch, by one workgroup of T threads. */
template <int T, int KIND, int WIN, int LV, int HOLD>
__device__ __forceinline__ void sweep_instance(const JobsDev &J, const GroupArg &G, const OutsDev &out,
                                               const uint32_t inst)
{
    constexpr int NW = T / 64;
    constexpr int kLevels = LV;          /* levels of the ladder this instantiation can hold */
    constexpr int kSlots = LV + kMaxM;   /* phase slots: one per level, one per merged first phase */
    constexpr bool EXPLICIT = (LV == kLevelsMax); /* explicit ladders get the large instantiation */
    static_assert(LV == kLevelsGeo || LV == kLevelsMax, "levels");
    constexpr bool PACKED = KIND != KIND_WIDE;   /* one-word entries */
    constexpr bool NESTED = KIND == KIND_NESTED;
    constexpr bool ALIVE = KIND == KIND_ALIVE;
    constexpr bool GATHERS = KIND == KIND_GATHER || KIND == KIND_STREAM;
    constexpr bool COPY = KIND == KIND_GATHER;   /* the instance is kept in LDS beside the phase buffer */
    static_assert(!GATHERS || PACKED, "the gathered entries are written as one word");

    /* Dynamic LDS.  Phase entries: n_jobs words, twice that when !PACKED.  COPY: behind them
     * the instance in input order, one word per job (prompt << 16 | length with per-job prompts,
     * else the length), and behind that one byte per job for its entry level. */
    extern __shared__ uint32_t buf[];

    static_assert(WIN % 64 == 0 && WIN <= kWinMax, "window size");
    __shared__ unsigned long long ev[NW][WIN];
    __shared__ uint32_t cumE[NW][kLevels]; /* per wavefront: jobs of its segment entering at levels <= l */
    __shared__ uint32_t cumL[NW][kLevels]; /* ... leaving at levels <= l                                  */
    __shared__ uint32_t totE[kLevels], totL[kLevels];
    __shared__ uint32_t upE[kLevels], upL[kLevels], upS[kLevels]; /* over the levels up to l: sums of totE, of totL, largest sMaxEnter */
    __shared__ uint8_t used[kSlots]; /* the slots that have a schedule of their own */
    __shared__ uint32_t n_used;
    __shared__ uint32_t sMaxPart[kLevels], sMaxEnter[kLevels];
    __shared__ uint32_t lad[kLevels]; /* slice of every level, saturated at 2^32 - 1 */
    __shared__ Slot slot[kSlots];
    __shared__ Sched sched[kMaxV][kSlots];
    __shared__ Result res[kMaxV][kSlots];
    __shared__ uint8_t order[kSlots];      /* GATHERS: the slots to evaluate, batch after batch */
    __shared__ uint8_t bstart[kSlots + 1]; /* ... batch b is order[bstart[b] .. bstart[b + 1])  */
    __shared__ uint32_t n_batches;
    __shared__ unsigned long long sumO_sh;
    __shared__ uint32_t flags, maxO_sh, maxS_sh, maxE_sh;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const uint32_t n = (uint32_t)J.n_jobs;
    const size_t row = (size_t)inst * n;
    const bool per_job_s = (J.s != nullptr);
    /* the one-phase instantiation is launched only for GBA on true lengths: saying so here lets
     * the compiler drop the other modes from it */
    /* what the host launches an instantiation for is said here, so that the compiler drops the
     * other modes from it */
    const int mode = (NESTED || GATHERS) ? MODE_GBA
                     : ALIVE ? ((int)G.mode == MODE_SINGLE ? MODE_SINGLE : MODE_GSA)
                             : (int)G.mode;
    const bool with_estimates = GATHERS || (!PACKED && mode == MODE_GBA && J.e != nullptr);
    const bool one_phase_each = NESTED || (!PACKED && mode == MODE_GBA && J.e == nullptr);
    const uint32_t m_min = G.m[0];
    uint32_t *const jobs_lds = buf + n;                                /* COPY only */
    uint8_t *const ga_lds = reinterpret_cast<uint8_t *>(buf + 2u * n); /* COPY only */

    /* each wavefront owns a contiguous segment of the jobs */
    const uint32_t seg = ((n + NW - 1) / NW + 63u) & ~63u; /* whole 64-job chunks: at most HOLD of them */
    const uint32_t seg_lo = (uint32_t)wave * seg < n ? (uint32_t)wave * seg : n;
    const uint32_t seg_hi = seg_lo + seg < n ? seg_lo + seg : n;

    if (tid < kLevels) {
        sMaxPart[tid] = 0;
        sMaxEnter[tid] = 0;
        if (EXPLICIT) {
            lad[tid] = (tid < (int)G.n_lv) ? G.ladder[tid] : 0xffffffffu;
        } else {
            const uint64_t tl = (uint64_t)G.base << tid;
            lad[tid] = tl > 0xffffffffull ? 0xffffffffu : (uint32_t)tl;
        }
    }
    for (int i = tid; i < NW * kLevels; i += T) {
        (&cumE[0][0])[i] = 0;
        (&cumL[0][0])[i] = 0;
    }
    if (tid == 0) {
        flags = 0;
        maxO_sh = 0;
        maxS_sh = 0;
        maxE_sh = 0;
        sumO_sh = 0;
    }
    __syncthreads();

    /* ---- pass 1: per wavefront, how many of its jobs enter / leave at each level ---- */
    {
        /* Most jobs fall into two or three levels, and lanes that add to the same counter are
         * served one after the other.  The wavefront's window, idle until phases are evaluated,
         * holds kRep copies of a level histogram, one per group of lanes (rows one word longer
         * than the levels, so equal levels of different copies sit in different banks): the
         * entry levels, or the levels at which the jobs complete where everybody enters at once
         * (ALIVE).  Where both differ from job to job (GATHERS) a second histogram with fewer
         * copies behind the first takes the completion levels. */
        constexpr int kRowE = kLevels + 1;
        constexpr int kRep = (2 * WIN / kRowE >= 8) ? 8 : (2 * WIN / kRowE >= 4) ? 4 : (2 * WIN / kRowE >= 2) ? 2 : 1;
        static_assert(kRep * kRowE <= 2 * WIN, "histogram copies fit the window");
        constexpr int kRoom2 = (2 * WIN - kRep * kRowE) / kRowE;
        constexpr int kRep2 = kRoom2 >= 4 ? 4 : kRoom2 >= 2 ? 2 : 1;
        static_assert(!GATHERS || kRoom2 >= 1, "the second histogram fits the window");
        uint32_t *histE = reinterpret_cast<uint32_t *>(ev[wave]);
        uint32_t *histL = histE + kRep * kRowE;
        for (int i = lane; i < (kRep + (GATHERS ? kRep2 : 0)) * kRowE; i += 64)
            histE[i] = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint32_t *myE = histE + (lane & (kRep - 1)) * kRowE;
        uint32_t *myL = histL + (lane & (kRep2 - 1)) * kRowE;
        unsigned long long sumO = 0;
        uint32_t mxO = 0, mxS = 0, mxG = 0;
        uint32_t badbits = 0;
        const bool want_e = with_estimates;
        /* first part of a job's accounting; returns the level that keeps its prompt, and the prompt */
        auto account_a = [&](const RawJob &raw, uint32_t i, uint32_t &g_out, uint32_t &s_out) {
            const JobView v = view_job<EXPLICIT>(raw, J, G, lad, mode, with_estimates);
            badbits |= v.bad;
            if (mode != MODE_SINGLE || v.go == 0)
                sumO += v.o; /* every job completes once; a lone invocation completes o <= tau */
            mxO = v.o > mxO ? v.o : mxO;
            mxS = v.s > mxS ? v.s : mxS;
            if (!NESTED) /* only the entry format of the other instantiations asks for it */
                mxG = v.gb > mxG ? v.gb : mxG;
            if (NESTED || ALIVE) /* the job as a phase entry (ALIVE: with its whole length), at its place in the input */
                buf[i] = per_job_s ? ((v.s << 16) | (v.o & 0xffffu)) : v.o;
            if (COPY) { /* the job itself, at its place in the input */
                jobs_lds[i] = per_job_s ? ((v.s << 16) | (v.o & 0xffffu)) : v.o;
                ga_lds[i] = (uint8_t)v.ga;
            }
            const uint32_t g_max = ALIVE ? v.gb : v.ga; /* the level that keeps this job's prompt */
            atomicAdd(&myE[g_max], 1u); /* the wavefront's own histogram */
            if (GATHERS)
                atomicAdd(&myL[v.gb], 1u);
            else if (!PACKED && !one_phase_each)
                atomicAdd(&cumL[wave][v.gb], 1u);
            if (per_job_s && !NESTED && !ALIVE) /* else one level says it all: the only one (NESTED), the last one (ALIVE) */
                for (uint32_t l = v.ga; l <= v.gb; l++)
                    if (v.s > sMaxPart[l]) /* the maxima settle after a few jobs; then this only reads */
                        atomicMax(&sMaxPart[l], v.s);
            g_out = g_max;
            s_out = v.s;
        };
        auto account = [&](const RawJob &raw, uint32_t i) {
            uint32_t g, s;
            account_a(raw, i, g, s);
            if (per_job_s && s > sMaxEnter[g]) /* settles after a few jobs; then this only reads */
                atomicMax(&sMaxEnter[g], s);
        };
        /* four jobs: their four looks at the prompt maxima travel to LDS together */
        auto account4 = [&](const RawJob &a, const RawJob &b, const RawJob &c, const RawJob &d, uint32_t i) {
            uint32_t g[4], s[4];
            account_a(a, i, g[0], s[0]);
            account_a(b, i + 1u, g[1], s[1]);
            account_a(c, i + 2u, g[2], s[2]);
            account_a(d, i + 3u, g[3], s[3]);
            if (per_job_s) {
                uint32_t cur[4];
#pragma unroll
                for (int q = 0; q < 4; q++)
                    cur[q] = sMaxEnter[g[q]];
#pragma unroll
                for (int q = 0; q < 4; q++)
                    if (s[q] > cur[q])
                        atomicMax(&sMaxEnter[g[q]], s[q]);
            }
        };
        if (J.vec4) {
            /* Four consecutive jobs per lane and 16-byte loads: pass 1 is bound by how many bytes a
             * wavefront keeps in flight, and nothing here depends on which lane sees which job.
             * (n_jobs and the segment bounds are multiples of 4, the rows 16-byte aligned.) */
            struct Quad {
                int4 o, s, e;
            };
            auto load4 = [&](uint32_t i) {
                Quad q;
                q.o = *reinterpret_cast<const int4 *>(J.o + row + i);
                q.s = J.s ? *reinterpret_cast<const int4 *>(J.s + row + i)
                          : make_int4((int)J.s_scalar, (int)J.s_scalar, (int)J.s_scalar, (int)J.s_scalar);
                q.e = want_e ? *reinterpret_cast<const int4 *>(J.e + row + i) : make_int4(1, 1, 1, 1);
                return q;
            };
            /* The loads of kDeep chunks are issued before the first is looked at: a segment is
             * only a few chunks long, and a workgroup in this pass has nothing else to wait with
             * (the registers are free: the evaluation's are not live yet). */
            constexpr uint32_t kDeep = 4;
            for (uint32_t base = seg_lo; base < seg_hi; base += 256u * kDeep) {
                Quad q[kDeep];
#pragma unroll
                for (uint32_t dch = 0; dch < kDeep; dch++) {
                    const uint32_t i = base + 256u * dch + 4u * (uint32_t)lane;
                    q[dch].o = q[dch].s = q[dch].e = make_int4(1, 1, 1, 1);
                    if (i < seg_hi)
                        q[dch] = load4(i);
                }
#pragma unroll
                for (uint32_t dch = 0; dch < kDeep; dch++) {
                    const uint32_t i = base + 256u * dch + 4u * (uint32_t)lane;
                    if (i < seg_hi) {
                        account4(RawJob{q[dch].o.x, q[dch].s.x, q[dch].e.x}, RawJob{q[dch].o.y, q[dch].s.y, q[dch].e.y},
                                 RawJob{q[dch].o.z, q[dch].s.z, q[dch].e.z}, RawJob{q[dch].o.w, q[dch].s.w, q[dch].e.w}, i);
                    }
                }
            }
        } else {
            RawJob nxt;
            nxt.o = nxt.s = nxt.e = 1;
            if (seg_lo + lane < seg_hi)
                nxt = load_job(J, row + seg_lo + lane, want_e);
            for (uint32_t base = seg_lo; base < seg_hi; base += 64) {
                const uint32_t i = base + lane;
                const RawJob raw = nxt;
                if (i + 64 < seg_hi) /* the next chunk's loads fly while this one is classified */
                    nxt = load_job(J, row + i + 64, want_e);
                if (i < seg_hi)
                    account(raw, i);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint32_t cntE = 0, cntL = 0;
        if (lane < kLevels) {
            for (int r = 0; r < kRep; r++)
                cntE += histE[r * kRowE + lane];
            if (GATHERS)
                for (int r = 0; r < kRep2; r++)
                    cntL += histL[r * kRowE + lane];
            else if (!PACKED && !one_phase_each)
                cntL = cumL[wave][lane];
            else
                cntL = cntE;
        }
        if (ALIVE) /* counted: the levels of completion; everybody enters at level 0 */
            cntE = (lane == 0) ? seg_hi - seg_lo : 0u;
        /* inclusive prefix over levels (lanes 0..31 hold the levels) */
        uint32_t pe = cntE, pl = cntL;
#pragma unroll
        for (int off = 1; off < kLevels; off <<= 1) {
            const uint32_t ue = __shfl_up(pe, off);
            const uint32_t ul = __shfl_up(pl, off);
            if (lane >= off) {
                pe += ue;
                pl += ul;
            }
        }
        if (lane < kLevels) {
            cumE[wave][lane] = pe;
            cumL[wave][lane] = pl;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            sumO += __shfl_xor(sumO, off);
            const uint32_t a = __shfl_xor(mxO, off), b = __shfl_xor(mxS, off),
                           c = __shfl_xor(mxG, off);
            mxO = a > mxO ? a : mxO;
            mxS = b > mxS ? b : mxS;
            mxG = c > mxG ? c : mxG;
        }
        if (lane == 0) {
            atomicAdd(&sumO_sh, sumO);
            atomicMax(&maxO_sh, mxO);
            atomicMax(&maxS_sh, mxS);
            atomicMax(&maxE_sh, mxG);
        }
        if (__any(badbits != 0)) {
#pragma unroll
            for (int off = 32; off > 0; off >>= 1)
                badbits |= __shfl_xor(badbits, off);
            if (lane == 0)
                atomicOr(&flags, badbits);
        }
    }
    __syncthreads();

    if (tid < kLevels) {
        uint32_t e = 0, l = 0;
        for (int w = 0; w < NW; w++) {
            e += cumE[w][tid] - (tid ? cumE[w][tid - 1] : 0u);
            l += cumL[w][tid] - (tid ? cumL[w][tid - 1] : 0u);
        }
        totE[tid] = e;
        totL[tid] = l;
        if (NESTED || ALIVE) {
            /* The partitions in LDS leave every wavefront the entries that came from its own
             * segment of the input, so what it keeps and where that goes follow from these counts
             * and nothing has to be counted again.  For that each count gets, beside it, the sum
             * over the wavefronts before: of cumE in cumL's place where every job has one phase
             * (the two are equal there), of cumL in cumE's place where everybody enters at once
             * (cumE is the segment length there). */
            uint32_t run = 0;
            for (int w = 0; w < NW; w++) {
                const uint32_t c = NESTED ? cumE[w][tid] : cumL[w][tid];
                (NESTED ? cumL : cumE)[w][tid] = run;
                run += c;
            }
        }
        /* the levels sit in the first lanes of the first wavefront: running sums and maximum */
        static_assert(kLevels <= 64, "one lane per level");
        uint32_t ue = e, ul = l, us = sMaxEnter[tid];
#pragma unroll
        for (int off = 1; off < kLevels; off <<= 1) {
            const uint32_t a = __shfl_up(ue, off), b = __shfl_up(ul, off), c = __shfl_up(us, off);
            if (tid >= off) {
                ue += a;
                ul += b;
                us = c > us ? c : us;
            }
        }
        upE[tid] = ue;
        upL[tid] = ul;
        upS[tid] = us;
        if (ALIVE && per_job_s) { /* a level's phase holds the jobs that complete there or later */
            uint32_t m = sMaxEnter[tid];
#pragma unroll
            for (int off = 1; off < kLevels; off <<= 1) {
                const uint32_t c = __shfl_down(m, off);
                if (tid + off < kLevels)
                    m = c > m ? c : m;
            }
            sMaxPart[tid] = m;
        }
    }
    __syncthreads();

    /* ---- entry format: does prompt | done | duration fit one word? ---- */
    /* One phase per job and values narrow enough for the copy pass 1 left in LDS (duration in
     * 16 bits under a 16-bit prompt, or a bare duration): every phase's entries are then cut out
     * of that copy inside LDS and the jobs are not read from memory again. */
    constexpr bool nested = NESTED; /* launched only when every job has one phase (no estimates, GBA) */
    if ((NESTED || ALIVE || COPY) && per_job_s && (maxO_sh >= 65536u || maxS_sh >= 65536u) && flags == 0) {
        /* too wide for the copy: left to the kernel with two-word entries */
        if (tid < G.n_pts)
            out.feasible[(size_t)G.pt_q[tid] * (size_t)J.n_inst + inst] = FEASIBLE_PENDING;
        return;
    }
    EntryFmt F;
    F.raw = ALIVE;
    if (nested || ALIVE) {
        F.dbits = per_job_s ? 16u : 31u;
        F.sshift = F.dbits;
        F.has_s = per_job_s;
        F.swidth = per_job_s ? 16u : 0u;
        F.all_done = nested;
    } else {
        /* durations are at most max(o), or a slice of a level some job reaches */
        uint64_t dmax = lad[maxE_sh];
        const uint64_t tau_m = lad[G.m[G.n_m - 1]];
        if (tau_m > dmax)
            dmax = tau_m;
        if (maxO_sh > dmax)
            dmax = maxO_sh;
        if (dmax > 0x7fffffffull)
            dmax = 0x7fffffffull; /* such a phase is out of range anyway */
        F.dbits = 32u - kvs_clz32((uint32_t)dmax);
        F.sshift = F.dbits + 1u;
        F.has_s = per_job_s && maxS_sh > 0; /* all-zero prompts need no field */
        F.all_done = false;
        const uint32_t sbits = F.has_s ? 32u - kvs_clz32(maxS_sh) : 0u;
        F.swidth = sbits;
        /* the prompt field is read with one shift, so it starts below bit 32 even when it is empty */
        const bool fits = F.dbits + 1u + sbits <= 32u && F.sshift <= 31u;
        if (PACKED && !fits && flags == 0) {
            if (tid < G.n_pts)
                out.feasible[(size_t)G.pt_q[tid] * (size_t)J.n_inst + inst] = FEASIBLE_PENDING;
            return;
        }
    }

    F.s_add = F.has_s ? 0u : J.s_scalar;

    /* ---- slots ---- */
    if (tid < kSlots) {
        Slot sl;
        sl.n = 0;
        sl.done = 0;
        sl.smax = J.s_scalar;
        sl.tau = 0;
        sl.off = 0;
        sl.alias = (uint32_t)tid;
        sl.bad = 0;
        sl.divtau = kvs_make_divisor(1);
        uint32_t lv = 0;
        bool used = false;
        if (tid < kLevels) {
            lv = (uint32_t)tid;
            used = (mode != MODE_SINGLE) && (lv > m_min);
            if (used) {
                const uint32_t enter = upE[lv], left = lv ? upL[lv - 1u] : 0u;
                sl.n = enter - left;
                sl.done = totL[lv];
                if (per_job_s)
                    sl.smax = NESTED ? sMaxEnter[lv] : sMaxPart[lv];
                if (one_phase_each) /* the multisplit keeps every level's jobs side by side */
                    sl.off = lv ? upE[lv - 1u] : 0u;
            }
        } else if (tid - kLevels < (int)G.n_m) {
            lv = G.m[tid - kLevels];
            used = true;
            const uint32_t enter = upE[lv], done = upL[lv], sm = upS[lv];
            const uint32_t below = lv ? upL[lv - 1u] : 0u; /* jobs that are through before level lv */
            sl.n = enter;
            sl.done = done;
            if (per_job_s)
                sl.smax = ALIVE ? maxS_sh : sm; /* ALIVE: everybody is in a first phase */
            /* Nobody is through below this level: everyone who has entered by now is still there,
             * so the merged phase holds exactly the jobs of the level's own phase, and the same of
             * them complete.  (One phase per job: nobody enters below.  Algorithm 1: no job is
             * shorter than the slice below.) */
            if (mode != MODE_SINGLE && lv > m_min && below == 0)
                sl.alias = lv;
        }
        if (used && sl.n > 0) {
            const uint64_t tau = lad[lv];
            if (tau * sl.n >= (1ull << 31)) { /* the points that use this phase are out of range */
                sl.bad = 1;
                sl.n = 0;
            } else {
                sl.tau = (uint32_t)tau;
                sl.divtau = kvs_make_divisor(sl.tau);
            }
        }
        if (!used)
            sl.n = 0;
        slot[tid] = sl;
    }
    __syncthreads();

    /* The slots that get schedules of their own (somebody takes part, and no other slot holds
     * the same phase), listed side by side: working out a schedule is a long serial piece of
     * code, and a wavefront pays for it in full however few of its lanes have one to do. */
    if (wave == 0) {
        uint32_t cu = 0;
        for (int base = 0; base < kSlots; base += 64) {
            const int si = base + lane;
            const bool u = si < kSlots && slot[si].n > 0 && slot[si].alias == (uint32_t)si;
            const uint64_t mk = __ballot(u);
            if (u)
                used[cu + lanes_below(mk)] = (uint8_t)si;
            cu += (uint32_t)__popcll(mk);
        }
        if (lane == 0)
            n_used = cu;
    }
    for (int i = tid; i < (int)G.n_v * kSlots; i += T) { /* the others: nothing to evaluate */
        const int vi = i / kSlots, si = i % kSlots;
        if (slot[si].n > 0 && slot[si].alias == (uint32_t)si)
            continue;
        Sched sc;
        sc.k = 1;
        sc.H = 0;
        sc.S = 64;
        sc.nslab = 0;
        sc.bad = 0;
        sc.narrow = 0;
        sc.div = kvs_make_divisor(1);
        sched[vi][si] = sc;
        res[vi][si].peak = 0;
        res[vi][si].sumF = 0;
    }
    __syncthreads();

    /* ---- the schedule of every (variant, slot) ---- */
    const int n_sched = (int)G.n_v * (int)n_used;
    for (int i = tid; i < n_sched; i += T) {
        const int vi = i / (int)n_used, si = used[i % (int)n_used];
        const Slot sl = slot[si];
        const bool sps = (G.v_sched[vi] == KVS_SCHED_SPS);
        Sched sc;
        sc.k = 1;
        sc.H = 0;
        sc.S = 64;
        sc.nslab = 0;
        sc.bad = 0;
        sc.narrow = 0;
        sc.div = kvs_make_divisor(1);
        if (sl.n > 0) {
            const uint64_t tau = sl.tau, smax = sl.smax, np = sl.n;
            uint64_t k;
            if (G.v_k[vi] > 0)
                k = G.v_k[vi];
            else if (sps)
                k = kvs_kstar(tau, smax, J.M);
            else
                k = kvs_udiv(J.M, smax + tau);
            if (k < 1)
                k = 1;
            const uint64_t kcap = sps ? tau * np : np; /* beyond this the offsets no longer change */
            if (k > kcap)
                k = kcap;
            const uint64_t act = (k < np) ? k : np;
            if (act * (smax + tau + 2 * WIN + 1) >= (1ull << 31)) /* window sums stay in 32 bits */
                sc.bad = 1;
            /* Every event of a round weighs at most smax + 1 + tau + (rounds of a slab) either way, and
             * at most `act` runs start and at most `act` end in one round: if that leaves a round's
             * sums within 23 and 9 signed bits, the phase is evaluated in narrow windows. */
            sc.narrow = (act < 256u && 2u * act * (smax + tau + 2 * WIN + 1) < (1ull << 22)) ? 1u : 0u;
            const uint32_t wcap = sc.narrow ? 2u * (uint32_t)WIN : (uint32_t)WIN;
            sc.k = (uint32_t)k;
            sc.div = kvs_make_divisor(sc.k);
            sc.H = start_offset(sl.n - 1, sl.tau, sc, sps) + sl.tau;
            /* slab length: about two wavefronts' share of the rounds, 64 to WIN rounds each (longer
             * slabs repeat less work at their edges, and that outweighs the balance);
             * SimS batches do not overlap, so whole batches per slab need no carry-in */
            uint32_t S = ((2 * sc.H + NW - 1) / NW + 63u) & ~63u;
            if (sps) { /* ... but long enough for about 1024 runs to start inside one: the work at
                          a slab's edges (window, carry-in, scan) is then small beside its runs */
                uint64_t need = kvs_udiv(1024u * tau, k);
                need = need > wcap ? wcap : need;
                S = S < (uint32_t)need ? (((uint32_t)need + 63u) & ~63u) : S;
            }
            S = S > wcap ? wcap : S;
            if (!sps && sl.tau <= wcap) {
                uint32_t b = S / sl.tau;
                S = sl.tau * (b ? b : 1u);
            }
            sc.S = S;
            sc.nslab = (sc.H + S - 1) / S;
            /* Long and thin: evaluating every run against the at most k + 1 runs around it is
             * cheaper than walking the rounds once a run's share of them, tau / k, is above a few
             * times k (a slab of S rounds costs about as much as 20 runs' neighbours). */
            if (sc.k * (uint64_t)sc.k < 4u * tau && sl.n > 64u) {
                sc.S = 0;
                sc.nslab = (sl.n + 63u) / 64u;
            }
            if (sl.n <= 64u)
                sc.nslab = 1; /* one wavefront, one run per lane */
            if (sc.bad)
                sc.nslab = 0; /* out of range: not evaluated, and its points say so */
        }
        sched[vi][si] = sc;
        res[vi][si].peak = 0;
        /* Sum of the start offsets of the completing runs.  When every run completes it is a
         * closed form of (n, tau, k) and nothing has to be summed over the runs. */
        unsigned long long sumF0 = 0;
        if (F.all_done && sl.n > 0 && (uint64_t)sl.n * sl.tau < (1ull << 31)) { /* else out of range: 1 <= k <= n tau needs it */
            if (sps) {
                sumF0 = kvs_floor_sum(sl.n, sc.k, sl.tau);
            } else {
                const uint64_t q = kvs_div(sl.n, sc.div), rem = sl.n - q * sc.k; /* q whole batches, then rem jobs */
                sumF0 = (uint64_t)sl.tau * ((uint64_t)sc.k * (q * (q - 1u) / 2u) + q * rem);
            }
        }
        res[vi][si].sumF = sumF0;
    }
    __syncthreads();

    const bool bad = (flags != 0);
    uint32_t next_item = 0; /* slabs are dealt to the wavefronts in turn */

    auto eval_slot = [&](int si) {
        const uint32_t n_runs = slot[si].n;
        if (n_runs == 0 || slot[si].alias != (uint32_t)si)
            return;
        for (int vi = 0; vi < (int)G.n_v; vi++) {
            /* work items of this (slot, variant): one for a phase of at most 64 runs, else its
             * slabs (or groups of runs).  This wavefront takes every NW-th, starting where the
             * dealing has got to, and reads the tables only if something falls to it. */
            const uint32_t items = sched[vi][si].nslab;
            const uint32_t first = ((uint32_t)wave + NW - next_item % NW) % NW;
            next_item += items;
            if (first >= items)
                continue;
            const Slot sl = slot[si];
            const Sched sc = sched[vi][si];
            const bool sps = (G.v_sched[vi] == KVS_SCHED_SPS);
            int32_t pk = 0;
            unsigned long long sumF = 0;
            if (n_runs <= 64u) {
                eval_sparse<PACKED>(sl, sc, sps, buf, n, J.s_scalar, F, lane, pk, sumF);
            } else {
                for (uint32_t j = first; j < items; j += NW) {
                    if (sc.S == 0)
                        eval_thin<PACKED>(sl, sc, sps, j, buf, n, J.s_scalar, F, lane, pk, sumF);
                    else if (sc.narrow)
                        eval_slab<PACKED, WIN, true>(sl, sc, sps, j, buf, n, J.s_scalar, F, ev[wave], lane, pk, sumF);
                    else
                        eval_slab<PACKED, WIN, false>(sl, sc, sps, j, buf, n, J.s_scalar, F, ev[wave], lane, pk, sumF);
                }
            }
            pk = wave_max_nonneg(pk);
            if (lane == 0)
                atomicMax(&res[vi][si].peak, pk);
            if (!F.all_done) { /* else the table holds the closed form */
                sumF = wave_sum_u63(sumF);
                if (lane == 0)
                    atomicAdd(&res[vi][si].sumF, sumF);
            }
        }
    };

    /* stable compaction of the jobs with ga <= lv (<= gb when `level`) into buf[0 ..) */
    auto compact = [&](uint32_t lv, bool level, uint32_t tau) {
        uint32_t pos0 = 0;
        for (int w = 0; w < wave; w++) {
            uint32_t c = cumE[w][lv];
            if (level && lv > 0)
                c -= cumL[w][lv - 1];
            pos0 += c;
        }
        /* Pass 1 has vouched for the instance's values, so membership is two comparisons with
         * slices: entry level <= lv  <=>  believed length <= tau_lv, and so on. */
        const bool want_e = with_estimates;
        const uint32_t tau_lv = lad[lv];
        const uint32_t tau_below = lv ? lad[lv - 1] : 0u;
        RawJob nxt;
        nxt.o = nxt.s = nxt.e = 1;
        if (seg_lo + lane < seg_hi)
            nxt = load_job(J, row + seg_lo + lane, want_e);
        for (uint32_t base = seg_lo; base < seg_hi; base += 64) {
            const uint32_t i = base + lane;
            bool take = false;
            const RawJob raw = nxt;
            if (i + 64 < seg_hi)
                nxt = load_job(J, row + i + 64, want_e);
            const uint32_t o = (uint32_t)raw.o, s = (uint32_t)raw.s;
            if (i < seg_hi) {
                uint32_t bel = 1u; /* what the scheduler believes: GSA and lone invocations take everybody */
                if (mode == MODE_GBA) {
                    bel = o;
                    if (want_e) {
                        uint64_t cap = J.M - s;
                        if (cap > kLenMax)
                            cap = kLenMax;
                        bel = (uint32_t)raw.e > (uint32_t)cap ? (uint32_t)cap : (uint32_t)raw.e;
                    }
                }
                take = bel <= tau_lv;
                if (level && lv > 0)
                    take = take && ((bel > o ? bel : o) > tau_below);
            }
            const uint64_t bal = __ballot(take);
            if (take) {
                const bool done = o <= tau_lv;
                put_entry<PACKED>(buf, n, pos0 + lanes_below(bal), done ? o : tau, done, s, F);
            }
            pos0 += (uint32_t)__popcll(bal);
        }
    };

    /*
     * GATHERS: the entries of the slots order[b0 .. b1) gathered from the copy of the instance
     * in LDS (or from memory), every slot's participants in input order at its own place in the
     * phase buffer.  A job takes part in the level slots from the level at which it enters to
     * the one at which it completes, and in the merged first phase of every shift at or above
     * its entry level.  Each wavefront walks its own segment of the jobs (the one it counted in
     * pass 1, so the per-wavefront counts tell where its entries of a slot begin); lane j keeps
     * what the wavefront needs to know about the j-th slot of the batch.  For every 64 jobs the
     * levels that any of them takes part in are or-ed into one mask, and only the batch's slots
     * at those levels are gone through.
     */
    auto gather = [&](uint32_t b0, uint32_t b1) {
        const uint32_t g_cnt = b1 - b0; /* at most 64 */
        uint32_t my_info = 0, my_tau = 0, my_cur = 0; /* info: the slot's level, bit 8: it is a level's own phase */
        if ((uint32_t)lane < g_cnt) {
            const uint32_t si = order[b0 + (uint32_t)lane];
            const uint32_t my_level = si < (uint32_t)kLevels ? 1u : 0u;
            const uint32_t my_lv = my_level ? si : (uint32_t)G.m[si - kLevels];
            my_info = my_lv | (my_level << 8);
            my_tau = lad[my_lv];
            my_cur = slot[si].off;
            for (int w = 0; w < wave; w++) {
                uint32_t c = cumE[w][my_lv];
                if (my_level && my_lv > 0)
                    c -= cumL[w][my_lv - 1u];
                my_cur += c;
            }
        }
        /* from memory: the loads of kAhead chunks of 64 jobs are issued together, a wavefront has
         * little else in flight here */
        constexpr uint32_t kAhead = COPY ? 1u : 4u;
        for (uint32_t base0 = seg_lo; base0 < seg_hi; base0 += 64u * kAhead) {
          RawJob ahead[kAhead];
          if (!COPY) {
#pragma unroll
              for (uint32_t u = 0; u < kAhead; u++) {
                  const uint32_t i = base0 + 64u * u + (uint32_t)lane;
                  ahead[u].o = ahead[u].s = ahead[u].e = 1;
                  if (i < seg_hi)
                      ahead[u] = load_job(J, row + i, true);
              }
          }
#pragma unroll
          for (uint32_t u = 0; u < kAhead; u++) {
            const uint32_t base = base0 + 64u * u;
            if (base >= seg_hi)
                break; /* the same for all lanes */
            const uint32_t i = base + (uint32_t)lane;
            const bool act = i < seg_hi;
            uint32_t o, s, ga;
            if (COPY) {
                const uint32_t w = act ? jobs_lds[i] : 0u;
                o = per_job_s ? (w & 0xffffu) : w;
                s = per_job_s ? (w >> 16) : J.s_scalar;
                ga = act ? (uint32_t)ga_lds[i] : 0u;
            } else {
                const JobView v = view_job<EXPLICIT>(ahead[u], J, G, lad, mode, true);
                o = v.o;
                s = v.s;
                ga = v.ga;
            }
            /* lowest entry level among these jobs (a merged phase below it gets none of them) and
             * the levels at which some of them is still unfinished: a job that enters at ga and
             * has the length o is there at the levels ga .. max(ga, level of o) */
            uint64_t here; /* bit l: some job takes part at level l; its lowest bit: the lowest entry level */
            bool ok = true; /* checked in pass 1 */
            const uint32_t go = act ? level_of<EXPLICIT>(o, G, lad, ok) : 0u; /* completes at this level ... */
            const uint32_t gb = go > ga ? go : ga;                            /* ... but not before it enters */
            {
                const uint64_t mine =
                    act ? (((gb >= 63u) ? ~0ull : ((2ull << gb) - 1ull)) & ~((1ull << ga) - 1ull)) : 0ull;
                here = (uint64_t)wave_or((uint32_t)mine);
                if (kLevels > 32)
                    here |= (uint64_t)wave_or((uint32_t)(mine >> 32)) << 32;
            }
            const uint32_t ga_min = here ? (uint32_t)__builtin_ctzll(here) : 0xffffffffu;
            const uint32_t ga_act = act ? ga : 0xffffffffu;          /* a lane without a job enters nowhere */
            const uint32_t s_part = F.has_s ? (s << F.sshift) : 0u; /* the entry's prompt field */
            for (uint32_t j = 0; j < g_cnt; j++) {
                const uint32_t info = __builtin_amdgcn_readlane(my_info, (int)j);
                const uint32_t lv = info & 0xffu;
                const bool level = (info >> 8) != 0;
                if (level ? !((here >> lv) & 1ull) : (ga_min > lv))
                    continue; /* none of these jobs is in that phase */
                /* entered by now; and, for a level's own phase, not through before it */
                const uint32_t stays = level ? gb : 0xffffffffu;
                const bool take = ga_act <= lv && stays >= lv;
                const uint64_t bal = __ballot(take);
                if (bal == 0)
                    continue;
                const uint32_t tau_lv = __builtin_amdgcn_readlane(my_tau, (int)j);
                const uint32_t at = __builtin_amdgcn_readlane(my_cur, (int)j);
                if (take) { /* the entry: duration | done | prompt (one word here) */
                    const bool done = go <= lv;
                    buf[at + lanes_below(bal)] = (done ? (o | (1u << F.dbits)) : tau_lv) | s_part;
                }
                if ((uint32_t)lane == j)
                    my_cur = at + (uint32_t)__popcll(bal);
            }
          }
        }
    };

    /* Chunks of 64 entries a wavefront holds in registers while LDS is rearranged under it. */
    constexpr int kHold = HOLD; /* the launch guarantees n_jobs <= HOLD * T */
    const uint32_t dmask = (F.dbits >= 32u) ? 0xffffffffu : ((1u << F.dbits) - 1u);

    /* Stable partition, wavefront by wavefront: this wavefront's entries buf[in_lo .. in_lo + in_len)
     * with duration <= theta go to buf[front ..) in their order, the others to buf[back ..) in
     * theirs (long_first: the other way round; !write_back: the others are dropped).  The caller
     * knows the places from the per-wavefront counts of pass 1.  The entries are held in
     * registers across the barrier that separates everybody's reads from everybody's writes. */
    auto split_owned = [&](uint32_t in_lo, uint32_t in_len, uint32_t theta, bool long_first, uint32_t front,
                           uint32_t back, bool write_back) {
        const uint32_t hi = in_lo + in_len;
        uint32_t held[kHold];
        /* all the reads first, none of them under a branch, so that they are in flight together
         * (an index past the stretch reads the stretch's last word, which is then ignored) */
        const uint32_t last = hi ? hi - 1u : 0u;
#pragma unroll
        for (int c = 0; c < kHold; c++) {
            const uint32_t idx = in_lo + (uint32_t)c * 64u + (uint32_t)lane;
            held[c] = buf[idx < last ? idx : last];
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < kHold; c++) {
            const uint32_t at = in_lo + (uint32_t)c * 64u;
            if (at >= hi)
                break; /* the rest of the stretch is empty (the same for all lanes) */
            /* the entries of a chunk sit in its first lanes, so a lane's rank among them is its
             * number, and its rank among the moved ones is that minus its rank among the kept */
            const bool act = at + (uint32_t)lane < hi;
            const bool keep = act && ((held[c] & dmask) <= theta) != long_first;
            const uint64_t bk = __builtin_amdgcn_ballot_w64(keep);
            const uint32_t rk = lanes_below(bk);
            if (keep)
                buf[front + rk] = held[c];
            else if (act && write_back)
                buf[back + ((uint32_t)lane - rk)] = held[c];
            const uint32_t nk = (uint32_t)__popcll(bk);
            const uint32_t na = hi - at < 64u ? hi - at : 64u;
            front += nk;
            back += na - nk;
        }
        __syncthreads();
    };

    /* Stable multisplit by level of this wavefront's entries buf[in_lo .. in_lo + in_len) (levels
     * above every merged phase, in input order) to where the level slots expect them: a level's
     * slot takes the wavefronts' shares one after the other.  pre: the sums over the wavefronts
     * before this one that the totals stage has put beside the counts. */
    auto split_tail_owned = [&](uint32_t in_lo, uint32_t in_len, const uint32_t *pre) {
        const uint32_t hi = in_lo + in_len;
        uint32_t held[kHold];
        const uint32_t last = hi ? hi - 1u : 0u;
#pragma unroll
        for (int c = 0; c < kHold; c++) {
            const uint32_t idx = in_lo + (uint32_t)c * 64u + (uint32_t)lane;
            held[c] = buf[idx < last ? idx : last];
        }
        uint32_t cur = 0; /* lane l: next free position of level l for this wavefront */
        if (lane > 0 && lane < kLevels)
            cur = slot[lane].off + (pre[lane] - pre[lane - 1]);
        __syncthreads();
#pragma unroll
        for (int c = 0; c < kHold; c++) {
            if (in_lo + (uint32_t)c * 64u >= hi)
                break; /* the rest of the stretch is empty (the same for all lanes) */
            const uint32_t idx = in_lo + (uint32_t)c * 64u + (uint32_t)lane;
            const bool act = idx < hi;
            bool ok = true; /* checked in pass 1 */
            const uint32_t lv = act ? level_of<EXPLICIT>(held[c] & dmask, G, lad, ok) : 0u;
            uint32_t pos = 0;
            uint64_t todo = __ballot(act);
            while (todo) {
                const int src = __ffsll((unsigned long long)todo) - 1;
                const uint32_t c0 = __builtin_amdgcn_readlane(lv, src);
                const uint64_t mk = __ballot(act && lv == c0);
                const uint32_t b = __builtin_amdgcn_readlane(cur, (int)c0);
                if (act && lv == c0)
                    pos = b + lanes_below(mk);
                if ((uint32_t)lane == c0)
                    cur += (uint32_t)__popcll(mk);
                todo &= ~mk;
            }
            if (act)
                buf[pos] = held[c];
        }
        __syncthreads();
    };

    if (ALIVE) {
        if (!bad) {
            /* ---- the list of unfinished jobs, in input order, is the phase ---- */
            /* first phases: everybody, whatever the shift (none of them moves the list) */
            for (int mi = 0; mi < (int)G.n_m; mi++)
                eval_slot(kLevels + mi);
            uint32_t cnt = n;   /* jobs in the list */
            uint32_t alive = n; /* of which are unfinished when the next level begins */
            for (uint32_t l = 0; l <= m_min; l++)
                alive -= totL[l];
            /* of this wavefront's segment, and of the segments before it, what has left the list
             * so far (cumL, and its sums over the wavefronts before in cumE's place) */
            uint32_t gone_own = 0, gone_before = 0;
            for (int si = (int)m_min + 1; si < kLevels && mode != MODE_SINGLE; si++) {
                const uint32_t left = alive; /* the jobs longer than the slice below */
                if (left == 0)
                    break;
                alive -= totL[si];
                if (left < cnt) {
                    /* no barrier here: the partition first only reads the list, as the phases
                     * evaluated so far do, and has a barrier of its own before it writes */
                    const uint32_t out_own = cumL[wave][si - 1], out_before = cumE[wave][si - 1];
                    split_owned(seg_lo - gone_before, (seg_hi - seg_lo) - gone_own, lad[si - 1], true,
                                seg_lo - out_before, 0u, false);
                    gone_own = out_own;
                    gone_before = out_before;
                    cnt = left;
                }
                eval_slot(si);
            }
            __syncthreads();
        }
    } else if (GATHERS) {
      if (!bad) {
        /* ---- batches of slots: as many as the phase buffer holds, gathered, then evaluated ---- */
        /* The slots in the order they are evaluated: the levels above the smallest shift, then
         * the merged first phases.  They are packed into batches one after the other (a batch is
         * closed when the next slot would overflow the phase buffer or the 64 lanes that keep
         * track of its slots).  The first wavefront fetches all the sizes at once and then goes
         * through them in scalar registers: one thread walking the table in LDS would make
         * every other wavefront wait for some hundred dependent reads. */
        if (wave == 0) {
            const uint32_t nlev = (uint32_t)kLevels - 1u - m_min;
            const uint32_t ncand = nlev + (uint32_t)G.n_m; /* at most kSlots <= 128 */
            static_assert(kSlots <= 128, "two candidates per lane");
            auto slot_of = [&](uint32_t k) { return k < nlev ? m_min + 1u + k : (uint32_t)kLevels + (k - nlev); };
            uint32_t size[2] = {0u, 0u};
#pragma unroll
            for (uint32_t h = 0; h < 2u; h++) {
                const uint32_t k = 64u * h + (uint32_t)lane;
                if (k < ncand) {
                    const uint32_t si = slot_of(k);
                    size[h] = (slot[si].alias == si) ? slot[si].n : 0u;
                }
            }
            uint32_t nb = 0, cnt = 0, first = 0, fill = 0;
            for (uint32_t k = 0; k < ncand; k++) {
                const uint32_t ns = (k < 64u) ? __builtin_amdgcn_readlane(size[0], (int)k)
                                              : __builtin_amdgcn_readlane(size[1], (int)(k - 64u));
                if (ns == 0)
                    continue;
                if (fill + ns > n || cnt - first >= 64u) {
                    nb++;
                    if (lane == 0)
                        bstart[nb] = (uint8_t)cnt;
                    first = cnt;
                    fill = 0;
                }
                if (lane == 0) {
                    slot[slot_of(k)].off = fill;
                    order[cnt] = (uint8_t)slot_of(k);
                }
                fill += ns;
                cnt++;
            }
            if (lane == 0) {
                bstart[0] = 0;
                if (cnt > 0)
                    bstart[++nb] = (uint8_t)cnt;
                n_batches = nb;
            }
        }
        __syncthreads();
        const uint32_t nb = n_batches;
        for (uint32_t b = 0; b < nb; b++) {
            const uint32_t b0 = bstart[b], b1 = bstart[b + 1];
            gather(b0, b1);
            __syncthreads();
            for (uint32_t j = b0; j < b1; j++)
                eval_slot((int)order[j]);
            __syncthreads();
        }
      }
    } else if (!bad) {
        if (nested) {
/* ---- every phase is cut out of the LDS copy of the instance ---- */
            const uint32_t m_max = G.m[G.n_m - 1];
            /* Of this wavefront's segment of the input, cumE[wave][g] jobs are of the levels up to g,
             * and cumL[wave][g] holds the same count summed over the wavefronts before it: that is
             * where its share of the merged phase of level g begins, and how long it is. */
            const uint32_t cnt0 = upE[m_max]; /* jobs of the levels up to m_max: the largest merged phase */
            if (cnt0 < n) {
                const uint32_t own = cumE[wave][m_max], before = cumL[wave][m_max];
                const uint32_t tail_lo = cnt0 + (seg_lo - before);
                if (cnt0 > 0)
                    split_owned(seg_lo, seg_hi - seg_lo, lad[m_max], false, before, tail_lo, true);
                split_tail_owned(tail_lo, (seg_hi - seg_lo) - own, cumL[wave]);
            }
            int mi = (int)G.n_m - 1;
            for (uint32_t g = m_max;; g--) {
                /* buf[0 .. cnt) holds the jobs of the levels 0 .. g in input order */
                if (mi >= 0 && G.m[mi] == g) {
                    const int si = kLevels + mi;
                    /* no barrier after it: whatever follows only reads the buffer until the
                     * barrier inside the next partition, which every wavefront reaches after its
                     * share of this phase */
                    if (slot[si].n > 0 && slot[si].alias == (uint32_t)si)
                        eval_slot(si);
                    mi--;
                }
                if (g == m_min)
                    break;
                const uint32_t below = upE[g - 1u];
                if (totE[g] > 0 && below > 0) /* level g's jobs move behind the lower levels', into the level's own slot */
                    split_owned(cumL[wave][g], cumE[wave][g], lad[g - 1u], false, cumL[wave][g - 1u],
                                below + (cumL[wave][g] - cumL[wave][g - 1u]), true);
            }
            for (int si = (int)m_min + 1; si < kLevels; si++)
                eval_slot(si);
            __syncthreads();
        } else if (one_phase_each && mode != MODE_SINGLE) {
            /* ---- stable multisplit by level: every level's jobs side by side, input order ---- */
            uint32_t cur = 0; /* lane l: next free position of level l for this wavefront */
            if (lane < kLevels) {
                for (uint32_t l = 0; l < (uint32_t)lane; l++)
                    cur += totE[l];
                for (int w = 0; w < wave; w++)
                    cur += cumE[w][lane] - (lane ? cumE[w][lane - 1] : 0u);
            }
            RawJob nxt;
            nxt.o = nxt.s = nxt.e = 1;
            if (seg_lo + lane < seg_hi)
                nxt = load_job(J, row + seg_lo + lane, false);
            for (uint32_t base = seg_lo; base < seg_hi; base += 64) {
                const uint32_t i = base + lane;
                const bool act = i < seg_hi;
                struct {
                    uint32_t ga, o, s;
                } v;
                v.ga = 0;
                const RawJob raw = nxt;
                if (i + 64 < seg_hi)
                    nxt = load_job(J, row + i + 64, false);
                v.o = (uint32_t)raw.o; /* valid: pass 1 has checked the instance */
                v.s = (uint32_t)raw.s;
                if (act) {
                    bool ok = true; /* checked in pass 1 */
                    v.ga = level_of<EXPLICIT>(v.o, G, lad, ok);
                }
                uint32_t pos = 0;
                uint64_t todo = __ballot(act);
                while (todo) {
                    const int src = __ffsll((unsigned long long)todo) - 1;
                    const uint32_t c0 = __builtin_amdgcn_readlane(v.ga, src);
                    const uint64_t mk = __ballot(act && v.ga == c0);
                    const uint32_t b0 = __builtin_amdgcn_readlane(cur, (int)c0);
                    if (act && v.ga == c0)
                        pos = b0 + lanes_below(mk);
                    if ((uint32_t)lane == c0)
                        cur += (uint32_t)__popcll(mk);
                    todo &= ~mk;
                }
                if (act && v.ga > m_min)
                    put_entry<PACKED>(buf, n, pos, v.o, true, v.s, F);
            }
            __syncthreads();
            for (int si = (int)m_min + 1; si < kLevels; si++)
                eval_slot(si);
            __syncthreads();
        } else if (mode != MODE_SINGLE) {
            for (int si = (int)m_min + 1; si < kLevels; si++) {
                if (slot[si].n == 0)
                    continue;
                compact((uint32_t)si, true, slot[si].tau);
                __syncthreads();
                eval_slot(si);
                __syncthreads();
            }
        }
        /* ---- merged first phases, one per shift (the LDS-only path has done them) ---- */
        for (int mi = 0; mi < (int)G.n_m && !nested; mi++) {
            const int si = kLevels + mi;
            if (slot[si].n == 0 || slot[si].alias != (uint32_t)si)
                continue;
            compact(G.m[mi], false, slot[si].tau);
            __syncthreads();
            eval_slot(si);
            __syncthreads();
        }
    }

    /* ---- put the phases of every point together ----
     * kLevels consecutive lanes per point: lane 0 takes the merged first phase, lane j the level
     * m + j.  A phase begins when the ones before it have ended (prefix sum of the phase lengths
     * over the lanes); flow = sum o + sum_p (done_p begin_p + start offsets of the completing
     * runs), job steps = sum o + sum_p tau_p (n_p - done_p), peak = max_p. */
    for (int item0 = 0; item0 < (int)G.n_pts * kLevels; item0 += T) {
        const int item = item0 + tid;
        const int q = item / kLevels, j = item % kLevels;
        const bool have = q < (int)G.n_pts;
        const int vi = have ? G.pt_v[q] : 0;
        const int mi = have ? G.pt_m[q] : 0;
        const int g = (int)G.m[mi] + j;
        const bool in_ladder = have && !bad && (j == 0 || (mode != MODE_SINGLE && g < kLevels));
        unsigned long long H = 0, sumF = 0;
        uint32_t n_p = 0, done_p = 0, tau_p = 0, err = 0;
        int32_t pk = 0;
        if (in_ladder) {
            const Slot sl = slot[j == 0 ? kLevels + mi : g];
            err = sl.bad | sched[vi][sl.alias].bad; /* a phase of this point left the 32-bit range */
            if (sl.n > 0) {
                const Result r = res[vi][sl.alias];
                n_p = sl.n;
                done_p = sl.done;
                tau_p = sl.tau;
                sumF = r.sumF;
                pk = r.peak;
                H = sched[vi][sl.alias].H;
            }
        }
        unsigned long long begin = H; /* inclusive prefix over the point's lanes, then exclusive */
#pragma unroll
        for (int d = 1; d < kLevels; d <<= 1) {
            const unsigned long long up = __shfl_up(begin, d, kLevels);
            if (j >= d)
                begin += up;
        }
        begin -= H;
        unsigned long long flow = (unsigned long long)done_p * begin + sumF;
        unsigned long long steps = (unsigned long long)tau_p * (unsigned long long)(n_p - done_p); /* killed runs use their whole slice */
        uint32_t done = done_p;
#pragma unroll
        for (int d = kLevels / 2; d >= 1; d >>= 1) {
            flow += __shfl_xor(flow, d, kLevels);
            steps += __shfl_xor(steps, d, kLevels);
            done += __shfl_xor(done, d, kLevels);
            err |= __shfl_xor(err, d, kLevels);
            const int32_t other = __shfl_xor(pk, d, kLevels);
            pk = other > pk ? other : pk;
        }
        if (have && j == 0) {
            int64_t peak = pk, fl = (int64_t)(flow + sumO_sh), st = (int64_t)(steps + sumO_sh);
            int64_t dn = done;
            uint8_t feas = (peak <= (int64_t)J.M) ? 1 : 0;
            if (flags & FLAG_EINVAL)
                feas = KVS_FEASIBLE_EINVAL;
            else if (flags & FLAG_ERANGE)
                feas = KVS_FEASIBLE_ERANGE;
            else if (flags & FLAG_EJOB)
                feas = KVS_FEASIBLE_EJOB;
            else if (err)
                feas = KVS_FEASIBLE_ERANGE;
            if (bad || err)
                peak = fl = st = dn = -1;
            const size_t oi = (size_t)G.pt_q[q] * (size_t)J.n_inst + inst;
            out.peak[oi] = peak;
            out.feasible[oi] = feas;
            out.flow[oi] = fl;
            if (out.job_steps)
                out.job_steps[oi] = st;
            if (out.n_completed)
                out.n_completed[oi] = (int32_t)dn;
        }
    }
}

/* Workgroups of the kernel with two-word entries: each looks after the instances
 * blockIdx.x, blockIdx.x + kWideGrid, ... and works on those the one-word kernel left behind. */
constexpr uint32_t kWideGrid = 1024;

/* 768 threads: two workgroups per compute unit need 6 wavefronts per SIMD, i.e. at most 80 VGPRs. */
template <int T, int KIND, int WIN, int LV, int HOLD>
__global__ __launch_bounds__(T, (T == 768 ? 6 : 1)) void kvs_sweep_kernel(JobsDev J, GroupArg G, OutsDev out)
{
    if (KIND != KIND_WIDE) { /* one workgroup per instance */
        sweep_instance<T, KIND, WIN, LV, HOLD>(J, G, out, blockIdx.x);
        return;
    }
    /* Two-word entries: only the instances that the one-word kernel marked in `feasible`, usually
     * none.  64 of the workgroup's instances at a time: every wavefront reads the same 64 marks
     * (lane l the mark of the l-th of them) and so arrives at the same list, then all work
     * through it together.  A mark is overwritten only by this workgroup, at the end of that
     * instance's evaluation, which no wavefront reaches before all have read the marks (the
     * evaluation takes workgroup barriers on the way). */
    const uint32_t n_inst = (uint32_t)J.n_inst;
    const int lane = threadIdx.x & 63;
    for (uint32_t first = blockIdx.x; first < n_inst; first += 64u * gridDim.x) {
        const uint64_t cand = (uint64_t)first + (uint64_t)lane * gridDim.x;
        const bool pending = cand < n_inst &&
                             (J.wide_all ||
                              out.feasible[(size_t)G.pt_q[0] * (size_t)n_inst + (size_t)cand] == FEASIBLE_PENDING);
        uint64_t todo = __ballot(pending);
        while (todo) {
            const uint32_t j = (uint32_t)__ffsll((unsigned long long)todo) - 1u;
            todo &= todo - 1u;
            sweep_instance<T, KIND, WIN, LV, HOLD>(J, G, out, first + j * gridDim.x);
            __syncthreads(); /* the tables in LDS are set up afresh for the next instance */
        }
    }
}

/* ---- input scan for kvs_validate ---- */
struct ValidateResult {
    uint32_t bad_value;  /* o < 1, s < 0 or o_est < 1 */
    uint32_t too_long;   /* a length above 2^30       */
    uint32_t infeasible; /* s + o > M                 */
};

__global__ __launch_bounds__(256) void kvs_validate_kernel(JobsDev J, ValidateResult *res)
{
    const size_t total = (size_t)J.n_inst * (size_t)J.n_jobs;
    uint32_t bad = 0, lng = 0, inf = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int64_t o = J.o[i];
        const int64_t s = J.s ? (int64_t)J.s[i] : (int64_t)J.s_scalar;
        const int64_t e = J.e ? (int64_t)J.e[i] : 1;
        if (o < 1 || s < 0 || e < 1)
            bad = 1;
        else {
            if (o > (int64_t)kLenMax || s > (int64_t)kLenMax || e > (int64_t)kLenMax)
                lng = 1;
            if ((uint64_t)(s + o) > J.M)
                inf = 1;
        }
    }
    if (__any(bad) && (threadIdx.x & 63) == 0)
        atomicOr(&res->bad_value, 1u);
    if (__any(lng) && (threadIdx.x & 63) == 0)
        atomicOr(&res->too_long, 1u);
    if (__any(inf) && (threadIdx.x & 63) == 0)
        atomicOr(&res->infeasible, 1u);
}

/*
 * Device memory for the entry point that allocates nothing: room for one ValidateResult.
 * Every GPU the library runs on holds its own copy until the process ends.  In host code the
 * name below is only a handle for hipGetSymbolAddress; kernels are handed the address that
 * call returns.
 */
constexpr size_t kScratchBytes = 256;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static_assert(sizeof(ValidateResult) <= kScratchBytes, "the scan's result fits the static scratch");

__global__ void kvs_clear_result_kernel(ValidateResult *res)
{
    if (threadIdx.x == 0) {
        res->bad_value = 0;
        res->too_long = 0;
        res->infeasible = 0;
    }
}

/* ---- host side ---- */

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_addr[kMaxDevices]; /* per device: where its copy of `scratch` lives, once asked */

/* Address of the current device's copy of the static scratch, looked up once per device. */
int32_t static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return KVS_EHIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_addr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return KVS_EHIP;
        scratch_addr[dev] = p;
    }
    *ptr = scratch_addr[dev];
    return KVS_OK;
}

int32_t check_jobs(const kvs_jobs_t *jobs)
{
    if (!jobs)
        return KVS_EINVAL;
    if (jobs->n_instances < 0 || jobs->n_jobs < 1)
        return KVS_EINVAL;
    if (jobs->n_instances > 0 && !jobs->o)
        return KVS_EINVAL;
    if (jobs->M < 1 || jobs->M >= (1ll << 40))
        return KVS_EINVAL;
    if (!jobs->s && (jobs->s_scalar < 0 || (uint32_t)jobs->s_scalar > kLenMax))
        return KVS_EINVAL;
    if (jobs->n_jobs > KVS_MAX_JOBS)
        return KVS_ELIMIT;
    return KVS_OK;
}

JobsDev to_dev(const kvs_jobs_t *jobs, bool use_estimates)
{
    JobsDev J;
    J.o = jobs->o;
    J.s = jobs->s;
    J.e = use_estimates ? jobs->o_est : nullptr;
    J.n_inst = jobs->n_instances;
    J.n_jobs = jobs->n_jobs;
    J.s_scalar = jobs->s ? 0u : (uint32_t)jobs->s_scalar;
    J.M = (uint64_t)jobs->M;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(J.o) | reinterpret_cast<uintptr_t>(J.s) |
                           reinterpret_cast<uintptr_t>(J.e);
    J.vec4 = (jobs->n_jobs % 4 == 0 && bits % 16 == 0) ? 1u : 0u;
    J.wide_all = 0;
    return J;
}

constexpr int32_t kNoRoom = -1;          /* internal: the instantiation's LDS need exceeds the compute unit's */
constexpr size_t kLdsPerGroup = 160 * 1024; /* LDS a workgroup can have on gfx950 */

template <int T, int KIND, int WIN, int LV, int HOLD>
int32_t launch_sweep(const JobsDev &J, const GroupArg &G, const OutsDev &out, hipStream_t st)
{
    /* phase entries; GATHER: also the instance itself, one word and one byte per job */
    const size_t n = (size_t)J.n_jobs;
    size_t lds = sizeof(uint32_t) * n * (KIND == KIND_WIDE ? 2 : 1);
    if (KIND == KIND_GATHER)
        lds += sizeof(uint32_t) * n + ((n + 3) & ~(size_t)3);
    static_assert((KIND != KIND_NESTED && KIND != KIND_ALIVE) || HOLD * T >= (T == 256 ? 4096 : 1), "hold");
    auto kern = kvs_sweep_kernel<T, KIND, WIN, LV, HOLD>;
    static std::atomic<int> static_lds{-1}; /* of this instantiation; the same on every device */
    int fixed = static_lds.load(std::memory_order_relaxed);
    if (fixed < 0) {
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(kern)) != hipSuccess)
            return KVS_EHIP;
        fixed = (int)attr.sharedSizeBytes;
        static_lds.store(fixed, std::memory_order_relaxed);
    }
    if (lds + (size_t)fixed > kLdsPerGroup)
        return kNoRoom;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return KVS_EHIP;
    const uint32_t grid = KIND != KIND_WIDE ? (uint32_t)J.n_inst
                                 : ((uint32_t)J.n_inst < kWideGrid ? (uint32_t)J.n_inst : kWideGrid);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(T), lds, st, J, G, out);
    return hipGetLastError() == hipSuccess ? KVS_OK : KVS_EHIP;
}

/*
 * First launch: one-word entries, the instantiation that fits the mode (see the list of
 * kinds above).  Second launch, only with per-job prompts: the instances the first one marked
 * as too wide, with two-word entries, every phase compacted from memory; it also takes every
 * instance should the first launch's LDS need ever exceed a compute unit's.
 */
template <int LV>
int32_t run_group_lv(const JobsDev &J, const GroupArg &G, const OutsDev &out, hipStream_t st)
{
    int32_t rc;
    const bool big = J.n_jobs > 4096;
    /* registers a thread needs to hold its share of an instance: n_jobs / threads, rounded up */
    constexpr int kHoldMid = 14, kHoldMax = (KVS_MAX_JOBS + 767) / 768;
    const bool mid = J.n_jobs <= kHoldMid * 768;
    /* Large instances: 12 wavefronts and 256-round windows keep two workgroups (24 wavefronts)
     * on a compute unit next to a 40 KB phase buffer; measured best among the shapes tried. */
    if (G.mode == MODE_GBA && J.e == nullptr) /* one phase per job */
        rc = !big ? launch_sweep<256, KIND_NESTED, 256, LV, 16>(J, G, out, st)
             : mid ? launch_sweep<768, KIND_NESTED, 256, LV, kHoldMid>(J, G, out, st)
                   : launch_sweep<768, KIND_NESTED, 256, LV, kHoldMax>(J, G, out, st);
    else if (G.mode != MODE_GBA) /* everybody in every phase until done */
        rc = !big ? launch_sweep<256, KIND_ALIVE, 256, LV, 16>(J, G, out, st)
             : mid ? launch_sweep<768, KIND_ALIVE, 256, LV, kHoldMid>(J, G, out, st)
                   : launch_sweep<768, KIND_ALIVE, 256, LV, kHoldMax>(J, G, out, st);
    else /* classes by estimates: two copies in LDS while several workgroups still share a compute unit */
        rc = !big ? launch_sweep<256, KIND_GATHER, 256, LV, 1>(J, G, out, st)
                  : launch_sweep<768, KIND_STREAM, 256, LV, 1>(J, G, out, st);
    JobsDev J2 = J;
    if (rc == kNoRoom)
        J2.wide_all = 1;
    else if (rc != KVS_OK || !J.s)
        return rc;
    constexpr int kWinBig = (LV == kLevelsMax) ? 128 : 256; /* 16384 two-word entries fill most of LDS */
    return big ? launch_sweep<512, KIND_WIDE, kWinBig, LV, 1>(J2, G, out, st)
               : launch_sweep<256, KIND_WIDE, 256, LV, 1>(J2, G, out, st);
}

int32_t run_group(const JobsDev &J, const GroupArg &G, const OutsDev &out, hipStream_t st)
{
    /* explicit ladder: the instantiations with room for KVS_MAX_LEVELS levels */
    return G.n_lv > 0 ? run_group_lv<kLevelsMax>(J, G, out, st) : run_group_lv<kLevelsGeo>(J, G, out, st);
}

struct HostPoint {
    uint32_t tau0, k;
    int sched, mode, q;
    const int32_t *ladder; /* explicit slices, or null for the geometric ladder from tau0 */
    int n_lv;
};

/*
 * Splits the points into launches.  Points share a launch when their initial
 * slices are base * 2^m for a common base (the odd part of tau0) and they
 * have the same mode; a launch holds at most kMaxM shifts and kMaxV variants.
 * A lone invocation of the subroutine has no ladder: its slice is the base.
 * Points with an explicit ladder share a launch when the ladders are equal.
 */
int32_t run_points(const JobsDev &J, const HostPoint *pts, int n_pts, const OutsDev &out,
                   hipStream_t st)
{
    bool taken[KVS_MAX_POINTS] = {false};
    for (int first = 0; first < n_pts; first++) {
        if (taken[first])
            continue;
        const int mode = pts[first].mode;
        const int32_t *ladder = pts[first].ladder;
        const uint32_t base = ladder ? (uint32_t)ladder[0]
                              : (mode == MODE_SINGLE)
                                  ? pts[first].tau0
                                  : pts[first].tau0 >> __builtin_ctz(pts[first].tau0);
        GroupArg G;
        memset(&G, 0, sizeof(G));
        G.base = base;
        G.lg_base = (uint8_t)kvs_ilog2_floor(base);
        G.mode = (uint8_t)mode;
        if (ladder) {
            G.n_lv = (uint8_t)pts[first].n_lv;
            for (int l = 0; l < pts[first].n_lv; l++)
                G.ladder[l] = (uint32_t)ladder[l];
        }
        for (int i = first; i < n_pts; i++) {
            if (taken[i] || pts[i].mode != mode || (pts[i].ladder != nullptr) != (ladder != nullptr))
                continue;
            uint32_t m = 0;
            if (ladder) {
                if (pts[i].n_lv != pts[first].n_lv ||
                    memcmp(pts[i].ladder, ladder, sizeof(int32_t) * (size_t)pts[i].n_lv) != 0)
                    continue;
            } else if (mode == MODE_SINGLE) {
                if (pts[i].tau0 != base)
                    continue;
            } else {
                m = (uint32_t)__builtin_ctz(pts[i].tau0);
                if ((pts[i].tau0 >> m) != base)
                    continue;
            }
            int mi = -1, vi = -1;
            for (int a = 0; a < G.n_m; a++)
                if (G.m[a] == m)
                    mi = a;
            for (int a = 0; a < G.n_v; a++)
                if (G.v_sched[a] == pts[i].sched && G.v_k[a] == pts[i].k)
                    vi = a;
            if ((mi < 0 && G.n_m == kMaxM) || (vi < 0 && G.n_v == kMaxV))
                continue; /* next launch */
            if (mi < 0) {
                mi = G.n_m++;
                G.m[mi] = (uint8_t)m;
            }
            if (vi < 0) {
                vi = G.n_v++;
                G.v_sched[vi] = (uint8_t)pts[i].sched;
                G.v_k[vi] = pts[i].k;
            }
            G.pt_m[G.n_pts] = (uint8_t)mi;
            G.pt_v[G.n_pts] = (uint8_t)vi;
            G.pt_q[G.n_pts] = (uint16_t)pts[i].q;
            G.n_pts++;
            taken[i] = true;
        }
        /* the kernel wants the shifts in ascending order */
        for (int a = 1; a < G.n_m; a++)
            for (int b = a; b > 0 && G.m[b] < G.m[b - 1]; b--) {
                const uint8_t t = G.m[b];
                G.m[b] = G.m[b - 1];
                G.m[b - 1] = t;
                for (int p = 0; p < G.n_pts; p++) {
                    if (G.pt_m[p] == b)
                        G.pt_m[p] = (uint8_t)(b - 1);
                    else if (G.pt_m[p] == b - 1)
                        G.pt_m[p] = (uint8_t)b;
                }
            }
        const int32_t rc = run_group(J, G, out, st);
        if (rc != KVS_OK)
            return rc;
    }
    return KVS_OK;
}

} /* namespace */

extern "C" {

int32_t kvs_gba_simulate(const kvs_jobs_t *jobs, const kvs_point_t *pts, int32_t n_pts,
                         int64_t *peak, uint8_t *feasible, int64_t *flow, int64_t *job_steps,
                         void *stream)
{
    int32_t rc = check_jobs(jobs);
    if (rc != KVS_OK)
        return rc;
    if (n_pts < 0 || (n_pts > 0 && !pts))
        return KVS_EINVAL;
    if (n_pts > KVS_MAX_POINTS)
        return KVS_ELIMIT;
    if (jobs->n_instances == 0 || n_pts == 0)
        return KVS_OK;
    if (!peak || !feasible || !flow)
        return KVS_EINVAL;
    HostPoint hp[KVS_MAX_POINTS];
    kvs_point_t refill[KVS_MAX_POINTS]; /* the points with dynamic refill go to their own kernel */
    int32_t refill_row[KVS_MAX_POINTS];
    int32_t n_hp = 0, n_refill = 0;
    for (int32_t q = 0; q < n_pts; q++) {
        const kvs_point_t &p = pts[q];
        if (p.tau0 < 1 || (uint32_t)p.tau0 > kLenMax || p.k < 0 ||
            (p.sched != KVS_SCHED_SPS && p.sched != KVS_SCHED_SIMS) ||
            (p.mode != KVS_MODE_GBA && p.mode != KVS_MODE_GSA && p.mode != KVS_MODE_GBAD))
            return KVS_EINVAL;
        if (p.mode == KVS_MODE_GBAD) {
            refill[n_refill] = p;
            refill_row[n_refill++] = q;
            continue;
        }
        hp[n_hp].tau0 = (uint32_t)p.tau0;
        hp[n_hp].k = (uint32_t)p.k;
        hp[n_hp].sched = p.sched;
        hp[n_hp].mode = (p.mode == KVS_MODE_GSA) ? MODE_GSA : MODE_GBA;
        hp[n_hp].q = q;
        hp[n_hp].ladder = nullptr;
        hp[n_hp].n_lv = 0;
        n_hp++;
    }
    OutsDev out{peak, feasible, flow, job_steps, nullptr};
    if (n_hp > 0) {
        rc = run_points(to_dev(jobs, true), hp, n_hp, out, static_cast<hipStream_t>(stream));
        if (rc != KVS_OK)
            return rc;
    }
    if (n_refill > 0)
        return kvs_gbad_run(jobs, refill, refill_row, n_refill, peak, feasible, flow, job_steps, stream);
    return KVS_OK;
}

int32_t kvs_schedule_eval(const kvs_jobs_t *jobs, const int32_t *tau, const int32_t *k,
                          const int32_t *sched, int32_t n_pts, int64_t *peak, uint8_t *feasible,
                          int64_t *flow, int32_t *n_completed, int64_t *job_steps, void *stream)
{
    int32_t rc = check_jobs(jobs);
    if (rc != KVS_OK)
        return rc;
    if (n_pts < 0 || (n_pts > 0 && (!tau || !k || !sched)))
        return KVS_EINVAL;
    if (n_pts > KVS_MAX_POINTS)
        return KVS_ELIMIT;
    if (jobs->n_instances == 0 || n_pts == 0)
        return KVS_OK;
    if (!peak || !feasible || !flow)
        return KVS_EINVAL;
    HostPoint hp[KVS_MAX_POINTS];
    for (int32_t q = 0; q < n_pts; q++) {
        if (tau[q] < 1 || (uint32_t)tau[q] > kLenMax || k[q] < 0 ||
            (sched[q] != KVS_SCHED_SPS && sched[q] != KVS_SCHED_SIMS))
            return KVS_EINVAL;
        hp[q].tau0 = (uint32_t)tau[q];
        hp[q].k = (uint32_t)k[q];
        hp[q].sched = sched[q];
        hp[q].mode = MODE_SINGLE;
        hp[q].q = q;
        hp[q].ladder = nullptr;
        hp[q].n_lv = 0;
    }
    OutsDev out{peak, feasible, flow, job_steps, n_completed};
    return run_points(to_dev(jobs, false), hp, n_pts, out, static_cast<hipStream_t>(stream));
}

int32_t kvs_ladder_simulate(const kvs_jobs_t *jobs, const int32_t *ladders,
                            const int32_t *n_levels, const int32_t *sched, const int32_t *k,
                            const int32_t *mode, int32_t n_pts, int64_t *peak, uint8_t *feasible,
                            int64_t *flow, int64_t *job_steps, void *stream)
{
    int32_t rc = check_jobs(jobs);
    if (rc != KVS_OK)
        return rc;
    if (n_pts < 0 || (n_pts > 0 && (!ladders || !n_levels || !sched || !k || !mode)))
        return KVS_EINVAL;
    if (n_pts > KVS_MAX_POINTS)
        return KVS_ELIMIT;
    if (jobs->n_instances == 0 || n_pts == 0)
        return KVS_OK;
    if (!peak || !feasible || !flow)
        return KVS_EINVAL;
    HostPoint hp[KVS_MAX_POINTS];
    for (int32_t q = 0; q < n_pts; q++) {
        const int32_t *lad = ladders + (size_t)q * KVS_MAX_LEVELS;
        if (n_levels[q] < 1 || n_levels[q] > KVS_MAX_LEVELS || k[q] < 0 ||
            (sched[q] != KVS_SCHED_SPS && sched[q] != KVS_SCHED_SIMS) ||
            (mode[q] != KVS_MODE_GBA && mode[q] != KVS_MODE_GSA))
            return KVS_EINVAL;
        for (int32_t l = 0; l < n_levels[q]; l++)
            if (lad[l] < 1 || (uint32_t)lad[l] > kLenMax || (l > 0 && lad[l] < lad[l - 1]))
                return KVS_EINVAL;
        hp[q].tau0 = (uint32_t)lad[0];
        hp[q].k = (uint32_t)k[q];
        hp[q].sched = sched[q];
        hp[q].mode = (mode[q] == KVS_MODE_GSA) ? MODE_GSA : MODE_GBA;
        hp[q].q = q;
        hp[q].ladder = lad;
        hp[q].n_lv = n_levels[q];
    }
    OutsDev out{peak, feasible, flow, job_steps, nullptr};
    return run_points(to_dev(jobs, true), hp, n_pts, out, static_cast<hipStream_t>(stream));
}

int32_t kvs_paper_ladder(int64_t M, int64_t s, int32_t alpha_num, int32_t alpha_den,
                         int32_t *ladder, int32_t *n_levels)
{
    if (!ladder || !n_levels || s < 0 || M <= s || M - s > (int64_t)kLenMax || alpha_den < 1 ||
        alpha_num <= alpha_den)
        return KVS_EINVAL;
    typedef unsigned __int128 u128;
    const u128 span = (u128)(M - s);
    const u128 limit = ((u128)1) << 126; /* no product below may reach it */
    /* l = max{ j : alpha^j <= M - s }  <=>  num^j <= (M - s) den^j */
    u128 pn = 1, pd = 1; /* num^l, den^l */
    int l = 0;
    for (;;) {
        if (pn > limit / (u128)alpha_num || pd > limit / ((u128)alpha_den * span))
            return KVS_ELIMIT;
        const u128 nn = pn * (u128)alpha_num, nd = pd * (u128)alpha_den;
        if (nn > span * nd)
            break;
        pn = nn;
        pd = nd;
        l++;
        if (l + 1 > KVS_MAX_LEVELS)
            return KVS_ELIMIT;
    }
    /* tau_p = floor(beta alpha^p) = floor((M - s) den^(l-p) / num^(l-p)), p = l, l-1, ..., 0 */
    u128 an = 1, ad = 1; /* num^(l-p), den^(l-p) */
    for (int p = l; p >= 0; p--) {
        ladder[p] = (int32_t)((span * ad) / an);
        an *= (u128)alpha_num;
        ad *= (u128)alpha_den;
    }
    *n_levels = l + 1;
    return KVS_OK;
}

int32_t kvs_paper_ladder_quadratic(int64_t M, int64_t s, int32_t a, int32_t b, int32_t c, int32_t d,
                                   int32_t *ladder, int32_t *n_levels)
{
    if (!ladder || !n_levels || s < 0 || M <= s || M - s > (int64_t)kLenMax || a < 0 || b < 0 || c < 0 ||
        d < 1)
        return KVS_EINVAL;
    typedef unsigned __int128 u128;
    /* alpha and its powers as intervals [lo, hi] of extended-precision numbers that contain the
     * true values: every operation below is correctly rounded to 64 bits (relative error at most
     * 2^-64), and widening its result by 2^-62 on either side covers that and leaves room for the
     * error of the operands' own widening to compound over at most 64 levels. */
    const long double eps = 0x1p-62L;
    const long double root = sqrtl((long double)c);
    const long double alpha = ((long double)a + (long double)b * root) / (long double)d;
    const long double a_lo = alpha * (1.0L - eps), a_hi = alpha * (1.0L + eps);
    if (!(a_lo > 1.0L))
        return KVS_EINVAL; /* alpha <= 1, or too close to 1 to tell */
    const u128 X = (u128)(M - s);
    const long double span = (long double)(M - s);
    /* Beside the intervals, alpha^q = (A_q + B_q sqrt(c)) / d^q in integers while they fit 128
     * bits: where an interval cannot decide a comparison (powers of sqrt(2) hit integers), it is
     * decided exactly:  y alpha^q <= X  <=>  X d^q - y A_q >= 0 and (y B_q)^2 c <= (X d^q - y A_q)^2. */
    u128 eA[KVS_MAX_LEVELS + 2], eB[KVS_MAX_LEVELS + 2], eD[KVS_MAX_LEVELS + 2];
    bool exact[KVS_MAX_LEVELS + 2];
    eA[0] = 1; eB[0] = 0; eD[0] = 1; exact[0] = true;
    auto mul = [](u128 x, u128 y, u128 &r) { return !__builtin_mul_overflow(x, y, &r); };
    auto next_exact = [&](int q) { /* level q + 1 from level q */
        u128 t1, t2, t3, t4, t5, nd;
        exact[q + 1] = exact[q] && mul(eA[q], (u128)a, t1) && mul(eB[q], (u128)b, t2) && mul(t2, (u128)c, t3) &&
                       mul(eA[q], (u128)b, t4) && mul(eB[q], (u128)a, t5) && mul(eD[q], (u128)d, nd) &&
                       !__builtin_add_overflow(t1, t3, &eA[q + 1]) && !__builtin_add_overflow(t4, t5, &eB[q + 1]);
        if (exact[q + 1])
            eD[q + 1] = nd;
    };
    /* 1: y alpha^q <= X, 0: not, -1: does not fit 128 bits */
    auto exact_le = [&](u128 y, int q) -> int {
        u128 xd, ya, yb, lhs, rhs;
        if (!exact[q] || !mul(X, eD[q], xd) || !mul(y, eA[q], ya) || !mul(y, eB[q], yb))
            return -1;
        if (xd < ya)
            return 0;
        const u128 r = xd - ya;
        if (!mul(yb, yb, lhs) || !mul(lhs, (u128)c, lhs) || !mul(r, r, rhs))
            return -1;
        return lhs <= rhs ? 1 : 0;
    };
    long double pw_lo[KVS_MAX_LEVELS + 2], pw_hi[KVS_MAX_LEVELS + 2]; /* alpha^j */
    pw_lo[0] = pw_hi[0] = 1.0L;
    int l = 0; /* the largest j with alpha^j <= M - s */
    for (;;) {
        if (l + 1 > KVS_MAX_LEVELS)
            return KVS_ELIMIT;
        const long double n_lo = pw_lo[l] * a_lo * (1.0L - eps), n_hi = pw_hi[l] * a_hi * (1.0L + eps);
        next_exact(l);
        if (n_lo > span)
            break; /* alpha^(l+1) > M - s for certain */
        if (!(n_hi <= span)) { /* too close to M - s for the interval */
            const int le = exact_le(1, l + 1);
            if (le < 0)
                return KVS_ELIMIT;
            if (le == 0)
                break;
        }
        pw_lo[l + 1] = n_lo;
        pw_hi[l + 1] = n_hi;
        l++;
    }
    /* tau_p = floor(beta alpha^p) = floor((M - s) / alpha^(l-p)); the top one is M - s itself */
    for (int p = 0; p <= l; p++) {
        const int q = l - p;
        if (q == 0) {
            ladder[p] = (int32_t)(M - s);
            continue;
        }
        const long double x_lo = span / pw_hi[q] * (1.0L - eps), x_hi = span / pw_lo[q] * (1.0L + eps);
        const long double f_lo = floorl(x_lo), f_hi = floorl(x_hi);
        if (f_lo == f_hi) {
            ladder[p] = (int32_t)f_lo;
            continue;
        }
        /* an integer lies inside the interval: the floor is it, or the one below */
        if (f_hi != f_lo + 1.0L || f_lo < 0.0L)
            return KVS_ELIMIT;
        const int le = exact_le((u128)f_hi, q);
        if (le < 0)
            return KVS_ELIMIT;
        ladder[p] = (int32_t)(le ? f_hi : f_lo);
    }
    *n_levels = l + 1;
    return KVS_OK;
}

int32_t kvs_validate(const kvs_jobs_t *jobs, void *stream)
{
    int32_t rc = check_jobs(jobs);
    if (rc != KVS_OK)
        return rc;
    if (jobs->n_instances == 0)
        return KVS_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ValidateResult *dres = nullptr;
    ValidateResult h{0, 0, 0};
    if (hipMalloc(reinterpret_cast<void **>(&dres), sizeof(ValidateResult)) != hipSuccess)
        return KVS_EHIP;
    rc = KVS_OK;
    if (hipMemsetAsync(dres, 0, sizeof(ValidateResult), st) != hipSuccess)
        rc = KVS_EHIP;
    if (rc == KVS_OK) {
        const size_t total = (size_t)jobs->n_instances * (size_t)jobs->n_jobs;
        size_t blocks = (total + 255) / 256;
        if (blocks > 256 * 32)
            blocks = 256 * 32;
        hipLaunchKernelGGL(kvs_validate_kernel, dim3((uint32_t)blocks), dim3(256), 0, st,
                           to_dev(jobs, true), dres);
        if (hipGetLastError() != hipSuccess)
            rc = KVS_EHIP;
    }
    if (rc == KVS_OK &&
        hipMemcpyAsync(&h, dres, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess)
        rc = KVS_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess)
        rc = KVS_EHIP;
    (void)hipFree(dres);
    if (rc != KVS_OK)
        return rc;
    if (h.bad_value)
        return KVS_EINVAL;
    if (h.too_long)
        return KVS_ERANGE;
    if (h.infeasible)
        return KVS_EJOB_INFEASIBLE;
    return KVS_OK;
}

int32_t kvs_validate_static(const kvs_jobs_t *jobs, void *stream)
{
    int32_t rc = check_jobs(jobs);
    if (rc != KVS_OK)
        return rc;
    if (jobs->n_instances == 0)
        return KVS_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *p = nullptr;
    rc = static_scratch(&p);
    if (rc != KVS_OK)
        return rc;
    ValidateResult *dres = static_cast<ValidateResult *>(p);
    ValidateResult h{0, 0, 0};
    /* the last call's findings are still there: cleared by a kernel, not by a memset node */
    hipLaunchKernelGGL(kvs_clear_result_kernel, dim3(1), dim3(64), 0, st, dres);
    if (hipGetLastError() != hipSuccess)
        return KVS_EHIP;
    const size_t total = (size_t)jobs->n_instances * (size_t)jobs->n_jobs;
    size_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32)
        blocks = 256 * 32;
    hipLaunchKernelGGL(kvs_validate_kernel, dim3((uint32_t)blocks), dim3(256), 0, st,
                       to_dev(jobs, true), dres);
    if (hipGetLastError() != hipSuccess)
        rc = KVS_EHIP;
    if (rc == KVS_OK &&
        hipMemcpyAsync(&h, dres, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess)
        rc = KVS_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess)
        rc = KVS_EHIP;
    if (rc != KVS_OK)
        return rc;
    if (h.bad_value)
        return KVS_EINVAL;
    if (h.too_long)
        return KVS_ERANGE;
    if (h.infeasible)
        return KVS_EJOB_INFEASIBLE;
    return KVS_OK;
}

const char *kvs_strerror(int32_t status)
{
    switch (status) {
    case KVS_OK: return "ok";
    case KVS_EINVAL: return "invalid argument or job data";
    case KVS_EJOB_INFEASIBLE: return "a job does not fit the memory budget on its own (s + o > M)";
    case KVS_ERANGE: return "a length exceeds 2^30";
    case KVS_EHIP: return "HIP runtime error";
    case KVS_ELIMIT: return "size above the compiled limits";
    default: return "unknown status";
    }
}

int32_t kvs_version(void) { return 600; }

/* Host evaluation of the kernels' integer helpers, for the host-side tests (kvsched_test.h). */
uint32_t kvs_host_class_index(uint32_t x, uint32_t tau0)
{
    return kvs_class_index(x, tau0, kvs_ilog2_floor(tau0));
}

uint32_t kvs_host_ladder_level(uint32_t x, const uint32_t *lad, uint32_t n_lv)
{
    return kvs_ladder_level(x, lad, n_lv);
}

uint32_t kvs_host_div(uint32_t x, uint32_t d) { return kvs_div(x, kvs_make_divisor(d)); }

uint64_t kvs_host_kstar(uint64_t tau, uint64_t s, uint64_t M) { return kvs_kstar(tau, s, M); }

} /* extern "C" */
