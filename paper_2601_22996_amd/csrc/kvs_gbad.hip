/*
 * kvs_gbad.hip -- Algorithm 2 with dynamic refill ("GBA-D") on gfx950.
 *
 * Paper: "Competitive Non-Clairvoyant KV-Cache Scheduling for LLM Inference"
 * (Feng, Yang, Zhang), appendix "Numerical Experiments", paragraph "Dynamic
 * Refill": a job is admitted as soon as the pipeline can go on with it without
 * violating memory feasibility, and no job is later than in the schedule of
 * Algorithm 2.  The paper gives no more than that; the rule evaluated here:
 *
 *   The baseline is Algorithm 2's schedule (classes on the ladder tau_0 * 2^p,
 *   Procedure 1 or the simultaneous schedule inside a class).  Every job first
 *   holds its baseline start with its actual run of o_i rounds.  In the
 *   baseline's order (class by class, input order inside a class) each job
 *   moves to the earliest round, not before the start of the job before it
 *   and not after its own baseline start, at which its whole run fits in every
 *   round (eq. (Memory-Feasibility)) on top of all other jobs where they stand:
 *   the earlier ones where they were moved, the later ones at their baseline
 *   starts.  A job can therefore always fall back on its baseline start.
 *
 * Unlike the other modes this one is sequential by nature: where a job goes
 * depends on where all the jobs before it went.  One wavefront evaluates one
 * (instance, point): the occupancy of every round of the schedule lives in
 * LDS, a run is taken out, tried and put back 64 rounds at a time, and a start
 * that fails is not followed by the next round but by the first start that the
 * failing rounds do not already rule out.
 */
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <initializer_list>

#include "kvs_internal.h"
#include "kvs_math.h"
#include "kvs_wave.h"
#include "kvsched.h"

namespace {

constexpr uint32_t kLenMax = 1u << 30;
constexpr int kLv = 32; /* classes that lengths up to 2^30 can reach on a ladder tau_0 * 2^p */

constexpr uint32_t FLAG_EINVAL = 1u, FLAG_ERANGE = 2u, FLAG_EJOB = 4u;

struct DJobs {
    const int32_t *o, *s;
    int32_t n_inst, n_jobs;
    uint32_t s_scalar;
    uint32_t cap; /* rounds of the schedule that fit LDS beside the jobs */
    uint32_t only_marked; /* take only the evaluations the launch before left behind            */
    uint32_t may_defer;   /* an evaluation that needs more rounds is left to the next launch */
    uint64_t M;
};

struct DPoints {
    uint32_t tau0[KVS_MAX_POINTS];
    uint32_t k[KVS_MAX_POINTS];
    uint16_t q[KVS_MAX_POINTS]; /* output row */
    uint8_t sched[KVS_MAX_POINTS];
    int32_t n;
};

/* What this wavefront wrote to LDS is seen by its later reads, whichever lane did either: a
 * workgroup here is one wavefront, whose LDS operations are carried out in order. */
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr uint8_t FEASIBLE_PENDING = 0xFD; /* internal: left for the launch with all of LDS */

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    /* values below 2^31 here */
    return (uint32_t)wave_max_nonneg((int32_t)v);
}

__global__ __launch_bounds__(64) void kvs_gbad_kernel(DJobs J, DPoints P, int64_t *peak, uint8_t *feasible,
                                                      int64_t *flow, int64_t *job_steps)
{
    /* dynamic LDS: the jobs in the baseline's order (length, prompt), then the occupancy of
     * every round */
    extern __shared__ uint32_t lds[];
    __shared__ uint32_t cnt[kLv], smax[kLv], off[kLv], tauc[kLv], kc[kLv], beginc[kLv];
    __shared__ kvs_divisor_t divc[kLv];
    __shared__ uint32_t flags, horizon;

    const int lane = threadIdx.x;
    const uint32_t inst = blockIdx.x, pt = blockIdx.y;
    if (J.only_marked && feasible[(size_t)P.q[pt] * (size_t)J.n_inst + inst] != FEASIBLE_PENDING)
        return; /* done by a launch before */
    const uint32_t n = (uint32_t)J.n_jobs;
    const size_t row = (size_t)inst * n;
    uint32_t *const ordO = lds, *const ordS = lds + n;
    int32_t *const occ = reinterpret_cast<int32_t *>(lds + 2u * n);
    const uint32_t tau0 = P.tau0[pt];
    const uint32_t lg_tau0 = kvs_ilog2_floor(tau0);
    const bool sps = P.sched[pt] == KVS_SCHED_SPS;

    if (lane < kLv) {
        cnt[lane] = 0;
        smax[lane] = J.s ? 0u : J.s_scalar;
    }
    if (lane == 0)
        flags = 0;
    __syncthreads();

    /* ---- classes: how many jobs, and the largest prompt ---- */
    unsigned long long sumO = 0;
    uint32_t badbits = 0;
    auto class_of = [&](uint32_t i, uint32_t &o, uint32_t &s) {
        const int32_t ro = J.o[row + i];
        const int32_t rs = J.s ? J.s[row + i] : (int32_t)J.s_scalar;
        uint32_t bad = 0;
        if (ro < 1 || rs < 0)
            bad = FLAG_EINVAL;
        else if ((uint32_t)ro > kLenMax || (uint32_t)rs > kLenMax)
            bad = FLAG_ERANGE;
        else if ((uint64_t)(uint32_t)rs + (uint64_t)(uint32_t)ro > J.M)
            bad = FLAG_EJOB;
        badbits |= bad;
        o = ro < 1 ? 1u : ((uint32_t)ro > kLenMax ? kLenMax : (uint32_t)ro);
        s = rs < 0 ? 0u : ((uint32_t)rs > kLenMax ? kLenMax : (uint32_t)rs);
        return kvs_class_index(o, tau0, lg_tau0);
    };
    for (uint32_t i = (uint32_t)lane; i < n; i += 64) {
        uint32_t o, s;
        const uint32_t c = class_of(i, o, s);
        sumO += o;
        atomicAdd(&cnt[c], 1u);
        if (J.s && s > smax[c])
            atomicMax(&smax[c], s);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        sumO += __shfl_xor(sumO, d, 64);
        badbits |= __shfl_xor(badbits, d, 64);
    }
    __syncthreads();

    /* ---- the baseline's phase table: one lane per class ---- */
    {
        uint32_t n_c = 0, err = 0;
        unsigned long long len = 0;   /* rounds the class lasts */
        unsigned long long most = 0;  /* bound on what its jobs hold together in a round */
        if (lane < kLv) {
            n_c = cnt[lane];
            const uint64_t tau = (uint64_t)tau0 << lane;
            uint64_t k = 1;
            if (n_c > 0) {
                if (tau * n_c >= (1ull << 31)) {
                    err = 1;
                } else {
                    const uint64_t sm = smax[lane];
                    if (P.k[pt] > 0)
                        k = P.k[pt];
                    else if (sps)
                        k = kvs_kstar(tau, sm, J.M);
                    else
                        k = J.M / (sm + tau);
                    if (k < 1)
                        k = 1;
                    const uint64_t kcap = sps ? tau * n_c : n_c; /* beyond this the offsets no longer change */
                    if (k > kcap)
                        k = kcap;
                    const uint64_t act = k < n_c ? k : n_c;
                    most = act * (sm + tau + 1u);
                    if (most >= (1ull << 31))
                        err = 1;
                    const uint64_t last = sps ? ((uint64_t)(n_c - 1u) * tau) / k : ((uint64_t)(n_c - 1u) / k) * tau;
                    len = last + tau;
                }
            }
            tauc[lane] = (uint32_t)(tau > 0xffffffffull ? 0xffffffffull : tau);
            kc[lane] = (uint32_t)k;
            divc[lane] = kvs_make_divisor((uint32_t)k);
        }
        unsigned long long pre = len; /* inclusive prefix over the classes */
        uint32_t pre_n = n_c;
#pragma unroll
        for (int d = 1; d < kLv; d <<= 1) {
            const unsigned long long up = __shfl_up(pre, d, 64);
            const uint32_t un = __shfl_up(pre_n, d, 64);
            if (lane >= d) {
                pre += up;
                pre_n += un;
            }
        }
        /* moved jobs of different classes can share a round: all classes together stay in 31 bits */
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1)
            most += __shfl_xor(most, d, 64);
        if (most >= (1ull << 31))
            err = 1;
        const unsigned long long total = __shfl(pre, kLv - 1, 64);
        if (lane < kLv) {
            beginc[lane] = (uint32_t)(pre - len); /* meaningful only when total fits */
            off[lane] = pre_n - n_c;
        }
        err = __any(err != 0) ? 1u : 0u;
        if (lane == 0) {
            uint32_t f = badbits;
            if (err)
                f |= 8u; /* this evaluation leaves the range in some class */
            else if (total > (unsigned long long)J.cap)
                f |= (J.may_defer && f == 0) ? 16u : 8u; /* more rounds than fit: the next launch has more room, or none has */
            flags = f;
            horizon = (uint32_t)(total > (unsigned long long)J.cap ? 0ull : total);
        }
    }
    __syncthreads();

    const uint32_t fl = flags;
    if (fl != 0) {
        if (lane == 0) {
            uint8_t code = KVS_FEASIBLE_ERANGE;
            if (fl == 16u)
                code = FEASIBLE_PENDING;
            if (fl & FLAG_EINVAL)
                code = KVS_FEASIBLE_EINVAL;
            else if (fl & FLAG_ERANGE)
                code = KVS_FEASIBLE_ERANGE;
            else if (fl & FLAG_EJOB)
                code = KVS_FEASIBLE_EJOB;
            const size_t oi = (size_t)P.q[pt] * (size_t)J.n_inst + inst;
            peak[oi] = -1;
            feasible[oi] = code;
            flow[oi] = -1;
            if (job_steps)
                job_steps[oi] = -1;
        }
        return;
    }
    const uint32_t H = horizon;

    /* ---- the jobs in the baseline's order: class by class, input order inside ---- */
    {
        uint32_t cur = lane < kLv ? off[lane] : 0u; /* lane c: next free place of class c */
        for (uint32_t b = 0; b < n; b += 64) {
            const uint32_t i = b + (uint32_t)lane;
            const bool act = i < n;
            uint32_t o = 1, s = 0, c = 0, pos = 0;
            if (act)
                c = class_of(i, o, s);
            uint64_t todo = __ballot(act);
            while (todo) {
                const int src = __ffsll((unsigned long long)todo) - 1;
                const uint32_t c0 = __builtin_amdgcn_readlane(c, src);
                const uint64_t mk = __ballot(act && c == c0);
                const uint32_t at = __builtin_amdgcn_readlane(cur, (int)c0);
                if (act && c == c0)
                    pos = at + lanes_below(mk);
                if ((uint32_t)lane == c0)
                    cur += (uint32_t)__popcll(mk);
                todo &= ~mk;
            }
            if (act) {
                ordO[pos] = o;
                ordS[pos] = s + 1u; /* what the job holds in its first round */
            }
        }
        for (uint32_t t = (uint32_t)lane; t < H; t += 64)
            occ[t] = 0;
    }
    __syncthreads();

    /* a run of o rounds from round t, first round s1: added to (sign = 1) or taken out of the rounds */
    /* (additions carried out by the LDS unit itself, in the order they are issued: nothing comes
     * back, so the wavefront does not wait for one round's old value before it goes on) */
    auto ramp = [&](uint32_t t, uint32_t o, uint32_t s1, int32_t sign) {
        for (uint32_t u = (uint32_t)lane; u < o; u += 64)
            atomicAdd(&occ[t + u], sign * (int32_t)(s1 + u));
    };
    /* The jobs are gone through in the baseline's order.  64 of them at a time sit in the lanes
     * (lane j: job pos0 + j) and are handed to the whole wavefront one after the other, and the
     * current class's slice, divisor and first round are kept in registers: per job nothing is
     * fetched from LDS but the rounds themselves. */
    uint32_t cls = 0, cls_r = 0;           /* class of the next job, and its place in the class */
    uint32_t cls_n = 0, cls_tau = 0, cls_begin = 0;
    kvs_divisor_t cls_div = kvs_make_divisor(1);
    auto load_class = [&]() {
        cls_n = cnt[cls];
        cls_tau = tauc[cls];
        cls_begin = beginc[cls];
        cls_div = divc[cls];
    };
    auto next_base = [&]() { /* baseline start of the next job; moves on to it */
        while (cls_r >= cls_n) { /* next class with a job */
            cls++;
            cls_r = 0;
            load_class();
        }
        const uint32_t f = sps ? kvs_div(cls_r * cls_tau, cls_div) : kvs_div(cls_r, cls_div) * cls_tau;
        cls_r++;
        return cls_begin + f;
    };

    /* ---- everybody at the baseline start ---- */
    load_class();
    for (uint32_t pos0 = 0; pos0 < n; pos0 += 64) {
        const uint32_t mine = pos0 + (uint32_t)lane < n ? pos0 + (uint32_t)lane : n - 1u;
        const uint32_t myO = ordO[mine], myS = ordS[mine];
        const uint32_t m = n - pos0 < 64u ? n - pos0 : 64u;
        for (uint32_t j = 0; j < m; j++)
            ramp(next_base(), __builtin_amdgcn_readlane(myO, (int)j), __builtin_amdgcn_readlane(myS, (int)j), 1);
    }
    __syncthreads();

    /* ---- refill, one job after the other ---- */
    unsigned long long fsum = 0;
    const uint32_t m32 = J.M > 0xffffffffull ? 0xffffffffu : (uint32_t)J.M; /* a round holds less than 2^32 */
    {
        uint32_t prev = 0;
        cls = 0;
        cls_r = 0;
        load_class();
        for (uint32_t pos0 = 0; pos0 < n; pos0 += 64) {
          const uint32_t mine = pos0 + (uint32_t)lane < n ? pos0 + (uint32_t)lane : n - 1u;
          const uint32_t myO = ordO[mine], myS = ordS[mine];
          const uint32_t m = n - pos0 < 64u ? n - pos0 : 64u;
          for (uint32_t j = 0; j < m; j++) {
            const uint32_t o = __builtin_amdgcn_readlane(myO, (int)j), s1 = __builtin_amdgcn_readlane(myS, (int)j);
            const uint32_t base = next_base();
            uint32_t t = prev;
            while (t < base) {
                /* every round of the run is looked at, 64 at a time; a round over the budget rules
                 * out every start up to it, or up to where the run would be that much smaller in
                 * it, whichever comes first; the largest such move over all failing rounds skips
                 * only starts that fail in one of them.  The lanes keep their own largest move and
                 * the wavefront is asked once per start, not once per 64 rounds: most starts fit. */
                uint32_t cand = 0;
                auto look = [&](uint32_t u, uint32_t held_all) {
                    /* what the others hold in that round: the job's own run, still at its baseline
                     * start, is taken off */
                    const uint32_t x = t + u;
                    const uint32_t own = (x >= base) ? s1 + (x - base) : 0u; /* x < base + o: t < base */
                    const uint32_t held = held_all - own + (s1 + u); /* both parts below 2^31 */
                    if (held > m32) {
                        const uint32_t over = held - m32;
                        const uint32_t c = (over < u + 1u) ? t + over : t + u + 1u;
                        cand = c > cand ? c : cand;
                    }
                };
                uint32_t u = (uint32_t)lane;
                for (; u + 192u < o; u += 256u) { /* four reads in flight */
                    const uint32_t h0 = (uint32_t)occ[t + u], h1 = (uint32_t)occ[t + u + 64u],
                                   h2 = (uint32_t)occ[t + u + 128u], h3 = (uint32_t)occ[t + u + 192u];
                    look(u, h0);
                    look(u + 64u, h1);
                    look(u + 128u, h2);
                    look(u + 192u, h3);
                }
                for (; u < o; u += 64u)
                    look(u, (uint32_t)occ[t + u]);
                const uint32_t next = __any(cand != 0) ? wave_max_u32(cand) : 0u;
                if (next == 0)
                    break; /* fits */
                t = next;
            }
            if (t < base) { /* it moves */
                ramp(base, o, s1, -1);
                ramp(t, o, s1, 1);
                wave_sync();
            } else {
                t = base;
            }
            prev = t;
            fsum += (unsigned long long)t + o;
          }
        }
    }

    /* ---- the largest occupancy of any round ---- */
    int32_t pk = 0;
    for (uint32_t t = (uint32_t)lane; t < H; t += 64)
        pk = occ[t] > pk ? occ[t] : pk;
    pk = wave_max_nonneg(pk);
    if (lane == 0) {
        const size_t oi = (size_t)P.q[pt] * (size_t)J.n_inst + inst;
        peak[oi] = pk;
        feasible[oi] = ((int64_t)pk <= (int64_t)J.M) ? 1 : 0;
        flow[oi] = (int64_t)fsum;
        if (job_steps)
            job_steps[oi] = (int64_t)sumO;
    }
}

constexpr size_t kLdsPerGroup = 160 * 1024;

} /* namespace */

int32_t kvs_gbad_run(const kvs_jobs_t *jobs, const kvs_point_t *pts, const int32_t *rows, int32_t n_pts,
                     int64_t *peak, uint8_t *feasible, int64_t *flow, int64_t *job_steps, void *stream)
{
    static std::atomic<int> static_lds{-1};
    int fixed = static_lds.load(std::memory_order_relaxed);
    if (fixed < 0) {
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(kvs_gbad_kernel)) != hipSuccess)
            return KVS_EHIP;
        fixed = (int)attr.sharedSizeBytes;
        static_lds.store(fixed, std::memory_order_relaxed);
    }
    DJobs J;
    J.o = jobs->o;
    J.s = jobs->s;
    J.n_inst = jobs->n_instances;
    J.n_jobs = jobs->n_jobs;
    J.s_scalar = jobs->s ? 0u : (uint32_t)jobs->s_scalar;
    J.M = (uint64_t)jobs->M;
    /* Up to three launches.  An evaluation is one wavefront working through dependent LDS
     * operations, and only company on its compute unit hides that; what limits the company is
     * the LDS an evaluation is given (the jobs, two words each, and one word per round of the
     * baseline schedule).  So the first launch gives every evaluation a quarter of a compute
     * unit's LDS, an evaluation whose baseline lasts longer marks itself, the second launch
     * takes only those with half of the LDS each, the third the rest with all of it.  Sizes at
     * which the jobs leave too little room for rounds are skipped. */
    const size_t whole = (kLdsPerGroup - (size_t)fixed) & ~(size_t)15;
    const size_t for_jobs = sizeof(uint32_t) * 2u * (size_t)jobs->n_jobs;
    if (for_jobs + 4096 > whole)
        return KVS_ELIMIT;
    DPoints P;
    P.n = n_pts;
    for (int32_t j = 0; j < n_pts; j++) {
        P.tau0[j] = (uint32_t)pts[j].tau0;
        P.k[j] = (uint32_t)pts[j].k;
        P.sched[j] = (uint8_t)pts[j].sched;
        P.q[j] = (uint16_t)rows[j];
    }
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kvs_gbad_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)whole) != hipSuccess)
        return KVS_EHIP;
    const dim3 grid((uint32_t)jobs->n_instances, (uint32_t)n_pts);
    size_t sizes[8];
    int n_sizes = 0;
    for (size_t parts : {4, 2}) { /* finer steps were measured: each launch has a tail of its own, and they add up to more */
        if (kLdsPerGroup / parts < (size_t)fixed + 64 + 16)
            continue;
        const size_t room = ((kLdsPerGroup / parts) - (size_t)fixed - 64) & ~(size_t)15;
        if (for_jobs + 8192 <= room)
            sizes[n_sizes++] = room;
    }
    sizes[n_sizes++] = whole;
    for (int i = 0; i < n_sizes; i++) {
        J.cap = (uint32_t)((sizes[i] - for_jobs) / sizeof(int32_t));
        J.only_marked = i > 0 ? 1u : 0u;
        J.may_defer = i + 1 < n_sizes ? 1u : 0u;
        hipLaunchKernelGGL(kvs_gbad_kernel, grid, dim3(64), sizes[i], static_cast<hipStream_t>(stream), J, P, peak,
                           feasible, flow, job_steps);
        if (hipGetLastError() != hipSuccess)
            return KVS_EHIP;
    }
    return KVS_OK;
}
