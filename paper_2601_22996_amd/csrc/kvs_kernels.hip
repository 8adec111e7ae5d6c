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
 * One workgroup evaluates one (instance, sweep point).  No round-by-round
 * stepping happens on the device: inside a phase the occupancy of round t is
 *     occ(t) = A(t) + t * C(t),
 *     C(t) = number of active runs,  A(t) = sum over them of (s + 1 - start),
 * and both are prefix sums over time of per-round event sums (a run adds
 * (s + 1 - start, 1) in its first round and takes it away in the round after
 * its last).  Events are scattered into LDS arrays one time window at a
 * time, scanned by the workgroup, and the maximum of occ is kept.  All values
 * are exact integers, so the result equals the stepped definition.
 */
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvsched.h"
#include "kvs_math.h"

namespace {

constexpr int kLevels = 32;            /* ladder levels tau0 * 2^p that 2^30-bounded lengths can reach */
constexpr uint32_t kLenMax = 1u << 30; /* largest length the 32-bit arithmetic is sized for */

constexpr uint32_t FLAG_EINVAL = 1u;
constexpr uint32_t FLAG_ERANGE = 2u;

constexpr int MODE_GBA = 0, MODE_GSA = 1, MODE_SINGLE = 2;

struct JobsDev {
    const int32_t *o;
    const int32_t *s;
    const int32_t *e;
    int32_t n_inst;
    int32_t n_jobs;
    uint32_t s_scalar;
    uint64_t M;
};

struct PointDev {
    uint32_t tau0;
    uint32_t k;
    uint8_t sched;
    uint8_t mode;
    uint8_t lg_tau0;
    uint8_t pad;
};

struct PointsArg {
    int32_t n;
    PointDev p[KVS_MAX_POINTS];
};

struct OutsDev {
    int64_t *peak;
    uint8_t *feasible;
    int64_t *flow;
    int64_t *job_steps;
    int32_t *n_completed;
};

/* One phase of one evaluation (a row of the phase table). */
struct Phase {
    uint32_t tau; /* slice length tau_p                                  */
    uint32_t n;   /* participants n_p                                    */
    uint32_t k;   /* parallelism k_p (SPS) or batch size (SimS), >= 1    */
    uint32_t H;   /* rounds the phase lasts: last start offset + tau_p   */
    kvs_divisor_t div;
    int64_t begin; /* round in which the phase begins                    */
};

/* What one job means at one sweep point. */
struct JobView {
    uint32_t o, s;
    uint32_t enter; /* first phase the job takes part in                 */
    uint32_t leave; /* last phase it takes part in                       */
    uint32_t done;  /* class of o: the job completes in phases >= done   */
    bool valid;
};

__device__ __forceinline__ JobView view_job(const JobsDev &J, size_t idx, const PointDev &pt)
{
    JobView v;
    int32_t o = J.o[idx];
    int32_t s = J.s ? J.s[idx] : (int32_t)J.s_scalar;
    v.valid = (o >= 1) && (s >= 0) && ((uint32_t)o <= kLenMax) && ((uint32_t)s <= kLenMax) &&
              ((uint64_t)(uint32_t)s + (uint64_t)(uint32_t)o <= J.M);
    v.o = (o < 1) ? 1u : ((uint32_t)o > kLenMax ? kLenMax : (uint32_t)o);
    v.s = (s < 0) ? 0u : ((uint32_t)s > kLenMax ? kLenMax : (uint32_t)s);
    v.done = kvs_class_index(v.o, pt.tau0, pt.lg_tau0);
    if (pt.mode == MODE_SINGLE) {
        v.enter = 0;
        v.leave = 0;
    } else if (pt.mode == MODE_GSA) {
        v.enter = 0;
        v.leave = v.done;
    } else if (J.e) {
        int32_t e = J.e[idx];
        v.valid = v.valid && (e >= 1);
        uint64_t cap = (J.M > v.s) ? (J.M - v.s) : 1u; /* M - s, at least 1 */
        if (cap > kLenMax)
            cap = kLenMax;
        uint32_t eu = (e < 1) ? 1u : (uint32_t)e;
        if (eu > (uint32_t)cap)
            eu = (uint32_t)cap;
        v.enter = kvs_class_index(eu, pt.tau0, pt.lg_tau0);
        v.leave = v.enter > v.done ? v.enter : v.done;
    } else {
        v.enter = v.done;
        v.leave = v.done;
    }
    return v;
}

/* Start offset of the r-th job of a phase: floor(r tau / k) for SPS
 * (Procedure 1), floor(r / k) tau for SimS. */
__device__ __forceinline__ uint32_t start_offset(uint32_t r, const Phase &f, bool sps)
{
    return sps ? kvs_div(r * f.tau, f.div) : kvs_div(r, f.div) * f.tau;
}

/* First r in [0, n] with start_offset(r) >= x. */
__device__ __forceinline__ uint32_t first_rank_at(uint64_t x, const Phase &f, bool sps)
{
    uint64_t r;
    if (sps)
        r = (x * f.k + f.tau - 1) / f.tau; /* floor(r tau / k) >= x  <=>  r >= x k / tau */
    else
        r = ((x + f.tau - 1) / f.tau) * f.k; /* floor(r / k) >= ceil(x / tau) */
    return r > f.n ? f.n : (uint32_t)r;
}

__device__ __forceinline__ int pad_idx(int i) { return i + (i >> 5); }

template <int T, int TW>
__global__ __launch_bounds__(T) void kvs_eval_kernel(JobsDev J, PointsArg P, OutsDev out)
{
    constexpr int NW = T / 64;
    constexpr int E = TW / T;
    constexpr int TWP = TW + TW / 32;
    static_assert(TW % T == 0, "window must be a multiple of the workgroup size");

    extern __shared__ int32_t smem[];
    int32_t *evA = smem;
    int32_t *evC = evA + TWP;
    uint32_t *cd = reinterpret_cast<uint32_t *>(evC + TWP);
    uint32_t *cs = cd + J.n_jobs;

    __shared__ Phase ph[kLevels];
    __shared__ uint32_t hEnter[kLevels], hLeave[kLevels], sMax[kLevels];
    __shared__ uint32_t flags;
    __shared__ uint32_t wtot[2][NW];
    __shared__ int32_t wsA[NW], wsC[NW];
    __shared__ int64_t red[4][NW];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    /* Workgroups g, g+8, g+16, ... share an XCD (and its L2).  All sweep
     * points of one instance are put on the same XCD, next to each other in
     * dispatch order, so the instance's jobs come from HBM once. */
    const uint32_t g = blockIdx.x;
    const uint32_t xcd = g & 7u;
    const uint32_t slot = g >> 3;
    const uint32_t inst = (slot / (uint32_t)P.n) * 8u + xcd;
    const uint32_t q = slot % (uint32_t)P.n;
    if (inst >= (uint32_t)J.n_inst)
        return;

    const PointDev pt = P.p[q];
    const bool sps = (pt.sched == KVS_SCHED_SPS);
    const uint32_t n = (uint32_t)J.n_jobs;
    const size_t row = (size_t)inst * n;
    const bool per_job_s = (J.s != nullptr);

    if (tid < kLevels) {
        hEnter[tid] = 0;
        hLeave[tid] = 0;
        sMax[tid] = 0;
    }
    if (tid == 0)
        flags = 0;
    __syncthreads();

    /* ---- pass 1: how many jobs enter / leave at each level, largest prompt per level ---- */
    for (uint32_t i = tid; i < n; i += T) {
        JobView v = view_job(J, row + i, pt);
        if (!v.valid)
            atomicOr(&flags, FLAG_EINVAL);
        atomicAdd(&hEnter[v.enter], 1u);
        atomicAdd(&hLeave[v.leave], 1u);
        for (uint32_t l = v.enter; l <= v.leave; l++)
            atomicMax(&sMax[l], v.s);
    }
    __syncthreads();

    /* ---- phase table ---- */
    if (tid < kLevels) {
        const uint32_t p = tid;
        uint32_t np = 0;
        for (uint32_t l = 0; l <= p; l++)
            np += hEnter[l];
        for (uint32_t l = 0; l < p; l++)
            np -= hLeave[l];
        Phase f;
        f.n = np;
        f.tau = 0;
        f.k = 1;
        f.H = 0;
        f.div = kvs_make_divisor(1);
        f.begin = 0;
        if (np > 0) {
            const uint64_t tau = (uint64_t)pt.tau0 << p;
            const uint64_t smax = sMax[p];
            if (tau * np >= (1ull << 31)) {
                atomicOr(&flags, FLAG_ERANGE);
                f.n = 0;
            } else {
                uint64_t k;
                if (pt.k > 0)
                    k = pt.k;
                else if (sps)
                    k = kvs_kstar(tau, smax, J.M);
                else
                    k = J.M / (smax + tau);
                if (k < 1)
                    k = 1;
                /* beyond these values the start offsets no longer change */
                const uint64_t kcap = sps ? tau * np : np;
                if (k > kcap)
                    k = kcap;
                const uint64_t act = (k < np) ? k : np;
                if (act * (smax + tau + TW + 1) >= (1ull << 31))
                    atomicOr(&flags, FLAG_ERANGE);
                f.tau = (uint32_t)tau;
                f.k = (uint32_t)k;
                f.div = kvs_make_divisor(f.k);
                f.H = start_offset(np - 1, f, sps) + f.tau;
            }
        }
        ph[p] = f;
    }
    __syncthreads();
    if (tid == 0) {
        int64_t b = 0;
        for (int p = 0; p < kLevels; p++) {
            ph[p].begin = b;
            if (ph[p].n > 0)
                b += ph[p].H;
        }
    }
    __syncthreads();

    int64_t acc_flow = 0, acc_steps = 0;
    int32_t acc_done = 0;
    int32_t pk = 0;
    uint32_t buf = 0;
    const bool bad = (flags != 0);

    for (uint32_t p = 0; p < (uint32_t)kLevels && !bad; p++) {
        const Phase f = ph[p];
        if (f.n == 0)
            continue;

        /* ---- the phase's jobs, in input order, into LDS ---- */
        uint32_t cnt = 0;
        for (uint32_t base = 0; base < n; base += T) {
            const uint32_t i = base + tid;
            bool take = false;
            JobView v;
            if (i < n) {
                v = view_job(J, row + i, pt);
                take = (v.enter <= p) && (p <= v.leave);
            }
            const uint64_t bal = __ballot(take);
            const uint32_t lrank = __popcll(bal & ((1ull << lane) - 1ull));
            if (lane == 0)
                wtot[buf][wave] = (uint32_t)__popcll(bal);
            __syncthreads();
            uint32_t wbase = 0, total = 0;
#pragma unroll
            for (int w = 0; w < NW; w++) {
                const uint32_t c = wtot[buf][w];
                if (w < wave)
                    wbase += c;
                total += c;
            }
            if (take) {
                const uint32_t r = cnt + wbase + lrank;
                const bool completes = (v.done <= p);
                const uint32_t d = completes ? v.o : f.tau;
                cd[r] = d;
                if (per_job_s)
                    cs[r] = v.s;
                acc_steps += d;
                if (completes) {
                    acc_flow += f.begin + (int64_t)start_offset(r, f, sps) + (int64_t)v.o;
                    acc_done += 1;
                }
            }
            cnt += total;
            buf ^= 1u;
        }
        __syncthreads();

        /* ---- occupancy of every round of the phase, one window at a time ---- */
        int32_t carryA = 0, carryC = 0;
        for (uint64_t t0 = 0; t0 < f.H; t0 += TW) {
#pragma unroll
            for (int j = 0; j < E; j++) {
                evA[pad_idx(tid + j * T)] = 0;
                evC[pad_idx(tid + j * T)] = 0;
            }
            __syncthreads();

            const uint64_t back = (t0 > f.tau) ? (t0 - f.tau) : 0;
            const uint32_t r_lo = first_rank_at(back, f, sps);
            const uint32_t r_hi = first_rank_at(t0 + TW, f, sps);
            for (uint32_t r = r_lo + tid; r < r_hi; r += T) {
                const int32_t st = (int32_t)((int64_t)start_offset(r, f, sps) - (int64_t)t0);
                const int32_t d = (int32_t)cd[r];
                const int32_t s = per_job_s ? (int32_t)cs[r] : (int32_t)J.s_scalar;
                const int32_t w = s + 1 - st;
                if ((uint32_t)st < (uint32_t)TW) {
                    atomicAdd(&evA[pad_idx(st)], w);
                    atomicAdd(&evC[pad_idx(st)], 1);
                }
                const int32_t en = st + d;
                if ((uint32_t)en < (uint32_t)TW) {
                    atomicAdd(&evA[pad_idx(en)], -w);
                    atomicAdd(&evC[pad_idx(en)], -1);
                }
            }
            __syncthreads();

            int32_t a[E], c[E];
            int32_t la = 0, lc = 0;
#pragma unroll
            for (int j = 0; j < E; j++) {
                a[j] = evA[pad_idx(tid * E + j)];
                c[j] = evC[pad_idx(tid * E + j)];
                la += a[j];
                lc += c[j];
            }
            int32_t va = la, vc = lc;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int32_t ua = __shfl_up(va, off);
                const int32_t uc = __shfl_up(vc, off);
                if (lane >= off) {
                    va += ua;
                    vc += uc;
                }
            }
            if (lane == 63) {
                wsA[wave] = va;
                wsC[wave] = vc;
            }
            __syncthreads();
            int32_t ba = 0, bc = 0, ta = 0, tc = 0;
#pragma unroll
            for (int w = 0; w < NW; w++) {
                const int32_t xa = wsA[w], xc = wsC[w];
                if (w < wave) {
                    ba += xa;
                    bc += xc;
                }
                ta += xa;
                tc += xc;
            }
            int32_t A = carryA + ba + va - la;
            int32_t C = carryC + bc + vc - lc;
            const uint64_t left = f.H - t0; /* rounds of the phase from t0 on */
#pragma unroll
            for (int j = 0; j < E; j++) {
                const int32_t t = tid * E + j;
                A += a[j];
                C += c[j];
                const int32_t occ = A + t * C;
                if ((uint64_t)t < left && occ > pk)
                    pk = occ;
            }
            /* the next window measures time from t0 + TW */
            carryC += tc;
            carryA += ta + TW * carryC;
            __syncthreads();
        }
    }

    /* ---- workgroup reduction and store ---- */
    int64_t r_pk = pk, r_flow = acc_flow, r_steps = acc_steps, r_done = acc_done;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const int64_t o_pk = __shfl_down(r_pk, off);
        r_pk = o_pk > r_pk ? o_pk : r_pk;
        r_flow += __shfl_down(r_flow, off);
        r_steps += __shfl_down(r_steps, off);
        r_done += __shfl_down(r_done, off);
    }
    if (lane == 0) {
        red[0][wave] = r_pk;
        red[1][wave] = r_flow;
        red[2][wave] = r_steps;
        red[3][wave] = r_done;
    }
    __syncthreads();
    if (tid == 0) {
        int64_t peak = 0, flow = 0, steps = 0, done = 0;
        for (int w = 0; w < NW; w++) {
            peak = red[0][w] > peak ? red[0][w] : peak;
            flow += red[1][w];
            steps += red[2][w];
            done += red[3][w];
        }
        uint8_t feas = (peak <= (int64_t)J.M) ? 1 : 0;
        if (flags & FLAG_EINVAL) {
            feas = KVS_FEASIBLE_EINVAL;
        } else if (flags & FLAG_ERANGE) {
            feas = KVS_FEASIBLE_ERANGE;
        }
        if (flags) {
            peak = -1;
            flow = -1;
            steps = -1;
            done = -1;
        }
        const size_t oi = (size_t)q * (size_t)J.n_inst + inst;
        out.peak[oi] = peak;
        out.feasible[oi] = feas;
        out.flow[oi] = flow;
        if (out.job_steps)
            out.job_steps[oi] = steps;
        if (out.n_completed)
            out.n_completed[oi] = (int32_t)done;
    }
}

/* ---- input scan for kvs_validate ---- */
struct ValidateResult {
    uint32_t bad_value; /* o < 1, s < 0 or o_est < 1 */
    uint32_t too_long;  /* a length above 2^30       */
    uint32_t infeasible; /* s + o > M                */
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

/* ---- host side ---- */

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
    return J;
}

template <int T, int TW>
int32_t launch_eval(const JobsDev &J, const PointsArg &P, const OutsDev &out, hipStream_t st)
{
    constexpr int TWP = TW + TW / 32;
    const size_t lds = sizeof(int32_t) * (2 * (size_t)TWP + (size_t)J.n_jobs * (J.s ? 2 : 1));
    auto kern = kvs_eval_kernel<T, TW>;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return KVS_EHIP;
    const uint64_t groups = ((uint64_t)(J.n_inst + 7) / 8) * 8 * (uint64_t)P.n;
    if (groups > 0x7fffffffull)
        return KVS_ELIMIT;
    hipLaunchKernelGGL(kern, dim3((uint32_t)groups), dim3(T), lds, st, J, P, out);
    return hipGetLastError() == hipSuccess ? KVS_OK : KVS_EHIP;
}

int32_t run_eval(const JobsDev &J, const PointsArg &P, const OutsDev &out, hipStream_t st)
{
    if (J.n_jobs <= 2048)
        return launch_eval<256, 2048>(J, P, out, st);
    return launch_eval<1024, 4096>(J, P, out, st);
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
    PointsArg P;
    P.n = n_pts;
    for (int32_t q = 0; q < n_pts; q++) {
        const kvs_point_t &p = pts[q];
        if (p.tau0 < 1 || (uint32_t)p.tau0 > kLenMax || p.k < 0 ||
            (p.sched != KVS_SCHED_SPS && p.sched != KVS_SCHED_SIMS) ||
            (p.mode != KVS_MODE_GBA && p.mode != KVS_MODE_GSA))
            return KVS_EINVAL;
        P.p[q].tau0 = (uint32_t)p.tau0;
        P.p[q].k = (uint32_t)p.k;
        P.p[q].sched = (uint8_t)p.sched;
        P.p[q].mode = (uint8_t)(p.mode == KVS_MODE_GSA ? MODE_GSA : MODE_GBA);
        P.p[q].lg_tau0 = (uint8_t)kvs_ilog2_floor((uint32_t)p.tau0);
        P.p[q].pad = 0;
    }
    OutsDev out{peak, feasible, flow, job_steps, nullptr};
    return run_eval(to_dev(jobs, true), P, out, static_cast<hipStream_t>(stream));
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
    PointsArg P;
    P.n = n_pts;
    for (int32_t q = 0; q < n_pts; q++) {
        if (tau[q] < 1 || (uint32_t)tau[q] > kLenMax || k[q] < 0 ||
            (sched[q] != KVS_SCHED_SPS && sched[q] != KVS_SCHED_SIMS))
            return KVS_EINVAL;
        P.p[q].tau0 = (uint32_t)tau[q];
        P.p[q].k = (uint32_t)k[q];
        P.p[q].sched = (uint8_t)sched[q];
        P.p[q].mode = (uint8_t)MODE_SINGLE;
        P.p[q].lg_tau0 = (uint8_t)kvs_ilog2_floor((uint32_t)tau[q]);
        P.p[q].pad = 0;
    }
    OutsDev out{peak, feasible, flow, job_steps, n_completed};
    return run_eval(to_dev(jobs, false), P, out, static_cast<hipStream_t>(stream));
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

int32_t kvs_version(void) { return 100; }

/* Host evaluation of the kernels' integer helpers, for the host-side tests. */
uint32_t kvs_host_class_index(uint32_t x, uint32_t tau0)
{
    return kvs_class_index(x, tau0, kvs_ilog2_floor(tau0));
}

uint32_t kvs_host_div(uint32_t x, uint32_t d) { return kvs_div(x, kvs_make_divisor(d)); }

uint64_t kvs_host_kstar(uint64_t tau, uint64_t s, uint64_t M) { return kvs_kstar(tau, s, M); }

} /* extern "C" */
