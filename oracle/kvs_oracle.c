/*
 * kvs_oracle.c -- CPU oracle for KV-cache schedule evaluation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * reference against which the GPU library is checked.  It is used by the
 * tests, by the smoke check and by the CPU-baseline leg of the benchmark, and
 * by nothing else; the product path never calls it.  It shares no code,
 * header, table or helper with the GPU sources.
 *
 * Everything here follows "Competitive Non-Clairvoyant KV-Cache Scheduling for
 * LLM Inference" (Feng, Yang, Zhang).  Citations name the section, equation,
 * lemma, procedure or algorithm of that paper.
 *
 *   - the discrete-time model, the occupancy of a round and the flow time:
 *     Section 2.1 ("Model and Objective"), eq. (Memory-Feasibility);
 *   - Staggered-Pipeline-Schedule (SPS): Procedure 1;
 *   - Simultaneous-Schedule (SimS): Appendix "Lower Bounds for SimS";
 *   - Peak(k, tau, s) and k*(tau, s): Lemma "Peak Memory Usage of SPS" and
 *     Lemma "Feasible Parallelism of SPS", eq. (max-parallelism);
 *   - Geometric-Slicing-Algorithm (GSA): Algorithm 1;
 *   - Geometric-Batching-Algorithm (GBA): Algorithm 2;
 *   - memory-time area: Definition "Memory-Time Area";
 *   - dynamic refill (GBA-D): appendix "Numerical Experiments", paragraph
 *     "Dynamic Refill";
 *   - OPT: Section 2.1 ("Objective and Benchmark") and its footnote that
 *     neither preemption nor pausing is needed in an optimal schedule.
 *
 * Readings taken where the paper is silent: scaling factor alpha = 2 and an integer initial slice tau_0,
 * so that tau_p = tau_0 * 2^p exactly; jobs inside a phase keep input order;
 * a phase lasts until the scheduled end of its last slice and an empty phase
 * takes no time; with per-job prompt lengths the phase uses the largest
 * prompt among its participants in Peak / in the SimS batch size; when an
 * estimate is given a job enters the first phase whose slice covers the
 * estimate, is killed at slice end while its true length exceeds the slice
 * and re-enters the next phase (Procedure 1's kill rule with Algorithm 1's
 * "keep the unfinished jobs").
 *
 * What pins what (tests/test_oracle_pins.py).  The stepper, SPS, SimS and
 * k*: the printed values of the toy example (180, 225, peak 15), the Peak
 * lemma against the stepped peak, the identical-jobs flow identity.  The
 * phase driver in GBA and GSA mode: the printed 14083 and 21632 of the uniform
 * experiment, the long-job closed form, the two-point experiment's bracket, a
 * second driver written independently, the ratio theorems against exhaustive
 * search.  The ladder of Algorithms 1 and 2: exact rational arithmetic.  The
 * bounds (kvo_upper_gba, kvo_area_lb): printed values, hand examples, the
 * lemmas as inequalities against the stepped flow and the exhaustive optimum.
 * Algorithm 2 with dynamic refill (kvo_gbad_simulate): hand-worked cases, a
 * second implementation, the paper's claims about it (no job later than in
 * Algorithm 2's schedule, within the budget) and the toy example, where
 * nothing can move (180).
 * Parity unpinned by anything the paper prints: the refill rule itself (one
 * sentence in the appendix; the reading is stated at the function); the treatment of estimates
 * other than the two ends (estimate = true length, estimate = 1) to which it
 * reduces; per-job prompt lengths (only the invariant MemPeak <= M); the
 * order of the jobs inside a phase; a job shorter than its slice leaving the
 * later starts where they are.
 *
 * All quantities are integers (tokens, rounds); 64-bit throughout.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KVO_OK 0
#define KVO_EINVAL 1
#define KVO_EJOB_INFEASIBLE 2
#define KVO_ENOMEM 3

/* ------------------------------------------------------------------------ */
/* Closed forms                                                              */
/* ------------------------------------------------------------------------ */

static int64_t gcd64(int64_t a, int64_t b)
{
    while (b != 0) {
        int64_t r = a % b;
        a = b;
        b = r;
    }
    return a;
}

/* Lemma "Peak Memory Usage of SPS":
 *   Peak(k, tau, s) = s*k + (tau*k + tau + k - gcd(tau, k)) / 2.
 * The bracket is always even (it is twice a count of lattice points). */
int64_t kvo_peak_formula(int64_t k, int64_t tau, int64_t s)
{
    return s * k + (tau * k + tau + k - gcd64(tau, k)) / 2;
}

/* eq. (max-parallelism): k*(tau, s) = max{k in N : Peak(k, tau, s) <= M}.
 * Peak is increasing in k (same lemma), so the set is an initial segment of
 * the naturals and an upward scan finds its maximum.  Returns 0 when even
 * k = 1 does not fit. */
int64_t kvo_kstar(int64_t tau, int64_t s, int64_t M)
{
    int64_t k = 0;
    while (kvo_peak_formula(k + 1, tau, s) <= M)
        k++;
    return k;
}

/* Definition "Memory-Time Area": A(o, s) = s*o + o*(o+1)/2. */
int64_t kvo_area(int64_t o, int64_t s)
{
    return s * o + o * (o + 1) / 2;
}

/* ------------------------------------------------------------------------ */
/* The model of Section 2.1, stepped one round at a time                     */
/* ------------------------------------------------------------------------ */

typedef struct {
    int64_t start; /* round in which the run is started (progress 0)        */
    int64_t dur;   /* rounds it stays active: completes or is killed after  */
    int64_t s;     /* prompt length of the job                              */
} kvo_run_t;

/*
 * Steps a set of runs through the rounds t = 0, 1, 2, ...  `runs` must be in
 * non-decreasing order of start.  In round t every active job with progress
 * u occupies s + u + 1 units (prompt, decoded tokens and the token being
 * decoded), the round's occupancy is the sum over the active batch
 * (eq. (Memory-Feasibility)), and every active job then receives one unit of
 * processing.  A run leaves the batch at the start of the round in which its
 * progress has reached `dur`.
 *
 * peak      = max over rounds of the occupancy (0 without runs)
 * job_steps = number of (job, round) pairs processed = sum of dur
 */
static int step_runs(const kvo_run_t *runs, int64_t n_runs, int64_t *peak,
                     int64_t *job_steps)
{
    int64_t *as = NULL, *au = NULL, *ad = NULL;
    int64_t na = 0, next = 0, t = 0, pk = 0, steps = 0;
    int64_t i, w;

    if (n_runs > 0) {
        as = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_runs);
        au = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_runs);
        ad = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_runs);
        if (!as || !au || !ad) {
            free(as); free(au); free(ad);
            return KVO_ENOMEM;
        }
    }
    for (i = 1; i < n_runs; i++)
        if (runs[i].start < runs[i - 1].start) {
            free(as); free(au); free(ad);
            return KVO_EINVAL;
        }

    while (next < n_runs || na > 0) {
        int64_t occ = 0;
        /* (Start) actions of round t */
        while (next < n_runs && runs[next].start == t) {
            as[na] = runs[next].s;
            au[na] = 0;
            ad[na] = runs[next].dur;
            na++;
            next++;
        }
        /* occupancy of round t */
        for (i = 0; i < na; i++)
            occ += as[i] + au[i] + 1;
        if (occ > pk)
            pk = occ;
        /* one unit of processing for every active job */
        for (i = 0; i < na; i++) {
            au[i] += 1;
            steps += 1;
        }
        /* jobs that are complete, or killed, leave before round t+1 */
        w = 0;
        for (i = 0; i < na; i++)
            if (au[i] < ad[i]) {
                as[w] = as[i];
                au[w] = au[i];
                ad[w] = ad[i];
                w++;
            }
        na = w;
        t++;
    }
    free(as); free(au); free(ad);
    *peak = pk;
    *job_steps = steps;
    return KVO_OK;
}

/* Exposed for tests: occupancy peak and job-steps of explicit runs. */
int kvo_step_runs(int64_t n_runs, const int64_t *start, const int64_t *dur,
                  const int64_t *s, int64_t *peak, int64_t *job_steps)
{
    kvo_run_t *runs;
    int64_t i;
    int rc;
    if (n_runs < 0)
        return KVO_EINVAL;
    runs = (kvo_run_t *)malloc(sizeof(kvo_run_t) * (size_t)(n_runs > 0 ? n_runs : 1));
    if (!runs)
        return KVO_ENOMEM;
    for (i = 0; i < n_runs; i++) {
        runs[i].start = start[i];
        runs[i].dur = dur[i];
        runs[i].s = s[i];
    }
    rc = step_runs(runs, n_runs, peak, job_steps);
    free(runs);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Per-phase subroutines: Procedure 1 (SPS) and SimS                         */
/* ------------------------------------------------------------------------ */

#define KVO_SPS 0
#define KVO_SIMS 1

/* Parallelism used by a phase with slice tau whose participants have largest
 * prompt s_max.  SPS: k*(tau, s_max) of eq. (max-parallelism).  SimS: batch
 * size floor(M / (s + o)) with the slice in the role of o.  A forced value
 * k_forced > 0 replaces either.  Never below 1. */
static int64_t phase_parallelism(int sched, int64_t tau, int64_t s_max,
                                 int64_t M, int64_t k_forced)
{
    int64_t k;
    if (k_forced > 0)
        return k_forced;
    if (sched == KVO_SPS)
        k = kvo_kstar(tau, s_max, M);
    else
        k = M / (s_max + tau);
    return k < 1 ? 1 : k;
}

/* Start offset of the job with index r of the phase's sequence.
 * SPS (Procedure 1): floor(r * tau / k).
 * SimS: batches of k jobs, one batch after the other, each tau rounds. */
static int64_t start_offset(int sched, int64_t r, int64_t tau, int64_t k)
{
    if (sched == KVO_SPS)
        return (r * tau) / k;
    return (r / k) * tau;
}

/*
 * One invocation of the subroutine on the whole job sequence with explicit
 * slice tau and parallelism k (k = 0: the memory-feasible maximum for the
 * largest prompt).  Job r starts at its offset and runs in [start, start+tau);
 * a job with o_r <= tau completes at start + o_r, any other is killed when
 * its slice ends and does not count towards the flow time.
 */
int kvo_schedule_eval(int64_t n, const int32_t *o, const int32_t *s,
                      int64_t s_scalar, int64_t M, int64_t tau, int64_t k,
                      int sched, int64_t *peak, int32_t *feasible,
                      int64_t *flow, int64_t *n_completed, int64_t *job_steps)
{
    kvo_run_t *runs;
    int64_t r, s_max = 0, kk, fl = 0, nc = 0;
    int rc;

    if (n < 0 || M <= 0 || tau < 1 || k < 0 || (sched != KVO_SPS && sched != KVO_SIMS))
        return KVO_EINVAL;
    for (r = 0; r < n; r++) {
        int64_t sr = s ? s[r] : s_scalar;
        if (o[r] < 1 || sr < 0)
            return KVO_EINVAL;
        if (sr + o[r] > M)
            return KVO_EJOB_INFEASIBLE;
        if (sr > s_max)
            s_max = sr;
    }
    runs = (kvo_run_t *)malloc(sizeof(kvo_run_t) * (size_t)(n > 0 ? n : 1));
    if (!runs)
        return KVO_ENOMEM;
    kk = phase_parallelism(sched, tau, s_max, M, k);
    for (r = 0; r < n; r++) {
        runs[r].start = start_offset(sched, r, tau, kk);
        runs[r].s = s ? s[r] : s_scalar;
        if (o[r] <= tau) {
            runs[r].dur = o[r];
            fl += runs[r].start + o[r];
            nc++;
        } else {
            runs[r].dur = tau;
        }
    }
    rc = step_runs(runs, n, peak, job_steps);
    free(runs);
    if (rc != KVO_OK)
        return rc;
    *feasible = (*peak <= M) ? 1 : 0;
    *flow = fl;
    *n_completed = nc;
    return KVO_OK;
}

/* ------------------------------------------------------------------------ */
/* Geometric phases: Algorithm 2 (GBA), Algorithm 1 (GSA), and the           */
/* estimate-driven interpolation between the two                             */
/* ------------------------------------------------------------------------ */

#define KVO_MODE_GBA 0 /* class by o_est (by o itself when o_est is NULL)   */
#define KVO_MODE_GSA 1 /* every unfinished job takes part in every phase    */

/*
 * Evaluates one instance at one sweep point.
 *
 * Phases p = 0, 1, ... use the slice tau_p = tau_0 * 2^p.  The set T of
 * unfinished jobs starts as all jobs.  Phase p invokes the subroutine on
 *     J_p = { i in T : e_i <= tau_p }            (input order)
 * where e_i is the length the scheduler believes: o_i itself (Algorithm 2),
 * the estimate o_est_i clamped to [1, M - s_i], or 1 in GSA mode, which makes
 * J_p = T (Algorithm 1).  A participant with o_i <= tau_p completes at
 * start + o_i and leaves T; any other is killed at the end of its slice and
 * stays in T.  The next phase begins when the last slice of this one ends.
 *
 * All runs of all phases are then stepped round by round for the occupancy
 * peak; the flow time is the sum of the completion rounds.
 */
static int phase_driver(int64_t n, const int32_t *o, const int32_t *s,
                        const int32_t *o_est, int64_t s_scalar, int64_t M,
                        int64_t tau0, const int32_t *ladder, int64_t n_levels,
                        int sched, int64_t k, int mode,
                        int64_t *peak, int32_t *feasible, int64_t *flow,
                        int64_t *job_steps, int64_t *n_phases_used)
{
    kvo_run_t *runs = NULL;
    int64_t cap = 0, nr = 0;
    int64_t *e = NULL;
    uint8_t *in_T = NULL;
    int64_t *J = NULL;
    int64_t i, left, begin = 0, fl = 0, phases_used = 0;
    int p, rc;

    if (n < 0 || M <= 0 || tau0 < 1 || k < 0 ||
        (sched != KVO_SPS && sched != KVO_SIMS) ||
        (mode != KVO_MODE_GBA && mode != KVO_MODE_GSA))
        return KVO_EINVAL;
    for (i = 0; i < n; i++) {
        int64_t si = s ? s[i] : s_scalar;
        if (o[i] < 1 || si < 0 || (o_est && o_est[i] < 1))
            return KVO_EINVAL;
        if (si + o[i] > M) /* per-job feasibility, Section 2.1 */
            return KVO_EJOB_INFEASIBLE;
    }

    e = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    in_T = (uint8_t *)malloc((size_t)(n > 0 ? n : 1));
    J = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    if (!e || !in_T || !J) {
        free(e); free(in_T); free(J);
        return KVO_ENOMEM;
    }
    for (i = 0; i < n; i++) {
        int64_t si = s ? s[i] : s_scalar;
        if (mode == KVO_MODE_GSA)
            e[i] = 1;
        else if (o_est) {
            e[i] = o_est[i];
            if (e[i] > M - si)
                e[i] = M - si;
            if (e[i] < 1)
                e[i] = 1;
        } else
            e[i] = o[i];
        in_T[i] = 1;
    }

    left = n;
    rc = KVO_OK;
    for (p = 0; left > 0; p++) {
        int64_t tau, nJ = 0, s_max = 0, kk, r;
        if (ladder) {
            if (p >= n_levels) { /* a job that no slice of the ladder covers */
                rc = KVO_EINVAL;
                break;
            }
            tau = ladder[p];
        } else {
            if (p > 40) { /* tau_0 * 2^40 exceeds any int32 length */
                rc = KVO_EINVAL;
                break;
            }
            tau = tau0 << p;
        }
        for (i = 0; i < n; i++)
            if (in_T[i] && e[i] <= tau)
                J[nJ++] = i;
        if (nJ == 0)
            continue; /* an empty class takes no time */
        phases_used++;
        for (r = 0; r < nJ; r++) {
            int64_t si = s ? s[J[r]] : s_scalar;
            if (si > s_max)
                s_max = si;
        }
        kk = phase_parallelism(sched, tau, s_max, M, k);
        if (nr + nJ > cap) {
            int64_t ncap = cap ? cap * 2 : 1024;
            kvo_run_t *nrs;
            while (ncap < nr + nJ)
                ncap *= 2;
            nrs = (kvo_run_t *)realloc(runs, sizeof(kvo_run_t) * (size_t)ncap);
            if (!nrs) {
                rc = KVO_ENOMEM;
                break;
            }
            runs = nrs;
            cap = ncap;
        }
        for (r = 0; r < nJ; r++) {
            int64_t j = J[r];
            int64_t st = begin + start_offset(sched, r, tau, kk);
            runs[nr].start = st;
            runs[nr].s = s ? s[j] : s_scalar;
            if (o[j] <= tau) {
                runs[nr].dur = o[j];
                fl += st + o[j]; /* completion round c_j */
                in_T[j] = 0;
                left--;
            } else {
                runs[nr].dur = tau; /* killed when the slice ends */
            }
            nr++;
        }
        begin += start_offset(sched, nJ - 1, tau, kk) + tau;
    }

    if (rc == KVO_OK)
        rc = step_runs(runs, nr, peak, job_steps);
    free(runs); free(e); free(in_T); free(J);
    if (rc != KVO_OK)
        return rc;
    *feasible = (*peak <= M) ? 1 : 0;
    *flow = fl;
    if (n_phases_used)
        *n_phases_used = phases_used;
    return KVO_OK;
}

/* Slices tau_p = tau_0 * 2^p (scaling factor 2, integer initial slice). */
int kvo_gba_simulate(int64_t n, const int32_t *o, const int32_t *s,
                     const int32_t *o_est, int64_t s_scalar, int64_t M,
                     int64_t tau0, int sched, int64_t k, int mode,
                     int64_t *peak, int32_t *feasible, int64_t *flow,
                     int64_t *job_steps, int64_t *n_phases_used)
{
    return phase_driver(n, o, s, o_est, s_scalar, M, tau0, NULL, 0, sched, k,
                        mode, peak, feasible, flow, job_steps, n_phases_used);
}

/* Slices given one by one: ladder[0] <= ladder[1] <= ... (n_levels of them),
 * e.g. tau_p = floor(beta alpha^p) for any scaling factor alpha. */
int kvo_ladder_simulate(int64_t n, const int32_t *o, const int32_t *s,
                        const int32_t *o_est, int64_t s_scalar, int64_t M,
                        const int32_t *ladder, int64_t n_levels, int sched,
                        int64_t k, int mode, int64_t *peak, int32_t *feasible,
                        int64_t *flow, int64_t *job_steps,
                        int64_t *n_phases_used)
{
    int64_t p;
    if (!ladder || n_levels < 1 || ladder[0] < 1)
        return KVO_EINVAL;
    for (p = 1; p < n_levels; p++)
        if (ladder[p] < ladder[p - 1])
            return KVO_EINVAL;
    return phase_driver(n, o, s, o_est, s_scalar, M, 1, ladder, n_levels, sched,
                        k, mode, peak, feasible, flow, job_steps,
                        n_phases_used);
}

/*
 * The initialisation of Algorithms 1 and 2 for a rational scaling factor
 * alpha = num / den > 1 and a common prompt length s:
 *   l = floor(log_alpha(M - s)), beta = (M - s) / alpha^l,
 *   tau_p = floor(beta alpha^p) for p = 0 .. l.
 * Exact: beta alpha^p = (M - s) * (den/num)^(l-p), and the powers are kept as
 * 128-bit integers.  Returns the number of levels l + 1, or -1 when more than
 * max_levels are needed or a power leaves the 128-bit range.
 */
int64_t kvo_paper_ladder(int64_t M, int64_t s, int64_t num, int64_t den,
                         int32_t *ladder, int64_t max_levels)
{
    unsigned __int128 span, top = ((unsigned __int128)1) << 126;
    unsigned __int128 pow_num[130], pow_den[130];
    int64_t l, p;
    if (M <= s || s < 0 || den < 1 || num <= den)
        return -1;
    span = (unsigned __int128)(M - s);
    pow_num[0] = 1;
    pow_den[0] = 1;
    /* largest l with alpha^l <= M - s, i.e. num^l <= (M - s) den^l */
    for (l = 0;; l++) {
        /* the next powers, and (M - s) times the power of den, must stay below 2^126 */
        if (l + 1 >= 129 || pow_num[l] > top / (unsigned __int128)num ||
            pow_den[l] > top / ((unsigned __int128)den * span))
            return -1;
        pow_num[l + 1] = pow_num[l] * (unsigned __int128)num;
        pow_den[l + 1] = pow_den[l] * (unsigned __int128)den;
        if (pow_num[l + 1] > span * pow_den[l + 1])
            break;
    }
    if (l + 1 > max_levels)
        return -1;
    for (p = 0; p <= l; p++)
        ladder[p] = (int32_t)((span * pow_den[l - p]) / pow_num[l - p]);
    return l + 1;
}

/* Batch form used by the parity tests and the CPU-baseline timing: instances
 * [i0, i1) of row-major [n_instances][n] arrays at every sweep point; outputs
 * are [n_pts][i1 - i0].  Stops at the first error. */
int kvo_gba_simulate_batch(int64_t i0, int64_t i1, int64_t n,
                           const int32_t *o, const int32_t *s,
                           const int32_t *o_est, int64_t s_scalar, int64_t M,
                           int64_t n_pts, const int32_t *tau0,
                           const int32_t *sched, const int32_t *k,
                           const int32_t *mode, int64_t *peak,
                           uint8_t *feasible, int64_t *flow,
                           int64_t *job_steps)
{
    int64_t q, i, cnt = i1 - i0;
    for (q = 0; q < n_pts; q++)
        for (i = i0; i < i1; i++) {
            int32_t feas = 0;
            int64_t idx = q * cnt + (i - i0);
            int rc = kvo_gba_simulate(n, o + i * n, s ? s + i * n : NULL,
                                      o_est ? o_est + i * n : NULL, s_scalar,
                                      M, tau0[q], sched[q], k[q], mode[q],
                                      &peak[idx], &feas, &flow[idx],
                                      &job_steps[idx], NULL);
            if (rc != KVO_OK)
                return rc;
            feasible[idx] = (uint8_t)feas;
        }
    return KVO_OK;
}

/* Same for explicit ladders: ladders is [n_pts][stride]. */
int kvo_ladder_simulate_batch(int64_t i0, int64_t i1, int64_t n,
                              const int32_t *o, const int32_t *s,
                              const int32_t *o_est, int64_t s_scalar, int64_t M,
                              int64_t n_pts, const int32_t *ladders,
                              int64_t stride, const int32_t *n_levels,
                              const int32_t *sched, const int32_t *k,
                              const int32_t *mode, int64_t *peak,
                              uint8_t *feasible, int64_t *flow,
                              int64_t *job_steps)
{
    int64_t q, i, cnt = i1 - i0;
    for (q = 0; q < n_pts; q++)
        for (i = i0; i < i1; i++) {
            int32_t feas = 0;
            int64_t idx = q * cnt + (i - i0);
            int rc = kvo_ladder_simulate(n, o + i * n, s ? s + i * n : NULL,
                                         o_est ? o_est + i * n : NULL, s_scalar,
                                         M, ladders + q * stride, n_levels[q],
                                         sched[q], k[q], mode[q], &peak[idx],
                                         &feas, &flow[idx], &job_steps[idx], NULL);
            if (rc != KVO_OK)
                return rc;
            feasible[idx] = (uint8_t)feas;
        }
    return KVO_OK;
}

int kvo_schedule_eval_batch(int64_t i0, int64_t i1, int64_t n,
                            const int32_t *o, const int32_t *s,
                            int64_t s_scalar, int64_t M, int64_t n_pts,
                            const int32_t *tau, const int32_t *k,
                            const int32_t *sched, int64_t *peak,
                            uint8_t *feasible, int64_t *flow,
                            int32_t *n_completed, int64_t *job_steps)
{
    int64_t q, i, cnt = i1 - i0;
    for (q = 0; q < n_pts; q++)
        for (i = i0; i < i1; i++) {
            int32_t feas = 0;
            int64_t nc = 0;
            int64_t idx = q * cnt + (i - i0);
            int rc = kvo_schedule_eval(n, o + i * n, s ? s + i * n : NULL,
                                       s_scalar, M, tau[q], k[q], sched[q],
                                       &peak[idx], &feas, &flow[idx], &nc,
                                       &job_steps[idx]);
            if (rc != KVO_OK)
                return rc;
            feasible[idx] = (uint8_t)feas;
            n_completed[idx] = (int32_t)nc;
        }
    return KVO_OK;
}

/* ------------------------------------------------------------------------ */
/* OPT by brute force (tiny instances only)                                  */
/* ------------------------------------------------------------------------ */

/* A schedule without kills or pauses is a vector of start rounds; job i then
 * occupies s + (t - S_i) + 1 in the rounds S_i <= t < S_i + o_i and completes
 * at S_i + o_i (Section 2.1; the footnote on OPT says such schedules
 * suffice).  occ[] holds the occupancy already committed per round. */

static int fits(const int64_t *occ, int64_t horizon, int64_t S, int64_t o,
                int64_t s, int64_t M)
{
    int64_t t;
    if (S + o > horizon)
        return 0;
    for (t = S; t < S + o; t++)
        if (occ[t] + s + (t - S) + 1 > M)
            return 0;
    return 1;
}

static void place(int64_t *occ, int64_t S, int64_t o, int64_t s, int64_t sign)
{
    int64_t t;
    for (t = S; t < S + o; t++)
        occ[t] += sign * (s + (t - S) + 1);
}

/*
 * Minimum over all n! orders of the list schedule that starts the jobs in
 * that order, each at the earliest round, not before its predecessor's
 * start, at which its whole trajectory fits on top of the jobs already
 * placed.  An upper bound on OPT (it is a feasible schedule) that is exact on
 * many tiny instances; kvo_opt_exact below is the true optimum.
 */
int kvo_opt_perm(int64_t n, const int32_t *o, int64_t s, int64_t M,
                 int64_t *best_flow)
{
    int64_t horizon = 0, i, best = -1;
    int64_t *occ;
    int perm[16], c[16];
    if (n < 1 || n > 10)
        return KVO_EINVAL;
    for (i = 0; i < n; i++) {
        if (o[i] < 1 || s + o[i] > M)
            return KVO_EJOB_INFEASIBLE;
        horizon += o[i];
    }
    occ = (int64_t *)calloc((size_t)horizon + 1, sizeof(int64_t));
    if (!occ)
        return KVO_ENOMEM;
    for (i = 0; i < n; i++) {
        perm[i] = (int)i;
        c[i] = 0;
    }
    /* Heap's algorithm, non-recursive, visits every permutation once. */
    i = 0;
    for (;;) {
        /* evaluate perm */
        {
            int64_t prev = 0, fl = 0, j;
            int64_t S_of[16];
            for (j = 0; j < n; j++) {
                int64_t oj = o[perm[j]];
                int64_t S = prev;
                while (!fits(occ, horizon, S, oj, s, M))
                    S++; /* running alone after everything else always fits */
                place(occ, S, oj, s, +1);
                S_of[j] = S;
                prev = S;
                fl += S + oj;
            }
            for (j = 0; j < n; j++)
                place(occ, S_of[j], o[perm[j]], s, -1);
            if (best < 0 || fl < best)
                best = fl;
        }
        /* next permutation */
        while (i < n) {
            if (c[i] < i) {
                int a = (i % 2 == 0) ? 0 : c[i];
                int tmp = perm[a];
                perm[a] = perm[i];
                perm[i] = tmp;
                c[i]++;
                i = 0;
                break;
            }
            c[i] = 0;
            i++;
        }
        if (i >= n)
            break;
    }
    free(occ);
    *best_flow = best;
    return KVO_OK;
}

typedef struct {
    int64_t n, s, M, horizon, best;
    const int32_t *o;
    int64_t *occ;
} dfs_t;

static void dfs_exact(dfs_t *d, int64_t j, int64_t flow_so_far)
{
    int64_t S, oj, rest = 0, q;
    if (j == d->n) {
        if (d->best < 0 || flow_so_far < d->best)
            d->best = flow_so_far;
        return;
    }
    oj = d->o[j];
    for (q = j + 1; q < d->n; q++)
        rest += d->o[q]; /* every later job completes no earlier than o_q */
    for (S = 0; S + oj <= d->horizon; S++) {
        if (d->best >= 0 && flow_so_far + S + oj + rest >= d->best)
            break; /* larger S only costs more */
        if (!fits(d->occ, d->horizon, S, oj, d->s, d->M))
            continue;
        place(d->occ, S, oj, d->s, +1);
        dfs_exact(d, j + 1, flow_so_far + S + oj);
        place(d->occ, S, oj, d->s, -1);
    }
}

/* True optimum over every vector of start rounds in [0, sum o): exhaustive
 * depth-first search with a cost bound.  An optimal schedule has no round
 * without an active job before its last completion (shifting the rest one
 * round earlier would keep it feasible and lower the flow time), so its last
 * completion is at most sum(o) and the horizon loses nothing. */
int kvo_opt_exact(int64_t n, const int32_t *o, int64_t s, int64_t M,
                  int64_t *best_flow)
{
    dfs_t d;
    int64_t i;
    if (n < 1 || n > 8)
        return KVO_EINVAL;
    d.n = n; d.s = s; d.M = M; d.o = o; d.best = -1; d.horizon = 0;
    for (i = 0; i < n; i++) {
        if (o[i] < 1 || s + o[i] > M)
            return KVO_EJOB_INFEASIBLE;
        d.horizon += o[i];
    }
    d.occ = (int64_t *)calloc((size_t)d.horizon + 1, sizeof(int64_t));
    if (!d.occ)
        return KVO_ENOMEM;
    dfs_exact(&d, 0, 0);
    free(d.occ);
    *best_flow = d.best;
    return KVO_OK;
}

/* ------------------------------------------------------------------------ */
/* Bounds of the analysis of GBA (Section "Analysis of GBA", Steps 1 and 3)   */
/* ------------------------------------------------------------------------ */

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

/*
 * Numerator of the memory-time area lower bound on OPT (proof of the
 * area-based lower bound for OPT, first display): with the jobs numbered by
 * non-decreasing area,
 *     OPT >= (1 / M) * sum_{j = 1..n} (n - j + 1) * Area(o_j, s_j),
 * because the first i completions of any schedule have consumed at least the
 * i smallest areas and a round offers M units.  Returns the sum; the caller
 * divides by M.  Per-job prompts enter through each job's own area.
 */
int kvo_area_lb(int64_t n, const int32_t *o, const int32_t *s, int64_t s_scalar,
                int64_t *numerator)
{
    int64_t *a, j;
    __int128 sum = 0;
    if (n < 1)
        return KVO_EINVAL;
    a = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!a)
        return KVO_ENOMEM;
    for (j = 0; j < n; j++) {
        int64_t sj = s ? s[j] : s_scalar;
        if (o[j] < 1 || sj < 0) {
            free(a);
            return KVO_EINVAL;
        }
        a[j] = kvo_area(o[j], sj);
    }
    qsort(a, (size_t)n, sizeof(int64_t), cmp_i64);
    for (j = 1; j <= n; j++)
        sum += (__int128)(n - j + 1) * a[j - 1];
    free(a);
    if (sum > (__int128)INT64_MAX)
        return KVO_EINVAL;
    *numerator = (int64_t)sum;
    return KVO_OK;
}

/*
 * The upper bound on the flow time of GBA from Step 3 of its analysis, on the
 * ladder tau_p = tau0 * 2^p with true lengths as classes:
 *     Q_p = n_p * tau_p + sum_{i < n_p} floor(i * tau_p / k_p)      (ladder term)
 *     S_p = sum_{q < p} (floor(n_q * tau_q / k_q) + tau_q)          (class-prefix term)
 *     UpperGBA = sum_p (n_p * S_p + Q_p)
 * over the classes p = 0 .. the last class that has a job; k_p is the largest
 * memory-feasible parallelism for tau_p and the largest prompt of the class
 * (never below 1; an empty class takes the prompt 0, its k_p multiplies
 * n_q = 0 and does not matter).
 */
int kvo_upper_gba(int64_t n, const int32_t *o, const int32_t *s, int64_t s_scalar,
                  int64_t M, int64_t tau0, int64_t *upper)
{
    enum { MAXC = 64 };
    int64_t cnt[MAXC], smax[MAXC], tau[MAXC], kk[MAXC];
    int64_t j, p, last = 0, total = 0;
    if (n < 1 || tau0 < 1 || M < 1)
        return KVO_EINVAL;
    for (p = 0; p < MAXC; p++)
        cnt[p] = smax[p] = 0;
    for (j = 0; j < n; j++) {
        int64_t sj = s ? s[j] : s_scalar, t = tau0;
        if (o[j] < 1 || sj < 0)
            return KVO_EINVAL;
        if (sj + o[j] > M)
            return KVO_EJOB_INFEASIBLE;
        for (p = 0; t < o[j]; p++)
            t *= 2;
        cnt[p]++;
        if (sj > smax[p])
            smax[p] = sj;
        if (p > last)
            last = p;
    }
    for (p = 0; p <= last; p++) {
        tau[p] = tau0 << p;
        kk[p] = phase_parallelism(KVO_SPS, tau[p], smax[p], M, 0);
    }
    for (p = 0; p <= last; p++) {
        int64_t Q = cnt[p] * tau[p], S = 0, i, q;
        for (i = 0; i < cnt[p]; i++)
            Q += (i * tau[p]) / kk[p];
        for (q = 0; q < p; q++)
            S += (cnt[q] * tau[q]) / kk[q] + tau[q];
        total += cnt[p] * S + Q;
    }
    *upper = total;
    return KVO_OK;
}

/* ------------------------------------------------------------------------ */
/* GBA with dynamic refill ("GBA-D", appendix "Numerical Experiments")        */
/* ------------------------------------------------------------------------ */

/*
 * The appendix describes the variant in one sentence: a job is admitted as
 * soon as the pipeline can go on with it without violating memory
 * feasibility, and no job is ever delayed relative to the schedule of
 * Algorithm 2, whose idle time it only fills.  The reading taken here (the
 * paper prints no value that would pin another):
 *
 *   - the baseline is the schedule of Algorithm 2 on the ladder tau_0 * 2^p
 *     (subroutine, parallelism as for kvo_gba_simulate, true lengths as
 *     classes); every job first holds its baseline slot with its actual run
 *     (o_i rounds from its baseline start);
 *   - the jobs are taken in the baseline's order (class by class, input order
 *     inside a class).  Each is moved to the earliest round, not before the
 *     start of the job before it in that order and not after its own baseline
 *     start, at which its whole run fits in every round on top of the runs of
 *     all the other jobs where they stand now: the earlier ones where they were
 *     moved to, the later ones still at their baseline starts.
 *
 * Because the later jobs keep their places in the test, every job can always
 * fall back on its baseline start: no job is delayed, and the schedule stays
 * within the budget whenever the baseline does.  (Testing against the earlier
 * jobs alone would not do: a job moved up is further along, hence larger,
 * when a later one wants its baseline slot.)
 *
 * start_out / base_start_out (may be NULL): start round of every job in the
 * refilled and in the baseline schedule.
 */
int kvo_gbad_simulate(int64_t n, const int32_t *o, const int32_t *s,
                      int64_t s_scalar, int64_t M, int64_t tau0, int sched,
                      int64_t k, int64_t *peak, int32_t *feasible,
                      int64_t *flow, int64_t *job_steps, int64_t *start_out,
                      int64_t *base_start_out)
{
    int64_t *cls = NULL, *order = NULL, *base = NULL, *start = NULL, *occ = NULL;
    int64_t i, j, p, maxcls = 0, pos = 0, begin = 0, horizon, prev = 0, pk = 0, fl = 0, steps = 0;
    int rc = KVO_OK;

    if (n < 0 || M <= 0 || tau0 < 1 || k < 0 || (sched != KVO_SPS && sched != KVO_SIMS))
        return KVO_EINVAL;
    for (i = 0; i < n; i++) {
        int64_t si = s ? s[i] : s_scalar;
        if (o[i] < 1 || si < 0)
            return KVO_EINVAL;
        if (si + o[i] > M)
            return KVO_EJOB_INFEASIBLE;
    }
    cls = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    order = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    base = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    start = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!cls || !order || !base || !start) {
        rc = KVO_ENOMEM;
        goto out;
    }
    /* classes of Algorithm 2: the first slice tau_0 * 2^p that covers the length */
    for (i = 0; i < n; i++) {
        int64_t t = tau0;
        for (p = 0; t < o[i]; p++)
            t *= 2;
        cls[i] = p;
        if (p > maxcls)
            maxcls = p;
    }
    /* the baseline: class after class, Procedure 1 (or the simultaneous schedule) inside */
    for (p = 0; p <= maxcls; p++) {
        int64_t tau = tau0 << p, n_p = 0, s_max = 0, kk, r = 0;
        for (i = 0; i < n; i++)
            if (cls[i] == p) {
                int64_t si = s ? s[i] : s_scalar;
                n_p++;
                if (si > s_max)
                    s_max = si;
            }
        if (n_p == 0)
            continue;
        kk = phase_parallelism(sched, tau, s_max, M, k);
        for (i = 0; i < n; i++)
            if (cls[i] == p) {
                base[i] = begin + start_offset(sched, r, tau, kk);
                order[pos++] = i;
                r++;
            }
        begin += start_offset(sched, n_p - 1, tau, kk) + tau;
    }
    horizon = begin + 1;
    occ = (int64_t *)calloc((size_t)horizon, sizeof(int64_t));
    if (!occ) {
        rc = KVO_ENOMEM;
        goto out;
    }
    for (i = 0; i < n; i++) {
        start[i] = base[i];
        place(occ, base[i], o[i], s ? s[i] : s_scalar, +1);
    }
    /* refill: one job after the other, in the baseline's order */
    for (j = 0; j < n; j++) {
        int64_t t, si;
        i = order[j];
        si = s ? s[i] : s_scalar;
        place(occ, base[i], o[i], si, -1);
        for (t = prev; t < base[i]; t++)
            if (fits(occ, horizon, t, o[i], si, M))
                break;
        start[i] = t; /* its baseline start if nothing earlier fits */
        place(occ, t, o[i], si, +1);
        prev = t;
    }
    for (i = 0; i < horizon; i++)
        if (occ[i] > pk)
            pk = occ[i];
    for (i = 0; i < n; i++) {
        fl += start[i] + o[i];
        steps += o[i];
        if (start_out)
            start_out[i] = start[i];
        if (base_start_out)
            base_start_out[i] = base[i];
    }
    *peak = pk;
    *feasible = pk <= M ? 1 : 0;
    *flow = fl;
    *job_steps = steps;
out:
    free(cls); free(order); free(base); free(start); free(occ);
    return rc;
}

/* Instances [i0, i1) at every point (tau0, sched, k); outputs [n_pts][i1 - i0]. */
int kvo_gbad_simulate_batch(int64_t i0, int64_t i1, int64_t n, const int32_t *o,
                            const int32_t *s, int64_t s_scalar, int64_t M,
                            int64_t n_pts, const int32_t *tau0,
                            const int32_t *sched, const int32_t *k,
                            int64_t *peak, uint8_t *feasible, int64_t *flow,
                            int64_t *job_steps)
{
    int64_t q, i, cnt = i1 - i0;
    for (q = 0; q < n_pts; q++)
        for (i = i0; i < i1; i++) {
            int32_t feas = 0;
            int64_t idx = q * cnt + (i - i0);
            int rc = kvo_gbad_simulate(n, o + i * n, s ? s + i * n : NULL, s_scalar, M, tau0[q],
                                       sched[q], k[q], &peak[idx], &feas, &flow[idx],
                                       &job_steps[idx], NULL, NULL);
            if (rc != KVO_OK)
                return rc;
            feasible[idx] = (uint8_t)feas;
        }
    return KVO_OK;
}
