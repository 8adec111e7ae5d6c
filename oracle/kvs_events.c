/*
 * kvs_events.c -- second CPU evaluator: the same schedules as kvs_oracle.c,
 * evaluated from start and end events instead of round by round.
 *
 * TEST INFRASTRUCTURE ONLY, like kvs_oracle.c, and for one purpose: the
 * literal stepper costs one operation per (job, round) and cannot cover every
 * instance of the largest workload in a test; this evaluator costs
 * O(n log k) per phase and can.  It is written independently of the stepper
 * (no shared function) and of the GPU sources, and it is trusted only as far
 * as tests/test_oracle_pins.py shows it equal to the literal stepper: on
 * random instances in every mode and on instances of the four smaller
 * workloads.  Where the two disagree the stepper is right by definition.
 *
 * Follows "Competitive Non-Clairvoyant KV-Cache Scheduling for LLM Inference"
 * (Feng, Yang, Zhang): Section 2.1 (occupancy s + u + 1 of an active job,
 * completion at start + o), Procedure 1 (SPS start offsets, kill at the end of
 * the slice), appendix "Lower Bounds for SimS" (SimS), eq. (max-parallelism)
 * with Lemma "Peak Memory Usage of SPS", Algorithms 1 and 2 (phases, "keep the
 * unfinished jobs").
 *
 * How the occupancy peak is found without stepping.  A run with start S,
 * duration d and prompt s occupies s + 1 + (t - S) in the rounds S <= t < S + d.
 * While the set of active runs does not change the total grows by one per
 * active run and round, and it jumps up when a run starts; it can only fall
 * when a run leaves.  So the maximum over all rounds is attained in the last
 * round of some run.  With C = number of active runs and A = sum of
 * (s + 1 - S) over them, the occupancy of round t is A + t C; runs are added in
 * start order and leave through a min-heap keyed by their end, and the
 * occupancy is read off in the round before each departure.
 */
#include <stdint.h>
#include <stdlib.h>

#define KVE_OK 0
#define KVE_EINVAL 1
#define KVE_EJOB_INFEASIBLE 2
#define KVE_ENOMEM 3

#define KVE_SPS 0
#define KVE_SIMS 1
#define KVE_MODE_GBA 0
#define KVE_MODE_GSA 1

typedef struct {
    int64_t end; /* first round in which the run is no longer active */
    int64_t w;   /* s + 1 - start                                    */
} kve_item_t;

static void heap_push(kve_item_t *h, int64_t *len, kve_item_t x)
{
    int64_t i = (*len)++;
    while (i > 0) {
        int64_t parent = (i - 1) / 2;
        if (h[parent].end <= x.end)
            break;
        h[i] = h[parent];
        i = parent;
    }
    h[i] = x;
}

static kve_item_t heap_pop(kve_item_t *h, int64_t *len)
{
    kve_item_t top = h[0], x = h[--(*len)];
    int64_t i = 0, n = *len;
    for (;;) {
        int64_t c = 2 * i + 1;
        if (c >= n)
            break;
        if (c + 1 < n && h[c + 1].end < h[c].end)
            c++;
        if (x.end <= h[c].end)
            break;
        h[i] = h[c];
        i = c;
    }
    if (n > 0)
        h[i] = x;
    return top;
}

static int64_t gcd_i64(int64_t a, int64_t b)
{
    while (b) {
        int64_t r = a % b;
        a = b;
        b = r;
    }
    return a;
}

/* Largest k with s k + (tau k + tau + k - gcd(tau, k)) / 2 <= M (eq. (max-parallelism)).
 * Lemma "Feasible Parallelism of SPS" puts it at or above floor((2M - tau + 1) / (2s + tau + 1));
 * from there the scan goes up while the next value still fits (Peak is increasing in k). */
static int64_t largest_parallelism(int64_t tau, int64_t s, int64_t M)
{
    int64_t k = (2 * M - tau + 1) / (2 * s + tau + 1);
    if (2 * M - tau + 1 < 0)
        k = 0;
    while (k > 0 && s * k + (tau * k + tau + k - gcd_i64(tau, k)) / 2 > M)
        k--; /* never taken if the lemma holds; keeps the answer right if it did not */
    for (;;) {
        int64_t c = k + 1;
        int64_t peak = s * c + (tau * c + tau + c - gcd_i64(tau, c)) / 2;
        if (peak > M)
            break;
        k = c;
    }
    return k;
}

/*
 * One instance at one sweep point.  Slices: ladder[0 .. n_levels) when ladder
 * is given, else tau0 * 2^p.  Returns KVE_EINVAL for malformed jobs or a job
 * that no slice covers, KVE_EJOB_INFEASIBLE for s + o > M.
 */
int kve_simulate(int64_t n, const int32_t *o, const int32_t *s, const int32_t *o_est,
                 int64_t s_scalar, int64_t M, int64_t tau0, const int32_t *ladder,
                 int64_t n_levels, int sched, int64_t k_forced, int mode, int64_t *peak,
                 int32_t *feasible, int64_t *flow, int64_t *job_steps)
{
    int64_t *todo = NULL;   /* unfinished jobs, input order            */
    int64_t *believed = NULL; /* length the scheduler assumes per job  */
    kve_item_t *heap = NULL;
    int64_t left, i, p, begin = 0, pk = 0, fl = 0, steps = 0;
    int rc = KVE_OK;

    if (n < 0 || M <= 0 || tau0 < 1 || k_forced < 0 || (sched != KVE_SPS && sched != KVE_SIMS) ||
        (mode != KVE_MODE_GBA && mode != KVE_MODE_GSA))
        return KVE_EINVAL;
    for (i = 0; i < n; i++) {
        int64_t si = s ? s[i] : s_scalar;
        if (o[i] < 1 || si < 0 || (o_est && o_est[i] < 1))
            return KVE_EINVAL;
        if (si + o[i] > M)
            return KVE_EJOB_INFEASIBLE;
    }
    todo = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    believed = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    heap = (kve_item_t *)malloc(sizeof(kve_item_t) * (size_t)(n + 1));
    if (!todo || !believed || !heap) {
        free(todo); free(believed); free(heap);
        return KVE_ENOMEM;
    }
    for (i = 0; i < n; i++) {
        int64_t si = s ? s[i] : s_scalar;
        todo[i] = i;
        if (mode == KVE_MODE_GSA)
            believed[i] = 1; /* Algorithm 1 knows nothing: everybody is tried from the first phase */
        else if (o_est) {
            int64_t e = o_est[i];
            if (e > M - si)
                e = M - si;
            believed[i] = e < 1 ? 1 : e;
        } else
            believed[i] = o[i]; /* Algorithm 2 */
    }
    left = n;

    for (p = 0; left > 0; p++) {
        int64_t tau, n_p = 0, s_max = 0, par, r, kept = 0, hl = 0, A = 0, C = 0, last_start = 0;
        if (ladder) {
            if (p >= n_levels) {
                rc = KVE_EINVAL;
                break;
            }
            tau = ladder[p];
        } else {
            if (p > 40) {
                rc = KVE_EINVAL;
                break;
            }
            tau = tau0 << p;
        }
        /* who takes part, and the largest prompt among them */
        for (i = 0; i < left; i++) {
            int64_t j = todo[i];
            if (believed[j] <= tau) {
                int64_t sj = s ? s[j] : s_scalar;
                if (sj > s_max)
                    s_max = sj;
                n_p++;
            }
        }
        if (n_p == 0)
            continue;
        if (k_forced > 0)
            par = k_forced;
        else if (sched == KVE_SPS)
            par = largest_parallelism(tau, s_max, M);
        else
            par = M / (s_max + tau);
        if (par < 1)
            par = 1;

        r = 0;
        for (i = 0; i < left; i++) {
            int64_t j = todo[i];
            int64_t sj, start, d;
            kve_item_t it;
            if (believed[j] > tau) {
                todo[kept++] = j; /* waits for a later phase */
                continue;
            }
            sj = s ? s[j] : s_scalar;
            start = begin + (sched == KVE_SPS ? (r * tau) / par : (r / par) * tau);
            last_start = start;
            r++;
            /* runs that end at or before this start leave first; the round before each
             * departure is a candidate for the peak */
            while (hl > 0 && heap[0].end <= start) {
                int64_t occ = A + (heap[0].end - 1) * C;
                kve_item_t out = heap_pop(heap, &hl);
                if (occ > pk)
                    pk = occ;
                A -= out.w;
                C -= 1;
            }
            if (o[j] <= tau) {
                d = o[j];
                fl += start + d; /* completes */
            } else {
                d = tau;         /* killed when the slice ends, tried again in the next phase */
                todo[kept++] = j;
            }
            steps += d;
            it.end = start + d;
            it.w = sj + 1 - start;
            heap_push(heap, &hl, it);
            A += it.w;
            C += 1;
        }
        while (hl > 0) {
            int64_t occ = A + (heap[0].end - 1) * C;
            kve_item_t out = heap_pop(heap, &hl);
            if (occ > pk)
                pk = occ;
            A -= out.w;
            C -= 1;
        }
        left = kept;
        begin = last_start + tau; /* the phase lasts until its last slice ends */
    }

    free(todo); free(believed); free(heap);
    if (rc != KVE_OK)
        return rc;
    *peak = pk;
    *feasible = pk <= M ? 1 : 0;
    *flow = fl;
    *job_steps = steps;
    return KVE_OK;
}

/* Instances [i0, i1) of row-major [.][n] arrays at every point (tau0, sched, k, mode) on the
 * doubling ladder; outputs [n_pts][i1 - i0].  Stops at the first error. */
int kve_gba_simulate_batch(int64_t i0, int64_t i1, int64_t n, const int32_t *o, const int32_t *s,
                           const int32_t *o_est, int64_t s_scalar, int64_t M, int64_t n_pts,
                           const int32_t *tau0, const int32_t *sched, const int32_t *k,
                           const int32_t *mode, int64_t *peak, uint8_t *feasible, int64_t *flow,
                           int64_t *job_steps)
{
    int64_t q, i, cnt = i1 - i0;
    for (i = i0; i < i1; i++)
        for (q = 0; q < n_pts; q++) {
            int32_t feas = 0;
            int64_t idx = q * cnt + (i - i0);
            int rc = kve_simulate(n, o + i * n, s ? s + i * n : NULL, o_est ? o_est + i * n : NULL,
                                  s_scalar, M, tau0[q], NULL, 0, sched[q], k[q], mode[q],
                                  &peak[idx], &feas, &flow[idx], &job_steps[idx]);
            if (rc != KVE_OK)
                return rc;
            feasible[idx] = (uint8_t)feas;
        }
    return KVE_OK;
}

/* One instance on an explicit ladder of slices. */
int kve_ladder_simulate(int64_t n, const int32_t *o, const int32_t *s, const int32_t *o_est,
                        int64_t s_scalar, int64_t M, const int32_t *ladder, int64_t n_levels,
                        int sched, int64_t k, int mode, int64_t *peak, int32_t *feasible,
                        int64_t *flow, int64_t *job_steps)
{
    int64_t p;
    if (!ladder || n_levels < 1 || ladder[0] < 1)
        return KVE_EINVAL;
    for (p = 1; p < n_levels; p++)
        if (ladder[p] < ladder[p - 1])
            return KVE_EINVAL;
    return kve_simulate(n, o, s, o_est, s_scalar, M, 1, ladder, n_levels, sched, k, mode, peak,
                        feasible, flow, job_steps);
}
