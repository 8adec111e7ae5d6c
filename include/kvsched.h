/*
 * kvsched.h -- C ABI of the MI355X (gfx950) schedule-evaluation library.
 *
 * Batched evaluation of the scheduling policies of "Competitive
 * Non-Clairvoyant KV-Cache Scheduling for LLM Inference" (Feng, Yang, Zhang)
 * over many independent instances and a sweep of parameters.  Citations name
 * sections, equations, procedures and algorithms of that paper.
 *
 * Model (Section 2.1, "Model and Objective").  An instance is a set of jobs;
 * job i has a prompt length s_i >= 0 and a response length o_i >= 1 (tokens).
 * Time runs in rounds t = 0, 1, ...; a job started in round S is active in
 * the rounds S .. S + d - 1 (d = o_i if it completes, the slice length if it
 * is killed), occupies s_i + (t - S) + 1 units of KV-cache memory in round t
 * (eq. (Memory-Feasibility)) and, if it completes, does so at round S + o_i.
 *   MemPeak  = max over rounds of the summed occupancy of the active jobs;
 *   feasible = MemPeak <= M;
 *   FlowTime = sum of the completion rounds.
 *
 * Conventions for every entry point
 *   - plain C, no exceptions; the return value is a status code, 0 = KVS_OK;
 *   - pointers inside kvs_jobs_t and all output pointers are DEVICE pointers
 *     (memory of the GPU that is current on the calling thread); the structs
 *     themselves and the arrays of sweep points are HOST memory, read before
 *     the call returns;
 *   - the caller owns every buffer; the library allocates nothing that
 *     outlives a call and keeps no state between calls;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without waiting; outputs are valid
 *     once the stream has been synchronised.  kvs_validate is the exception:
 *     it waits and reports what it found;
 *   - job arrays are row-major [n_instances][n_jobs], int32;
 *   - outputs are row-major [n_pts][n_instances].
 *
 * Errors that depend on the job data cannot be returned by an asynchronous
 * call; they are reported in-band, per evaluation, in `feasible`:
 *   0 / 1                  the schedule exceeds / respects the budget M;
 *   KVS_FEASIBLE_EINVAL    some job of the instance has o < 1, s < 0 or
 *                          o_est < 1 (every point of the instance);
 *   KVS_FEASIBLE_EJOB      some job has s + o > M: it does not fit the budget
 *                          on its own, the per-job feasibility assumption of
 *                          Section 2.1 fails (every point of the instance);
 *   KVS_FEASIBLE_ERANGE    a length of the instance exceeds 2^30 (every
 *                          point), or this evaluation would leave the 32-bit
 *                          range of the device arithmetic in one of its own
 *                          phases (see "Limits"; only the points whose phases
 *                          do so).
 * When several apply the order is EINVAL, ERANGE for a length, EJOB, ERANGE
 * for a phase -- the order in which kvs_validate reports the first three.
 * In every error case peak, flow and the remaining outputs of that evaluation
 * are -1.
 *
 * Limits: 1 <= n_jobs <= KVS_MAX_JOBS; lengths (o, s, o_est, tau) at most
 * 2^30; 1 <= M < 2^40; per phase, n_p * tau_p < 2^31 and
 * min(n_p, k_p) * (s_max + tau_p + 513) < 2^31 (n_p jobs take part in the
 * phase, tau_p is its slice, k_p its parallelism, s_max its largest prompt).
 *
 * Cost: a phase of n_p jobs that lasts H_p rounds costs O(n_p + H_p / 64) per
 * (subroutine, parallelism) variant, or O(n_p k_p) where that is less (long
 * slices with few jobs in flight); phases of at most 64 jobs cost O(n_p^2).
 * No cost grows with the number of rounds alone.
 */
#ifndef KVSCHED_H
#define KVSCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVS_OK 0
#define KVS_EINVAL 1          /* bad argument: null pointer, size or parameter out of range */
#define KVS_EJOB_INFEASIBLE 2 /* kvs_validate: some job has s + o > M (in-band: KVS_FEASIBLE_EJOB) */
#define KVS_ERANGE 3          /* kvs_validate: a length exceeds 2^30                */
#define KVS_EHIP 4            /* a HIP runtime call failed                          */
#define KVS_ELIMIT 5          /* n_jobs or n_pts above the compiled limits          */

#define KVS_FEASIBLE_EJOB 0xFC
#define KVS_FEASIBLE_EINVAL 0xFE
#define KVS_FEASIBLE_ERANGE 0xFF

#define KVS_MAX_JOBS 16384 /* jobs per instance (one instance's phase lives in LDS) */
#define KVS_MAX_POINTS 64  /* sweep points per call                               */
#define KVS_MAX_LEVELS 64  /* slices of an explicit ladder                        */

#define KVS_SCHED_SPS 0  /* Staggered-Pipeline-Schedule, Procedure 1               */
#define KVS_SCHED_SIMS 1 /* Simultaneous-Schedule, appendix "Lower Bounds for SimS" */

#define KVS_MODE_GBA 0 /* Algorithm 2; with o_est: classes by the estimate        */
#define KVS_MODE_GSA 1 /* Algorithm 1: every unfinished job in every phase        */
#define KVS_MODE_GBAD 2 /* Algorithm 2 with dynamic refill ("GBA-D"), see below    */

/* One batch of instances (Section 2.1: jobs with prompt length s and response
 * length o; the estimate is what a non-clairvoyant scheduler believes). */
typedef struct {
    int32_t n_instances;
    int32_t n_jobs;
    const int32_t *o;     /* device, [n_instances][n_jobs], true response lengths >= 1   */
    const int32_t *s;     /* device, same shape, per-job prompt lengths; NULL: s_scalar  */
    const int32_t *o_est; /* device, same shape, estimated lengths >= 1; NULL: none      */
    int32_t s_scalar;     /* common prompt length when s == NULL                         */
    int64_t M;            /* KV-cache budget in tokens                                   */
} kvs_jobs_t;

/* One sweep point of kvs_gba_simulate. */
typedef struct {
    int32_t tau0;  /* initial slice length tau_0 >= 1; slices are tau_0 * 2^p (Algorithms 1, 2
                      with scaling factor 2 and a tunable integer initial slice)            */
    int32_t sched; /* KVS_SCHED_SPS or KVS_SCHED_SIMS: the per-phase subroutine              */
    int32_t k;     /* 0: per phase the largest memory-feasible parallelism, k*(tau_p, s) of
                      eq. (max-parallelism) for SPS, floor(M / (s + tau_p)) for SimS, with s
                      the largest prompt among the phase's jobs, never below 1;
                      > 0: this parallelism in every phase                                  */
    int32_t mode;  /* KVS_MODE_GBA, KVS_MODE_GSA or KVS_MODE_GBAD                           */
} kvs_point_t;

/*
 * Geometric phases (Algorithm 2 "GBA", Algorithm 1 "GSA") evaluated for every
 * instance at every sweep point.
 *
 * Phase p = 0, 1, ... has the slice tau_p = tau0 * 2^p.  Among the jobs not
 * yet completed, those the scheduler believes to fit the slice (o_i <= tau_p
 * in GBA mode without estimates; min(o_est_i, M - s_i) <= tau_p with
 * estimates; all of them in GSA mode) are run, in input order, by the
 * subroutine `sched` with slice tau_p: job number r of the phase starts
 * floor(r * tau_p / k_p) rounds (SPS) or floor(r / k_p) * tau_p rounds (SimS)
 * after the phase begins, completes after o_i rounds if o_i <= tau_p and is
 * otherwise killed at the end of its slice and tried again in the next phase.
 * A phase ends when its last slice ends; a phase without jobs takes no time.
 *
 * KVS_MODE_GBAD (appendix "Numerical Experiments", paragraph "Dynamic Refill":
 * a job is admitted as soon as the pipeline can go on with it without violating
 * memory feasibility, and never later than in Algorithm 2's schedule; the
 * paper says no more, this is the rule evaluated).  The baseline is the
 * schedule of KVS_MODE_GBA at the same (tau0, sched, k) on the true lengths
 * (o_est is ignored), every job holding its baseline start with its actual run
 * of o_i rounds.  In the baseline's order (class by class, input order inside a
 * class) each job moves to the earliest round, not before the start of the job
 * before it and not after its own baseline start, at which its whole run fits
 * in every round on top of all other jobs where they stand: the earlier ones
 * where they were moved to, the later ones at their baseline starts.  This
 * mode is sequential per instance and keeps the occupancy of every round of
 * the schedule in LDS: besides the limits above, the baseline may last at most
 * (about 160 KB - 8 n_jobs) / 4 rounds (KVS_FEASIBLE_ERANGE otherwise), and a
 * job's cost grows with its length and with the starts it has to try.
 *
 * Outputs (device, [n_pts][n_instances]; job_steps may be NULL):
 *   peak      MemPeak;  feasible  see above;  flow  FlowTime;
 *   job_steps number of (job, round) pairs the schedule processes, i.e. the
 *             simulated decode steps.
 *
 * Returns KVS_EINVAL for null required pointers, n_instances < 0, n_jobs < 1,
 * n_pts < 0, M outside [1, 2^40), s_scalar outside [0, 2^30], tau0 outside
 * [1, 2^30], k < 0, unknown sched / mode; KVS_ELIMIT above the limits;
 * KVS_EHIP if the launch fails.  n_instances == 0 or n_pts == 0 is a no-op.
 */
int32_t kvs_gba_simulate(const kvs_jobs_t *jobs, const kvs_point_t *pts, int32_t n_pts,
                         int64_t *peak, uint8_t *feasible, int64_t *flow,
                         int64_t *job_steps, void *stream);

/*
 * One invocation of the per-phase subroutine (Procedure 1 for SPS, the
 * simultaneous schedule for SimS) on the whole job sequence of every
 * instance, with explicit slice tau[q] and parallelism k[q] (0: automatic as
 * above) for every point q.  o_est is ignored.  Jobs with o_i <= tau complete
 * and count towards flow and n_completed; the others are killed when their
 * slice ends.
 *
 * tau, k, sched: host arrays of n_pts entries.  Outputs as above;
 * n_completed (device, int32, may be NULL) is the number of completed jobs.
 */
int32_t kvs_schedule_eval(const kvs_jobs_t *jobs, const int32_t *tau, const int32_t *k,
                          const int32_t *sched, int32_t n_pts, int64_t *peak,
                          uint8_t *feasible, int64_t *flow, int32_t *n_completed,
                          int64_t *job_steps, void *stream);

/*
 * kvs_gba_simulate on explicit ladders of slice lengths: any scaling factor
 * alpha and initial slice of Algorithms 1 and 2, whose phases use the integer
 * slices tau_p = floor(beta alpha^p).  Point q runs its phases p = 0, 1, ...
 * with the slices ladders[q * KVS_MAX_LEVELS + p], p < n_levels[q]; a job's
 * class is the first slice that covers its (believed) length.  sched, k, mode
 * as in kvs_point_t.  Everything else as kvs_gba_simulate.
 *
 * ladders: host, int32 [n_pts][KVS_MAX_LEVELS], each row non-decreasing with
 * entries in [1, 2^30] (else KVS_EINVAL); n_levels, sched, k, mode: host,
 * n_pts entries.  An instance with a length above the last slice of a ladder
 * has no class there and is reported in-band as KVS_FEASIBLE_EINVAL.
 */
int32_t kvs_ladder_simulate(const kvs_jobs_t *jobs, const int32_t *ladders,
                            const int32_t *n_levels, const int32_t *sched, const int32_t *k,
                            const int32_t *mode, int32_t n_pts, int64_t *peak, uint8_t *feasible,
                            int64_t *flow, int64_t *job_steps, void *stream);

/*
 * The ladder Algorithms 1 and 2 initialise for a common prompt length s and a
 * rational scaling factor alpha = alpha_num / alpha_den > 1:
 *   l = floor(log_alpha(M - s)),  beta = (M - s) / alpha^l  (so 1 <= beta < alpha),
 *   tau_p = floor(beta alpha^p),  p = 0 .. l,  tau_l = M - s,
 * in exact integer arithmetic.  Host only.  ladder: room for KVS_MAX_LEVELS
 * entries; *n_levels receives l + 1.  KVS_EINVAL for M <= s, s < 0,
 * M - s > 2^30 or alpha <= 1; KVS_ELIMIT if the ladder needs more than
 * KVS_MAX_LEVELS levels or the exact arithmetic would leave 128 bits.
 */
int32_t kvs_paper_ladder(int64_t M, int64_t s, int32_t alpha_num, int32_t alpha_den,
                         int32_t *ladder, int32_t *n_levels);

/*
 * The same ladder for a scaling factor that is a quadratic irrational,
 *   alpha = (a + b sqrt(c)) / d > 1,   a, b, c >= 0, d >= 1
 * (the factor that minimises the competitive ratio of Algorithm 1 in Theorem
 * "Competitive Ratio Guarantee of GSA" is (7 + sqrt(13)) / 6).  The powers of
 * alpha are carried as intervals of 64-bit-mantissa floating-point numbers
 * that contain the true values; a level or a floor on which the whole interval
 * agrees is accepted, any other is decided in exact 128-bit integer arithmetic
 * on alpha^q = (A + B sqrt(c)) / d^q.  Host only.  KVS_EINVAL as above, also
 * for alpha <= 1; KVS_ELIMIT if more than KVS_MAX_LEVELS levels are needed, or
 * if some floor(beta alpha^p) lies within about 2^-24 of an integer while the
 * exact integers no longer fit 128 bits: the call then fails rather than
 * guess.  The result, when there is one, is exact.
 */
int32_t kvs_paper_ladder_quadratic(int64_t M, int64_t s, int32_t a, int32_t b, int32_t c, int32_t d,
                                   int32_t *ladder, int32_t *n_levels);

/*
 * Scans the job arrays on the device, waits for the result and returns
 * KVS_OK, KVS_EINVAL (some o < 1, s < 0 or o_est < 1), KVS_ERANGE (a length
 * above 2^30) or KVS_EJOB_INFEASIBLE (some s + o > M, Section 2.1).  Optional:
 * the evaluation entry points report the same conditions per instance.
 */
int32_t kvs_validate(const kvs_jobs_t *jobs, void *stream);

/*
 * kvs_validate for callers that cannot allocate device memory (tight serving
 * loops, harnesses that forbid hipMalloc): the same scan and the same return
 * values, but the scan's 12-byte result lives in a 256-byte array that is
 * part of the library's device image (one copy per GPU, held until the
 * process ends) instead of being allocated and freed by the call.  The result
 * does not grow with the input, so no input is too large for it; the call
 * allocates and frees nothing.  Every call on a GPU uses that GPU's one array
 * (cleared by a small kernel at the start of each call): calls that overlap
 * on the same GPU, from any threads or streams, race and may report each
 * other's findings.  Waits for the stream like kvs_validate.
 */
int32_t kvs_validate_static(const kvs_jobs_t *jobs, void *stream);

/*
 * The two bounds between which the analysis of GBA places its flow time
 * (Section "Analysis of GBA"), per instance, next to the schedules themselves:
 *
 * upper_gba (device, int64 [n_pts][n_instances]): the upper bound of Step 3
 * (Lemma "GBA Upper Bound via Packing Efficiency") on the ladder
 * tau_p = tau0[q] * 2^p with the true lengths as classes,
 *     Q_p = n_p tau_p + sum_{i < n_p} floor(i tau_p / k_p)          (ladder term),
 *     S_p = sum_{q < p} (floor(n_q tau_q / k_q) + tau_q)            (class-prefix term),
 *     UpperGBA = sum_p (n_p S_p + Q_p),  p = 0 .. the last class with a job,
 * k_p = max(1, k*(tau_p, s)) of eq. (max-parallelism) with s the largest prompt
 * of the class (0 for an empty class).  Always >= the flow of kvs_gba_simulate
 * at (tau0, SPS, k = 0, GBA) without estimates.
 *
 * area_lb_num (device, int64 [n_instances]): numerator of the memory-time area
 * lower bound on OPT (Step 1, first display of the proof of Lemma "Area-Based
 * Lower Bound for OPT"): with the jobs numbered by non-decreasing area
 * Area(o, s) = s o + o (o + 1) / 2,
 *     OPT >= (1 / M) sum_{j = 1..n} (n - j + 1) Area(o_j, s_j);
 * the sum is returned, the caller divides by M.
 *
 * tau0: host, n_pts entries in [1, 2^30].  o_est is ignored.  Either output
 * may be NULL (upper_gba only with n_pts == 0).  In-band errors, value -1: an
 * invalid job (as KVS_FEASIBLE_EINVAL); upper_gba also when some class has
 * n_p tau_p >= 2^31; area_lb_num also when n (n + 1) / 2 times the largest
 * area reaches 2^63.  Return values as kvs_gba_simulate.
 */
int32_t kvs_flow_bounds(const kvs_jobs_t *jobs, const int32_t *tau0, int32_t n_pts,
                        int64_t *upper_gba, int64_t *area_lb_num, void *stream);

#define KVS_MAX_PERM_JOBS 10          /* jobs per instance of kvs_opt_perm (10! orders) */
#define KVS_MAX_PERM_ROUNDS (1 << 20) /* largest sum of the lengths of such an instance  */

/*
 * Best list schedule over every order of the jobs, for tiny instances: a
 * feasible schedule without kills or pauses, hence an upper bound on OPT
 * (Section 2.1: OPT needs neither), and OPT itself on many tiny instances.
 * For an order, the
 * jobs are started one after the other, each at the earliest round, not before
 * its predecessor's start, at which its whole run s + 1 .. s + o fits on top
 * of the runs already placed in every round (eq. (Memory-Feasibility)); the
 * flow time of the order is the sum of start + o.  best_flow (device, int64
 * [n_instances]) receives the minimum over all n_jobs! orders, or -1 for an
 * instance with an invalid job or with lengths that sum to more than
 * KVS_MAX_PERM_ROUNDS.
 *
 * Needs a common prompt length (jobs->s == NULL, else KVS_EINVAL) and
 * n_jobs <= KVS_MAX_PERM_JOBS (else KVS_ELIMIT); o_est is ignored.
 */
int32_t kvs_opt_perm(const kvs_jobs_t *jobs, int64_t *best_flow, void *stream);

/* Static, human-readable text for a status code. */
const char *kvs_strerror(int32_t status);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t kvs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVSCHED_H */
