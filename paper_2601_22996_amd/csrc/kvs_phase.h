/*
 * kvs_phase.h -- evaluation of one phase of the geometric-slicing algorithms on
 * gfx950: the slot / schedule tables, the LDS entry of a run, and the occupancy
 * of a slab of rounds in exact event / prefix-sum form.
 *
 * Citations: "Competitive Non-Clairvoyant KV-Cache Scheduling for LLM
 * Inference" (Feng, Yang, Zhang): Section 2.1 (occupancy of a round, flow time),
 * Procedure 1 (start offsets of SPS), appendix "Lower Bounds for SimS" (SimS).
 */
#ifndef KVS_PHASE_H
#define KVS_PHASE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvs_math.h"
#include "kvs_wave.h"

namespace {

constexpr int kWinMax = 512; /* most rounds a wavefront's window can hold */

/* Slot: the jobs of one phase (a level, or the merged first phase of a shift). */
struct Slot {
    uint32_t n;     /* participants                                      */
    uint32_t done;  /* of which complete in this phase                   */
    uint32_t smax;  /* largest prompt among them                         */
    uint32_t tau;   /* slice length                                      */
    uint32_t off;   /* where its entries start in the phase buffer       */
    uint32_t alias; /* slot whose results it shares, or its own index    */
    uint32_t bad;   /* n * tau leaves 31 bits: the phase is not evaluated */
    kvs_divisor_t divtau; /* division by tau                             */
};

/* Variant of a slot: the schedule the subroutine builds on it. */
struct Sched {
    uint32_t k; /* parallelism (SPS) or batch size (SimS), >= 1          */
    uint32_t H; /* rounds the phase lasts                                */
    uint32_t S; /* slab length used to evaluate it; 0: by runs, not by rounds (eval_thin) */
    uint32_t nslab; /* work items: slabs of S rounds, groups of 64 runs, 1 for a phase of at most
                       64 runs, 0 when there is nothing to evaluate        */
    uint32_t bad;   /* the window sums could leave 32 bits: not evaluated  */
    uint32_t narrow; /* the event sums of a round fit one 32-bit word (see WinFmt): slabs twice as long */
    kvs_divisor_t div;
};

struct Result {
    int32_t peak;
    unsigned long long sumF; /* sum of the start offsets of the completing runs */
};

/* Start offset of the r-th job of a phase: floor(r tau / k) for SPS
 * (Procedure 1), floor(r / k) tau for SimS. */
__device__ __forceinline__ uint32_t start_offset(uint32_t r, uint32_t tau, const Sched &c, bool sps)
{
    return sps ? kvs_div(r * tau, c.div) : kvs_div(r, c.div) * tau;
}

/*
 * Number of runs of the phase whose start offset is below x, for x <= H.
 * SPS: floor(r tau / k) < x  <=>  r tau < x k  <=>  r < ceil(x k / tau).
 * SimS: floor(r / k) tau < x <=>  floor(r / k) < ceil(x / tau).
 * Past the last start offset the answer is n, which also keeps x * k inside
 * 31 bits: below it x k <= (n - 1) tau.
 */
__device__ __forceinline__ uint32_t ranks_before(uint32_t x, const Slot &sl, const Sched &sc,
                                                 bool sps)
{
    if (x == 0)
        return 0;
    if (x > sc.H - sl.tau)
        return sl.n;
    uint32_t r;
    if (sps)
        r = kvs_div(x * sc.k - 1u, sl.divtau) + 1u;
    else
        r = (kvs_div(x - 1u, sl.divtau) + 1u) * sc.k;
    return r > sl.n ? sl.n : r;
}

/* How phase entries are laid out in LDS.  One word: prompt | done-bit |
 * duration, with the field width taken from the instance's largest values;
 * two words when that does not fit 32 bits. */
struct EntryFmt {
    uint32_t dbits;  /* duration in bits [0, dbits), done-bit at dbits, prompt above          */
    uint32_t sshift; /* where the prompt starts: dbits + 1, or dbits when no done-bit is kept */
    uint32_t swidth; /* bits of the prompt field, 0 when no prompt is stored                  */
    uint32_t s_add;  /* the common prompt length when none is stored, else 0                  */
    bool has_s;      /* per-job prompts are stored at all                                     */
    bool all_done;   /* every run completes: no done-bit                                      */
    bool raw;        /* the duration field holds the job's whole length: the run completes if
                        that is within the slice and is cut off at the slice otherwise         */
};

template <bool PACKED>
__device__ __forceinline__ void put_entry(uint32_t *buf, uint32_t n_cap, uint32_t pos, uint32_t d,
                                          bool done, uint32_t s, const EntryFmt &F)
{
    if (PACKED) {
        uint32_t w = d;
        if (!F.all_done)
            w |= (uint32_t)done << F.dbits;
        if (F.has_s)
            w |= s << F.sshift;
        buf[pos] = w;
    } else {
        buf[pos] = d | ((uint32_t)done << 31);
        buf[n_cap + pos] = s;
    }
}

template <bool PACKED>
__device__ __forceinline__ void get_entry(const uint32_t *buf, uint32_t n_cap, uint32_t pos,
                                          uint32_t &d, bool &done, uint32_t &s, uint32_t s_scalar,
                                          const EntryFmt &F, uint32_t tau)
{
    const uint32_t w = buf[pos];
    if (PACKED) {
        d = w & ((1u << F.dbits) - 1u);
        if (F.raw) {
            done = d <= tau;
            d = done ? d : tau;
        } else {
            done = F.all_done || ((w >> F.dbits) & 1u);
        }
        s = (w >> F.sshift) + F.s_add; /* the prompt is the topmost field; nothing above sshift <= 31 when none is stored */
    } else {
        d = w & 0x7fffffffu;
        done = w >> 31;
        s = buf[n_cap + pos];
    }
}

/* The same for an entry whose first word has been read already (a loop that reads two entries
 * with one LDS instruction and then works through them). */
template <bool PACKED>
__device__ __forceinline__ void entry_of_word(uint32_t w, const uint32_t *buf, uint32_t n_cap, uint32_t pos,
                                              uint32_t &d, bool &done, uint32_t &s, const EntryFmt &F,
                                              uint32_t tau)
{
    if (PACKED) {
        d = w & ((1u << F.dbits) - 1u);
        if (F.raw) {
            done = d <= tau;
            d = done ? d : tau;
        } else {
            done = F.all_done || ((w >> F.dbits) & 1u);
        }
        s = (w >> F.sshift) + F.s_add;
    } else {
        d = w & 0x7fffffffu;
        done = w >> 31;
        s = buf[n_cap + pos];
    }
}

/* An end event: one run less, and its weight w = s + 1 - start taken out: -(2^32 + w), as
 * this constant plus the sign-extended -w. */
constexpr unsigned long long kEndOne = 0xffffffff00000000ull;

/*
 * The entry of a round in a wavefront's window: the number of runs that start there minus those
 * whose first round off it is, C, above the sum A of their weights (s + 1 - start offset, signed),
 * in one integer C * 2^shift + A, so that one LDS atomic adds both.  Wide: 64 bits, shift 32.
 * Narrow: 32 bits, shift 23 -- for phases in which no round's events can leave |A| < 2^22 and
 * |C| < 2^8 (the schedule stage checks it from the parallelism, the largest prompt and the
 * slice); the window then holds twice the rounds and its atomics are half as wide.  Whatever the
 * order of the additions, the final sums decode exactly while they are in range.
 */
template <bool NARROW> struct WinFmt;
template <> struct WinFmt<false> {
    typedef unsigned long long T;
    static __device__ __forceinline__ T starts(uint32_t cnt, int32_t a)
    {
        return ((T)cnt << 32) + (T)(long long)a;
    }
    static __device__ __forceinline__ T end(int32_t w) { return kEndOne + (T)(long long)(-w); }
    static __device__ __forceinline__ void decode(T e, int32_t &a, int32_t &c)
    {
        a = (int32_t)(uint32_t)e;                        /* signed low word            */
        c = (int32_t)(uint32_t)(e >> 32) - (a >> 31);    /* undo the low word's borrow */
    }
};
template <> struct WinFmt<true> {
    typedef uint32_t T;
    static constexpr uint32_t kShift = 23;
    static __device__ __forceinline__ T starts(uint32_t cnt, int32_t a) { return (cnt << kShift) + (uint32_t)a; }
    static __device__ __forceinline__ T end(int32_t w) { return (0u - (1u << kShift)) + (uint32_t)(-w); }
    static __device__ __forceinline__ void decode(T e, int32_t &a, int32_t &c)
    {
        a = (int32_t)(e << (32u - kShift)) >> (32u - kShift); /* the low 23 bits, signed */
        c = ((int32_t)e - a) >> kShift;                       /* exact: a multiple of 2^23 is left */
    }
};

/*
 * One slab [t_s, t_s + len) of one phase variant, by one wavefront.
 * ev: the wavefront's window of packed (C << 32) + A event sums, one per round of the slab.
 * sumF collects the start offsets of the completing runs that start here.
 */
template <bool PACKED, int WIN, bool NARROW>
__device__ __forceinline__ void eval_slab(const Slot &sl, const Sched &sc, bool sps, uint32_t slab,
                                          const uint32_t *buf, uint32_t n_cap, uint32_t s_scalar,
                                          const EntryFmt &F, unsigned long long *window, int lane,
                                          int32_t &pk, unsigned long long &sumF)
{
    typedef WinFmt<NARROW> W;
    typename W::T *const ev = reinterpret_cast<typename W::T *>(window); /* WIN wide or 2 WIN narrow entries */
    const uint32_t t_s = slab * sc.S;
    const uint32_t len = (sc.H - t_s < sc.S) ? (sc.H - t_s) : sc.S;
    const int per = (int)((len + 63u) >> 6); /* window entries per lane */

    for (int j = 0; j < per; j++)
        ev[j * 64 + lane] = 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    /* ranks [r0, r1) started less than tau rounds before the slab, [r1, r2) start inside it */
    const uint32_t r0 = ranks_before((t_s + 1u > sl.tau) ? (t_s + 1u - sl.tau) : 0u, sl, sc, sps);
    const uint32_t r1 = ranks_before(t_s, sl, sc, sps);
    const uint32_t r2 = ranks_before(t_s + len, sl, sc, sps);

    int32_t A0 = 0, C0 = 0;
    bool touched = (r2 > r1);
    for (uint32_t r = r0 + lane; r < r1; r += 64) {
        uint32_t d, s;
        bool done;
        get_entry<PACKED>(buf, n_cap, sl.off + r, d, done, s, s_scalar, F, sl.tau);
        const int32_t st = (int32_t)(start_offset(r, sl.tau, sc, sps) - t_s); /* in (-tau, 0) */
        const int32_t en = st + (int32_t)d;
        if (en > 0) { /* still running when the slab begins */
            const int32_t w = (int32_t)s + 1 - st;
            A0 += w;
            C0 += 1;
            if (en < (int32_t)len) {
                atomicAdd(&ev[en], W::end(w));
                touched = true;
            }
        }
    }
    /* Runs that start inside the slab.  Each lane takes a block of consecutive ranks, so the
     * runs of one round sit in one lane (two at a block's edge): their start events are summed
     * in registers and added once, and different lanes work on different rounds -- no lane
     * fights another for a window entry.  The block length is odd, which spreads the lanes'
     * LDS reads over all banks. */
    uint32_t sum_st = 0, n_done = 0; /* per lane: a few runs, offsets below the window size */
    {
        const uint32_t blk = ((r2 - r1 + 63u) >> 6) | 1u;
        const uint32_t rb = r1 + (uint32_t)lane * blk;
        const uint32_t cnt = rb < r2 ? (r2 - rb < blk ? r2 - rb : blk) : 0u;
        /* each subroutine has a loop of its own over the runs that start in the slab */
        if (sps) {
            /* inside a block the start offset is carried from rank to rank (quotient and
             * remainder of r tau / k) instead of divided out each time: per rank the remainder
             * grows by tau mod k, and the offset by floor(tau / k) and one more when it wraps */
            uint32_t f = 0, rem = 0;
            if (cnt) {
                f = kvs_div(rb * sl.tau, sc.div);
                rem = rb * sl.tau - f * sc.k;
            }
            const uint32_t q_step = kvs_div(sl.tau, sc.div);
            const uint32_t r_step = sl.tau - q_step * sc.k;
            uint32_t cur = f - t_s, accS = 0, accN = 0;
            auto one = [&](uint32_t w, uint32_t at) {
                uint32_t d, s;
                bool done;
                entry_of_word<PACKED>(w, buf, n_cap, at, d, done, s, F, sl.tau);
                const uint32_t st = f - t_s; /* in [0, len) */
                if (st != cur) { /* cur is the round of the run before: something is held */
                    atomicAdd(&ev[cur], W::starts(accN, (int32_t)(accS - __umul24(accN, cur))));
                    accS = 0;
                    accN = 0;
                }
                cur = st;
                accS += s + 1u;
                accN += 1u;
                const uint32_t en = st + d;
                if (en < len)
                    atomicAdd(&ev[en], W::end((int32_t)((s + 1u) - st)));
                if (!F.all_done) { /* else the caller has the sum of the start offsets in closed form */
                    sum_st += done ? st : 0u;
                    n_done += done ? 1u : 0u;
                }
                rem += r_step;
                const bool over = rem >= sc.k;
                rem -= over ? sc.k : 0u;
                f += q_step + (over ? 1u : 0u);
            };
            const uint32_t pos = sl.off + rb;
            uint32_t j = 0;
            for (; j + 3u < cnt; j += 4u) { /* four entries per round trip to LDS */
                const uint32_t w0 = buf[pos + j], w1 = buf[pos + j + 1u], w2 = buf[pos + j + 2u], w3 = buf[pos + j + 3u];
                one(w0, pos + j);
                one(w1, pos + j + 1u);
                one(w2, pos + j + 2u);
                one(w3, pos + j + 3u);
            }
            for (; j < cnt; j++)
                one(buf[pos + j], pos + j);
            if (accN)
                atomicAdd(&ev[cur], W::starts(accN, (int32_t)(accS - __umul24(accN, cur))));
        } else {
            /* SimS: the runs of a batch start together, so a block is gone through batch by
             * batch with the round fixed, and each stretch adds its start events once */
            uint32_t left = cnt, pos = sl.off + rb, inb = 0, st = 0;
            if (cnt) {
                const uint32_t b = kvs_div(rb, sc.div);
                inb = rb - b * sc.k;       /* place of the first rank in its batch */
                st = b * sl.tau - t_s;     /* in [0, len) */
            }
            while (left) {
                uint32_t seg = sc.k - inb;
                seg = seg < left ? seg : left;
                uint32_t accS = 0, seg_done = 0;
                auto one = [&](uint32_t w, uint32_t at) {
                    uint32_t d, s;
                    bool done;
                    entry_of_word<PACKED>(w, buf, n_cap, at, d, done, s, F, sl.tau);
                    accS += s + 1u;
                    const uint32_t en = st + d;
                    if (en < len)
                        atomicAdd(&ev[en], W::end((int32_t)((s + 1u) - st)));
                    if (!F.all_done)
                        seg_done += done ? 1u : 0u;
                };
                uint32_t j = 0;
                for (; j + 3u < seg; j += 4u) { /* four entries per round trip to LDS */
                    const uint32_t w0 = buf[pos + j], w1 = buf[pos + j + 1u], w2 = buf[pos + j + 2u], w3 = buf[pos + j + 3u];
                    one(w0, pos + j);
                    one(w1, pos + j + 1u);
                    one(w2, pos + j + 2u);
                    one(w3, pos + j + 3u);
                }
                for (; j < seg; j++)
                    one(buf[pos + j], pos + j);
                atomicAdd(&ev[st], W::starts(seg, (int32_t)(accS - __umul24(seg, st))));
                if (!F.all_done) { /* st < 2^10, a stretch is a part of a lane's block */
                    sum_st += __umul24(seg_done, st);
                    n_done += seg_done;
                }
                pos += seg;
                left -= seg;
                inb = 0;
                st += sl.tau;
            }
        }
    }
    if (!F.all_done) /* else the caller has the sum in closed form */
        sumF += (unsigned long long)sum_st + (unsigned long long)n_done * (unsigned long long)t_s;
    if (r0 < r1) { /* the same for every lane */
        A0 = wave_sum(A0);
        C0 = wave_sum(C0);
    }
    if (!__any(touched)) {
        /* nothing starts or ends inside: the occupancy only grows, the last round is the largest */
        const int32_t occ = A0 + (int32_t)(len - 1u) * C0;
        pk = occ > pk ? occ : pk;
        return;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    constexpr int kPer = (NARROW ? 2 * WIN : WIN) / 64; /* window entries per lane, at most */
    int32_t la[kPer], lc[kPer];
    int32_t sa = 0, sc_ = 0;
#pragma unroll
    for (int j = 0; j < kPer; j++) {
        const typename W::T e = (j < per) ? ev[lane * per + j] : (typename W::T)0;
        W::decode(e, la[j], lc[j]);
        sa += la[j];
        sc_ += lc[j];
    }
    int32_t A = A0 + wave_prefix_add(sa) - sa;
    int32_t C = C0 + wave_prefix_add(sc_) - sc_;
#pragma unroll
    for (int j = 0; j < kPer; j++) {
        if (j < per) {
            A += la[j];
            C += lc[j];
            const int32_t t = lane * per + j;
            const int32_t occ = A + __mul24(t, C); /* t < 2^10, |C| < 2^22 by the range check */
            if ((uint32_t)t < len && occ > pk)
                pk = occ;
        }
    }
}

/*
 * A phase of at most 64 runs, by one wavefront, one run per lane.  The
 * occupancy can only fall right after a run's last round, so its maximum is
 * attained in the last round of some run: every lane evaluates the round in
 * which its own run ends, summing over all runs of the phase.
 */
template <bool PACKED>
__device__ __forceinline__ void eval_sparse(const Slot &sl, const Sched &sc, bool sps,
                                            const uint32_t *buf, uint32_t n_cap, uint32_t s_scalar,
                                            const EntryFmt &F, int lane, int32_t &pk,
                                            unsigned long long &sumF)
{
    uint32_t d = 0, s = 0, f = 0;
    bool done = false;
    const bool act = (uint32_t)lane < sl.n;
    if (act) {
        get_entry<PACKED>(buf, n_cap, sl.off + (uint32_t)lane, d, done, s, s_scalar, F, sl.tau);
        f = start_offset((uint32_t)lane, sl.tau, sc, sps);
        if (done)
            sumF += f;
    }
    const uint32_t s1 = s + 1u;
    const uint32_t e = f + d;  /* first round after the run */
    const uint32_t t = e - 1u; /* its last round            */
    uint32_t occ = 0;
    for (uint32_t q = 0; q < sl.n; q++) {
        const uint32_t fq = __builtin_amdgcn_readlane(f, (int)q);
        const uint32_t eq = __builtin_amdgcn_readlane(e, (int)q);
        const uint32_t sq = __builtin_amdgcn_readlane(s1, (int)q);
        if (fq <= t && t < eq)
            occ += sq + (t - fq);
    }
    if (act && (int32_t)occ > pk)
        pk = (int32_t)occ;
}

/*
 * 64 consecutive runs of a phase that is long and thin (many more rounds than runs in
 * flight): one run per lane, evaluated like eval_sparse in the last round of the lane's own
 * run, but summing only over the runs that can be active then -- those that started less
 * than tau rounds before that round, a contiguous stretch of at most k + 1 ranks.
 * Cost O(k) per run instead of O(rounds / 64) per phase.
 */
template <bool PACKED>
__device__ __forceinline__ void eval_thin(const Slot &sl, const Sched &sc, bool sps, uint32_t group,
                                          const uint32_t *buf, uint32_t n_cap, uint32_t s_scalar,
                                          const EntryFmt &F, int lane, int32_t &pk,
                                          unsigned long long &sumF)
{
    const uint32_t r = group * 64u + (uint32_t)lane;
    if (r >= sl.n)
        return;
    uint32_t d, s;
    bool done;
    get_entry<PACKED>(buf, n_cap, sl.off + r, d, done, s, s_scalar, F, sl.tau);
    const uint32_t f = start_offset(r, sl.tau, sc, sps);
    if (done)
        sumF += f;
    const uint32_t t = f + d - 1u; /* the run's last round */
    const uint32_t q_lo = ranks_before(t + 1u > sl.tau ? t + 1u - sl.tau : 0u, sl, sc, sps);
    const uint32_t q_hi = ranks_before(t + 1u, sl, sc, sps);
    uint32_t occ = 0;
    auto other = [&](uint32_t word, uint32_t q) {
        uint32_t dq, sq;
        bool doneq;
        entry_of_word<PACKED>(word, buf, n_cap, sl.off + q, dq, doneq, sq, F, sl.tau);
        const uint32_t fq = start_offset(q, sl.tau, sc, sps);
        if (fq <= t && t < fq + dq)
            occ += sq + 1u + (t - fq);
    };
    uint32_t q = q_lo;
    for (; q + 3u < q_hi; q += 4u) { /* four entries per round trip to LDS */
        const uint32_t w0 = buf[sl.off + q], w1 = buf[sl.off + q + 1u], w2 = buf[sl.off + q + 2u],
                       w3 = buf[sl.off + q + 3u];
        other(w0, q);
        other(w1, q + 1u);
        other(w2, q + 2u);
        other(w3, q + 3u);
    }
    for (; q < q_hi; q++)
        other(buf[sl.off + q], q);
    if ((int32_t)occ > pk)
        pk = (int32_t)occ;
}

} // namespace

#endif /* KVS_PHASE_H */
