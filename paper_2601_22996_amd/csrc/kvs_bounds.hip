/*
 * kvs_bounds.hip -- the bounds that frame a schedule's flow time, on gfx950:
 * UpperGBA and the memory-time area lower bound on OPT (analysis of GBA,
 * Steps 3 and 1), and the best list schedule over all orders of a tiny
 * instance.  Paper: "Competitive Non-Clairvoyant KV-Cache Scheduling for LLM
 * Inference" (Feng, Yang, Zhang).
 *
 * Entry points: kvs_flow_bounds, kvs_opt_perm (see kvsched.h).
 */
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <type_traits>

#include "kvs_math.h"
#include "kvs_wave.h"
#include "kvsched.h"
#include "kvsched_test.h"

namespace {

constexpr uint32_t kLenMax = 1u << 30;
constexpr int kWave = 64;
constexpr int kLevels = 32;     /* levels of a ladder base * 2^g that lengths <= 2^30 can reach */
constexpr int kMaxBases = 64;   /* distinct odd parts among the initial slices of a call       */

struct BJobs {
    const int32_t *o, *s;
    int32_t n_inst, n_jobs;
    uint32_t s_scalar;
    uint32_t mant_bits; /* buckets of the area ranking: 2^mant_bits per power of two (0: sort instead) */
    uint64_t M;
};

/* Points of one call: point q has the initial slice base[grp[q]] << shift[q]. */
struct BPoints {
    uint32_t base[kMaxBases];
    uint8_t lg_base[kMaxBases];
    uint8_t grp[KVS_MAX_POINTS];
    uint8_t shift[KVS_MAX_POINTS];
    int32_t n_pts, n_bases;
};

__device__ __forceinline__ uint64_t wave_sum64(uint64_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1)
        v += __shfl_xor(v, d, kWave);
    return v;
}

__device__ __forceinline__ uint64_t wave_max64(uint64_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        uint64_t w = __shfl_xor(v, d, kWave);
        v = w > v ? w : v;
    }
    return v;
}


/* ---- bitonic sort in LDS, 16 keys per thread and pass ---- */


/* One unused word after every 16 keys: a thread that reads 16 consecutive keys and its
 * neighbours then fall into different banks. */
__device__ __forceinline__ uint32_t slot_of(uint32_t i) { return i + (i >> 4); }

template <typename KT> __device__ __forceinline__ void order_pair(KT &a, KT &b)
{
    const KT lo = a < b ? a : b, hi = a < b ? b : a;
    a = lo;
    b = hi;
}

/*
 * The stages j = 2^(b_low + R - 1) .. 2^b_low of the bitonic merge of block
 * length k, fused: a thread takes the 2^R keys whose indices differ only in
 * those R bits, runs the R stages in registers and writes them back.  The
 * direction of a merge is the same for all keys of a thread (bit log2 k of the
 * index); descending blocks are merged ascending on the complemented keys.
 */
template <typename KT, int R, int T>
__device__ __forceinline__ void merge_stages(KT *key, uint32_t n_pad, KT *key2, uint32_t n_pad2, uint32_t k,
                                             uint32_t b_low, uint32_t tid)
{
    /* the groups of the first run, then (while its merges are this long) those of the second */
    const uint32_t g1 = n_pad >> R, g2 = (k <= n_pad2) ? (n_pad2 >> R) : 0u;
    for (uint32_t gg = tid; gg < g1 + g2; gg += T) {
        KT *run = gg < g1 ? key : key2;
        const uint32_t g = gg < g1 ? gg : gg - g1;
        const uint32_t base = ((g >> b_low) << (b_low + R)) | (g & ((1u << b_low) - 1u));
        const KT flip = (base & k) ? ~(KT)0 : (KT)0;
        KT v[1 << R];
#pragma unroll
        for (int e = 0; e < (1 << R); e++)
            v[e] = run[slot_of(base + ((uint32_t)e << b_low))] ^ flip;
#pragma unroll
        for (int bit = R - 1; bit >= 0; bit--)
#pragma unroll
            for (int e = 0; e < (1 << R); e++)
                if (!(e & (1 << bit)))
                    order_pair(v[e], v[e | (1 << bit)]);
#pragma unroll
        for (int e = 0; e < (1 << R); e++)
            run[slot_of(base + ((uint32_t)e << b_low))] = v[e] ^ flip;
    }
    __syncthreads();
}

/* Sorts two runs ascending in the same sequence of passes: key[slot_of(0 .. n_pad-1)] and
 * key2[slot_of(0 .. n_pad2-1)], n_pad >= n_pad2, each a power of two >= 16 (n_pad2 may be 0).
 * Every thread of the workgroup must call it. */
template <typename KT, int T>
__device__ void bitonic_sort(KT *key, uint32_t n_pad, KT *key2, uint32_t n_pad2, uint32_t tid)
{
    /* blocks of 16 consecutive keys: the merges k = 2, 4, 8, 16 entirely in registers */
    const uint32_t g1 = n_pad / 16, g2 = n_pad2 / 16;
    for (uint32_t gg = tid; gg < g1 + g2; gg += T) {
        KT *run = gg < g1 ? key : key2;
        const uint32_t base = (gg < g1 ? gg : gg - g1) * 16;
        KT v[16];
#pragma unroll
        for (int e = 0; e < 16; e++)
            v[e] = run[slot_of(base + e)];
#pragma unroll
        for (int k = 2; k <= 8; k <<= 1)
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1)
#pragma unroll
                for (int e = 0; e < 16; e++)
                    if (!(e & j)) {
                        if (e & k)
                            order_pair(v[e | j], v[e]);
                        else
                            order_pair(v[e], v[e | j]);
                    }
        /* the run of 16 is sorted upwards on its own, and in a longer run by bit 4 of its place */
        const uint32_t len = gg < g1 ? n_pad : n_pad2;
        const KT flip = (len > 16u && (base & 16u)) ? ~(KT)0 : (KT)0;
#pragma unroll
        for (int j = 8; j > 0; j >>= 1)
#pragma unroll
            for (int e = 0; e < 16; e++)
                if (!(e & j)) {
                    KT a = v[e] ^ flip, b = v[e | j] ^ flip;
                    order_pair(a, b);
                    v[e] = a ^ flip;
                    v[e | j] = b ^ flip;
                }
#pragma unroll
        for (int e = 0; e < 16; e++)
            run[slot_of(base + e)] = v[e];
    }
    __syncthreads();
    for (uint32_t m = 5; (1u << m) <= n_pad; m++) {
        const uint32_t k = 1u << m;
        uint32_t b = m; /* stages of the bits b-1 .. 0 are still to do */
        switch (m % 4) {
        case 1: merge_stages<KT, 1, T>(key, n_pad, key2, n_pad2, k, b - 1, tid); b -= 1; break;
        case 2: merge_stages<KT, 2, T>(key, n_pad, key2, n_pad2, k, b - 2, tid); b -= 2; break;
        case 3: merge_stages<KT, 3, T>(key, n_pad, key2, n_pad2, k, b - 3, tid); b -= 3; break;
        default: break;
        }
        for (; b >= 4; b -= 4)
            merge_stages<KT, 4, T>(key, n_pad, key2, n_pad2, k, b - 4, tid);
    }
}

/* The keys are sorted as one or two runs of power-of-two length: all of them in one run when
 * n is close below a power of two, else the first 2^floor(log2 n) in run A and the rest, padded
 * to a power of two, in run B (10 000 keys: 8192 + 2048 instead of 16 384). */
struct TwoRuns {
    uint32_t a, b; /* lengths of the runs, b == 0: one run */
};

__host__ __device__ inline TwoRuns split_runs(uint32_t n)
{
    TwoRuns r;
    uint32_t a = 16;
    while (a * 2u <= n)
        a *= 2u;
    if (n <= a) { /* n <= 16, or a power of two */
        r.a = a;
        r.b = 0;
        return r;
    }
    uint32_t b = 16;
    while (b < n - a)
        b *= 2u;
    if (b == a) {
        r.a = 2u * a;
        r.b = 0;
    } else {
        r.a = a;
        r.b = b;
    }
    return r;
}

/* number of keys below x (or not above it, when `or_equal`) in a sorted run of `len` keys */
template <typename KT>
__device__ __forceinline__ uint32_t rank_in_run(const KT *run, uint32_t len, KT x, bool or_equal)
{
    uint32_t lo = 0, hi = len;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        const KT v = run[slot_of(mid)];
        if (v < x || (or_equal && v == x))
            lo = mid + 1u;
        else
            hi = mid;
    }
    return lo;
}

/*
 * Sorts the n keys laid out as split_runs(n) says (run A at key[slot_of(0..)), run B behind it,
 * padded with the largest value) and returns this thread's share of sum_j (n - j) * key_(j) over
 * the ascending sequence j = 0 .. n-1.  A key's place in that sequence is its place in its own
 * run plus the number of keys of the other run in front of it (equal keys: run A first).
 */
template <typename KT, int T>
__device__ uint64_t ranked_sum(KT *key, uint32_t n, TwoRuns runs, uint32_t tid)
{
    KT *run_b = key + slot_of(runs.a); /* runs.a is a multiple of 16 */
    bitonic_sort<KT, T>(key, runs.a, run_b, runs.b, tid);
    uint64_t sum = 0;
    const uint32_t in_a = n < runs.a ? n : runs.a, in_b = n - in_a; /* real keys; padding sorts behind them */
    for (uint32_t i = tid; i < in_a; i += T) {
        const KT x = key[slot_of(i)];
        const uint32_t j = i + (runs.b ? rank_in_run(run_b, in_b, x, false) : 0u);
        sum += (uint64_t)(n - j) * x;
    }
    for (uint32_t i = tid; i < in_b; i += T) {
        const KT x = run_b[slot_of(i)];
        const uint32_t j = i + rank_in_run(key, in_a, x, true);
        sum += (uint64_t)(n - j) * x;
    }
    return sum;
}

constexpr int64_t kAreaPending = INT64_MIN; /* internal: areas too wide for 32-bit keys, left to the second launch */

/* ---- ranks by buckets ---- */

/* Bucket of a key a >= 1: the position of its leading bit and the mb bits below it; keys below
 * 2^mb have a bucket each.  Non-decreasing in a, so all keys of a lower bucket are smaller. */
__device__ __forceinline__ uint32_t bucket_of(uint32_t a, uint32_t mb)
{
    const uint32_t t = 31u - (uint32_t)__clz((int)a);
    return t < mb ? a : (((t - mb + 1u) << mb) | ((a >> (t - mb)) & ((1u << mb) - 1u)));
}
__host__ __device__ inline uint32_t bucket_count(uint32_t mb) { return (33u - mb) << mb; }

/* A bucket with more keys than this sends the instance to the sort: every key is compared with
 * all keys of its bucket, which is cheap only while buckets are small. */
constexpr uint32_t kBucketLimit = 128;

/*
 * One workgroup per instance (T threads, n_jobs <= 16 T).  LDS holds only the sort keys --
 * 32-bit in the first launch
 * (WIDE = false), which leaves an instance whose largest area needs more to the second launch
 * with 64-bit keys (WIDE = true, twice the LDS, one workgroup per compute unit instead of two)
 * -- beside the bucket table of the first launch, and per wavefront one histogram of the levels
 * of the current base.
 *
 * 1. load and check the jobs, find the largest area; the level histogram of the first base is
 *    counted on the way;
 * 2. UpperGBA (first launch only): per distinct base the jobs are counted and the largest
 *    prompt kept per level g (smallest g with base * 2^g >= o; further bases read the jobs
 *    again, from cache).  The class of a job at the point base * 2^m is max(0, g - m), so a
 *    point's class table is the level table with the levels 0..m merged.  32 consecutive lanes
 *    take the classes of one point: each computes k_p, Q_p and floor(n_p tau_p / k_p) + tau_p,
 *    a prefix sum over the lanes gives S_p, a sum n_p S_p + Q_p the bound (Step 3 of the
 *    analysis of GBA);
 * 3. the sum of (n - j) * area_j over the ascending sequence j = 0 .. n-1 (Step 1, proof of the
 *    lower bound).  First launch: the areas (jobs read again, from cache) are dealt into buckets
 *    by their leading bits and a key's place is its bucket's start plus its rank among the keys
 *    of its bucket; an instance with a crowded bucket, and the second launch, sort the areas as
 *    one or two runs instead (bitonic, 16 keys per thread, up to four stages per pass over LDS).
 */
template <int T, bool WIDE>
__global__ __launch_bounds__(T, (T == 1024 && !WIDE) ? 8 : 1) void kvs_bounds_kernel(BJobs J, BPoints P, int64_t *upper,
                                                        int64_t *area_num)
{
    using KT = typename std::conditional<WIDE, uint64_t, uint32_t>::type;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    KT *key = reinterpret_cast<KT *>(lds_raw);
    constexpr int NW = T / kWave;
    __shared__ uint32_t hist[NW][kLevels];
    __shared__ uint32_t smax_lv[kLevels];
    __shared__ uint32_t cnt_lv[kLevels];
    __shared__ uint32_t bad;
    __shared__ uint64_t red[NW];

    const uint32_t inst = blockIdx.x, tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const uint32_t n = (uint32_t)J.n_jobs;
    const size_t row = (size_t)inst * n;
    if (WIDE && area_num[inst] != kAreaPending)
        return; /* the first launch has finished this instance */
    const bool want_upper = !WIDE && upper && P.n_pts > 0;

    auto clear_hist = [&]() {
        for (uint32_t i = tid; i < NW * kLevels; i += T)
            (&hist[0][0])[i] = 0;
        if (tid < kLevels)
            smax_lv[tid] = 0;
    };
    /* a job as it counts: an invalid one marks the instance and is replaced by (o, s) = (1, 0) */
    auto read_job = [&](uint32_t i, uint32_t &o, uint32_t &s) -> bool {
        const int32_t oi = J.o[row + i];
        const int64_t si = J.s ? (int64_t)J.s[row + i] : (int64_t)J.s_scalar;
        const bool ok = !(oi < 1 || si < 0 || (uint32_t)oi > kLenMax || si > (int64_t)kLenMax ||
                          (uint64_t)si + (uint64_t)oi > J.M);
        o = ok ? (uint32_t)oi : 1u;
        s = ok ? (uint32_t)si : 0u;
        return ok;
    };
    auto count_level = [&](uint32_t o, uint32_t s, uint32_t base, uint32_t lg) {
        const uint32_t g = kvs_class_index(o, base, lg);
        atomicAdd(&hist[wave][g], 1u);
        if (s > smax_lv[g])
            atomicMax(&smax_lv[g], s);
    };

    if (tid == 0)
        bad = 0;
    if (want_upper)
        clear_hist();
    __syncthreads();

    /* 1. load */
    auto area_of = [](uint32_t o, uint32_t s) { /* Area(o, s) < 2^61 */
        return (uint64_t)s * o + (uint64_t)o * (o + 1u) / 2u;
    };
    uint64_t amax = 0;
    uint32_t my_bad = 0;
    for (uint32_t i = tid; i < n; i += T) {
        uint32_t o, s;
        if (!read_job(i, o, s))
            my_bad = 1;
        const uint64_t a = area_of(o, s);
        amax = a > amax ? a : amax;
        if (want_upper)
            count_level(o, s, P.base[0], P.lg_base[0]);
    }
    if (my_bad)
        atomicOr(&bad, 1u);
    __syncthreads();
    const bool invalid = bad != 0;

    /* 2. class tables and UpperGBA: 32 consecutive lanes hold the 32 classes of one point */
    if (want_upper) {
        for (int b = 0; b < P.n_bases; b++) {
            const uint32_t base = P.base[b], lg = P.lg_base[b];
            if (b > 0) {
                clear_hist();
                __syncthreads();
                for (uint32_t i = tid; i < n; i += T) {
                    uint32_t o, s;
                    read_job(i, o, s);
                    count_level(o, s, base, lg);
                }
                __syncthreads();
            }
            if (tid < kLevels) {
                uint32_t c = 0;
                for (int w = 0; w < NW; w++)
                    c += hist[w][tid];
                cnt_lv[tid] = c;
            }
            __syncthreads();
            for (uint32_t item0 = 0; item0 < (uint32_t)P.n_pts * kLevels; item0 += T) {
                const uint32_t item = item0 + tid;
                const uint32_t q = item / kLevels, p = item % kLevels; /* p == lane % 32 */
                const bool mine = q < (uint32_t)P.n_pts && P.grp[q < KVS_MAX_POINTS ? q : 0] == b;
                const uint32_t m = mine ? P.shift[q] : 0u;
                uint32_t np = 0, sp = 0;
                if (mine && p == 0) {
                    for (uint32_t g = 0; g <= m && g < kLevels; g++) {
                        np += cnt_lv[g];
                        sp = smax_lv[g] > sp ? smax_lv[g] : sp;
                    }
                } else if (mine && p + m < kLevels) {
                    np = cnt_lv[p + m];
                    sp = smax_lv[p + m];
                }
                const uint64_t tau = ((uint64_t)base << m) << p; /* < 2^62 */
                uint64_t Q = 0, L = tau;                         /* L = floor(n tau / k) + tau */
                uint32_t wide = 0;
                if (np > 0) {
                    if ((uint64_t)np * tau >= (1ull << 31)) {
                        wide = 1;
                    } else {
                        uint64_t k = kvs_kstar(tau, sp, J.M);
                        k = k < 1 ? 1 : k;
                        Q = (uint64_t)np * tau + kvs_floor_sum(np, k, tau);
                        L = ((uint64_t)np * tau) / k + tau;
                    }
                }
                /* S_p: exclusive prefix sum of L over the 32 lanes of the point */
                uint64_t S = L;
#pragma unroll
                for (int d = 1; d < kLevels; d <<= 1) {
                    const uint64_t v = __shfl_up(S, d, kLevels);
                    if ((int)p >= d)
                        S += v;
                }
                S -= L;
                uint64_t term = (uint64_t)np * S + Q;
#pragma unroll
                for (int d = kLevels / 2; d >= 1; d >>= 1) {
                    term += __shfl_xor(term, d, kLevels);
                    wide |= __shfl_xor(wide, d, kLevels);
                }
                if (mine && p == 0)
                    upper[(size_t)q * J.n_inst + inst] = (invalid || wide) ? -1 : (int64_t)term;
            }
            __syncthreads();
        }
    }

    if (!area_num)
        return;

    /* 3. areas, sorted ascending */
    amax = wave_max64(amax);
    if (lane == 0)
        red[wave] = amax;
    __syncthreads();
    amax = 0;
    for (int w = 0; w < NW; w++)
        amax = red[w] > amax ? red[w] : amax;
    __syncthreads();
    if (invalid) {
        if (tid == 0)
            area_num[inst] = -1;
        return;
    }
    if (!WIDE && amax >= 0xffffffffull) { /* needs 64-bit keys (the padding takes the largest 32-bit value) */
        if (tid == 0)
            area_num[inst] = kAreaPending;
        return;
    }
    if (!WIDE && J.mant_bits != 0) {
        /* 3a. The place of a key in the ascending sequence without sorting everything: the keys
         * are dealt into buckets by their leading bits (a counting sort: count, running sums,
         * scatter; inside a bucket in any order), and a key's place is where its bucket begins
         * plus the number of keys of its bucket that are smaller, or equal and in front of it. */
        const uint32_t mb = J.mant_bits, nb = bucket_count(mb);
        uint32_t *const srt = reinterpret_cast<uint32_t *>(lds_raw); /* n keys in bucket order */
        uint32_t *const cntb = srt + n;                              /* nb + 1 counts, then starts */
        __shared__ uint32_t scan_w[NW];
        __shared__ uint32_t biggest;
        for (uint32_t i = tid; i <= nb; i += T)
            cntb[i] = 0;
        if (tid == 0)
            biggest = 0;
        __syncthreads();
        uint32_t my_a[16], my_bp[16]; /* this thread's keys, and bucket << 16 | place in the bucket */
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const uint32_t i = tid + (uint32_t)k * T;
            my_a[k] = 0;
            my_bp[k] = 0;
            if (i < n) { /* the jobs again, from cache */
                uint32_t o, s;
                read_job(i, o, s);
                const uint32_t a = (uint32_t)area_of(o, s);
                const uint32_t b = bucket_of(a, mb);
                my_a[k] = a;
                my_bp[k] = (b << 16) | atomicAdd(&cntb[b], 1u);
            }
        }
        __syncthreads();
        /* running sums over the buckets: every thread takes a stretch of them */
        {
            const uint32_t per = (nb + T) / T; /* covers the nb + 1 entries */
            const uint32_t lo = tid * per, hi = lo + per < nb + 1u ? lo + per : nb + 1u;
            uint32_t sum = 0, mx = 0;
            for (uint32_t b = lo; b < hi; b++) {
                const uint32_t c = cntb[b];
                sum += c;
                mx = c > mx ? c : mx;
            }
            const uint32_t incl = (uint32_t)wave_prefix_add((int32_t)sum);
            if (lane == kWave - 1)
                scan_w[wave] = incl;
            mx = (uint32_t)wave_max_nonneg((int32_t)mx);
            if (lane == 0)
                atomicMax(&biggest, mx);
            __syncthreads();
            uint32_t before = incl - sum;
            for (uint32_t w = 0; w < wave; w++)
                before += scan_w[w];
            for (uint32_t b = lo; b < hi; b++) {
                const uint32_t c = cntb[b];
                cntb[b] = before;
                before += c;
            }
        }
        __syncthreads();
        if (biggest <= kBucketLimit) {
#pragma unroll
            for (int k = 0; k < 16; k++) {
                const uint32_t i = tid + (uint32_t)k * T;
                if (i < n)
                    srt[cntb[my_bp[k] >> 16] + (my_bp[k] & 0xffffu)] = my_a[k];
            }
            __syncthreads();
            /* consecutive lanes take consecutive places, so a wavefront's lanes look at the same
             * few buckets */
            uint64_t sum = 0;
            for (uint32_t p = tid; p < n; p += T) {
                const uint32_t a = srt[p];
                const uint32_t b = bucket_of(a, mb);
                const uint32_t lo = cntb[b], hi = cntb[b + 1u];
                uint32_t r = 0;
                auto cmp = [&](uint32_t v, uint32_t q) { r += (v < a || (v == a && q < p)) ? 1u : 0u; };
                uint32_t q = lo;
                for (; q + 3u < hi; q += 4u) { /* four keys per round trip to LDS */
                    const uint32_t v0 = srt[q], v1 = srt[q + 1u], v2 = srt[q + 2u], v3 = srt[q + 3u];
                    cmp(v0, q);
                    cmp(v1, q + 1u);
                    cmp(v2, q + 2u);
                    cmp(v3, q + 3u);
                }
                for (; q < hi; q++)
                    cmp(srt[q], q);
                sum += (uint64_t)(n - (lo + r)) * a;
            }
            sum = wave_sum64(sum);
            if (lane == 0)
                red[wave] = sum;
            __syncthreads();
            if (tid == 0) {
                uint64_t tot = 0;
                for (int w = 0; w < NW; w++)
                    tot += red[w];
                const uint64_t tri = (uint64_t)n * (n + 1u) / 2u;
                const bool wide = __umul64hi(tri, amax) != 0 || tri * amax >= (1ull << 63);
                area_num[inst] = wide ? -1 : (int64_t)tot;
            }
            return;
        }
        __syncthreads(); /* a crowded bucket: the sort below takes over the same memory */
    }
    const TwoRuns runs = split_runs(n);
    const uint32_t b0 = slot_of(runs.a); /* where run B begins */
    for (uint32_t i = tid; i < runs.a + runs.b; i += T) { /* the jobs again, from cache */
        KT a = (KT) ~(KT)0; /* padding sorts to the end */
        if (i < n) {
            uint32_t o, s;
            read_job(i, o, s);
            a = (KT)area_of(o, s);
        }
        key[i < runs.a ? slot_of(i) : b0 + slot_of(i - runs.a)] = a;
    }
    __syncthreads();
    uint64_t sum = ranked_sum<KT, T>(key, n, runs, tid);
    sum = wave_sum64(sum);
    if (lane == 0)
        red[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        uint64_t tot = 0;
        for (int w = 0; w < NW; w++)
            tot += red[w];
        const uint64_t tri = (uint64_t)n * (n + 1u) / 2u;
        const bool wide = __umul64hi(tri, amax) != 0 || tri * amax >= (1ull << 63);
        area_num[inst] = wide ? -1 : (int64_t)tot;
    }
}

/* ---- best list schedule over all orders ---- */

constexpr int kPermT = 256;          /* threads per workgroup                  */
constexpr int kPN = KVS_MAX_PERM_JOBS;
constexpr uint64_t kPermRounds = KVS_MAX_PERM_ROUNDS; /* largest sum of lengths of an instance */

__global__ void kvs_opt_init_kernel(BJobs J, int64_t *best)
{
    const uint32_t inst = blockIdx.x * blockDim.x + threadIdx.x;
    if (inst >= (uint32_t)J.n_inst)
        return;
    bool ok = true;
    uint64_t total = 0;
    for (int j = 0; j < J.n_jobs; j++) {
        const int32_t o = J.o[(size_t)inst * J.n_jobs + j];
        ok = ok && o >= 1 && (uint32_t)o <= kLenMax && (uint64_t)J.s_scalar + (uint64_t)o <= J.M;
        total += ok ? (uint64_t)o : 0u;
    }
    best[inst] = (ok && total <= kPermRounds) ? INT64_MAX : -1;
}

/*
 * Earliest start, not before `prev`, of a run of length o on top of the J runs already placed
 * (starts S_of[0..J), ends E_of[0..J), all started at or before prev).  From the candidate
 * start S on, the placed load only falls when one of them ends and rises by one per job and
 * round in between: the new run fits iff it fits in its own last round and in the last round
 * of every placed run that ends inside it.  When some round t is over the budget by x, every
 * start before min(S + x, t + 1) still has round t inside the run and still over the budget,
 * so the search jumps there instead of trying them.
 */
template <int J>
__host__ __device__ inline int64_t earliest_start(const int64_t *S_of, const int64_t *E_of, int64_t o,
                                                   int64_t prev, int64_t s1, int64_t M)
{
    int64_t S = prev;
    for (;;) {
        const int64_t E = S + o;
        int64_t jump = 0;
#pragma unroll
        for (int c = 0; c <= J; c++) {
            int64_t t;
            if (c == J)
                t = E - 1;
            else if (E_of[c] > S && E_of[c] < E)
                t = E_of[c] - 1;
            else
                continue;
            int64_t occ = s1 + (t - S);
#pragma unroll
            for (int i = 0; i < J; i++)
                if (E_of[i] > t) /* started at or before S <= t */
                    occ += s1 + (t - S_of[i]);
            if (occ > M) {
                const int64_t by = occ - M < t + 1 - S ? occ - M : t + 1 - S;
                jump = by > jump ? by : jump;
            }
        }
        if (jump == 0)
            return S;
        S += jump;
    }
}

/* Takes the c-th of the job ids packed four bits each into `avail` and closes the gap. */
__host__ __device__ inline uint32_t take_job(uint64_t &avail, uint32_t c)
{
    const uint32_t id = (uint32_t)(avail >> (4 * c)) & 15u;
    const uint64_t low = avail & ((1ull << (4 * c)) - 1ull);
    avail = low | ((avail >> (4 * c + 4)) << (4 * c));
    return id;
}

/*
 * All orders of the jobs still in `avail` behind the J runs already placed, depth first: an
 * order's list schedule shares the placement of every prefix with the orders that begin alike,
 * so a prefix is placed once for all of them.  Keeps the smallest flow time in `best`.
 */
template <int N, int J>
__host__ __device__ inline void orders_below(uint64_t avail, int64_t *S_of, int64_t *E_of, int64_t prev,
                                             int64_t flow, const uint32_t *len, int64_t s1, int64_t M,
                                             int64_t &best)
{
    if constexpr (J == N) {
        best = flow < best ? flow : best;
    } else {
        for (uint32_t c = 0; c < (uint32_t)(N - J); c++) {
            uint64_t rest = avail;
            const int64_t o = len[take_job(rest, c)];
            const int64_t S = earliest_start<J>(S_of, E_of, o, prev, s1, M);
            S_of[J] = S;
            E_of[J] = S + o;
            orders_below<N, J + 1>(rest, S_of, E_of, S, flow + S + o, len, s1, M, best);
        }
    }
}

constexpr int kPermTail = 4; /* the last jobs of an order are enumerated by one thread */

template <int N> struct PermShape {
    static constexpr int D = N < kPermTail ? N : kPermTail; /* jobs in a thread's subtree   */
    static constexpr int P = N - D;                         /* jobs in the prefix that names it */
};

/*
 * Work unit `unit` of an instance of N jobs: the prefix of N - D jobs it names in the factorial
 * number system (digit j picks among the N - j jobs not yet placed) is placed, then all D!
 * orders of the rest are evaluated.  Returns the smallest flow time among them.
 */
template <int N>
__host__ __device__ inline int64_t best_of_unit(uint32_t unit, const uint32_t *len, int64_t s1, int64_t M)
{
    constexpr int P = PermShape<N>::P;
    uint64_t avail = 0x9876543210ull;
    int64_t S_of[N], E_of[N];
    int64_t prev = 0, flow = 0;
    auto place = [&](auto jc) {
        constexpr int J = decltype(jc)::value;
        const uint32_t radix = (uint32_t)(N - J);
        const uint32_t d = unit % radix;
        unit /= radix;
        const int64_t o = len[take_job(avail, d)];
        const int64_t S = earliest_start<J>(S_of, E_of, o, prev, s1, M);
        S_of[J] = S;
        E_of[J] = S + o;
        prev = S;
        flow += S + o;
    };
    /* P <= 6 prefix positions, each with its own compile-time count of placed runs */
    if constexpr (P > 0) place(std::integral_constant<int, 0>{});
    if constexpr (P > 1) place(std::integral_constant<int, 1>{});
    if constexpr (P > 2) place(std::integral_constant<int, 2>{});
    if constexpr (P > 3) place(std::integral_constant<int, 3>{});
    if constexpr (P > 4) place(std::integral_constant<int, 4>{});
    if constexpr (P > 5) place(std::integral_constant<int, 5>{});
    static_assert(P <= 6, "prefix positions");
    int64_t best = INT64_MAX;
    orders_below<N, P>(avail, S_of, E_of, prev, flow, len, s1, M, best);
    return best;
}

/* number of work units of an instance of n jobs: n! / D! */
__host__ __device__ inline uint32_t perm_units(int n)
{
    const int d = n < kPermTail ? n : kPermTail;
    uint32_t u = 1;
    for (int j = d + 1; j <= n; j++)
        u *= (uint32_t)j;
    return u;
}

/*
 * Workgroup (instance, chunk): every thread evaluates one work unit and the minimum goes to
 * best[instance] with one atomic per wavefront.
 */
template <int N>
__global__ __launch_bounds__(kPermT) void kvs_opt_perm_kernel(BJobs J, int64_t *best, uint32_t n_units,
                                                               uint32_t chunks)
{
    const uint32_t inst = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
    __shared__ uint32_t len[kPN];
    if (threadIdx.x < (uint32_t)N)
        len[threadIdx.x] = (uint32_t)J.o[(size_t)inst * N + threadIdx.x];
    __syncthreads();
    if (best[inst] < 0) /* invalid or too long: reported by the first kernel */
        return;
    const int64_t s1 = (int64_t)J.s_scalar + 1, M = (int64_t)J.M;
    const uint32_t unit = chunk * kPermT + threadIdx.x;
    int64_t mine = INT64_MAX;
    if (unit < n_units)
        mine = best_of_unit<N>(unit, len, s1, M);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int64_t w = __shfl_xor(mine, d, kWave);
        mine = w < mine ? w : mine;
    }
    if (threadIdx.x % kWave == 0 && mine != INT64_MAX)
        atomicMin(reinterpret_cast<long long *>(best + inst), (long long)mine);
}

template <int N>
void launch_opt_perm(const BJobs &J, int64_t *best, uint32_t n_units, uint32_t chunks, hipStream_t st)
{
    hipLaunchKernelGGL(kvs_opt_perm_kernel<N>, dim3(chunks * (uint32_t)J.n_inst), dim3(kPermT), 0, st, J,
                       best, n_units, chunks);
}

/* smallest flow time of one work unit, on the host (tests) */
int64_t host_best_of_unit(int n, uint32_t unit, const uint32_t *len, int64_t s1, int64_t M)
{
    switch (n) {
    case 1: return best_of_unit<1>(unit, len, s1, M);
    case 2: return best_of_unit<2>(unit, len, s1, M);
    case 3: return best_of_unit<3>(unit, len, s1, M);
    case 4: return best_of_unit<4>(unit, len, s1, M);
    case 5: return best_of_unit<5>(unit, len, s1, M);
    case 6: return best_of_unit<6>(unit, len, s1, M);
    case 7: return best_of_unit<7>(unit, len, s1, M);
    case 8: return best_of_unit<8>(unit, len, s1, M);
    case 9: return best_of_unit<9>(unit, len, s1, M);
    case 10: return best_of_unit<10>(unit, len, s1, M);
    default: return -1;
    }
}

int32_t check_bound_jobs(const kvs_jobs_t *jobs)
{
    if (!jobs || jobs->n_instances < 0 || jobs->n_jobs < 1)
        return KVS_EINVAL;
    if (jobs->n_instances > 0 && !jobs->o)
        return KVS_EINVAL;
    if (jobs->M < 1 || jobs->M >= (1ll << 40))
        return KVS_EINVAL;
    if (!jobs->s && (jobs->s_scalar < 0 || (uint32_t)jobs->s_scalar > kLenMax))
        return KVS_EINVAL;
    return KVS_OK;
}

BJobs to_bjobs(const kvs_jobs_t *jobs)
{
    BJobs J;
    J.o = jobs->o;
    J.s = jobs->s;
    J.n_inst = jobs->n_instances;
    J.n_jobs = jobs->n_jobs;
    J.s_scalar = jobs->s ? 0u : (uint32_t)jobs->s_scalar;
    J.mant_bits = 0;
    J.M = (uint64_t)jobs->M;
    return J;
}

} // namespace

extern "C" {

int32_t kvs_flow_bounds(const kvs_jobs_t *jobs, const int32_t *tau0, int32_t n_pts,
                        int64_t *upper_gba, int64_t *area_lb_num, void *stream)
{
    int32_t rc = check_bound_jobs(jobs);
    if (rc != KVS_OK)
        return rc;
    if (n_pts < 0 || (n_pts > 0 && (!tau0 || !upper_gba)))
        return KVS_EINVAL;
    if (jobs->n_jobs > KVS_MAX_JOBS || n_pts > KVS_MAX_POINTS)
        return KVS_ELIMIT;
    BPoints P;
    memset(&P, 0, sizeof(P));
    P.n_pts = n_pts;
    for (int32_t q = 0; q < n_pts; q++) {
        if (tau0[q] < 1 || (uint32_t)tau0[q] > kLenMax)
            return KVS_EINVAL;
        const uint32_t m = (uint32_t)__builtin_ctz((uint32_t)tau0[q]);
        const uint32_t base = (uint32_t)tau0[q] >> m;
        int b = 0;
        while (b < P.n_bases && P.base[b] != base)
            b++;
        if (b == P.n_bases) {
            P.base[b] = base;
            P.lg_base[b] = (uint8_t)kvs_ilog2_floor(base);
            P.n_bases++;
        }
        P.grp[q] = (uint8_t)b;
        P.shift[q] = (uint8_t)m;
    }
    if (jobs->n_instances == 0 || (n_pts == 0 && !area_lb_num))
        return KVS_OK;
    /* the runs of keys with one unused slot per 16: 32-bit keys in the first launch, 64-bit in
     * the second, which takes the instances the first one left (areas of 2^32 and more) */
    const uint32_t n = (uint32_t)jobs->n_jobs;
    const TwoRuns runs = split_runs(n);
    const size_t slots = (size_t)runs.a + runs.a / 16 + runs.b + runs.b / 16 + 1;
    /* the first launch ranks by buckets where it can: the keys and the bucket table beside them;
     * 256 buckets per power of two while two workgroups of the largest kind still fit a compute
     * unit's LDS, else 128 */
    BJobs J32 = to_bjobs(jobs);
    J32.mant_bits = (sizeof(uint32_t) * ((size_t)n + bucket_count(8) + 1) <= 72 * 1024) ? 8u : 7u;
    const size_t lds_b = sizeof(uint32_t) * ((size_t)n + bucket_count(J32.mant_bits) + 1);
    const size_t lds64 = sizeof(uint64_t) * slots;
    const size_t lds32 = sizeof(uint32_t) * slots > lds_b ? sizeof(uint32_t) * slots : lds_b;
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto launch = [&](auto kern, int threads, size_t lds) -> int32_t {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return KVS_EHIP;
        hipLaunchKernelGGL(kern, dim3((uint32_t)jobs->n_instances), dim3(threads), lds, st,
                           J32, P, n_pts > 0 ? upper_gba : nullptr, area_lb_num);
        return hipGetLastError() == hipSuccess ? KVS_OK : KVS_EHIP;
    };
    rc = n > 4096   ? launch(kvs_bounds_kernel<1024, false>, 1024, lds32)
         : n > 1024 ? launch(kvs_bounds_kernel<256, false>, 256, lds32)
                    : launch(kvs_bounds_kernel<64, false>, 64, lds32);
    if (rc != KVS_OK || !area_lb_num)
        return rc;
    return n > 4096   ? launch(kvs_bounds_kernel<1024, true>, 1024, lds64)
           : n > 1024 ? launch(kvs_bounds_kernel<256, true>, 256, lds64)
                      : launch(kvs_bounds_kernel<64, true>, 64, lds64);
}

int32_t kvs_opt_perm(const kvs_jobs_t *jobs, int64_t *best_flow, void *stream)
{
    int32_t rc = check_bound_jobs(jobs);
    if (rc != KVS_OK)
        return rc;
    if (jobs->s)
        return KVS_EINVAL;
    if (jobs->n_jobs > KVS_MAX_PERM_JOBS)
        return KVS_ELIMIT;
    if (jobs->n_instances == 0)
        return KVS_OK;
    if (!best_flow)
        return KVS_EINVAL;
    const uint32_t n_units = perm_units(jobs->n_jobs);
    const uint32_t chunks = (n_units + kPermT - 1) / kPermT;
    if ((uint64_t)chunks * (uint64_t)jobs->n_instances > 0x7fffffffull)
        return KVS_ELIMIT;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const BJobs J = to_bjobs(jobs);
    hipLaunchKernelGGL(kvs_opt_init_kernel, dim3((uint32_t)(jobs->n_instances + 255) / 256), dim3(256),
                       0, st, J, best_flow);
    switch (jobs->n_jobs) {
    case 1: launch_opt_perm<1>(J, best_flow, n_units, chunks, st); break;
    case 2: launch_opt_perm<2>(J, best_flow, n_units, chunks, st); break;
    case 3: launch_opt_perm<3>(J, best_flow, n_units, chunks, st); break;
    case 4: launch_opt_perm<4>(J, best_flow, n_units, chunks, st); break;
    case 5: launch_opt_perm<5>(J, best_flow, n_units, chunks, st); break;
    case 6: launch_opt_perm<6>(J, best_flow, n_units, chunks, st); break;
    case 7: launch_opt_perm<7>(J, best_flow, n_units, chunks, st); break;
    case 8: launch_opt_perm<8>(J, best_flow, n_units, chunks, st); break;
    case 9: launch_opt_perm<9>(J, best_flow, n_units, chunks, st); break;
    default: launch_opt_perm<10>(J, best_flow, n_units, chunks, st); break;
    }
    return hipGetLastError() == hipSuccess ? KVS_OK : KVS_EHIP;
}

/* Host-side access to the kernels' arithmetic, for tests without a GPU. */
uint64_t kvs_host_floor_sum(uint64_t n, uint64_t k, uint64_t tau) { return kvs_floor_sum(n, k, tau); }

/* Smallest flow time of work unit `unit` (of kvs_host_perm_units(n)) of one instance. */
int64_t kvs_host_best_of_unit(uint32_t unit, int32_t n, const int32_t *o, int64_t s, int64_t M)
{
    uint32_t len[kPN] = {0};
    if (n < 1 || n > kPN || unit >= perm_units(n))
        return -1;
    for (int j = 0; j < n; j++)
        len[j] = (uint32_t)o[j];
    return host_best_of_unit(n, unit, len, s + 1, M);
}

uint32_t kvs_host_perm_units(int32_t n) { return (n < 1 || n > kPN) ? 0u : perm_units(n); }

} // extern "C"
