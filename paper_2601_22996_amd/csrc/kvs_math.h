/*
 * kvs_math.h -- small integer helpers of the schedule-evaluation kernels.
 *
 * Host- and device-callable so that the host tests can drive exactly the
 * arithmetic the kernels use (class index of the geometric ladder, division
 * by a per-phase constant, the largest feasible parallelism).
 *
 * Citations: "Competitive Non-Clairvoyant KV-Cache Scheduling for LLM
 * Inference" (Feng, Yang, Zhang).
 */
#ifndef KVS_MATH_H
#define KVS_MATH_H

#include <stdint.h>

#if defined(__HIPCC__)
#define KVS_HD __host__ __device__ __forceinline__
#else
#define KVS_HD static inline
#endif

/* Count of leading zero bits; 32 for x == 0. */
KVS_HD uint32_t kvs_clz32(uint32_t x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint32_t)__clz((int)x);
#else
    return x ? (uint32_t)__builtin_clz(x) : 32u;
#endif
}

KVS_HD uint32_t kvs_mulhi32(uint32_t a, uint32_t b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32);
#endif
}

/* floor(log2 x) for x >= 1. */
KVS_HD uint32_t kvs_ilog2_floor(uint32_t x) { return 31u - kvs_clz32(x); }

/*
 * Class of a length x on the ladder tau_p = tau0 * 2^p (Algorithm 2: class p
 * holds the lengths in (tau_{p-1}, tau_p], class 0 those up to tau_0):
 * the smallest p >= 0 with tau0 * 2^p >= x.  Needs 1 <= x, tau0 <= 2^30;
 * lg_tau0 = floor(log2 tau0).
 *
 * With g = ceil(log2 x) and m = lg_tau0, 2^m <= tau0 < 2^(m+1) brackets the
 * answer between g - m - 1 and g - m, so one comparison decides.
 */
KVS_HD uint32_t kvs_class_index(uint32_t x, uint32_t tau0, uint32_t lg_tau0)
{
    uint32_t g = (x <= 1u) ? 0u : 32u - kvs_clz32(x - 1u);
    int32_t p1 = (int32_t)g - (int32_t)lg_tau0 - 1;
    if (p1 < 0)
        p1 = 0;
    return ((tau0 << p1) >= x) ? (uint32_t)p1 : (uint32_t)p1 + 1u;
}

/*
 * floor(a / b) for a < 2^63 and 1 <= b < 2^53 whose quotient is below 2^52: one double-precision
 * division and a correction by at most one.  (The quotient of the two roundings and of the
 * division itself is off by less than 1; the remainder, in wrapping 64-bit arithmetic, says
 * which way.)  On the GPU a 64-bit integer division is some hundred instructions of one
 * wavefront while the others wait for the phase tables; this is a dozen.
 */
KVS_HD uint64_t kvs_udiv(uint64_t a, uint64_t b)
{
    uint64_t q = (uint64_t)((double)a / (double)b);
    int64_t r = (int64_t)(a - q * b);
    if (r < 0) {
        q -= 1u;
        r += (int64_t)b;
    }
    if ((uint64_t)r >= b)
        q += 1u;
    return q;
}

/*
 * Level of a length x on an explicit ladder lad[0] <= lad[1] <= ... <= lad[n_lv - 1]
 * (1 <= n_lv <= 64): the number of slices below x, which is the index of the first slice
 * that covers x, or n_lv when none does.  Six halving steps find the largest p <= 63 whose
 * p slices in front are all below x; the last slice of a 64-slice ladder is then looked at
 * on its own.
 */
KVS_HD uint32_t kvs_ladder_level(uint32_t x, const uint32_t *lad, uint32_t n_lv)
{
    uint32_t p = 0;
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
#endif
    for (uint32_t b = 32u; b > 0u; b >>= 1)
        if (p + b - 1u < n_lv && lad[p + b - 1u] < x)
            p += b;
    if (p < n_lv && lad[p] < x)
        p++;
    return p;
}

/*
 * Division of 31-bit dividends by a constant d >= 1 through one multiply-high
 * and a shift: with l = ceil(log2 d) and mul = floor(2^(31+l) / d) + 1,
 * floor(x * mul / 2^(31+l)) = floor(x / d) for every 0 <= x < 2^31
 * (round-up method for N = 31; the error mul*d - 2^(31+l) is at most d <= 2^l).
 */
typedef struct {
    uint32_t mul;   /* 0 encodes d == 1 */
    uint32_t shift; /* l - 1            */
} kvs_divisor_t;

KVS_HD kvs_divisor_t kvs_make_divisor(uint32_t d)
{
    kvs_divisor_t r;
    if (d <= 1u) {
        r.mul = 0u;
        r.shift = 0u;
        return r;
    }
    uint32_t l = 32u - kvs_clz32(d - 1u); /* ceil(log2 d), >= 1 */
    r.mul = (uint32_t)kvs_udiv(((uint64_t)1) << (31u + l), d) + 1u;
    r.shift = l - 1u;
    return r;
}

KVS_HD uint32_t kvs_div(uint32_t x, kvs_divisor_t d)
{
    return d.mul ? (kvs_mulhi32(x, d.mul) >> d.shift) : x;
}

/* gcd(a, b) for a >= 1, by halving and subtracting (no division). */
KVS_HD uint32_t kvs_gcd32(uint32_t a, uint32_t b)
{
    if (b == 0)
        return a;
    const uint32_t za = 31u - kvs_clz32(a & (0u - a)), zb = 31u - kvs_clz32(b & (0u - b)); /* trailing zeros */
    const uint32_t shift = za < zb ? za : zb;
    a >>= za;
    b >>= zb;
    while (a != b) { /* both odd */
        if (a > b) {
            a -= b;
            a >>= 31u - kvs_clz32(a & (0u - a));
        } else {
            b -= a;
            b >>= 31u - kvs_clz32(b & (0u - b));
        }
    }
    return a << shift;
}

/*
 * k*(tau, s) = max{k : Peak(k, tau, s) <= M}, eq. (max-parallelism), with
 * Peak(k, tau, s) = s k + (tau k + tau + k - gcd(tau, k)) / 2 (Lemma "Peak
 * Memory Usage of SPS").  The proof of Lemma "Feasible Parallelism of SPS"
 * rewrites the condition as
 *     k (2s + tau + 1) <= 2M - tau + gcd(tau, k).
 * As 1 <= gcd <= tau, every feasible k is at most K = floor(2M / (2s+tau+1)),
 * and K - 1 is feasible whenever it is positive, so only K has to be tested.
 * Returns 0 if no k >= 1 fits.
 */
KVS_HD uint64_t kvs_kstar(uint64_t tau, uint64_t s, uint64_t M)
{
    uint64_t den = 2u * s + tau + 1u;
    uint64_t K = kvs_udiv(2u * M, den);
    if (K == 0)
        return 0;
    /* gcd(tau, K) = gcd(tau, K mod tau); tau is below 2^32 wherever this is called */
    const uint64_t g = kvs_gcd32((uint32_t)tau, (uint32_t)(K - kvs_udiv(K, tau) * tau));
    /* K * den <= 2M always; compare without forming a negative right side */
    if (K * den + tau <= 2u * M + g)
        return K;
    return K - 1u;
}

/*
 * sum_{i = 0}^{n-1} floor(i * tau / k): the start offsets of Procedure 1 summed
 * over a phase of n jobs (the second part of the ladder term Q_p in the analysis
 * of GBA).  Euclid-like reduction: whole multiples of k in tau are summed in
 * closed form, then the lattice points under the line are counted from the
 * other axis, which swaps the roles of tau and k; O(log) steps.  Needs k >= 1
 * and a result below 2^63 (n <= 2^14, tau < 2^31, k < 2^41 are safe).
 */
KVS_HD uint64_t kvs_floor_sum(uint64_t n, uint64_t k, uint64_t tau)
{
    uint64_t ans = 0, a = tau, m = k, b = 0;
    for (;;) {
        if (a >= m) {
            const uint64_t q = kvs_udiv(a, m);
            ans += (n - 1u) * n / 2u * q;
            a -= q * m;
        }
        if (b >= m) {
            const uint64_t q = kvs_udiv(b, m);
            ans += n * q;
            b -= q * m;
        }
        uint64_t y = a * n + b;
        if (y < m)
            return ans;
        n = kvs_udiv(y, m);
        b = y - n * m;
        uint64_t t = m;
        m = a;
        a = t;
    }
}

#endif /* KVS_MATH_H */
