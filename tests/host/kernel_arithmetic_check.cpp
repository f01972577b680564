/*
 * The arithmetic shortcuts of the HIP kernels, run on the CPU against the plain definitions over
 * (near-)exhaustive input sets.  The sequences under test are NOT re-typed here: this program
 * includes paper_2605_08565_amd/csrc/mxq_arith.hpp, the very header the kernels are built from
 * (make_recip / quot, sixth_of / quarter_of and the scale encode, pow2_code, div_by_T
 * with its range predicates, sf_decode_bias), and compares every DECISION they lead to with
 * exact arithmetic in double precision.  It shares nothing with the oracle.
 *
 * Prints one line per check: "<name> cases=<n> bad=<m>"; exit status 0 iff all bad == 0.
 * Build: g++ -O2 -std=c++17 -ffp-contract=off -mfma -fopenmp.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../paper_2605_08565_amd/csrc/mxq_arith.hpp"

using mxq::f2u;
using mxq::u2f;

/* E2M1 magnitude index by the conversion instruction's rule (RNE, saturate) */
static int e2m1_index(double ay)
{
    return (ay > 0.25) + (ay >= 0.75) + (ay > 1.25) + (ay >= 1.75) + (ay > 2.5) + (ay >= 3.5) + (ay > 5.0);
}
/* the same decision taken exactly: compare v with t*S (exact products in double) */
static int e2m1_index_exact(double v, double S)
{
    static const double t[7] = {0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0};
    static const int incl[7] = {0, 1, 0, 1, 0, 1, 0};
    int m = 0;
    for (int i = 0; i < 7; ++i) m += incl[i] ? (v >= t[i] * S) : (v > t[i] * S);
    return m;
}

/* check 1: quotient decisions for every fp32 mantissa of v, every scale mantissa, and the
 * binades of v/S that contain a rounding threshold */
static long check_quot(long* cases)
{
    long bad = 0, n = 0;
    for (int mi = 0; mi < 8; ++mi) {
        const float S = 1.0f + mi * 0.125f;
        const mxq::Recip r = mxq::make_recip(S);
#pragma omp parallel for reduction(+ : bad, n) schedule(static)
        for (int64_t m = 0; m < (1 << 23); ++m) {
            for (int e = -4; e <= 3; ++e) {
                const float v = ldexpf(u2f(0x3F800000u | (uint32_t)m), e);
                const int a = e2m1_index((double)mxq::quot(v, r));
                const int b = e2m1_index_exact((double)v, (double)S);
                ++n;
                if (a != b) ++bad;
            }
        }
    }
    *cases = n;
    return bad;
}

/* the kernel's Round_SF on the bit pattern (clip, then mxq::sf_encode_bits) */
static uint32_t sf_encode(float y, int bias, float maxv)
{
    if (y > maxv) y = maxv;
    return bias == 7 ? mxq::sf_encode_bits<7>(y) : mxq::sf_encode_bits<15>(y);
}
static double sf_value(int bias, int c)
{
    const int e = c >> 3, m = c & 7;
    return e ? ldexp(1.0 + m / 8.0, e - bias) : ldexp((double)m, 1 - bias - 3);
}
/* exact nearest-even code of a/M: walk up from the kernel's answer's neighbourhood */
static int sf_exact(double a, double M, int bias, int maxc)
{
    /* a/M compared with midpoints mu via a ? M*mu (exact: mu has <= 5 significant bits, M <= 3) */
    int lo = 0, hi = maxc;
    while (lo < hi) {                       /* largest c with value(c) <= a/M */
        const int mid = (lo + hi + 1) / 2;
        if (M * sf_value(bias, mid) <= a) lo = mid; else hi = mid - 1;
    }
    if (lo == maxc) return maxc;
    const double mu = (sf_value(bias, lo) + sf_value(bias, lo + 1)) / 2;
    if (a > M * mu) return lo + 1;
    if (a < M * mu) return lo;
    return (lo % 2 == 0) ? lo : lo + 1;
}

static long check_scale_encode(long* cases)
{
    long bad = 0, n = 0;
    for (int f = 0; f < 2; ++f) {
        const int bias = f ? 15 : 7, maxc = f ? 0xFE : 0x7E;
        const float maxv = (float)sf_value(bias, maxc);
        const int e_lo = 1 - bias - 3 - 3, e_hi = (maxc >> 3) - bias + 4;
#pragma omp parallel for reduction(+ : bad, n) schedule(static)
        for (int64_t m = 0; m < (1 << 23); m += 3) {
            for (int e = e_lo; e <= e_hi; ++e) {
                const float a = ldexpf(u2f(0x3F800000u | (uint32_t)m), e);
                const float y6 = mxq::sixth_of(a);
                const float y4 = mxq::quarter_of(a);
                n += 2;
                if ((int)sf_encode(y6, bias, maxv) != sf_exact((double)a, 6.0, bias, maxc)) ++bad;
                if ((int)sf_encode(y4, bias, maxv) != sf_exact((double)a, 4.0, bias, maxc)) ++bad;
            }
        }
    }
    *cases = n;
    return bad;
}

/* check 3: Eq. 1 code from the bit pattern vs floor(log2(a/6)) by exact comparison */
static long check_pow2(long* cases)
{
    long bad = 0, n = 0;
#pragma omp parallel for reduction(+ : bad, n) schedule(static)
    for (int64_t b = 0; b < 0x7F800000LL; b += 5) {
        const float a = u2f((uint32_t)b);
        const int got = (int)mxq::pow2_code(a);
        int want = 0;
        if (a > 0.0f) {
            int ex;
            const double fr = frexp((double)a / 6.0, &ex);    /* a/6 = fr * 2^ex, fr in [.5,1): not exact */
            (void)fr;
            int k = ex - 1;                                   /* candidate floor(log2) */
            while (ldexp(6.0, k) > (double)a) --k;            /* exact comparisons fix it */
            while (ldexp(6.0, k + 1) <= (double)a) ++k;
            want = k + 127;
            if (want < 0) want = 0;
            if (want > 254) want = 254;
        }
        ++n;
        if (got != want) ++bad;
    }
    *cases = n;
    return bad;
}

/* check 4: division by the per-tensor scale, reciprocal + one FMA refinement; the remainder is
 * taken with the opposite sign so that signed zeros survive (every bf16 value includes -0) */
static long check_div(long* cases)
{
    long bad = 0, n = 0;
#pragma omp parallel for reduction(+ : bad, n) schedule(dynamic, 8)
    for (int ti = 0; ti < 3000; ++ti) {
        uint64_t rng = 88172645463325252ull + 7919ull * (uint64_t)ti;
#define NEXT() (rng ^= rng << 13, rng ^= rng >> 7, rng ^= rng << 17, rng)
        uint32_t tm = (uint32_t)(NEXT() & 0x7FFFFF);
        if (ti < 32) tm = 0x7FFFFEu - (uint32_t)ti;           /* near all-ones mantissas */
        const int te = (int)(NEXT() % 41) - 20;
        const float T = ldexpf(u2f(0x3F800000u | tm), te);
        if (!mxq::fast_division_ok(T)) continue;
        const float rT = 1.0f / T;
        for (uint32_t b = 0; b < 0x10000; ++b) {              /* every bf16 value */
            const float v = u2f(b << 16);
            if (isnan(v) || isinf(v)) continue;
            const float q = v / T;
            const float aq = fabsf(q);
            if (aq != 0.0f && (aq < 0x1p-78f || aq > 0x1p90f)) continue;   /* see below */
            ++n;
            if (f2u(mxq::div_by_T(v, T, rT)) != f2u(q)) ++bad;
        }
        for (int k = 0; k < 30000; ++k) {                     /* random fp32 values */
            const uint32_t u = (uint32_t)NEXT();
            const int e = (int)(NEXT() % 121) - 60;
            const float v = ldexpf(u2f(0x3F800000u | (u & 0x7FFFFF)), e) * ((u >> 31) ? -1.0f : 1.0f);
            const float q = v / T;
            const float aq = fabsf(q);
            /* above 2^90 the block's abs-max sends the wavefront to the plain division; below
             * 2^-78 the remainder may underflow and the quotient be off by one ulp, which nothing
             * observes: such an element is either the block's abs-max (< 2^-40: plain division)
             * or quantises to a signed zero with a squared residual that underflows to zero */
            if (aq < 0x1p-78f || aq > 0x1p90f) continue;
            ++n;
            if (f2u(mxq::div_by_T(v, T, rT)) != f2u(q)) ++bad;
        }
    }
    *cases = n;
    return bad;
}

/* check 5: the same division, every case in which it could fail.
 *
 * With r = RN(1/T), q0 = RN(v r) is within 1.5 ulp of Q = v/T, the FMA remainder and the final
 * FMA perturb the exact quotient by less than 3 * 2^-24 ulp before the last rounding, so q1 can
 * differ from RN(Q) only if Q lies that close to a midpoint of two neighbouring floats.  For
 * integer mantissas V, T' in [2^23, 2^24) the distance of Q = V/T' to the midpoint odd/2^k
 * (k = 24 for Q >= 1, 25 for Q < 1) is |N| / (2 T') ulp with N = V 2^k - odd T', a non-zero
 * integer: only |N| < 6 can fail.  This enumerates EVERY (V, T') with |N| <= 64 by solving the
 * congruence V 2^k = N (mod T') and runs the sequence on each; the all-ones mantissa of T is
 * the one the kernel's host code routes to the plain division. */
static int64_t egcd(int64_t a, int64_t b, int64_t* x, int64_t* y)
{
    if (!b) { *x = 1; *y = 0; return a; }
    int64_t x1, y1;
    const int64_t g = egcd(b, a % b, &x1, &y1);
    *x = y1;
    *y = x1 - (a / b) * y1;
    return g;
}
static long check_div_midpoints(long* cases)
{
    long bad = 0, n = 0;
#pragma omp parallel for reduction(+ : bad, n) schedule(dynamic, 4096)
    for (int64_t Tp = (1 << 23); Tp < (1 << 24) - 1; ++Tp) {
        const float T = (float)Tp;
        const float r = 1.0f / T;
        for (int k = 24; k <= 25; ++k) {
            const int64_t lo = (k == 24) ? Tp : (1 << 23), hi = (k == 24) ? (1 << 24) : Tp;   /* V in [lo, hi) */
            int64_t x, y;
            const int64_t g = egcd(((int64_t)1 << k) % Tp, Tp, &x, &y);
            const int64_t m = Tp / g;
            for (int N = -64; N <= 64; ++N) {
                if (N == 0 || N % g) continue;
                int64_t V0 = (int64_t)(((__int128)x * (N / g)) % m);
                if (V0 < 0) V0 += m;
                for (int64_t V = lo + ((V0 - lo) % m + m) % m; V < hi; V += m) {
                    const int64_t M = (int64_t)(((((__int128)V) << k) - N) / Tp);
                    if (!(M & 1)) continue;                     /* next to a float, not to a midpoint */
                    ++n;
                    const float v = (float)V;
                    if (f2u(mxq::div_by_T(v, T, r)) != f2u(v / T)) ++bad;
                }
            }
        }
    }
    *cases = n;
    return bad;
}

/* check 6: the quotient for every finite bf16 value against every finite positive code of both
 * scale formats (value and reciprocal exactly as the kernels' scale table holds them: many of
 * these pairs are exact ties), incl. the sign of zero results */
static long check_quot_bf16(long* cases)
{
    long bad = 0, n = 0;
    for (int f = 0; f < 2; ++f) {
        const int maxc = f ? 0xFE : 0x7E;
#pragma omp parallel for reduction(+ : bad, n) schedule(static)
        for (int c = 1; c <= maxc; ++c) {
            const float S = f ? mxq::sf_decode_bias<15>((uint32_t)c) : mxq::sf_decode_bias<7>((uint32_t)c);
            const mxq::Recip r = mxq::make_recip(S);
            for (uint32_t b = 0; b < 0x10000u; ++b) {
                const float v = u2f(b << 16);
                if (isnan(v) || isinf(v)) continue;
                const float y = mxq::quot(v, r);
                ++n;
                if (e2m1_index(fabs((double)y)) != e2m1_index_exact(fabs((double)v), (double)S)) ++bad;
                if ((f2u(y) >> 31) != (b >> 15)) ++bad;
            }
        }
    }
    *cases = n;
    return bad;
}

/* check 7: scale values built from bits against ldexp, every finite code of both formats; the
 * range predicate of the fast division against its definition */
static long check_decode(long* cases)
{
    long bad = 0, n = 0;
    for (int c = 0; c <= 0x7E; ++c, ++n) bad += ((double)mxq::sf_decode_bias<7>((uint32_t)c) != sf_value(7, c));
    for (int c = 0; c <= 0xFE; ++c, ++n) bad += ((double)mxq::sf_decode_bias<15>((uint32_t)c) != sf_value(15, c));
    for (int64_t b = 0; b < 0x7F800000LL; b += 7, ++n) {
        const float a = u2f((uint32_t)b);
        const bool want = a != 0.0f && (a < 0x1p-40f || a > 0x1p90f);
        bad += (mxq::fast_division_unsafe_amax(a) != want);
    }
    *cases = n;
    return bad;
}

int main(void)
{
    long n, bad, total = 0;
    bad = check_quot(&n);          printf("quotient_decisions cases=%ld bad=%ld\n", n, bad); total += bad;
    bad = check_scale_encode(&n);  printf("scale_encode cases=%ld bad=%ld\n", n, bad); total += bad;
    bad = check_pow2(&n);          printf("pow2_code cases=%ld bad=%ld\n", n, bad); total += bad;
    bad = check_div(&n);           printf("tensor_scale_division cases=%ld bad=%ld\n", n, bad); total += bad;
    bad = check_div_midpoints(&n); printf("tensor_scale_division_midpoints cases=%ld bad=%ld\n", n, bad); total += bad;
    bad = check_quot_bf16(&n);     printf("bf16_quotient_decisions cases=%ld bad=%ld\n", n, bad); total += bad;
    bad = check_decode(&n);        printf("scale_decode_and_range cases=%ld bad=%ld\n", n, bad); total += bad;
    return total == 0 ? 0 : 1;
}
