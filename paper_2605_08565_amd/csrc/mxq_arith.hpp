// Scalar arithmetic of the libmxq kernels that replaces a literal IEEE division (or a search over
// a value table) by a cheaper instruction sequence.  Every function here is plain fp32 / integer
// C++ without any GPU intrinsic, so the SAME source is compiled twice: by hipcc into the gfx950
// kernels (mxq_device.hpp includes this file) and by the host compiler into
// tests/host/kernel_arithmetic_check.cpp, which runs each sequence over (near-)exhaustive input
// sets against exact arithmetic.  An edit here is therefore re-proved by the CPU test suite.
//
// The operations follow Section 2 of "Finer is Better (with the Right Scaling)": Eq. 1 (power-of-
// two scale), Eq. 2 (abs-max scale rounded to the scale format), the element quotient v / S in
// front of the E2M1 rounding, and the division by the per-tensor scale of hierarchical scaling.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define MXQ_HD __host__ __device__ __forceinline__
#else
#define MXQ_HD inline
#endif

namespace mxq {

MXQ_HD uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
MXQ_HD float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// ---------------------------------------------------------------------------------------
// 8-bit floating-point scale formats with 3 mantissa bits and exponent bias BIAS (Background;
// eps under Eq. 3): E4M3 has bias 7, UE5M3 bias 15.
// ---------------------------------------------------------------------------------------

// Value of a finite scale code: m * 2^(1-bias-3) below the first binade, else
// (1 + m/8) * 2^(e-bias), built directly as fp32 bits.
template <int BIAS>
MXQ_HD float sf_decode_bias(uint32_t code)
{
    const float sub = (float)(code & 7u) * u2f((uint32_t)(127 + 1 - BIAS - 3) << 23);
    const float nrm = u2f((code + ((127u - (uint32_t)BIAS) << 3)) << 20);
    return (code < 8u) ? sub : nrm;
}

// Round_SF of Eq. 2 for 0 <= y <= max_value (the caller clips): round to nearest even into the
// format.  Normal range: RNE of the fp32 mantissa to 3 bits by the usual
// add-half-minus-one-plus-lsb on the bit pattern.  Sub-normal range: adding 2^(emin+20) makes
// the fp32 adder itself round y to a multiple of eps (ties to even).
template <int BIAS>
MXQ_HD uint32_t sf_encode_bits(float y)
{
    const uint32_t b = f2u(y);
    const uint32_t nrm = ((b + 0x7FFFFu + ((b >> 20) & 1u)) >> 20) - ((127u - (uint32_t)BIAS) << 3);
    const float magic = u2f((uint32_t)(127 + (1 - BIAS) + 20) << 23);
    const uint32_t sub = f2u(y + magic) - f2u(magic);
    const float min_normal = u2f((uint32_t)(127 + 1 - BIAS) << 23);
    return (y < min_normal) ? sub : nrm;
}

// ---------------------------------------------------------------------------------------
// Quotients whose rounding decisions are exact.
//
// The method divides in IEEE fp32 (v / S, amax / M) and then rounds the quotient to a very
// coarse grid (E2M1, or an 8-bit scale format).  Only the side of each grid mid-point t the
// quotient falls on matters.  For a divisor d with at most 4 significant bits and a
// mid-point t with at most 5, the product t*d is exact in fp32, and for fp32 v
//     fl32(v / d) <, =, > t   <=>   v <, =, > t*d,
// because v != t*d implies |v/(t*d) - 1| >= 2^-24, which is more than half an ulp of t away.
// The same holds for  y = fl32(v*r_hi + fl32(v*r_lo))  with r_hi + r_lo = 1/d to 2^-47
// relative (r_hi need not be the nearest float for that): y is within 2^-46 relative of v/d
// before its single rounding, far inside the 2^-28 margin the inequality above leaves.  So y
// may stand in for the IEEE quotient wherever only the rounded code is needed.  (The residual
// v - q*S is computed from v, q and S, never from y.)
// ---------------------------------------------------------------------------------------
struct Recip { float hi, lo; };

// r_hi = 1/d rounded toward zero, r_lo = fl32(rho * r_hi) >= 0 with rho = 1 - r_hi*d exact (fma).
// Both parts are non-negative, so both products in quot() carry the sign of v and a zero
// quotient (v = -0, or an underflowing product) keeps the sign bit of v.
MXQ_HD Recip make_recip(float d)
{
    Recip r;
    r.hi = 1.0f / d;
    if (__builtin_fmaf(-r.hi, d, 1.0f) < 0.0f) r.hi = u2f(f2u(r.hi) - 1u);      // was rounded up
    const float rho = __builtin_fmaf(-r.hi, d, 1.0f);
    r.lo = rho * r.hi;
    return r;
}

MXQ_HD float quot(float v, Recip r)
{
    return __builtin_fmaf(v, r.hi, v * r.lo);
}

// A single multiplication by a rounded reciprocal is NOT enough, not even for bf16 inputs with
// their 8 significant bits: an input that sits exactly on a tie (v = t*d) must produce exactly t
// for the ties-to-even rule of the E2M1 rounding, and t*d*fl(1/d) misses t by an ulp for most d
// (the host-side check shows the failures when quot is replaced by one product).

// amax / 6 and amax / 4 in front of Round_SF (Eq. 2, M = 6; Eq. 4, M = 4): the first by the
// two-part reciprocal above (6 has 2 significant bits), the second is exact.
constexpr float kSixthHi = (float)(1.0 / 6.0);
constexpr float kSixthLo = (float)(1.0 / 6.0 - (double)kSixthHi);
MXQ_HD float sixth_of(float amax) { return __builtin_fmaf(amax, kSixthHi, amax * kSixthLo); }
MXQ_HD float quarter_of(float amax) { return amax * 0.25f; }

// Eq. 1: k = floor(log2(amax / 6)).  With amax = m * 2^e, 1 <= m < 2: k = e - 2 when
// m >= 1.5, else e - 3; byte = k + 127, never below 0 (sub-normal or zero amax gives 0).
MXQ_HD uint32_t pow2_code(float amax)
{
    const uint32_t b = f2u(amax);
    const int c = (int)(b >> 23) - 3 + (int)((b >> 22) & 1u);
    return (uint32_t)(c > 0 ? c : 0);
}

// ---------------------------------------------------------------------------------------
// Hierarchical scaling divides every input by the per-tensor scale T in IEEE fp32.  T is the
// same for the whole tensor, so its correctly rounded reciprocal r is formed once and each
// quotient is refined once:
//     q0 = v*r;  q1 = q0 - r*(q0*T - v)                                 (remainder by FMA)
// q0 is within 1.5 ulp of v/T and the value rounded into q1 differs from the exact quotient by
// less than 3 * 2^-24 ulp, so q1 is the correctly rounded quotient unless v/T lies that close
// to the midpoint of two floats; all mantissa pairs that come so close (an integer congruence
// lists them) are checked one by one on the host, the all-ones mantissa of T excluded.  The
// remainder is formed with the opposite sign (q0*T - v) and subtracted, which keeps a signed
// zero: for v = -0 the last step is (-0)*r + (-0) = -0, whereas v - q0*T would give +0 and
// lose the sign.  The argument needs intermediate results free of
// overflow and underflow: the host takes this path only for 2^-20 <= T <= 2^20 with a
// mantissa that is not all ones, and a block whose adjusted abs-max leaves [2^-40, 2^90]
// (zero excepted) sends its whole wavefront through the plain division instead.  An element far
// below its block's abs-max can still have |v/T| < 2^-78, where the remainder may underflow and
// q1 be off by one ulp; nothing observes that: the element quantises to a signed zero and its
// squared residual underflows to zero either way.
// ---------------------------------------------------------------------------------------
MXQ_HD float div_by_T(float v, float T, float rT)
{
    const float q0 = v * rT;
    const float neg_rem = __builtin_fmaf(q0, T, -v);                 // q0*T - v, exact
    return __builtin_fmaf(-neg_rem, rT, q0);
}

// The reciprocal-refined division is exact for these T only.
MXQ_HD bool fast_division_ok(float T)
{
    return T >= 0x1p-20f && T <= 0x1p20f && (f2u(T) & 0x7FFFFFu) != 0x7FFFFFu;
}

// An adjusted block abs-max a >= 0 outside [2^-40, 2^90], zero excepted, falls back to the plain
// division.
MXQ_HD bool fast_division_unsafe_amax(float a)
{
    return (f2u(a) - 0x2B800000u) > (0x6C800000u - 0x2B800000u) && f2u(a) != 0u;
}

// Per-tensor scale of hierarchical scaling (Section 2, two-stage process) from the tensor
// abs-max: the abs-max lands on (largest element magnitude) x (largest scale value); 1 for an
// all-zero tensor or when the quotient vanishes or overflows.
MXQ_HD float tensor_scale_from(float absmax, float sf_max)
{
    if (!(absmax > 0.0f)) return 1.0f;
    const float t = absmax / (6.0f * sf_max);
    return (t > 0.0f && t < __builtin_inff()) ? t : 1.0f;
}

}  // namespace mxq
