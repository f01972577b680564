// Device-side building blocks of libmxq (gfx950): number formats, exact-decision quotients,
// E2M1 rounding, wavefront reductions.  Everything here follows Section 2 of "Finer is Better
// (with the Right Scaling)" (Eq. 1-4); the places where a cheaper instruction sequence
// replaces a literal IEEE division carry the argument for why every rounding DECISION is
// unchanged.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mxq_arith.hpp"      // the division-free sequences, shared with the host-side proof

namespace mxq {

constexpr int kE8M0 = 0, kE4M3 = 1, kUE5M3 = 2;
constexpr int kBF16 = 0, kF32 = 1;

// ---------------------------------------------------------------------------------------
// 8-bit floating-point scale formats (Background; eps under Eq. 3).
// ---------------------------------------------------------------------------------------
template <int FMT> struct ScaleFmt;
template <> struct ScaleFmt<kE4M3> {
    static constexpr int kBias = 7;              // eps = 2^(1-7-3) = 2^-9
    static constexpr int kMaxCode = 0x7E;        // 1.75 * 2^8 = 448
    static constexpr float kMaxValue = 448.0f;
};
template <> struct ScaleFmt<kUE5M3> {
    static constexpr int kBias = 15;             // eps = 2^-17
    static constexpr int kMaxCode = 0xFE;        // 1.75 * 2^16
    static constexpr float kMaxValue = 114688.0f;
};

template <int FMT>
__device__ __forceinline__ float sf_decode(uint32_t code) { return sf_decode_bias<ScaleFmt<FMT>::kBias>(code); }

// Round_SF of Eq. 2: round-to-nearest-even of y >= 0 into the format, clipped to the largest
// finite value.  For E4M3 the gfx950 conversion v_cvt_pk_fp8_f32 does the rounding (OCP E4M3,
// nearest even, sub-normals included) in one instruction; it turns values beyond 448 into NaN
// rather than clipping, hence the clamp in front of it.  UE5M3 rounds on the bit pattern.
template <int FMT>
__device__ __forceinline__ uint32_t sf_encode_rne(float y)
{
    y = fminf(y, ScaleFmt<FMT>::kMaxValue);
    if constexpr (FMT == kE4M3) {
        return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(y, y, 0, false) & 0xFFu;
    } else {
        return sf_encode_bits<ScaleFmt<FMT>::kBias>(y);
    }
}

// Value of any scale byte of any format (NaN for bytes that are not finite numbers); used where
// the format is a run-time argument (de-quantise, diagnostics).
__device__ __forceinline__ float scale_byte_value(int fmt, uint32_t code)
{
    const float nan = u2f(0x7FC00000u);
    if (fmt == kE8M0) {
        if (code == 255u) return nan;
        return (code == 0u) ? u2f(0x00400000u) : u2f(code << 23);      // 2^-127 is sub-normal
    }
    if (fmt == kE4M3) return (code > (uint32_t)ScaleFmt<kE4M3>::kMaxCode) ? nan : sf_decode<kE4M3>(code);
    return (code > (uint32_t)ScaleFmt<kUE5M3>::kMaxCode) ? nan : sf_decode<kUE5M3>(code);
}

// Per-tensor scale of hierarchical scaling from the tensor abs-max: the same function as the
// host helper of the C ABI, so both give the same bits.
template <int FMT>
__device__ __forceinline__ float tensor_scale_of(float absmax)
{
    float sf_max;
    if constexpr (FMT == kE8M0) sf_max = u2f(254u << 23);
    else sf_max = ScaleFmt<FMT>::kMaxValue;
    return tensor_scale_from(absmax, sf_max);
}

// (scale value, reciprocal hi/lo) for every scale byte, filled once per workgroup into LDS.
struct __align__(16) ScaleEntry { float S, rhi, rlo, pad; };

template <int FMT>
__device__ __forceinline__ void fill_scale_table(ScaleEntry* tab)
{
    for (uint32_t c = threadIdx.x; c < 256u; c += blockDim.x) {
        ScaleEntry e{0.0f, 0.0f, 0.0f, 0.0f};
        if (c >= 1u && c <= (uint32_t)ScaleFmt<FMT>::kMaxCode) {
            e.S = sf_decode<FMT>(c);
            const Recip r = make_recip(e.S);
            e.rhi = r.hi;
            e.rlo = r.lo;
        }
        tab[c] = e;     // code 0: S = 0 and a zero "reciprocal" -> every quotient is a signed 0
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------
// E2M1 (Section 2 value set {0, .5, 1, 1.5, 2, 3, 4, 6}).
// ---------------------------------------------------------------------------------------

// Rounding to E2M1 uses the gfx950 conversion instructions v_cvt_scalef32_pk_fp4_f32 /
// v_cvt_scalef32_pk_f32_fp4.  The forward one divides two fp32 inputs by a power-of-two scale
// (only the exponent of the scale operand is used), rounds to nearest even onto
// {0, .5, 1, 1.5, 2, 3, 4, 6}, saturates at 6, keeps the sign bit also for zero results, and
// writes the two 4-bit codes (first input in the low nibble) into the selected byte of the
// destination; the inverse one returns the two values times the scale.  Mid-points go to the
// even code: 0.25->0, 0.75->1, 1.25->1, 1.75->2, 2.5->2, 3.5->4, 5->4.
using f32x2 = float __attribute__((ext_vector_type(2)));
using u32x4 = uint32_t __attribute__((ext_vector_type(4)));

template <int SEL>
__device__ __forceinline__ uint32_t e2m1_pack2(uint32_t old, float a, float b, float scale)
{
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(old, a, b, scale, SEL);
}

template <int SEL>
__device__ __forceinline__ void e2m1_unpack2(uint32_t packed, float scale, float& a, float& b)
{
    const f32x2 r = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(packed, scale, SEL);
    a = r.x;
    b = r.y;
}

// 8 values -> one dword of codes (element j in nibble j).  The four conversions overwrite all
// four bytes, so the register they accumulate into needs no initial value; the empty asm
// statement defines it without emitting an instruction.
__device__ __forceinline__ uint32_t e2m1_pack8(const float (&y)[8], float scale)
{
    uint32_t r;
    asm volatile("" : "=v"(r));
    r = e2m1_pack2<0>(r, y[0], y[1], scale);
    r = e2m1_pack2<1>(r, y[2], y[3], scale);
    r = e2m1_pack2<2>(r, y[4], y[5], scale);
    r = e2m1_pack2<3>(r, y[6], y[7], scale);
    return r;
}

// The same with one power-of-two scale per block of EPB elements inside the lane (EPB even, so
// a pair never straddles two blocks).
template <int EPB>
__device__ __forceinline__ uint32_t e2m1_pack8_scales(const float (&y)[8], const float (&scale)[8 / EPB])
{
    uint32_t r;
    asm volatile("" : "=v"(r));
    r = e2m1_pack2<0>(r, y[0], y[1], scale[0 / EPB]);
    r = e2m1_pack2<1>(r, y[2], y[3], scale[2 / EPB]);
    r = e2m1_pack2<2>(r, y[4], y[5], scale[4 / EPB]);
    r = e2m1_pack2<3>(r, y[6], y[7], scale[6 / EPB]);
    return r;
}

__device__ __forceinline__ void e2m1_unpack8(uint32_t packed, float scale, float (&q)[8])
{
    e2m1_unpack2<0>(packed, scale, q[0], q[1]);
    e2m1_unpack2<1>(packed, scale, q[2], q[3]);
    e2m1_unpack2<2>(packed, scale, q[4], q[5]);
    e2m1_unpack2<3>(packed, scale, q[6], q[7]);
}

// ---------------------------------------------------------------------------------------
// Wavefront helpers.  A block of more than 8 elements is spread over 2, 4, 8 or 16
// neighbouring lanes (8 elements each); xor-butterflies inside a 16-lane DPP row combine
// them.  After a butterfly level every lane of a pair holds the same value, so the mirror
// patterns (lane i <-> 7-i, i <-> 15-i) deliver the partner group's value for the xor-4 and
// xor-8 levels.  fp32 addition is commutative, so all lanes of a block end with the same
// bits, equal to the balanced binary tree in index order.
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return u2f((uint32_t)__builtin_amdgcn_update_dpp(0, (int)f2u(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each group of 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each row of 16

// Maximum of non-negative floats: their bit patterns order like unsigned integers.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

template <int LANES>
__device__ __forceinline__ float group_max(float nonneg)
{
    uint32_t v = f2u(nonneg);
    if constexpr (LANES >= 2) v = max(v, dpp_u<kDppXor1>(v));
    if constexpr (LANES >= 4) v = max(v, dpp_u<kDppXor2>(v));
    if constexpr (LANES >= 8) v = max(v, dpp_u<kDppHalfMirror>(v));
    if constexpr (LANES >= 16) v = max(v, dpp_u<kDppMirror>(v));
    return u2f(v);
}

template <int LANES>
__device__ __forceinline__ float group_sum(float v)
{
    if constexpr (LANES >= 2) v = v + dpp_f<kDppXor1>(v);
    if constexpr (LANES >= 4) v = v + dpp_f<kDppXor2>(v);
    if constexpr (LANES >= 8) v = v + dpp_f<kDppHalfMirror>(v);
    if constexpr (LANES >= 16) v = v + dpp_f<kDppMirror>(v);
    return v;
}

// ---------------------------------------------------------------------------------------
// Loads: 8 consecutive elements per lane, widened to fp32.
// ---------------------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void load8(const void* x, int64_t first, float (&v)[8])
{
    if constexpr (DT == kBF16) {
        const uint4 r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(x) + first);
        v[0] = u2f(r.x << 16); v[1] = u2f(r.x & 0xFFFF0000u);
        v[2] = u2f(r.y << 16); v[3] = u2f(r.y & 0xFFFF0000u);
        v[4] = u2f(r.z << 16); v[5] = u2f(r.z & 0xFFFF0000u);
        v[6] = u2f(r.w << 16); v[7] = u2f(r.w & 0xFFFF0000u);
    } else {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(x) + first);
        const float4 a = p[0], b = p[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
}

// Ragged tail: `count` < 8 valid elements, the rest read as +0.
template <int DT>
__device__ __forceinline__ void load_partial(const void* x, int64_t first, int count, float (&v)[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float f = 0.0f;
        if (i < count) {
            if constexpr (DT == kBF16)
                f = u2f((uint32_t)static_cast<const uint16_t*>(x)[first + i] << 16);
            else
                f = static_cast<const float*>(x)[first + i];
        }
        v[i] = f;
    }
}

}  // namespace mxq
