// Streaming recipes of Section 2: abs-max scale (Eq. 2; Eq. 1 for power-of-two scales),
// prevent-zero clamp (Eq. 3) and 4-over-6 (Eq. 4), one pass over the tensor.
//
// Mapping: every lane owns 8 consecutive elements (one 128-bit load for bf16, two for fp32),
// so a block of b >= 8 elements is b/8 neighbouring lanes of one DPP row and a block of
// b < 8 sits inside a lane.  Per lane the kernel emits one dword of packed codes; the first
// lane of a block emits the scale byte and the block SSE.  HBM-bound by design: algorithmic
// traffic is sizeof(in) + 0.5 + 5/b bytes per element.
#include "mxq_device.hpp"
#include "mxq_launch.hpp"

namespace mxq {

// (scale value, reciprocal hi/lo) for every scale byte, filled once per workgroup.
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
        tab[c] = e;     // code 0: S = 0 and a zero "reciprocal" -> every quotient is 0
    }
    __syncthreads();
}

// Eq. 2 / Eq. 3: scale code from the block abs-max for M = 6 or M = 4.
template <int FMT, int M>
__device__ __forceinline__ uint32_t absmax_code(float amax, bool pz)
{
    float y;
    if constexpr (M == 6) y = __builtin_fmaf(amax, kSixthHi, amax * kSixthLo);
    else y = amax * 0.25f;
    uint32_t c = sf_encode_rne<FMT>(y);
    if (pz) c = max(c, 1u);                 // eps_SF is code 1 in both formats
    return c;
}

// Eq. 1: k = floor(log2(amax / 6)).  With amax = m * 2^e, 1 <= m < 2: k = e - 2 when
// m >= 1.5, else e - 3; byte = k + 127, never below 0 (sub-normal or zero amax gives 0).
__device__ __forceinline__ uint32_t pow2_code(float amax)
{
    const uint32_t b = f2u(amax);
    const int c = (int)(b >> 23) - 3 + (int)((b >> 22) & 1u);
    return (uint32_t)max(c, 0);
}

// Quantise the lane's 8 values (NBLK blocks of EPB elements, one scale code each): packed
// nibbles and the 8 squared residuals.
template <int NBLK, int EPB>
__device__ __forceinline__ void quant_lane(const float (&v)[8], const uint32_t (&code)[NBLK],
                                           const ScaleEntry* tab, uint32_t& packed, float (&sq)[8])
{
    packed = 0u;
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        const ScaleEntry se = tab[code[k]];
        const Recip r{se.rhi, se.rlo};
#pragma unroll
        for (int i = 0; i < EPB; ++i) {
            const int j = k * EPB + i;
            const float y = quot(v[j], r);
            const uint32_t mag = e2m1_round_mag(__builtin_fabsf(y));
            const uint32_t sign = f2u(v[j]) >> 31;
            const float q = u2f(f2u(e2m1_mag_value(mag)) | (sign << 31));
            const float e = __builtin_fmaf(-q, se.S, v[j]);    // q*S is exact: one rounding
            sq[j] = e * e;
            packed |= ((sign << 3) | mag) << (4 * j);
        }
    }
}

// Block SSE: balanced tree in index order, inside the lane and then across the block's lanes.
// For b < 8 the lane holds 8/b blocks; their sums come back in sse[0 .. 8/b).
template <int B>
__device__ __forceinline__ void block_sse(const float (&sq)[8], float (&sse)[4])
{
    const float p0 = sq[0] + sq[1], p1 = sq[2] + sq[3], p2 = sq[4] + sq[5], p3 = sq[6] + sq[7];
    if constexpr (B == 2) {
        sse[0] = p0; sse[1] = p1; sse[2] = p2; sse[3] = p3;
    } else if constexpr (B == 4) {
        sse[0] = p0 + p1; sse[1] = p2 + p3;
    } else {
        sse[0] = group_sum<B / 8>((p0 + p1) + (p2 + p3));
    }
}

template <int DT, int B, int FMT, bool FOUR6>
__global__ void __launch_bounds__(kThreads)
stream_kernel(const void* __restrict__ x, int64_t n, float T, int pz,
              uint32_t* __restrict__ codes, uint8_t* __restrict__ scales, float* __restrict__ sse_out)
{
    constexpr int NBLK = (B < 8) ? 8 / B : 1;          // blocks inside one lane
    constexpr int LANES = (B < 8) ? 1 : B / 8;         // lanes per block
    constexpr int EPB = (B < 8) ? B : 8;               // elements of one block inside a lane

    __shared__ ScaleEntry tab[(FMT == kE8M0) ? 1 : 256];
    if constexpr (FMT != kE8M0) fill_scale_table<FMT>(tab);

    const int64_t n_chunks = (n + 7) >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t wave_first = (int64_t)blockIdx.x * kThreads + (threadIdx.x & ~63);

    for (int64_t base = wave_first; base < n_chunks; base += stride) {
        const int64_t chunk = base + (threadIdx.x & 63);
        const int64_t first = chunk << 3;
        const int count = (int)min((int64_t)8, n - first);      // <= 0 past the end
        float v[8];
        if (count == 8) load8<DT>(x, first, v);
        else load_partial<DT>(x, first, count, v);

        if (T != 1.0f) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = v[i] / T;        // IEEE division (hierarchical)
        }

        // block abs-max
        float amax[NBLK];
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < EPB; ++i) a = fmaxf(a, __builtin_fabsf(v[k * EPB + i]));
            amax[k] = group_max<LANES>(a);
        }

        uint32_t packed = 0u, code_out[NBLK];
        float sse_sel[4];

        if constexpr (FMT == kE8M0) {
            // power-of-two scale: v / 2^k is exact, multiply by 2^-k
            float sq[8];
#pragma unroll
            for (int k = 0; k < NBLK; ++k) {
                const uint32_t c = pow2_code(amax[k]);
                code_out[k] = c;
                const float S = (c == 0u) ? u2f(0x00400000u) : u2f(c << 23);
                const float Sinv = (c == 254u) ? u2f(0x00400000u) : u2f((254u - c) << 23);
#pragma unroll
                for (int i = 0; i < EPB; ++i) {
                    const int j = k * EPB + i;
                    const uint32_t mag = e2m1_round_mag(__builtin_fabsf(v[j] * Sinv));
                    const uint32_t sign = f2u(v[j]) >> 31;
                    const float q = u2f(f2u(e2m1_mag_value(mag)) | (sign << 31));
                    const float e = __builtin_fmaf(-q, S, v[j]);
                    sq[j] = e * e;
                    packed |= ((sign << 3) | mag) << (4 * j);
                }
            }
            block_sse<B>(sq, sse_sel);
        } else {
            // one scale per block inside the lane; gather per-element scale operands
            uint32_t c6[NBLK], c4[NBLK];
#pragma unroll
            for (int k = 0; k < NBLK; ++k) {
                c6[k] = absmax_code<FMT, 6>(amax[k], pz != 0);
                if constexpr (FOUR6) c4[k] = absmax_code<FMT, 4>(amax[k], pz != 0);
            }
            float sq6[8], sse6[4];
            quant_lane<NBLK, EPB>(v, c6, tab, packed, sq6);
            block_sse<B>(sq6, sse6);
#pragma unroll
            for (int k = 0; k < NBLK; ++k) { code_out[k] = c6[k]; sse_sel[k] = sse6[k]; }

            if constexpr (FOUR6) {
                float sq4[8], sse4[4];
                uint32_t packed4;
                quant_lane<NBLK, EPB>(v, c4, tab, packed4, sq4);
                block_sse<B>(sq4, sse4);
                // Eq. 4: M = 4 only when its SSE is strictly lower
#pragma unroll
                for (int k = 0; k < NBLK; ++k) {
                    if (sse4[k] < sse6[k]) {
                        constexpr uint32_t m = (EPB == 8) ? 0xFFFFFFFFu : ((1u << (4 * EPB)) - 1u);
                        const uint32_t mask = m << (4 * EPB * k);
                        packed = (packed & ~mask) | (packed4 & mask);
                        code_out[k] = c4[k];
                        sse_sel[k] = sse4[k];
                    }
                }
            }
        }

        if (count <= 0) continue;
        if (count == 8) {
            codes[chunk] = packed;
        } else {
            uint8_t* cb = reinterpret_cast<uint8_t*>(codes) + chunk * 4;
            for (int i = 0; i < count / 2; ++i) cb[i] = (uint8_t)(packed >> (8 * i));
        }
        if constexpr (B >= 8) {
            if ((threadIdx.x & (LANES - 1)) == 0) {
                const int64_t blk = chunk / LANES;
                scales[blk] = (uint8_t)code_out[0];
                if (sse_out) sse_out[blk] = sse_sel[0];
            }
        } else {
            const int64_t blk0 = chunk * NBLK;
            const int nvalid = count / B;
            if (nvalid == NBLK) {
                if constexpr (NBLK == 2) {
                    *reinterpret_cast<uint16_t*>(scales + blk0) = (uint16_t)(code_out[0] | (code_out[1] << 8));
                    if (sse_out) *reinterpret_cast<float2*>(sse_out + blk0) = make_float2(sse_sel[0], sse_sel[1]);
                } else {
                    *reinterpret_cast<uint32_t*>(scales + blk0) =
                        code_out[0] | (code_out[1] << 8) | (code_out[2] << 16) | (code_out[3] << 24);
                    if (sse_out)
                        *reinterpret_cast<float4*>(sse_out + blk0) =
                            make_float4(sse_sel[0], sse_sel[1], sse_sel[2], sse_sel[3]);
                }
            } else {
                for (int k = 0; k < nvalid; ++k) {
                    scales[blk0 + k] = (uint8_t)code_out[k];
                    if (sse_out) sse_out[blk0 + k] = sse_sel[k];
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------ dispatch

template <int DT, int B, int FMT>
static hipError_t launch_fmt(const StreamArgs& a)
{
    const int64_t n_chunks = (a.n + 7) / 8;
    const int grid = stream_grid(n_chunks);
    const bool four6 = (a.recipe == 2 || a.recipe == 3);
    const int pz = (a.recipe == 1 || a.recipe == 3) ? 1 : 0;
    if constexpr (FMT == kE8M0) {
        hipLaunchKernelGGL((stream_kernel<DT, B, FMT, false>), dim3(grid), dim3(kThreads), 0, a.stream,
                           a.x, a.n, a.T, 0, (uint32_t*)a.codes, a.scales, a.sse);
    } else {
        if (four6)
            hipLaunchKernelGGL((stream_kernel<DT, B, FMT, true>), dim3(grid), dim3(kThreads), 0, a.stream,
                               a.x, a.n, a.T, pz, (uint32_t*)a.codes, a.scales, a.sse);
        else
            hipLaunchKernelGGL((stream_kernel<DT, B, FMT, false>), dim3(grid), dim3(kThreads), 0, a.stream,
                               a.x, a.n, a.T, pz, (uint32_t*)a.codes, a.scales, a.sse);
    }
    return hipGetLastError();
}

template <int DT, int B>
static hipError_t launch_block(const StreamArgs& a)
{
    switch (a.scale_fmt) {
        case kE8M0: return launch_fmt<DT, B, kE8M0>(a);
        case kE4M3: return launch_fmt<DT, B, kE4M3>(a);
        default: return launch_fmt<DT, B, kUE5M3>(a);
    }
}

template <int DT>
static hipError_t launch_dt(const StreamArgs& a)
{
    switch (a.block) {
        case 2: return launch_block<DT, 2>(a);
        case 4: return launch_block<DT, 4>(a);
        case 8: return launch_block<DT, 8>(a);
        case 16: return launch_block<DT, 16>(a);
        case 32: return launch_block<DT, 32>(a);
        case 64: return launch_block<DT, 64>(a);
        default: return launch_block<DT, 128>(a);
    }
}

hipError_t launch_stream(const StreamArgs& a)
{
    return (a.dtype == kBF16) ? launch_dt<kBF16>(a) : launch_dt<kF32>(a);
}

}  // namespace mxq
