// Brute-force scale search (last paragraph of Section 2): for every block, every finite,
// strictly positive scale code is tried; the code of minimal block SSE wins, the lowest code
// on a tie.  Same lane mapping as the streaming kernels (8 elements per lane); the tensor is
// read once and each candidate costs only ALU work, so this kernel is bound by the fp32
// vector units, not by HBM.
#include "mxq_device.hpp"
#include "mxq_launch.hpp"

namespace mxq {

struct __align__(16) BruteEntry { float S, rhi, rlo, pad; };

template <int B>
__device__ __forceinline__ void brute_block_sse(const float (&sq)[8], float (&sse)[4])
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

template <int DT, int B, int FMT>
__global__ void __launch_bounds__(kThreads)
brute_kernel(const void* __restrict__ x, int64_t n, float T,
             uint32_t* __restrict__ codes, uint8_t* __restrict__ scales, float* __restrict__ sse_out)
{
    constexpr int NBLK = (B < 8) ? 8 / B : 1;
    constexpr int LANES = (B < 8) ? 1 : B / 8;
    constexpr int EPB = (B < 8) ? B : 8;
    constexpr uint32_t kMax = ScaleFmt<FMT>::kMaxCode;

    __shared__ BruteEntry tab[256];
    for (uint32_t c = threadIdx.x; c < 256u; c += blockDim.x) {
        BruteEntry e{0.0f, 0.0f, 0.0f, 0.0f};
        if (c >= 1u && c <= kMax) {
            e.S = sf_decode<FMT>(c);
            const Recip r = make_recip(e.S);
            e.rhi = r.hi;
            e.rlo = r.lo;
        }
        tab[c] = e;
    }
    __syncthreads();

    const int64_t n_chunks = (n + 7) >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t wave_first = (int64_t)blockIdx.x * kThreads + (threadIdx.x & ~63);

    for (int64_t base = wave_first; base < n_chunks; base += stride) {
        const int64_t chunk = base + (threadIdx.x & 63);
        const int64_t first = chunk << 3;
        const int count = (int)min((int64_t)8, n - first);
        float v[8];
        if (count == 8) load8<DT>(x, first, v);
        else load_partial<DT>(x, first, count, v);
        if (T != 1.0f) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = v[i] / T;
        }

        float best_sse[NBLK];
        uint32_t best_code[NBLK];
#pragma unroll
        for (int k = 0; k < NBLK; ++k) { best_sse[k] = __builtin_inff(); best_code[k] = 1u; }

        for (uint32_t c = 1u; c <= kMax; ++c) {          // ascending: a tie keeps the lowest code
            const BruteEntry se = tab[c];
            const Recip r{se.rhi, se.rlo};
            float sq[8], s[4];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float y = quot(v[j], r);
                const uint32_t mag = e2m1_round_mag(__builtin_fabsf(y));
                const float q = u2f(f2u(e2m1_mag_value(mag)) | (f2u(v[j]) & 0x80000000u));
                const float e = __builtin_fmaf(-q, se.S, v[j]);
                sq[j] = e * e;
            }
            brute_block_sse<B>(sq, s);
#pragma unroll
            for (int k = 0; k < NBLK; ++k) {
                if (s[k] < best_sse[k]) { best_sse[k] = s[k]; best_code[k] = c; }
            }
        }

        // codes of the winning candidate
        uint32_t packed = 0u;
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            const BruteEntry se = tab[best_code[k]];
            const Recip r{se.rhi, se.rlo};
#pragma unroll
            for (int i = 0; i < EPB; ++i) {
                const int j = k * EPB + i;
                const uint32_t mag = e2m1_round_mag(__builtin_fabsf(quot(v[j], r)));
                packed |= (((f2u(v[j]) >> 31) << 3) | mag) << (4 * j);
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
                scales[blk] = (uint8_t)best_code[0];
                if (sse_out) sse_out[blk] = best_sse[0];
            }
        } else {
            const int64_t blk0 = chunk * NBLK;
            const int nvalid = count / B;
            for (int k = 0; k < NBLK; ++k) {
                if (k < nvalid) {
                    scales[blk0 + k] = (uint8_t)best_code[k];
                    if (sse_out) sse_out[blk0 + k] = best_sse[k];
                }
            }
        }
    }
}

template <int DT, int B>
static hipError_t launch_b(const StreamArgs& a)
{
    const int64_t n_chunks = (a.n + 7) / 8;
    const int64_t need = (n_chunks + kThreads - 1) / kThreads;
    const int grid = (int)(need < 1 ? 1 : (need < 256 * 8 ? need : 256 * 8));
    if (a.scale_fmt == kE4M3)
        hipLaunchKernelGGL((brute_kernel<DT, B, kE4M3>), dim3(grid), dim3(kThreads), 0, a.stream,
                           a.x, a.n, a.T, (uint32_t*)a.codes, a.scales, a.sse);
    else
        hipLaunchKernelGGL((brute_kernel<DT, B, kUE5M3>), dim3(grid), dim3(kThreads), 0, a.stream,
                           a.x, a.n, a.T, (uint32_t*)a.codes, a.scales, a.sse);
    return hipGetLastError();
}

template <int DT>
static hipError_t launch_d(const StreamArgs& a)
{
    switch (a.block) {
        case 2: return launch_b<DT, 2>(a);
        case 4: return launch_b<DT, 4>(a);
        case 8: return launch_b<DT, 8>(a);
        case 16: return launch_b<DT, 16>(a);
        case 32: return launch_b<DT, 32>(a);
        case 64: return launch_b<DT, 64>(a);
        default: return launch_b<DT, 128>(a);
    }
}

hipError_t launch_brute(const StreamArgs& a)
{
    return (a.dtype == kBF16) ? launch_d<kBF16>(a) : launch_d<kF32>(a);
}

}  // namespace mxq
