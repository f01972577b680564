// Diagnostics of the paper's appendix: the clipping-only part of the block SSE ("Clipping only
// MSE" figure) and the histograms of quantised entries and of chosen scales.  Both read what
// mxq_quantize wrote; neither is on the hot path.
#include "mxq_device.hpp"
#include "mxq_launch.hpp"

namespace mxq {

// One lane = 8 consecutive elements.  An element clips when fl32(|v| / S) > 6, which for the
// short significands of S is the same as |v| > 6 * S (6 * S is exact); its residual is
// v - (+-6) * S, one FMA because the product is exact.
template <int DT, int B>
__global__ void __launch_bounds__(kThreads)
clip_sse_kernel(const void* __restrict__ x, const uint8_t* __restrict__ scales, int64_t n, int fmt,
                float T, float* __restrict__ out)
{
    constexpr int NBLK = (B < 8) ? 8 / B : 1;
    constexpr int LANES = (B < 8) ? 1 : B / 8;
    constexpr int EPB = (B < 8) ? B : 8;
    const int64_t n_chunks = (n + 7) >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t c0 = (int64_t)blockIdx.x * kThreads; c0 < n_chunks; c0 += stride) {     // uniform
        const int64_t chunk = c0 + threadIdx.x;
        const int64_t first = chunk << 3;
        const int count = (int)max((int64_t)0, min((int64_t)8, n - first));
        float v[8];
        if (count == 8) load8<DT>(x, first, v);
        else load_partial<DT>(x, first, count, v);
        if (T != 1.0f) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = v[i] / T;
        }
        float sq[8];
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            float S = 0.0f;
            if (k * EPB < count) S = scale_byte_value(fmt, scales[(B >= 8) ? chunk / LANES : chunk * NBLK + k]);
            const float lim = 6.0f * S;
#pragma unroll
            for (int i = 0; i < EPB; ++i) {
                const int j = k * EPB + i;
                const float q = u2f(0x40C00000u | (f2u(v[j]) & 0x80000000u));      // +-6
                const float e = __builtin_fmaf(-q, S, v[j]);
                const float s = e * e;
                sq[j] = (__builtin_fabsf(v[j]) > lim && S > 0.0f) ? s : 0.0f;
            }
        }
        const float p0 = sq[0] + sq[1], p1 = sq[2] + sq[3], p2 = sq[4] + sq[5], p3 = sq[6] + sq[7];
        if constexpr (B >= 8) {
            const float s = group_sum<LANES>((p0 + p1) + (p2 + p3));
            if (count > 0 && (threadIdx.x & (LANES - 1)) == 0) out[chunk / LANES] = s;
        } else if constexpr (B == 4) {
            if (count >= 4) out[chunk * 2] = p0 + p1;
            if (count >= 8) out[chunk * 2 + 1] = p2 + p3;
        } else {
            if (count >= 2) out[chunk * 4] = p0;
            if (count >= 4) out[chunk * 4 + 1] = p1;
            if (count >= 6) out[chunk * 4 + 2] = p2;
            if (count >= 8) out[chunk * 4 + 3] = p3;
        }
    }
}

template <int DT>
static void launch_clip_dt(const void* x, const uint8_t* scales, int64_t n, int block, int fmt, float T,
                           float* out, hipStream_t stream, int grid)
{
#define MXQ_CLIP(BB)                                                                                  \
    hipLaunchKernelGGL((clip_sse_kernel<DT, BB>), dim3(grid), dim3(kThreads), 0, stream, x, scales, n, fmt, T, out)
    switch (block) {
        case 2: MXQ_CLIP(2); break;
        case 4: MXQ_CLIP(4); break;
        case 8: MXQ_CLIP(8); break;
        case 16: MXQ_CLIP(16); break;
        case 32: MXQ_CLIP(32); break;
        case 64: MXQ_CLIP(64); break;
        default: MXQ_CLIP(128); break;
    }
#undef MXQ_CLIP
}

hipError_t launch_clip_sse(const void* x, const uint8_t* scales, int64_t n, int dtype, int block,
                           int scale_fmt, float T, float* out, hipStream_t stream)
{
    const int grid = stream_grid((n + 7) / 8);
    if (dtype == kBF16) launch_clip_dt<kBF16>(x, scales, n, block, scale_fmt, T, out, stream, grid);
    else launch_clip_dt<kF32>(x, scales, n, block, scale_fmt, T, out, stream, grid);
    return hipGetLastError();
}

// Histograms.  Element magnitudes are counted per lane in registers over the whole grid-stride
// loop (nibble-parallel compares on the packed dword), scale bytes go through a per-workgroup
// LDS histogram; both meet in 64-bit atomics on the caller's arrays, which a small kernel
// clears first.
__global__ void hist_clear_kernel(unsigned long long* elem_hist, unsigned long long* scale_hist)
{
    const uint32_t t = threadIdx.x;
    if (t < 8u) elem_hist[t] = 0ull;
    scale_hist[t] = 0ull;
}

// number of nibbles of w whose low three bits equal k
__device__ __forceinline__ uint32_t count_mag(uint32_t w, uint32_t k)
{
    const uint32_t d = (w ^ (k * 0x11111111u)) & 0x77777777u;          // zero nibble <=> match
    const uint32_t nz = (d | (d >> 1) | (d >> 2)) & 0x11111111u;       // 1 per non-matching nibble
    return 8u - (uint32_t)__builtin_popcount(nz);
}

static_assert(kThreads == 256, "the scale histogram uses one LDS counter per thread");

__global__ void __launch_bounds__(kThreads)
histogram_kernel(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales, int64_t n,
                 int64_t n_blocks, unsigned long long* __restrict__ elem_hist,
                 unsigned long long* __restrict__ scale_hist)
{
    __shared__ uint32_t sh_scale[256];
    __shared__ uint32_t sh_elem[8];
    sh_scale[threadIdx.x] = 0u;
    if (threadIdx.x < 8) sh_elem[threadIdx.x] = 0u;
    __syncthreads();

    uint32_t cnt[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    const int64_t n_dwords = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t t0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    for (int64_t i = t0; i < n_dwords; i += stride) {
        const uint32_t w = __builtin_nontemporal_load(codes + i);
#pragma unroll
        for (uint32_t k = 0; k < 8u; ++k) cnt[k] += count_mag(w, k);
    }
    if (t0 == 0) {                                                   // ragged tail: < 8 elements
        const uint8_t* cb = reinterpret_cast<const uint8_t*>(codes);
        for (int64_t e = n_dwords << 3; e < n; ++e) cnt[(cb[e >> 1] >> ((e & 1) * 4)) & 7u] += 1u;
    }
    for (int64_t b = t0; b < n_blocks; b += stride) atomicAdd(&sh_scale[scales[b]], 1u);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t c = cnt[k];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) c += (uint32_t)__shfl_xor((int)c, off, 64);
        if ((threadIdx.x & 63) == 0) atomicAdd(&sh_elem[k], c);
    }
    __syncthreads();
    if (threadIdx.x < 8 && sh_elem[threadIdx.x]) atomicAdd(&elem_hist[threadIdx.x], (unsigned long long)sh_elem[threadIdx.x]);
    if (sh_scale[threadIdx.x]) atomicAdd(&scale_hist[threadIdx.x], (unsigned long long)sh_scale[threadIdx.x]);
}

hipError_t launch_histogram(const uint8_t* codes, const uint8_t* scales, int64_t n, int block,
                            unsigned long long* elem_hist, unsigned long long* scale_hist,
                            hipStream_t stream)
{
    hipLaunchKernelGGL(hist_clear_kernel, dim3(1), dim3(256), 0, stream, elem_hist, scale_hist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    // a lane's register counters are 32-bit and a workgroup's LDS counters too: bound the work
    // per workgroup to < 2^32 elements by using enough workgroups (one per 2^21 dwords at least)
    const int64_t n_dwords = (n + 7) / 8;
    int64_t grid = (n_dwords + kThreads * 16 - 1) / (kThreads * 16);
    if (grid > 1024) grid = 1024;
    const int64_t min_grid = (n_dwords >> 21) + 1;
    if (grid < min_grid) grid = min_grid;
    hipLaunchKernelGGL(histogram_kernel, dim3((unsigned)grid), dim3(kThreads), 0, stream,
                       reinterpret_cast<const uint32_t*>(codes), scales, n, n / block, elem_hist, scale_hist);
    return hipGetLastError();
}

}  // namespace mxq
