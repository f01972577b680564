// De-quantisation ("de-quantization simply multiplies by S", Section 2) and the tensor
// abs-max of hierarchical scaling (first stage of the two-stage process, Section 2).
#include "mxq_device.hpp"
#include "mxq_launch.hpp"

namespace mxq {

__device__ __forceinline__ float scale_value_any(int fmt, uint32_t code)
{
    const float nan = u2f(0x7FC00000u);
    if (fmt == kE8M0) {
        if (code == 255u) return nan;
        return (code == 0u) ? u2f(0x00400000u) : u2f(code << 23);
    }
    if (fmt == kE4M3) return (code > (uint32_t)ScaleFmt<kE4M3>::kMaxCode) ? nan : sf_decode<kE4M3>(code);
    return (code > (uint32_t)ScaleFmt<kUE5M3>::kMaxCode) ? nan : sf_decode<kUE5M3>(code);
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    const uint32_t u = f2u(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;       // keep NaN a NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// One lane = 8 consecutive elements = one dword of codes.
template <int DT>
__global__ void __launch_bounds__(kThreads)
dequant_kernel(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales, int64_t n,
               int block_shift, int fmt, float T, void* __restrict__ out)
{
    const int64_t n_chunks = (n + 7) >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t chunk = (int64_t)blockIdx.x * kThreads + threadIdx.x; chunk < n_chunks; chunk += stride) {
        const int64_t first = chunk << 3;
        const int count = (int)min((int64_t)8, n - first);
        uint32_t packed = 0u;
        if (count == 8) {
            packed = codes[chunk];
        } else {
            const uint8_t* cb = reinterpret_cast<const uint8_t*>(codes) + chunk * 4;
            for (int i = 0; i < count / 2; ++i) packed |= (uint32_t)cb[i] << (8 * i);
        }
        float r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float val = 0.0f;
            if (i < count) {
                const uint32_t c = (packed >> (4 * i)) & 0xFu;
                const float S = scale_value_any(fmt, scales[(first + i) >> block_shift]);
                const float q = u2f(f2u(e2m1_mag_value(c & 7u)) | ((c & 8u) << 28));
                val = (q * S) * T;
            }
            r[i] = val;
        }
        if (count == 8) {
            if constexpr (DT == kBF16) {
                uint4 o;
                o.x = f32_to_bf16_rne(r[0]) | (f32_to_bf16_rne(r[1]) << 16);
                o.y = f32_to_bf16_rne(r[2]) | (f32_to_bf16_rne(r[3]) << 16);
                o.z = f32_to_bf16_rne(r[4]) | (f32_to_bf16_rne(r[5]) << 16);
                o.w = f32_to_bf16_rne(r[6]) | (f32_to_bf16_rne(r[7]) << 16);
                *reinterpret_cast<uint4*>(static_cast<uint16_t*>(out) + first) = o;
            } else {
                float4* p = reinterpret_cast<float4*>(static_cast<float*>(out) + first);
                p[0] = make_float4(r[0], r[1], r[2], r[3]);
                p[1] = make_float4(r[4], r[5], r[6], r[7]);
            }
        } else {
            for (int i = 0; i < count; ++i) {
                if constexpr (DT == kBF16) static_cast<uint16_t*>(out)[first + i] = (uint16_t)f32_to_bf16_rne(r[i]);
                else static_cast<float*>(out)[first + i] = r[i];
            }
        }
    }
}

hipError_t launch_dequant(const DequantArgs& a)
{
    const int64_t n_chunks = (a.n + 7) / 8;
    const int grid = stream_grid(n_chunks);
    int shift = 0;
    while ((1 << shift) < a.block) ++shift;
    if (a.dtype == kBF16)
        hipLaunchKernelGGL((dequant_kernel<kBF16>), dim3(grid), dim3(kThreads), 0, a.stream,
                           (const uint32_t*)a.codes, a.scales, a.n, shift, a.scale_fmt, a.T, a.out);
    else
        hipLaunchKernelGGL((dequant_kernel<kF32>), dim3(grid), dim3(kThreads), 0, a.stream,
                           (const uint32_t*)a.codes, a.scales, a.n, shift, a.scale_fmt, a.T, a.out);
    return hipGetLastError();
}

// Tensor abs-max.  |x| of finite fp32 values orders like the unsigned integer bits & 0x7fffffff,
// so the reduction is an integer max; partial results meet in one 32-bit atomic max on the
// output word, which a one-thread kernel clears first (no memset node, so the pair can be
// captured in a graph).
__global__ void absmax_clear_kernel(uint32_t* out) { *out = 0u; }

template <int DT>
__global__ void __launch_bounds__(kThreads)
absmax_kernel(const void* __restrict__ x, int64_t n, uint32_t* __restrict__ out)
{
    const int64_t n_chunks = (n + 7) >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    uint32_t m = 0u;
    for (int64_t chunk = (int64_t)blockIdx.x * kThreads + threadIdx.x; chunk < n_chunks; chunk += stride) {
        const int64_t first = chunk << 3;
        const int count = (int)min((int64_t)8, n - first);
        float v[8];
        if (count == 8) load8<DT>(x, first, v);
        else load_partial<DT>(x, first, count, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) m = max(m, f2u(v[i]) & 0x7FFFFFFFu);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
    __shared__ uint32_t part[kThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t w = part[0];
        for (int i = 1; i < kThreads / 64; ++i) w = max(w, part[i]);
        atomicMax(out, w);
    }
}

hipError_t launch_absmax(const void* x, int64_t n, int dtype, float* out, hipStream_t stream)
{
    hipLaunchKernelGGL(absmax_clear_kernel, dim3(1), dim3(1), 0, stream, (uint32_t*)out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    const int64_t n_chunks = (n + 7) / 8;
    const int grid = stream_grid(n_chunks);
    if (dtype == kBF16)
        hipLaunchKernelGGL((absmax_kernel<kBF16>), dim3(grid), dim3(kThreads), 0, stream, x, n, (uint32_t*)out);
    else
        hipLaunchKernelGGL((absmax_kernel<kF32>), dim3(grid), dim3(kThreads), 0, stream, x, n, (uint32_t*)out);
    return hipGetLastError();
}

}  // namespace mxq
