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
        uint32_t sb[NBLK];                          // the lane's scale bytes; one load for a full chunk
        if (B < 8 && count == 8) {
            uint32_t w;
            if constexpr (NBLK == 4) w = *reinterpret_cast<const uint32_t*>(scales + chunk * 4);
            else w = *reinterpret_cast<const uint16_t*>(scales + chunk * 2);
#pragma unroll
            for (int k = 0; k < NBLK; ++k) sb[k] = (w >> (8 * k)) & 0xFFu;
        } else {
#pragma unroll
            for (int k = 0; k < NBLK; ++k)
                sb[k] = (k * EPB < count) ? (uint32_t)scales[(B >= 8) ? chunk / LANES : chunk * NBLK + k] : 0u;
        }
        float sq[8];
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            const float S = (k * EPB < count) ? scale_byte_value(fmt, sb[k]) : 0.0f;
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
            if (count == 8) {
                reinterpret_cast<float2*>(out)[chunk] = make_float2(p0 + p1, p2 + p3);
            } else if (count >= 4) {
                out[chunk * 2] = p0 + p1;
            }
        } else {
            if (count == 8) {
                reinterpret_cast<float4*>(out)[chunk] = make_float4(p0, p1, p2, p3);
            } else {
                if (count >= 2) out[chunk * 4] = p0;
                if (count >= 4) out[chunk * 4 + 1] = p1;
                if (count >= 6) out[chunk * 4 + 2] = p2;
            }
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

// Histograms.  Both arrays are read with 128-bit loads.
//
// Element magnitudes: the low three bits of the 32 nibbles in a 128-bit vector are transposed
// into three 32-bit planes (plane p holds bit p of every nibble: the four dwords' bit-p masks
// 0x11111111 << p are shifted to interleave), and each of the 8 magnitudes is one boolean
// function of the three planes followed by a population count that adds into a per-lane
// register counter: about 40 vector instructions per 32 elements.
//
// Scale bytes: a per-workgroup LDS histogram with one copy per lane of a wavefront (64 copies,
// word [code][lane]: 64 KiB), so that the lanes of one LDS atomic never meet on a word, however
// popular a code is, and fall on the banks like any 64-lane access.
//
// Partial results meet in 64-bit atomics on the caller's arrays, which a small kernel clears
// first; few, large workgroups keep the number of those atomics small.  The scale bytes are
// counted first, so that those atomics are on their way while the codes are counted.  The bytes before the
// first 16-byte boundary, those after the last complete vector and a ragged last dword are
// counted serially by one thread.
__global__ void hist_clear_kernel(unsigned long long* elem_hist, unsigned long long* scale_hist)
{
    const uint32_t t = threadIdx.x;
    if (t < 8u) elem_hist[t] = 0ull;
    scale_hist[t] = 0ull;
}

constexpr int kHistThreads = 1024;
constexpr int kHistCopies = 64;
constexpr int kHistMaxGrid = 256;      // more workgroups lose more in same-address atomics than they gain (measured)
static_assert(kHistThreads == 4 * 256 && kHistCopies == 64, "the closing reduction maps four threads to a code");

// cnt[k] += number of nibbles of the four dwords whose low three bits equal k
__device__ __forceinline__ void count_magnitudes(const u32x4 w, uint32_t (&cnt)[8])
{
    constexpr uint32_t M0 = 0x11111111u, M1 = 0x22222222u, M2 = 0x44444444u;
    const uint32_t p0 = (w.x & M0) | ((w.y & M0) << 1) | ((w.z & M0) << 2) | ((w.w & M0) << 3);
    const uint32_t p1 = ((w.x & M1) >> 1) | (w.y & M1) | ((w.z & M1) << 1) | ((w.w & M1) << 2);
    const uint32_t p2 = ((w.x & M2) >> 2) | ((w.y & M2) >> 1) | (w.z & M2) | ((w.w & M2) << 1);
    cnt[0] += (uint32_t)__builtin_popcount(~p2 & ~p1 & ~p0);
    cnt[1] += (uint32_t)__builtin_popcount(~p2 & ~p1 & p0);
    cnt[2] += (uint32_t)__builtin_popcount(~p2 & p1 & ~p0);
    cnt[3] += (uint32_t)__builtin_popcount(~p2 & p1 & p0);
    cnt[4] += (uint32_t)__builtin_popcount(p2 & ~p1 & ~p0);
    cnt[5] += (uint32_t)__builtin_popcount(p2 & ~p1 & p0);
    cnt[6] += (uint32_t)__builtin_popcount(p2 & p1 & ~p0);
    cnt[7] += (uint32_t)__builtin_popcount(p2 & p1 & p0);
}

__global__ void __launch_bounds__(kHistThreads)
histogram_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales, int64_t n,
                 int64_t n_blocks, unsigned long long* __restrict__ elem_hist,
                 unsigned long long* __restrict__ scale_hist)
{
    __shared__ uint32_t sh_scale[kHistCopies * 256];
    __shared__ uint32_t sh_elem[8];

    const int64_t stride = (int64_t)gridDim.x * kHistThreads;
    const int64_t t0 = (int64_t)blockIdx.x * kHistThreads + threadIdx.x;

    // packed codes: n / 2 bytes = head bytes, n_vec aligned 16-byte vectors, tail bytes
    const int64_t code_bytes = n >> 1;
    const int64_t c_head = min(code_bytes, (int64_t)((16u - (uint32_t)(reinterpret_cast<uintptr_t>(codes) & 15u)) & 15u));
    const int64_t c_vec = (code_bytes - c_head) >> 4;
    const u32x4* cv = reinterpret_cast<const u32x4*>(codes + c_head);
    // scale bytes: the same split
    const int64_t s_head = min(n_blocks, (int64_t)((16u - (uint32_t)(reinterpret_cast<uintptr_t>(scales) & 15u)) & 15u));
    const int64_t s_vec = (n_blocks - s_head) >> 4;
    const u32x4* sv = reinterpret_cast<const u32x4*>(scales + s_head);

    // The first loads of both arrays leave before the LDS is cleared, so that their latency
    // covers the clearing and, for the codes, the whole scale phase.
    u32x4 rs[2] = {}, rc[4] = {};
    if (s_vec > 0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) rs[u] = __builtin_nontemporal_load(sv + min(t0 + u * stride, s_vec - 1));
    }
    if (c_vec > 0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) rc[u] = __builtin_nontemporal_load(cv + min(t0 + u * stride, c_vec - 1));
    }

    for (uint32_t i = threadIdx.x; i < (uint32_t)(kHistCopies * 256); i += kHistThreads) sh_scale[i] = 0u;
    if (threadIdx.x < 8) sh_elem[threadIdx.x] = 0u;
    __syncthreads();

    // Scales first: their partial histogram reaches the caller's array while the codes, by far
    // the larger array, are still being counted.
    uint32_t* mine = sh_scale + (threadIdx.x & (kHistCopies - 1));        // word of code c: mine[c * 64]
    for (int64_t i = t0; i < s_vec; i += 2 * stride) {               // two loads in flight per lane
        if (i != t0) {
#pragma unroll
            for (int u = 0; u < 2; ++u) rs[u] = __builtin_nontemporal_load(sv + min(i + u * stride, s_vec - 1));
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (i + u * stride >= s_vec) continue;
            const uint32_t d[4] = {rs[u].x, rs[u].y, rs[u].z, rs[u].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                atomicAdd(&mine[(d[j] & 0xFFu) * kHistCopies], 1u);
                atomicAdd(&mine[((d[j] >> 8) & 0xFFu) * kHistCopies], 1u);
                atomicAdd(&mine[((d[j] >> 16) & 0xFFu) * kHistCopies], 1u);
                atomicAdd(&mine[(d[j] >> 24) * kHistCopies], 1u);
            }
        }
    }
    if (t0 == 0) {                                                   // the few bytes outside the vectors
        for (int64_t b = 0; b < n_blocks; ++b) {
            if (b == s_head) b += s_vec << 4;
            if (b >= n_blocks) break;
            atomicAdd(&mine[(uint32_t)scales[b] * kHistCopies], 1u);
        }
    }
    __syncthreads();
    {   // four threads per code, 16 copies each
        const uint32_t code = threadIdx.x >> 2, part = threadIdx.x & 3u;
        uint32_t c = 0u;
#pragma unroll
        for (int r = 0; r < kHistCopies / 4; ++r) c += sh_scale[code * kHistCopies + part * (kHistCopies / 4) + r];
        c += dpp_u<kDppXor1>(c);
        c += dpp_u<kDppXor2>(c);
        if (part == 0u && c) atomicAdd(&scale_hist[code], (unsigned long long)c);
    }

    uint32_t cnt[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    for (int64_t i = t0; i < c_vec; i += 4 * stride) {               // four loads in flight per lane
        if (i != t0) {
#pragma unroll
            for (int u = 0; u < 4; ++u) rc[u] = __builtin_nontemporal_load(cv + min(i + u * stride, c_vec - 1));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * stride < c_vec) count_magnitudes(rc[u], cnt);
    }
    if (t0 == 0) {
        for (int64_t b = 0; b < code_bytes; ++b) {
            if (b == c_head) b += c_vec << 4;
            if (b >= code_bytes) break;
            cnt[codes[b] & 7u] += 1u;
            cnt[(codes[b] >> 4) & 7u] += 1u;
        }
    }

    // the 16 lanes of a DPP row add up in registers; one lane per row adds into the LDS
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t c = cnt[k];
        c += dpp_u<kDppXor1>(c);
        c += dpp_u<kDppXor2>(c);
        c += dpp_u<kDppHalfMirror>(c);
        c += dpp_u<kDppMirror>(c);
        if ((threadIdx.x & 15) == 0 && c) atomicAdd(&sh_elem[k], c);
    }
    __syncthreads();
    if (threadIdx.x < 8 && sh_elem[threadIdx.x]) atomicAdd(&elem_hist[threadIdx.x], (unsigned long long)sh_elem[threadIdx.x]);
}

hipError_t launch_histogram(const uint8_t* codes, const uint8_t* scales, int64_t n, int block,
                            unsigned long long* elem_hist, unsigned long long* scale_hist,
                            hipStream_t stream)
{
    hipLaunchKernelGGL(hist_clear_kernel, dim3(1), dim3(256), 0, stream, elem_hist, scale_hist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    // a lane's register counters and a workgroup's LDS counters are 32-bit: keep the elements
    // per workgroup below 2^32 by using enough workgroups (at least one per 2^31 elements)
    const int64_t n_vec = (n + 31) / 32;
    int64_t grid = (n_vec + kHistThreads - 1) / kHistThreads;
    if (grid > kHistMaxGrid) grid = kHistMaxGrid;
    const int64_t min_grid = (n >> 31) + 1;
    if (grid < min_grid) grid = min_grid;
    hipLaunchKernelGGL(histogram_kernel, dim3((unsigned)grid), dim3(kHistThreads), 0, stream,
                       codes, scales, n, n / block, elem_hist, scale_hist);
    return hipGetLastError();
}

}  // namespace mxq
