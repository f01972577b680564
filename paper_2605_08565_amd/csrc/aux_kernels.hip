// De-quantisation (Section 2, paragraph after Eq. 2: the codes times the block scale) and the tensor
// abs-max of hierarchical scaling (first stage of the two-stage process, Section 2).
#include "mxq_device.hpp"
#include "mxq_launch.hpp"

#include <mutex>

namespace mxq {

using bf16x2 = __bf16 __attribute__((ext_vector_type(2)));

// Two fp32 -> two bf16 (round to nearest even, v_cvt_pk_bf16_f32), first value in the low half.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// bf16 output: one lane = 8 consecutive elements = one dword of codes = one 128-bit store; a
// block of b >= 8 elements spans b/8 lanes that all read the same scale byte, a block of b < 8
// lies inside the lane.
template <int B>
__global__ void __launch_bounds__(kThreads)
dequant_bf16_kernel(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales, int64_t n,
                    int fmt, float T_arg, const float* __restrict__ t_dev, uint16_t* __restrict__ out)
{
    const float T = t_dev ? *t_dev : T_arg;                         // per-tensor scale by value or from device memory
    constexpr int NBLK = (B < 8) ? 8 / B : 1;
    constexpr int LANES = (B < 8) ? 1 : B / 8;
    constexpr int EPB = (B < 8) ? B : 8;
    const int64_t n_chunks = (n + 7) >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t c0 = (int64_t)blockIdx.x * kThreads; c0 < n_chunks; c0 += stride) {     // uniform
        const uint32_t tid = threadIdx.x;
        if (tid >= (uint32_t)min((int64_t)kThreads, n_chunks - c0)) continue;
        const int64_t chunk = c0 + tid;
        const int64_t first = chunk << 3;
        const int count = (int)min((int64_t)8, n - first);
        uint32_t packed = 0u;
        if (count == 8) {
            packed = __builtin_nontemporal_load(codes + chunk);
        } else {
            const uint8_t* cb = reinterpret_cast<const uint8_t*>(codes) + chunk * 4;
            for (int i = 0; i < count / 2; ++i) packed |= (uint32_t)cb[i] << (8 * i);
        }
        float S[NBLK];
        if (B < 8 && count == 8) {                  // the lane's 8/B scale bytes in one load
            uint32_t sb;
            if constexpr (NBLK == 4) sb = *reinterpret_cast<const uint32_t*>(scales + chunk * 4);
            else sb = *reinterpret_cast<const uint16_t*>(scales + chunk * 2);
#pragma unroll
            for (int k = 0; k < NBLK; ++k) S[k] = scale_byte_value(fmt, (sb >> (8 * k)) & 0xFFu);
        } else {
#pragma unroll
            for (int k = 0; k < NBLK; ++k) {
                const int64_t blk = (B >= 8) ? chunk / LANES : chunk * NBLK + k;
                S[k] = (B >= 8 || k < count / B) ? scale_byte_value(fmt, scales[blk]) : 0.0f;
            }
        }
        float r[8];
        e2m1_unpack8(packed, 1.0f, r);
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = (r[i] * S[i / EPB]) * T;
        if (count == 8) {
            u32x4 o;
            o.x = pack_bf16x2(r[0], r[1]);
            o.y = pack_bf16x2(r[2], r[3]);
            o.z = pack_bf16x2(r[4], r[5]);
            o.w = pack_bf16x2(r[6], r[7]);
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(out + first));
        } else {
            for (int i = 0; i < count; ++i) out[first + i] = (uint16_t)(pack_bf16x2(r[i], 0.0f) & 0xFFFFu);
        }
    }
}

// fp32 output: one lane = 4 consecutive elements = 16 bits of codes = one 128-bit store, so a
// store instruction of a wavefront covers 1 KiB without gaps (with 8 elements per lane its two
// stores would each leave every other 16 bytes untouched).  n is even, so the ragged last lane
// holds 2 elements.
template <int B>
__global__ void __launch_bounds__(kThreads)
dequant_f32_kernel(const uint16_t* __restrict__ codes, const uint8_t* __restrict__ scales, int64_t n,
                   int fmt, float T_arg, const float* __restrict__ t_dev, float* __restrict__ out)
{
    const float T = t_dev ? *t_dev : T_arg;
    constexpr int NBLK = (B < 4) ? 4 / B : 1;
    constexpr int EPB = (B < 4) ? B : 4;
    const int64_t n_half = (n + 3) >> 2;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t h0 = (int64_t)blockIdx.x * kThreads; h0 < n_half; h0 += stride) {       // uniform
        const uint32_t tid = threadIdx.x;
        if (tid >= (uint32_t)min((int64_t)kThreads, n_half - h0)) continue;
        const int64_t h = h0 + tid;
        const int64_t first = h << 2;
        const int count = (int)min((int64_t)4, n - first);
        const uint32_t packed = (count == 4) ? (uint32_t)__builtin_nontemporal_load(codes + h)
                                             : (uint32_t)reinterpret_cast<const uint8_t*>(codes)[h * 2];
        float S[NBLK];
        if (B == 2 && count == 4) {                 // both scale bytes of the lane in one load
            const uint32_t sb = *reinterpret_cast<const uint16_t*>(scales + h * 2);
#pragma unroll
            for (int k = 0; k < NBLK; ++k) S[k] = scale_byte_value(fmt, (sb >> (8 * k)) & 0xFFu);
        } else {
#pragma unroll
            for (int k = 0; k < NBLK; ++k) {
                const int64_t blk = (B >= 4) ? first / B : h * NBLK + k;
                S[k] = (B >= 4 || k < count / B) ? scale_byte_value(fmt, scales[blk]) : 0.0f;
            }
        }
        float r[4];
        e2m1_unpack2<0>(packed, 1.0f, r[0], r[1]);
        e2m1_unpack2<1>(packed, 1.0f, r[2], r[3]);
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (r[i] * S[i / EPB]) * T;
        if (count == 4) {
            const u32x4 o = {f2u(r[0]), f2u(r[1]), f2u(r[2]), f2u(r[3])};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(out + first));
        } else {
            for (int i = 0; i < count; ++i) out[first + i] = r[i];
        }
    }
}

static void launch_dequant_f32(const DequantArgs& a)
{
    const int grid = stream_grid((a.n + 3) / 4);
#define MXQ_DQF(BB)                                                                                  \
    hipLaunchKernelGGL((dequant_f32_kernel<BB>), dim3(grid), dim3(kThreads), 0, a.stream,           \
                       (const uint16_t*)a.codes, a.scales, a.n, a.scale_fmt, a.T, a.t_dev, (float*)a.out)
    switch (a.block) {
        case 2: MXQ_DQF(2); break;
        case 4: MXQ_DQF(4); break;
        case 8: MXQ_DQF(8); break;
        case 16: MXQ_DQF(16); break;
        case 32: MXQ_DQF(32); break;
        case 64: MXQ_DQF(64); break;
        default: MXQ_DQF(128); break;
    }
#undef MXQ_DQF
}

static void launch_dequant_bf16(const DequantArgs& a)
{
    const int grid = stream_grid((a.n + 7) / 8);
#define MXQ_DQ(BB)                                                                                   \
    hipLaunchKernelGGL((dequant_bf16_kernel<BB>), dim3(grid), dim3(kThreads), 0, a.stream,          \
                       (const uint32_t*)a.codes, a.scales, a.n, a.scale_fmt, a.T, a.t_dev, (uint16_t*)a.out)
    switch (a.block) {
        case 2: MXQ_DQ(2); break;
        case 4: MXQ_DQ(4); break;
        case 8: MXQ_DQ(8); break;
        case 16: MXQ_DQ(16); break;
        case 32: MXQ_DQ(32); break;
        case 64: MXQ_DQ(64); break;
        default: MXQ_DQ(128); break;
    }
#undef MXQ_DQ
}

hipError_t launch_dequant(const DequantArgs& a)
{
    if (a.dtype == kBF16) launch_dequant_bf16(a);
    else launch_dequant_f32(a);
    return hipGetLastError();
}

// Tensor abs-max.  |x| of finite fp32 values orders like the unsigned integer bits & 0x7fffffff,
// so the reduction is an integer max; the workgroups' partial results meet in one 32-bit atomic
// max on a device word.  Two closing schemes:
//   * no workspace: the word is the caller's output, which a one-thread kernel clears first (a
//     kernel, not a memset node, so the pair can be captured in a graph) -- two launches -- or
//     which the caller guarantees to hold zero (or a maximum to be continued) -- one launch; that
//     form can clear a second word on the way, the output of the caller's next call;
//   * workspace (two words: accumulator, ticket; both zero between calls): every workgroup adds
//     its maximum to the accumulator, then takes a ticket; the workgroup that draws the last
//     ticket copies the accumulator to the output and returns both words to zero -- one launch.
__global__ void absmax_clear_kernel(uint32_t* out) { *out = 0u; }

// One workgroup of 1024 threads per compute unit walks tiles of 4 x 1024 vectors with four
// independent 128-bit loads per lane in flight (16 MiB over the chip); the ragged last chunk (n
// not a multiple of 8) is read element-wise by one lane.  Few, large workgroups because the
// closing accesses to the one word serialise at about 5 ns each, whatever their kind.
constexpr int kAbsItems = 4;
constexpr int kAbsThreads = 1024;
constexpr int kAbsMaxGrid = 256;

template <int DT, bool TICKET>
__global__ void __launch_bounds__(kAbsThreads)
absmax_kernel(const void* __restrict__ x, int64_t n, uint32_t* __restrict__ out, uint32_t* __restrict__ ws,
              uint32_t* __restrict__ clear_word)
{
    if (clear_word && blockIdx.x == 0 && threadIdx.x == 0) *clear_word = 0u;      // for a LATER launch
    constexpr int64_t kVec = (DT == kBF16) ? 1 : 2;               // 128-bit vectors per chunk
    const int64_t n_vec = (n >> 3) * kVec;                         // complete vectors
    const int64_t tile = (int64_t)kAbsThreads * kAbsItems;
    const int64_t stride = (int64_t)gridDim.x * tile;
    const u32x4* xv = static_cast<const u32x4*>(x);
    uint32_t m = 0u;
    for (int64_t v0 = (int64_t)blockIdx.x * tile; v0 < n_vec; v0 += stride) {            // uniform
        u32x4 r[kAbsItems];
#pragma unroll
        for (int i = 0; i < kAbsItems; ++i) {
            const int64_t vi = v0 + (int64_t)i * kAbsThreads;
            r[i] = u32x4{0u, 0u, 0u, 0u};
            if (vi < n_vec) {                                                               // uniform
                const uint32_t left = (uint32_t)min((int64_t)kAbsThreads, n_vec - vi);
                r[i] = __builtin_nontemporal_load(xv + vi + min((uint32_t)threadIdx.x, left - 1u));
            }
        }
#pragma unroll
        for (int i = 0; i < kAbsItems; ++i) {
            if constexpr (DT == kBF16) {
                // two bf16 per dword: compare the high halves and the low halves separately
                const uint32_t hi = max(max(r[i].x & 0x7FFF0000u, r[i].y & 0x7FFF0000u),
                                        max(r[i].z & 0x7FFF0000u, r[i].w & 0x7FFF0000u));
                const uint32_t lo = max(max(r[i].x & 0x7FFFu, r[i].y & 0x7FFFu),
                                        max(r[i].z & 0x7FFFu, r[i].w & 0x7FFFu));
                m = max(m, max(hi, lo << 16));
            } else {
                m = max(m, max(max(r[i].x & 0x7FFFFFFFu, r[i].y & 0x7FFFFFFFu),
                               max(r[i].z & 0x7FFFFFFFu, r[i].w & 0x7FFFFFFFu)));
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        for (int64_t i = (n >> 3) << 3; i < n; ++i) {
            uint32_t b;
            if constexpr (DT == kBF16) b = (uint32_t)static_cast<const uint16_t*>(x)[i] << 16;
            else b = static_cast<const uint32_t*>(x)[i];
            m = max(m, b & 0x7FFFFFFFu);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
    __shared__ uint32_t part[kAbsThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t w = part[0];
        for (int i = 1; i < kAbsThreads / 64; ++i) w = max(w, part[i]);
        if constexpr (!TICKET) {
            // The word only grows during a call, so a workgroup whose maximum does not exceed the
            // value it reads (at device scope, past the per-CU cache) has nothing to add: after
            // the first few workgroups almost none issues the atomic max.
            if (w > __hip_atomic_load(out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(out, w);
        } else {
            // Read-modify-writes at device scope are performed at the one point all compute dies
            // share.  The ticket is requested only after the value returned by the max has arrived
            // (its increment depends on it), i.e. after the max was performed there; the workgroup
            // that draws the last ticket therefore exchanges out a word that already holds every
            // other workgroup's contribution.  No cache-wide fence is needed (one costs several
            // microseconds here, more than the second launch it would save).
            const uint32_t before = atomicMax(ws, w);
            const uint32_t ticket = atomicAdd(ws + 1, 1u + (before >> 31));      // bit 31 is never set
            if (ticket == gridDim.x - 1u) {
                *out = atomicExch(ws, 0u);
                atomicExch(ws + 1, 0u);
            }
        }
    }
}

// `ws`: the two-word workspace of the ticket scheme, or NULL.  `accumulate` (without ws): the output
// word is not cleared first; `clear_word` (accumulate only, may be NULL) is set to zero instead.
hipError_t launch_absmax(const void* x, int64_t n, int dtype, float* out, uint32_t* ws, bool accumulate,
                         float* clear_word, hipStream_t stream)
{
    if (accumulate && n == 0) {
        if (!clear_word) return hipSuccess;
        hipLaunchKernelGGL(absmax_clear_kernel, dim3(1), dim3(1), 0, stream, (uint32_t*)clear_word);
        return hipGetLastError();
    }
    if ((!ws && !accumulate) || n == 0) {
        hipLaunchKernelGGL(absmax_clear_kernel, dim3(1), dim3(1), 0, stream, (uint32_t*)out);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess || n == 0) return e;
    }
    const int64_t n_tiles = ((n + 7) / 8 + kAbsThreads * kAbsItems - 1) / (kAbsThreads * kAbsItems);
    const int64_t capw = kAbsMaxGrid;
    const dim3 grid((unsigned)(n_tiles < 1 ? 1 : (n_tiles < capw ? n_tiles : capw))), block(kAbsThreads);
    uint32_t* o = (uint32_t*)out;
    uint32_t* cw = (uint32_t*)clear_word;
    if (dtype == kBF16) {
        if (ws) hipLaunchKernelGGL((absmax_kernel<kBF16, true>), grid, block, 0, stream, x, n, o, ws, cw);
        else hipLaunchKernelGGL((absmax_kernel<kBF16, false>), grid, block, 0, stream, x, n, o, ws, cw);
    } else {
        if (ws) hipLaunchKernelGGL((absmax_kernel<kF32, true>), grid, block, 0, stream, x, n, o, ws, cw);
        else hipLaunchKernelGGL((absmax_kernel<kF32, false>), grid, block, 0, stream, x, n, o, ws, cw);
    }
    return hipGetLastError();
}

// Workspace of the entry point that may not allocate and takes no workspace argument: the two
// words of the ticket scheme (the rest is padding to the alignment) live in the library's own
// device image, one copy per GPU, zero when the image is loaded and returned to zero by every call.
// In host code the array's name is only a handle for hipGetSymbolAddress; the address it yields for
// the current device is what kernels and launches are given.
constexpr int kStaticScratchWords = 64;
static __device__ __align__(256) uint32_t scratch[kStaticScratchWords];

constexpr int kMaxDevices = 64;
static uint32_t* g_scratch_ptr[kMaxDevices];      // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch`, resolved once per device.
static hipError_t static_scratch(uint32_t** ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<uint32_t*>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

// The ticket scheme on the library's own workspace: no allocation, no workspace argument.
hipError_t launch_absmax_static(const void* x, int64_t n, int dtype, float* out, hipStream_t stream)
{
    uint32_t* ws = nullptr;
    const hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return e;
    return launch_absmax(x, n, dtype, out, ws, false, nullptr, stream);
}

}  // namespace mxq
