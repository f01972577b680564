// Host-side launch descriptors shared by the kernel translation units and the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mxq {

constexpr int kThreads = 256;          // 4 wavefronts per workgroup
constexpr int kMaxBatch = 8;           // tensors per launch of the batched streaming kernel

// Arguments of one quantise call after host validation; n = rows * cols (blocks never
// straddle rows because cols % block == 0, so the tensor is a flat run of blocks).
struct StreamArgs {
    const void* x;
    int64_t n;
    int dtype, block, scale_fmt, recipe;
    float T;                   // per-tensor scale by value; ignored when absmax_dev is set
    const float* absmax_dev;   // device: tensor abs-max from which the kernels derive T, or NULL
    float* t_out;              // device: receives the derived T, or NULL
    uint8_t* codes;
    uint8_t* scales;
    float* sse;
    float* clip;               // device: clipping-only block SSE, or NULL
    hipStream_t stream;
};

struct DequantArgs {
    const uint8_t* codes;
    const uint8_t* scales;
    int64_t n;
    int block, scale_fmt, dtype;
    float T;                   // per-tensor scale by value; ignored when t_dev is set
    const float* t_dev;        // device: per-tensor scale, or NULL
    void* out;
    hipStream_t stream;
};

// Grid for the streaming kernels: enough workgroups to cover the tensor once, capped so that
// each workgroup loops (the scale table is filled once per workgroup).  MI355X has 256 CUs;
// 8 resident workgroups of 4 waves each per CU.
inline int stream_grid(int64_t n_chunks)
{
    const int64_t need = (n_chunks + kThreads - 1) / kThreads;
    const int64_t cap = 256 * 8;
    return (int)(need < 1 ? 1 : (need < cap ? need : cap));
}

hipError_t launch_stream(const StreamArgs& a);       // ABSMAX, ABSMAX_PZ, 4OVER6, 4OVER6_PZ
hipError_t launch_stream_batch(const StreamArgs* t, int count, hipStream_t stream);   // the same, several tensors per launch
hipError_t launch_brute(const StreamArgs& a);        // BRUTE
hipError_t launch_dequant(const DequantArgs& a);
hipError_t launch_clip_sse(const void* x, const uint8_t* scales, int64_t n, int dtype, int block,
                           int scale_fmt, float T, float* out, hipStream_t stream);
hipError_t launch_histogram(const uint8_t* codes, const uint8_t* scales, int64_t n, int block,
                            unsigned long long* elem_hist, unsigned long long* scale_hist,
                            hipStream_t stream);
hipError_t launch_absmax(const void* x, int64_t n, int dtype, float* out, uint32_t* ws, bool accumulate,
                         float* clear_word, hipStream_t stream);
hipError_t launch_absmax_static(const void* x, int64_t n, int dtype, float* out, hipStream_t stream);

}  // namespace mxq
