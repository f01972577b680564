// C ABI of libmxq (see include/mxq.h): host-side validation and dispatch.  No allocation, no
// synchronisation, no global state.
#include "../../include/mxq.h"
#include "mxq_arith.hpp"
#include "mxq_launch.hpp"

#include <cmath>
#include <cstddef>
#include <cstdint>

namespace {

bool valid_block(int b)
{
    return b == 2 || b == 4 || b == 8 || b == 16 || b == 32 || b == 64 || b == 128;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Host copy of the scale decode, for mxq_scale_decode only.
float host_scale_decode(int fmt, unsigned code)
{
    if (fmt == MXQ_SCALE_E8M0) return code == 255u ? NAN : std::ldexp(1.0f, (int)code - 127);
    int bias, maxc;
    if (fmt == MXQ_SCALE_E4M3) { bias = 7; maxc = 0x7E; }
    else if (fmt == MXQ_SCALE_UE5M3) { bias = 15; maxc = 0xFE; }
    else return NAN;
    if ((int)code > maxc) return NAN;
    const int e = (int)(code >> 3), m = (int)(code & 7u);
    if (e == 0) return std::ldexp((float)m, 1 - bias - 3);
    return std::ldexp((float)(8 + m), e - bias - 3);
}

}  // namespace

extern "C" {

// Validation and launch shared by mxq_quantize (T by value) and mxq_quantize_hier (T derived on
// the device from *absmax_dev).
static int quantize_common(const void* x, int64_t rows, int64_t cols, int block,
                           int elem_fmt, int scale_fmt, int recipe, float tensor_scale,
                           const float* absmax_dev, float* t_out,
                           uint8_t* codes_out, uint8_t* scales_out, float* sse_out, float* clip_out,
                           int x_dtype, void* stream)
{
    if (rows < 0 || cols < 0) return MXQ_ERR_INVALID_ARG;
    if (!valid_block(block) || cols % block != 0) return MXQ_ERR_INVALID_ARG;
    if (elem_fmt != MXQ_ELEM_E2M1) return MXQ_ERR_INVALID_ARG;
    if (scale_fmt < MXQ_SCALE_E8M0 || scale_fmt > MXQ_SCALE_UE5M3) return MXQ_ERR_INVALID_ARG;
    if (recipe < MXQ_RECIPE_ABSMAX || recipe > MXQ_RECIPE_BRUTE_PRUNED) return MXQ_ERR_INVALID_ARG;
    if (x_dtype != MXQ_DT_BF16 && x_dtype != MXQ_DT_F32) return MXQ_ERR_INVALID_ARG;
    if (!(tensor_scale > 0.0f) || std::isinf(tensor_scale)) return MXQ_ERR_INVALID_ARG;
    if (rows > 0 && cols > INT64_MAX / rows) return MXQ_ERR_INVALID_ARG;
    if (scale_fmt == MXQ_SCALE_E8M0 && recipe >= MXQ_RECIPE_4OVER6 && recipe != MXQ_RECIPE_BRUTE)
        return MXQ_ERR_UNSUPPORTED;
    const int64_t n = rows * cols;
    if (n == 0) return MXQ_OK;
    if (n >= ((int64_t)1 << 42)) return MXQ_ERR_UNSUPPORTED;        // 32-bit slice counters
    if (!x || !codes_out || !scales_out) return MXQ_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(codes_out, 4) || !aligned(scales_out, 4) ||
        (sse_out && !aligned(sse_out, 16)) || (clip_out && !aligned(clip_out, 16)) ||
        !aligned(absmax_dev, 4) || !aligned(t_out, 4))
        return MXQ_ERR_ALIGNMENT;

    mxq::StreamArgs a;
    a.x = x; a.n = n; a.dtype = x_dtype; a.block = block; a.scale_fmt = scale_fmt;
    a.recipe = recipe; a.T = tensor_scale; a.absmax_dev = absmax_dev; a.t_out = t_out;
    a.codes = codes_out; a.scales = scales_out;
    a.sse = sse_out; a.clip = clip_out; a.stream = static_cast<hipStream_t>(stream);
    const hipError_t e = (recipe >= MXQ_RECIPE_BRUTE) ? mxq::launch_brute(a) : mxq::launch_stream(a);
    return e == hipSuccess ? MXQ_OK : MXQ_ERR_HIP;
}

int mxq_quantize(const void* x, int64_t rows, int64_t cols, int block,
                 int elem_fmt, int scale_fmt, int recipe, float tensor_scale,
                 uint8_t* codes_out, uint8_t* scales_out, float* sse_out,
                 int x_dtype, void* stream)
{
    return quantize_common(x, rows, cols, block, elem_fmt, scale_fmt, recipe, tensor_scale, nullptr, nullptr,
                           codes_out, scales_out, sse_out, nullptr, x_dtype, stream);
}

int mxq_quantize_clip(const void* x, int64_t rows, int64_t cols, int block,
                      int elem_fmt, int scale_fmt, int recipe, float tensor_scale,
                      uint8_t* codes_out, uint8_t* scales_out, float* sse_out, float* clip_sse_out,
                      int x_dtype, void* stream)
{
    return quantize_common(x, rows, cols, block, elem_fmt, scale_fmt, recipe, tensor_scale, nullptr, nullptr,
                           codes_out, scales_out, sse_out, clip_sse_out, x_dtype, stream);
}

int mxq_quantize_batch(const mxq_tensor* tensors, int count, int block,
                       int elem_fmt, int scale_fmt, int recipe, int x_dtype, void* stream)
{
    if (count < 0 || (count > 0 && !tensors)) return MXQ_ERR_INVALID_ARG;
    if (!valid_block(block)) return MXQ_ERR_INVALID_ARG;
    if (elem_fmt != MXQ_ELEM_E2M1) return MXQ_ERR_INVALID_ARG;
    if (scale_fmt < MXQ_SCALE_E8M0 || scale_fmt > MXQ_SCALE_UE5M3) return MXQ_ERR_INVALID_ARG;
    if (recipe < MXQ_RECIPE_ABSMAX || recipe > MXQ_RECIPE_BRUTE_PRUNED) return MXQ_ERR_INVALID_ARG;
    if (x_dtype != MXQ_DT_BF16 && x_dtype != MXQ_DT_F32) return MXQ_ERR_INVALID_ARG;
    if (recipe >= MXQ_RECIPE_BRUTE) return MXQ_ERR_UNSUPPORTED;               // the search is never launch-bound
    if (scale_fmt == MXQ_SCALE_E8M0 && recipe >= MXQ_RECIPE_4OVER6) return MXQ_ERR_UNSUPPORTED;
    // every tensor is validated before anything is launched
    int64_t total = 0;
    for (int i = 0; i < count; ++i) {
        const mxq_tensor& t = tensors[i];
        if (t.rows < 0 || t.cols < 0 || t.cols % block != 0) return MXQ_ERR_INVALID_ARG;
        if (t.rows > 0 && t.cols > INT64_MAX / t.rows) return MXQ_ERR_INVALID_ARG;
        const int64_t n = t.rows * t.cols;
        if (n == 0) continue;
        if (n >= ((int64_t)1 << 40) || (total += n) >= ((int64_t)1 << 40)) return MXQ_ERR_UNSUPPORTED;   // 32-bit slice counters
        if (!t.x || !t.codes_out || !t.scales_out) return MXQ_ERR_INVALID_ARG;
        if (!aligned(t.x, 16) || !aligned(t.codes_out, 4) || !aligned(t.scales_out, 4) ||
            (t.sse_out && !aligned(t.sse_out, 16)))
            return MXQ_ERR_ALIGNMENT;
    }
    constexpr int kGroup = 64;
    mxq::StreamArgs a[kGroup];
    int m = 0;
    for (int i = 0; i <= count; ++i) {
        if (i < count) {
            const mxq_tensor& t = tensors[i];
            const int64_t n = t.rows * t.cols;
            if (n == 0) continue;
            mxq::StreamArgs& s = a[m++];
            s.x = t.x; s.n = n; s.dtype = x_dtype; s.block = block; s.scale_fmt = scale_fmt; s.recipe = recipe;
            s.T = 1.0f; s.absmax_dev = nullptr; s.t_out = nullptr; s.codes = t.codes_out; s.scales = t.scales_out;
            s.sse = t.sse_out; s.clip = nullptr; s.stream = static_cast<hipStream_t>(stream);
        }
        if (m == kGroup || (i == count && m > 0)) {
            if (mxq::launch_stream_batch(a, m, static_cast<hipStream_t>(stream)) != hipSuccess) return MXQ_ERR_HIP;
            m = 0;
        }
    }
    return MXQ_OK;
}

int mxq_quantize_hier(const void* x, int64_t rows, int64_t cols, int block,
                      int elem_fmt, int scale_fmt, int recipe,
                      const float* absmax, float* tensor_scale_out,
                      uint8_t* codes_out, uint8_t* scales_out, float* sse_out,
                      int x_dtype, void* stream)
{
    if (!absmax) return MXQ_ERR_INVALID_ARG;
    return quantize_common(x, rows, cols, block, elem_fmt, scale_fmt, recipe, 1.0f, absmax, tensor_scale_out,
                           codes_out, scales_out, sse_out, nullptr, x_dtype, stream);
}

static int dequantize_common(const uint8_t* codes, const uint8_t* scales,
                             int64_t rows, int64_t cols, int block,
                             int elem_fmt, int scale_fmt, float tensor_scale, const float* t_dev,
                             void* x_out, int out_dtype, void* stream)
{
    if (rows < 0 || cols < 0) return MXQ_ERR_INVALID_ARG;
    if (!valid_block(block) || cols % block != 0) return MXQ_ERR_INVALID_ARG;
    if (elem_fmt != MXQ_ELEM_E2M1) return MXQ_ERR_INVALID_ARG;
    if (scale_fmt < MXQ_SCALE_E8M0 || scale_fmt > MXQ_SCALE_UE5M3) return MXQ_ERR_INVALID_ARG;
    if (out_dtype != MXQ_DT_BF16 && out_dtype != MXQ_DT_F32) return MXQ_ERR_INVALID_ARG;
    if (!(tensor_scale > 0.0f) || std::isinf(tensor_scale)) return MXQ_ERR_INVALID_ARG;
    if (rows > 0 && cols > INT64_MAX / rows) return MXQ_ERR_INVALID_ARG;
    const int64_t n = rows * cols;
    if (n == 0) return MXQ_OK;
    if (!codes || !scales || !x_out) return MXQ_ERR_INVALID_ARG;
    if (!aligned(codes, 4) || !aligned(scales, 4) || !aligned(x_out, 16) || !aligned(t_dev, 4))
        return MXQ_ERR_ALIGNMENT;

    mxq::DequantArgs a;
    a.codes = codes; a.scales = scales; a.n = n; a.block = block; a.scale_fmt = scale_fmt;
    a.dtype = out_dtype; a.T = tensor_scale; a.t_dev = t_dev; a.out = x_out;
    a.stream = static_cast<hipStream_t>(stream);
    return mxq::launch_dequant(a) == hipSuccess ? MXQ_OK : MXQ_ERR_HIP;
}

int mxq_dequantize(const uint8_t* codes, const uint8_t* scales,
                   int64_t rows, int64_t cols, int block,
                   int elem_fmt, int scale_fmt, float tensor_scale,
                   void* x_out, int out_dtype, void* stream)
{
    return dequantize_common(codes, scales, rows, cols, block, elem_fmt, scale_fmt, tensor_scale, nullptr,
                             x_out, out_dtype, stream);
}

int mxq_dequantize_hier(const uint8_t* codes, const uint8_t* scales,
                        int64_t rows, int64_t cols, int block,
                        int elem_fmt, int scale_fmt, const float* tensor_scale,
                        void* x_out, int out_dtype, void* stream)
{
    if (!tensor_scale) return MXQ_ERR_INVALID_ARG;
    return dequantize_common(codes, scales, rows, cols, block, elem_fmt, scale_fmt, 1.0f, tensor_scale,
                             x_out, out_dtype, stream);
}

static int absmax_common(const void* x, int64_t rows, int64_t cols, int x_dtype,
                         float* absmax_out, uint32_t* ws, bool accumulate, float* clear_word, void* stream)
{
    if (rows < 0 || cols < 0 || !absmax_out) return MXQ_ERR_INVALID_ARG;
    if (x_dtype != MXQ_DT_BF16 && x_dtype != MXQ_DT_F32) return MXQ_ERR_INVALID_ARG;
    if (rows > 0 && cols > INT64_MAX / rows) return MXQ_ERR_INVALID_ARG;
    const int64_t n = rows * cols;
    if (n > 0 && !x) return MXQ_ERR_INVALID_ARG;
    if ((n > 0 && !aligned(x, 16)) || !aligned(absmax_out, 4)) return MXQ_ERR_ALIGNMENT;
    if (!aligned(clear_word, 4)) return MXQ_ERR_ALIGNMENT;
    if (clear_word == absmax_out) return MXQ_ERR_INVALID_ARG;
    return mxq::launch_absmax(x, n, x_dtype, absmax_out, ws, accumulate, clear_word,
                              static_cast<hipStream_t>(stream)) == hipSuccess ? MXQ_OK : MXQ_ERR_HIP;
}

int mxq_tensor_absmax(const void* x, int64_t rows, int64_t cols, int x_dtype,
                      float* absmax_out, void* stream)
{
    return absmax_common(x, rows, cols, x_dtype, absmax_out, nullptr, false, nullptr, stream);
}

int mxq_tensor_absmax_acc(const void* x, int64_t rows, int64_t cols, int x_dtype,
                          float* absmax_inout, float* clear_word, void* stream)
{
    return absmax_common(x, rows, cols, x_dtype, absmax_inout, nullptr, true, clear_word, stream);
}

size_t mxq_tensor_absmax_workspace_size(void) { return MXQ_ABSMAX_WORKSPACE_BYTES; }

int mxq_tensor_absmax_ws(const void* x, int64_t rows, int64_t cols, int x_dtype,
                         float* absmax_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!workspace || workspace_bytes < MXQ_ABSMAX_WORKSPACE_BYTES) return MXQ_ERR_INVALID_ARG;
    if (!aligned(workspace, 8)) return MXQ_ERR_ALIGNMENT;
    return absmax_common(x, rows, cols, x_dtype, absmax_out, static_cast<uint32_t*>(workspace), false, nullptr, stream);
}

int mxq_tensor_absmax_static(const void* x, int64_t rows, int64_t cols, int x_dtype,
                             float* absmax_out, void* stream)
{
    if (rows < 0 || cols < 0 || !absmax_out) return MXQ_ERR_INVALID_ARG;
    if (x_dtype != MXQ_DT_BF16 && x_dtype != MXQ_DT_F32) return MXQ_ERR_INVALID_ARG;
    if (rows > 0 && cols > INT64_MAX / rows) return MXQ_ERR_INVALID_ARG;
    const int64_t n = rows * cols;
    if (n > MXQ_ABSMAX_STATIC_MAX_ELEMENTS) return MXQ_ERR_UNSUPPORTED;
    if (n > 0 && !x) return MXQ_ERR_INVALID_ARG;
    if ((n > 0 && !aligned(x, 16)) || !aligned(absmax_out, 4)) return MXQ_ERR_ALIGNMENT;
    return mxq::launch_absmax_static(x, n, x_dtype, absmax_out, static_cast<hipStream_t>(stream)) == hipSuccess
               ? MXQ_OK : MXQ_ERR_HIP;
}

int mxq_clip_sse(const void* x, const uint8_t* scales, int64_t rows, int64_t cols, int block,
                 int elem_fmt, int scale_fmt, float tensor_scale, float* clip_sse_out,
                 int x_dtype, void* stream)
{
    if (rows < 0 || cols < 0) return MXQ_ERR_INVALID_ARG;
    if (!valid_block(block) || cols % block != 0) return MXQ_ERR_INVALID_ARG;
    if (elem_fmt != MXQ_ELEM_E2M1) return MXQ_ERR_INVALID_ARG;
    if (scale_fmt < MXQ_SCALE_E8M0 || scale_fmt > MXQ_SCALE_UE5M3) return MXQ_ERR_INVALID_ARG;
    if (x_dtype != MXQ_DT_BF16 && x_dtype != MXQ_DT_F32) return MXQ_ERR_INVALID_ARG;
    if (!(tensor_scale > 0.0f) || std::isinf(tensor_scale)) return MXQ_ERR_INVALID_ARG;
    if (rows > 0 && cols > INT64_MAX / rows) return MXQ_ERR_INVALID_ARG;
    const int64_t n = rows * cols;
    if (n == 0) return MXQ_OK;
    if (!x || !scales || !clip_sse_out) return MXQ_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(scales, 4) || !aligned(clip_sse_out, 16)) return MXQ_ERR_ALIGNMENT;
    return mxq::launch_clip_sse(x, scales, n, x_dtype, block, scale_fmt, tensor_scale, clip_sse_out,
                                static_cast<hipStream_t>(stream)) == hipSuccess ? MXQ_OK : MXQ_ERR_HIP;
}

int mxq_histogram(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                  int block, int elem_fmt, uint64_t* elem_hist, uint64_t* scale_hist, void* stream)
{
    if (rows < 0 || cols < 0) return MXQ_ERR_INVALID_ARG;
    if (!valid_block(block) || cols % block != 0) return MXQ_ERR_INVALID_ARG;
    if (elem_fmt != MXQ_ELEM_E2M1) return MXQ_ERR_INVALID_ARG;
    if (rows > 0 && cols > INT64_MAX / rows) return MXQ_ERR_INVALID_ARG;
    if (!elem_hist || !scale_hist) return MXQ_ERR_INVALID_ARG;
    const int64_t n = rows * cols;
    if (n > 0 && (!codes || !scales)) return MXQ_ERR_INVALID_ARG;
    if (!aligned(elem_hist, 8) || !aligned(scale_hist, 8)) return MXQ_ERR_ALIGNMENT;
    if (n > 0 && (!aligned(codes, 4) || !aligned(scales, 4))) return MXQ_ERR_ALIGNMENT;
    return mxq::launch_histogram(codes, scales, n, block,
                                 reinterpret_cast<unsigned long long*>(elem_hist),
                                 reinterpret_cast<unsigned long long*>(scale_hist),
                                 static_cast<hipStream_t>(stream)) == hipSuccess ? MXQ_OK : MXQ_ERR_HIP;
}

float mxq_tensor_scale_from_absmax(float absmax, int elem_fmt, int scale_fmt)
{
    if (elem_fmt != MXQ_ELEM_E2M1) return NAN;
    float sf_max;
    if (scale_fmt == MXQ_SCALE_E8M0) sf_max = host_scale_decode(scale_fmt, 254);
    else if (scale_fmt == MXQ_SCALE_E4M3) sf_max = 448.0f;
    else if (scale_fmt == MXQ_SCALE_UE5M3) sf_max = 114688.0f;
    else return NAN;
    return mxq::tensor_scale_from(absmax, sf_max);      // the function the kernels call
}

float mxq_scale_decode(int scale_fmt, uint8_t code) { return host_scale_decode(scale_fmt, code); }

int mxq_num_candidates(int scale_fmt)
{
    if (scale_fmt == MXQ_SCALE_E8M0) return 255;
    if (scale_fmt == MXQ_SCALE_E4M3) return 126;
    if (scale_fmt == MXQ_SCALE_UE5M3) return 254;
    return -1;
}

const char* mxq_status_string(int status)
{
    switch (status) {
        case MXQ_OK: return "MXQ_OK";
        case MXQ_ERR_INVALID_ARG: return "MXQ_ERR_INVALID_ARG";
        case MXQ_ERR_UNSUPPORTED: return "MXQ_ERR_UNSUPPORTED";
        case MXQ_ERR_ALIGNMENT: return "MXQ_ERR_ALIGNMENT";
        case MXQ_ERR_HIP: return "MXQ_ERR_HIP";
        default: return "MXQ_ERR_UNKNOWN";
    }
}

}  // extern "C"
