// The argument-validation path of the C ABI under AddressSanitizer / UndefinedBehaviorSanitizer.
//
// Linked with paper_2605_08565_amd/csrc/mxq_api.hip itself; the kernel launchers it calls are
// replaced by the counting stubs below, so no GPU is needed and nothing is ever dereferenced: a
// valid call must reach its launcher exactly once, an invalid one must be refused before it.
// Build: hipcc --offload-arch=gfx950 -O1 -g -Xarch_host -fsanitize=address -Xarch_host
//        -fsanitize=undefined -Xarch_host -fno-sanitize-recover=all  this file + mxq_api.hip
#include <cmath>
#include <cstdio>
#include <cstdlib>

#include "../../include/mxq.h"
#include "../../paper_2605_08565_amd/csrc/mxq_launch.hpp"

static int g_launches = 0;
static mxq::StreamArgs g_last;

namespace mxq {
hipError_t launch_stream(const StreamArgs& a) { ++g_launches; g_last = a; return hipSuccess; }
hipError_t launch_brute(const StreamArgs& a) { ++g_launches; g_last = a; return hipSuccess; }
hipError_t launch_stream_batch(const StreamArgs* t, int count, hipStream_t) { ++g_launches; g_last = t[count - 1]; return hipSuccess; }
hipError_t launch_dequant(const DequantArgs&) { ++g_launches; return hipSuccess; }
hipError_t launch_clip_sse(const void*, const uint8_t*, int64_t, int, int, int, float, float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_histogram(const uint8_t*, const uint8_t*, int64_t, int, unsigned long long*, unsigned long long*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_absmax(const void*, int64_t, int, float*, uint32_t*, bool, float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_absmax_static(const void*, int64_t, int, float*, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace mxq

static int g_bad = 0, g_checks = 0;
#define EXPECT(call, status, launches)                                                                      \
    do {                                                                                                    \
        const int before_ = g_launches;                                                                     \
        const int got_ = (call);                                                                            \
        ++g_checks;                                                                                         \
        if (got_ != (status) || g_launches - before_ != (launches)) {                                       \
            ++g_bad;                                                                                        \
            std::printf("line %d: status %d (want %d), launches %d (want %d)\n", __LINE__, got_, (int)(status), \
                        g_launches - before_, (int)(launches));                                             \
        }                                                                                                   \
    } while (0)

int main()
{
    // fake, aligned, never dereferenced device addresses
    uint8_t* const P = reinterpret_cast<uint8_t*>(0x10000);
    float* const F = reinterpret_cast<float*>(0x20000);
    const float inf = INFINITY, nan = NAN;

    // ---- mxq_quantize / mxq_quantize_clip
    for (int block : {2, 4, 8, 16, 32, 64, 128})
        for (int fmt = 0; fmt < 3; ++fmt)
            for (int rec = 0; rec < 6; ++rec)
                for (int dt = 0; dt < 2; ++dt) {
                    const bool unsupported = fmt == 0 && rec >= 2 && rec != 4;
                    EXPECT(mxq_quantize(P, 3, 128, block, 0, fmt, rec, 1.0f, P, P, F, dt, nullptr),
                           unsupported ? MXQ_ERR_UNSUPPORTED : MXQ_OK, unsupported ? 0 : 1);
                    EXPECT(mxq_quantize_clip(P, 3, 128, block, 0, fmt, rec, 0.5f, P, P, nullptr, F, dt, nullptr),
                           unsupported ? MXQ_ERR_UNSUPPORTED : MXQ_OK, unsupported ? 0 : 1);
                }
    if (g_last.n != 3 * 128 || g_last.clip != F || g_last.sse != nullptr || g_last.T != 0.5f) { ++g_bad; std::printf("arguments not forwarded\n"); }
    EXPECT(mxq_quantize(nullptr, 4, 64, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, 0, 1.0f, nullptr, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, 0, 1.0f, P, nullptr, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P, -1, 64, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P, 4, -64, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    for (int block : {0, 1, 3, 5, 24, 256, -16})
        EXPECT(mxq_quantize(P, 4, 1536, block, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P, 4, 72, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P, 4, 64, 16, 1, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    for (int fmt : {-1, 3, 1000})
        EXPECT(mxq_quantize(P, 4, 64, 16, 0, fmt, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    for (int rec : {-1, 6, 99})
        EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, rec, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    for (int dt : {-1, 2})
        EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, 0, 1.0f, P, P, F, dt, nullptr), MXQ_ERR_INVALID_ARG, 0);
    for (float T : {0.0f, -1.0f, inf, -inf, nan})
        EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, 0, T, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P + 2, 4, 64, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, 0, 1.0f, P + 1, P, F, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, 0, 1.0f, P, P + 2, F, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_quantize(P, 4, 64, 16, 0, 1, 0, 1.0f, P, P, F + 1, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_quantize_clip(P, 4, 64, 16, 0, 1, 0, 1.0f, P, P, F, F + 2, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_quantize(P, (int64_t)1 << 40, (int64_t)1 << 40, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize(P, (int64_t)1 << 30, (int64_t)1 << 12, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_ERR_UNSUPPORTED, 0);
    EXPECT(mxq_quantize(P, 0, 64, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_OK, 0);
    EXPECT(mxq_quantize(nullptr, 0, 64, 16, 0, 1, 0, 1.0f, nullptr, nullptr, nullptr, 0, nullptr), MXQ_OK, 0);
    EXPECT(mxq_quantize(P, 3, 0, 16, 0, 1, 0, 1.0f, P, P, F, 0, nullptr), MXQ_OK, 0);

    // ---- mxq_quantize_batch: one launcher call per group of up to 64 non-empty tensors
    {
        mxq_tensor t[70];
        for (int i = 0; i < 70; ++i) t[i] = mxq_tensor{P, 2, 64, P, P, (i & 1) ? F : nullptr};
        t[3].rows = 0;                                                       // skipped
        EXPECT(mxq_quantize_batch(t, 70, 16, 0, 1, 2, 0, nullptr), MXQ_OK, 2);
        if (g_last.n != 128 || g_last.recipe != 2 || g_last.T != 1.0f) { ++g_bad; std::printf("batch arguments not forwarded\n"); }
        EXPECT(mxq_quantize_batch(t, 5, 16, 0, 1, 0, 1, nullptr), MXQ_OK, 1);
        EXPECT(mxq_quantize_batch(t, 0, 16, 0, 1, 0, 1, nullptr), MXQ_OK, 0);
        EXPECT(mxq_quantize_batch(nullptr, 3, 16, 0, 1, 0, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
        EXPECT(mxq_quantize_batch(t, 70, 16, 0, 1, 4, 0, nullptr), MXQ_ERR_UNSUPPORTED, 0);
        EXPECT(mxq_quantize_batch(t, 70, 16, 0, 0, 3, 0, nullptr), MXQ_ERR_UNSUPPORTED, 0);
        t[69].cols = 72;
        EXPECT(mxq_quantize_batch(t, 70, 16, 0, 1, 0, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
        t[69].cols = 64; t[68].x = P + 4;
        EXPECT(mxq_quantize_batch(t, 70, 16, 0, 1, 0, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
        t[68].x = nullptr;
        EXPECT(mxq_quantize_batch(t, 70, 16, 0, 1, 0, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
        t[68].x = P; t[0].rows = (int64_t)1 << 28; t[0].cols = (int64_t)1 << 12;
        EXPECT(mxq_quantize_batch(t, 70, 16, 0, 1, 0, 0, nullptr), MXQ_ERR_UNSUPPORTED, 0);
    }

    // ---- mxq_quantize_hier
    EXPECT(mxq_quantize_hier(P, 4, 64, 16, 0, 1, 2, F, F, P, P, F, 0, nullptr), MXQ_OK, 1);
    EXPECT(mxq_quantize_hier(P, 4, 64, 16, 0, 1, 2, F, nullptr, P, P, nullptr, 1, nullptr), MXQ_OK, 1);
    EXPECT(mxq_quantize_hier(P, 4, 64, 16, 0, 1, 2, nullptr, F, P, P, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_quantize_hier(P, 4, 64, 16, 0, 0, 5, F, F, P, P, F, 0, nullptr), MXQ_ERR_UNSUPPORTED, 0);
    EXPECT(mxq_quantize_hier(P, 4, 64, 16, 0, 1, 2, reinterpret_cast<float*>(0x20002), F, P, P, F, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_quantize_hier(P, 4, 64, 16, 0, 1, 2, F, reinterpret_cast<float*>(0x20001), P, P, F, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_quantize_hier(P, 0, 64, 16, 0, 1, 2, F, F, P, P, F, 0, nullptr), MXQ_OK, 0);

    // ---- de-quantise
    EXPECT(mxq_dequantize(P, P, 4, 64, 16, 0, 1, 1.0f, P, 1, nullptr), MXQ_OK, 1);
    EXPECT(mxq_dequantize(P, P, 4, 64, 16, 0, 2, 0.25f, P, 0, nullptr), MXQ_OK, 1);
    EXPECT(mxq_dequantize(nullptr, P, 4, 64, 16, 0, 1, 1.0f, P, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize(P, nullptr, 4, 64, 16, 0, 1, 1.0f, P, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize(P, P, 4, 64, 16, 0, 1, 1.0f, nullptr, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize(P, P, 4, 64, 5, 0, 1, 1.0f, P, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize(P, P, 4, 64, 16, 0, -1, 1.0f, P, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize(P, P, 4, 64, 16, 0, 1, 1.0f, P, 3, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize(P, P, 4, 64, 16, 0, 1, 0.0f, P, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize(P, P, 4, 64, 16, 0, 1, 1.0f, P + 8, 1, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_dequantize(P, P, 0, 64, 16, 0, 1, 1.0f, P, 1, nullptr), MXQ_OK, 0);
    EXPECT(mxq_dequantize_hier(P, P, 4, 64, 16, 0, 1, F, P, 1, nullptr), MXQ_OK, 1);
    EXPECT(mxq_dequantize_hier(P, P, 4, 64, 16, 0, 1, nullptr, P, 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_dequantize_hier(P, P, 4, 64, 16, 0, 1, reinterpret_cast<float*>(0x20002), P, 1, nullptr), MXQ_ERR_ALIGNMENT, 0);

    // ---- tensor abs-max, all four forms
    EXPECT(mxq_tensor_absmax(P, 4, 4, 0, F, nullptr), MXQ_OK, 1);
    EXPECT(mxq_tensor_absmax(P, 4, 4, 0, nullptr, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax(nullptr, 4, 4, 0, F, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax(P, 4, 4, 5, F, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax(P + 4, 4, 4, 0, F, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_tensor_absmax(nullptr, 0, 4, 0, F, nullptr), MXQ_OK, 1);
    EXPECT(mxq_tensor_absmax_acc(P, 4, 4, 1, F, F + 1, nullptr), MXQ_OK, 1);
    EXPECT(mxq_tensor_absmax_acc(P, 4, 4, 1, F, nullptr, nullptr), MXQ_OK, 1);
    EXPECT(mxq_tensor_absmax_acc(P, 4, 4, 1, F, F, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax_acc(P, 4, 4, 1, nullptr, F, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax_acc(P, 4, 4, 1, F, reinterpret_cast<float*>(0x20006), nullptr), MXQ_ERR_ALIGNMENT, 0);
    const size_t wsz = mxq_tensor_absmax_workspace_size();
    if (wsz != MXQ_ABSMAX_WORKSPACE_BYTES) { ++g_bad; std::printf("workspace size\n"); }
    EXPECT(mxq_tensor_absmax_ws(P, 4, 4, 0, F, P, wsz, nullptr), MXQ_OK, 1);
    EXPECT(mxq_tensor_absmax_ws(P, 4, 4, 0, F, nullptr, wsz, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax_ws(P, 4, 4, 0, F, P, wsz - 1, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax_ws(P, 4, 4, 0, F, P + 4, wsz, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_tensor_absmax_static(P, 4, 4, 0, F, nullptr), MXQ_OK, 1);
    EXPECT(mxq_tensor_absmax_static(P, 4, 4, 0, nullptr, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_tensor_absmax_static(P, (int64_t)1 << 21, ((int64_t)1 << 19) + 8, 0, F, nullptr), MXQ_ERR_UNSUPPORTED, 0);

    // ---- diagnostics
    EXPECT(mxq_clip_sse(P, P, 4, 64, 16, 0, 1, 1.0f, F, 0, nullptr), MXQ_OK, 1);
    EXPECT(mxq_clip_sse(nullptr, P, 4, 64, 16, 0, 1, 1.0f, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_clip_sse(P, nullptr, 4, 64, 16, 0, 1, 1.0f, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_clip_sse(P, P, 4, 64, 16, 0, 1, 1.0f, nullptr, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_clip_sse(P, P, 4, 64, 7, 0, 1, 1.0f, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_clip_sse(P, P, 4, 64, 16, 0, 1, -2.0f, F, 0, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_clip_sse(P, P, 4, 64, 16, 0, 1, 1.0f, F + 1, 0, nullptr), MXQ_ERR_ALIGNMENT, 0);
    uint64_t* const H = reinterpret_cast<uint64_t*>(0x30000);
    EXPECT(mxq_histogram(P, P, 4, 64, 16, 0, H, H + 8, nullptr), MXQ_OK, 1);
    EXPECT(mxq_histogram(nullptr, P, 4, 64, 16, 0, H, H + 8, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_histogram(P, P, 4, 64, 16, 0, nullptr, H + 8, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_histogram(P, P, 4, 70, 16, 0, H, H + 8, nullptr), MXQ_ERR_INVALID_ARG, 0);
    EXPECT(mxq_histogram(P, P, 4, 64, 16, 0, reinterpret_cast<uint64_t*>(0x30004), H + 8, nullptr), MXQ_ERR_ALIGNMENT, 0);
    EXPECT(mxq_histogram(P + 2, P, 4, 64, 16, 0, H, H + 8, nullptr), MXQ_ERR_ALIGNMENT, 0);

    // ---- host helpers
    if (mxq_num_candidates(0) != 255 || mxq_num_candidates(1) != 126 || mxq_num_candidates(2) != 254 ||
        mxq_num_candidates(3) != -1) { ++g_bad; std::printf("num_candidates\n"); }
    for (int fmt = -1; fmt < 4; ++fmt)
        for (int c = 0; c < 256; ++c) (void)mxq_scale_decode(fmt, (uint8_t)c);
    if (mxq_scale_decode(1, 0x7E) != 448.0f || mxq_scale_decode(1, 1) != 0x1p-9f || !std::isnan(mxq_scale_decode(1, 0x7F)) ||
        mxq_scale_decode(2, 0xFE) != 114688.0f || mxq_scale_decode(0, 127) != 1.0f) { ++g_bad; std::printf("scale_decode\n"); }
    if (mxq_tensor_scale_from_absmax(2688.0f, 0, 1) != 1.0f || mxq_tensor_scale_from_absmax(0.0f, 0, 1) != 1.0f ||
        !std::isnan(mxq_tensor_scale_from_absmax(1.0f, 0, 9)) || !std::isnan(mxq_tensor_scale_from_absmax(1.0f, 1, 1))) { ++g_bad; std::printf("tensor_scale\n"); }
    for (int st = -6; st < 3; ++st) if (!mxq_status_string(st)) { ++g_bad; std::printf("status_string\n"); }

    std::printf("boundary_sanitize checks=%d launches=%d bad=%d\n", g_checks, g_launches, g_bad);
    return g_bad ? 1 : 0;
}
