/*
 * mxq.h -- C ABI of libmxq: block-wise microscaled FP4 (E2M1) quantise / de-quantise with
 * per-block scale selection, as hand-written HIP kernels for gfx950 (AMD Instinct MI355X).
 *
 * The operations follow "Finer is Better (with the Right Scaling)", Section 2
 * ("Experimental Setup"): Eq. 1 (power-of-two scale), Eq. 2 (abs-max scale rounded to the
 * scale format), Eq. 3 (prevent-zero clamp), Eq. 4 (4-over-6), the hierarchical-scaling
 * paragraph and the brute-force paragraph that close that section.
 *
 * Conventions common to every entry point
 *   - Every pointer named "device" is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or synchronises: work is enqueued on `stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and the call returns at once.
 *   - Tensors are row-major `rows x cols`, contiguous.  A block is `block` consecutive
 *     elements of one row; `cols % block == 0`; block is one of 2,4,8,16,32,64,128.
 *   - Every function that can fail returns an mxq_status (0 = success).  Arguments are
 *     validated on the host before anything is launched; the library never aborts, throws
 *     or prints.  Inputs are assumed finite: NaN/Inf elements give unspecified codes, never
 *     a fault.
 *   - Outputs are overwritten in full; they must not alias the input.
 *   - Calls are re-entrant; there is no global mutable state (one documented exception:
 *     mxq_tensor_absmax_static).
 */
#ifndef MXQ_H
#define MXQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MXQ_API __attribute__((visibility("default")))

typedef enum {
    MXQ_OK = 0,
    MXQ_ERR_INVALID_ARG = -1,   /* NULL pointer, bad shape, unknown enum, bad tensor_scale  */
    MXQ_ERR_UNSUPPORTED = -2,   /* well-formed request outside what the paper defines       */
    MXQ_ERR_ALIGNMENT = -3,     /* a pointer is not aligned as stated below                 */
    MXQ_ERR_HIP = -4            /* the HIP runtime reported an error at launch              */
} mxq_status;

/* Element format. E2M1 (OCP FP4): magnitudes {0, .5, 1, 1.5, 2, 3, 4, 6} (Section 2).
 * A 4-bit code is sign<<3 | magnitude index. */
typedef enum { MXQ_ELEM_E2M1 = 0 } mxq_elem_fmt;

/* Scale format: one byte per block.
 *   E8M0   power of two, value 2^(byte-127), chosen by the floor rule of Eq. 1.
 *   E4M3   OFP8 E4M3 with the sign bit unused (Background): bias 7, subnormals m*2^-9
 *          (eps = 2^-9, stated under Eq. 3), largest value 0x7E = 448, 0x7F = NaN (never
 *          written).
 *   UE5M3  unsigned, 5 exponent + 3 mantissa bits (Background; Results, "Downstream LLM Perplexity").  The paper
 *          gives no encoding; this library uses bias 15, subnormals m*2^-17, largest value
 *          0xFE = 1.75*2^16, 0xFF = NaN (never written). */
typedef enum { MXQ_SCALE_E8M0 = 0, MXQ_SCALE_E4M3 = 1, MXQ_SCALE_UE5M3 = 2 } mxq_scale_fmt;

/* Scale-selection recipe.
 *   ABSMAX     S = Round_SF(amax / 6), round to nearest even, clipped to the largest finite
 *              value (Eq. 2); for E8M0 the floor rule S = 2^floor(log2(amax/6)) (Eq. 1).
 *   ABSMAX_PZ  S = max(S_absmax, eps_SF) (Eq. 3).  No effect for E8M0.
 *   4OVER6     S_absmax(6) or S_absmax(4), whichever has the lower block SSE; M = 6 on a
 *              tie (Eq. 4).
 *   4OVER6_PZ  both candidates clamped by Eq. 3 first (Fig. 1(d) of the paper).
 *   BRUTE      every finite, strictly positive scale code is tried; the lowest code of
 *              minimal SSE is kept (brute-force paragraph, Section 2).  126 candidates for
 *              E4M3, 254 for UE5M3, the 255 powers of two 2^(byte-127), byte 0 .. 254, for E8M0.
 *   BRUTE_PRUNED  the same result as BRUTE, bit for bit, but candidates that provably cannot
 *              win are skipped: scales so large that the elements certain to quantise to zero
 *              alone cost more than the abs-max scale's whole SSE, and scales so small that the
 *              clipping error of the abs-max element alone does.  2 to 5 times faster than
 *              BRUTE.  A step toward cheaper near-optimal selection (Conclusion).
 * 4OVER6* and BRUTE_PRUNED with E8M0 return MXQ_ERR_UNSUPPORTED (Eq. 4 rounds amax / M to the
 * scale format, which the floor rule of Eq. 1 does not define). */
typedef enum {
    MXQ_RECIPE_ABSMAX = 0,
    MXQ_RECIPE_ABSMAX_PZ = 1,
    MXQ_RECIPE_4OVER6 = 2,
    MXQ_RECIPE_4OVER6_PZ = 3,
    MXQ_RECIPE_BRUTE = 4,
    MXQ_RECIPE_BRUTE_PRUNED = 5
} mxq_recipe;

typedef enum { MXQ_DT_BF16 = 0, MXQ_DT_F32 = 1 } mxq_dtype;

/*
 * mxq_quantize -- quantise one tensor (Section 2, Eq. 1-4).
 *
 * Per block: v_i = x_i / tensor_scale (IEEE fp32 division; skipped when tensor_scale == 1),
 * amax = max |v_i|, scale S by `recipe`, q_i = E2M1 value nearest to v_i / S (ties to the
 * even code, |v_i / S| > 5 gives 6; S == 0 gives magnitude 0), e_i = v_i - q_i * S,
 * SSE = sum e_i^2 in fp32 (squares rounded separately, summed by the balanced binary tree in
 * index order).  The sign bit of a code is the sign bit of x_i, also for zero magnitudes.
 *
 *   x            device, rows*cols elements of x_dtype, 16-byte aligned
 *   tensor_scale the per-tensor scale T of hierarchical scaling, finite and > 0;
 *                1.0f = no hierarchical scaling
 *   codes_out    device, rows*cols/2 bytes, 4-byte aligned; byte j = code of element 2j in
 *                bits 3:0, of element 2j+1 in bits 7:4
 *   scales_out   device, rows*cols/block bytes, 4-byte aligned, row-major
 *   sse_out      device, rows*cols/block floats, 16-byte aligned, row-major (SSE of the
 *                selected scale, in the domain of v); NULL to skip
 *   stream       hipStream_t, NULL = default stream
 *
 * rows*cols == 0 is a valid no-op.  Errors: INVALID_ARG (NULL x/codes_out/scales_out,
 * negative size, bad block, cols % block != 0, unknown enum, tensor_scale not finite or
 * <= 0), UNSUPPORTED (see mxq_recipe; rows*cols >= 2^42), ALIGNMENT, HIP.
 */
MXQ_API int mxq_quantize(const void* x, int64_t rows, int64_t cols, int block,
                 int elem_fmt, int scale_fmt, int recipe, float tensor_scale,
                 uint8_t* codes_out, uint8_t* scales_out, float* sse_out,
                 int x_dtype, void* stream);

/*
 * mxq_quantize_clip -- mxq_quantize with one more per-block output, the clipping-only part of
 * the block SSE (appendix figure "Clipping only MSE"): the sum, over the elements that saturate
 * at the largest E2M1 magnitude (|v_i / S| > 6) under the SELECTED scale, of their squared
 * residuals; elements that do not clip contribute +0; same fp32 tree as the block SSE.  Equal,
 * bit for bit, to mxq_clip_sse run afterwards on the scales this call writes, without the second
 * read of x (4 / block extra bytes per element instead of sizeof(x) + 5 / block).
 *
 *   clip_sse_out  device, rows*cols/block floats, 16-byte aligned, row-major; NULL to skip (then
 *                 the call is mxq_quantize)
 * Everything else, and all errors, as for mxq_quantize.
 */
MXQ_API int mxq_quantize_clip(const void* x, int64_t rows, int64_t cols, int block,
                      int elem_fmt, int scale_fmt, int recipe, float tensor_scale,
                      uint8_t* codes_out, uint8_t* scales_out, float* sse_out, float* clip_sse_out,
                      int x_dtype, void* stream);

/*
 * mxq_quantize_batch -- mxq_quantize (streaming recipes, no per-tensor scale) on several tensors
 * with as few launches as possible: up to 8 tensors share one grid.  Same outputs, bit for bit,
 * as one mxq_quantize call per tensor.  For the many small matrices of a model (Results,
 * "Downstream LLM Perplexity": the MLP weights of every layer), whose individual launches are
 * shorter than a launch's start-up and drain.
 *
 *   tensors  HOST array of `count` descriptors (read during the call, not kept); the pointers
 *            inside are device pointers with the alignment mxq_quantize asks for; sse_out may
 *            be NULL per tensor; tensors with rows*cols == 0 are skipped
 *   block, elem_fmt, scale_fmt, recipe, x_dtype   shared by all tensors
 * Every tensor is validated before anything is launched.  Errors as for mxq_quantize, plus
 * UNSUPPORTED for BRUTE / BRUTE_PRUNED (a search launch is never short) and for more than 2^40
 * elements in one call.
 */
typedef struct mxq_tensor {
    const void* x;          /* device, rows*cols elements, 16-byte aligned            */
    int64_t rows, cols;
    uint8_t* codes_out;     /* device, rows*cols/2 bytes, 4-byte aligned               */
    uint8_t* scales_out;    /* device, rows*cols/block bytes, 4-byte aligned           */
    float* sse_out;         /* device, rows*cols/block floats, 16-byte aligned, or NULL */
} mxq_tensor;
MXQ_API int mxq_quantize_batch(const mxq_tensor* tensors, int count, int block,
                       int elem_fmt, int scale_fmt, int recipe, int x_dtype, void* stream);

/*
 * mxq_quantize_hier -- hierarchical scaling without a round trip to the host (the two-stage
 * process of Section 2 as a dynamic activation tensor needs it): mxq_quantize with the
 * per-tensor scale derived on the device from the tensor abs-max that mxq_tensor_absmax left
 * in device memory,
 *     T = mxq_tensor_scale_from_absmax(*absmax, elem_fmt, scale_fmt)      (the same bits),
 * so that "abs-max, then quantise" is two launches on one stream with nothing in between, and
 * a captured graph of the pair follows the data from replay to replay.
 *
 *   absmax            device, 1 float, 4-byte aligned; read when the kernel runs
 *   tensor_scale_out  device, 1 float, 4-byte aligned, receives T (de-quantisation needs it);
 *                     NULL to skip
 * Everything else as for mxq_quantize.  rows*cols == 0 is a no-op that leaves
 * tensor_scale_out untouched.  Errors as for mxq_quantize, plus INVALID_ARG for a NULL absmax.
 */
MXQ_API int mxq_quantize_hier(const void* x, int64_t rows, int64_t cols, int block,
                      int elem_fmt, int scale_fmt, int recipe,
                      const float* absmax, float* tensor_scale_out,
                      uint8_t* codes_out, uint8_t* scales_out, float* sse_out,
                      int x_dtype, void* stream);

/*
 * mxq_dequantize -- x^_i = (q_i * S) * tensor_scale, rounded to nearest even into out_dtype
 * (de-quantisation, Section 2, paragraph after Eq. 2).
 *
 *   codes, scales  device, layouts as written by mxq_quantize, 4-byte aligned
 *   x_out          device, rows*cols elements of out_dtype, 16-byte aligned
 * A scale byte that is not a finite value of scale_fmt de-quantises to NaN.
 */
MXQ_API int mxq_dequantize(const uint8_t* codes, const uint8_t* scales,
                   int64_t rows, int64_t cols, int block,
                   int elem_fmt, int scale_fmt, float tensor_scale,
                   void* x_out, int out_dtype, void* stream);

/*
 * mxq_dequantize_hier -- mxq_dequantize with the per-tensor scale read from device memory (the
 * word mxq_quantize_hier wrote to tensor_scale_out) when the kernel runs.
 *   tensor_scale   device, 1 float, 4-byte aligned
 * Errors as for mxq_dequantize, plus INVALID_ARG for a NULL tensor_scale.
 */
MXQ_API int mxq_dequantize_hier(const uint8_t* codes, const uint8_t* scales,
                        int64_t rows, int64_t cols, int block,
                        int elem_fmt, int scale_fmt, const float* tensor_scale,
                        void* x_out, int out_dtype, void* stream);

/*
 * mxq_tensor_absmax -- first stage of hierarchical scaling (Section 2): max |x_i| over the
 * whole tensor, written as one float to absmax_out (device, 4-byte aligned).  x 16-byte
 * aligned.  An empty tensor writes 0.
 */
MXQ_API int mxq_tensor_absmax(const void* x, int64_t rows, int64_t cols, int x_dtype,
                      float* absmax_out, void* stream);

/*
 * mxq_tensor_absmax_acc -- the reduction as a running maximum, in ONE launch and with the
 * shortest tail: *absmax_inout = max(*absmax_inout, max |x_i|).  For the dynamic-activation use of
 * hierarchical scaling (Section 2), where the pre-pass is on the critical path, and for a tensor
 * that arrives in several pieces (row shards: call once per piece on the same word).
 *
 *   absmax_inout  device, 1 float, 4-byte aligned.  Must hold +0 (or the non-negative maximum to
 *                 be continued) when the kernel runs; nothing clears it here.
 *   clear_word    device, 1 float, 4-byte aligned, or NULL.  Set to +0 by this call, to be the
 *                 absmax_inout of a LATER call on the same stream: a caller that alternates
 *                 between two words (this call's result in one, the next call's in the other)
 *                 never needs a separate clear.  Must differ from absmax_inout.
 * An empty tensor leaves absmax_inout untouched (and still clears clear_word).
 * Errors as for mxq_tensor_absmax, plus INVALID_ARG when clear_word == absmax_inout.
 */
MXQ_API int mxq_tensor_absmax_acc(const void* x, int64_t rows, int64_t cols, int x_dtype,
                          float* absmax_inout, float* clear_word, void* stream);

/*
 * mxq_tensor_absmax_ws -- mxq_tensor_absmax in ONE launch (that one needs a second, tiny launch
 * that clears the output word first) and without a precondition on the output word (unlike
 * mxq_tensor_absmax_acc): the workgroups meet in a caller-owned workspace, and the one that
 * arrives last writes the output.  One graph node instead of two; the tail of the kernel is
 * longer than that of the other two forms (three dependent device-scope atomics), so on large
 * tensors it is the slowest of the three (first stage of hierarchical scaling, Section 2).
 *
 *   workspace        device, at least mxq_tensor_absmax_workspace_size() bytes, 8-byte aligned.
 *                    It must hold zeros before its first use (one hipMemset when it is allocated);
 *                    every call leaves it zeroed again, so it can be reused from call to call.
 *   workspace_bytes  size of the buffer behind `workspace`
 * Calls that share one workspace must not overlap in time (give each concurrent stream its own).
 * Errors as for mxq_tensor_absmax, plus INVALID_ARG for a NULL or too small workspace and
 * ALIGNMENT for a misaligned one.
 */
#define MXQ_ABSMAX_WORKSPACE_BYTES 256
MXQ_API size_t mxq_tensor_absmax_workspace_size(void);
MXQ_API int mxq_tensor_absmax_ws(const void* x, int64_t rows, int64_t cols, int x_dtype,
                         float* absmax_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * mxq_tensor_absmax_static -- mxq_tensor_absmax_ws for callers that can neither allocate device
 * memory nor carry a workspace around: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernels, same result; the two-word workspace is a
 * 256-byte array inside the library's own device image (one copy per GPU, held until the process
 * ends).  The call allocates and frees nothing.
 *
 *   - rows*cols may not exceed MXQ_ABSMAX_STATIC_MAX_ELEMENTS (2^40): MXQ_ERR_UNSUPPORTED beyond.
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two host threads) race and may both return wrong maxima; calls on one stream, or
 *     otherwise ordered, are safe.  Each call returns the array to zero, which is the state the
 *     next call needs.  This is the library's only global state.
 *   - The device must be current.  The first call on each device looks the array's address up
 *     (hipGetSymbolAddress); make that call outside graph capture.
 * Other arguments and errors as for mxq_tensor_absmax; MXQ_ERR_HIP also when the address
 * look-up fails.
 */
#define MXQ_ABSMAX_STATIC_MAX_ELEMENTS ((int64_t)1 << 40)
MXQ_API int mxq_tensor_absmax_static(const void* x, int64_t rows, int64_t cols, int x_dtype,
                             float* absmax_out, void* stream);

/*
 * mxq_clip_sse -- diagnostic of the paper's appendix ("Clipping only MSE"): for every block,
 * the part of the squared error that comes from elements saturating at the largest E2M1
 * magnitude: sum over the elements with |v_i / S| > 6 of (v_i - sign(v_i) * 6 * S)^2, with
 * v_i = x_i / tensor_scale and S the block's scale byte; elements that do not clip contribute
 * +0; same fp32 tree as the block SSE.  Works on the scales written by any recipe.
 *
 *   x               device, as for mxq_quantize
 *   scales          device, rows*cols/block bytes, 4-byte aligned
 *   clip_sse_out    device, rows*cols/block floats, 16-byte aligned
 */
MXQ_API int mxq_clip_sse(const void* x, const uint8_t* scales, int64_t rows, int64_t cols, int block,
                         int elem_fmt, int scale_fmt, float tensor_scale, float* clip_sse_out,
                         int x_dtype, void* stream);

/*
 * mxq_histogram -- diagnostic of the paper's appendix (entry and scale histograms): counts of
 * the 8 E2M1 magnitude indices over all elements and of the 256 scale bytes over all blocks.
 *
 *   codes, scales   device, layouts as written by mxq_quantize, 4-byte aligned
 *   elem_hist       device, 8 x uint64, 8-byte aligned, overwritten
 *   scale_hist      device, 256 x uint64, 8-byte aligned, overwritten
 */
MXQ_API int mxq_histogram(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                          int block, int elem_fmt, uint64_t* elem_hist, uint64_t* scale_hist,
                          void* stream);

/* Host helper: the per-tensor scale that maps the tensor abs-max onto (largest element
 * value) x (largest scale value): absmax / (6 * SF_max), e.g. absmax / 2688 for E4M3; 1 for
 * an all-zero tensor or a format whose range makes the quotient vanish.  NaN on a bad enum. */
MXQ_API float mxq_tensor_scale_from_absmax(float absmax, int elem_fmt, int scale_fmt);

/* Host helper: value of a scale byte; NaN for a code that is not a finite number. */
MXQ_API float mxq_scale_decode(int scale_fmt, uint8_t code);

/* Host helper: number of candidates BRUTE tries (finite positive codes): 126 for E4M3,
 * 254 for UE5M3, 255 for E8M0; -1 on a bad enum. */
MXQ_API int mxq_num_candidates(int scale_fmt);

/* Host helper: static, human-readable name of a status code. */
MXQ_API const char* mxq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MXQ_H */
