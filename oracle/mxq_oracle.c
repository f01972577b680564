/*
 * mxq_oracle.c -- plain CPU oracle for block-wise microscaled FP4 quantisation with
 * per-block scale selection ("Finer is Better (with the Right Scaling)").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU library can be
 * checked element by element against something that can be compared with the paper by eye.
 * It shares no code, table, header or constant generator with the HIP library, is never
 * called from the product path, and is only used by the tests, by the smoke check and by the
 * benchmark's "cpu_baseline" leg.  It is deliberately slow: every rounding is a
 * nearest-value search over the whole value set of the target format, every recipe is the
 * definition written out, there is no blocking, fusion or reordering.  OpenMP over blocks is
 * the only concession to run time and does not change any result.
 *
 * What is computed, per block V = (v_0 .. v_{b-1}) of b consecutive row elements
 * (Section 2 "Experimental Setup" of the paper unless another place is named):
 *
 *   step 0  hierarchical adjust: v_i <- fl32(v_i / T) when a per-tensor scale T != 1 is given
 *           (hierarchical scaling paragraph).
 *   step 1  amax = max_i |v_i|                                             (Eq. 1, Eq. 2)
 *   step 2  scale candidates
 *             power-of-two (E8M0): S = 2^floor(log2(amax / M))              (Eq. 1)
 *             E4M3 / UE5M3:        S = Round_SF(fl32(amax / M)), round to nearest even,
 *                                  clipped to the largest finite value      (Eq. 2)
 *             prevent-zero:        S <- max(S, eps_SF)                      (Eq. 3)
 *             4-over-6:            M in {6, 4}                              (Eq. 4)
 *             brute force:         every finite, strictly positive scale code
 *                                  (brute-force paragraph at the end of Section 2)
 *   step 3  q_i = quant(fl32(v_i / S)): nearest value of the E2M1 set
 *           {0, .5, 1, 1.5, 2, 3, 4, 6}, ties to the code with even mantissa, magnitudes
 *           above 6 clip to 6; S == 0 sets every magnitude to zero.  The sign bit of the
 *           code is the sign bit of the input.
 *   step 4  e_i = fl32(v_i - q_i * S);  SSE = sum e_i^2   ("MSE(v, S)" under Eq. 4)
 *   step 5  selection: 4-over-6 keeps M = 6 unless SSE_4 < SSE_6 strictly; brute force keeps
 *           the lowest code among those of minimal SSE.
 *   step 6  outputs: one scale byte per block, two 4-bit codes per byte (element 2j in the
 *           low nibble), one fp32 SSE per block.
 *
 * Arithmetic of the SSE used for selection and reported ("pinned" mode, ORC_SEL_PINNED):
 * fp32, s_i = fl32(e_i * e_i) (no fused multiply-add), summed by the balanced binary tree in
 * index order: sum(lo,hi) = fl32(sum(lo,mid) + sum(mid,hi)), mid = (lo+hi)/2.  The paper
 * states MSE in real arithmetic; the tree is this build's reading, chosen so that the
 * result does not depend on how a kernel spreads a block over lanes.  ORC_SEL_EXACT selects
 * with the SSE accumulated in long double instead; it is used by tests only, to show that
 * the pinned selection differs from the exact one only on near ties.
 *
 * Besides the path itself the file holds the appendix diagnostic orc_clip_sse (the histograms
 * are numpy bincounts in the Python wrapper).
 *
 * Parity pins (tests/, CPU only): the E2M1 value set the paper prints; eps_E4M3 = 2^-9; the
 * closed form of Eq. 1; a library float8 cast for the E4M3 table and its rounding; worked
 * blocks under tests/golden/; exhaustive enumeration on tiny blocks in exact rational
 * arithmetic; the chain SSE_absmax >= SSE_4over6 >= SSE_brute; nesting of brute-force SSE.
 * Parity unpinned (the paper does not define them; fixed by this build's written reading
 * only): the UE5M3 bias / special codes, the sign bit of zero codes, the nibble order, the
 * tie-breaks of step 5.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -fPIC -shared (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_DT_BF16 = 0, ORC_DT_F32 = 1 };
enum { ORC_SCALE_E8M0 = 0, ORC_SCALE_E4M3 = 1, ORC_SCALE_UE5M3 = 2 };
enum { ORC_ABSMAX = 0, ORC_ABSMAX_PZ = 1, ORC_4OVER6 = 2, ORC_4OVER6_PZ = 3, ORC_BRUTE = 4 };
enum { ORC_SEL_PINNED = 0, ORC_SEL_EXACT = 1 };

/* ------------------------------------------------------------------------------------ */
/* Formats                                                                              */
/* ------------------------------------------------------------------------------------ */

/* The FP4 (OCP E2M1) magnitudes, as the paper lists them in Section 2. Index = 3-bit
 * magnitude code (2 exponent bits, 1 mantissa bit, bias 1). */
static const float E2M1_SET[8] = { 0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f };

float orc_e2m1_decode(int code)
{
    float m = E2M1_SET[code & 7];
    return (code & 8) ? -m : m;
}

/* Value of a scale byte, NaN for codes that are not finite numbers.
 *   E8M0  : 2^(code-127), 255 = NaN                  (MX v1.0 power-of-two scale, Background)
 *   E4M3  : OFP8 E4M3 with the sign bit unused: bias 7, subnormals m*2^-9, 0x7F = NaN,
 *           largest 0x7E = 448; smallest nonzero 2^-9 as the paper states under Eq. 3.
 *   UE5M3 : 5 exponent + 3 mantissa bits, bias 15, subnormals m*2^-17, 0xFF = NaN,
 *           largest 0xFE = 1.75*2^16 (this build's reading; the paper gives no encoding). */
float orc_scale_decode(int fmt, int code)
{
    if (code < 0 || code > 255) return NAN;
    if (fmt == ORC_SCALE_E8M0) {
        if (code == 255) return NAN;
        return ldexpf(1.0f, code - 127);
    }
    if (fmt == ORC_SCALE_E4M3) {
        if (code >= 0x7F) return NAN;              /* 0x7F NaN; bit 7 is the unused sign */
        int e = code >> 3, m = code & 7;
        if (e == 0) return ldexpf((float)m, -9);
        return ldexpf(1.0f + (float)m / 8.0f, e - 7);
    }
    if (fmt == ORC_SCALE_UE5M3) {
        if (code == 0xFF) return NAN;
        int e = code >> 3, m = code & 7;
        if (e == 0) return ldexpf((float)m, -17);
        return ldexpf(1.0f + (float)m / 8.0f, e - 15);
    }
    return NAN;
}

/* Largest finite code of a scale format. */
int orc_scale_max_code(int fmt)
{
    if (fmt == ORC_SCALE_E8M0) return 254;
    if (fmt == ORC_SCALE_E4M3) return 0x7E;
    if (fmt == ORC_SCALE_UE5M3) return 0xFE;
    return -1;
}

/* Number of finite, strictly positive codes = the brute-force candidate set. */
int orc_num_candidates(int fmt)
{
    int n = 0;
    for (int c = 0; c <= orc_scale_max_code(fmt); ++c)
        if (orc_scale_decode(fmt, c) > 0.0f) ++n;
    return n;
}

/* eps_SF of Eq. 3: smallest nonzero value of the scale format. */
float orc_scale_eps(int fmt)
{
    float best = INFINITY;
    for (int c = 0; c <= orc_scale_max_code(fmt); ++c) {
        float s = orc_scale_decode(fmt, c);
        if (s > 0.0f && s < best) best = s;
    }
    return best;
}

/* Round_SF of Eq. 2 for the 8-bit floating-point scale formats: the finite code whose value
 * is nearest to r; a tie goes to the even code; anything beyond the largest value clips to
 * it.  Written as the definition: a search over every finite code.  Differences are taken
 * in long double, where they are exact for r inside the format's range. */
int orc_round_sf(int fmt, float r)
{
    int top = orc_scale_max_code(fmt);
    if (r >= orc_scale_decode(fmt, top)) return top;        /* clipping, stated separately */
    int best = 0;
    long double best_d = INFINITY;
    for (int c = 0; c <= orc_scale_max_code(fmt); ++c) {
        long double d = fabsl((long double)r - (long double)orc_scale_decode(fmt, c));
        if (d < best_d || (d == best_d && (c % 2 == 0) && (best % 2 != 0))) {
            best_d = d;
            best = c;
        }
    }
    return best;
}

/* Eq. 1: the power-of-two scale 2^k with k = floor(log2(amax / M)), i.e. the largest k with
 * M * 2^k <= amax, stored as the E8M0 byte k + 127 clamped to [0, 254].  amax == 0 has no
 * such k; it takes the smallest code. */
int orc_pow2_code(float amax, float M)
{
    if (!(amax > 0.0f)) return 0;
    int k = -200;
    for (int t = 200; t >= -200; --t) {
        if (ldexp((double)M, t) <= (double)amax) { k = t; break; }
    }
    int code = k + 127;
    if (code < 0) code = 0;
    if (code > 254) code = 254;
    return code;
}

/* quant() of Section 2: 3-bit magnitude code of the E2M1 value nearest to |y|; ties to the
 * even code (mantissa bit 0); |y| at or beyond the largest value 6 clips to 6 (stated
 * separately so that huge or infinite quotients do not depend on cancellation). */
int orc_e2m1_round_mag(float y)
{
    double ay = fabs((double)y);
    if (ay >= (double)E2M1_SET[7]) return 7;
    int best = 0;
    double best_d = INFINITY;
    for (int c = 0; c < 8; ++c) {
        double d = fabs(ay - (double)E2M1_SET[c]);
        if (d < best_d || (d == best_d && (c % 2 == 0) && (best % 2 != 0))) {
            best_d = d;
            best = c;
        }
    }
    return best;
}

/* ------------------------------------------------------------------------------------ */
/* One block                                                                            */
/* ------------------------------------------------------------------------------------ */

static float load_elem(const void* x, int dt, int64_t i)
{
    if (dt == ORC_DT_F32) return ((const float*)x)[i];
    uint32_t bits = (uint32_t)((const uint16_t*)x)[i] << 16;   /* bf16 widens exactly */
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* Balanced binary tree in index order over the fp32 squares. */
static float tree_sum(const float* s, int lo, int hi)
{
    if (hi - lo == 1) return s[lo];
    int mid = (lo + hi) / 2;
    float a = tree_sum(s, lo, mid);
    float b = tree_sum(s, mid, hi);
    return a + b;
}

/* Steps 3 and 4 for one scale S: 4-bit codes, pinned fp32 SSE, exact SSE. */
static void quant_under_scale(const float* v, int b, float S, uint8_t* code4,
                              float* sse_pinned, long double* sse_exact)
{
    float sq[128];
    long double ex = 0.0L;
    for (int i = 0; i < b; ++i) {
        int mag = 0;
        if (S != 0.0f) {
            float y = v[i] / S;                      /* IEEE round-to-nearest-even divide */
            mag = orc_e2m1_round_mag(y);
        }
        int sign = signbit(v[i]) ? 1 : 0;
        code4[i] = (uint8_t)((sign << 3) | mag);
        float q = sign ? -E2M1_SET[mag] : E2M1_SET[mag];
        float qS = q * S;                            /* exact: at most 6 significant bits */
        float e = v[i] - qS;
        sq[i] = e * e;
        long double ee = (long double)v[i] - (long double)q * (long double)S;
        ex += ee * ee;
    }
    *sse_pinned = tree_sum(sq, 0, b);
    *sse_exact = ex;
}

/* Eq. 2 (+ Eq. 3 when pz) for the floating-point scale formats, Eq. 1 for E8M0. */
static int absmax_scale_code(int fmt, float amax, float M, int pz)
{
    if (fmt == ORC_SCALE_E8M0) return orc_pow2_code(amax, M);
    float r = amax / M;
    int code = orc_round_sf(fmt, r);
    if (pz && orc_scale_decode(fmt, code) < orc_scale_eps(fmt)) {
        /* max(S, eps): the only value below eps is 0; eps is code 1 in both formats */
        for (int c = 0; c <= orc_scale_max_code(fmt); ++c)
            if (orc_scale_decode(fmt, c) == orc_scale_eps(fmt)) { code = c; break; }
    }
    return code;
}

static int less_sel(int mode, float a_p, long double a_e, float b_p, long double b_e)
{
    return (mode == ORC_SEL_EXACT) ? (a_e < b_e) : (a_p < b_p);
}

static void quantize_block(const float* v, int b, int fmt, int recipe, int mode,
                           uint8_t* code4_out, uint8_t* scale_out, float* sse_out,
                           double* sse_exact_out)
{
    float amax = 0.0f;
    for (int i = 0; i < b; ++i) {
        float a = fabsf(v[i]);
        if (a > amax) amax = a;
    }

    uint8_t best_codes[128], cand_codes[128];
    int best_code = -1;
    float best_p = 0.0f, cand_p;
    long double best_e = 0.0L, cand_e;

    if (recipe == ORC_ABSMAX || recipe == ORC_ABSMAX_PZ) {
        best_code = absmax_scale_code(fmt, amax, 6.0f, recipe == ORC_ABSMAX_PZ);
        quant_under_scale(v, b, orc_scale_decode(fmt, best_code), best_codes, &best_p, &best_e);
    } else if (recipe == ORC_4OVER6 || recipe == ORC_4OVER6_PZ) {
        int pz = (recipe == ORC_4OVER6_PZ);
        int c6 = absmax_scale_code(fmt, amax, 6.0f, pz);
        int c4 = absmax_scale_code(fmt, amax, 4.0f, pz);
        quant_under_scale(v, b, orc_scale_decode(fmt, c6), best_codes, &best_p, &best_e);
        best_code = c6;
        quant_under_scale(v, b, orc_scale_decode(fmt, c4), cand_codes, &cand_p, &cand_e);
        if (less_sel(mode, cand_p, cand_e, best_p, best_e)) {      /* M = 4 only if strictly lower */
            best_code = c4; best_p = cand_p; best_e = cand_e;
            memcpy(best_codes, cand_codes, (size_t)b);
        }
    } else { /* ORC_BRUTE */
        for (int c = 0; c <= orc_scale_max_code(fmt); ++c) {
            float S = orc_scale_decode(fmt, c);
            if (!(S > 0.0f)) continue;                              /* finite and positive only */
            quant_under_scale(v, b, S, cand_codes, &cand_p, &cand_e);
            if (best_code < 0 || less_sel(mode, cand_p, cand_e, best_p, best_e)) {
                best_code = c; best_p = cand_p; best_e = cand_e;   /* ascending: ties keep lowest */
                memcpy(best_codes, cand_codes, (size_t)b);
            }
        }
    }
    memcpy(code4_out, best_codes, (size_t)b);
    *scale_out = (uint8_t)best_code;
    *sse_out = best_p;
    if (sse_exact_out) *sse_exact_out = (double)best_e;
}

/* ------------------------------------------------------------------------------------ */
/* Whole tensors (host pointers)                                                        */
/* ------------------------------------------------------------------------------------ */

static int valid_block(int b)
{
    return b == 2 || b == 4 || b == 8 || b == 16 || b == 32 || b == 64 || b == 128;
}

/* Quantise a row-major rows x cols tensor; blocks are `block` consecutive elements of a row.
 *   codes      rows*cols/2 bytes, element 2j in bits 3:0 and 2j+1 in bits 7:4 of byte j
 *   scales     rows*cols/block bytes, row-major
 *   sse        rows*cols/block floats (pinned fp32 SSE of the selected scale), may be NULL
 *   sse_exact  rows*cols/block doubles (same candidate, long-double accumulation), may be NULL
 * Returns 0, or -1 on an argument the method does not define. */
int orc_quantize(const void* x, int x_dtype, int64_t rows, int64_t cols, int block,
                 int scale_fmt, int recipe, float tensor_scale, int sel_mode,
                 uint8_t* codes, uint8_t* scales, float* sse, double* sse_exact)
{
    if (!x || !codes || !scales) return -1;
    if (rows < 0 || cols < 0 || !valid_block(block) || cols % block != 0) return -1;
    if (x_dtype != ORC_DT_BF16 && x_dtype != ORC_DT_F32) return -1;
    if (scale_fmt < 0 || scale_fmt > 2 || recipe < 0 || recipe > 4) return -1;
    /* Eq. 4 chooses between two roundings of amax / M, which the floor rule of Eq. 1 does not
     * define; the brute-force search over the values of the scale format applies to the power-of-two
     * format as it stands: all 255 bytes 0x00 .. 0xFE are finite positive values. */
    if (scale_fmt == ORC_SCALE_E8M0 && (recipe == ORC_4OVER6 || recipe == ORC_4OVER6_PZ)) return -1;
    if (!(tensor_scale > 0.0f) || isinf(tensor_scale)) return -1;

    int64_t nb = rows * cols / block;
#pragma omp parallel for schedule(static)
    for (int64_t blk = 0; blk < nb; ++blk) {
        float v[128];
        uint8_t c4[128];
        for (int i = 0; i < block; ++i) {
            float f = load_elem(x, x_dtype, blk * block + i);
            if (tensor_scale != 1.0f) f = f / tensor_scale;       /* step 0 */
            v[i] = f;
        }
        uint8_t sc;
        float sp;
        double se;
        quantize_block(v, block, scale_fmt, recipe, sel_mode, c4, &sc, &sp, &se);
        for (int i = 0; i < block; i += 2)
            codes[(blk * block + i) / 2] = (uint8_t)(c4[i] | (c4[i + 1] << 4));
        scales[blk] = sc;
        if (sse) sse[blk] = sp;
        if (sse_exact) sse_exact[blk] = se;
    }
    return 0;
}

/* Pinned and exact SSE of one block under one given scale code (tests use it to probe
 * individual candidates). v holds `block` fp32 values already adjusted by T. */
int orc_block_sse(const float* v, int block, int scale_fmt, int code,
                  uint8_t* code4_out, float* sse_pinned, double* sse_exact)
{
    if (!valid_block(block)) return -1;
    float S = orc_scale_decode(scale_fmt, code);
    if (isnan(S)) return -1;
    uint8_t c4[128];
    float sp;
    long double se;
    quant_under_scale(v, block, S, c4, &sp, &se);
    if (code4_out) memcpy(code4_out, c4, (size_t)block);
    if (sse_pinned) *sse_pinned = sp;
    if (sse_exact) *sse_exact = (double)se;
    return 0;
}

/* Clipping-only part of the block SSE (appendix figure "Clipping only MSE"): the squared
 * error of the elements whose quotient v_i / S lies beyond the largest E2M1 magnitude 6, i.e.
 * that saturate; every other element contributes +0.  Same fp32 tree as the block SSE.  The
 * paper shows this quantity only as a figure; taking "the clipping portion" of the MSE to be
 * the error of the saturating elements is this build's reading.  scales holds one byte per
 * block, as written by orc_quantize. */
int orc_clip_sse(const void* x, int x_dtype, int64_t rows, int64_t cols, int block, int scale_fmt,
                 float tensor_scale, const uint8_t* scales, float* clip_sse)
{
    if (!x || !scales || !clip_sse) return -1;
    if (rows < 0 || cols < 0 || !valid_block(block) || cols % block != 0) return -1;
    int64_t nb = rows * cols / block;
#pragma omp parallel for schedule(static)
    for (int64_t blk = 0; blk < nb; ++blk) {
        float sq[128];
        float S = orc_scale_decode(scale_fmt, scales[blk]);
        for (int i = 0; i < block; ++i) {
            float v = load_elem(x, x_dtype, blk * block + i);
            if (tensor_scale != 1.0f) v = v / tensor_scale;
            sq[i] = 0.0f;
            if (S > 0.0f) {
                float y = v / S;
                if (fabsf(y) > E2M1_SET[7]) {
                    float q = signbit(v) ? -E2M1_SET[7] : E2M1_SET[7];
                    float e = v - q * S;
                    sq[i] = e * e;
                }
            }
        }
        clip_sse[blk] = tree_sum(sq, 0, block);
    }
    return 0;
}

static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);   /* NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* De-quantisation: x^_i = fl32(fl32(q_i * S) * T), rounded to nearest even into the output
 * type (de-quantisation, Section 2, paragraph after Eq. 2). */
int orc_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                   int block, int scale_fmt, float tensor_scale, void* x_out, int out_dtype)
{
    if (!codes || !scales || !x_out) return -1;
    if (rows < 0 || cols < 0 || !valid_block(block) || cols % block != 0) return -1;
    if (out_dtype != ORC_DT_BF16 && out_dtype != ORC_DT_F32) return -1;
    int64_t n = rows * cols;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int c = (codes[i / 2] >> ((i & 1) * 4)) & 0xF;
        float S = orc_scale_decode(scale_fmt, scales[i / block]);
        float qS = orc_e2m1_decode(c) * S;
        float r = qS * tensor_scale;
        if (out_dtype == ORC_DT_F32) ((float*)x_out)[i] = r;
        else ((uint16_t*)x_out)[i] = f32_to_bf16_rne(r);
    }
    return 0;
}

/* First stage of hierarchical scaling: abs-max across the entire tensor. */
float orc_tensor_absmax(const void* x, int x_dtype, int64_t n)
{
    float a = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float f = fabsf(load_elem(x, x_dtype, i));
        if (f > a) a = f;
    }
    return a;
}

/* Per-tensor scale that maps the tensor abs-max onto (largest element value) x (largest
 * scale value): T = A / (6 * SF_max); an all-zero tensor takes T = 1. */
float orc_tensor_scale(float absmax, int scale_fmt)
{
    if (!(absmax > 0.0f)) return 1.0f;
    float denom = 6.0f * orc_scale_decode(scale_fmt, orc_scale_max_code(scale_fmt));
    float T = absmax / denom;
    return (T > 0.0f) ? T : 1.0f;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
