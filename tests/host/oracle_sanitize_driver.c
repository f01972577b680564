/*
 * The CPU oracle under AddressSanitizer / UndefinedBehaviorSanitizer.
 *
 * Includes oracle/mxq_oracle.c itself (no second copy of anything), reads a case file written by
 * tests/test_sanitizers.py and runs every case through orc_quantize, orc_dequantize, orc_clip_sse
 * and orc_tensor_absmax on exactly sized heap buffers, so that any access one element past an
 * input or output is an ASan report.  Each result is compared byte for byte with what the file
 * expects (the hand-derived worked blocks of tests/golden/, and outputs of the ordinary,
 * unsanitised oracle build for the rest).
 *
 * Case record (little endian): int32 dtype, rows, cols, block, fmt, recipe; float T;
 *   x (rows*cols elements), codes (rows*cols/2), scales (nb), sse (nb floats).
 * Exit status 0 iff every case matches and no sanitizer fired.
 * Build: gcc -O1 -g -std=c11 -ffp-contract=off -fopenmp -fsanitize=address,undefined
 *        -fno-sanitize-recover=all -static-libasan
 */
#include <stdio.h>

#include "../../oracle/mxq_oracle.c"

static void* exact_alloc(size_t n) { void* p = malloc(n ? n : 1); if (!p) { perror("malloc"); exit(2); } return p; }

static int read_exact(FILE* f, void* p, size_t n) { return fread(p, 1, n, f) == n; }

int main(int argc, char** argv)
{
    if (argc < 2) { fprintf(stderr, "usage: %s cases.bin\n", argv[0]); return 2; }
    FILE* f = fopen(argv[1], "rb");
    if (!f) { perror(argv[1]); return 2; }
    int32_t n_cases = 0;
    if (!read_exact(f, &n_cases, 4)) return 2;
    int bad = 0;
    for (int c = 0; c < n_cases; ++c) {
        int32_t h[6];
        float T;
        if (!read_exact(f, h, sizeof h) || !read_exact(f, &T, 4)) return 2;
        const int dtype = h[0], block = h[3], fmt = h[4], recipe = h[5];
        const int64_t rows = h[1], cols = h[2], n = rows * cols, nb = n / block;
        const size_t xb = (size_t)n * (dtype == ORC_DT_BF16 ? 2 : 4);
        void* x = exact_alloc(xb);
        uint8_t* want_codes = exact_alloc((size_t)n / 2);
        uint8_t* want_scales = exact_alloc((size_t)nb);
        float* want_sse = exact_alloc((size_t)nb * 4);
        if (!read_exact(f, x, xb) || !read_exact(f, want_codes, (size_t)n / 2) ||
            !read_exact(f, want_scales, (size_t)nb) || !read_exact(f, want_sse, (size_t)nb * 4)) return 2;

        uint8_t* codes = exact_alloc((size_t)n / 2);
        uint8_t* scales = exact_alloc((size_t)nb);
        float* sse = exact_alloc((size_t)nb * 4);
        double* ex = exact_alloc((size_t)nb * 8);
        int rc = orc_quantize(x, dtype, rows, cols, block, fmt, recipe, T, ORC_SEL_PINNED, codes, scales, sse, ex);
        int ok = rc == 0 && !memcmp(codes, want_codes, (size_t)n / 2) && !memcmp(scales, want_scales, (size_t)nb) &&
                 !memcmp(sse, want_sse, (size_t)nb * 4);
        /* the other entry points on the same buffers: results are checked for self-consistency */
        float* deq = exact_alloc((size_t)n * 4);
        uint16_t* deq16 = exact_alloc((size_t)n * 2);
        float* clip = exact_alloc((size_t)nb * 4);
        ok = ok && orc_dequantize(codes, scales, rows, cols, block, fmt, T, deq, ORC_DT_F32) == 0;
        ok = ok && orc_dequantize(codes, scales, rows, cols, block, fmt, T, deq16, ORC_DT_BF16) == 0;
        ok = ok && orc_clip_sse(x, dtype, rows, cols, block, fmt, T, scales, clip) == 0;
        for (int64_t b = 0; ok && b < nb; ++b) ok = clip[b] <= sse[b];          /* a part of the block SSE */
        const float amax = orc_tensor_absmax(x, dtype, n);
        ok = ok && amax >= 0.0f;
        /* the exact-selection mode walks the same buffers */
        ok = ok && orc_quantize(x, dtype, rows, cols, block, fmt, recipe, T, ORC_SEL_EXACT, codes, scales, sse, NULL) == 0;
        if (!ok) { ++bad; printf("case %d MISMATCH (dtype %d %lldx%lld b=%d fmt=%d recipe=%d T=%g rc=%d)\n", c, dtype,
                                 (long long)rows, (long long)cols, block, fmt, recipe, (double)T, rc); }
        free(x); free(want_codes); free(want_scales); free(want_sse); free(codes); free(scales); free(sse); free(ex);
        free(deq); free(deq16); free(clip);
    }
    fclose(f);
    /* argument errors must be refusals, not accesses */
    uint8_t one[8] = {0};
    float fone[2] = {0};
    bad += orc_quantize(NULL, 0, 1, 2, 2, 1, 0, 1.0f, 0, one, one, fone, NULL) != -1;
    bad += orc_quantize(one, 0, 1, 2, 3, 1, 0, 1.0f, 0, one, one, fone, NULL) != -1;
    bad += orc_quantize(one, 0, 1, 6, 4, 1, 0, 1.0f, 0, one, one, fone, NULL) != -1;
    bad += orc_quantize(one, 0, 1, 2, 2, 0, 2, 1.0f, 0, one, one, fone, NULL) != -1;
    bad += orc_quantize(one, 0, 1, 2, 2, 1, 0, 0.0f, 0, one, one, fone, NULL) != -1;
    bad += orc_quantize(one, 7, 1, 2, 2, 1, 0, 1.0f, 0, one, one, fone, NULL) != -1;
    printf("oracle_sanitize cases=%d bad=%d\n", (int)n_cases, bad);
    return bad ? 1 : 0;
}
