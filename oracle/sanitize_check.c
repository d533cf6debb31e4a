/*
 * Sanitizer driver of the CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * Compiled together with mx_oracle.c under -fsanitize=address,undefined (tests/test_oracle_sanitized.py), it calls
 * every routine of the oracle on heap buffers of exactly the documented sizes, over ragged shapes, every width,
 * narrow exponents, subnormals, zero blocks and the largest finite values, so that an access outside a buffer, a
 * shift by too much or a signed overflow anywhere in the oracle ends the run with a report.  It checks no values
 * (the pins do that); it returns 0 when every call returned its expected status.
 */
#include "mx_oracle.c"

#include <stdio.h>
#include <stdlib.h>

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }

static float draw(int kind) {
    const float u = (float)(rnd() & 0xFFFF) / 65536.0f - 0.5f;
    switch (kind % 5) {
        case 0: return u;
        case 1: return ldexpf(u, (int)(rnd() % 200) - 100);
        case 2: return (rnd() & 3) ? 0.0f : u;
        case 3: return ldexpf(u, -140);                          /* subnormals */
        default: return (rnd() & 1) ? 3.0e38f : -3.0e38f * u;    /* the top of the range */
    }
}

#define EXPECT(call, want) do { int s__ = (call); if (s__ != (want)) { \
    fprintf(stderr, "%s:%d: status %d, expected %d\n", __FILE__, __LINE__, s__, (want)); return 1; } } while (0)

int main(void) {
    const int blocks[] = {1, 8, 16, 32, 64};
    int calls = 0;
    for (int bi = 0; bi < 5; ++bi) {
        const int block = blocks[bi];
        for (int w = 2; w <= 8; ++w) {
            for (int e = 2; e <= 8; e += 3) {
                const int64_t rows = 1 + (int64_t)(rnd() % 5), nb = 1 + (int64_t)(rnd() % 4), cols = nb * block;
                const int64_t stride = cols + (int64_t)(rnd() % 3);
                float *x = malloc(sizeof(float) * (size_t)(rows * stride));
                int8_t *q = malloc((size_t)(rows * cols)), *q2 = malloc((size_t)(rows * cols));
                uint8_t *ex = malloc((size_t)(rows * nb)), *ex2 = malloc((size_t)(rows * nb));
                uint8_t *bits = malloc((size_t)(rows * ((cols * w + 7) / 8)));
                double *y = malloc(sizeof(double) * (size_t)(rows * cols));
                for (int64_t i = 0; i < rows * stride; ++i) x[i] = draw(bi + w + e);
                for (int rounding = 0; rounding < 2; ++rounding) {
                    EXPECT(mxo_quantize(x, rows, cols, stride, block, e, w, rounding, q, ex), MXO_OK);
                    EXPECT(mxo_dequantize(q, ex, rows, cols, block, e, w, y), MXO_OK);
                    const int whole = (cols * w) % 8 == 0 ? MXO_OK : MXO_BAD_ARG;   /* rows are whole bytes */
                    EXPECT(mxo_pack_bits(q, rows, cols, w, bits), whole);
                    EXPECT(mxo_unpack_bits(bits, rows, cols, w, q2), whole);
                    for (int wd = 2; wd <= 8; wd += 2)
                        EXPECT(mxo_cast(q, ex, rows, cols, block, e, w, 8 - (e % 3), wd, rounding, q2, ex2), MXO_OK);
                    calls += 8;
                }
                /* blocks down the columns: rows must be a multiple of the block */
                {
                    const int64_t r0 = block * 2, c0 = 3;
                    float *xa = malloc(sizeof(float) * (size_t)(r0 * (c0 + 1)));
                    int8_t *qa = malloc((size_t)(r0 * c0));
                    uint8_t *ea = malloc((size_t)(c0 * 2));
                    for (int64_t i = 0; i < r0 * (c0 + 1); ++i) xa[i] = draw(w);
                    EXPECT(mxo_quantize_axis0(xa, r0, c0, c0 + 1, block, e, w, 0, qa, ea), MXO_OK);
                    free(xa); free(qa); free(ea);
                }
                /* product of the quantized matrix with itself (rows x rows), whole and one row window */
                {
                    double *Y = malloc(sizeof(double) * (size_t)(rows * rows)), *mag = malloc(sizeof(double) * (size_t)(rows * rows));
                    EXPECT(mxo_gemm(q, ex, w, q, ex, w, rows, rows, cols, block, e, 0, rows, Y, mag), MXO_OK);
                    EXPECT(mxo_gemm(q, ex, w, q, ex, w, rows, rows, cols, block, e, rows - 1, rows, Y, NULL), MXO_OK);
                    EXPECT(mxo_gemm_at(q, ex, w, q, ex, w, cols, block, e, Y, mag), MXO_OK);
                    free(Y); free(mag);
                }
                free(x); free(q); free(q2); free(ex); free(ex2); free(bits); free(y);
            }
        }
        /* the other block formats: every (e, m) with 1 + e + m <= 8 */
        for (int e = 1; e <= 7; ++e)
            for (int m = 0; 1 + e + m <= 8; ++m) {
                const int64_t rows = 3, cols = 2 * block;
                float *x = malloc(sizeof(float) * (size_t)(rows * cols));
                uint8_t *codes = malloc((size_t)(rows * cols)), *sh = malloc((size_t)(rows * 2));
                double *y = malloc(sizeof(double) * (size_t)(rows * cols));
                for (int64_t i = 0; i < rows * cols; ++i) x[i] = draw(e + m);
                for (int rounding = 0; rounding < 2; ++rounding)
                    EXPECT(mxo_quantize_minifloat(x, rows, cols, cols, block, e, m, rounding, codes, sh), MXO_OK);
                EXPECT(mxo_dequantize_minifloat(codes, sh, rows, cols, block, e, m, y), MXO_OK);
                free(x); free(codes); free(sh); free(y);
                calls += 3;
            }
    }
    /* rejections touch nothing */
    EXPECT(mxo_quantize(NULL, 1, 15, 15, 16, 8, 8, 0, NULL, NULL), MXO_BAD_ARG);
    EXPECT(mxo_quantize(NULL, 1, 16, 16, 16, 9, 8, 0, NULL, NULL), MXO_BAD_ARG);
    EXPECT(mxo_gemm(NULL, NULL, 8, NULL, NULL, 4, 1, 1, 17, 16, 8, 0, 1, NULL, NULL), MXO_BAD_ARG);
    {
        float bad[16] = {0};
        int8_t q[16];
        uint8_t ex[1];
        bad[3] = NAN;
        EXPECT(mxo_quantize(bad, 1, 16, 16, 16, 8, 8, 0, q, ex), MXO_NONFINITE);
    }
    printf("sanitize_check: %d calls clean\n", calls);
    return 0;
}
