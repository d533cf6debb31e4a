/*
 * MXInt CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step implementation of the MXInt (block floating
 * point) format and of the MXInt x MXInt matrix product, written from the
 * paper's description of the format.  It exists to check the GPU library; it
 * shares no code with it, is never called by it, and is never tuned.
 *
 * What the paper fixes, and where:
 *   - an MXInt value is a 3-tuple (B, e, m): a block of Pi(B) elements shares
 *     one e-bit exponent, every element has an m-bit mantissa and a sign bit
 *     (Section 4.1, Eq. 1: average bits p = e/Pi(B) + m + 1);
 *   - the shared exponent bounds the range of the values in its block
 *     (Section 2, "What are MX Formats?");
 *   - software emulation of an operator = quantize the inputs, run the
 *     ordinary floating-point operator on the dequantized values
 *     (Section 3.2);
 *   - the hardware dot product multiplies integer mantissas, adds them, and
 *     handles the two shared exponents once per block (Section 3.2, Fig. 3).
 *
 * What the paper leaves open, and the reading taken here (all of them are
 * choices of this implementation, not of the paper):
 *   - w := m + 1 is the number of stored bits per element, sign included;
 *     mantissa values are the symmetric range -qmax..+qmax, qmax = 2^(w-1)-1,
 *     stored in two's complement;
 *   - shared exponent E = floor(log2(max |x|)) of the block, stored biased by
 *     2^(e-1)-1 and clamped to the e-bit range; an all-zero block stores 0;
 *   - one mantissa unit is worth 2^(E-(w-2)), so the block maximum lands in
 *     [2^(w-2), 2^(w-1)); a value that rounds up to 2^(w-1) saturates at qmax
 *     and the exponent is not changed;
 *   - rounding is to nearest, ties to the even integer (rounding = 0), or
 *     toward zero (rounding = 1);
 *   - fp32 subnormal inputs count with their true value; inputs are finite;
 *   - blocks are 1-D runs of `block` consecutive elements of a row;
 *   - mantissas are packed little-endian: element k of a row occupies bits
 *     [k*w, (k+1)*w) of the row's bit stream, bit i of the stream being bit
 *     (i mod 8) of byte (i div 8).
 *
 * All floating point here is IEEE double: scaling by a power of two is done
 * with ldexp (exact), rounding with nearbyint under the default rounding mode
 * (ties to even), the exponent with frexp (exact).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define MXO_OK 0
#define MXO_BAD_ARG 1
#define MXO_NONFINITE 2

static int mxo_check_format(int block, int e, int w, int rounding) {
    if (block < 1 || e < 2 || e > 8 || w < 2 || w > 8) return MXO_BAD_ARG;
    if (rounding != 0 && rounding != 1) return MXO_BAD_ARG;
    return MXO_OK;
}

/* Exponent bias of an e-bit shared exponent. */
static int mxo_bias(int e) { return (1 << (e - 1)) - 1; }

/*
 * Quantize one block of n values (Section 4.1 format; Section 2 range rule).
 * q receives the signed mantissas, the return value is the stored exponent
 * byte, or -1 if an input is not finite.
 */
static int mxo_quantize_block(const float *x, int64_t stride, int n, int e, int w, int rounding,
                              int8_t *q) {
    double amax = 0.0;
    for (int i = 0; i < n; ++i) {
        double v = (double)x[i * stride];
        if (!isfinite(v)) return -1;
        if (fabs(v) > amax) amax = fabs(v);
    }
    if (amax == 0.0) {
        for (int i = 0; i < n; ++i) q[i] = 0;
        return 0;
    }
    const int bias = mxo_bias(e);
    const int qmax = (1 << (w - 1)) - 1;
    int ex;
    (void)frexp(amax, &ex);          /* amax = f * 2^ex, f in [0.5, 1)  =>  floor(log2 amax) = ex - 1 */
    int E = ex - 1;
    const int Emin = -bias, Emax = ((1 << e) - 1) - bias;
    if (E < Emin) E = Emin;
    if (E > Emax) E = Emax;
    const int s = E - (w - 2);       /* one mantissa unit = 2^s */
    for (int i = 0; i < n; ++i) {
        double v = ldexp((double)x[i * stride], -s);
        double r = (rounding == 0) ? nearbyint(v) : trunc(v);
        if (r > (double)qmax) r = (double)qmax;
        if (r < (double)-qmax) r = (double)-qmax;
        q[i] = (int8_t)r;
    }
    return E + bias;
}

/*
 * x: rows x cols floats, element (r, c) at x[r*row_stride + c].
 * Blocks run along the columns of each row; cols must be a multiple of block.
 * q:    rows*cols signed mantissas (one int8 each, unpacked), row-major.
 * exps: rows*(cols/block) exponent bytes, row-major.
 */
int mxo_quantize(const float *x, int64_t rows, int64_t cols, int64_t row_stride, int block, int e,
                 int w, int rounding, int8_t *q, uint8_t *exps) {
    if (mxo_check_format(block, e, w, rounding) != MXO_OK) return MXO_BAD_ARG;
    if (rows < 0 || cols < 0 || cols % block != 0) return MXO_BAD_ARG;
    const int64_t nb = cols / block;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t b = 0; b < nb; ++b) {
            int eb = mxo_quantize_block(x + r * row_stride + b * block, 1, block, e, w, rounding,
                                        q + r * cols + b * block);
            if (eb < 0) { bad = 1; eb = 0; }
            exps[r * nb + b] = (uint8_t)eb;
        }
    }
    return bad ? MXO_NONFINITE : MXO_OK;
}

/*
 * Same, with the blocks running down the rows of each column (the strided
 * axis).  The result is written as the quantization of the transposed matrix:
 * q is cols x rows, exps is cols x (rows/block).
 */
int mxo_quantize_axis0(const float *x, int64_t rows, int64_t cols, int64_t row_stride, int block,
                       int e, int w, int rounding, int8_t *q, uint8_t *exps) {
    if (mxo_check_format(block, e, w, rounding) != MXO_OK) return MXO_BAD_ARG;
    if (rows < 0 || cols < 0 || rows % block != 0) return MXO_BAD_ARG;
    const int64_t nb = rows / block;
    int bad = 0;
    for (int64_t c = 0; c < cols; ++c) {
        for (int64_t b = 0; b < nb; ++b) {
            int eb = mxo_quantize_block(x + (b * block) * row_stride + c, row_stride, block, e, w,
                                        rounding, q + c * rows + b * block);
            if (eb < 0) { bad = 1; eb = 0; }
            exps[c * nb + b] = (uint8_t)eb;
        }
    }
    return bad ? MXO_NONFINITE : MXO_OK;
}

/*
 * Dequantize: value = q * 2^(Ebiased - bias - (w-2)).  Output in double, so no
 * rounding or underflow can occur.
 */
int mxo_dequantize(const int8_t *q, const uint8_t *exps, int64_t rows, int64_t cols, int block,
                   int e, int w, double *y) {
    if (mxo_check_format(block, e, w, 0) != MXO_OK) return MXO_BAD_ARG;
    if (rows < 0 || cols < 0 || cols % block != 0) return MXO_BAD_ARG;
    const int64_t nb = cols / block;
    const int bias = mxo_bias(e);
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int s = (int)exps[r * nb + c / block] - bias - (w - 2);
            y[r * cols + c] = ldexp((double)q[r * cols + c], s);
        }
    return MXO_OK;
}

/*
 * Bit packing of one tensor of signed mantissas: w-bit two's complement,
 * little-endian bit stream per row.  rows*cols*w must make whole bytes per row.
 */
int mxo_pack_bits(const int8_t *q, int64_t rows, int64_t cols, int w, uint8_t *out) {
    if (w < 2 || w > 8 || rows < 0 || cols < 0 || (cols * w) % 8 != 0) return MXO_BAD_ARG;
    const int64_t row_bytes = cols * w / 8;
    memset(out, 0, (size_t)(rows * row_bytes));
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            unsigned code = (unsigned)(int)q[r * cols + c] & ((1u << w) - 1u);
            for (int i = 0; i < w; ++i) {
                int64_t bit = c * w + i;
                if ((code >> i) & 1u) out[r * row_bytes + bit / 8] |= (uint8_t)(1u << (bit % 8));
            }
        }
    return MXO_OK;
}

int mxo_unpack_bits(const uint8_t *in, int64_t rows, int64_t cols, int w, int8_t *q) {
    if (w < 2 || w > 8 || rows < 0 || cols < 0 || (cols * w) % 8 != 0) return MXO_BAD_ARG;
    const int64_t row_bytes = cols * w / 8;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            unsigned code = 0;
            for (int i = 0; i < w; ++i) {
                int64_t bit = c * w + i;
                code |= (unsigned)((in[r * row_bytes + bit / 8] >> (bit % 8)) & 1u) << i;
            }
            int v = (int)code;
            if (code & (1u << (w - 1))) v -= (1 << w);   /* sign-extend the w-bit code */
            q[r * cols + c] = (int8_t)v;
        }
    return MXO_OK;
}

/*
 * MXInt x MXInt product (Section 3.2: integer mantissa products and sums, the
 * two shared exponents applied once per block).
 *   qa [M,K] with exponents ea [M,K/block];  qb [N,K] with exponents eb [N,K/block]
 *   Y[m,n]  = sum_b ( sum_{k in block b} qa[m,k]*qb[n,k] ) * 2^(Ea[m,b] + Eb[n,b] - (wa-2) - (wb-2))
 * Block sums are exact integers (int64); the sum over blocks is taken in
 * double, in increasing block order.  mag (may be NULL) receives
 * sum_b |term_b|, the scale against which a tolerance is stated.
 * Only rows m with m_begin <= m < m_end are computed (Y and mag are still
 * indexed by the full m).
 */
int mxo_gemm(const int8_t *qa, const uint8_t *ea, int wa, const int8_t *qb, const uint8_t *eb,
             int wb, int64_t M, int64_t N, int64_t K, int block, int e, int64_t m_begin,
             int64_t m_end, double *Y, double *mag) {
    if (mxo_check_format(block, e, wa, 0) != MXO_OK || mxo_check_format(block, e, wb, 0) != MXO_OK)
        return MXO_BAD_ARG;
    if (M < 0 || N < 0 || K < 0 || K % block != 0 || m_begin < 0 || m_end > M) return MXO_BAD_ARG;
    const int64_t nb = K / block;
    const int bias = mxo_bias(e);
#pragma omp parallel for schedule(static)
    for (int64_t m = m_begin; m < m_end; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, amag = 0.0;
            for (int64_t b = 0; b < nb; ++b) {
                int64_t d = 0;
                for (int k = 0; k < block; ++k)
                    d += (int64_t)qa[m * K + b * block + k] * (int64_t)qb[n * K + b * block + k];
                int s = ((int)ea[m * nb + b] - bias - (wa - 2)) + ((int)eb[n * nb + b] - bias - (wb - 2));
                double term = ldexp((double)d, s);
                acc += term;
                amag += fabs(term);
            }
            Y[m * N + n] = acc;
            if (mag) mag[m * N + n] = amag;
        }
    }
    return MXO_OK;
}

/* One output element of the product above (for sampled checks at large sizes). */
int mxo_gemm_at(const int8_t *qa_row, const uint8_t *ea_row, int wa, const int8_t *qb_row,
                const uint8_t *eb_row, int wb, int64_t K, int block, int e, double *y, double *mag) {
    return mxo_gemm(qa_row, ea_row, wa, qb_row, eb_row, wb, 1, 1, K, block, e, 0, 1, y, mag);
}

/*
 * Cast between two precisions of the same MXInt block shape without leaving
 * the format (Section 4, paragraph on mixed-precision quantization: casting
 * mantissas is bit extension or truncation, the exponent needs a shift).
 *
 * Reading taken here: the cast gives exactly what quantizing the block's exact
 * values to the destination format gives.  In integers: with mx = max |q_i| and
 * p = floor(log2 mx), the block maximum is mx * 2^(E - (ws-2)), so the new
 * shared exponent is E' = E - (ws-2) + p (clamped to the destination's e-bit
 * range), and every mantissa is q_i * 2^sh in units of the destination,
 * sh = (E - (ws-2)) - (E' - (wd-2)): a left shift when sh >= 0 (extension,
 * exact), a right shift by -sh with the destination's rounding (to nearest,
 * ties to even; or truncation toward zero) otherwise, then saturation at
 * +-qmax.  A block of zeros stores exponent byte 0.
 */
static int mxo_floor_log2(int v) {      /* v >= 1 */
    int p = 0;
    while (v > 1) { v >>= 1; ++p; }
    return p;
}

int mxo_cast(const int8_t *q, const uint8_t *exps, int64_t rows, int64_t cols, int block, int es,
             int ws, int ed, int wd, int rounding, int8_t *q_out, uint8_t *exps_out) {
    if (mxo_check_format(block, es, ws, 0) != MXO_OK) return MXO_BAD_ARG;
    if (mxo_check_format(block, ed, wd, rounding) != MXO_OK) return MXO_BAD_ARG;
    if (rows < 0 || cols < 0 || cols % block != 0) return MXO_BAD_ARG;
    const int64_t nb = cols / block;
    const int bias_s = mxo_bias(es), bias_d = mxo_bias(ed);
    const int Emin = -bias_d, Emax = ((1 << ed) - 1) - bias_d;
    const int qmax = (1 << (wd - 1)) - 1;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t b = 0; b < nb; ++b) {
            const int8_t *src = q + r * cols + b * block;
            int8_t *dst = q_out + r * cols + b * block;
            int mx = 0;
            for (int i = 0; i < block; ++i) {
                int a = src[i] < 0 ? -(int)src[i] : (int)src[i];
                if (a > mx) mx = a;
            }
            if (mx == 0) {
                for (int i = 0; i < block; ++i) dst[i] = 0;
                exps_out[r * nb + b] = 0;
                continue;
            }
            const int E = (int)exps[r * nb + b] - bias_s;
            int E2 = E - (ws - 2) + mxo_floor_log2(mx);
            if (E2 < Emin) E2 = Emin;
            if (E2 > Emax) E2 = Emax;
            const int sh = (E - (ws - 2)) - (E2 - (wd - 2));
            for (int i = 0; i < block; ++i) {
                const int v = src[i];
                int64_t res;
                if (sh >= 0) {
                    res = sh >= 40 ? (v > 0 ? INT64_MAX / 2 : (v < 0 ? -(INT64_MAX / 2) : 0))
                                   : (int64_t)v * ((int64_t)1 << sh);
                } else {
                    const int k = -sh;
                    const int64_t a = v < 0 ? -(int64_t)v : (int64_t)v;     /* magnitude: both roundings are odd-symmetric */
                    int64_t m;
                    if (k >= 40) {
                        m = 0;
                    } else {
                        m = a >> k;                                          /* truncation */
                        if (rounding == 0) {
                            const int64_t rem = a - (m << k), half = (int64_t)1 << (k - 1);
                            if (rem > half || (rem == half && (m & 1))) ++m;  /* nearest, ties to even */
                        }
                    }
                    res = v < 0 ? -m : m;
                }
                if (res > qmax) res = qmax;
                if (res < -qmax) res = -qmax;
                dst[i] = (int8_t)res;
            }
            exps_out[r * nb + b] = (uint8_t)(E2 + bias_d);
        }
    }
    return MXO_OK;
}

/*
 * ------------------------------------------------------------------------------------------
 * The paper's two other block formats (Section 2, "What are MX Formats?"): Block Minifloat
 * (BMF), whose elements are small floating-point numbers that share the exponent *bias* of
 * their block, and Block Logarithm (BL), which is BMF without mantissa bits -- every value a
 * power of two.  The paper gives the idea and no bit-level definition; the reading taken here
 * (all of it a choice of this implementation):
 *   - an element is sign | c (e bits) | f (m bits), m = 0 for BL; with cmax = 2^e - 1 and the
 *     block's shared top exponent T,
 *         c >= 1:  value = +-2^(c - cmax + T) * (1 + f / 2^m)
 *         c == 0:  value = +-2^(1 - cmax + T) * (f / 2^m)          (gradual underflow; zero)
 *     i.e. the shared bias is cmax - T; every code is a finite number;
 *   - the shared byte stores T + 127, T clamped to [-126, 127]; an all-zero block stores 0;
 *   - T is the exponent of the block maximum after rounding: floor(log2 amax), plus one when
 *     amax is at or above the midpoint between the largest value of that binade and the next
 *     power of two (so that rounding never has to saturate); toward-zero rounding never
 *     carries, T = floor(log2 amax);
 *   - an element is rounded to the nearest representable value, a tie to the neighbour whose
 *     code integer (c << m | f) is even (rounding = 0), or toward zero (rounding = 1); a value
 *     above the largest representable one (only possible when T was clamped) saturates.
 * ------------------------------------------------------------------------------------------
 */
static int mxo_check_minifloat(int block, int e, int m, int rounding) {
    if (block < 1 || e < 1 || m < 0 || 1 + e + m > 8) return MXO_BAD_ARG;
    if (rounding != 0 && rounding != 1) return MXO_BAD_ARG;
    return MXO_OK;
}

/* codes: one byte per element (sign << (e+m) | c << m | f); shared: one byte per block. */
int mxo_quantize_minifloat(const float *x, int64_t rows, int64_t cols, int64_t row_stride, int block,
                           int e, int m, int rounding, uint8_t *codes, uint8_t *shared) {
    if (mxo_check_minifloat(block, e, m, rounding) != MXO_OK) return MXO_BAD_ARG;
    if (rows < 0 || cols < 0 || cols % block != 0) return MXO_BAD_ARG;
    const int64_t nb = cols / block;
    const int cmax = (1 << e) - 1;
    int bad = 0;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t b = 0; b < nb; ++b) {
            const float *src = x + r * row_stride + b * block;
            uint8_t *dst = codes + r * cols + b * block;
            double amax = 0.0;
            for (int i = 0; i < block; ++i) {
                if (!isfinite(src[i])) bad = 1;
                const double a = fabs((double)src[i]);
                if (a > amax) amax = a;
            }
            if (amax == 0.0 || bad) {
                for (int i = 0; i < block; ++i) dst[i] = 0;
                shared[r * nb + b] = 0;
                continue;
            }
            int ex;
            frexp(amax, &ex);                       /* amax = fr * 2^ex, fr in [0.5, 1) */
            int T = ex - 1;                         /* floor(log2 amax) */
            if (rounding == 0) {
                /* midpoint between the binade's largest value (2 - 2^-m) * 2^T and 2^(T+1) */
                const double mid = ldexp(1.0, T + 1) - ldexp(1.0, T - m - 1);
                if (amax >= mid) T += 1;
            }
            if (T < -126) T = -126;
            if (T > 127) T = 127;
            const int L = T - cmax + 1;             /* exponent of the smallest normal binade */
            for (int i = 0; i < block; ++i) {
                const double a = fabs((double)src[i]);
                const int sign = signbit(src[i]) ? 1 : 0;
                int c = 0, f = 0;
                if (a > 0.0) {
                    int ea;
                    frexp(a, &ea);
                    int k = ea - 1;
                    if (k < L) k = L;
                    const double qv = ldexp(a, m - k);          /* in units of the binade's step: exact */
                    double lo = floor(qv);
                    const double rem = qv - lo;
                    long n = (long)lo;
                    if (rounding == 0 && rem > 0.0) {
                        /* code integer of the lower neighbour: its parity decides a tie */
                        const long c_lo = n >= (1L << m) ? (long)(k - L + 1) : 0;
                        const long code_lo = (c_lo << m) | (n & ((1L << m) - 1));
                        if (rem > 0.5 || (rem == 0.5 && (code_lo & 1))) n += 1;
                    }
                    if (n == (1L << (m + 1))) { k += 1; n = 1L << m; }     /* carry into the next binade */
                    if (k > T) { k = T; n = (1L << (m + 1)) - 1; }         /* saturate (clamped T only) */
                    if (n >= (1L << m)) { c = k - L + 1; f = (int)(n - (1L << m)); }
                    else { c = 0; f = (int)n; }
                }
                dst[i] = (uint8_t)((sign << (e + m)) | (c << m) | f);
            }
            shared[r * nb + b] = (uint8_t)(T + 127);
        }
    }
    return bad ? MXO_NONFINITE : MXO_OK;
}

int mxo_dequantize_minifloat(const uint8_t *codes, const uint8_t *shared, int64_t rows, int64_t cols,
                             int block, int e, int m, double *y) {
    if (mxo_check_minifloat(block, e, m, 0) != MXO_OK) return MXO_BAD_ARG;
    if (rows < 0 || cols < 0 || cols % block != 0) return MXO_BAD_ARG;
    const int64_t nb = cols / block;
    const int cmax = (1 << e) - 1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t cidx = 0; cidx < cols; ++cidx) {
            const int code = codes[r * cols + cidx];
            const int sb = shared[r * nb + cidx / block];
            const int sign = (code >> (e + m)) & 1, c = (code >> m) & cmax, f = code & ((1 << m) - 1);
            double v = 0.0;
            if (sb != 0) {
                const int T = sb - 127;
                if (c >= 1) v = ldexp(1.0 + ldexp((double)f, -m), c - cmax + T);
                else v = ldexp(ldexp((double)f, -m), 1 - cmax + T);
            }
            y[r * cols + cidx] = sign ? -v : v;
        }
    return MXO_OK;
}

int mxo_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}
