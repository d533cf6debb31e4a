/*
 * mx.h -- C ABI of the MXInt library for MI355X (gfx950).
 *
 * MXInt is the block floating-point format of the paper "A Dataflow Compiler for
 * Efficient LLM Inference using Custom Microscaling Formats": a block of elements
 * shares one exponent, every element keeps its own signed integer mantissa
 * (Section 2, "What are MX Formats?"; Section 4.1, the 3-tuple (B, e, m) and Eq. 1).
 * This library holds the data-parallel part of inference in that format: the block
 * quantizer, its inverse, a re-layout of quantized operands for the matrix cores,
 * and the MXInt x MXInt matrix product (Section 3.2: integer mantissa products and
 * sums, the two shared exponents applied once per block).
 *
 * Conventions for every entry point
 *   - Pointers named x, y, Y, mant, exps, packed, A_packed, B_packed are DEVICE
 *     pointers (e.g. a torch tensor's data_ptr()).  The library allocates nothing,
 *     frees nothing and never synchronizes (mx_check_finite, which returns an answer
 *     about device data, is the one exception): all work is enqueued on `stream` (a
 *     hipStream_t passed as void*, NULL = default stream).  Between calls it keeps no
 *     data; the only host state is, per kernel that needs more than 64 KB of LDS, a
 *     set of the devices on which that limit has been raised (set once, thread-safe).
 *   - The return value is an mx_status.  Nothing throws or aborts across this
 *     boundary.  MX_ERR_BAD_ARG: a null pointer, a negative size, a size that is not
 *     a whole number of blocks, a format outside the ranges stated at mx_format, or
 *     a misaligned pointer.  MX_ERR_UNSUPPORTED: a legal request this library has no
 *     kernel for.  MX_ERR_DEVICE: the HIP runtime refused the launch.
 *   - Inputs must be finite; NaN and infinity give unspecified mantissas (no fault).
 *     mx_check_finite tests that precondition for callers who want it tested.
 *
 * Canonical form of a quantized tensor of `rows` rows and `cols` columns with the
 * blocks running along the columns (this is the form bit-exactness is stated on):
 *   mant: rows * (cols*w/8) bytes.  Element k of a row occupies bits [k*w, (k+1)*w)
 *         of that row's bit stream; bit i of the stream is bit (i mod 8) of byte
 *         (i div 8); mantissas are w-bit two's complement.
 *   exps: rows * (cols/block) bytes, one per block: E + (2^(e-1) - 1).
 *   A batch is `batch` such tensors back to back.
 * The value of an element is  q * 2^(E - (w - 2)).
 */
#ifndef MX_H_
#define MX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MX_API __attribute__((visibility("default")))

/*
 * One MXInt format (Section 4.1).  The paper writes MXInt(B, e, m) with m the
 * mantissa width WITHOUT the sign bit (Eq. 1: p = e/prod(B) + m + 1); here
 * mant_bits = m + 1 is the stored width of an element, so the paper's
 * MXInt((16,2), 8, 7) has block = 16, block_rows = 2, exp_bits = 8, mant_bits = 8.
 */
typedef struct {
    int32_t block;     /* elements of a row sharing one exponent, consecutive along the reduction axis:
                          8, 16, 32 or 64 for mx_quantize / mx_dequantize / mx_cast;
                          16, 32 or 64 for mx_pack / mx_unpack / mx_gemm / mx_linear */
    int32_t exp_bits;  /* e, 2..8 (the paper fixes 8 for every tensor, Section 4.1) */
    int32_t mant_bits; /* w = m + 1, 2..8; mantissas lie in -(2^(w-1)-1) .. +(2^(w-1)-1) */
    int32_t rounding;  /* MX_RNE or MX_RTZ */
    int32_t block_rows;/* 1 or 2: adjacent rows that share the exponent, i.e. the second entry of the
                          paper's block shape -- MXInt((16,2),8,7) is block 16, block_rows 2, mant_bits 8.
                          With 2, rows must be even and the canonical exponent array is
                          [rows/2][cols/block]; the packed layouts repeat the byte for both rows, so
                          mx_gemm does not care (along axis 0 the rows are those of the transposed
                          matrix: two columns of x). */
} mx_format;

enum { MX_RNE = 0,  /* round to nearest, ties to the even mantissa */
       MX_RTZ = 1   /* round toward zero (the "truncation" of a width cast, Section 4) */ };

typedef enum { MX_OK = 0, MX_ERR_BAD_ARG = 1, MX_ERR_UNSUPPORTED = 2, MX_ERR_DEVICE = 3 } mx_status;

/*
 * Device layouts mx_pack can write.  The bytes are opaque to the caller;
 * mx_unpack restores the canonical form bit for bit.
 *   MX_LAYOUT_FRAGMENT: w bits per element + 1 byte per block, i.e. exactly the
 *       density of the canonical form (Eq. 1), arranged in the order the matrix
 *       cores' lanes consume it.  Rows are padded to a multiple of 32 and columns to
 *       a multiple of 4 blocks with zeros.  Either operand of mx_gemm, any M, block 16, 32 or 64.
 *   MX_LAYOUT_MATRIX: the operand as the floating-point matrix cores of gfx950 read it; the
 *       layout of the compute-bound (prefill, attention) path.  Both operands of one mx_gemm use
 *       the same layout.
 *       Block 32 or 64 (block-scaled matrix instruction): every mantissa is carried exactly in 6-bit
 *       float codes, one code for up to 4 stored bits and two codes (q = 16*h + l) for 5..8 bits,
 *       i.e. 6 or 12 bits per element plus the exponent bytes; rows are padded to 32 (64 for
 *       one-code operands) and K to 256.  Restriction: exponent bytes above 250 (|x| >= 2^124 at
 *       e = 8) are not representable next to the +4 offset of the high code; such blocks give
 *       unspecified products.
 *       Accuracy of products in this layout (both block forms): mantissa products and their sums inside a
 *       block are exact, but the matrix instruction aligns the running fp32 sum to the largest SINGLE product
 *       it adds and keeps 24 bits below that, not below the block sums.  A block whose large products cancel
 *       can therefore push out low bits that much smaller blocks had contributed.  Guaranteed for any in-range
 *       input:  |err| <= 1e-5 * sum_blocks |block term|  +  1e-6 * sum_k |product_k|.  The first term alone
 *       holds whenever, for an output element, the exponent sums Ea + Eb of its blocks span at most
 *       24 - wa - wb binades (12 for 8-bit by 4-bit operands: a product of mantissa pieces has at most
 *       wa + wb - 1 bits, so nothing is pushed out then) -- and it
 *       holds on LLM-shaped data (heavy tails, outlier channels), where products do not cancel inside blocks
 *       to that degree.  The weaker bound is still tighter than that of a float product of the dequantized
 *       operands, Section 3.2's emulated operator.  Callers that need the first term alone on arbitrary data
 *       use MX_LAYOUT_FRAGMENT.
 *       Block 16 (that instruction scales runs of 32, not 16): every element is stored as the
 *       bfloat16 number mantissa * 2^exponent, which is exact, 16 bits per element plus the
 *       exponent bytes; rows are padded to 32 and K to 64.  Restriction: nonzero elements must be
 *       normal bfloat16 numbers, i.e. at e = 8 the exponent byte of a block with nonzero mantissas
 *       lies in [mant_bits - 1, 253] (always so for blocks quantized from |x| >= 2^-120); other
 *       blocks give unspecified products and do not survive mx_unpack.
 */
enum { MX_LAYOUT_FRAGMENT = 0, MX_LAYOUT_MATRIX = 1 };

/* Library version: major*10000 + minor*100 + patch. */
MX_API int32_t mx_version(void);

/* Static, NUL-terminated description of a status code. */
MX_API const char* mx_status_string(mx_status s);

/* Bytes of the canonical mantissa / exponent arrays of batch x rows x cols; 0 on a bad format. */
MX_API size_t mx_mant_bytes(int64_t batch, int64_t rows, int64_t cols, mx_format f);
MX_API size_t mx_exps_bytes(int64_t batch, int64_t rows, int64_t cols, mx_format f);

/*
 * Block quantizer (Section 3.2 "quantize ... between the given format and
 * floating-point numbers"; format of Section 4.1).  Per block of f.block elements:
 *   E = floor(log2(max |x|)) clamped to the e-bit range [-(2^(e-1)-1), 2^(e-1)]; a zero
 *   block stores exponent byte 0;  q = round(x * 2^-(E-(w-2))) with f.rounding, then
 *   clamped to +-(2^(w-1)-1).  fp32 subnormals count with their true value.
 *
 * x: batch matrices of rows x cols floats; element (b, r, c) at x[b*batch_stride +
 *    r*row_stride + c] (strides in elements; the columns are contiguous).
 * axis = 1: blocks run along the columns; cols % block == 0.
 *           mant, exps receive the canonical form of batch x rows x cols.
 * axis = 0: blocks run down the rows of each column; rows % block == 0.
 *           mant, exps receive the canonical form of the TRANSPOSED matrices,
 *           batch x cols x rows (the layout the right operand of a product needs
 *           when the reduction runs over the rows of x).
 * x must be 4-byte aligned; row_stride >= cols; mant and exps are written densely; mant must be
 * 16-byte aligned (any allocation's start is).
 */
MX_API mx_status mx_quantize(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                      int64_t batch_stride, int32_t axis, mx_format f, uint8_t* mant, uint8_t* exps,
                      void* stream);

/*
 * The precondition of the calls that take fp32 input (finite values), checked as a call of its own for callers and
 * tests that want it; the quantizers themselves do not look (a pass over the input would cost as much as they do).
 * Returns MX_ERR_BAD_ARG when one of the batch x rows x cols elements, addressed as in mx_quantize, is a NaN or an
 * infinity, MX_OK when all are finite.  The only entry point that waits: it enqueues its kernels on `stream`, copies
 * the answer to the host and synchronizes that stream before it returns (so it cannot be captured into a graph).
 * flag: 4 bytes of caller-owned device memory, 4-byte aligned, overwritten (1 = a non-finite value was found).
 */
MX_API mx_status mx_check_finite(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                 int64_t batch_stride, int32_t* flag, void* stream);

/*
 * Inverse of the quantizer's encoding (Section 3.2 "dequantize"): y[b][r][c] =
 * q * 2^(E - (w-2)) as fp32, dense batch x rows x cols, from the canonical form of
 * batch x rows x cols (blocks along the columns).  Exact whenever the value is
 * representable in fp32 (always, except below the fp32 subnormal spacing).  y must be 16-byte aligned.
 */
MX_API mx_status mx_dequantize(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows,
                        int64_t cols, mx_format f, float* y, void* stream);

/*
 * The paper's two other block formats (Section 2, "What are MX Formats?"): Block Minifloat, whose
 * elements are small floating-point numbers sharing the exponent bias of their block, and Block
 * Logarithm, the same without mantissa bits (every value a power of two or zero).
 * An element is one byte: sign << (e+m) | c << m | f, with c the exp_bits-wide exponent field and f
 * the mant_bits-wide mantissa field, 1 + exp_bits + mant_bits <= 8.  With cmax = 2^exp_bits - 1
 * and the block's shared top exponent T:
 *     c >= 1:  +-2^(c - cmax + T) * (1 + f / 2^mant_bits)
 *     c == 0:  +-2^(1 - cmax + T) * (f / 2^mant_bits)         (gradual underflow, and zero)
 * The shared byte is T + 127 (T in -126..127), 0 for an all-zero block.  T is the exponent of the
 * block maximum after rounding, elements round to the nearest representable value with ties to the
 * even code (MX_RNE) or toward zero (MX_RTZ).
 */
typedef struct {
    int32_t block;     /* elements of a row sharing the bias: 8, 16, 32 or 64 */
    int32_t exp_bits;  /* e, 1..7 */
    int32_t mant_bits; /* m, 0..6; 0 is the Block Logarithm format */
    int32_t rounding;  /* MX_RNE or MX_RTZ */
} mx_minifloat_format;

/*
 * Quantizer and its inverse for the formats above, blocks along the columns.
 * x: device fp32, element (b, r, c) at x[b*batch_stride + r*row_stride + c], finite values;
 *    16-byte aligned with strides that are multiples of 4 elements (else MX_ERR_UNSUPPORTED).
 * codes: device, batch*rows*cols bytes, 4-byte aligned; shared: batch*rows*(cols/block) bytes.
 * cols must be a multiple of block.  y: device fp32, dense batch x rows x cols, 16-byte aligned.
 */
MX_API mx_status mx_quantize_minifloat(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                int64_t batch_stride, mx_minifloat_format f, uint8_t* codes, uint8_t* shared,
                                void* stream);
MX_API mx_status mx_dequantize_minifloat(const uint8_t* codes, const uint8_t* shared, int64_t batch, int64_t rows,
                                  int64_t cols, mx_minifloat_format f, float* y, void* stream);

/*
 * Width cast inside the format, without going through floating point (Section 4, the paragraph
 * on mixed-precision quantization: casting mantissas is bit extension or truncation, the
 * exponent takes a shift): canonical form in format fs -> canonical form in format fd, same
 * block size, same batch x rows x cols (blocks along the columns).  The result is what
 * mx_quantize would give on the exact values of the source: per block the shared exponent is
 * re-derived from the largest mantissa (a block that is not normalised gains mantissa bits), the
 * mantissas are shifted left (exact) or right with fd.rounding and saturate at +-qmax of fd; the
 * exponent is clamped to fd.exp_bits.  mant and mant_out 4-byte aligned, dense, distinct buffers
 * (MX_ERR_BAD_ARG for in-place use, fs.block != fd.block or fs.block_rows != fd.block_rows);
 * fs.rounding is ignored.
 */
MX_API mx_status mx_cast(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                  mx_format fs, mx_format fd, uint8_t* mant_out, uint8_t* exps_out, void* stream);

/* Bytes mx_pack writes for batch x rows x cols in `layout`; 0 on a bad argument. */
MX_API size_t mx_packed_bytes(int64_t batch, int64_t rows, int64_t cols, mx_format f, int32_t layout);

/*
 * Canonical form -> device layout (the format's memory density is the point of
 * Table 1 and Eq. 1; the layouts keep it).  rows x cols is the operand as mx_gemm
 * sees it: rows = M (left operand) or N (right operand), cols = K, blocks along K.
 * `packed` must be 256-byte aligned and hold mx_packed_bytes(...) bytes.
 */
MX_API mx_status mx_pack(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                  mx_format f, int32_t layout, void* packed, void* stream);

/*
 * mx_quantize (axis 1) and mx_pack in one pass over the fp32 input: `packed` receives exactly
 * the bytes that mx_pack would produce from mx_quantize's output, without the canonical form
 * going through memory.  Same argument rules as mx_quantize; for MX_LAYOUT_MATRIX x must be
 * 16-byte aligned and the strides multiples of 4 elements (else MX_ERR_UNSUPPORTED).
 */
MX_API mx_status mx_quantize_pack(const float* x, int64_t batch, int64_t rows, int64_t cols,
                                  int64_t row_stride, int64_t batch_stride, mx_format f, int32_t layout,
                                  void* packed, void* stream);

/*
 * mx_quantize along axis 0 and mx_pack in one pass: x [rows x cols] is quantized with blocks of
 * f.block consecutive elements DOWN each column (the strided axis) and written as the packed operand
 * of the transposed matrix, cols x rows -- exactly the bytes mx_pack gives from the canonical form
 * that mx_quantize (axis 0) produces.  This is how the V operand of P V is prepared (V [keys x d] is
 * reduced over the keys: Fig. 1, and mx_attention's Vt_packed).  rows must be a multiple of f.block.
 * Same pointer rules as mx_quantize_pack; `packed` holds mx_packed_bytes(batch, cols, rows, f, layout)
 * bytes.  With f.block_rows = 2 (cols even) columns 2p and 2p+1 of x, the rows of the operand, share
 * their exponents: the bytes of mx_quantize_pack on the transposed matrix.
 * Built for MX_LAYOUT_MATRIX with blocks of 16; else MX_ERR_UNSUPPORTED.
 */
MX_API mx_status mx_quantize_pack_axis0(const float* x, int64_t batch, int64_t rows, int64_t cols,
                                        int64_t row_stride, int64_t batch_stride, mx_format f, int32_t layout,
                                        void* packed, void* stream);

/* Exact inverse of mx_pack. */
MX_API mx_status mx_unpack(const void* packed, int64_t batch, int64_t rows, int64_t cols, mx_format f,
                    int32_t layout, uint8_t* mant, uint8_t* exps, void* stream);

/*
 * MXInt x MXInt product (Section 3.2, the MXInt dot-product operator):
 *   Y[b][m][n] = sum over K-blocks j of
 *        ( sum_{k in block j} qa[m][k] * qb[n][k] )  *  2^(Ea[m][j] + Eb[n][j] - (wa-2) - (wb-2))
 * The inner sum is exact (integer matrix instructions on MX_LAYOUT_FRAGMENT; small integers in
 * float codes on MX_LAYOUT_MATRIX); the blocks' scaled values are added in fp32.  Error against the
 * exact value: MX_LAYOUT_FRAGMENT |err| <= 1e-5 * sum_blocks |block term| for any input;
 * MX_LAYOUT_MATRIX the bound stated at the layout (an extra 1e-6 * sum_k |product_k| on
 * adversarial exponent spreads).  Both operands come from mx_pack in the same layout.  The left operand is M x K; the right operand is given as
 * N x K (one row per output column, like torch.nn.Linear.weight).
 * fa.block == fb.block and fa.exp_bits == fb.exp_bits are required.
 * Y: fp32, element (b, m, n) at Y[b*batch_stride_y + m*ldy + n]; ldy >= N.
 * With MX_LAYOUT_FRAGMENT, M <= 8 takes the bandwidth-bound decode path (one pass over the
 * right operand); MX_LAYOUT_MATRIX runs the tiled kernel whatever M is.
 */
MX_API mx_status mx_gemm(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A_packed, mx_format fa,
                  const void* B_packed, mx_format fb, int32_t layout, float* Y, int64_t ldy,
                  int64_t batch_stride_y, void* stream);

/*
 * The emulated operator in full (Section 3.2: quantize the inputs, the operator, quantize the result;
 * Fig. 2b: a linear layer whose bias is MXInt as well): the product of mx_gemm, plus an optional
 * bias, quantized to format `fo` with blocks along N (the axis the next layer reduces over), without
 * the fp32 result going through memory:
 *     out = mx_quantize_pack( fp32(A x B^T) + fp32(bias), fo, layout )       [batch x M x N]
 * bias_mant / bias_exps: canonical form of one row of N elements in format fbias (block_rows 1, same
 * block as fo), shared by the batch; both null for no bias.  The fp32 sum is rounded once more by the
 * addition; the quantizer arithmetic is that of mx_quantize.  out_packed: mx_packed_bytes(batch, M, N,
 * fo, layout) bytes, 256-byte aligned.  Built for MX_LAYOUT_MATRIX with inputs and output in the same
 * form of it: blocks of 16 on both sides, or blocks of 32/64 on both sides with a right operand of at
 * most 4 stored bits; anything else is MX_ERR_UNSUPPORTED.  M must be a multiple of fo.block_rows.
 */
MX_API mx_status mx_gemm_q(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A_packed, mx_format fa,
                    const void* B_packed, mx_format fb, int32_t layout, const uint8_t* bias_mant,
                    const uint8_t* bias_exps, mx_format fbias, mx_format fo, void* out_packed, void* stream);

/*
 * Attention with both matrix products in MXInt (Fig. 1: the two products of the attention layer take
 * quantized operands; Section 3.2: an emulated operator computes on quantized inputs), per batch
 * entry (head) b, in one kernel:
 *     S  = Q K^T                     MXInt x MXInt product as in mx_gemm                      [Sq x Sk]
 *     P  = softmax(scale * S)        along the keys, in fp32
 *     P^ = MXInt(P, fp)              blocks of fp.block along the keys, the arithmetic of mx_quantize
 *     O  = P^ V                      MXInt x MXInt product as in mx_gemm                      [Sq x D]
 * Neither S nor P goes through memory (at 32 heads x 2048 x 2048 they are 537 MB each in fp32).
 * Q_packed: [batch][Sq x D] in format fq and K_packed: [batch][Sk x D] in fk, blocks along D.
 * Vt_packed: [batch][D x Sk] in fv: V quantized in blocks along the keys (mx_quantize with axis 0)
 *   and packed as a D x Sk matrix, i.e. the right operand mx_gemm would take for P V.
 * All three come from mx_pack / mx_quantize_pack (device, 256-byte aligned, padding as written there).
 * fp: format of P^ (fp.exp_bits == fv.exp_bits; fp.block is fv.block or a multiple of it); P^ is never
 *   stored.
 * O: device fp32, element (b, i, d) at O[b*o_batch_stride + i*ldo + d], ldo >= D.
 * Sk >= 1, Sk a multiple of fp.block, D a multiple of fq.block; scale finite.
 * Numerics: S and O accumulate in fp32 like mx_gemm.  P is computed in fp32 with the hardware's
 * exp2/log2 and differs from the exactly rounded softmax of S by a few 1e-6 relative (plus the
 * accumulation error of S times scale); a probability that close to a rounding tie of the quantizer,
 * or a block maximum that close to a power of two, can take the neighbouring mantissa or exponent.
 * Blocks of P^ whose elements are below 2^-126 count as zero.
 * Two-row blocks (block_rows = 2, the paper's own block shape, Section 3, the MASE IR example; Section 4.1) are taken for every tensor:
 * the packed operands carry their exponents inside the elements, so fq, fk, fv only need sizes that
 * hold whole pairs (Sq for Q, Sk for K, D for V^T); with fp.block_rows = 2 (Sq even) queries 2t and
 * 2t+1 share the exponent of each block of 16 probabilities.
 * Built for the form MX_LAYOUT_MATRIX takes with blocks of 16 (fq, fk, fv declare block 16), D <= 128,
 * and fp.block 16 or 32; anything else is MX_ERR_UNSUPPORTED.  That form carries the exponent inside
 * every element, so a tensor quantized with blocks of 32 or 64 enters it as the block-16 tensor of the
 * same values: mx_pack with block 16 and each exponent byte repeated for the runs of 16 it covers.
 */
MX_API mx_status mx_attention(int64_t batch, int64_t Sq, int64_t Sk, int64_t D, const void* Q_packed, mx_format fq,
                       const void* K_packed, mx_format fk, const void* Vt_packed, mx_format fv, mx_format fp,
                       float scale, int32_t layout, float* O, int64_t ldo, int64_t o_batch_stride, void* stream);

/*
 * Linear layer on fp32 activations for decode (M <= 8): quantizes x [M x K] with fx
 * on the fly (same arithmetic as mx_quantize, axis 1), then the product above
 * against B_packed [N x K] (Section 3.2: quantize the input, then the operator).  The result
 * equals mx_quantize + mx_pack + mx_gemm.  One launch when x is 16-byte aligned, row_stride a
 * multiple of 4 and fx.block_rows = 1: the weights are split over column groups and K slices so that
 * every compute unit streams its share once, each workgroup quantizes only its slice of x, and the
 * slices' partial sums are added in slice order by the last workgroup to finish (the result does not
 * depend on the order of arrival).  Otherwise two launches (quantize, then the decode product).
 * workspace: device buffer of mx_linear_workspace_bytes(M, K, N, fx, fb, layout) bytes, 256-byte
 *   aligned, caller-owned.  Its first 16384 bytes are arrival counters: they must be zero when the call
 *   starts and every call leaves them zero again, so a buffer that was zero-filled once serves call after
 *   call, also for other shapes it is large enough for.  The rest (partial sums, packed activations) needs
 *   no initial value and holds nothing of use afterwards.  Calls that may overlap in time (different
 *   streams) need a workspace each.
 * Y: device fp32, 4-byte aligned, element (m, n) at Y[m*ldy + n]; B_packed 256-byte aligned.
 * fx.block_rows = 2 (rows 2p and 2p+1 of x share their exponents) needs an even M.
 */
MX_API size_t mx_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, mx_format fx, mx_format fb,
                                        int32_t layout);
MX_API mx_status mx_linear(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx,
                    void* workspace, const void* B_packed, int64_t N, mx_format fb, int32_t layout,
                    float* Y, int64_t ldy, void* stream);

/*
 * mx_linear for callers that cannot allocate or pass device memory of their own for it: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, arithmetic, kernels and
 * results as mx_linear, without the workspace argument: the workspace is an array the library holds in
 * device memory itself, mx_linear_static_workspace_max() bytes (8 MiB) on every GPU the library is used on,
 * from load until the process ends.  The call allocates and frees nothing; it first clears the arrival
 * counters with a small kernel on `stream`.  MX_ERR_UNSUPPORTED when
 * mx_linear_workspace_bytes(M, K, N, fx, fb, layout) exceeds that size (the LLaMA-13B decode shapes need under
 * 4 MiB); MX_ERR_DEVICE when the array's address cannot be obtained.  The device of `stream` must be the
 * current device.  Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU
 * (different streams, different host threads) race -- give those mx_linear with a workspace each.
 */
MX_API size_t mx_linear_static_workspace_max(void);
MX_API mx_status mx_linear_static_workspace(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx,
                                     const void* B_packed, int64_t N, mx_format fb, int32_t layout,
                                     float* Y, int64_t ldy, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MX_H_ */
