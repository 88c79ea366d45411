/*
 * deepgemm_hip.h -- C ABI of the MI355X (gfx950) 2-bit lookup-table GEMM / convolution library.
 *
 * The method (DeepGEMM, arXiv 2304.09049): weights and activations are quantised to 2-bit codes,
 * every product of a weight level and an activation level is precomputed into a 16-entry table,
 * and a dot product is formed by fetching table entries and adding them (Sec. 3.1; Sec. 3
 * "LUT-16"; Algorithm 1).  Codes are packed four per byte (Sec. 3.1, Fig. 1).
 *
 * Notation: M = output channels / weight rows, N = output pixels x batch / activation rows,
 * K = reduction length (KH*KW*Cin for a convolution).  Wc[m][k], Ac[n][k] are codes in {0..3};
 * lw[4], la[4] are the level tables; LUT[4*w + a] = lw[w] * la[a].
 *
 * Conventions common to every call
 *   - Every function returns a dg_status, never throws, never aborts, never synchronises the
 *     device.  Arguments are validated on the host BEFORE anything is launched; on error nothing
 *     has been launched and dg_last_error() holds a description (thread-local, static storage).
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; all other pointers are host
 *     pointers.  Buffers must not alias.  The library allocates no device memory.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously on it; results are valid once the caller has synchronised.
 *   - The only library-owned object is dg_lut (a small host struct), freed by dg_lut_destroy.
 */
#ifndef DEEPGEMM_HIP_H
#define DEEPGEMM_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
/* the library is built with hidden visibility: only what this header declares is exported */
#pragma GCC visibility push(default)

typedef enum {
    DG_OK = 0,
    DG_ERR_NULL = 1,        /* a required pointer is NULL */
    DG_ERR_SHAPE = 2,       /* a dimension is <= 0, K or Cin is not a multiple of 4, empty output */
    DG_ERR_RANGE = 3,       /* a table entry does not fit its type, or K*max|LUT| could overflow int32 */
    DG_ERR_BUFFER = 4,      /* a buffer-size argument is too small */
    DG_ERR_UNSUPPORTED = 5, /* the requested kernel variant cannot run this shape / table */
    DG_ERR_HIP = 6          /* a HIP call failed; dg_last_error() carries hipGetErrorString */
} dg_status;

/* Name of a status code; static storage. */
const char *dg_status_string(dg_status s);
/* Detail of the calling thread's most recent failure ("" if none); thread-local static storage. */
const char *dg_last_error(void);

/* ---- the table (Sec. 3 "LUT-16": all 16 products w*a; Table 2: 2+2 index bits) ---------------- */

/* Entry type.  The paper's tables hold 8-bit entries and assume no overflow, with wider entries
 * "if required" (Sec. 3.2 "LUT Versions"); here the width is explicit and checked. */
typedef enum { DG_LUT_I8 = 0, DG_LUT_I16 = 1, DG_LUT_F32 = 2 } dg_lut_dtype;

typedef struct dg_lut dg_lut; /* opaque, immutable after build, usable from any thread */

/*
 * Build the table LUT[4*w + a] = levels_w[w] * levels_a[a] for codes w, a in {0..3}.
 * levels_w / levels_a: host arrays of 4 signed levels in code order (signed or unsigned, uniform or
 * not: Sec. 5.3).  Returns DG_ERR_RANGE if a product is not representable in `entry`
 * (int8: [-128,127]; int16 always fits), DG_ERR_NULL for NULL arguments.  *out owns the result.
 */
dg_status dg_build_lut(const int8_t levels_w[4], const int8_t levels_a[4], dg_lut_dtype entry,
                       dg_lut **out);
/*
 * The same table for b-bit codes, b = 2, 3 or 4 (Sec. 3.3 and Table 2: index b + b bits, 2^(2b) = 16 / 64 / 256
 * entries; the paper describes this scaling without implementing it).  levels_w / levels_a hold 2^b levels each;
 * entry index = (w << b) | a.  Tables with b > 2 run on the one-hot matrix-core kernels (int8 entries, Cin % 16 == 0)
 * or on the LDS kernel.  bits outside 2..4 -> DG_ERR_UNSUPPORTED.  dg_build_lut is the b = 2 case.
 */
dg_status dg_build_lut_bits(int32_t bits, const int8_t *levels_w, const int8_t *levels_a,
                            dg_lut_dtype entry, dg_lut **out);
/*
 * A 2-bit table given as such: entries[4*w + a] may be ANY 16 integers, not only products of two level vectors
 * (the table stores results, Sec. 5.3).  entry = DG_LUT_I8 checks every value against [-128, 127]
 * (DG_ERR_RANGE); DG_LUT_I16 accepts all.  The table kernels run such tables unchanged; the matrix-core
 * comparison kernel needs the level vectors and returns DG_ERR_UNSUPPORTED for them.
 */
dg_status dg_build_lut_entries(const int16_t entries[16], dg_lut_dtype entry, dg_lut **out);
/*
 * A 2-bit table of binary32 products of floating-point levels (non-uniform quantisation, Sec. 5.3):
 * entry[4*w + a] = levels_w[w] * levels_a[a], one binary32 multiply each.  With such a table dg_gemm_lut /
 * dg_conv2d_lut write binary32 to Cf_dev / Yf_dev (required; the int32 pointer is ignored): the sum of the
 * fetched entries taken in binary32, one addition per reduction position in ascending k (for a convolution kh,
 * then kw, then ci; taps outside the image skipped), starting from +0; then, if a scale is given, one multiply by
 * scale[m].  Only the LDS kernel runs binary32 tables (AUTO selects it).
 */
dg_status dg_build_lut_f32(const float levels_w[4], const float levels_a[4], dg_lut **out);
/* Copy the 16 binary32 entries of a DG_LUT_F32 table (DG_ERR_UNSUPPORTED for integer tables). */
dg_status dg_lut_entries_f32(const dg_lut *lut, float out[16]);
/* Code width of a table (0 for NULL). */
int32_t dg_lut_bits(const dg_lut *lut);
/* Copy all 2^(2b) entries, widened to int16; count must equal that number (else DG_ERR_BUFFER). */
dg_status dg_lut_entries_all(const dg_lut *lut, int16_t *out, int32_t count);
/* Copy the 16 entries of a 2-bit table, widened to int16, to host array out16 (out16[4*w + a]). */
dg_status dg_lut_entries(const dg_lut *lut, int16_t out16[16]);
/* Free a table; NULL is allowed. */
void dg_lut_destroy(dg_lut *lut);

/* ---- packing (Sec. 3.1: several 2-bit values shift/OR-ed into a byte; weights offline, ------
 *      activations at run time, Sec. 5.2) ------------------------------------------------------ */

/*
 * Bytes of a packed [rows][K] code matrix: rows*K/4.  0 if rows or K is negative or K % 4 != 0.
 * Packed ACTIVATION layout (public): code k of a row is in byte k/4 of that row, bits
 * [2*(k%4)+1 : 2*(k%4)]; rows are contiguous (K/4 bytes each).  For NHWC use rows = B*H*W, K = C.
 * Packed WEIGHT layout: private to the library (Sec. 3 allows an offline re-arrangement); only
 * its size, dg_packed_weight_bytes, is public.
 */
size_t dg_packed_activation_bytes(int64_t rows, int64_t K);
size_t dg_packed_weight_bytes(int64_t M, int64_t K);
/* Bytes of a packed [rows][K] matrix of b-bit codes: 3- and 4-bit codes sit two per byte, each in a 4-bit slot
 * (code k in byte k/2, bits [4*(k%2)+b-1 : 4*(k%2)]), for weights and activations alike.  0 on bad arguments. */
size_t dg_packed_bytes_bits(int64_t rows, int64_t K, int32_t bits);

/*
 * Pack codes (one uint8 per code, values 0..3; higher bits are masked off) four per byte.
 * codes_dev: device, [rows][K] row-major.  packed_dev: device, packed_bytes >= the size above
 * (else DG_ERR_BUFFER).  K % 4 != 0 or rows/K <= 0 -> DG_ERR_SHAPE.  Asynchronous on hip_stream.
 * A convolution's weights [Cout][KH][KW][Cin] are packed with M = Cout, K = KH*KW*Cin.
 */
dg_status dg_pack_weights(const uint8_t *codes_dev, int64_t M, int64_t K, void *packed_dev,
                          size_t packed_bytes, void *hip_stream);
dg_status dg_pack_activations(const uint8_t *codes_dev, int64_t N, int64_t K, void *packed_dev,
                              size_t packed_bytes, void *hip_stream);
/* Pack b-bit codes (weights or activations); b = 2 is dg_pack_activations.  K must be a multiple of the codes per
 * byte (4 for b = 2, else 2). */
dg_status dg_pack_codes_bits(const uint8_t *codes_dev, int64_t rows, int64_t K, int32_t bits, void *packed_dev,
                             size_t packed_bytes, void *hip_stream);

/*
 * Fused activation quantise + pack (the two stages that precede the table convolution in Sec. 5.4, with the
 * quantiser of Sec. 2.1, Eq. 1):
 *     q = clip(round(scale * x + zero_point), lo, lo + 3),   code = q - lo,   then packed as above.
 * x_dev: device, fp32 [N][K] (NHWC: N = B*H*W, K = C).  The decision is taken in binary32 exactly as written:
 * one multiply, one add (never fused), round-half-to-even, then the clip; NaN gives code 0.  lo = -2 for signed
 * codes, 0 for unsigned ones (any lo is accepted).  Errors and buffer rules as dg_pack_activations.
 */
dg_status dg_quantize_pack_activations(const float *x_dev, int64_t N, int64_t K, float scale,
                                       float zero_point, int32_t lo, void *packed_dev,
                                       size_t packed_bytes, void *hip_stream);

/*
 * The matching dequantise stage (Sec. 5.4 names it as the operator after the table convolution), for callers that
 * keep the int32 sums: out[r][c] = (float)acc[r][c] * scale_c[c] -- one int32 -> binary32 conversion (round to
 * nearest even) and one binary32 multiply, exactly what the scale epilogue of dg_gemm_lut / dg_conv2d_lut does.
 * acc_dev: device, int32 [rows][C] contiguous (NHWC: rows = B*OH*OW, C = Cout); scale_c_dev: device, fp32 [C];
 * out_dev: device, fp32 [rows][C] (may be acc_dev itself: element by element in place).
 * Errors: DG_ERR_NULL; DG_ERR_SHAPE if rows <= 0 or C <= 0.
 */
dg_status dg_dequantize(const int32_t *acc_dev, int64_t rows, int64_t C, const float *scale_c_dev,
                        float *out_dev, void *hip_stream);

/* ---- the kernels ------------------------------------------------------------------------------ */

/*
 * Which kernel runs.  AUTO picks the fastest table kernel for the shape.  The others exist for
 * A/B measurement:
 *   PERM     table rows held in registers, entries fetched with the byte-permute instruction
 *   LDS      table held in LDS, one indexed read per product (any shape the library accepts)
 *   MFMA_I8  NOT a table kernel: decodes codes to int8 levels and multiplies on the matrix cores (the
 *            one-hot kernels' frame with the selection replaced by a multiply); the measured comparison.
 *            Needs a table built from level vectors, 2-bit codes and Cin % 32 == 0
 *   SMALLN   table kernel for few activation rows: K split across lanes + wavefront reduction
 *   LUT65K   the paper's second table (Sec. 3 "LUT-65k"): one entry per (weight byte, activation byte) holding
 *            the dot product of the four code pairs, kept in LDS; one fetch per four products
 *   ONEHOT_MFMA  table kernel on the matrix cores: each int8 MFMA multiply is by a one-hot byte of the activation
 *            code, i.e. it selects one entry of the weight code's table row; any int8 entries, 2-, 3- or 4-bit
 *            codes (2^bits times the MFMA work of a plain int8 product); 2-bit tables with wider entries (up to
 *            32639) are selected from two int8 planes; needs Cin % 32 == 0 (2-bit) or % 16 (3-, 4-bit)
 *   ONEHOT_SMFMAC  the same selection on the sparse matrix instruction, at half the matrix work: a one-hot run
 *            of four bytes is 1-of-4 sparse, so the activation operand is a constant and its index register
 *            is the packed code word itself -- the instruction's index multiplexer does the table lookup;
 *            2-bit codes (Cin % 32 == 0; entries up to 32639, those beyond int8 as two planes under the
 *            same index registers) or 4-bit codes (Cin % 16 == 0, int8 entries); outputs whose stride-1
 *            axis is the channel axis (NHWC), or plain GEMMs without scale (run transposed)
 * A variant that cannot run the given shape or table returns DG_ERR_UNSUPPORTED.
 *
 * Test and measurement overrides.  They are honoured only when the environment variable DG_TEST_OVERRIDES is "1" at
 * the library's first call (that one is read once); otherwise none of them is looked at.  The results are the same
 * under any of them, only the kernel shape changes:
 *   DG_ONEHOT_PLAN   forces the one-hot kernels' shape: "split" (split-K kernel), "<wn>" (tile 32*wn columns wide,
 *                    wn = 1, 2, 4, 7) or "<wn>k<s>" (s = 2, 4 wavefronts sharing a tile); "44" is the comparison
 *                    kernel's 128 x 128 tile; "ws" the sparse-instruction kernel with stationary weight operands
 *                    (K = 64, 128, 256, and 512 on packed codes, without a filter window) whatever the size.  While it is set AUTO does not
 *                    move to the sparse-instruction forms on its own.
 *                    "fewn" the few-columns kernel on the sparse instruction (K % 256 == 0, no filter window).
 *                    "12", "14" (optionally followed by "k2" or "k4"), "16", "17", "24": the sparse-instruction kernel
 *                    that stages its operands through LDS (Cin % 128 == 0; "12" and "14" alone also
 *                    Cin % 128 == 64), tile 32 x 64, 32 x 128, 32 x 192, 32 x 224, 64 x 128;
 *                    the other values keep that kernel out.
 *   DG_ONEHOT_STAGED "0" keeps the staged kernel out altogether (the direct-load kernels run instead)
 *   DG_STAGED_BIAS   "0": the staged kernel multiplies with the table as it is; "1": with every entry raised by
 *                    minus the smallest one, the sums starting at the matching negative value (its default on
 *                    problems of 2MNK >= 2e10, where that lowers the matrix pipe's power draw)
 *   DG_WS_WAVES      target number of wavefronts of the "ws" kernel (default: one per SIMD)
 *   DG_WS_STRIDED    "0": AUTO never takes the "ws" kernel for a 1x1 layer with a stride, "1": for every such layer
 *   DG_WS_COUNT_STORES "0": the "ws" kernel that packs codes itself waits for its stores too whenever it waits for
 *                    staged codes (by default it counts the stores it has issued and lets them drain)
 *   DG_FEWN_WAVES    wavefronts per workgroup of the "fewn" kernel (1..8)
 *   DG_FEWN_ROWS     weight rows per workgroup of the "fewn" kernel (16 or 32)
 *   DG_ONEHOT_WAVES  target number of wavefronts of the split-K kernel (default 2048; 3072 for K = 2304 ... 4608)
 *   DG_ONEHOT_SHARE_BELOW  tiles per SIMD from which the planner does not let wavefronts share a tile (default 2)
 *   DG_ONEHOT_CH2_MAX  the dense instruction's split-K kernel walks K in chunks of 64 positions instead of 128 where K
 *                    has at most this many chunks of 128 and twice as many wavefronts per tile are wanted (default 4)
 *   DG_ONEHOT_CH2_SMAX and where that gives a tile more wavefronts, up to this many (default 12)
 *   DG_ONEHOT_CODES_TILED "0": the one-call entry points never use the tiled kernel that packs the codes itself,
 *                    "1": wherever it applies (default: where it was measured shorter than two kernels)
 *   DG_ONEHOT_CODES_SPARSE "0": that kernel on the dense instruction only, "1": on the sparse one wherever the output's
 *                    channel axis is contiguous (the default)
 *   DG_PERM_PLAN     index of the permute kernel's tile shape
 */
typedef enum {
    DG_KERNEL_AUTO = 0,
    DG_KERNEL_PERM = 1,
    DG_KERNEL_LDS = 2,
    DG_KERNEL_MFMA_I8 = 3,
    DG_KERNEL_SMALLN = 4,
    DG_KERNEL_LUT65K = 5,
    DG_KERNEL_ONEHOT_MFMA = 6,
    DG_KERNEL_ONEHOT_SMFMAC = 7
} dg_kernel;

/*
 * GEMM by table lookup (Algorithm 1 over all rows):
 *     C[m][n] = sum_{k<K} LUT[4*Wc[m][k] + Ac[n][k]]          (exact, int32)
 * Wp_dev: weights packed by dg_pack_weights(M, K).  Ap_dev: activations packed by
 * dg_pack_activations(N, K) (or any buffer in the public activation layout).
 * Output, one of:
 *   scale_m_dev == NULL : C_dev[m*stride_cm + n*stride_cn] = sum (int32; strides in elements,
 *                         both non-zero, the M*N addresses distinct)
 *   scale_m_dev != NULL : Cf_dev[m*stride_cm + n*stride_cn] = (float)sum * scale_m_dev[m]
 *                         (int32 -> binary32 round-to-nearest-even, then ONE binary32 multiply:
 *                         the dequantisation stage of Sec. 5.4); C_dev is ignored and may be NULL.
 * Errors: DG_ERR_NULL; DG_ERR_SHAPE (M, N, K <= 0 or K % 4 != 0); DG_ERR_RANGE if
 * K * max|LUT| >= 2^31.
 */
dg_status dg_gemm_lut(const dg_lut *lut, const void *Wp_dev, const void *Ap_dev, int64_t M,
                      int64_t N, int64_t K, int32_t *C_dev, int64_t stride_cm, int64_t stride_cn,
                      const float *scale_m_dev, float *Cf_dev, dg_kernel variant,
                      void *hip_stream);

/* Convolution geometry; dilation 1, groups 1. */
typedef struct {
    int32_t B, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w;
} dg_conv_desc;

/* Output height/width: floor((in + 2*pad - k) / stride) + 1, or 0 if the kernel does not fit. */
int64_t dg_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad);

/*
 * NHWC convolution by table lookup with implicit im2col (no expanded matrix is ever formed):
 *     Y[b][oh][ow][co] = sum_{kh,kw,ci} LUT[4*Wc[co][kh][kw][ci] + Xc[b][ih][iw][ci]],
 *     ih = oh*stride_h - pad_h + kh, iw = ow*stride_w - pad_w + kw;
 *     taps outside the image add 0 to the sum whatever the level tables are.
 * Wp_dev: dg_pack_weights(codes [Cout][KH][KW][Cin], M = Cout, K = KH*KW*Cin).
 * Xp_dev: dg_pack_activations(codes [B][H][W][Cin], N = B*H*W, K = Cin).
 * Output NHWC [B][OH][OW][Cout], contiguous: Y_dev (int32) when scale_cout_dev == NULL, else
 * Yf_dev[...][co] = (float)sum * scale_cout_dev[co] (as in dg_gemm_lut) and Y_dev is ignored.
 * Errors: DG_ERR_NULL; DG_ERR_SHAPE (a dimension <= 0, pad < 0, Cin % 4 != 0, OH or OW <= 0);
 * DG_ERR_RANGE if KH*KW*Cin * max|LUT| >= 2^31.
 */
dg_status dg_conv2d_lut(const dg_lut *lut, const void *Wp_dev, const void *Xp_dev,
                        const dg_conv_desc *desc, int32_t *Y_dev, const float *scale_cout_dev,
                        float *Yf_dev, dg_kernel variant, void *hip_stream);

/*
 * The run-time packing stage (Sec. 5.2) and the convolution as ONE call, from activations that are still one code
 * per byte: Xc_dev is device memory, [B][H][W][Cin] uint8, values below 2^bits (higher bits of 2-bit codes are
 * masked off, as dg_pack_activations does), 16-byte aligned for the fused form.  Where a second kernel launch
 * costs a good part of the layer itself the kernel reads the codes as they are and packs them while loading -- one
 * launch, and Xp_work_dev is not touched.  Those are, for 2-bit codes: the layers the library runs on the one-hot
 * split-K kernel (Cin % 32 == 0, K <= 3072; variant ONEHOT_MFMA, or AUTO while Cout is small enough that packing
 * once per 32 output channels costs less than the launch); layers of a few microseconds on the one-hot tiled
 * kernel's 64 x 32 and 64 x 64 tiles (Cin % 64 == 0; AUTO, ONEHOT_MFMA or ONEHOT_SMFMAC -- on the sparse instruction
 * where the output's channel axis is contiguous unless ONEHOT_MFMA is named -- up to about 2 * 10^9 table operations,
 * more where there is much to pack or Cin % 128 != 0); the layers of the stationary-weight
 * kernel (K = 64, 128, 256 without a filter window; AUTO or ONEHOT_SMFMAC); and the few-columns kernel (AUTO or
 * SMALLN).  Every other layer is packed into
 * Xp_work_dev (device, work_bytes >= dg_packed_bytes_bits(B*H*W, Cin, bits), else DG_ERR_BUFFER; DG_ERR_NULL if it
 * is needed and NULL) by the packing kernel and then run as dg_conv2d_lut would run it, on the same stream (of a
 * 1x1 layer with a stride and no padding only the pixels it reads are packed, [B][OH][OW][Cin/4] at the start of the
 * buffer, and the layer runs on those without the stride).
 * Outputs, scale, variant and the other errors as dg_conv2d_lut; the results are identical to dg_pack_activations
 * followed by dg_conv2d_lut.  dg_conv_codes_kernel_name names the convolution kernel that would run: "codes_..."
 * for the fused form, else dg_conv_kernel_name's answer.
 */
dg_status dg_conv2d_lut_codes(const dg_lut *lut, const void *Wp_dev, const uint8_t *Xc_dev,
                              const dg_conv_desc *desc, void *Xp_work_dev, size_t work_bytes,
                              int32_t *Y_dev, const float *scale_cout_dev, float *Yf_dev,
                              dg_kernel variant, void *hip_stream);
const char *dg_conv_codes_kernel_name(const dg_lut *lut, const dg_conv_desc *desc, dg_kernel variant);
/*
 * dg_conv2d_lut_codes for callers that cannot allocate device memory and so have no work buffer to hand over (code
 * under HIP graph capture, serving loops, harnesses that forbid hipMalloc): the packed activations are staged in a
 * buffer the library holds in static device memory, dg_static_work_bytes() = 8 MiB per GPU (33 554 432 2-bit codes),
 * kept until the process ends.  The call allocates and frees nothing.  Arguments, results and errors as
 * dg_conv2d_lut_codes without Xp_work_dev / work_bytes; a layer whose packed activations exceed the staging buffer
 * returns DG_ERR_BUFFER (nothing launched).  The staging buffer is written before it is read on every call (nothing
 * needs clearing), and it is shared by all calls on a GPU: calls that overlap in time on one GPU (two streams, two
 * threads) race on it -- serialise them, or use dg_conv2d_lut_codes with buffers of their own.
 */
size_t dg_static_work_bytes(void);
dg_status dg_conv2d_lut_codes_static(const dg_lut *lut, const void *Wp_dev, const uint8_t *Xc_dev,
                                     const dg_conv_desc *desc, int32_t *Y_dev, const float *scale_cout_dev,
                                     float *Yf_dev, dg_kernel variant, void *hip_stream);
/*
 * The same for a GEMM: Ac_dev is device memory, [N][K] uint8 codes; Ap_work_dev (work_bytes >=
 * dg_packed_bytes_bits(N, K, bits)) is used when the packing is not fused (K % 32 != 0, a large problem, another
 * variant, 3- or 4-bit codes: the conditions above with Cin = K).  Outputs, strides, scale and the other errors as dg_gemm_lut.
 */
dg_status dg_gemm_lut_codes(const dg_lut *lut, const void *Wp_dev, const uint8_t *Ac_dev, int64_t M, int64_t N,
                            int64_t K, void *Ap_work_dev, size_t work_bytes, int32_t *C_dev, int64_t stride_cm,
                            int64_t stride_cn, const float *scale_m_dev, float *Cf_dev, dg_kernel variant,
                            void *hip_stream);
const char *dg_gemm_codes_kernel_name(const dg_lut *lut, int64_t M, int64_t N, int64_t K, dg_kernel variant);

/*
 * A whole layer in one kernel: table convolution, dequantise, re-quantise (Sec. 2.1, Eq. 1) and pack -- the stages
 * Sec. 5.4 lists after one another -- so that the output is the packed activation tensor of the next layer:
 *     y    = (float)sum * scale_cout_dev[co]                               (as in dg_conv2d_lut)
 *     code = clip(round(q_scale * y + q_zero), lo, lo + 3) - lo            (as in dg_quantize_pack_activations)
 * packed_out_dev: device, dg_packed_activation_bytes(B*OH*OW, Cout) bytes, the public layout ([pixel][Cout/4]).
 * Every decision is taken in binary32, operation by operation, so the result equals dg_conv2d_lut followed by
 * dg_quantize_pack_activations bit for bit.  Needs Cout % 4 == 0 and a table and shape the one-hot matrix-core
 * kernel accepts (variant AUTO, ONEHOT_MFMA or ONEHOT_SMFMAC; otherwise DG_ERR_UNSUPPORTED -- run the two calls
 * instead).
 * Errors: as dg_conv2d_lut; DG_ERR_SHAPE if Cout % 4 != 0; DG_ERR_BUFFER if packed_bytes is too small.
 */
dg_status dg_conv2d_lut_requant(const dg_lut *lut, const void *Wp_dev, const void *Xp_dev,
                                const dg_conv_desc *desc, const float *scale_cout_dev, float q_scale,
                                float q_zero, int32_t lo, void *packed_out_dev, size_t packed_bytes,
                                dg_kernel variant, void *hip_stream);

/* Measurement aid: launch a kernel that does nothing, `blocks` workgroups of `threads` threads (a multiple of 64,
 * at most 1024), on `hip_stream`.  Its duration is what a launch of that shape costs before any work is done, the
 * floor under the duration of a small layer's kernel.  Errors: DG_ERR_SHAPE. */
dg_status dg_launch_empty(int64_t blocks, int32_t threads, void *hip_stream);

/* Name of the kernel that AUTO would pick (or that `variant` maps to) for this GEMM / convolution
 * shape; static storage.  For reports only. */
const char *dg_gemm_kernel_name(const dg_lut *lut, int64_t M, int64_t N, int64_t K,
                                dg_kernel variant);
const char *dg_conv_kernel_name(const dg_lut *lut, const dg_conv_desc *desc, dg_kernel variant);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* DEEPGEMM_HIP_H */
