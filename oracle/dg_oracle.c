/*
 * CPU oracle for the 2-bit lookup-table GEMM / convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of WHAT the GPU library must compute.  It is not a fallback: nothing in the
 * product path may call it.  It shares no code, header, table or constant with
 * the HIP library.
 *
 * What is computed (paper, Sec. 3 "LUT-16": the table holds every product w*a
 * of a weight level and an activation level, and a dot product is the sum of
 * the fetched products).  Because the table stores exact products, the result
 * of the table method has a plain definition, and the oracle is that
 * definition written out: decode each 2-bit code to its integer level,
 * multiply, and sum.  No table is built here, nothing is packed, nothing is
 * blocked, fused or reordered.
 *
 *   GEMM : C[m][n] = sum_k  lw[Wc[m][k]] * la[Ac[n][k]]
 *   CONV : Y[b][oh][ow][co] = sum_{kh,kw,ci} lw[Wc[co][kh][kw][ci]] * la[Xc[b][ih][iw][ci]]
 *          ih = oh*stride_h - pad_h + kh,  iw = ow*stride_w - pad_w + kw,
 *          taps that fall outside the image are left out of the sum
 *          (the feature map is zero-padded in the real domain; Sec. 2.1 speaks
 *          only of "padded activations", the value is this build's reading).
 *   EPI  : Yf = (float)Y * scale[co]   (Sec. 5.4: dequantisation is a separate,
 *          cheap stage; one binary32 multiply, no fused multiply-add).
 *
 * Inputs are UNPACKED codes, one uint8 per code, plus the two level tables of
 * `nlev` entries each: nlev = 4 for the paper's 2-bit kernels, 8 or 16 for the
 * 3- and 4-bit extension it describes (Sec. 3.3, Table 2).  Sums are taken in
 * int64 and narrowed with a check.
 *
 * Return codes: 0 ok, 1 a code was >= nlev, 2 a sum does not fit int32,
 *               3 bad shape.
 *
 * OpenMP is used on the outermost output loop only; it changes no sum.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int dgo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void dgo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* One dot product over K codes on decoded levels.  Returns 1 on a bad code. */
static int dot_levels(const uint8_t *w, const uint8_t *a, int64_t K,
                      const int32_t *lw, const int32_t *la, int nlev, int64_t *out)
{
    int64_t s = 0;
    for (int64_t k = 0; k < K; ++k) {
        if (w[k] >= nlev || a[k] >= nlev) return 1;
        s += (int64_t)lw[w[k]] * (int64_t)la[a[k]];
    }
    *out = s;
    return 0;
}

/* GEMM.  Wc is [M][K], Ac is [N][K], C is [M][N] row-major. */
int dgo_gemm(const uint8_t *Wc, const uint8_t *Ac,
             const int32_t *lw, const int32_t *la, int nlev,
             int64_t M, int64_t N, int64_t K, int32_t *C)
{
    if (M < 0 || N < 0 || K < 0 || nlev < 1 || nlev > 16) return 3;
    int err = 0;
#pragma omp parallel for schedule(static) reduction(max : err)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s;
            if (dot_levels(Wc + m * K, Ac + n * K, K, lw, la, nlev, &s)) {
                if (err < 1) err = 1;
                continue;
            }
            if (s > INT32_MAX || s < INT32_MIN) {
                if (err < 2) err = 2;
                continue;
            }
            C[m * N + n] = (int32_t)s;
        }
    }
    return err;
}

/* GEMM at a list of sampled output positions: out[i] = C[ms[i]][ns[i]]. */
int dgo_gemm_sampled(const uint8_t *Wc, const uint8_t *Ac,
                     const int32_t *lw, const int32_t *la, int nlev,
                     int64_t M, int64_t N, int64_t K,
                     const int64_t *ms, const int64_t *ns, int64_t count,
                     int32_t *out)
{
    if (M < 0 || N < 0 || K < 0 || count < 0 || nlev < 1 || nlev > 16) return 3;
    int err = 0;
#pragma omp parallel for schedule(static) reduction(max : err)
    for (int64_t i = 0; i < count; ++i) {
        int64_t m = ms[i], n = ns[i], s;
        if (m < 0 || m >= M || n < 0 || n >= N) {
            if (err < 3) err = 3;
            continue;
        }
        if (dot_levels(Wc + m * K, Ac + n * K, K, lw, la, nlev, &s)) {
            if (err < 1) err = 1;
            continue;
        }
        if (s > INT32_MAX || s < INT32_MIN) {
            if (err < 2) err = 2;
            continue;
        }
        out[i] = (int32_t)s;
    }
    return err;
}

/* Output extent of a convolution along one axis (floor division). */
int64_t dgo_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad)
{
    if (stride <= 0) return -1;
    int64_t span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* One output element of the direct convolution. */
static int conv_point(const uint8_t *Wc, const uint8_t *Xc,
                      const int32_t *lw, const int32_t *la, int nlev,
                      int64_t H, int64_t W, int64_t Cin,
                      int64_t KH, int64_t KW,
                      int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                      int64_t b, int64_t oh, int64_t ow, int64_t co,
                      int64_t *out)
{
    int64_t s = 0;
    for (int64_t kh = 0; kh < KH; ++kh) {
        int64_t ih = oh * sh - ph + kh;
        if (ih < 0 || ih >= H) continue;
        for (int64_t kw = 0; kw < KW; ++kw) {
            int64_t iw = ow * sw - pw + kw;
            if (iw < 0 || iw >= W) continue;
            const uint8_t *x = Xc + ((b * H + ih) * W + iw) * Cin;
            const uint8_t *w = Wc + ((co * KH + kh) * KW + kw) * Cin;
            for (int64_t ci = 0; ci < Cin; ++ci) {
                if (w[ci] >= nlev || x[ci] >= nlev) return 1;
                s += (int64_t)lw[w[ci]] * (int64_t)la[x[ci]];
            }
        }
    }
    *out = s;
    return 0;
}

/*
 * Direct NHWC convolution.  Xc is [B][H][W][Cin], Wc is [Cout][KH][KW][Cin],
 * Y is [B][OH][OW][Cout].  Dilation 1, groups 1.
 */
int dgo_conv2d(const uint8_t *Wc, const uint8_t *Xc,
               const int32_t *lw, const int32_t *la, int nlev,
               int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
               int64_t KH, int64_t KW, int64_t sh, int64_t sw,
               int64_t ph, int64_t pw, int32_t *Y)
{
    if (B < 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 ||
        KW <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0 || nlev < 1 || nlev > 16)
        return 3;
    const int64_t OH = dgo_conv_out_dim(H, KH, sh, ph);
    const int64_t OW = dgo_conv_out_dim(W, KW, sw, pw);
    int err = 0;
#pragma omp parallel for schedule(static) reduction(max : err)
    for (int64_t row = 0; row < B * OH; ++row) {
        const int64_t b = row / OH, oh = row % OH;
        for (int64_t ow = 0; ow < OW; ++ow) {
            for (int64_t co = 0; co < Cout; ++co) {
                int64_t s;
                if (conv_point(Wc, Xc, lw, la, nlev, H, W, Cin, KH, KW, sh, sw, ph,
                               pw, b, oh, ow, co, &s)) {
                    if (err < 1) err = 1;
                    continue;
                }
                if (s > INT32_MAX || s < INT32_MIN) {
                    if (err < 2) err = 2;
                    continue;
                }
                Y[((b * OH + oh) * OW + ow) * Cout + co] = (int32_t)s;
            }
        }
    }
    return err;
}

/* Convolution at sampled output positions; pos[i] is a flat NHWC output index. */
int dgo_conv2d_sampled(const uint8_t *Wc, const uint8_t *Xc,
                       const int32_t *lw, const int32_t *la, int nlev,
                       int64_t B, int64_t H, int64_t W, int64_t Cin,
                       int64_t Cout, int64_t KH, int64_t KW, int64_t sh,
                       int64_t sw, int64_t ph, int64_t pw,
                       const int64_t *pos, int64_t count, int32_t *out)
{
    if (B < 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 ||
        KW <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0 || count < 0 || nlev < 1 || nlev > 16)
        return 3;
    const int64_t OH = dgo_conv_out_dim(H, KH, sh, ph);
    const int64_t OW = dgo_conv_out_dim(W, KW, sw, pw);
    const int64_t total = B * OH * OW * Cout;
    int err = 0;
#pragma omp parallel for schedule(static) reduction(max : err)
    for (int64_t i = 0; i < count; ++i) {
        int64_t p = pos[i], s;
        if (p < 0 || p >= total) {
            if (err < 3) err = 3;
            continue;
        }
        const int64_t co = p % Cout;
        const int64_t ow = (p / Cout) % OW;
        const int64_t oh = (p / (Cout * OW)) % OH;
        const int64_t b = p / (Cout * OW * OH);
        if (conv_point(Wc, Xc, lw, la, nlev, H, W, Cin, KH, KW, sh, sw, ph, pw, b,
                       oh, ow, co, &s)) {
            if (err < 1) err = 1;
            continue;
        }
        if (s > INT32_MAX || s < INT32_MIN) {
            if (err < 2) err = 2;
            continue;
        }
        out[i] = (int32_t)s;
    }
    return err;
}

/*
 * Per-channel dequantisation epilogue: out[r][c] = (float)acc[r][c] * scale[c],
 * acc and out are [rows][channels] with channels fastest (NHWC).
 * int32 -> binary32 conversion rounds to nearest even (C default), then one
 * binary32 multiply.  Build with -ffp-contract=off.
 */
void dgo_scale_epilogue_nhwc(const int32_t *acc, const float *scale,
                             int64_t rows, int64_t channels, float *out)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < channels; ++c) {
            volatile float f = (float)acc[r * channels + c];
            out[r * channels + c] = f * scale[c];
        }
}

/* Same epilogue for a GEMM result stored [M][N]: the scale belongs to row m. */
void dgo_scale_epilogue_rows(const int32_t *acc, const float *scale,
                             int64_t M, int64_t N, float *out)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            volatile float f = (float)acc[m * N + n];
            out[m * N + n] = f * scale[m];
        }
}

/*
 * Uniform quantisation of activations to 2-bit codes (paper Sec. 2.1, Eq. 1):
 *     x_q = clip(round(s * x + z), lo, hi),        code = x_q - lo   (so that code 0 is the lowest level)
 * The printed equation has its closing parenthesis misplaced and its value set ends at 2^(b-1); it is read as
 * clip(round(s*x + z), -2^(b-1), 2^(b-1) - 1) for signed data, and the range [lo, hi] = [lo, lo + 3] is an
 * argument here so that unsigned (post-ReLU) activations use [0, 3].  The paper does not say how ties round;
 * round-half-to-even is taken (the IEEE default, rintf).  The decision is taken in binary32, the precision of
 * the input: t = s * x (one rounding), t + z (one rounding), rintf, compare.  NaN maps to code of `lo`
 * (every comparison with NaN is false, so it falls through the clip as the lower bound).
 * Returns 3 for a bad range.
 */
#include <math.h>
int dgo_quantize_codes(const float *x, int64_t count, float s, float z, int32_t lo, int32_t hi,
                       uint8_t *codes)
{
    if (count < 0 || hi - lo != 3) return 3;
    for (int64_t i = 0; i < count; ++i) {
        volatile float t = s * x[i];
        volatile float u = t + z;
        const float r = rintf(u);
        int32_t q = lo;
        if (r > (float)lo) q = r >= (float)hi ? hi : (int32_t)r;
        codes[i] = (uint8_t)(q - lo);
    }
    return 0;
}

/*
 * Table-defined variants.  Sec. 5.3 stresses that the table stores RESULTS, so it may hold anything: products of
 * non-uniform levels, signed or unsigned, integer or floating point.  A table need not even factor into level
 * vectors.  For such tables the result has this plain definition:
 *     C[m][n] = sum_k  T[ nlev * Wc[m][k] + Ac[n][k] ]
 * Integer tables: exact (int64 sum, checked).  binary32 tables: the sum is taken in binary32, one addition per
 * reduction position in ascending order of k (for a convolution: kh, then kw, then ci, taps outside the image
 * skipped), starting from +0.0f -- the order is part of the definition because float addition does not commute
 * with rounding.  The paper gives no order; this one is this build's reading.
 */
int dgo_gemm_table(const uint8_t *Wc, const uint8_t *Ac, const int32_t *table, int nlev,
                   int64_t M, int64_t N, int64_t K, int32_t *C)
{
    if (M < 0 || N < 0 || K < 0 || nlev < 1 || nlev > 16) return 3;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) {
                const uint8_t w = Wc[m * K + k], a = Ac[n * K + k];
                if (w >= nlev || a >= nlev) return 1;
                s += table[nlev * w + a];
            }
            if (s > INT32_MAX || s < INT32_MIN) return 2;
            C[m * N + n] = (int32_t)s;
        }
    return 0;
}

int dgo_conv2d_table(const uint8_t *Wc, const uint8_t *Xc, const int32_t *table, int nlev,
                     int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                     int64_t KH, int64_t KW, int64_t sh, int64_t sw, int64_t ph, int64_t pw, int32_t *Y)
{
    if (B < 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || sh <= 0 || sw <= 0 ||
        ph < 0 || pw < 0 || nlev < 1 || nlev > 16)
        return 3;
    const int64_t OH = dgo_conv_out_dim(H, KH, sh, ph), OW = dgo_conv_out_dim(W, KW, sw, pw);
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oh = 0; oh < OH; ++oh)
            for (int64_t ow = 0; ow < OW; ++ow)
                for (int64_t co = 0; co < Cout; ++co) {
                    int64_t s = 0;
                    for (int64_t kh = 0; kh < KH; ++kh) {
                        const int64_t ih = oh * sh - ph + kh;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            const int64_t iw = ow * sw - pw + kw;
                            if (iw < 0 || iw >= W) continue;
                            for (int64_t ci = 0; ci < Cin; ++ci) {
                                const uint8_t w = Wc[((co * KH + kh) * KW + kw) * Cin + ci];
                                const uint8_t a = Xc[((b * H + ih) * W + iw) * Cin + ci];
                                if (w >= nlev || a >= nlev) return 1;
                                s += table[nlev * w + a];
                            }
                        }
                    }
                    if (s > INT32_MAX || s < INT32_MIN) return 2;
                    Y[((b * OH + oh) * OW + ow) * Cout + co] = (int32_t)s;
                }
    return 0;
}

/* table[4*w + a] = lw[w] * la[a], one binary32 multiply each */
void dgo_build_lut_f32(const float lw[4], const float la[4], float table[16])
{
    for (int w = 0; w < 4; ++w)
        for (int a = 0; a < 4; ++a) {
            volatile float p = lw[w] * la[a];
            table[4 * w + a] = p;
        }
}

int dgo_gemm_table_f32(const uint8_t *Wc, const uint8_t *Ac, const float table[16],
                       int64_t M, int64_t N, int64_t K, float *C)
{
    if (M < 0 || N < 0 || K < 0) return 3;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            volatile float s = 0.0f;
            for (int64_t k = 0; k < K; ++k) {
                const uint8_t w = Wc[m * K + k], a = Ac[n * K + k];
                if (w > 3 || a > 3) return 1;
                s = s + table[4 * w + a];
            }
            C[m * N + n] = s;
        }
    return 0;
}

int dgo_conv2d_table_f32(const uint8_t *Wc, const uint8_t *Xc, const float table[16],
                         int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                         int64_t KH, int64_t KW, int64_t sh, int64_t sw, int64_t ph, int64_t pw, float *Y)
{
    if (B < 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || sh <= 0 || sw <= 0 ||
        ph < 0 || pw < 0)
        return 3;
    const int64_t OH = dgo_conv_out_dim(H, KH, sh, ph), OW = dgo_conv_out_dim(W, KW, sw, pw);
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oh = 0; oh < OH; ++oh)
            for (int64_t ow = 0; ow < OW; ++ow)
                for (int64_t co = 0; co < Cout; ++co) {
                    volatile float s = 0.0f;
                    for (int64_t kh = 0; kh < KH; ++kh) {
                        const int64_t ih = oh * sh - ph + kh;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            const int64_t iw = ow * sw - pw + kw;
                            if (iw < 0 || iw >= W) continue;
                            for (int64_t ci = 0; ci < Cin; ++ci) {
                                const uint8_t w = Wc[((co * KH + kh) * KW + kw) * Cin + ci];
                                const uint8_t a = Xc[((b * H + ih) * W + iw) * Cin + ci];
                                if (w > 3 || a > 3) return 1;
                                s = s + table[4 * w + a];
                            }
                        }
                    }
                    Y[((b * OH + oh) * OW + ow) * Cout + co] = s;
                }
    return 0;
}
