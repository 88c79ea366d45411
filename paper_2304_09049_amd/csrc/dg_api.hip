// Host side of the C ABI: argument validation, table construction, kernel selection.
// Every entry point validates on the host before launching anything and never synchronises.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "dg_common.h"

// Staging for packed activations owned by the library, for dg_conv2d_lut_codes_static: callers that cannot allocate
// (HIP graph capture, serving loops) have no work buffer to pass.  8 MiB hold 33 554 432 2-bit codes; every GPU the
// library runs on keeps its own copy of the array until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress: kernels and copies take the per-device address kept in g_static_work.
#define DG_STATIC_WORK_BYTES ((size_t)8 << 20)
static __device__ __align__(256) unsigned char scratch[DG_STATIC_WORK_BYTES];

namespace {
thread_local char g_error[512] = "";

__global__ void empty_kernel() {}

constexpr int MAX_DEVICES = 64;
void *g_static_work[MAX_DEVICES];       // device address of `scratch` on each device, looked up at first use
std::mutex g_static_work_mutex;
}

dg_status dg_fail(dg_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return s;
}

const char *dg_override(const char *name)
{
    static const bool enabled = [] {
        const char *e = getenv("DG_TEST_OVERRIDES");
        return e != nullptr && e[0] == '1' && e[1] == 0;
    }();
    return enabled ? getenv(name) : nullptr;
}

int dg_simd_count()
{
    static const int simds = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;                                      // (no device to ask: the MI355X figure)
        return 4 * cus;
    }();
    return simds;
}

dg_status dg_check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return dg_fail(DG_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return DG_OK;
}

extern "C" {

const char *dg_status_string(dg_status s)
{
    switch (s) {
    case DG_OK: return "DG_OK";
    case DG_ERR_NULL: return "DG_ERR_NULL";
    case DG_ERR_SHAPE: return "DG_ERR_SHAPE";
    case DG_ERR_RANGE: return "DG_ERR_RANGE";
    case DG_ERR_BUFFER: return "DG_ERR_BUFFER";
    case DG_ERR_UNSUPPORTED: return "DG_ERR_UNSUPPORTED";
    case DG_ERR_HIP: return "DG_ERR_HIP";
    }
    return "DG_ERR_UNKNOWN";
}

const char *dg_last_error(void) { return g_error; }

// Sec. 3 "LUT-16": the table holds all possible results of w*a; index = weight code (high two
// bits) concatenated with activation code (low two bits).
dg_status dg_build_lut(const int8_t levels_w[4], const int8_t levels_a[4], dg_lut_dtype entry,
                       dg_lut **out)
{
    return dg_build_lut_bits(2, levels_w, levels_a, entry, out);
}

// Table 2: b + b index bits, 2^(2b) entries (16, 64, 256 for b = 2, 3, 4).
dg_status dg_build_lut_bits(int32_t bits, const int8_t *levels_w, const int8_t *levels_a,
                            dg_lut_dtype entry, dg_lut **out)
{
    if (!levels_w || !levels_a || !out) return dg_fail(DG_ERR_NULL, "dg_build_lut: NULL argument");
    if (bits < 2 || bits > 4) return dg_fail(DG_ERR_UNSUPPORTED, "dg_build_lut: %d-bit codes (2, 3 or 4)", bits);
    if (entry != DG_LUT_I8 && entry != DG_LUT_I16)
        return dg_fail(DG_ERR_UNSUPPORTED, "dg_build_lut: unknown entry type %d", (int)entry);
    const int nlev = 1 << bits;
    dg_lut t;
    memset(&t, 0, sizeof(t));
    t.bits = bits;
    t.dtype = entry;
    t.separable = true;
    t.min_entry = INT32_MAX;
    t.max_entry = INT32_MIN;
    for (int w = 0; w < nlev; ++w) {
        t.levels_w[w] = levels_w[w];
        t.levels_a[w] = levels_a[w];
    }
    for (int w = 0; w < nlev; ++w)
        for (int a = 0; a < nlev; ++a) {
            const int32_t prod = (int32_t)levels_w[w] * (int32_t)levels_a[a];
            if (entry == DG_LUT_I8 && (prod < -128 || prod > 127))
                return dg_fail(DG_ERR_RANGE,
                               "dg_build_lut: product %d of levels_w[%d]=%d and levels_a[%d]=%d "
                               "does not fit an int8 table entry",
                               prod, w, (int)levels_w[w], a, (int)levels_a[a]);
            t.entry[(w << bits) | a] = (int16_t)prod;   // |prod| <= 128*128 = 16384 always fits int16
            if (prod < t.min_entry) t.min_entry = prod;
            if (prod > t.max_entry) t.max_entry = prod;
        }
    t.max_abs = t.max_entry > -t.min_entry ? t.max_entry : -t.min_entry;
    dg_lut *p = new (std::nothrow) dg_lut(t);
    if (!p) return dg_fail(DG_ERR_BUFFER, "dg_build_lut: out of host memory");
    *out = p;
    return DG_OK;
}

dg_status dg_lut_entries(const dg_lut *lut, int16_t out16[16])
{
    if (!lut || !out16) return dg_fail(DG_ERR_NULL, "dg_lut_entries: NULL argument");
    if (lut->bits != 2) return dg_fail(DG_ERR_UNSUPPORTED, "dg_lut_entries: a %d-bit table has more than 16 entries", lut->bits);
    if (lut->dtype == DG_LUT_F32) return dg_fail(DG_ERR_UNSUPPORTED, "dg_lut_entries: a binary32 table (use dg_lut_entries_f32)");
    for (int i = 0; i < 16; ++i) out16[i] = lut->entry[i];
    return DG_OK;
}

int32_t dg_lut_bits(const dg_lut *lut) { return lut ? lut->bits : 0; }

dg_status dg_build_lut_entries(const int16_t entries[16], dg_lut_dtype entry, dg_lut **out)
{
    if (!entries || !out) return dg_fail(DG_ERR_NULL, "dg_build_lut_entries: NULL argument");
    if (entry != DG_LUT_I8 && entry != DG_LUT_I16)
        return dg_fail(DG_ERR_UNSUPPORTED, "dg_build_lut_entries: entry type %d is not an integer type", (int)entry);
    dg_lut t;
    memset(&t, 0, sizeof(t));
    t.bits = 2;
    t.dtype = entry;
    t.separable = false;
    t.min_entry = INT32_MAX;
    t.max_entry = INT32_MIN;
    for (int i = 0; i < 16; ++i) {
        const int32_t v = entries[i];
        if (entry == DG_LUT_I8 && (v < -128 || v > 127))
            return dg_fail(DG_ERR_RANGE, "dg_build_lut_entries: entry %d = %d does not fit int8", i, v);
        t.entry[i] = (int16_t)v;
        if (v < t.min_entry) t.min_entry = v;
        if (v > t.max_entry) t.max_entry = v;
    }
    t.max_abs = t.max_entry > -t.min_entry ? t.max_entry : -t.min_entry;
    dg_lut *p = new (std::nothrow) dg_lut(t);
    if (!p) return dg_fail(DG_ERR_BUFFER, "dg_build_lut_entries: out of host memory");
    *out = p;
    return DG_OK;
}

dg_status dg_build_lut_f32(const float levels_w[4], const float levels_a[4], dg_lut **out)
{
    if (!levels_w || !levels_a || !out) return dg_fail(DG_ERR_NULL, "dg_build_lut_f32: NULL argument");
    dg_lut t;
    memset(&t, 0, sizeof(t));
    t.bits = 2;
    t.dtype = DG_LUT_F32;
    t.separable = true;
    for (int w = 0; w < 4; ++w)
        for (int a = 0; a < 4; ++a) {
            volatile float prod = levels_w[w] * levels_a[a];     // one binary32 multiply, kept out of wider registers
            t.fentry[4 * w + a] = prod;
        }
    dg_lut *p = new (std::nothrow) dg_lut(t);
    if (!p) return dg_fail(DG_ERR_BUFFER, "dg_build_lut_f32: out of host memory");
    *out = p;
    return DG_OK;
}

dg_status dg_lut_entries_f32(const dg_lut *lut, float out[16])
{
    if (!lut || !out) return dg_fail(DG_ERR_NULL, "dg_lut_entries_f32: NULL argument");
    if (lut->dtype != DG_LUT_F32) return dg_fail(DG_ERR_UNSUPPORTED, "dg_lut_entries_f32: an integer table");
    for (int i = 0; i < 16; ++i) out[i] = lut->fentry[i];
    return DG_OK;
}

dg_status dg_lut_entries_all(const dg_lut *lut, int16_t *out, int32_t count)
{
    if (!lut || !out) return dg_fail(DG_ERR_NULL, "dg_lut_entries_all: NULL argument");
    if (count != 1 << (2 * lut->bits))
        return dg_fail(DG_ERR_BUFFER, "dg_lut_entries_all: the table has %d entries, not %d", 1 << (2 * lut->bits), count);
    for (int i = 0; i < count; ++i) out[i] = lut->entry[i];
    return DG_OK;
}

void dg_lut_destroy(dg_lut *lut) { delete lut; }

size_t dg_packed_activation_bytes(int64_t rows, int64_t K) { return dg_packed_bytes_bits(rows, K, 2); }

size_t dg_packed_bytes_bits(int64_t rows, int64_t K, int32_t bits)
{
    if (bits < 2 || bits > 4) return 0;
    const int per_byte = bits == 2 ? 4 : 2;
    if (rows < 0 || K < 0 || K % per_byte != 0) return 0;
    return (size_t)rows * (size_t)(K / per_byte);
}

// The private weight layout currently coincides with the activation layout: with the table rows
// and selectors expanded once per tile in LDS, no offline re-ordering of weights saves work here.
size_t dg_packed_weight_bytes(int64_t M, int64_t K) { return dg_packed_activation_bytes(M, K); }

static dg_status pack_common(const char *name, const uint8_t *codes_dev, int64_t rows, int64_t K, int32_t bits,
                             void *packed_dev, size_t packed_bytes, void *hip_stream)
{
    if (!codes_dev || !packed_dev) return dg_fail(DG_ERR_NULL, "%s: NULL buffer", name);
    if (bits < 2 || bits > 4) return dg_fail(DG_ERR_UNSUPPORTED, "%s: %d-bit codes (2, 3 or 4)", name, bits);
    const int per_byte = bits == 2 ? 4 : 2;
    if (rows <= 0 || K <= 0 || K % per_byte != 0)
        return dg_fail(DG_ERR_SHAPE, "%s: rows=%lld K=%lld (need rows > 0, K > 0, K %% %d == 0)", name,
                       (long long)rows, (long long)K, per_byte);
    if (rows > INT32_MAX || K > INT32_MAX)
        return dg_fail(DG_ERR_SHAPE, "%s: rows and K must each fit int32", name);
    const size_t need = dg_packed_bytes_bits(rows, K, bits);
    if (packed_bytes < need)
        return dg_fail(DG_ERR_BUFFER, "%s: packed buffer has %zu bytes, %zu needed", name,
                       packed_bytes, need);
    return dg_launch_pack(codes_dev, rows, K, bits, (uint8_t *)packed_dev, (hipStream_t)hip_stream);
}

dg_status dg_pack_codes_bits(const uint8_t *codes_dev, int64_t rows, int64_t K, int32_t bits, void *packed_dev,
                             size_t packed_bytes, void *hip_stream)
{
    return pack_common("dg_pack_codes_bits", codes_dev, rows, K, bits, packed_dev, packed_bytes, hip_stream);
}

dg_status dg_pack_weights(const uint8_t *codes_dev, int64_t M, int64_t K, void *packed_dev,
                          size_t packed_bytes, void *hip_stream)
{
    return pack_common("dg_pack_weights", codes_dev, M, K, 2, packed_dev, packed_bytes, hip_stream);
}

dg_status dg_pack_activations(const uint8_t *codes_dev, int64_t N, int64_t K, void *packed_dev,
                              size_t packed_bytes, void *hip_stream)
{
    return pack_common("dg_pack_activations", codes_dev, N, K, 2, packed_dev, packed_bytes, hip_stream);
}

dg_status dg_quantize_pack_activations(const float *x_dev, int64_t N, int64_t K, float scale,
                                       float zero_point, int32_t lo, void *packed_dev,
                                       size_t packed_bytes, void *hip_stream)
{
    const char *name = "dg_quantize_pack_activations";
    if (!x_dev || !packed_dev) return dg_fail(DG_ERR_NULL, "%s: NULL buffer", name);
    if (N <= 0 || K <= 0 || K % 4 != 0)
        return dg_fail(DG_ERR_SHAPE, "%s: N=%lld K=%lld (need N > 0, K > 0, K %% 4 == 0)", name, (long long)N,
                       (long long)K);
    if (N > INT32_MAX || K > INT32_MAX) return dg_fail(DG_ERR_SHAPE, "%s: N and K must each fit int32", name);
    if (lo < -(1 << 24) || lo > (1 << 24)) return dg_fail(DG_ERR_RANGE, "%s: lo=%d is not exact in binary32", name, lo);
    const size_t need = dg_packed_activation_bytes(N, K);
    if (packed_bytes < need)
        return dg_fail(DG_ERR_BUFFER, "%s: packed buffer has %zu bytes, %zu needed", name, packed_bytes, need);
    return dg_launch_quantize_pack(x_dev, N, K, scale, zero_point, lo, (uint8_t *)packed_dev,
                                   (hipStream_t)hip_stream);
}

dg_status dg_dequantize(const int32_t *acc_dev, int64_t rows, int64_t C, const float *scale_c_dev, float *out_dev,
                        void *hip_stream)
{
    const char *name = "dg_dequantize";
    if (!acc_dev || !scale_c_dev || !out_dev) return dg_fail(DG_ERR_NULL, "%s: NULL buffer", name);
    if (rows <= 0 || C <= 0 || C > INT32_MAX || rows > INT64_MAX / C)
        return dg_fail(DG_ERR_SHAPE, "%s: rows=%lld C=%lld", name, (long long)rows, (long long)C);
    return dg_launch_dequantize(acc_dev, rows, C, scale_c_dev, out_dev, (hipStream_t)hip_stream);
}

int64_t dg_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad)
{
    if (stride <= 0 || k <= 0 || in <= 0 || pad < 0) return 0;
    const int64_t span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

}   // extern "C"

namespace {

enum class Pick { Perm, Lds, LdsF32, Mfma, SmallN, Lut65k, OneHot, Sparse, Sparse4, Sparse2p, SparseWs, FewN, Unsupported };

Pick pick_kernel(const dg_lut *lut, const DgProblem &p, dg_kernel variant)
{
    // binary32 tables run on the plain LDS kernel only; 3- and 4-bit tables on the one-hot matrix-core kernel or the LDS kernel
    if (lut->dtype == DG_LUT_F32)
        return (variant == DG_KERNEL_AUTO || variant == DG_KERNEL_LDS) ? Pick::LdsF32 : Pick::Unsupported;
    if (lut->bits != 2) {
        if (variant == DG_KERNEL_LDS) return Pick::Lds;
        if (variant == DG_KERNEL_AUTO) {
            if (dg_sparse4_preferred(lut, p)) return Pick::Sparse4;
            return dg_onehot_supports(lut, p) ? Pick::OneHot : Pick::Lds;
        }
        if (variant == DG_KERNEL_ONEHOT_MFMA && dg_onehot_supports(lut, p)) return Pick::OneHot;
        if (variant == DG_KERNEL_ONEHOT_SMFMAC && dg_sparse4_supports(lut, p)) return Pick::Sparse4;
        return Pick::Unsupported;
    }
    switch (variant) {
    case DG_KERNEL_PERM: return dg_perm_supports(lut, p) ? Pick::Perm : Pick::Unsupported;
    case DG_KERNEL_LDS: return Pick::Lds;
    case DG_KERNEL_MFMA_I8: return dg_decode_supports(lut, p) ? Pick::Mfma : Pick::Unsupported;
    case DG_KERNEL_SMALLN: return dg_smalln_supports(lut, p) ? Pick::SmallN : Pick::Unsupported;
    case DG_KERNEL_LUT65K: return dg_lut65k_supports(lut, p) ? Pick::Lut65k : Pick::Unsupported;
    case DG_KERNEL_ONEHOT_MFMA: return dg_onehot_supports(lut, p) ? Pick::OneHot : Pick::Unsupported;
    case DG_KERNEL_ONEHOT_SMFMAC:
        if (dg_fewn_preferred(lut, p)) return Pick::FewN;
        if (dg_sparse_ws_preferred(lut, p)) return Pick::SparseWs;
        if (dg_sparse2p_supports(lut, p)) return Pick::Sparse2p;
        return dg_sparse_supports(lut, p) ? Pick::Sparse : Pick::Unsupported;
    case DG_KERNEL_AUTO:
        // AUTO stays within the table kernels: the decode-and-multiply matrix-core kernel is a comparison only.
        // few columns, long rows: the weights stream once through the sparse instruction's index operand
        if (dg_fewn_preferred(lut, p)) return Pick::FewN;
        // one or two columns: K across the lanes of a wavefront streams the weights once at full width
        if (p.N <= 2 && p.K >= 1024 && dg_smalln_supports(lut, p)) return Pick::SmallN;
        // int8 tables: selecting entries with one-hot operands on the matrix cores outruns the permute loop at every
        // size measured (1.5x on a 0.2 GOP layer, 5x - 10x from 3 GOP upwards)
        // (large layers: the same selection on the sparse instruction, about half the matrix work)
        if (dg_sparse2p_preferred(lut, p)) return Pick::Sparse2p;
        // short reductions with many output blocks: the dense operand of the weights is built once per wavefront
        if (dg_sparse_ws_preferred(lut, p)) return Pick::SparseWs;
        if (dg_onehot_supports(lut, p)) return dg_sparse_preferred(lut, p) ? Pick::Sparse : Pick::OneHot;
        if (p.N <= 32 && p.K >= 1024 && dg_smalln_supports(lut, p)) return Pick::SmallN;
        if (dg_perm_supports(lut, p)) return Pick::Perm;
        return Pick::Lds;
    }
    return Pick::Unsupported;
}

dg_status run(const dg_lut *lut, const DgProblem &p, dg_kernel variant, hipStream_t stream)
{
    switch (pick_kernel(lut, p, variant)) {
    case Pick::Perm: return dg_launch_perm(lut, p, stream);
    case Pick::Lds: return dg_launch_lds(lut, p, stream);
    case Pick::LdsF32: return dg_launch_lds_f32(lut, p, stream);
    case Pick::Mfma: return dg_launch_decode(lut, p, stream);
    case Pick::SmallN: return dg_launch_smalln(lut, p, stream);
    case Pick::Lut65k: return dg_launch_lut65k(lut, p, stream);
    case Pick::OneHot: return dg_launch_onehot(lut, p, stream);
    case Pick::Sparse: return dg_launch_sparse(lut, p, stream);
    case Pick::Sparse4: return dg_launch_sparse4(lut, p, stream);
    case Pick::Sparse2p: return dg_launch_sparse2p(lut, p, stream);
    case Pick::SparseWs: return dg_launch_sparse_ws(lut, p, stream);
    case Pick::FewN: return dg_launch_fewn(lut, p, stream);
    case Pick::Unsupported: break;
    }
    return dg_fail(DG_ERR_UNSUPPORTED,
                   "kernel variant %d cannot run M=%d N=%d K=%d (Cin=%d) with this table",
                   (int)variant, p.M, p.N, p.K, p.Cin);
}

const char *pick_name(const dg_lut *lut, const DgProblem &p, dg_kernel variant)
{
    switch (pick_kernel(lut, p, variant)) {
    case Pick::Perm: return dg_perm_config_name(lut, p);
    case Pick::Lds: return "lds";
    case Pick::LdsF32: return "lds_f32";
    case Pick::Mfma: return dg_decode_config_name(lut, p);
    case Pick::SmallN: return "smalln";
    case Pick::Lut65k: return "lut65k";
    case Pick::OneHot: return dg_onehot_config_name(lut, p);
    case Pick::Sparse: return dg_sparse_config_name(lut, p);
    case Pick::Sparse4: return "onehot_smfmac4_64x128";
    case Pick::Sparse2p: return "onehot_smfmac_2p_32x128";
    case Pick::SparseWs: return "onehot_smfmac_ws_32xK";
    case Pick::FewN: return "onehot_smfmac_fewn_16";
    case Pick::Unsupported: break;
    }
    return "unsupported";
}

dg_status check_range(const char *name, const dg_lut *lut, int64_t K)
{
    // int32 accumulator: |sum| <= K * max|LUT| must stay below 2^31 (binary32 tables have no such bound)
    if (lut->dtype != DG_LUT_F32 && (int64_t)lut->max_abs * K >= ((int64_t)1 << 31))
        return dg_fail(DG_ERR_RANGE, "%s: K=%lld times max|LUT|=%d could overflow int32", name,
                       (long long)K, lut->max_abs);
    return DG_OK;
}

dg_status fill_gemm(const char *name, const dg_lut *lut, int64_t M, int64_t N, int64_t K,
                    DgProblem *p)
{
    if (!lut) return dg_fail(DG_ERR_NULL, "%s: NULL table", name);
    const int per_byte = lut->bits == 2 ? 4 : 2;
    if (M <= 0 || N <= 0 || K <= 0 || K % per_byte != 0)
        return dg_fail(DG_ERR_SHAPE, "%s: M=%lld N=%lld K=%lld (need all > 0 and K %% %d == 0)", name,
                       (long long)M, (long long)N, (long long)K, per_byte);
    if (M > INT32_MAX / 2 || N > INT32_MAX / 2 || K > INT32_MAX / 2)
        return dg_fail(DG_ERR_SHAPE, "%s: a dimension exceeds 2^30", name);
    memset(p, 0, sizeof(*p));
    p->M = (int32_t)M;
    p->N = (int32_t)N;
    p->K = (int32_t)K;
    p->H = p->W = p->KH = p->KW = p->sh = p->sw = p->OH = p->OW = 1;
    p->Cin = (int32_t)K;
    p->stride_cm = N;             // row-major [M][N] unless the caller says otherwise
    p->stride_cn = 1;
    return check_range(name, lut, K);
}

dg_status fill_conv(const char *name, const dg_lut *lut, const dg_conv_desc *d, DgProblem *p)
{
    if (!lut || !d) return dg_fail(DG_ERR_NULL, "%s: NULL table or descriptor", name);
    if (d->B <= 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0 || d->KH <= 0 ||
        d->KW <= 0 || d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return dg_fail(DG_ERR_SHAPE, "%s: every dimension and stride must be > 0 and pads >= 0", name);
    const int per_byte = lut->bits == 2 ? 4 : 2;
    if (d->Cin % per_byte != 0)
        return dg_fail(DG_ERR_SHAPE, "%s: Cin=%d is not a multiple of %d", name, d->Cin, per_byte);
    const int64_t OH = dg_conv_out_dim(d->H, d->KH, d->stride_h, d->pad_h);
    const int64_t OW = dg_conv_out_dim(d->W, d->KW, d->stride_w, d->pad_w);
    if (OH <= 0 || OW <= 0) return dg_fail(DG_ERR_SHAPE, "%s: the filter does not fit the padded image", name);
    const int64_t N = (int64_t)d->B * OH * OW;
    const int64_t K = (int64_t)d->KH * d->KW * d->Cin;
    const int64_t pixels = (int64_t)d->B * d->H * d->W;
    if (N > INT32_MAX / 2 || K > INT32_MAX / 2 || pixels > INT32_MAX / 2 || d->Cout > INT32_MAX / 2)
        return dg_fail(DG_ERR_SHAPE, "%s: a dimension exceeds 2^30", name);
    memset(p, 0, sizeof(*p));
    p->M = d->Cout;
    p->N = (int32_t)N;
    p->K = (int32_t)K;
    p->H = d->H;
    p->W = d->W;
    p->Cin = d->Cin;
    p->KH = d->KH;
    p->KW = d->KW;
    p->sh = d->stride_h;
    p->sw = d->stride_w;
    p->ph = d->pad_h;
    p->pw = d->pad_w;
    p->OH = (int32_t)OH;
    p->OW = (int32_t)OW;
    p->stride_cm = 1;             // NHWC: channel fastest
    p->stride_cn = p->M;
    return check_range(name, lut, K);
}

}   // namespace

extern "C" {

dg_status dg_gemm_lut(const dg_lut *lut, const void *Wp_dev, const void *Ap_dev, int64_t M,
                      int64_t N, int64_t K, int32_t *C_dev, int64_t stride_cm, int64_t stride_cn,
                      const float *scale_m_dev, float *Cf_dev, dg_kernel variant, void *hip_stream)
{
    DgProblem p;
    dg_status s = fill_gemm("dg_gemm_lut", lut, M, N, K, &p);
    if (s != DG_OK) return s;
    if (!Wp_dev || !Ap_dev) return dg_fail(DG_ERR_NULL, "dg_gemm_lut: NULL operand");
    if ((scale_m_dev || lut->dtype == DG_LUT_F32) ? !Cf_dev : !C_dev)
        return dg_fail(DG_ERR_NULL, "dg_gemm_lut: NULL output");
    if (stride_cm == 0 || stride_cn == 0) return dg_fail(DG_ERR_SHAPE, "dg_gemm_lut: zero output stride");
    p.Wp = (const uint8_t *)Wp_dev;
    p.Xp = (const uint8_t *)Ap_dev;
    p.C = C_dev;
    p.Cf = Cf_dev;
    p.scale = scale_m_dev;
    p.stride_cm = stride_cm;
    p.stride_cn = stride_cn;
    return run(lut, p, variant, (hipStream_t)hip_stream);
}

dg_status dg_conv2d_lut(const dg_lut *lut, const void *Wp_dev, const void *Xp_dev,
                        const dg_conv_desc *desc, int32_t *Y_dev, const float *scale_cout_dev,
                        float *Yf_dev, dg_kernel variant, void *hip_stream)
{
    DgProblem p;
    dg_status s = fill_conv("dg_conv2d_lut", lut, desc, &p);
    if (s != DG_OK) return s;
    if (!Wp_dev || !Xp_dev) return dg_fail(DG_ERR_NULL, "dg_conv2d_lut: NULL operand");
    if ((scale_cout_dev || lut->dtype == DG_LUT_F32) ? !Yf_dev : !Y_dev)
        return dg_fail(DG_ERR_NULL, "dg_conv2d_lut: NULL output");
    p.Wp = (const uint8_t *)Wp_dev;
    p.Xp = (const uint8_t *)Xp_dev;
    p.C = Y_dev;
    p.Cf = Yf_dev;
    p.scale = scale_cout_dev;
    p.stride_cm = 1;          // NHWC: channel fastest
    p.stride_cn = p.M;
    return run(lut, p, variant, (hipStream_t)hip_stream);
}

namespace {

// The one-call entry points fuse the packing into the kernel where the library's own choice for the problem (or the
// variant the caller names) is the one-hot split-K kernel or the few-columns kernel, i.e. on problems so small that a
// second launch costs a good part of the whole.
enum class Fuse { None, OneHot, OneHotSparse, SmallN, SparseWs };

Fuse fuses_packing(const dg_lut *lut, const DgProblem &p_codes, dg_kernel variant)
{
    // (the unpacked buffer's 16-byte alignment satisfies every kernel's test of the packed one)
    if ((uintptr_t)p_codes.Xp % 16 != 0 || lut->bits != 2) return Fuse::None;
    if ((variant == DG_KERNEL_AUTO || variant == DG_KERNEL_ONEHOT_MFMA) && dg_onehot_codes_supports(lut, p_codes) &&
        (variant == DG_KERNEL_ONEHOT_MFMA ||
         (dg_onehot_codes_pays(p_codes) && pick_kernel(lut, p_codes, DG_KERNEL_AUTO) == Pick::OneHot)))
        return Fuse::OneHot;
    // layers of a few microseconds on the tiled kernels: the narrow tiles pack per 64-row tile -- on the sparse instruction
    // where the output's channel axis is the contiguous one and the caller has not named the dense one's variant
    if ((variant == DG_KERNEL_AUTO || variant == DG_KERNEL_ONEHOT_MFMA || variant == DG_KERNEL_ONEHOT_SMFMAC) &&
        dg_onehot_codes_tiled_supports(lut, p_codes)) {
        const bool sparse = variant != DG_KERNEL_ONEHOT_MFMA && dg_onehot_codes_tiled_sparse(lut, p_codes);
        if ((sparse || variant != DG_KERNEL_ONEHOT_SMFMAC) && dg_onehot_codes_tiled_pays(lut, p_codes, sparse)) {
            const Pick pick = pick_kernel(lut, p_codes, variant);
            if (pick == Pick::OneHot || pick == Pick::Sparse) return sparse ? Fuse::OneHotSparse : Fuse::OneHot;
        }
    }
    // (the few-columns kernel packs once per row block and pass of four columns, about 7 % more work for it: less than
    // a launch while the columns are few, which is where AUTO uses that kernel anyway)
    if ((variant == DG_KERNEL_SMALLN || (variant == DG_KERNEL_AUTO && p_codes.N <= 4)) &&
        pick_kernel(lut, p_codes, variant) == Pick::SmallN)
        return Fuse::SmallN;
    // the stationary-weight kernel stages and packs the codes of its pixel blocks itself
    if ((variant == DG_KERNEL_AUTO || variant == DG_KERNEL_ONEHOT_SMFMAC) && dg_sparse_ws_codes_supports(lut, p_codes) &&
        pick_kernel(lut, p_codes, variant) == Pick::SparseWs)
        return Fuse::SparseWs;
    // (one column: on packed activations the few-columns sparse-instruction kernel is the faster by 6 %, which is less
    // than the packing launch it would need here)
    if (variant == DG_KERNEL_AUTO && p_codes.N == 1 && p_codes.K >= 1024 && dg_smalln_supports(lut, p_codes) &&
        pick_kernel(lut, p_codes, variant) == Pick::FewN)
        return Fuse::SmallN;
    return Fuse::None;
}

// A 1x1 layer with a stride and no padding reads one input pixel in sh * sw: where the packing is not fused only those
// are packed (2-bit codes in whole 16-code groups), and the layer then runs on them without a stride -- 56x56x256 -> 512
// with stride 2 at batch 32 packs 6.4 MB of codes instead of 25.7 MB.
bool packs_strided_pixels(const dg_lut *lut, const DgProblem &p_codes)
{
    return lut->bits == 2 && p_codes.KH == 1 && p_codes.KW == 1 && p_codes.ph == 0 && p_codes.pw == 0 &&
           (p_codes.sh > 1 || p_codes.sw > 1) && p_codes.Cin % 16 == 0 && (uintptr_t)p_codes.Xp % 16 == 0 &&
           (int64_t)p_codes.N * (p_codes.Cin / 16) < ((int64_t)1 << 31);
}

DgProblem without_stride(const DgProblem &p)
{
    DgProblem c = p;
    c.H = p.OH, c.W = p.OW, c.sh = 1, c.sw = 1;
    return c;
}

// Launch the fused form, or pack into the work buffer and run the problem as the two-call path would.
dg_status run_codes(const char *name, const dg_lut *lut, DgProblem &p, const uint8_t *codes, int64_t rows, int64_t row_codes,
                    void *work, size_t work_bytes, dg_kernel variant, void *hip_stream)
{
    p.Xp = codes;
    switch (fuses_packing(lut, p, variant)) {
    case Fuse::OneHot: return dg_launch_onehot_codes(lut, p, (hipStream_t)hip_stream);
    case Fuse::OneHotSparse: return dg_launch_onehot_codes(lut, p, (hipStream_t)hip_stream, true);
    case Fuse::SmallN: return dg_launch_smalln_codes(lut, p, (hipStream_t)hip_stream);
    case Fuse::SparseWs: return dg_launch_sparse_ws_codes(lut, p, (hipStream_t)hip_stream);
    case Fuse::None: break;
    }
    if (packs_strided_pixels(lut, p)) {
        if (!work) return dg_fail(DG_ERR_NULL, "%s: NULL buffer", name);
        const size_t need = dg_packed_bytes_bits(rows, row_codes, lut->bits);       // (the documented size, not the smaller one used)
        if (work_bytes < need) return dg_fail(DG_ERR_BUFFER, "%s: packed buffer has %zu bytes, %zu needed", name, work_bytes, need);
        const int64_t images = rows / ((int64_t)p.H * p.W);
        const dg_status st = dg_launch_pack_strided_pixels(codes, images, p.H, p.W, p.OH, p.OW, p.sh, p.sw, p.Cin, (uint8_t *)work,
                                                           (hipStream_t)hip_stream);
        if (st != DG_OK) return st;
        DgProblem c = without_stride(p);
        c.Xp = (const uint8_t *)work;
        return run(lut, c, variant, (hipStream_t)hip_stream);
    }
    const dg_status s = pack_common(name, codes, rows, row_codes, lut->bits, work, work_bytes, hip_stream);
    if (s != DG_OK) return s;
    p.Xp = (const uint8_t *)work;
    return run(lut, p, variant, (hipStream_t)hip_stream);
}

const char *codes_name(const dg_lut *lut, const DgProblem &p, dg_kernel variant)
{
    switch (fuses_packing(lut, p, variant)) {
    case Fuse::OneHot: return dg_onehot_codes_config_name(lut, p);
    case Fuse::OneHotSparse: return dg_onehot_codes_config_name(lut, p, true);
    case Fuse::SmallN: return "codes_smalln";
    case Fuse::SparseWs: return "codes_onehot_smfmac_ws_32xK";
    case Fuse::None: break;
    }
    if (packs_strided_pixels(lut, p)) return pick_name(lut, without_stride(p), variant);
    return pick_name(lut, p, variant);
}

}   // namespace

dg_status dg_gemm_lut_codes(const dg_lut *lut, const void *Wp_dev, const uint8_t *Ac_dev, int64_t M, int64_t N,
                            int64_t K, void *Ap_work_dev, size_t work_bytes, int32_t *C_dev, int64_t stride_cm,
                            int64_t stride_cn, const float *scale_m_dev, float *Cf_dev, dg_kernel variant,
                            void *hip_stream)
{
    const char *name = "dg_gemm_lut_codes";
    DgProblem p;
    dg_status s = fill_gemm(name, lut, M, N, K, &p);
    if (s != DG_OK) return s;
    if (!Wp_dev || !Ac_dev) return dg_fail(DG_ERR_NULL, "%s: NULL operand", name);
    if ((scale_m_dev || lut->dtype == DG_LUT_F32) ? !Cf_dev : !C_dev) return dg_fail(DG_ERR_NULL, "%s: NULL output", name);
    if (stride_cm == 0 || stride_cn == 0) return dg_fail(DG_ERR_SHAPE, "%s: zero output stride", name);
    p.Wp = (const uint8_t *)Wp_dev;
    p.C = C_dev;
    p.Cf = Cf_dev;
    p.scale = scale_m_dev;
    p.stride_cm = stride_cm;
    p.stride_cn = stride_cn;
    return run_codes(name, lut, p, Ac_dev, N, K, Ap_work_dev, work_bytes, variant, hip_stream);
}

const char *dg_gemm_codes_kernel_name(const dg_lut *lut, int64_t M, int64_t N, int64_t K, dg_kernel variant)
{
    DgProblem p;
    if (fill_gemm("dg_gemm_codes_kernel_name", lut, M, N, K, &p) != DG_OK) return "invalid";
    return codes_name(lut, p, variant);
}

dg_status dg_conv2d_lut_codes(const dg_lut *lut, const void *Wp_dev, const uint8_t *Xc_dev, const dg_conv_desc *desc,
                              void *Xp_work_dev, size_t work_bytes, int32_t *Y_dev, const float *scale_cout_dev,
                              float *Yf_dev, dg_kernel variant, void *hip_stream)
{
    const char *name = "dg_conv2d_lut_codes";
    DgProblem p;
    dg_status s = fill_conv(name, lut, desc, &p);
    if (s != DG_OK) return s;
    if (!Wp_dev || !Xc_dev) return dg_fail(DG_ERR_NULL, "%s: NULL operand", name);
    if ((scale_cout_dev || lut->dtype == DG_LUT_F32) ? !Yf_dev : !Y_dev) return dg_fail(DG_ERR_NULL, "%s: NULL output", name);
    p.Wp = (const uint8_t *)Wp_dev;
    p.C = Y_dev;
    p.Cf = Yf_dev;
    p.scale = scale_cout_dev;
    p.stride_cm = 1;
    p.stride_cn = p.M;
    return run_codes(name, lut, p, Xc_dev, (int64_t)desc->B * desc->H * desc->W, desc->Cin, Xp_work_dev, work_bytes, variant,
                     hip_stream);
}

const char *dg_conv_codes_kernel_name(const dg_lut *lut, const dg_conv_desc *desc, dg_kernel variant)
{
    DgProblem p;
    if (fill_conv("dg_conv_codes_kernel_name", lut, desc, &p) != DG_OK) return "invalid";
    p.stride_cm = 1;
    p.stride_cn = p.M;
    return codes_name(lut, p, variant);
}

size_t dg_static_work_bytes(void) { return DG_STATIC_WORK_BYTES; }

dg_status dg_conv2d_lut_codes_static(const dg_lut *lut, const void *Wp_dev, const uint8_t *Xc_dev, const dg_conv_desc *desc,
                                     int32_t *Y_dev, const float *scale_cout_dev, float *Yf_dev, dg_kernel variant,
                                     void *hip_stream)
{
    const char *name = "dg_conv2d_lut_codes_static";
    if (!lut || !desc) return dg_fail(DG_ERR_NULL, "%s: NULL table or descriptor", name);
    if (desc->B > 0 && desc->H > 0 && desc->W > 0 && desc->Cin > 0) {
        // (bad dimensions are reported by the shared validation below; here only the size limit)
        const int per_byte = lut->bits == 2 ? 4 : 2;
        const unsigned long long need = (unsigned long long)desc->B * desc->H * desc->W * (unsigned long long)(desc->Cin / per_byte);
        if (need > DG_STATIC_WORK_BYTES)
            return dg_fail(DG_ERR_BUFFER, "%s: the packed activations take %llu bytes, the library's staging holds %zu "
                           "(use dg_conv2d_lut_codes with a work buffer)", name, need, DG_STATIC_WORK_BYTES);
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return dg_fail(DG_ERR_HIP, "%s: hipGetDevice: %s", name, hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return dg_fail(DG_ERR_UNSUPPORTED, "%s: device %d (at most %d devices)", name, dev, MAX_DEVICES);
    void *work = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_static_work_mutex);
        if (!g_static_work[dev]) {
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));      // the current device's copy of the array
            if (e != hipSuccess || !ptr)
                return dg_fail(DG_ERR_HIP, "%s: hipGetSymbolAddress: %s", name, hipGetErrorString(e));
            g_static_work[dev] = ptr;
        }
        work = g_static_work[dev];
    }
    return dg_conv2d_lut_codes(lut, Wp_dev, Xc_dev, desc, work, DG_STATIC_WORK_BYTES, Y_dev, scale_cout_dev, Yf_dev, variant,
                               hip_stream);
}

dg_status dg_conv2d_lut_requant(const dg_lut *lut, const void *Wp_dev, const void *Xp_dev, const dg_conv_desc *desc,
                                const float *scale_cout_dev, float q_scale, float q_zero, int32_t lo,
                                void *packed_out_dev, size_t packed_bytes, dg_kernel variant, void *hip_stream)
{
    const char *name = "dg_conv2d_lut_requant";
    DgProblem p;
    dg_status s = fill_conv(name, lut, desc, &p);
    if (s != DG_OK) return s;
    if (p.M % 4 != 0) return dg_fail(DG_ERR_SHAPE, "%s: Cout=%d is not a multiple of 4", name, p.M);
    if (!Wp_dev || !Xp_dev || !scale_cout_dev || !packed_out_dev) return dg_fail(DG_ERR_NULL, "%s: NULL buffer", name);
    if (lo < -(1 << 24) || lo > (1 << 24)) return dg_fail(DG_ERR_RANGE, "%s: lo=%d is not exact in binary32", name, lo);
    const size_t need = dg_packed_activation_bytes(p.N, p.M);
    if (packed_bytes < need)
        return dg_fail(DG_ERR_BUFFER, "%s: packed buffer has %zu bytes, %zu needed", name, packed_bytes, need);
    p.Wp = (const uint8_t *)Wp_dev;
    p.Xp = (const uint8_t *)Xp_dev;
    p.scale = scale_cout_dev;
    p.stride_cm = 1;
    p.stride_cn = p.M;
    p.Qp = (uint8_t *)packed_out_dev;
    p.q_scale = q_scale;
    p.q_zero = q_zero;
    p.q_lo = lo;
    // the re-quantising epilogue lives in the one-hot matrix-core kernels (both instruction forms share it)
    if ((variant == DG_KERNEL_ONEHOT_SMFMAC || variant == DG_KERNEL_AUTO) && dg_sparse_ws_preferred(lut, p))
        return dg_launch_sparse_ws(lut, p, (hipStream_t)hip_stream);
    if (variant == DG_KERNEL_ONEHOT_SMFMAC && lut->bits == 2 && dg_sparse_supports(lut, p))
        return dg_launch_sparse(lut, p, (hipStream_t)hip_stream);
    if (variant == DG_KERNEL_ONEHOT_SMFMAC && dg_sparse2p_supports(lut, p))
        return dg_launch_sparse2p(lut, p, (hipStream_t)hip_stream);
    if (variant == DG_KERNEL_ONEHOT_SMFMAC && dg_sparse4_supports(lut, p))
        return dg_launch_sparse4(lut, p, (hipStream_t)hip_stream);
    if ((variant != DG_KERNEL_AUTO && variant != DG_KERNEL_ONEHOT_MFMA) || lut->dtype == DG_LUT_F32 ||
        !dg_onehot_supports(lut, p))
        return dg_fail(DG_ERR_UNSUPPORTED, "%s: needs the one-hot matrix-core kernel (variant %d, Cin=%d, table range %d..%d)",
                       name, (int)variant, p.Cin, lut->min_entry, lut->max_entry);
    if (variant == DG_KERNEL_AUTO && dg_sparse2p_preferred(lut, p)) return dg_launch_sparse2p(lut, p, (hipStream_t)hip_stream);
    if (variant == DG_KERNEL_AUTO && dg_sparse4_preferred(lut, p)) return dg_launch_sparse4(lut, p, (hipStream_t)hip_stream);
    if (variant == DG_KERNEL_AUTO && dg_sparse_preferred(lut, p)) return dg_launch_sparse(lut, p, (hipStream_t)hip_stream);
    return dg_launch_onehot(lut, p, (hipStream_t)hip_stream);
}

dg_status dg_launch_empty(int64_t blocks, int32_t threads, void *hip_stream)
{
    if (blocks <= 0 || blocks > INT32_MAX || threads <= 0 || threads > 1024 || threads % 64 != 0)
        return dg_fail(DG_ERR_SHAPE, "dg_launch_empty: blocks=%lld threads=%d", (long long)blocks, threads);
    hipLaunchKernelGGL(empty_kernel, dim3((unsigned)blocks), dim3((unsigned)threads), 0, (hipStream_t)hip_stream);
    return dg_check_launch("empty_kernel");
}

const char *dg_gemm_kernel_name(const dg_lut *lut, int64_t M, int64_t N, int64_t K, dg_kernel variant)
{
    DgProblem p;
    if (fill_gemm("dg_gemm_kernel_name", lut, M, N, K, &p) != DG_OK) return "invalid";
    return pick_name(lut, p, variant);
}

const char *dg_conv_kernel_name(const dg_lut *lut, const dg_conv_desc *desc, dg_kernel variant)
{
    DgProblem p;
    if (fill_conv("dg_conv_kernel_name", lut, desc, &p) != DG_OK) return "invalid";
    return pick_name(lut, p, variant);
}

}   // extern "C"
