// Internal declarations shared by the host API and the gfx950 kernels of libdeepgemm_hip.
// Nothing here is part of the public ABI (that is include/deepgemm_hip.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "deepgemm_hip.h"

// The opaque table object: levels, the 16 products, and what the kernels need to know about them.
struct dg_lut {
    int32_t bits;        // code width: 2 (the paper's kernels), 3 or 4 (Sec. 3.3); 2^bits levels per side
    int8_t levels_w[16];
    int8_t levels_a[16];
    int16_t entry[256];  // entry[(w << bits) | a] = levels_w[w] * levels_a[a]; 2^(2*bits) entries are used
    dg_lut_dtype dtype;
    bool separable;      // built from level vectors (the matrix-core comparison kernel needs them)
    float fentry[16];    // DG_LUT_F32 tables only: binary32 products of floating-point levels
    int32_t min_entry;   // smallest product
    int32_t max_entry;   // largest product
    int32_t max_abs;     // max |product|
};

// 16 table entries passed to kernels by value (no device allocation is needed for a table).
struct DgTable16 {
    int16_t e[16];
};

// One implicit-GEMM problem.  A plain GEMM is the convolution with B = N, H = W = 1, a 1x1 filter
// and Cin = K: "pixel" n is activation row n.
//   M = Cout, N = B*OH*OW, K = KH*KW*Cin, reduction index k = (kh*KW + kw)*Cin + ci.
struct DgProblem {
    int32_t M, N, K;
    int32_t H, W, Cin, KH, KW, sh, sw, ph, pw, OH, OW;
    const uint8_t *Wp;    // packed weights, [M][K/4]
    const uint8_t *Xp;    // packed activations, [B*H*W][Cin/4]
    int32_t *C;           // int32 output (used when scale == nullptr)
    float *Cf;            // fp32 output (used when scale != nullptr)
    const float *scale;   // per-m scale or nullptr
    int64_t stride_cm, stride_cn;   // element strides of the output
    // Re-quantising epilogue (the packed activations of the next layer instead of C / Cf), used when Qp != nullptr:
    // code = clip(rint(q_scale * (float(sum) * scale[m]) + q_zero), q_lo, q_lo + 3) - q_lo, four channels per byte.
    uint8_t *Qp;          // [N][M/4]; requires scale, M % 4 == 0 and the NHWC output order (stride_cm == 1)
    float q_scale, q_zero;
    int32_t q_lo;
};

// n / d for 0 <= n < 2^31 by multiply-high and shift, d fixed per launch and prepared on the host:
// n / d == umulhi(n, mul) >> shift for d >= 2 with L = ceil(log2 d), mul = ceil(2^(31+L) / d) < 2^32 and shift = L - 1
// (the error mul * d - 2^(31+L) is below d <= 2^L = 2^((31+L) - 31)); d = 1 is passed through.
struct DgFastDiv {
    uint32_t mul, shift, d;
};

__device__ __forceinline__ uint32_t dg_fdiv(uint32_t n, const DgFastDiv &f)
{
    return f.d == 1 ? n : __umulhi(n, f.mul) >> f.shift;
}

inline DgFastDiv dg_make_div(uint32_t d)
{
    DgFastDiv f = {0u, 0u, d};
    if (d < 2) return f;
    uint32_t L = 0;
    while ((1ull << L) < d) ++L;
    f.mul = (uint32_t)(((1ull << (31 + L)) + d - 1) / d);
    f.shift = L - 1;
    return f;
}

// Value of a test / measurement override (an environment variable), or nullptr.  Overrides are looked at only when
// DG_TEST_OVERRIDES=1 was set when the library was first called; otherwise this returns nullptr without reading anything.
const char *dg_override(const char *name);
// Number of SIMD units of the current device (compute units x 4), asked from the runtime once.
int dg_simd_count();
// Record the calling thread's error detail and return `s`.
dg_status dg_fail(dg_status s, const char *fmt, ...);
// Turn the launch status of the last kernel into a dg_status.
dg_status dg_check_launch(const char *what);

// Kernel launchers (each validates nothing: the API layer has done that).
dg_status dg_launch_pack(const uint8_t *codes, int64_t rows, int64_t K, int bits, uint8_t *packed,
                         hipStream_t stream);
// 2-bit codes of the pixels (b, oh * sh, ow * sw) only, [B][H][W][Cin] -> [B][OH][OW][Cin / 4]; Cin % 16 == 0, codes
// 16-byte and packed 4-byte aligned (the caller checks)
dg_status dg_launch_pack_strided_pixels(const uint8_t *codes, int64_t B, int32_t H, int32_t W, int32_t OH, int32_t OW, int32_t sh,
                                        int32_t sw, int32_t Cin, uint8_t *packed, hipStream_t stream);
dg_status dg_launch_quantize_pack(const float *x, int64_t rows, int64_t K, float scale, float zero_point,
                                  int32_t lo, uint8_t *packed, hipStream_t stream);
dg_status dg_launch_dequantize(const int32_t *acc, int64_t rows, int64_t C, const float *scale, float *out,
                               hipStream_t stream);
dg_status dg_launch_lds(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
dg_status dg_launch_lds_f32(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
bool dg_perm_supports(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_perm(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
const char *dg_perm_config_name(const dg_lut *lut, const DgProblem &p);
bool dg_decode_supports(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_decode(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
const char *dg_decode_config_name(const dg_lut *lut, const DgProblem &p);
bool dg_lut65k_supports(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_lut65k(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
bool dg_onehot_supports(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_onehot(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
const char *dg_onehot_config_name(const dg_lut *lut, const DgProblem &p);
// the one-hot split-K kernel reading activations one code per byte (p.Xp = those bytes) and packing them as it loads
bool dg_onehot_codes_supports(const dg_lut *lut, const DgProblem &p);
bool dg_onehot_codes_pays(const DgProblem &p);      // AUTO: the repeated packing costs less than the saved launch
// (`sparse_tiles`: the tiled form on the sparse instruction, where dg_onehot_codes_tiled_sparse says it applies)
dg_status dg_launch_onehot_codes(const dg_lut *lut, const DgProblem &p, hipStream_t stream, bool sparse_tiles = false);
const char *dg_onehot_codes_config_name(const dg_lut *lut, const DgProblem &p, bool sparse_tiles = false);
// the one-hot tiled kernel (64 x 32 and 64 x 64 tiles) doing the same on layers of a few microseconds
bool dg_onehot_codes_tiled_supports(const dg_lut *lut, const DgProblem &p);
bool dg_onehot_codes_tiled_sparse(const dg_lut *lut, const DgProblem &p);  // on the sparse instruction (channel axis contiguous)
bool dg_onehot_codes_tiled_pays(const dg_lut *lut, const DgProblem &p, bool sparse_tiles);   // AUTO: shorter than packing kernel + AUTO's kernel
bool dg_sparse_supports(const dg_lut *lut, const DgProblem &p);
bool dg_sparse_preferred(const dg_lut *lut, const DgProblem &p);     // AUTO's choice between the two one-hot kernels
dg_status dg_launch_sparse(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
const char *dg_sparse_config_name(const dg_lut *lut, const DgProblem &p);
bool dg_sparse4_supports(const dg_lut *lut, const DgProblem &p);      // 4-bit codes on the sparse instruction
bool dg_sparse4_preferred(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_sparse4(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
bool dg_sparse2p_supports(const dg_lut *lut, const DgProblem &p);     // two-plane 2-bit tables on the sparse instruction
bool dg_sparse2p_preferred(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_sparse2p(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
bool dg_sparse_ws_supports(const dg_lut *lut, const DgProblem &p);    // short K: weight operands stationary in registers
bool dg_sparse_ws_preferred(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_sparse_ws(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
bool dg_sparse_ws_codes_supports(const dg_lut *lut, const DgProblem &p);                       // p.Xp: codes one per byte
dg_status dg_launch_sparse_ws_codes(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
bool dg_fewn_supports(const dg_lut *lut, const DgProblem &p);         // few activation rows: weights as the sparse operand
bool dg_fewn_preferred(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_fewn(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
bool dg_smalln_supports(const dg_lut *lut, const DgProblem &p);
dg_status dg_launch_smalln(const dg_lut *lut, const DgProblem &p, hipStream_t stream);
dg_status dg_launch_smalln_codes(const dg_lut *lut, const DgProblem &p, hipStream_t stream);   // p.Xp: codes one per byte
