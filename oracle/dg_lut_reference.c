/*
 * CPU statement of the table METHOD itself (test infrastructure only).
 *
 * dg_oracle.c states the result (multiply decoded levels).  This file walks the
 * steps of the method in the paper's own order and notation, so that tests can
 * check "table path == explicit multiply" on the CPU, and so that the packed
 * byte format has a definition independent of the GPU library:
 *
 *   - Sec. 3.1: packing puts several 2-bit values into one byte with shifts
 *     and ORs; unpacking masks them out again; the weight code and the
 *     activation code are concatenated into the table index.
 *   - Sec. 3 "LUT-16": the table holds all 16 products w*a.
 *   - Algorithm 1: for i in the four 2-bit slots of a byte, shift = 2*i,
 *     index from the masked weight and activation fields, fetch, then a
 *     reduction sum.  (The printed loop bound "0 to 4" is read as the four
 *     slots 0..3; the printed index ORs two fields masked to the same two
 *     bits, which is read as the concatenation the prose describes:
 *     index = 4*w + a.)
 *
 * Packed layout used here: code k of a row sits in byte k/4, bits
 * [2*(k%4)+1 : 2*(k%4)].  Nothing here is shared with the HIP library.
 */
#include <stdint.h>

/* table[4*w + a] = lw[w] * la[a] */
void dgo_build_lut(const int32_t lw[4], const int32_t la[4], int32_t table[16])
{
    for (int w = 0; w < 4; ++w)
        for (int a = 0; a < 4; ++a)
            table[4 * w + a] = lw[w] * la[a];
}

/* Pack `count` codes (count % 4 == 0), four per byte, by shift and OR. */
int dgo_pack_codes(const uint8_t *codes, int64_t count, uint8_t *packed)
{
    if (count < 0 || count % 4 != 0) return 3;
    for (int64_t j = 0; j < count / 4; ++j) {
        uint8_t byte = 0;
        for (int i = 0; i < 4; ++i) {
            uint8_t c = codes[4 * j + i];
            if (c > 3) return 1;
            byte = (uint8_t)(byte | (c << (2 * i)));
        }
        packed[j] = byte;
    }
    return 0;
}

/* Inverse of dgo_pack_codes: mask each 2-bit field out again. */
void dgo_unpack_codes(const uint8_t *packed, int64_t count, uint8_t *codes)
{
    const uint8_t mask = 3;
    for (int64_t j = 0; j < count / 4; ++j)
        for (int i = 0; i < 4; ++i)
            codes[4 * j + i] = (uint8_t)((packed[j] >> (2 * i)) & mask);
}

/*
 * GEMM by table lookup on packed operands.  Wp is [M][K/4], Ap is [N][K/4],
 * C is [M][N].  The inner loop is Algorithm 1 on one byte at a time.
 */
int dgo_lut_gemm_packed(const uint8_t *Wp, const uint8_t *Ap,
                        const int32_t table[16],
                        int64_t M, int64_t N, int64_t K, int32_t *C)
{
    if (M < 0 || N < 0 || K < 0 || K % 4 != 0) return 3;
    const int64_t KB = K / 4;
    const uint8_t mask = 3;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t sum = 0;
            for (int64_t j = 0; j < KB; ++j) {
                const uint8_t vec_w = Wp[m * KB + j];
                const uint8_t vec_a = Ap[n * KB + j];
                for (int i = 0; i < 4; ++i) {
                    const int shift = i * 2;
                    const int indx = (((vec_w >> shift) & mask) << 2) |
                                     ((vec_a >> shift) & mask);
                    sum += table[indx];
                }
            }
            if (sum > INT32_MAX || sum < INT32_MIN) return 2;
            C[m * N + n] = (int32_t)sum;
        }
    return 0;
}
