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
 *
 * Sec. 3.3 / Table 2 describe (without implementing) the same scheme for 3- and
 * 4-bit codes: index = b + b bits, 2^(2b) entries.  For those widths the functions
 * below take `bits`; a byte then holds TWO codes, each in a 4-bit slot (code k in
 * byte k/2, bits [4*(k%2)+bits-1 : 4*(k%2)]) -- the paper does not give a layout for
 * them, this is this build's reading.  The index is w * 2^bits + a.
 */
#include <stdint.h>

/* table[nlev*w + a] = lw[w] * la[a], nlev = 2^bits levels per side (16 entries for 2 bits, 64, 256) */
void dgo_build_lut(const int32_t *lw, const int32_t *la, int nlev, int32_t *table)
{
    for (int w = 0; w < nlev; ++w)
        for (int a = 0; a < nlev; ++a)
            table[nlev * w + a] = lw[w] * la[a];
}

static int slot_bits(int bits) { return bits == 2 ? 2 : 4; }

/* Pack `count` codes of `bits` bits, 8/slot_bits per byte, by shift and OR. */
int dgo_pack_codes(const uint8_t *codes, int64_t count, int bits, uint8_t *packed)
{
    if (bits < 2 || bits > 4) return 3;
    const int sb = slot_bits(bits), per = 8 / sb;
    if (count < 0 || count % per != 0) return 3;
    for (int64_t j = 0; j < count / per; ++j) {
        uint8_t byte = 0;
        for (int i = 0; i < per; ++i) {
            uint8_t c = codes[per * j + i];
            if (c >= (1 << bits)) return 1;
            byte = (uint8_t)(byte | (c << (sb * i)));
        }
        packed[j] = byte;
    }
    return 0;
}

/* Inverse of dgo_pack_codes: mask each field out again. */
void dgo_unpack_codes(const uint8_t *packed, int64_t count, int bits, uint8_t *codes)
{
    const int sb = slot_bits(bits), per = 8 / sb;
    const uint8_t mask = (uint8_t)((1 << bits) - 1);
    for (int64_t j = 0; j < count / per; ++j)
        for (int i = 0; i < per; ++i)
            codes[per * j + i] = (uint8_t)((packed[j] >> (sb * i)) & mask);
}

/* The code in slot `slot` of a packed byte (slots are `sb` bits apart, a code is `bits` bits wide). */
static unsigned code_in_slot(uint8_t packed, int slot, int sb, int bits)
{
    return (unsigned)(packed >> (slot * sb)) & ((1u << bits) - 1u);
}

/*
 * GEMM by table lookup on packed operands (Algorithm 1 over all rows).  Wp is [M][K/per], Ap is [N][K/per],
 * C is [M][N].  A dot product walks the two rows byte by byte; in every slot of a byte pair the weight code and
 * the activation code side by side (weight code in the high bits) address the table, and the entries are added.
 */
int dgo_lut_gemm_packed(const uint8_t *Wp, const uint8_t *Ap,
                        const int32_t *table, int bits,
                        int64_t M, int64_t N, int64_t K, int32_t *C)
{
    if (bits < 2 || bits > 4) return 3;
    const int sb = slot_bits(bits), per = 8 / sb;
    if (M < 0 || N < 0 || K < 0 || K % per != 0) return 3;
    const int64_t row_bytes = K / per;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            const uint8_t *wrow = Wp + m * row_bytes, *arow = Ap + n * row_bytes;
            int64_t sum = 0;
            for (int64_t j = 0; j < row_bytes; ++j)
                for (int slot = 0; slot < per; ++slot) {
                    const unsigned w = code_in_slot(wrow[j], slot, sb, bits), a = code_in_slot(arow[j], slot, sb, bits);
                    sum += table[(w << bits) | a];
                }
            if (sum > INT32_MAX || sum < INT32_MIN) return 2;
            C[m * N + n] = (int32_t)sum;
        }
    return 0;
}
