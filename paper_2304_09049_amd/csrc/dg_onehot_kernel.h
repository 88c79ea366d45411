// Table lookup on the matrix cores by one-hot selection -- TABLE kernels (they work for any int8 entries, whether or
// not they factor into level vectors), unlike the decode-and-multiply comparison kernel.
//
//   C[m][n] = sum_k T[w(m,k)][a(n,k)] = sum_k sum_{v<L} T[w(m,k)][v] * [a(n,k) == v],      L = 2^BITS levels
//
// so with A'[m][(k,v)] = T[w(m,k)][v] (the table ROW of the weight code, L int8) and B'[n][(k,v)] = [a(n,k) == v]
// (a one-hot run of L bytes) the layer is an int8 contraction of length L*K: each multiply is by 0 or 1, i.e. the
// MFMA unit SELECTS one table entry per reduction position and adds it.  L times the MFMA work of the rank-1 decode
// kernel, but every table is accepted and the VALU only expands codes.  BITS = 2 is the paper's LUT-16 (Sec. 3);
// BITS = 3 and 4 are the 64- and 256-entry tables of its Sec. 3.3 / Table 2 (codes two per byte in 4-bit slots).
//
// Expansion, without LDS: the order of the (k,v) axis is free as long as both operands use the same one, so the 16
// operand bytes of a lane are laid out value-major: each dword holds, for ONE value v and 4 reduction positions,
// T[w(k)][v] (weights) or [a(k) == v] (activations); a lane's operand of one MFMA step is the 4 dwords of a group of
// 4 values, and a selector of 4 positions feeds L/4 steps.  With the codes of a packed word's four bytes spread into
// the bytes of a selector ((word >> slot) & mask), a dword is a byte permute (v_perm_b32 picks 4 bytes out of 8):
//   weights      BITS 2: of the 4 bytes T[0..3][v];  BITS 3: of the 8 bytes T[0..7][v];
//                BITS 4: of T[0..7][v] with the selector of the codes below 8, OR'd with that of T[8..15][v] with
//                the selector of the codes from 8 up (each selector reads 0x0C = "constant 0" where it does not apply)
//   activations  of a constant holding a single 1 at byte v % 4, in the lower or upper permute source as v / 4 says
// A filter tap outside the image, or a column beyond N, gets selector bytes 0x0C: it selects nothing.
//
// BITS = 0 is not a table kernel but the measured comparison, built in the same frame so that it has every advantage
// the table kernels have (tiles, K sharing, split K, epilogues): tables that are outer products of level vectors make
// the layer a plain int8 contraction, so the operands are the decoded levels themselves -- a dword of 4 positions is a
// byte permute of the 4 weight (activation) levels, an MFMA step consumes a whole packed word (16 positions) per lane,
// and the MFMA work is a quarter of the 2-bit one-hot kernel's.
//
// BITS = 20 is the 2-bit table kernel on the SPARSE matrix instruction (v_smfmac_i32_32x32x64_i8), at half the matrix
// work.  A one-hot run of 4 bytes is 1-of-4 sparse, and that instruction takes one operand as two kept bytes out of
// every four plus their 2-bit positions -- which, for a one-hot run, are the constant bytes (1, 0) and the CODE itself.
// So the activation operand needs no expansion at all: its values are a constant and its index register is the packed
// word itself -- a 4-bit field of it holds an even and an odd code, the indices of the first and the second kept byte,
// so with kept bytes (1, 0) the instruction selects by the even codes, and by the odd ones with kept bytes (0, 1) or
// with the word shifted by one code (the byte that is 0 may select anything) -- and the hardware's index multiplexer
// performs the table lookup: it picks, out of the 4 bytes T[w(k)][0..3] that the dense operand holds for a
// position, the entry of the activation code.  The dense operand is a dword per position, the table ROW of the weight
// code, fetched from a 16-entry table of row pairs in LDS (one 8-byte read serves two positions, without bank
// conflicts).  One instruction covers 16 positions per lane pair in the time the dense MFMA takes for 8.
// Layout of that instruction (measured): with A the sparse operand (rows), lane (row, h) holds kept bytes j = 0..15
// and 2-bit fields j of its index register; byte j multiplies byte 16h + 4((j % 8) / 2) + field_j of the dense lane
// (column, j / 8).  The accumulator layout is the dense instruction's.
//
// Entries beyond int8 (2-bit codes only): the table is split into two int8 planes, T = 256 * hi + lo with
// lo = ((T + 128) mod 256) - 128, each selected into an accumulator of its own (the two planes take the places of the
// tile's two weight row blocks, so a tile covers 32 rows instead of 64), and the result is 256 * acc_hi + acc_lo.
#pragma once

#include "dg_codes.h"
#include "dg_mfma_tile.h"

namespace dgoh {

typedef dg_v4i v4i;
typedef dg_v16i v16i;

// pool[v * (L/4) + q] = bytes T[4q .. 4q+3][v] (signed int8, as stored): column v of the table, 4 weight codes per word.
// A second plane (two-plane tables, 2-bit codes) sits at word 32.
struct Pools {
    uint32_t w[64];
};

typedef DgFastDiv FastDiv;

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) { return dg_fdiv(n, f); }
inline FastDiv make_div(uint32_t d) { return dg_make_div(d); }

struct Args {
    DgProblem p;
    Pools pools;
    FastDiv div_ow, div_oh, div_cin, div_kw;
    int32_t tiles_m;
    int64_t wave_tiles;
    // dg_sparse_staged_kernel.h: division by the 32-byte runs of packed codes per filter tap; tile numbering in bands
    FastDiv div_runs, div_band, div_last, div_cpt;
    int32_t tiles_n, band_log2, m_log2;
    uint32_t band_tiles;
    // dg_sparse_staged_kernel.h: what was added to every table entry (the sums start at minus this per position of K)
    int32_t bias;
};

struct SplitArgs {
    DgProblem p;
    Pools pools;
    FastDiv div_ow, div_oh, div_cin, div_kw;
    int32_t tiles_m;
    int32_t chunks;          // K / (codes per chunk)
    int32_t cpw;             // chunks per wavefront
};

template <int BITS>
struct Fmt {
    static constexpr bool DECODE = BITS == 0;                   // the decode-and-multiply comparison (2-bit codes)
    static constexpr bool SPARSE = BITS == 20;                  // 2-bit codes selected by the sparse MFMA's index
    static constexpr int SLOT = (BITS == 2 || DECODE || SPARSE) ? 2 : 4;  // bits per code slot in a packed byte
    static constexpr int PER_BYTE = 8 / SLOT;                  // codes per packed byte
    static constexpr int SELS = DECODE ? 1 : 8 / SLOT;         // selectors per 32-bit word (decode: the word itself)
    static constexpr int GROUPS = DECODE ? 1 : (1 << BITS) / 4; // MFMA steps per selector: groups of 4 values
    static constexpr int STEPS = SELS * GROUPS;                // MFMA steps per 32-bit word
    static constexpr uint32_t MASK = ((1u << (DECODE ? 2 : BITS)) - 1u) * 0x01010101u;
    static constexpr int QW = DECODE ? 1 : (1 << BITS) / 4;    // pool words per value
    // rough VALU instruction counts of building one operand of one step (for the scheduling groups)
    static constexpr int VALU_W = BITS == 4 ? 14 : (DECODE ? 11 : 6);
    static constexpr int VALU_A = BITS == 4 ? 7 : (DECODE ? 15 : 6);
};

template <int CH>
struct Words {
    uint32_t v[CH];
};

template <int CH>
__device__ __forceinline__ Words<CH> load_words(const uint8_t *ptr)
{
    Words<CH> w;
    if (CH == 4) {
        const uint4 t = *(const uint4 *)ptr;
        w.v[0] = t.x, w.v[1 % CH] = t.y, w.v[2 % CH] = t.z, w.v[3 % CH] = t.w;
    } else if (CH == 2) {
        const uint2 t = *(const uint2 *)ptr;
        w.v[0] = t.x, w.v[1 % CH] = t.y;
    } else {
        w.v[0] = *(const uint32_t *)ptr;
    }
    return w;
}

// CH up to 8: two 128-bit loads
template <int CH>
__device__ __forceinline__ Words<CH> load_words_any(const uint8_t *ptr)
{
    if constexpr (CH <= 4) {
        return load_words<CH>(ptr);
    } else {
        static_assert(CH == 8 || CH == 16, "1, 2, 4, 8 or 16 words");
        Words<CH> w;
#pragma unroll
        for (int q = 0; q < CH / 4; ++q) {
            const Words<4> part = load_words<4>(ptr + 16 * q);
#pragma unroll
            for (int i = 0; i < 4; ++i) w.v[4 * q + i] = part.v[i];
        }
        return w;
    }
}

// The same words from codes that are still one per byte (the run-time packing stage done in the load stage).
template <int CH>
__device__ __forceinline__ Words<CH> load_codes(const uint8_t *ptr)
{
    uint4 t[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) t[i] = ((const uint4 *)ptr)[i];
    Words<CH> w;
#pragma unroll
    for (int i = 0; i < CH; ++i) w.v[i] = dg_pack_codes16(t[i]);
    return w;
}

// Selector of 4 reduction positions.  BITS < 4: `lo` holds the codes.  BITS 4: `lo` the codes below 8 (0x0C
// elsewhere), `hi` the codes from 8 up, minus 8 (0x0C elsewhere).
struct Sel {
    uint32_t lo, hi;
};

constexpr uint32_t NOTHING = 0x0C0C0C0Cu;                      // permute selector bytes that read as 0

template <int BITS>
__device__ __forceinline__ Sel make_sel(uint32_t word, int j, bool valid)
{
    typedef Fmt<BITS> F;
    // decoding: the packed word and what to OR into its selectors (an invalid tap: word 0, every selector "zero byte")
    if (F::DECODE) return Sel{valid ? word : 0u, valid ? 0u : NOTHING};
    const uint32_t raw = (word >> (F::SLOT * j)) & F::MASK;
    Sel s;
    if (BITS == 4) {
        const uint32_t flag = (raw & 0x08080808u) >> 3;          // 1 in the bytes whose code is 8 or more
        const uint32_t up = (flag << 8) - flag;                  // 0xFF in those bytes
        s.lo = (up & NOTHING) | (~up & raw);
        s.hi = (up & (raw & 0x07070707u)) | (~up & NOTHING);
        if (!valid) s.lo = NOTHING, s.hi = NOTHING;
    } else {
        s.lo = valid ? raw : NOTHING;
        s.hi = 0;
    }
    return s;
}

// the weight operand of value group g: T[w(k)][4g + i] for the selector's 4 positions, i = 0..3
template <int BITS>
__device__ __forceinline__ v4i weight_operand(const Pools &pl, Sel s, int g, int plane = 0)
{
    typedef Fmt<BITS> F;
    v4i r;
    if (F::DECODE) {                                           // dword i: the levels of code i of the word's four bytes
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (int)__builtin_amdgcn_perm(0u, pl.w[0], (s.lo >> (2 * i)) & 0x03030303u);
        return r;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t *c = pl.w + 32 * plane + (4 * g + i) * F::QW;
        uint32_t d;
        if (BITS == 2)
            d = __builtin_amdgcn_perm(0u, c[0], s.lo);
        else if (BITS == 3)
            d = __builtin_amdgcn_perm(c[1 % F::QW], c[0], s.lo);
        else
            d = __builtin_amdgcn_perm(c[1 % F::QW], c[0], s.lo) | __builtin_amdgcn_perm(c[3 % F::QW], c[2 % F::QW], s.hi);
        r[i] = (int)d;
    }
    return r;
}

// the activation operand of value group g: [a(k) == 4g + i]
template <int BITS>
__device__ __forceinline__ v4i onehot_operand(const Pools &pl, Sel s, int g)
{
    v4i r;
    if (Fmt<BITS>::DECODE) {                                   // the activation levels (pool word 1); invalid: zeros
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (int)__builtin_amdgcn_perm(0u, pl.w[1], ((s.lo >> (2 * i)) & 0x03030303u) | s.hi);
        return r;
    }
    const uint32_t sel = (BITS == 4 && g >= 2) ? s.hi : s.lo;   // values 8..15 of 4-bit codes use the upper selector
    const bool upper = (g & 1) != 0;                            // values 4..7 (12..15): the permute's upper source
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t one = 1u << (8 * i);
        r[i] = (int)(upper ? __builtin_amdgcn_perm(one, 0u, sel) : __builtin_amdgcn_perm(0u, one, sel));
    }
    return r;
}

template <int N>
__device__ __forceinline__ void sched_valu()
{
    __builtin_amdgcn_sched_group_barrier(0x002, N, 0);
}

typedef int v8i __attribute__((ext_vector_type(8)));

// Sparse-instruction form (BITS = 20).  Per wavefront, 16 entries of 8 bytes in LDS: entry (c0 | c1 << 2) holds the
// table rows of weight codes c0 and c1, row w = bytes T[w][0..3] (pool words 0..3).  A wavefront writes and reads only
// its own copy, so no barrier is involved (LDS operations of one wavefront execute in order).
__device__ __forceinline__ void sparse_fill_rows(uint2 *rows, const Pools &pl, int lane)
{
    if (lane < 16) {
        const int c0 = lane & 3, c1 = lane >> 2;
        const uint32_t r0 = c0 == 0 ? pl.w[0] : (c0 == 1 ? pl.w[1] : (c0 == 2 ? pl.w[2] : pl.w[3]));
        const uint32_t r1 = c1 == 0 ? pl.w[0] : (c1 == 1 ? pl.w[1] : (c1 == 2 ? pl.w[2] : pl.w[3]));
        rows[lane] = make_uint2(r0, r1);
    }
    __builtin_amdgcn_wave_barrier();
}

// The dense operands of the two instructions (even codes, odd codes) that consume one packed word per lane half.  w0
// and w1 are the weight row's words at the positions of lane half 0's and lane half 1's activation words; this lane
// supplies the rows of their codes 8*half .. 8*half+7, i.e. of one 16-bit half of each word -- `pick` is the byte
// permute that puts those two halves side by side (see sparse_pick) -- as dwords 0-3 (from w0) and 4-7 (from w1) of the
// two operands: the even codes to `even`, the odd ones to `odd` (see the layout above).  Two codes two apart are first
// brought together as a 4-bit table index, for both words at once, so that one 8-byte read fills two consecutive
// operand registers.
__device__ __forceinline__ uint32_t sparse_pick(int half)
{
    return half ? 0x07060302u : 0x05040100u;                     // bytes 2,3 (or 0,1) of the lower source, then of the upper
}

__device__ __forceinline__ void sparse_dense_rows(const uint2 *rows, uint32_t w0, uint32_t w1, uint32_t pick, v8i &even, v8i &odd)
{
    const uint32_t v = __builtin_amdgcn_perm(w1, w0, pick), t = v >> 2;
    const uint32_t e = (v & 0x03030303u) | (t & 0x0C0C0C0Cu);    // byte b: codes 4b and 4b+2 of the 32 bits
    const uint32_t o = (t & 0x03030303u) | ((v >> 4) & 0x0C0C0C0Cu);    // byte b: codes 4b+1 and 4b+3
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const uint2 x = rows[(e >> (8 * b)) & 255u], y = rows[(o >> (8 * b)) & 255u];
        even[2 * b] = (int)x.x, even[2 * b + 1] = (int)x.y;
        odd[2 * b] = (int)y.x, odd[2 * b + 1] = (int)y.y;
    }
}

// The same with ONE table for the whole workgroup, at a fixed LDS address: threads 0-15 fill it and the workgroup meets
// at a barrier before the first read.  A read's address is then nothing but the 4-bit index times 8, and with the
// indices kept pre-multiplied, a byte each, it is one bit-field extract per read (three instructions per read otherwise:
// shift, mask, add the wavefront's table base).
__device__ __forceinline__ void sparse_fill_table(uint2 *table, const Pools &pl, int tid)
{
    if (tid < 16) {
        const int c0 = tid & 3, c1 = tid >> 2;
        const uint32_t r0 = c0 == 0 ? pl.w[0] : (c0 == 1 ? pl.w[1] : (c0 == 2 ? pl.w[2] : pl.w[3]));
        const uint32_t r1 = c1 == 0 ? pl.w[0] : (c1 == 1 ? pl.w[1] : (c1 == 2 ? pl.w[2] : pl.w[3]));
        table[tid] = make_uint2(r0, r1);
    }
}

__device__ __forceinline__ void sparse_dense_rows_shared(const uint2 *table, uint32_t w0, uint32_t w1, uint32_t pick, v8i &even, v8i &odd)
{
    const uint32_t v = __builtin_amdgcn_perm(w1, w0, pick), t = v >> 2;
    uint32_t e = ((v & 0x03030303u) | (t & 0x0C0C0C0Cu)) << 3;          // byte b: 8 * (code 4b | code 4b+2 << 2)
    uint32_t o = ((t & 0x03030303u) | ((v >> 4) & 0x0C0C0C0Cu)) << 3;   // byte b: 8 * (code 4b+1 | code 4b+3 << 2)
    // (kept as they are: a byte of them IS an LDS offset; left to itself the compiler folds the multiplication into a
    // shift and a mask per read)
    asm volatile("" : "+v"(e), "+v"(o));
    const char *base = (const char *)table;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const uint2 x = *(const uint2 *)(base + ((e >> (8 * b)) & 255u)), y = *(const uint2 *)(base + ((o >> (8 * b)) & 255u));
        even[2 * b] = (int)x.x, even[2 * b + 1] = (int)x.y;
        odd[2 * b] = (int)y.x, odd[2 * b + 1] = (int)y.y;
    }
}

// Position bookkeeping shared by the two kernels: output column n -> image coordinates, and the filter tap of a chunk.
// Workgroups are dealt to the 8 XCDs, each with an L2 of its own, round-robin.  Renumbered this way each XCD works on a
// contiguous run of tiles, so that neighbouring pixels' filter windows and a tile row's weights meet in one L2
// (any bijection is correct; this one is a guess at the dealing order that costs nothing when it is wrong).
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t block, uint32_t blocks)
{
    const uint32_t per = blocks / 8, rem = blocks % 8, x = block % 8, i = block / 8;
    return x * per + min(x, rem) + i;
}

struct Column {
    bool ok;
    int ih0, iw0;
    int64_t off0;
};

__device__ __forceinline__ Column make_column(const DgProblem &p, const FastDiv &div_ow, const FastDiv &div_oh, int n,
                                              int bytes_per_pixel, int lane_byte)
{
    Column c;
    c.ok = n < p.N;
    const int nn = c.ok ? n : 0;
    const int t = (int)fdiv((uint32_t)nn, div_ow), ow = nn - t * p.OW;
    const int b = (int)fdiv((uint32_t)t, div_oh), oh = t - b * p.OH;
    c.ih0 = oh * p.sh - p.ph;
    c.iw0 = ow * p.sw - p.pw;
    c.off0 = (((int64_t)b * p.H + c.ih0) * p.W + c.iw0) * bytes_per_pixel + lane_byte;
    return c;
}

// Large layers: each wavefront owns a (WM*32) x (WN*32) tile; operands come straight from global memory (L2), one
// chunk ahead.  SKW = 1: a wavefront walks all of K, there is no LDS and no barrier.  SKW = 2 or 4 (layers whose tiles
// alone would leave SIMDs idle or with a single wavefront): SKW wavefronts of the workgroup share a tile and split K
// between them in contiguous runs of chunks; their accumulators meet in LDS by integer atomics (exact in any order)
// and each of them stores a share of the tile's blocks.
// RAW (the narrow tiles of 2-bit codes on the dense instruction): the activations are codes one per byte and are
// packed in registers as they are loaded -- once per 64-row tile; on layers of a few microseconds that is less than
// the launch of the packing kernel.
template <int BITS, int WM, int WN, int CH, bool TR, bool TWO, int SKW, bool RAW = false>
__global__ void __launch_bounds__(256, (WM * WN > 8 ? 1 : 2))
onehot_mfma_kernel(Args a)
{
    typedef Fmt<BITS> F;
    static_assert(!RAW || ((BITS == 2 || BITS == 20) && !TWO), "unpacked activations: 2-bit codes, one plane");
    static_assert(!TWO || (WM == 2 && BITS == 2), "two planes stand in for the two weight row blocks of 2-bit tiles");
    static_assert(BITS == 0 || BITS == 2 || BITS == 3 || BITS == 4 || BITS == 20,
                  "code widths 2, 3, 4; 0 = the decode comparison; 20 = 2-bit codes on the sparse instruction");
    static_assert(!F::SPARSE || (TR && !TWO), "the sparse operand is the MFMA's row operand: activations on the rows");
    constexpr int RB = TWO ? 1 : WM;                       // weight row blocks of 32 rows
    constexpr int WRUNS = F::SPARSE ? 2 : 1;               // runs of CH words a weight lane reads: its half's, or both
    __shared__ uint2 s_rows[F::SPARSE ? 16 : 1];            // the sparse form's table of row pairs, one for the workgroup
    constexpr int TPW = 4 / SKW;                           // tiles per workgroup
    constexpr int NB = RB * WN;                            // 32x32 output blocks per tile
    extern __shared__ int32_t s_acc[];                      // SKW > 1: [TPW][NB][16][64] sums
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, w4 = threadIdx.x >> 6;
    const int ks = w4 % SKW, tw = w4 / SKW;                 // this wavefront's share of K, and its tile within the workgroup
    const int64_t my_tile = (int64_t)xcd_contiguous(blockIdx.x, gridDim.x) * TPW + tw;
    const bool active = my_tile < a.wave_tiles;
    if (F::SPARSE) {
        sparse_fill_table(s_rows, a.pools, threadIdx.x);
        __syncthreads();                                   // (every wavefront of the workgroup, also one without a tile)
    }
    if (SKW == 1 && !active) return;                       // whole waves leave; no barrier follows on this path
    const int64_t wave_tile = active ? my_tile : 0;        // (an idle wavefront of a shared workgroup adds zeros)
    if (SKW > 1)
        for (int i = threadIdx.x; i < TPW * NB * 1024; i += 256) s_acc[i] = 0;
    const int r = lane & 31, h = lane >> 5;
    const int m0 = (int)(wave_tile % a.tiles_m) * (RB * 32);
    const int n0 = (int)(wave_tile / a.tiles_m) * (WN * 32);
    const int cq = p.Cin / F::PER_BYTE;                     // packed bytes per pixel
    constexpr int CHUNK = 8 * CH * F::PER_BYTE;             // codes of K per chunk: 4*CH packed bytes per lane half
    const int chunks = p.K / CHUNK;
    const int cps = (chunks + SKW - 1) / SKW;               // chunks per share of K
    const int c0 = min(ks * cps, chunks), c1 = active ? min(c0 + cps, chunks) : c0;

    const uint8_t *w_ptr[RB];
#pragma unroll
    for (int bm = 0; bm < RB; ++bm) {
        int m = m0 + bm * 32 + r;
        if (m >= p.M) m = p.M - 1;
        w_ptr[bm] = p.Wp + (int64_t)m * (p.K / F::PER_BYTE) + (F::SPARSE ? 0 : h * (4 * CH));
    }
    Column col[WN];
    constexpr int LANE_BYTE = RAW ? 16 * CH : 4 * CH;      // activation bytes a lane half reads per chunk
    const int bpp = RAW ? p.Cin : cq;                       // activation bytes per pixel
#pragma unroll
    for (int bn = 0; bn < WN; ++bn) col[bn] = make_column(p, a.div_ow, a.div_oh, n0 + bn * 32 + r, bpp, h * LANE_BYTE);

    v16i acc[WM][WN];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[bm][bn][e] = 0;
    float sc_cols[RB];                                      // the epilogue's scales, fetched now
    dg_mfma_column_scales<RB, TR>(p, m0, lane, sc_cols);

    // filter tap of this wavefront's first chunk
    int kh = 0, kw = 0, ci = 0;
    if (SKW > 1) {
        const int pos = c0 * CHUNK, tap = (int)fdiv((uint32_t)pos, a.div_cin);
        kh = (int)fdiv((uint32_t)tap, a.div_kw);
        kw = tap - kh * p.KW;
        ci = pos - tap * p.Cin;
    }
    Words<CH> wa[RB][WRUNS], wb[WN];
    // Where the next chunk's words of each column are read, and whether that filter tap lies inside the image.  A tap
    // outside the image points at the first pixel instead and is masked by its selector: the loads are unconditional,
    // because a load under a branch would make the compiler wait for it at once and the prefetch would hide nothing.
    // STEPPED (the sparse instruction's widest tile, where every VALU instruction is paid in full -- that instruction
    // does not overlap with them): offsets and validity are recomputed only when the walk enters a new tap and just
    // stepped by a chunk otherwise, and the kept bytes are rebuilt per tap too (VGG layer 61.4 -> 58.6 us, 8192-cube
    // 946 -> 931 us).  On the other tiles and forms that was measured 2 - 20 % slower, so they recompute per chunk.
    // (32-bit byte offsets from the activations' base: the host sends only inputs of less than 2^31 packed bytes here)
    constexpr bool STEPPED = F::SPARSE && SKW == 1 && WN == 4;
    uint32_t x_off[STEPPED ? WN : 1];
    bool vb[WN];
    bool starts_tap = true;                                  // the chunk fetched last is the first of its tap (or of the share)
    auto next_position = [&]() {                             // (kh, kw, ci) of the chunk after this one; true: a new tap
        ci += CHUNK;
        if (ci != p.Cin) return false;
        ci = 0;
        if (++kw == p.KW) {
            kw = 0;
            ++kh;
        }
        return true;
    };
    auto enter_tap = [&]() {
        if constexpr (STEPPED) {
            const int32_t tap_off = (kh * p.W + kw) * cq + ci / F::PER_BYTE;
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) {
                const int ih = col[bn].ih0 + kh, iw = col[bn].iw0 + kw;
                vb[bn] = col[bn].ok & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
                // (outside: the first pixel at the same channel offset, so that stepping stays inside that pixel)
                x_off[bn] = vb[bn] ? (uint32_t)((int32_t)col[bn].off0 + tap_off) : (uint32_t)(h * (4 * CH) + ci / F::PER_BYTE);
            }
        }
    };
    enter_tap();
    auto fetch = [&](int chunk) {                            // `chunk` is clamped: a fetch past the share is unused
        const int cw = min(chunk, chunks - 1);
#pragma unroll
        for (int bm = 0; bm < RB; ++bm)
#pragma unroll
            for (int run = 0; run < WRUNS; ++run)
                wa[bm][run] = load_words<CH>(w_ptr[bm] + (int64_t)cw * (8 * CH) + run * (4 * CH));
        if constexpr (STEPPED) {
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) wb[bn] = load_words<CH>(p.Xp + x_off[bn]);
        } else {
            const int64_t tap_off = ((int64_t)kh * p.W + kw) * bpp + (RAW ? ci : ci / F::PER_BYTE);
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) {
                const int ih = col[bn].ih0 + kh, iw = col[bn].iw0 + kw;
                vb[bn] = col[bn].ok & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
                const uint8_t *ptr = vb[bn] ? p.Xp + col[bn].off0 + tap_off : p.Xp + h * LANE_BYTE;
                if constexpr (RAW)
                    wb[bn] = load_codes<CH>(ptr);
                else
                    wb[bn] = load_words<CH>(ptr);
            }
            next_position();
        }
    };
    auto advance = [&]() {                                   // STEPPED: to the chunk after the one fetched last
        starts_tap = next_position();
        if (starts_tap) {                                    // (uniform)
            enter_tap();
        } else {
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) x_off[bn] += CHUNK / F::PER_BYTE;
        }
    };

    fetch(c0);
    // every wavefront's zeroes are in LDS before any wavefront adds to them; the loads above stay in flight across
    // this barrier (it waits for LDS only)
    if (SKW > 1) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    v4i ones[F::SPARSE ? WN : 1];                            // sparse form: the kept bytes of the one-hot operand
    for (int c = c0; c < c1; ++c) {
        Words<CH> ca[RB], ca1[RB], cb[WN];
        bool valid[WN];
#pragma unroll
        for (int bm = 0; bm < RB; ++bm) ca[bm] = wa[bm][0], ca1[bm] = wa[bm][WRUNS - 1];
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            cb[bn] = wb[bn];
            valid[bn] = vb[bn];
        }
        const bool new_tap = starts_tap;                    // of the chunk about to be computed
        if constexpr (STEPPED) advance();
        fetch(c + 1 < c1 ? c + 1 : c);                      // unconditional (the last one re-reads in bounds and is unused)
        if constexpr (F::SPARSE) {
            // The kept bytes: (1, 0) per position, or zeros for a tap outside the image; they change with the tap only.
            // The index register is the packed word as it is for the even codes and shifted by one code for the odd
            // ones: of a 4-bit field the low half is the index of the first kept byte (the 1), and what the high half
            // makes the second kept byte (the 0) pick does not matter.  (Kept bytes (0, 1) would spare the shift too,
            // but a second set of them does not fit the widest tile's registers.)
            if (!STEPPED || new_tap) {
#pragma unroll
                for (int bn = 0; bn < WN; ++bn) {
                    const int x = valid[bn] ? 0x00010001 : 0;
                    ones[bn] = (v4i){x, x, x, x};
                }
            }
            // Step t = the chunk's word t: two instructions (even codes, odd codes) per block of the tile.  The operands
            // of step t+1 -- per weight block a unit of table reads, per activation block a shift -- are made between
            // the instructions of step t.
            v8i dn[2][WM][2];
            int odd_ix[2][WN];
            const uint32_t pick = sparse_pick(h);
            auto prepare = [&](int t, int u, int buf) {      // unit u < WM: a weight block; else an activation block
                if (u < WM)
                    sparse_dense_rows_shared(s_rows, ca[u].v[t], ca1[u].v[t], pick, dn[buf][u][0], dn[buf][u][1]);
                else
                    odd_ix[buf][u - WM] = (int)(cb[u - WM].v[t] >> 2);
            };
            constexpr int U = WM + WN, MN = WM * WN;
#pragma unroll
            for (int u = 0; u < U; ++u) prepare(0, u, 0);
#pragma unroll
            for (int t = 0; t < CH; ++t) {
                const int cur = t & 1;
#pragma unroll
                for (int i = 0; i < 2 * MN; ++i) {
                    const int par = i / MN, bm = (i % MN) / WN, bn = i % WN;      // all blocks with the even codes, then the odd
                    acc[bm][bn] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones[bn], dn[cur][bm][par], acc[bm][bn],
                                                                          par ? odd_ix[cur][bn] : (int)cb[bn].v[t], 0, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (t + 1 < CH) {
                        // the table reads go first (over the first instructions) so that their latency is covered
                        const int u0 = i * U / (2 * MN), u1 = (i + 1) * U / (2 * MN);
#pragma unroll
                        for (int u = u0; u < u1; ++u) {
                            prepare(t + 1, u, cur ^ 1);
                            if (u < WM)
                                __builtin_amdgcn_sched_group_barrier(0x102, 31, 0);      // 23 VALU and 8 LDS reads
                            else
                                __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
                        }
                    }
                }
            }
            continue;
        }
        // Step t = one MFMA per block of the tile: word t / STEPS, selector j of it, value group g.  The operands of
        // step t+1 are built between the MFMAs of step t so that the matrix unit and the VALU of a single wavefront
        // overlap; the scheduling groups pin that interleaving.
        constexpr int T = F::STEPS * CH;
        v4i fa[2][WM], fb[2][WN];
        Sel sa[RB], sb[WN];
        auto expand = [&](int t, int u, int buf) {           // operand u of step t: u < WM weights, else activations
            const int word = t / F::STEPS, j = (t % F::STEPS) / F::GROUPS, g = t % F::GROUPS;
            if (u < WM) {
                const int rb = TWO ? 0 : u, plane = TWO ? u : 0;    // two planes: one row block, selector made once
                if (g == 0 && plane == 0) sa[rb] = make_sel<BITS>(ca[rb].v[word], j, true);
                fa[buf][u] = weight_operand<BITS>(a.pools, sa[rb], g, plane);
            } else {
                if (g == 0) sb[u - WM] = make_sel<BITS>(cb[u - WM].v[word], j, valid[u - WM]);
                fb[buf][u - WM] = onehot_operand<BITS>(a.pools, sb[u - WM], g);
            }
        };
#pragma unroll
        for (int u = 0; u < WM + WN; ++u) expand(0, u, 0);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int cur = t & 1;
#pragma unroll
            for (int i = 0; i < WM * WN; ++i) {
                const int bm = i / WN, bn = i % WN;
                acc[bm][bn] = dg_mfma_step<TR>(fa[cur][bm], fb[cur][bn], acc[bm][bn]);
                // the WM + WN operands of the next step are spread evenly over the WM * WN MFMAs of this one
                constexpr int U = WM + WN, MN = WM * WN;
                const int u0 = i * U / MN, u1 = (i + 1) * U / MN;
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                         // one MFMA ...
                if (t + 1 < T) {
#pragma unroll
                    for (int u = u0; u < u1; ++u) {
                        expand(t + 1, u, cur ^ 1);
                        if (u < WM)
                            sched_valu<F::VALU_W>();                                       // ... then that VALU work
                        else
                            sched_valu<F::VALU_A>();
                    }
                }
            }
        }
    }

    // the tile's blocks as they go to memory: two planes merge into one block row, 256 * hi + lo
    v16i out[RB][WN];
#pragma unroll
    for (int bm = 0; bm < RB; ++bm)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                out[bm][bn][e] = TWO ? (int)((uint32_t)acc[0][bn][e] + ((uint32_t)acc[WM - 1][bn][e] << 8)) : acc[bm][bn][e];
    if (SKW == 1) {
        dg_mfma_store_tile<RB, WN, TR>(p, out, m0, n0, lane, sc_cols);
        return;
    }
    int32_t *sums = s_acc + tw * (NB * 1024);
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            __hip_atomic_fetch_add(&sums[(i * 16 + e) * 64 + lane], out[i / WN][i % WN][e], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
    __syncthreads();
    if (!active) return;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        if (i % SKW != ks) continue;                        // each wavefront of the tile stores a share of its blocks
        v16i blk;
#pragma unroll
        for (int e = 0; e < 16; ++e) blk[e] = sums[(i * 16 + e) * 64 + lane];
        dg_mfma_store_block<TR>(p, blk, m0 + (i / WN) * 32, n0 + (i % WN) * 32, lane, sc_cols[i / WN]);
    }
}

// Small layers: too few 64 x 32 tiles to occupy the chip, and a wavefront that walks all of K alone pays the memory
// latency once per chunk.  Here a workgroup owns ONE 32 x 32 output block and its S wavefronts split K between them
// (whole chunks each), so a layer with T blocks puts T*S wavefronts in flight and each of them waits for memory once
// or twice.  Partial blocks meet in LDS: every wavefront adds its 16 accumulator registers to the block's sums with
// LDS integer atomics (exact in any order), one barrier, then the threads scale and store the sums -- 128 contiguous
// bytes per half wavefront, as in the large-layer kernel.
// RAW: the activations are codes one per byte ([pixel][Cin] bytes at p.Xp) and are packed in registers as they are
// loaded, which saves a layer this small the launch of the packing kernel (as long as the whole layer itself).
template <int BITS, int CH, bool TR, bool TWO, bool RAW = false>
__global__ void __launch_bounds__(1024)
onehot_splitk_kernel(SplitArgs a)
{
    typedef Fmt<BITS> F;
    static_assert(!F::SPARSE || (TR && !TWO), "the sparse operand is the MFMA's row operand: activations on the rows");
    static_assert(!RAW || BITS == 2, "unpacked activations: 2-bit codes on the dense instruction");
    __shared__ int32_t s_sum[16 * 64];                      // the block's sums, [accumulator register][lane]
    __shared__ uint2 s_rows[F::SPARSE ? 16 * 16 : 1];
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, ws = threadIdx.x >> 6;
    for (int idx = threadIdx.x; idx < 1024; idx += blockDim.x) s_sum[idx] = 0;
    const int r = lane & 31, h = lane >> 5;
    const int block = (int)xcd_contiguous(blockIdx.x, gridDim.x);
    const int m0 = (block % a.tiles_m) * 32;
    const int n0 = (block / a.tiles_m) * 32;
    const int cq = p.Cin / F::PER_BYTE;
    constexpr int CHUNK = 8 * CH * F::PER_BYTE;
    // every wavefront has at least one chunk (the host sizes S that way); the max only keeps an odd launch harmless
    const int c0 = ws * a.cpw, c1 = max(c0, min(c0 + a.cpw, a.chunks));

    v16i acc, acc_hi;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0, acc_hi[e] = 0;

    // The prologue is most of this kernel's life, so it is ordered for latency: the weight load needs no division and
    // goes first; the scale of the epilogue (NHWC: one channel per thread whatever element it sums) is fetched now.
    const int mw = min(m0 + r, p.M - 1);
    const uint8_t *w_ptr = p.Wp + (int64_t)mw * (p.K / F::PER_BYTE) + (F::SPARSE ? 0 : h * (4 * CH));
    Words<CH> wa = load_words<CH>(w_ptr + (int64_t)min(c0, a.chunks - 1) * (8 * CH)), wa1 = wa, wb;
    if (F::SPARSE) wa1 = load_words<CH>(w_ptr + (int64_t)min(c0, a.chunks - 1) * (8 * CH) + 4 * CH);
    float sc = 0.0f;
    if (TR && p.scale) sc = p.scale[mw];
    if (F::SPARSE) sparse_fill_rows(s_rows + 16 * ws, a.pools, lane);
    {
        constexpr int LANE_BYTE = RAW ? 16 * CH : 4 * CH;  // bytes a lane half reads per chunk
        const int bpp = RAW ? p.Cin : cq;                  // activation bytes per pixel
        const Column col = make_column(p, a.div_ow, a.div_oh, n0 + r, bpp, h * LANE_BYTE);
        // filter tap of this wavefront's first chunk
        const int pos = c0 * CHUNK, tap = (int)fdiv((uint32_t)pos, a.div_cin), tkh = (int)fdiv((uint32_t)tap, a.div_kw);
        int ci = pos - tap * p.Cin, kh = tkh, kw = tap - tkh * p.KW;

        bool vb;
        auto fetch_x = [&]() {
            const int ih = col.ih0 + kh, iw = col.iw0 + kw;
            vb = col.ok & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
            const int64_t tap_off = ((int64_t)kh * p.W + kw) * bpp + (RAW ? ci : ci / F::PER_BYTE);
            const uint8_t *ptr = vb ? p.Xp + col.off0 + tap_off : p.Xp + h * LANE_BYTE;
            if constexpr (RAW)
                wb = load_codes<CH>(ptr);
            else
                wb = load_words<CH>(ptr);
            ci += CHUNK;
            if (ci == p.Cin) {
                ci = 0;
                if (++kw == p.KW) {
                    kw = 0;
                    ++kh;
                }
            }
        };
        fetch_x();
        // every wavefront's zeroes are in LDS before any wavefront adds to them; the global loads issued above stay in
        // flight across this barrier (it waits for LDS only), so the wavefronts' staggered starts cost nothing here
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        for (int c = c0; c < c1; ++c) {
            const Words<CH> ca = wa, ca1 = wa1, cb = wb;
            const bool valid = vb;
            // unconditional prefetch (the last one re-reads in bounds and is unused)
            wa = load_words<CH>(w_ptr + (int64_t)(c + 1 < c1 ? c + 1 : c) * (8 * CH));
            if (F::SPARSE) wa1 = load_words<CH>(w_ptr + (int64_t)(c + 1 < c1 ? c + 1 : c) * (8 * CH) + 4 * CH);
            fetch_x();
            if constexpr (F::SPARSE) {
                // (kept bytes (1, 0) with the even codes, (0, 1) with the odd; the packed word is the index of both)
                const int x = valid ? 0x00010001 : 0, y = valid ? 0x01000100 : 0;
                const v4i ones_even = {x, x, x, x}, ones_odd = {y, y, y, y};
#pragma unroll
                for (int word = 0; word < CH; ++word) {
                    v8i even, odd;
                    sparse_dense_rows(s_rows + 16 * ws, ca.v[word], ca1.v[word], sparse_pick(h), even, odd);
                    acc = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones_even, even, acc, (int)cb.v[word], 0, 0);
                    acc = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones_odd, odd, acc, (int)cb.v[word], 0, 0);
                }
                continue;
            }
#pragma unroll
            for (int word = 0; word < CH; ++word)
#pragma unroll
                for (int j = 0; j < F::SELS; ++j) {
                    const Sel sa = make_sel<BITS>(ca.v[word], j, true), sb = make_sel<BITS>(cb.v[word], j, valid);
#pragma unroll
                    for (int g = 0; g < F::GROUPS; ++g) {
                        const v4i fb = onehot_operand<BITS>(a.pools, sb, g);
                        acc = dg_mfma_step<TR>(weight_operand<BITS>(a.pools, sa, g, 0), fb, acc);
                        if (TWO) acc_hi = dg_mfma_step<TR>(weight_operand<BITS>(a.pools, sa, g, 1), fb, acc_hi);
                    }
                }
        }
    }
    if (TWO) {
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = (int)((uint32_t)acc[e] + ((uint32_t)acc_hi[e] << 8));       // 256 * hi + lo
    }

    // the wavefronts' partial blocks meet by LDS integer atomics (exact in any order)
#pragma unroll
    for (int e = 0; e < 16; ++e)
        __hip_atomic_fetch_add(&s_sum[e * 64 + lane], acc[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __syncthreads();

    if (TR && p.Qp) {
        // re-quantising epilogue: the four channels of a quad make one packed byte of the next layer's activations
        // (a wavefront's 64 elements share the accumulator register e, so the trip count is uniform and DPP is safe)
        const float lo_f = (float)p.q_lo, hi_f = (float)(p.q_lo + 3);
        for (int idx = threadIdx.x; idx < 1024; idx += blockDim.x) {
            const int e = idx >> 6, l = idx & 63, c = l & 31;
            const int m = m0 + c, n = n0 + 8 * (e / 4) + 4 * (l >> 5) + (e % 4);
            const bool live = m < p.M;
            const float y = __fmul_rn((float)s_sum[idx], sc);
            const uint32_t code = live ? dg_quantize_code(y, p.q_scale, p.q_zero, lo_f, hi_f, p.q_lo) : 0u;
            const uint32_t byte = dg_quad_or(code << (2 * (c & 3)));
            if (live && (c & 3) == 0 && n < p.N) p.Qp[(int64_t)n * (p.M / 4) + m / 4] = (uint8_t)byte;
        }
        return;
    }
    for (int idx = threadIdx.x; idx < 1024; idx += blockDim.x) {
        const int e = idx >> 6, l = idx & 63;
        const int32_t sum = s_sum[idx];
        const int row = 8 * (e / 4) + 4 * (l >> 5) + (e % 4), c = l & 31;       // MFMA block coordinates
        const int m = m0 + (TR ? c : row), n = n0 + (TR ? row : c);
        if (m >= p.M || n >= p.N) continue;
        const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
        if (p.scale)
            p.Cf[o] = (float)sum * (TR ? sc : p.scale[m]);      // TR: m = m0 + thread % 32, the channel fetched above
        else
            p.C[o] = sum;
    }
}

// What runs a problem: the split-K kernel with S wavefronts per block, or the large-layer kernel with a
// (32*wm) x (32*wn) tile.
struct Plan {
    int ch;          // 32-bit words of packed codes per lane half and chunk
    bool two;        // entries beyond int8: two int8 planes
    bool decode;     // the decode-and-multiply comparison instead of a table kernel
    bool split;
    int wm;          // 2; 1 with two planes; 4 for the comparison's 128 x 128 tile
    int wn;
    int skw;         // large-layer kernel: wavefronts sharing a tile (1, 2 or 4)
    int S, cpw, chunks;
    bool staged;     // sparse instruction: the kernel that stages its operands through LDS (dg_sparse_staged_kernel.h)
};

// dynamic LDS of the large-layer kernel: the shared tiles' sums
template <int WM, int WN, bool TWO, int SKW>
constexpr size_t main_lds_bytes()
{
    return SKW == 1 ? 0 : (size_t)(4 / SKW) * (TWO ? 1 : WM) * WN * 1024 * sizeof(int32_t);
}

template <int BITS, int WM, int WN, bool TR, bool TWO, int SKW>
void launch_ch(const Args &a, int ch, dim3 grid, hipStream_t stream)
{
    constexpr size_t lds = main_lds_bytes<WM, WN, TWO, SKW>();
    static_assert(lds <= 64 * 1024, "the host plans only shapes whose sums fit 64 KB of LDS");
    // (4-bit codes: the host never plans 4-word chunks -- 32 MFMA steps -- so they are not instantiated; nor for the
    // sparse instruction's 64 x 128 and shared tiles, which would spill with them)
    if constexpr (BITS != 4 && !(BITS == 20 && (WN > 2 || SKW > 1))) {
        if (ch == 4) {
            hipLaunchKernelGGL((onehot_mfma_kernel<BITS, WM, WN, 4, TR, TWO, SKW>), grid, dim3(256), lds, stream, a);
            return;
        }
    }
    // (nor 2-word chunks on their widest tile: 16 steps of 14 MFMAs take the compiler minutes; the host plans 1 word)
    if constexpr (!(BITS == 4 && WN == 7)) {
        if (ch == 2) {
            hipLaunchKernelGGL((onehot_mfma_kernel<BITS, WM, WN, 2, TR, TWO, SKW>), grid, dim3(256), lds, stream, a);
            return;
        }
    }
    hipLaunchKernelGGL((onehot_mfma_kernel<BITS, WM, WN, 1, TR, TWO, SKW>), grid, dim3(256), lds, stream, a);
}

// The large-layer kernel on `wave_tiles` tiles of the planned width, 64 rows high (32 with two planes); a workgroup
// holds 4 / SKW of them.  The widest tile shares only among 4 wavefronts (two tiles of sums would not fit 64 KB).
template <int BITS, bool TR, bool TWO, int SKW>
void launch_main(const DgProblem &p, const Pools &pools, const Plan &q, int64_t wave_tiles, hipStream_t stream)
{
    Args a;
    a.p = p;
    a.pools = pools;
    a.tiles_m = (p.M + q.wm * 32 - 1) / (q.wm * 32);
    a.wave_tiles = wave_tiles;
    a.div_ow = make_div((uint32_t)p.OW), a.div_oh = make_div((uint32_t)p.OH);
    a.div_cin = make_div((uint32_t)p.Cin), a.div_kw = make_div((uint32_t)p.KW);
    constexpr int TPW = 4 / SKW;
    const dim3 grid((unsigned)((wave_tiles + TPW - 1) / TPW));
    if (q.wm == 4) {
        // (decoding costs VALU work per operand, not per MFMA: only a 128 x 128 tile has enough MFMAs per operand for
        // the matrix pipe to be the limit, so the comparison gets one)
        if constexpr (BITS == 0 && SKW == 1) launch_ch<0, 4, 4, TR, false, 1>(a, q.ch, grid, stream);
    } else if (q.wn == 7) {
        // (the sparse instruction's accumulators cannot live in the accumulation registers: 14 blocks do not fit)
        if constexpr (SKW != 2 && BITS != 20) launch_ch<BITS, 2, 7, TR, TWO, SKW>(a, q.ch, grid, stream);
    } else if (q.wn == 4) {
        launch_ch<BITS, 2, 4, TR, TWO, SKW>(a, q.ch, grid, stream);
    } else if (q.wn == 2) {
        launch_ch<BITS, 2, 2, TR, TWO, SKW>(a, q.ch, grid, stream);
    } else {
        launch_ch<BITS, 2, 1, TR, TWO, SKW>(a, q.ch, grid, stream);
    }
}

// The split-K kernel on `blocks11` 32 x 32 blocks of the output.
template <int BITS, bool TR, bool TWO, bool RAW = false>
void launch_split(const DgProblem &p, const Pools &pools, const Plan &q, int64_t blocks11, hipStream_t stream)
{
    SplitArgs b;
    b.p = p;
    b.pools = pools;
    b.chunks = q.chunks;
    b.cpw = q.cpw;
    b.tiles_m = (p.M + 31) / 32;
    b.div_ow = make_div((uint32_t)p.OW), b.div_oh = make_div((uint32_t)p.OH);
    b.div_cin = make_div((uint32_t)p.Cin), b.div_kw = make_div((uint32_t)p.KW);
    const dim3 grid((unsigned)blocks11), block(64 * q.S);
    if constexpr (BITS != 4 && BITS != 20 && !RAW) {        // (on unpacked codes the host plans 2-word chunks at most)
        if (q.ch == 4) {
            hipLaunchKernelGGL((onehot_splitk_kernel<BITS, 4, TR, TWO, RAW>), grid, block, 0, stream, b);
            return;
        }
    }
    if (q.ch == 2)
        hipLaunchKernelGGL((onehot_splitk_kernel<BITS, 2, TR, TWO, RAW>), grid, block, 0, stream, b);
    else
        hipLaunchKernelGGL((onehot_splitk_kernel<BITS, 1, TR, TWO, RAW>), grid, block, 0, stream, b);
}

// One translation unit per (code width, output layout, K share) instantiates these (the kernels are many: 4 tiles x
// 3 chunk sizes each).  TR: the output axis with stride 1 goes on the MFMA columns (see dg_mfma_tile.h).
// Unit "bBtTkK" defines unit_main_bB_tT_kK, and for K = 1 also unit_split_bB_tT; B = 22 stands for 2-bit codes in two
// planes, B = 0 for the decode-and-multiply comparison, B = 20 for 2-bit codes on the sparse instruction (T = 1 only).
typedef void (*MainFn)(const DgProblem &, const Pools &, const Plan &, int64_t, hipStream_t);
#define DGOH_UNIT(B, T, K) \
    void unit_main_b##B##_t##T##_k##K(const DgProblem &, const Pools &, const Plan &, int64_t, hipStream_t);
#define DGOH_UNIT_SPLIT(B, T) \
    void unit_split_b##B##_t##T(const DgProblem &, const Pools &, const Plan &, int64_t, hipStream_t);
DGOH_UNIT(2, 0, 1) DGOH_UNIT(2, 0, 2) DGOH_UNIT(2, 0, 4) DGOH_UNIT(2, 1, 1) DGOH_UNIT(2, 1, 2) DGOH_UNIT(2, 1, 4)
DGOH_UNIT(3, 0, 1) DGOH_UNIT(3, 1, 1) DGOH_UNIT(4, 0, 1) DGOH_UNIT(4, 1, 1) DGOH_UNIT(22, 0, 1) DGOH_UNIT(22, 1, 1)
DGOH_UNIT(20, 1, 1) DGOH_UNIT(20, 1, 2) DGOH_UNIT(20, 1, 4)
DGOH_UNIT(0, 0, 1) DGOH_UNIT(0, 0, 2) DGOH_UNIT(0, 0, 4) DGOH_UNIT(0, 1, 1) DGOH_UNIT(0, 1, 2) DGOH_UNIT(0, 1, 4)
DGOH_UNIT_SPLIT(2, 0) DGOH_UNIT_SPLIT(2, 1) DGOH_UNIT_SPLIT(3, 0) DGOH_UNIT_SPLIT(3, 1) DGOH_UNIT_SPLIT(4, 0)
DGOH_UNIT_SPLIT(4, 1) DGOH_UNIT_SPLIT(22, 0) DGOH_UNIT_SPLIT(22, 1) DGOH_UNIT_SPLIT(0, 0) DGOH_UNIT_SPLIT(0, 1) DGOH_UNIT_SPLIT(20, 1)
void unit_sparse4(const DgProblem &, const uint32_t (&)[16][4], int, hipStream_t);      // dg_sparse4_kernel.h
void unit_sparse2p(const DgProblem &, const uint32_t (&)[2][4], int, hipStream_t);      // dg_sparse2p_kernel.h
void unit_sparse_ws(const DgProblem &, const uint32_t (&)[4], int, bool raw, hipStream_t);      // dg_sparse_ws_kernel.h
void unit_sparse_staged(const DgProblem &, const Pools &, int32_t bias, const Plan &, int64_t, hipStream_t);      // dg_sparse_staged_kernel.h
// the split-K kernel on activations still one code per byte (one- and two-plane tables, either output layout)
void unit_split_codes(const DgProblem &, const Pools &, const Plan &, bool two, bool tr, int64_t, hipStream_t);
// the tiled kernel on unpacked codes: 64 x 32 and 64 x 64 tiles (q.wn = 1, 2), 2-word chunks, any sharing of K;
// `sparse`: on the sparse instruction (its pools; outputs whose channel axis has stride 1 only)
void unit_main_codes(const DgProblem &, const Pools &, const Plan &, bool tr, bool sparse, int64_t wave_tiles, hipStream_t);
#undef DGOH_UNIT
#undef DGOH_UNIT_SPLIT

}   // namespace dgoh
