// Table lookup on the matrix cores by one-hot selection -- a TABLE kernel (it works for any 16 int8 entries,
// whether or not they factor into level vectors), unlike the decode-and-multiply comparison kernel.
//
//   C[m][n] = sum_k T[w(m,k)][a(n,k)] = sum_k sum_{v<4} T[w(m,k)][v] * [a(n,k) == v]
//
// so with A'[m][4k+v] = T[w(m,k)][v] (the table ROW of the weight code, 4 int8) and B'[n][4k+v] = [a(n,k) == v]
// (a one-hot byte quadruple) the layer is an int8 contraction of length 4K: each multiply is by 0 or 1, i.e. the
// MFMA unit SELECTS one table entry per reduction position and adds it.  Four times the MFMA work of the
// rank-1 decode kernel, but every table is accepted and the VALU only expands codes.
//
// Expansion, without LDS: the order of the 4K axis is free as long as both operands use the same one, so the 16 operand
// bytes of a lane are laid out value-major: dword v holds, for 4 reduction positions, T[w(k)][v] (weights) or
// [a(k) == v] (activations).  With the four 2-bit codes spread into the bytes of a selector word
// ((word >> 2j) & 0x03030303 takes code j of each of a word's four bytes), each operand dword is ONE byte permute:
// of the table's column v for the weights, of the constant 1 << 8v for the activations.  A filter tap outside the
// image gets selector bytes 4 (the permute's upper, all-zero source), so it selects nothing.
// Wave tiles, global loads and the epilogue follow the comparison kernel: each wave owns (WM*32) x (WN*32) outputs,
// operands come straight from global memory, and there is no LDS and no barrier.
#include <cstdlib>

#include "dg_mfma_tile.h"

namespace {

typedef dg_v4i v4i;
typedef dg_v16i v16i;

struct OneHotArgs {
    DgProblem p;
    uint32_t cols[4];        // cols[v] = bytes T[0..3][v] (signed int8, as stored): the permute pool of value v
    int32_t tiles_m;
    int64_t wave_tiles;
};

template <int CH>
struct Words {
    uint32_t v[CH];
};

template <int CH>
__device__ __forceinline__ Words<CH> load_words(const uint8_t *ptr, bool ok)
{
    Words<CH> w;
    if (CH == 4) {
        const uint4 t = ok ? *(const uint4 *)ptr : make_uint4(0, 0, 0, 0);
        w.v[0] = t.x, w.v[1 % CH] = t.y, w.v[2 % CH] = t.z, w.v[3 % CH] = t.w;
    } else if (CH == 2) {
        const uint2 t = ok ? *(const uint2 *)ptr : make_uint2(0, 0);
        w.v[0] = t.x, w.v[1 % CH] = t.y;
    } else {
        w.v[0] = ok ? *(const uint32_t *)ptr : 0u;
    }
    return w;
}

// selector word of 4 reduction positions -> the 4 operand dwords (one per activation value v)
__device__ __forceinline__ v4i select4(uint32_t p0, uint32_t p1, uint32_t p2, uint32_t p3, uint32_t sel)
{
    v4i r;
    r[0] = (int)__builtin_amdgcn_perm(0u, p0, sel);
    r[1] = (int)__builtin_amdgcn_perm(0u, p1, sel);
    r[2] = (int)__builtin_amdgcn_perm(0u, p2, sel);
    r[3] = (int)__builtin_amdgcn_perm(0u, p3, sel);
    return r;
}

template <int WM, int WN, int CH, bool TR>
__global__ void __launch_bounds__(256, (WM * WN > 8 ? 1 : 2))
onehot_mfma_kernel(OneHotArgs a)
{
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63;
    const int64_t wave_tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wave_tile >= a.wave_tiles) return;                 // whole waves leave; there is no barrier below
    const int r = lane & 31, h = lane >> 5;
    const int m0 = (int)(wave_tile % a.tiles_m) * (WM * 32);
    const int n0 = (int)(wave_tile / a.tiles_m) * (WN * 32);
    const int cq = p.Cin / 4;
    constexpr int CHUNK = 32 * CH;                          // codes of K per chunk (16*CH per lane half)

    const uint8_t *w_ptr[WM];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm) {
        int m = m0 + bm * 32 + r;
        if (m >= p.M) m = p.M - 1;
        w_ptr[bm] = p.Wp + (int64_t)m * (p.K / 4) + h * (4 * CH);
    }
    bool x_ok[WN];
    int x_ih0[WN], x_iw0[WN];
    int64_t x_off0[WN];
#pragma unroll
    for (int bn = 0; bn < WN; ++bn) {
        const int n = n0 + bn * 32 + r;
        x_ok[bn] = n < p.N;
        const int nn = x_ok[bn] ? n : 0;
        const int ow = nn % p.OW, oh = (nn / p.OW) % p.OH, b = nn / (p.OW * p.OH);
        x_ih0[bn] = oh * p.sh - p.ph;
        x_iw0[bn] = ow * p.sw - p.pw;
        x_off0[bn] = (((int64_t)b * p.H + x_ih0[bn]) * p.W + x_iw0[bn]) * cq + h * (4 * CH);
    }

    v16i acc[WM][WN];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[bm][bn][e] = 0;

    int kh = 0, kw = 0, ci = 0;
    Words<CH> wa[WM], wb[WN];
    bool vb[WN];
    auto fetch = [&](int chunk) {
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) wa[bm] = load_words<CH>(w_ptr[bm] + (int64_t)chunk * (CHUNK / 4), true);
        const int64_t tap_off = ((int64_t)kh * p.W + kw) * cq + ci / 4;
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            const int ih = x_ih0[bn] + kh, iw = x_iw0[bn] + kw;
            vb[bn] = x_ok[bn] & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
            // always load (a tap outside the image reads the first pixel instead and is masked later): a load under
            // a branch would make the compiler wait for it at once, and the prefetch would hide nothing
            wb[bn] = load_words<CH>(vb[bn] ? p.Xp + x_off0[bn] + tap_off : p.Xp + h * (4 * CH), true);
        }
        ci += CHUNK;
        if (ci == p.Cin) {
            ci = 0;
            if (++kw == p.KW) {
                kw = 0;
                ++kh;
            }
        }
    };

    const int chunks = p.K / CHUNK;
    fetch(0);
    for (int c = 0; c < chunks; ++c) {
        Words<CH> ca[WM], cb[WN];
        uint32_t pad[WN];
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) ca[bm] = wa[bm];
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            cb[bn] = wb[bn];
            pad[bn] = vb[bn] ? 0u : 0x04040404u;
        }
        fetch(c + 1 < chunks ? c + 1 : c);                  // unconditional (the last one re-reads in bounds and is unused)
        // Step t (word t/4, code t%4 of its four bytes) is one MFMA step.  The operands of step t+1 are built between
        // the MFMAs of step t so that the matrix unit and the VALU of a single
        // wavefront overlap; the scheduling groups pin that interleaving.
        constexpr int T = 4 * CH;
        v4i fa[2][WM], fb[2][WN];
        auto expand = [&](int t, int u, int buf) {           // operand u of step t: u < WM weights, else activations
            const int sw = t / 4, sh = 2 * (t % 4);
            if (u < WM)
                fa[buf][u] = select4(a.cols[0], a.cols[1], a.cols[2], a.cols[3], (ca[u].v[sw] >> sh) & 0x03030303u);
            else
                fb[buf][u - WM] = select4(0x00000001u, 0x00000100u, 0x00010000u, 0x01000000u,
                                          ((cb[u - WM].v[sw] >> sh) & 0x03030303u) | pad[u - WM]);
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
                    for (int u = u0; u < u1; ++u) expand(t + 1, u, cur ^ 1);
                    if (u1 - u0 == 1) __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);   // ... then that VALU work
                    if (u1 - u0 == 2) __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);
                }
            }
        }
    }

    dg_mfma_store_tile<WM, WN, TR>(p, acc, m0, n0, lane);
}

template <int WM, int WN, bool TR>
void launch_ch(const OneHotArgs &a, int ch, dim3 grid, hipStream_t stream)
{
    if (ch == 4)
        hipLaunchKernelGGL((onehot_mfma_kernel<WM, WN, 4, TR>), grid, dim3(256), 0, stream, a);
    else if (ch == 2)
        hipLaunchKernelGGL((onehot_mfma_kernel<WM, WN, 2, TR>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((onehot_mfma_kernel<WM, WN, 1, TR>), grid, dim3(256), 0, stream, a);
}

template <bool TR>
void launch_wn(const OneHotArgs &a, int wn, int ch, dim3 grid, hipStream_t stream)
{
    if (wn == 7)
        launch_ch<2, 7, TR>(a, ch, grid, stream);
    else if (wn == 4)
        launch_ch<2, 4, TR>(a, ch, grid, stream);
    else if (wn == 2)
        launch_ch<2, 2, TR>(a, ch, grid, stream);
    else
        launch_ch<2, 1, TR>(a, ch, grid, stream);
}

// Small layers: too few 64 x 32 tiles to occupy the chip, and a wavefront that walks all of K alone pays the memory
// latency once per chunk.  Here a workgroup owns ONE 32 x 32 output block and its S wavefronts split K between them
// (whole chunks of 32*CH reduction positions each), so a layer with T blocks puts T*S wavefronts in flight and each
// of them waits for memory once or twice.  Partial blocks meet in LDS: every wavefront writes its 16 accumulator
// registers, one barrier, then the threads add the S partials of each output element (integer, so exact in any order)
// and store it -- 128 contiguous bytes per half wavefront, as in the large-layer kernel.
struct OneHotSplitArgs {
    DgProblem p;
    uint32_t cols[4];
    int32_t tiles_m;
    int32_t chunks;          // K / (32*CH)
    int32_t cpw;             // chunks per wavefront
};

template <int CH, bool TR>
__global__ void __launch_bounds__(1024)
onehot_splitk_kernel(OneHotSplitArgs a)
{
    extern __shared__ int32_t s_part[];                     // [S][16][64]
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, ws = threadIdx.x >> 6, S = blockDim.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int m0 = ((int)blockIdx.x % a.tiles_m) * 32;
    const int n0 = ((int)blockIdx.x / a.tiles_m) * 32;
    const int cq = p.Cin / 4;
    constexpr int CHUNK = 32 * CH;
    const int c0 = ws * a.cpw, c1 = min(c0 + a.cpw, a.chunks);

    v16i acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0;

    if (c0 < c1) {
        const int m = min(m0 + r, p.M - 1);
        const uint8_t *w_ptr = p.Wp + (int64_t)m * (p.K / 4) + h * (4 * CH);
        const int n = n0 + r;
        const bool x_ok = n < p.N;
        const int nn = x_ok ? n : 0;
        const int ow = nn % p.OW, oh = (nn / p.OW) % p.OH, b = nn / (p.OW * p.OH);
        const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
        const int64_t x_off0 = (((int64_t)b * p.H + ih0) * p.W + iw0) * cq + h * (4 * CH);
        // filter tap of this wavefront's first chunk
        const int pos = c0 * CHUNK, tap = pos / p.Cin;
        int ci = pos - tap * p.Cin, kh = tap / p.KW, kw = tap - (tap / p.KW) * p.KW;

        Words<CH> wa, wb;
        bool vb;
        auto fetch = [&](int chunk) {
            wa = load_words<CH>(w_ptr + (int64_t)chunk * (CHUNK / 4), true);
            const int ih = ih0 + kh, iw = iw0 + kw;
            vb = x_ok & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
            const int64_t tap_off = ((int64_t)kh * p.W + kw) * cq + ci / 4;
            wb = load_words<CH>(vb ? p.Xp + x_off0 + tap_off : p.Xp + h * (4 * CH), true);
            ci += CHUNK;
            if (ci == p.Cin) {
                ci = 0;
                if (++kw == p.KW) {
                    kw = 0;
                    ++kh;
                }
            }
        };
        fetch(c0);
        for (int c = c0; c < c1; ++c) {
            const Words<CH> ca = wa, cb = wb;
            const uint32_t pad = vb ? 0u : 0x04040404u;
            fetch(c + 1 < c1 ? c + 1 : c);                  // unconditional (the last one re-reads in bounds and is unused)
#pragma unroll
            for (int t = 0; t < 4 * CH; ++t) {
                const int sw = t / 4, sh = 2 * (t % 4);
                const v4i fa = select4(a.cols[0], a.cols[1], a.cols[2], a.cols[3], (ca.v[sw] >> sh) & 0x03030303u);
                const v4i fb = select4(0x00000001u, 0x00000100u, 0x00010000u, 0x01000000u,
                                       ((cb.v[sw] >> sh) & 0x03030303u) | pad);
                acc = dg_mfma_step<TR>(fa, fb, acc);
            }
        }
    }

#pragma unroll
    for (int e = 0; e < 16; ++e) s_part[(ws * 16 + e) * 64 + lane] = acc[e];
    __syncthreads();

    for (int idx = threadIdx.x; idx < 1024; idx += blockDim.x) {
        const int e = idx >> 6, l = idx & 63;
        int32_t sum = 0;
        for (int w = 0; w < S; ++w) sum += s_part[(w * 16 + e) * 64 + l];
        const int row = 8 * (e / 4) + 4 * (l >> 5) + (e % 4), col = l & 31;     // MFMA block coordinates
        const int m = m0 + (TR ? col : row), n = n0 + (TR ? row : col);
        if (m >= p.M || n >= p.N) continue;
        const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
        if (p.scale)
            p.Cf[o] = (float)sum * p.scale[m];
        else
            p.C[o] = sum;
    }
}

template <bool TR>
void launch_splitk(const OneHotSplitArgs &a, int ch, dim3 grid, int S, hipStream_t stream)
{
    const dim3 block(64 * S);
    const size_t lds = (size_t)S * 16 * 64 * sizeof(int32_t);
    if (ch == 4)
        hipLaunchKernelGGL((onehot_splitk_kernel<4, TR>), grid, block, lds, stream, a);
    else if (ch == 2)
        hipLaunchKernelGGL((onehot_splitk_kernel<2, TR>), grid, block, lds, stream, a);
    else
        hipLaunchKernelGGL((onehot_splitk_kernel<1, TR>), grid, block, lds, stream, a);
}

}   // namespace

bool dg_onehot_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->min_entry < -128 || lut->max_entry > 127) return false;   // entries are MFMA int8 operands
    if (p.Cin % 32 != 0) return false;
    const int ch = p.Cin % 128 == 0 ? 4 : (p.Cin % 64 == 0 ? 2 : 1);
    if ((uintptr_t)p.Wp % (4 * ch) != 0 || (uintptr_t)p.Xp % (4 * ch) != 0) return false;
    return true;
}

namespace {

// Which of the two kernels runs a problem, and its shape.
struct OneHotPlan {
    int ch;          // 32-bit words of packed codes per lane half and chunk
    bool split;      // small layer: 32 x 32 block per workgroup, K split over S wavefronts
    int wn;          // large layer: the wave tile is 64 x (32*wn)
    int S, cpw, chunks;
};

int64_t tile_count(const DgProblem &p, int wm, int wn)
{
    return ((int64_t)(p.M + wm * 32 - 1) / (wm * 32)) * (((int64_t)p.N + wn * 32 - 1) / (wn * 32));
}

OneHotPlan plan_for(const DgProblem &p)
{
    OneHotPlan q;
    q.ch = p.Cin % 128 == 0 ? 4 : (p.Cin % 64 == 0 ? 2 : 1);
    q.chunks = p.K / (32 * q.ch);
    q.wn = 1, q.S = 1, q.cpw = q.chunks;
    // too few 64 x 32 tiles to give every SIMD a wavefront (or barely enough, and a long K to walk): split K
    const int64_t t21 = tile_count(p, 2, 1);
    const bool few_tiles = t21 < 512 || (t21 < 1024 && q.chunks >= 32);
    q.split = few_tiles && q.chunks > 1;
    // DG_ONEHOT_PLAN = split | 1 | 2 | 4 | 7 overrides the choice (tuning, and tests that must reach every plan)
    const char *force = getenv("DG_ONEHOT_PLAN");
    int force_wn = 0;
    if (force) {
        if (force[0] == 's') q.split = true;
        else if (atoi(force) == 1 || atoi(force) == 2 || atoi(force) == 4 || atoi(force) == 7) force_wn = atoi(force), q.split = false;
    }
    if (q.split) {
        // about 2048 wavefronts in all, at most 16 per workgroup, whole chunks each
        const int64_t blocks = tile_count(p, 1, 1);
        int S = (int)((2048 + blocks - 1) / blocks);
        S = S < 1 ? 1 : (S > 16 ? 16 : S);
        if (S > q.chunks) S = q.chunks;
        q.cpw = (q.chunks + S - 1) / S;
        q.S = (q.chunks + q.cpw - 1) / q.cpw;
        return q;
    }
    // Wave tile 64 x (32*wn): the one with the least modelled time on the busiest SIMD, in cycles.  A SIMD's
    // wavefronts share its matrix pipe, so its time is (tiles per SIMD, rounded up) x (32x32 blocks per tile) x (MFMA
    // steps of K) x (cycles per MFMA: 32, more where the VALU work of building operands or the operand loads show --
    // measured 42 for one block column, 33 for two), plus what no other wavefront hides: one prologue (~3000 cycles)
    // and the last tile's stores (~600 cycles per block).  7 blocks wide fits the 56 x 56 and 28 x 28 images of
    // ImageNet networks (N = 49 * 2^k) where 4 wide leaves the last round of tiles half empty.  The constants are
    // fitted to timings of 50 layer shapes; ties go to the wider tile (fewer operand loads).
    static const int widths[4] = {7, 4, 2, 1};
    static const double mfma_cycles[4] = {32.0, 32.0, 33.0, 42.0};
    const double steps = p.K / 8.0;
    double best = 0.0;
    for (int i = 0; i < 4; ++i) {
        const int wn = widths[i];
        const double per_simd = (double)((tile_count(p, 2, wn) + 1023) / 1024);
        const double cost = per_simd * 2 * wn * steps * mfma_cycles[i] + 3000.0 + 600.0 * 2 * wn;
        if (i == 0 || cost < best * 0.999) best = cost, q.wn = wn;
    }
    if (force_wn) q.wn = force_wn;
    return q;
}

}   // namespace

const char *dg_onehot_config_name(const dg_lut *, const DgProblem &p)
{
    static const char *const split_names[17] = {
        "", "onehot_mfma_splitk_s1", "onehot_mfma_splitk_s2", "onehot_mfma_splitk_s3", "onehot_mfma_splitk_s4",
        "onehot_mfma_splitk_s5", "onehot_mfma_splitk_s6", "onehot_mfma_splitk_s7", "onehot_mfma_splitk_s8",
        "onehot_mfma_splitk_s9", "onehot_mfma_splitk_s10", "onehot_mfma_splitk_s11", "onehot_mfma_splitk_s12",
        "onehot_mfma_splitk_s13", "onehot_mfma_splitk_s14", "onehot_mfma_splitk_s15", "onehot_mfma_splitk_s16"};
    const OneHotPlan q = plan_for(p);
    if (q.split) return split_names[q.S];
    return q.wn == 7 ? "onehot_mfma_64x224"
                     : (q.wn == 4 ? "onehot_mfma_64x128" : (q.wn == 2 ? "onehot_mfma_64x64" : "onehot_mfma_64x32"));
}

dg_status dg_launch_onehot(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    OneHotArgs a;
    a.p = p;
    for (int w = 0; w < 4; ++w) {
        uint32_t r = 0;
        for (int c = 0; c < 4; ++c) r |= (uint32_t)(uint8_t)(int8_t)lut->entry[4 * c + w] << (8 * c);
        a.cols[w] = r;
    }
    const OneHotPlan q = plan_for(p);
    const bool tr = p.stride_cm == 1 && p.stride_cn != 1;   // the output axis with stride 1 goes on the MFMA columns
    if (q.split) {
        OneHotSplitArgs b;
        b.p = p;
        for (int v = 0; v < 4; ++v) b.cols[v] = a.cols[v];
        b.chunks = q.chunks;
        b.cpw = q.cpw;
        b.tiles_m = (p.M + 31) / 32;
        const int64_t blocks = tile_count(p, 1, 1);
        if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel: too many tiles for one grid");
        if (tr)
            launch_splitk<true>(b, q.ch, dim3((unsigned)blocks), q.S, stream);
        else
            launch_splitk<false>(b, q.ch, dim3((unsigned)blocks), q.S, stream);
        return dg_check_launch("onehot_splitk_kernel");
    }
    a.tiles_m = (p.M + 63) / 64;
    a.wave_tiles = tile_count(p, 2, q.wn);
    const int64_t blocks = (a.wave_tiles + 3) / 4;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel: too many tiles for one grid");
    const dim3 grid((unsigned)blocks);
    if (tr)
        launch_wn<true>(a, q.wn, q.ch, grid, stream);
    else
        launch_wn<false>(a, q.wn, q.ch, grid, stream);
    return dg_check_launch("onehot_mfma_kernel");
}
