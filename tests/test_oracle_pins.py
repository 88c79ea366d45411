"""Pins for the CPU oracle: it is checked against things other than itself.

Hand-computed fixtures (tests/golden/), brute force over the 16 code pairs,
closed forms, library routines on decoded levels (numpy int64 matmul, torch
float64 conv2d), invariants of the sum, and statistical moments of the seeded
workload.  A dropped term, a wrong sign, a transposed operand or a swapped
kh/kw in the oracle fails at least one of these.  No GPU is used here.
"""
import itertools
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2304_09049_amd import workloads as wl

LW = np.array(wl.LEVELS_W_SIGNED, dtype=np.int32)
LA = np.array(wl.LEVELS_A_UNSIGNED, dtype=np.int32)
LEVEL_SETS = [
    (LW, LA),
    (np.array([0, 1, -2, -1], dtype=np.int32), np.array([3, 1, 0, 2], dtype=np.int32)),   # two's-complement order
    (np.array([-8, 7, 3, -5], dtype=np.int32), np.array([-7, 6, -8, 1], dtype=np.int32)),  # non-uniform
    (np.array([127, -128, 5, 0], dtype=np.int32), np.array([-128, 127, 1, 0], dtype=np.int32)),
]


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


# ---- fixtures worked out by hand ---------------------------------------------------------

def test_golden_tiny_gemm(golden_dir):
    g = _load(golden_dir, "tiny_gemm.json")
    C = oracle.gemm(g["Wc"], g["Ac"], g["levels_w"], g["levels_a"])
    assert C.tolist() == g["C"]


def test_golden_packed_bytes(golden_dir):
    g = _load(golden_dir, "tiny_gemm.json")
    assert oracle.pack_codes(np.array(g["Wc"], dtype=np.uint8)).tolist() == g["Wp"]
    assert oracle.pack_codes(np.array(g["Ac"], dtype=np.uint8)).tolist() == g["Ap"]
    assert oracle.unpack_codes(np.array(g["Wp"], dtype=np.uint8)).tolist() == g["Wc"]
    table = oracle.build_lut(g["levels_w"], g["levels_a"])
    C = oracle.lut_gemm_packed(g["Wp"], g["Ap"], table, 8)
    assert C.tolist() == g["C"]


def test_golden_lut16_table(golden_dir):
    g = _load(golden_dir, "lut16_signed_unsigned.json")
    table = oracle.build_lut(g["levels_w"], g["levels_a"])
    assert table.tolist() == g["table"]
    assert len(table) == g["entries"] == 2 ** g["index_bits"]


def _tiny_conv_weights(g):
    Wc = np.zeros((4, 3, 3, 4), dtype=np.uint8)
    for co in range(4):
        spec = g["W_taps"][str(co)]
        Wc[co, :, :, :] = np.array(spec["default"], dtype=np.uint8)
        for key, codes in spec.items():
            if key == "default":
                continue
            kh, kw = (int(t) for t in key.split(","))
            Wc[co, kh, kw, :] = np.array(codes, dtype=np.uint8)
    return Wc


@pytest.mark.parametrize("stride,key", [((1, 1), "Y_stride1"), ((2, 2), "Y_stride2")])
def test_golden_tiny_conv(golden_dir, stride, key):
    g = _load(golden_dir, "tiny_conv.json")
    Wc = _tiny_conv_weights(g)
    Xc = np.array(g["X"], dtype=np.uint8)
    Y = oracle.conv2d(Wc, Xc, g["levels_w"], g["levels_a"], stride=stride, pad=(1, 1))
    want = np.array(g[key], dtype=np.int32)              # [co][oh][ow]
    assert Y.shape == (1,) + want.shape[1:] + (4,)
    assert np.array_equal(Y[0].transpose(2, 0, 1), want)


# ---- brute force over the 16 code pairs --------------------------------------------------

@pytest.mark.parametrize("lw,la", LEVEL_SETS)
def test_all_16_code_pairs(lw, la):
    Wc = np.repeat(np.arange(4, dtype=np.uint8)[:, None], 4, axis=1)     # row m = code m, K = 4
    Ac = np.repeat(np.arange(4, dtype=np.uint8)[:, None], 4, axis=1)
    C = oracle.gemm(Wc, Ac, lw, la)
    for m, n in itertools.product(range(4), range(4)):
        assert C[m, n] == 4 * int(lw[m]) * int(la[n])


@pytest.mark.parametrize("lw,la", LEVEL_SETS[:3])
def test_each_slot_alone(lw, la):
    # K = 4: one slot carries the code pair (c, d), the other three carry the filler pair (f, g)
    for slot, c, d, f, g in itertools.product(range(4), range(4), range(4), (0, 3), (1, 2)):
        w = np.full((1, 4), f, dtype=np.uint8)
        a = np.full((1, 4), g, dtype=np.uint8)
        w[0, slot], a[0, slot] = c, d
        want = int(lw[c]) * int(la[d]) + 3 * int(lw[f]) * int(la[g])
        assert oracle.gemm(w, a, lw, la)[0, 0] == want
        table = oracle.build_lut(lw, la)
        assert oracle.lut_gemm_packed(oracle.pack_codes(w), oracle.pack_codes(a), table, 4)[0, 0] == want


def test_lut_index_is_weight_high_activation_low():
    lw = np.array([1, 10, 100, 1000], dtype=np.int32)
    la = np.array([1, 2, 3, 4], dtype=np.int32)
    t = oracle.build_lut(lw, la)
    for w, a in itertools.product(range(4), range(4)):
        assert t[4 * w + a] == lw[w] * la[a]


# ---- closed forms ------------------------------------------------------------------------

@pytest.mark.parametrize("lw,la", LEVEL_SETS)
def test_constant_codes_closed_form(lw, la):
    K = 52
    for c, d in itertools.product(range(4), range(4)):
        C = oracle.gemm(np.full((3, K), c, np.uint8), np.full((5, K), d, np.uint8), lw, la)
        assert np.all(C == K * int(lw[c]) * int(la[d]))


def test_conv_constant_input_tap_counts():
    # 3x3, pad 1 on a constant image: interior sees 9 taps, edges 6, corners 4
    Cin, Cout, H, W = 8, 3, 5, 6
    lw, la = LEVEL_SETS[2]
    Wc = np.full((Cout, 3, 3, Cin), 1, np.uint8)
    Xc = np.full((2, H, W, Cin), 3, np.uint8)
    Y = oracle.conv2d(Wc, Xc, lw, la, pad=(1, 1))
    unit = Cin * int(lw[1]) * int(la[3])
    taps_h = np.array([2] + [3] * (H - 2) + [2])
    taps_w = np.array([2] + [3] * (W - 2) + [2])
    want = unit * np.outer(taps_h, taps_w)
    for b in range(2):
        for co in range(Cout):
            assert np.array_equal(Y[b, :, :, co], want)


def test_conv_out_dim_floor():
    assert oracle.conv_out_dim(56, 3, 1, 1) == 56
    assert oracle.conv_out_dim(56, 3, 2, 1) == 28
    assert oracle.conv_out_dim(7, 3, 2, 0) == 3
    assert oracle.conv_out_dim(8, 3, 2, 0) == 3      # floor, not ceil
    assert oracle.conv_out_dim(224, 7, 2, 3) == 112
    assert oracle.conv_out_dim(2, 3, 1, 0) == 0


# ---- library routines on decoded levels --------------------------------------------------

@pytest.mark.parametrize("lw,la", LEVEL_SETS)
@pytest.mark.parametrize("M,N,K", [(7, 5, 12), (33, 17, 100), (64, 196, 576)])
def test_gemm_equals_numpy_matmul(lw, la, M, N, K):
    inp = wl.small_gemm(M, N, K, seed=M + N + K)
    want = lw.astype(np.int64)[inp.Wc] @ la.astype(np.int64)[inp.Ac].T
    assert np.array_equal(oracle.gemm(inp.Wc, inp.Ac, lw, la).astype(np.int64), want)


CONV_CASES = [
    # B, H, W, Cin, Cout, KH, KW, stride, pad
    (2, 7, 9, 8, 5, 3, 3, (1, 1), (1, 1)),
    (1, 8, 8, 4, 6, 3, 3, (2, 2), (1, 1)),
    (2, 9, 6, 12, 4, 1, 1, (1, 1), (0, 0)),
    (1, 10, 7, 4, 3, 5, 3, (2, 1), (2, 0)),
    (1, 6, 11, 8, 2, 1, 7, (1, 3), (0, 3)),
    (3, 5, 5, 16, 7, 3, 3, (1, 1), (0, 0)),
]


@pytest.mark.parametrize("case", CONV_CASES)
@pytest.mark.parametrize("lw,la", LEVEL_SETS[:3])
def test_conv_equals_torch_float64(case, lw, la):
    B, H, W, Cin, Cout, KH, KW, stride, pad = case
    inp = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H * W + Cin)
    x = torch.from_numpy(la.astype(np.float64)[inp.Ac]).permute(0, 3, 1, 2)       # NCHW levels
    w = torch.from_numpy(lw.astype(np.float64)[inp.Wc]).permute(0, 3, 1, 2)       # [Cout][Cin][KH][KW]
    want = torch.nn.functional.conv2d(x, w, stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()
    got = oracle.conv2d(inp.Wc, inp.Ac, lw, la, stride=stride, pad=pad)
    assert got.shape == want.shape
    assert np.array_equal(got.astype(np.float64), want)       # exact: every value is a small integer


# ---- invariants of the sum ---------------------------------------------------------------

def test_table_path_equals_multiply_path():
    for lw, la in LEVEL_SETS:
        inp = wl.small_gemm(19, 23, 64, seed=5)
        table = oracle.build_lut(lw, la)
        via_table = oracle.lut_gemm_packed(oracle.pack_codes(inp.Wc), oracle.pack_codes(inp.Ac), table, 64)
        assert np.array_equal(via_table, oracle.gemm(inp.Wc, inp.Ac, lw, la))


def test_k_additivity_and_permutation():
    lw, la = LEVEL_SETS[2]
    inp = wl.small_gemm(9, 11, 40, seed=3)
    full = oracle.gemm(inp.Wc, inp.Ac, lw, la)
    left = oracle.gemm(inp.Wc[:, :16], inp.Ac[:, :16], lw, la)
    right = oracle.gemm(inp.Wc[:, 16:], inp.Ac[:, 16:], lw, la)
    assert np.array_equal(full, left + right)
    perm = np.random.default_rng(0).permutation(40)
    assert np.array_equal(full, oracle.gemm(inp.Wc[:, perm], inp.Ac[:, perm], lw, la))


def test_relabelling_codes_with_levels():
    lw, la = LEVEL_SETS[2]
    inp = wl.small_gemm(6, 7, 24, seed=8)
    base = oracle.gemm(inp.Wc, inp.Ac, lw, la)
    pw, pa = np.array([2, 0, 3, 1]), np.array([1, 3, 0, 2])     # new code = p[old code]
    lw2, la2 = np.empty_like(lw), np.empty_like(la)
    lw2[pw], la2[pa] = lw, la
    assert np.array_equal(base, oracle.gemm(pw[inp.Wc].astype(np.uint8), pa[inp.Ac].astype(np.uint8), lw2, la2))


def test_scaling_weight_levels_scales_result():
    lw, la = LEVEL_SETS[0]
    inp = wl.small_gemm(5, 5, 32, seed=9)
    assert np.array_equal(3 * oracle.gemm(inp.Wc, inp.Ac, lw, la), oracle.gemm(inp.Wc, inp.Ac, 3 * lw, la))
    assert np.array_equal(-oracle.gemm(inp.Wc, inp.Ac, lw, la), oracle.gemm(inp.Wc, inp.Ac, lw, -la))


def test_transposed_operands_are_not_interchangeable():
    # guards the tests themselves: with these levels swapping the two sides must change the result
    lw, la = LEVEL_SETS[0]
    inp = wl.small_gemm(8, 8, 32, seed=1)
    assert not np.array_equal(oracle.gemm(inp.Wc, inp.Ac, lw, la), oracle.gemm(inp.Wc, inp.Ac, la, lw))


def test_conv1x1_is_gemm():
    lw, la = LEVEL_SETS[2]
    inp = wl.small_conv(2, 5, 4, 16, 6, 1, 1, seed=4)
    Y = oracle.conv2d(inp.Wc, inp.Ac, lw, la)
    C = oracle.gemm(inp.Wc.reshape(6, 16), inp.Ac.reshape(-1, 16), lw, la)        # [Cout][pixels]
    assert np.array_equal(Y.reshape(-1, 6), C.T)


def test_conv3x3_is_gemm_on_explicit_im2col():
    # K index = (kh*KW + kw)*Cin + ci on both sides; a padded position uses a code whose level is 0
    lw, la = LEVEL_SETS[0]                       # activation code 0 decodes to 0
    inp = wl.small_conv(1, 6, 5, 4, 3, 3, 3, pad=(1, 1), seed=6)
    Xpad = np.zeros((1, 8, 7, 4), np.uint8)
    Xpad[:, 1:-1, 1:-1, :] = inp.Ac
    cols = np.stack([Xpad[0, oh:oh + 3, ow:ow + 3, :].reshape(-1) for oh in range(6) for ow in range(5)])
    C = oracle.gemm(inp.Wc.reshape(3, -1), cols, lw, la)
    Y = oracle.conv2d(inp.Wc, inp.Ac, lw, la, pad=(1, 1))
    assert np.array_equal(Y.reshape(-1, 3), C.T)


def test_padding_contributes_zero_whatever_the_levels():
    # out-of-image taps add nothing even when no activation code decodes to 0:
    # compare with an un-padded convolution over an image padded with a code, minus that code's share
    lw = np.array([-3, 2, 5, -1], dtype=np.int32)
    la = np.array([4, -2, 7, 1], dtype=np.int32)                 # no zero level
    inp = wl.small_conv(1, 5, 5, 4, 2, 3, 3, pad=(1, 1), seed=2)
    Y = oracle.conv2d(inp.Wc, inp.Ac, lw, la, pad=(1, 1))
    Xpad = np.zeros((1, 7, 7, 4), np.uint8)                      # padded with code 0 (level 4)
    Xpad[:, 1:-1, 1:-1, :] = inp.Ac
    ring = oracle.conv2d(inp.Wc, Xpad, lw, la) - Y               # what the ring of code-0 pixels added
    # the same ring computed alone: image of code 0 everywhere minus the interior part
    mask_levels = np.array([int(la[0]), 0, 0, 0], dtype=np.int32)
    ring_codes = np.ones((1, 7, 7, 4), np.uint8)                 # code 1 -> level 0 under mask_levels
    ring_codes[:, 0, :, :] = ring_codes[:, -1, :, :] = 0
    ring_codes[:, :, 0, :] = ring_codes[:, :, -1, :] = 0
    assert np.array_equal(ring, oracle.conv2d(inp.Wc, ring_codes, lw, mask_levels))


def test_stride2_samples_stride1():
    lw, la = LEVEL_SETS[2]
    inp = wl.small_conv(1, 9, 9, 8, 3, 3, 3, pad=(1, 1), seed=12)
    Y1 = oracle.conv2d(inp.Wc, inp.Ac, lw, la, stride=(1, 1), pad=(1, 1))
    Y2 = oracle.conv2d(inp.Wc, inp.Ac, lw, la, stride=(2, 2), pad=(1, 1))
    assert np.array_equal(Y2, Y1[:, ::2, ::2, :])


def test_batch_items_are_independent():
    lw, la = LEVEL_SETS[1]
    inp = wl.small_conv(3, 6, 6, 8, 4, 3, 3, pad=(1, 1), seed=13)
    Y = oracle.conv2d(inp.Wc, inp.Ac, lw, la, pad=(1, 1))
    for b in range(3):
        assert np.array_equal(Y[b:b + 1], oracle.conv2d(inp.Wc, inp.Ac[b:b + 1], lw, la, pad=(1, 1)))


def test_sampled_variants_agree_with_full():
    lw, la = LEVEL_SETS[2]
    g = wl.small_gemm(13, 17, 48, seed=14)
    full = oracle.gemm(g.Wc, g.Ac, lw, la)
    ms, ns = np.array([0, 12, 5, 5]), np.array([16, 0, 3, 3])
    assert np.array_equal(oracle.gemm_sampled(g.Wc, g.Ac, lw, la, ms, ns), full[ms, ns])
    c = wl.small_conv(2, 6, 7, 8, 5, 3, 3, (2, 1), (1, 1), seed=15)
    Y = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=(2, 1), pad=(1, 1))
    pos = np.array([0, Y.size - 1, 17, 101])
    assert np.array_equal(oracle.conv2d_sampled(c.Wc, c.Ac, lw, la, pos, stride=(2, 1), pad=(1, 1)),
                          Y.reshape(-1)[pos])


# ---- moments of the seeded workload (generator + decode sanity) --------------------------

def test_moments_of_small_gemm_workload():
    # uniform codes: E[lw] = -0.5, E[la] = 1.5, E[lw^2] = 1.5, E[la^2] = 3.5
    # E[C] = 576 * (-0.75) = -432, Var[C] = 576 * (1.5*3.5 - 0.5625) = 2700
    inp = wl.make_inputs(wl.CONFIGS["gemm_64x196x576"])
    C = oracle.gemm(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a).astype(np.float64)
    # C splits into a row part (64 samples, variance 1620), a column part (196 samples, 180) and an
    # interaction part (900): the sample mean has sd ~5.1 and the pooled sample variance sd ~300
    assert abs(C.mean() + 432.0) < 16.0
    assert abs(C.var() / 2700.0 - 1.0) < 0.35
    inter = C - C.mean(axis=0, keepdims=True) - C.mean(axis=1, keepdims=True) + C.mean()
    assert abs(inter.var() / 900.0 - 1.0) < 0.1          # 576 * Var[lw] * Var[la] = 576 * 1.25 * 1.25


def test_relu_skew_distribution():
    codes = wl.draw_codes(np.random.default_rng(0), (200000,), "relu_skew")
    freq = np.bincount(codes, minlength=4) / codes.size
    assert abs(freq[0] - 0.5) < 0.01
    assert np.all(np.abs(freq[1:] - 1.0 / 6.0) < 0.01)


# ---- epilogue ------------------------------------------------------------------------------

def test_scale_epilogue_is_one_float32_multiply():
    acc = np.array([[1, -3, 16777217], [0, 2 ** 30 + 1, -(2 ** 24) - 3]], dtype=np.int32)
    scale = np.array([0.1, 0.037, 0.5], dtype=np.float32)
    want = acc.astype(np.float32) * scale            # numpy: int32 -> float32 (RNE), then float32 multiply
    assert np.array_equal(oracle.scale_epilogue_nhwc(acc, scale), want)
    # the conversion itself rounds to nearest even: 2^24 + 1 -> 2^24
    assert oracle.scale_epilogue_nhwc(np.array([[16777217]], np.int32), np.array([1.0], np.float32))[0, 0] == 16777216.0
    rows = oracle.scale_epilogue_rows(acc.T.copy(), scale)
    assert np.array_equal(rows, want.T)


# ---- error reporting ---------------------------------------------------------------------

def test_oracle_rejects_bad_codes_and_overflow():
    with pytest.raises(oracle.OracleError):
        oracle.gemm(np.full((1, 4), 4, np.uint8), np.zeros((1, 4), np.uint8), LW, LA)
    big = np.array([2 ** 15, 0, 0, 0], dtype=np.int32)
    with pytest.raises(oracle.OracleError):
        oracle.gemm(np.zeros((1, 8), np.uint8), np.zeros((1, 8), np.uint8), big, big)


# ---- activation quantiser (Eq. 1) ------------------------------------------------------------

def test_quantizer_hand_values():
    # s = 2, z = 0.5, signed range [-2, 1]: t = 2x + 0.5, ties go to the even integer
    x = np.array([-10.0, -1.3, -1.25, -1.0, -0.75, -0.5, -0.25, 0.0, 0.2, 0.25, 0.5, 0.75, 3.0], dtype=np.float32)
    #   2x+.5 =   -19.5  -2.1  -2.0  -1.5  -1.0  -0.5   0.0  0.5  0.9   1.0  1.5   2.0  6.5
    #   rint  =   -20    -2    -2    -2    -1    -0     0    0    1     1    2     2    6
    #   clip  =   -2     -2    -2    -2    -1     0     0    0    1     1    1     1    1
    want = np.array([0, 0, 0, 0, 1, 2, 2, 2, 3, 3, 3, 3, 3], dtype=np.uint8)
    assert oracle.quantize_codes(x, 2.0, 0.5, -2, 1).tolist() == want.tolist()
    # unsigned range [0, 3], s = 1, z = 0: rint(0.5) = 0, rint(1.5) = 2, rint(2.5) = 2
    x = np.array([-1.0, 0.0, 0.49, 0.5, 0.51, 1.5, 2.5, 2.51, 3.4, 3.5, 100.0], dtype=np.float32)
    want = np.array([0, 0, 0, 0, 1, 2, 2, 3, 3, 3, 3], dtype=np.uint8)
    assert oracle.quantize_codes(x, 1.0, 0.0, 0, 3).tolist() == want.tolist()


def test_quantizer_matches_numpy_float32_pipeline():
    rng = np.random.default_rng(7)
    x = rng.normal(0, 1.5, size=20000).astype(np.float32)
    for s, z, lo in ((1.7, 0.3, -2), (0.9, -0.2, 0), (3.0, 0.5, -2)):
        t = (np.float32(s) * x).astype(np.float32) + np.float32(z)          # two float32 roundings, no FMA
        want = (np.clip(np.rint(t), lo, lo + 3) - lo).astype(np.uint8)
        assert np.array_equal(oracle.quantize_codes(x, s, z, lo, lo + 3), want)


def test_quantizer_special_values_and_range_check():
    x = np.array([np.nan, np.inf, -np.inf, 1e30, -1e30], dtype=np.float32)
    assert oracle.quantize_codes(x, 1.0, 0.0, -2, 1).tolist() == [0, 3, 0, 3, 0]
    with pytest.raises(oracle.OracleError):
        oracle.quantize_codes(x, 1.0, 0.0, 0, 4)


def test_quantize_then_levels_recovers_a_uniform_grid():
    # a value that already sits on the grid x = (q - z) / s quantises to q: the inverse of Eq. 1 on its range
    s, z = 4.0, 1.0
    q = np.arange(-2, 2)
    x = ((q - z) / s).astype(np.float32)
    assert oracle.quantize_codes(x, s, z, -2, 1).tolist() == [0, 1, 2, 3]


# ---- 3- and 4-bit codes (Sec. 3.3, Table 2: index 3+3 / 4+4 bits, 64 / 256 entries) ---------------------

WIDE_LEVELS = {
    3: (np.array([-4, -3, -2, -1, 0, 1, 2, 3], dtype=np.int32), np.array([0, 1, 2, 3, 4, 5, 6, 7], dtype=np.int32)),
    4: (np.arange(-8, 8, dtype=np.int32), np.array([0, 3, 1, 7, 2, 9, 4, 15, 5, 6, 8, 10, 11, 12, 13, 14], dtype=np.int32)),
}


@pytest.mark.parametrize("bits", [3, 4])
def test_table_sizes_follow_table2(bits):
    lw, la = WIDE_LEVELS[bits]
    table = oracle.build_lut(lw, la)
    assert len(table) == 2 ** (2 * bits) == {3: 64, 4: 256}[bits]        # Table 2: 2^6 = 64, 2^8 = 256 entries
    for w, a in itertools.product(range(2 ** bits), repeat=2):
        assert table[(w << bits) | a] == lw[w] * la[a]


@pytest.mark.parametrize("bits", [3, 4])
def test_wide_codes_all_pairs_and_matmul(bits):
    lw, la = WIDE_LEVELS[bits]
    nlev = 2 ** bits
    Wc = np.repeat(np.arange(nlev, dtype=np.uint8)[:, None], 2, axis=1)
    C = oracle.gemm(Wc, Wc, lw, la)
    for m, n in itertools.product(range(nlev), repeat=2):
        assert C[m, n] == 2 * int(lw[m]) * int(la[n])
    rng = np.random.default_rng(bits)
    Wc, Ac = wl.draw_codes(rng, (13, 40), nlev=nlev), wl.draw_codes(rng, (9, 40), nlev=nlev)
    want = lw.astype(np.int64)[Wc] @ la.astype(np.int64)[Ac].T
    assert np.array_equal(oracle.gemm(Wc, Ac, lw, la).astype(np.int64), want)
    via_table = oracle.lut_gemm_packed(oracle.pack_codes(Wc, bits), oracle.pack_codes(Ac, bits),
                                       oracle.build_lut(lw, la), 40, bits)
    assert np.array_equal(via_table.astype(np.int64), want)
    with pytest.raises(oracle.OracleError):
        oracle.gemm(np.full((1, 2), nlev, np.uint8), np.zeros((1, 2), np.uint8), lw, la)    # code out of range


def test_wide_codes_packing_hand_values():
    # two codes per byte in 4-bit slots: [5, 10] -> 5 + 10*16 = 165; [7, 1] -> 7 + 16 = 23; [0, 15] -> 240
    assert oracle.pack_codes(np.array([[5, 10, 0, 15]], np.uint8), 4).tolist() == [[165, 240]]
    assert oracle.pack_codes(np.array([[7, 1, 3, 0]], np.uint8), 3).tolist() == [[23, 3]]
    assert oracle.unpack_codes(np.array([[165, 240]], np.uint8), 4).tolist() == [[5, 10, 0, 15]]
    with pytest.raises(oracle.OracleError):
        oracle.pack_codes(np.array([[8, 0]], np.uint8), 3)                 # 8 is not a 3-bit code


@pytest.mark.parametrize("bits", [3, 4])
def test_wide_codes_conv_equals_torch(bits):
    lw, la = WIDE_LEVELS[bits]
    rng = np.random.default_rng(10 + bits)
    Wc = wl.draw_codes(rng, (5, 3, 3, 6), nlev=2 ** bits)
    Xc = wl.draw_codes(rng, (2, 7, 8, 6), nlev=2 ** bits)
    x = torch.from_numpy(la.astype(np.float64)[Xc]).permute(0, 3, 1, 2)
    w = torch.from_numpy(lw.astype(np.float64)[Wc]).permute(0, 3, 1, 2)
    want = torch.nn.functional.conv2d(x, w, stride=(2, 1), padding=(1, 1)).permute(0, 2, 3, 1).numpy()
    got = oracle.conv2d(Wc, Xc, lw, la, stride=(2, 1), pad=(1, 1))
    assert np.array_equal(got.astype(np.float64), want)


# ---- tables given as such: non-separable integer tables, binary32 tables (Sec. 5.3) -----------------------

def test_table_oracle_equals_level_oracle_for_product_tables():
    for lw, la in LEVEL_SETS:
        g = wl.small_gemm(11, 13, 36, seed=21)
        assert np.array_equal(oracle.gemm_table(g.Wc, g.Ac, oracle.build_lut(lw, la)), oracle.gemm(g.Wc, g.Ac, lw, la))
        c = wl.small_conv(2, 6, 5, 8, 3, 3, 3, (2, 1), (1, 1), seed=22)
        assert np.array_equal(oracle.conv2d_table(c.Wc, c.Ac, oracle.build_lut(lw, la), stride=(2, 1), pad=(1, 1)),
                              oracle.conv2d(c.Wc, c.Ac, lw, la, stride=(2, 1), pad=(1, 1)))


def test_table_oracle_on_a_non_separable_table_by_one_hot_matmul():
    rng = np.random.default_rng(23)
    table = rng.integers(-100, 100, size=16).astype(np.int32)           # rank 4 with overwhelming probability
    assert np.linalg.matrix_rank(table.reshape(4, 4)) > 1
    g = wl.small_gemm(9, 12, 28, seed=24)
    # C = sum_v  T[Wc][:, :, v] @ onehot(Ac == v)^T : an independent formulation in numpy int64
    want = sum(table.reshape(4, 4).astype(np.int64)[g.Wc][:, :, v] @ (g.Ac == v).astype(np.int64).T for v in range(4))
    assert np.array_equal(oracle.gemm_table(g.Wc, g.Ac, table).astype(np.int64), want)
    assert np.array_equal(oracle.lut_gemm_packed(oracle.pack_codes(g.Wc), oracle.pack_codes(g.Ac), table, 28), want)
    # single-pair brute force: K = 1 picks exactly one entry
    for w, a in itertools.product(range(4), range(4)):
        assert oracle.gemm_table(np.array([[w]], np.uint8), np.array([[a]], np.uint8), table)[0, 0] == table[4 * w + a]


def test_f32_table_is_one_multiply_per_entry():
    lw = np.array([0.1, -0.37, 1.5, 3.0e-3], np.float32)
    la = np.array([0.0, 0.7, 1.9, 2.25], np.float32)
    want = (lw[:, None] * la[None, :]).astype(np.float32).reshape(-1)       # numpy float32 multiply
    assert np.array_equal(oracle.build_lut_f32(lw, la), want)


def test_f32_sum_is_sequential_in_k():
    table = oracle.build_lut_f32(np.array([1.0e8, -1.0e8, 1.0, 0.5], np.float32), np.array([1.0, 1.0, 1.0, 1.0], np.float32))
    # weights: big, small, small, -big.  Sequential float32: ((1e8 + 1) + 0.5) - 1e8 = 0 (both small terms are absorbed);
    # any other order gives 1.5 or 1 or 0.5
    Wc = np.array([[0, 2, 3, 1]], np.uint8)
    Ac = np.zeros((1, 4), np.uint8)
    assert oracle.gemm_table_f32(Wc, Ac, table)[0, 0] == 0.0
    Wc = np.array([[2, 3, 0, 1]], np.uint8)                               # small terms first: (1 + 0.5 + 1e8) - 1e8 = 0 too,
    assert oracle.gemm_table_f32(Wc, Ac, table)[0, 0] == np.float32(np.float32(np.float32(1.5) + np.float32(1e8)) - np.float32(1e8))
    # against numpy's sequential float32 accumulate on random data
    rng = np.random.default_rng(25)
    t = rng.normal(0, 1, 16).astype(np.float32)
    g = wl.small_gemm(5, 6, 200, seed=26)
    got = oracle.gemm_table_f32(g.Wc, g.Ac, t)
    for m, n in itertools.product(range(5), range(6)):
        terms = t[4 * g.Wc[m].astype(np.int64) + g.Ac[n]]
        assert got[m, n] == np.add.accumulate(terms, dtype=np.float32)[-1]


def test_f32_conv_sum_order_is_kh_then_kw_then_ci():
    """Order-sensitive pin of the binary32 convolution (the reading: ascending kh, then kw, then ci, taps outside the
    image skipped, from +0).  Entries depend on the weight code only: 1e8, -1e8, 1, 0.5 (activation levels all 1), and
    1e8 absorbs any 1 or 0.5 added to it in binary32.  Filter, Cin = 2 (code of channel 0 | channel 1 per tap):
        kh=0:  big|0.5   1|0.5   1|0.5
        kh=1: -big|0.5   1|0.5   1|0.5
        kh=2:    1|0.5   1|0.5   1|0.5
    Centre pixel of a 3x3 input with pad 1 (all 9 taps), in the order kh, kw, ci:
        row 0: 1e8, then five absorbed terms -> 1e8;  row 1: -1e8 -> 0, then 0.5 + 1 + 0.5 + 1 + 0.5 = 3.5;
        row 2: + 4.5 = 8.0.
    Other orders give other values: kw before kh 11.0, ci outermost 9.5, any axis descending differs too.
    Corner pixel (0, 0): taps (1,1), (1,2), (2,1), (2,2) only = 4 * 1.5 = 6.0 (the big entries are outside)."""
    table = oracle.build_lut_f32(np.array([1.0e8, -1.0e8, 1.0, 0.5], np.float32), np.ones(4, np.float32))
    BIG, NEG, ONE, HALF = 0, 1, 2, 3
    Wc = np.full((1, 3, 3, 2), ONE, np.uint8)
    Wc[0, :, :, 1] = HALF
    Wc[0, 0, 0, 0], Wc[0, 1, 0, 0] = BIG, NEG
    Xc = np.zeros((1, 3, 3, 2), np.uint8)
    y = oracle.conv2d_table_f32(Wc, Xc, table, pad=(1, 1))
    assert y.shape == (1, 3, 3, 1)
    assert y[0, 1, 1, 0] == 8.0
    assert y[0, 0, 0, 0] == 6.0
    # bottom-right corner (2, 2): taps (0,0), (0,1), (1,0), (1,1): 1e8 (+0.5, +1, +0.5 absorbed) - 1e8 = 0, + 0.5 + 1 + 0.5 = 2.0
    assert y[0, 2, 2, 0] == 2.0


def test_f32_conv_equals_f32_gemm_on_explicit_im2col():
    """With no padding every tap is inside the image, so the convolution is the GEMM on rows gathered in the order
    k = (kh * KW + kw) * Cin + ci -- and the GEMM's sequential order is pinned by test_f32_sum_is_sequential_in_k."""
    rng = np.random.default_rng(31)
    table = rng.normal(0.0, 1.0, 16).astype(np.float32)
    c = wl.small_conv(2, 6, 7, 4, 5, 3, 2, (2, 1), (0, 0), seed=32)
    B, H, W, Cin = c.Ac.shape
    Cout, KH, KW, _ = c.Wc.shape
    sh, sw = 2, 1
    OH, OW = (H - KH) // sh + 1, (W - KW) // sw + 1
    rows = np.empty((B * OH * OW, KH * KW * Cin), np.uint8)
    for b, oh, ow in itertools.product(range(B), range(OH), range(OW)):
        rows[(b * OH + oh) * OW + ow] = c.Ac[b, oh * sh:oh * sh + KH, ow * sw:ow * sw + KW, :].reshape(-1)
    want = oracle.gemm_table_f32(c.Wc.reshape(Cout, -1), rows, table)             # [Cout][N]
    got = oracle.conv2d_table_f32(c.Wc, c.Ac, table, stride=(sh, sw))
    assert np.array_equal(got.reshape(B * OH * OW, Cout), want.T)


def test_f32_table_with_integer_levels_equals_integer_oracle():
    lw, la = LEVEL_SETS[0]
    c = wl.small_conv(1, 6, 6, 8, 4, 3, 3, pad=(1, 1), seed=27)
    t = oracle.build_lut_f32(lw.astype(np.float32), la.astype(np.float32))
    got = oracle.conv2d_table_f32(c.Wc, c.Ac, t, pad=(1, 1))
    assert np.array_equal(got, oracle.conv2d(c.Wc, c.Ac, lw, la, pad=(1, 1)).astype(np.float32))


def test_quantiser_multiply_and_add_are_two_roundings():
    """Eq. 1 decided in binary32 as one multiply, then one add: with s = 1 + 2^-23, x = 0.5 - 2^-23, z = 1 the product
    0.5 - 2^-24 - 2^-46 rounds to 0.5 - 2^-24, the sum 1.5 - 2^-24 is a tie that rounds to 1.5, and rint(1.5) = 2;
    a fused multiply-add would keep the 2^-46, round the sum down to 1.5 - 2^-23 and give 1."""
    s, x, z = np.float32(1 + 2.0 ** -23), np.float32(0.5 - 2.0 ** -23), np.float32(1.0)
    two_step = np.rint(np.float32(np.float32(s * x) + z))
    fused = np.rint(np.float32(np.float64(s) * np.float64(x) + np.float64(z)))
    assert two_step == 2.0 and fused == 1.0                      # the case does tell the two apart
    codes = oracle.quantize_codes(np.full((1, 4), x, np.float32), float(s), float(z), 0, 3)
    assert codes.tolist() == [[2, 2, 2, 2]]
