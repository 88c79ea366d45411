"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bar: bit-exact on int32 accumulators; fp32 epilogue within 1e-6 relative (it is one int->float
conversion and one multiply, so equality is expected and also checked).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2304_09049_amd import binding as dg
from paper_2304_09049_amd import workloads as wl
from gpu_helpers import GpuCase, run_or_unsupported

pytestmark = pytest.mark.gpu

VARIANTS = ["auto", "lds", "perm", "mfma_i8", "smalln", "lut65k", "onehot_mfma", "onehot_smfmac"]

LEVELS = {
    "signed_unsigned": ((-2, -1, 0, 1), (0, 1, 2, 3), dg.DG_LUT_I8),
    "twos_complement": ((0, 1, -2, -1), (3, 1, 0, 2), dg.DG_LUT_I8),
    "nonuniform_i8": ((-8, 7, 3, -5), (-7, 6, -8, 1), dg.DG_LUT_I8),
    "nonuniform_i16": ((-8, 7, 3, -5), (-7, 6, -8, 1), dg.DG_LUT_I16),
    "wide_i8": ((127, -128, 5, 0), (1, 0, 1, 1), dg.DG_LUT_I8),
    "extreme_i16": ((127, -128, 5, 0), (-128, 127, 1, 0), dg.DG_LUT_I16),
    "all_positive": ((1, 2, 3, 4), (4, 3, 2, 1), dg.DG_LUT_I8),
}

GEMM_SHAPES = [
    (1, 1, 4), (3, 5, 8), (4, 4, 4), (17, 9, 20), (64, 196, 576), (70, 130, 192), (129, 257, 320),
    (8, 1, 64), (1, 300, 128), (256, 512, 64), (33, 1000, 1024), (200, 3, 2048), (5, 16, 4096),
]


def _assert_same(got, want, what):
    assert got.shape == want.shape, what
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        first = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {got.size} differ; first at {first}: "
                             f"got {got[first]} want {want[first]}")


def test_pack_activations_matches_the_public_layout():
    rng = np.random.default_rng(0)
    # the last case is large enough for the unrolled kernel, with a remainder for each of the other two
    for rows, K in [(1, 4), (3, 8), (7, 20), (196, 576), (5, 4096), (1000, 36), (4101, 1028)]:
        codes = wl.draw_codes(rng, (rows, K))
        got = dg.dg_pack_activations(torch.from_numpy(codes).cuda(), rows, K).cpu().numpy()
        _assert_same(got.reshape(rows, K // 4), oracle.pack_codes(codes), f"pack {rows}x{K}")


def test_pack_masks_high_bits_and_handles_unaligned_buffers():
    rng = np.random.default_rng(1)
    codes = wl.draw_codes(rng, (9, 52))
    dirty = codes | (rng.integers(0, 64, size=codes.shape, dtype=np.uint8) << 2)   # garbage above bit 1
    base = torch.zeros(9 * 52 + 3, dtype=torch.uint8, device="cuda")
    view = base[3:]                                                                 # 3-byte offset
    view.copy_(torch.from_numpy(dirty.reshape(-1)))
    out = torch.zeros(9 * 13 + 1, dtype=torch.uint8, device="cuda")[1:]
    dg.dg_pack_activations(view, 9, 52, out=out)
    _assert_same(out.cpu().numpy().reshape(9, 13), oracle.pack_codes(codes), "unaligned pack")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("shape", GEMM_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_gemm_parity(shape, variant):
    M, N, K = shape
    inp = wl.small_gemm(M, N, K, seed=M * 7 + N * 3 + K)
    case = GpuCase(inp)
    got = run_or_unsupported(case, variant)
    if got is None:
        pytest.skip(f"{variant} declares {shape} unsupported")
    _assert_same(got, oracle.gemm(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a), f"gemm {shape} {variant}")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("shape", [(64, 196, 576), (37, 41, 4096), (130, 70, 64)], ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("levels", sorted(LEVELS))
def test_gemm_parity_level_tables(levels, shape, variant):
    lw, la, entry = LEVELS[levels]
    M, N, K = shape
    inp = wl.small_gemm(M, N, K, seed=11 + K)
    case = GpuCase(inp, levels=(lw, la), entry=entry)
    got = run_or_unsupported(case, variant)
    if got is None:
        pytest.skip(f"{variant} declares {levels} {shape} unsupported")
    _assert_same(got, oracle.gemm(inp.Wc, inp.Ac, lw, la), f"gemm {levels} {shape} {variant}")


CONV_CASES = [
    # B, H, W, Cin, Cout, KH, KW, stride, pad
    (1, 3, 3, 4, 4, 3, 3, (1, 1), (1, 1)),
    (2, 7, 9, 8, 5, 3, 3, (1, 1), (1, 1)),
    (1, 8, 8, 16, 6, 3, 3, (2, 2), (1, 1)),
    (2, 9, 6, 12, 4, 1, 1, (1, 1), (0, 0)),
    (1, 10, 7, 4, 3, 5, 3, (2, 1), (2, 0)),
    (1, 6, 11, 8, 2, 1, 7, (1, 3), (0, 3)),
    (3, 5, 5, 16, 7, 3, 3, (1, 1), (0, 0)),
    (1, 14, 14, 64, 64, 3, 3, (1, 1), (1, 1)),
    (2, 13, 11, 64, 70, 3, 3, (1, 1), (1, 1)),
    (1, 28, 28, 128, 33, 3, 3, (2, 2), (1, 1)),
    (3, 9, 9, 256, 64, 1, 1, (1, 1), (0, 0)),
    (1, 12, 12, 32, 40, 3, 3, (1, 1), (2, 2)),
    (1, 17, 15, 48, 24, 5, 5, (1, 1), (2, 2)),
    (2, 16, 16, 16, 130, 3, 3, (1, 1), (1, 1)),
    (1, 9, 9, 64, 16, 7, 7, (2, 2), (3, 3)),
]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("levels", ["signed_unsigned", "nonuniform_i8"])      # the second has no zero activation level
@pytest.mark.parametrize("case_", CONV_CASES, ids=lambda c: "-".join(map(str, c[:7])))
def test_conv_parity(case_, levels, variant):
    B, H, W, Cin, Cout, KH, KW, stride, pad = case_
    lw, la, entry = LEVELS[levels]
    inp = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H * W + Cin + Cout)
    case = GpuCase(inp, levels=(lw, la), entry=entry)
    got = run_or_unsupported(case, variant)
    if got is None:
        pytest.skip(f"{variant} declares {case_} {levels} unsupported")
    want = oracle.conv2d(inp.Wc, inp.Ac, lw, la, stride=stride, pad=pad)
    _assert_same(got, want, f"conv {case_} {levels} {variant}")


ONEHOT_PLANS = {"split": "onehot_mfma_splitk_s", "1": "onehot_mfma_64x32", "2": "onehot_mfma_64x64",
                "4": "onehot_mfma_64x128", "7": "onehot_mfma_64x224",
                # 2 or 4 wavefronts sharing a tile and splitting K
                "1k2": "onehot_mfma_64x32_k2", "1k4": "onehot_mfma_64x32_k4", "2k2": "onehot_mfma_64x64_k2",
                "2k4": "onehot_mfma_64x64_k4", "4k2": "onehot_mfma_64x128_k2", "4k4": "onehot_mfma_64x128_k4",
                "7k4": "onehot_mfma_64x224_k4",
                # the decode-and-multiply comparison's own 128 x 128 tile
                "44": "mfma_i8_128x128"}


@pytest.mark.parametrize("table", ["signed_unsigned", "extreme_i16", "decode", "sparse"])
@pytest.mark.parametrize("plan", sorted(ONEHOT_PLANS))
def test_onehot_every_plan(plan, table, monkeypatch):
    """Every wave tile of the one-hot matrix-core kernel and its split-K form, forced on shapes with ragged edges in
    M and N (the library picks among them by a cost model that small test shapes would never move off one plan):
    GEMM with row-major and column-major output, convolution with padding and stride, int32 and scaled fp32 output.
    Once with an int8 table (one plane), once with entries up to 16384 (two int8 planes), and once as the
    decode-and-multiply comparison kernel and once as the sparse-instruction table kernel, which are built in the same
    frame and have the same plans."""
    if "k" in plan and table == "extreme_i16":
        pytest.skip("tiles are shared only by the one-plane kernels")
    if plan == "44" and table != "decode":
        pytest.skip("only the comparison kernel has the 128 x 128 tile")
    if plan.startswith("7") and table == "sparse":
        pytest.skip("the sparse instruction's sums stay in the vector registers: no 64 x 224 tile")
    monkeypatch.setenv("DG_ONEHOT_PLAN", plan)
    glw, gla, gentry = LEVELS[{"decode": "extreme_i16", "sparse": "nonuniform_i8"}.get(table, table)]
    kernel = {"decode": "mfma_i8", "sparse": "onehot_smfmac"}.get(table, "onehot_mfma")
    prefix = ONEHOT_PLANS[plan]
    if table == "extreme_i16":
        prefix = prefix.replace("onehot_mfma_", "onehot_mfma_2p_").replace("_64x", "_32x")
    if table == "decode":
        prefix = prefix.replace("onehot_mfma_", "mfma_i8_")
    if table == "sparse":
        prefix = prefix.replace("onehot_mfma_", "onehot_smfmac_")

    def chunk_codes(c):                  # codes a wavefront takes at a time: 4, 2 or 1 words per lane half (sparse, where a
        return 128 if c % 128 == 0 and table != "sparse" else (64 if c % 64 == 0 else 32)     # K share matters: 2 or 1)

    def right_kernel(name, chunks, channels):
        if plan == "split":
            return name.startswith(prefix)
        want = prefix
        if "k" in plan and chunks < int(plan.split("k")[1]):
            want = prefix.rsplit("_k", 1)[0]                # fewer chunks than sharers: the unshared kernel
        return name == want

    for (M, N, K) in [(70, 1000, 96), (130, 777, 64), (64, 300, 256), (33, 250, 1024)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K)
        case = GpuCase(inp, levels=(glw, gla), entry=gentry)
        assert right_kernel(case.kernel_name(kernel), K // chunk_codes(K), K)
        want = oracle.gemm(inp.Wc, inp.Ac, glw, gla)
        _assert_same(case.run(kernel).cpu().numpy(), want, f"gemm {(M, N, K)} plan {plan}")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant=kernel, strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"gemm {(M, N, K)} column-major plan {plan}")
    # no zero activation level: padding must still add 0
    lw, la, entry = LEVELS["nonuniform_i8"] if table in ("signed_unsigned", "sparse") else ((127, -128, 5, 3), (-128, 127, 1, 2), dg.DG_LUT_I16)
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in [(2, 24, 24, 32, 70, 3, 3, (1, 1), (1, 1)),
                                                      (1, 30, 30, 128, 40, 3, 3, (2, 2), (1, 1)),
                                                      (3, 16, 16, 64, 33, 1, 1, (1, 1), (0, 0)),
                                                      (1, 20, 20, 64, 96, 5, 5, (1, 1), (2, 2))]:
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert right_kernel(case.kernel_name(kernel), KH * KW * Cin // chunk_codes(Cin), Cin)
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
        _assert_same(case.run(kernel).cpu().numpy(), acc, f"conv {(B, H, W, Cin, Cout)} plan {plan}")
        got = case.run(kernel, scale=True).cpu().numpy()
        assert np.array_equal(got, oracle.scale_epilogue_nhwc(acc, c.scale)), f"scaled conv plan {plan}"


def test_two_plane_tables_on_the_sparse_instruction():
    """Entries beyond int8 through the sparse-instruction kernel (two int8 planes selected by the same index registers):
    GEMMs with ragged edges in both output layouts, convolutions with padding and stride under a table with no zero
    activation level, int32 and scaled fp32 output, chunk widths of one and two words."""
    kernel = "onehot_smfmac"
    glw, gla, gentry = LEVELS["extreme_i16"]
    for (M, N, K) in [(70, 1000, 96), (130, 777, 64), (33, 250, 1024), (1, 129, 32), (300, 5, 128)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K)
        case = GpuCase(inp, levels=(glw, gla), entry=gentry)
        assert case.kernel_name(kernel) == "onehot_smfmac_2p_32x128"
        want = oracle.gemm(inp.Wc, inp.Ac, glw, gla)
        _assert_same(case.run(kernel).cpu().numpy(), want, f"gemm {(M, N, K)}")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant=kernel, strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"gemm {(M, N, K)} column-major")
    lw, la, entry = (127, -128, 5, 3), (-128, 127, 1, 2), dg.DG_LUT_I16
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in [(2, 24, 24, 32, 70, 3, 3, (1, 1), (1, 1)),
                                                      (1, 30, 30, 128, 40, 3, 3, (2, 2), (1, 1)),
                                                      (3, 16, 16, 64, 33, 1, 1, (1, 1), (0, 0)),
                                                      (1, 20, 20, 64, 96, 5, 5, (1, 1), (2, 2)),
                                                      (1, 7, 9, 96, 3, 3, 3, (1, 1), (2, 2))]:
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert case.kernel_name(kernel) == "onehot_smfmac_2p_32x128"
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
        _assert_same(case.run(kernel).cpu().numpy(), acc, f"conv {(B, H, W, Cin, Cout)}")
        got = case.run(kernel, scale=True).cpu().numpy()
        assert np.array_equal(got, oracle.scale_epilogue_nhwc(acc, c.scale)), "scaled conv"
    # AUTO takes it where its 32 x 128 tiles fill the chip, and the dense-instruction kernel below that
    big = GpuCase(wl.small_conv(16, 56, 56, 64, 96, 3, 3, (1, 1), (1, 1), seed=5), levels=(lw, la), entry=entry)
    assert big.kernel_name("auto") == "onehot_smfmac_2p_32x128"
    want = oracle.conv2d(big.inp.Wc, big.inp.Ac, lw, la, stride=(1, 1), pad=(1, 1))
    _assert_same(big.run("auto").cpu().numpy(), want, "AUTO on a large two-plane layer")
    # the fused layer on the same large layer (AUTO: the same sparse-instruction kernel with the re-quantising epilogue)
    cb = wl.small_conv(16, 56, 56, 64, 96, 3, 3, (1, 1), (1, 1), seed=5, scale=True)
    bigs = GpuCase(cb, levels=(lw, la), entry=entry)
    y = oracle.scale_epilogue_nhwc(want, cb.scale)
    qs = float(np.float32(3.0 / max(1e-6, float(np.percentile(np.abs(y), 90)))))
    packed = oracle.pack_codes(oracle.quantize_codes(y, qs, 0.5, 0, 3).reshape(-1, 96))
    got = dg.dg_conv2d_lut_requant(bigs.lut, bigs.Wp, bigs.Ap, bigs.desc, bigs.scale, qs, 0.5, 0)
    torch.cuda.synchronize()
    _assert_same(got.cpu().numpy().reshape(-1, 24), packed, "fused large two-plane layer")
    small = GpuCase(wl.small_conv(1, 14, 14, 32, 96, 1, 1, (1, 1), (0, 0), seed=5), levels=(lw, la), entry=entry)
    assert small.kernel_name("auto").startswith("onehot_mfma_2p_")


def test_convolution_from_unpacked_codes(monkeypatch):
    """dg_conv2d_lut_codes (packing stage + convolution in one call) against the oracle's convolution of the same
    codes: small layers, where the split-K kernel packs the codes itself as it loads them (padding, stride, ragged
    Cout and pixel counts, chunk widths of 1, 2 and 4 words, one- and two-plane tables, int32 and scaled output, codes
    with garbage above their two bits), and layers it hands to the packing kernel and another convolution kernel."""
    cases = [(2, 24, 24, 32, 70, 3, 3, (1, 1), (1, 1)), (1, 30, 30, 128, 40, 3, 3, (2, 2), (1, 1)),
             (3, 16, 16, 64, 33, 1, 1, (1, 1), (0, 0)), (1, 20, 20, 64, 96, 5, 5, (1, 1), (2, 2)),
             (1, 7, 9, 96, 3, 3, 3, (1, 1), (2, 2)), (1, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1)),
             (1, 5, 5, 256, 130, 3, 3, (1, 1), (1, 1))]
    rng = np.random.default_rng(77)
    for table in ("nonuniform_i8", "extreme_i16"):
        monkeypatch.setenv("DG_ONEHOT_PLAN", "split")       # (the 1 x 1 layer would otherwise run on a tiled kernel)
        lw, la, entry = LEVELS[table] if table == "nonuniform_i8" else ((127, -128, 5, 3), (-128, 127, 1, 2), dg.DG_LUT_I16)
        for (B, H, W, Cin, Cout, KH, KW, stride, pad) in cases:
            c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout, scale=True)
            case = GpuCase(c, levels=(lw, la), entry=entry)
            name = dg.dg_conv_codes_kernel_name(case.lut, case.desc)
            assert name.startswith("codes_onehot_mfma_2p_splitk_s" if table == "extreme_i16" else "codes_onehot_mfma_splitk_s"), name
            dirty = c.Ac | (rng.integers(0, 64, size=c.Ac.shape, dtype=np.uint8) << 2)      # garbage above bit 1
            Xc = torch.from_numpy(dirty).cuda()
            acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
            got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc)                   # no work buffer: must fuse
            torch.cuda.synchronize()
            _assert_same(got.cpu().numpy(), acc, f"codes conv {(B, H, W, Cin, Cout)} {table}")
            got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, scale=case.scale)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), oracle.scale_epilogue_nhwc(acc, c.scale)), "scaled codes conv"
    # codes at an address that is not 16-byte aligned: not fused (the packing kernel takes any address), same result
    c = wl.small_conv(1, 12, 12, 64, 40, 3, 3, (1, 1), (1, 1), seed=9)
    case = GpuCase(c, levels=LEVELS["nonuniform_i8"][:2], entry=dg.DG_LUT_I8)
    base = torch.zeros(c.Ac.size + 3, dtype=torch.uint8, device="cuda")
    base[3:].copy_(torch.from_numpy(c.Ac.reshape(-1)))
    got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, base[3:], case.desc, work=torch.empty_like(case.Ap))
    torch.cuda.synchronize()
    _assert_same(got.cpu().numpy(), oracle.conv2d(c.Wc, c.Ac, *LEVELS["nonuniform_i8"][:2], stride=(1, 1), pad=(1, 1)), "unaligned codes")
    with pytest.raises(dg.DgError) as e:
        dg.dg_conv2d_lut_codes(case.lut, case.Wp, base[3:], case.desc)
    assert e.value.status == 1
    # layers that are not fused: a channel count the one-hot kernels do not take, a variant that never fuses, and a
    # layer for the tiled kernels whose channels are not whole 64-code chunks -- packed into the work buffer, then run
    # as dg_conv2d_lut runs them
    monkeypatch.delenv("DG_ONEHOT_PLAN")
    monkeypatch.setenv("DG_ONEHOT_CODES_TILED", "0")      # (the tiled kernel that packs would take the last one)
    lw, la, entry = LEVELS["nonuniform_i8"]
    for (shape, variant) in (((2, 9, 9, 16, 20, 3, 3, (1, 1), (1, 1)), "auto"), ((1, 14, 14, 64, 64, 3, 3, (1, 1), (1, 1)), "lds"),
                             ((8, 56, 56, 96, 64, 3, 3, (1, 1), (1, 1)), "auto"),
                             # 1x1 with a stride, no padding: only the pixels read are packed, and the layer runs on them
                             # without the stride (odd image sizes, different strides, a layer for the stationary-weight kernel)
                             ((8, 56, 56, 48, 64, 1, 1, (2, 2), (0, 0)), "auto"), ((4, 30, 31, 16, 40, 1, 1, (2, 3), (0, 0)), "auto"),
                             ((3, 29, 30, 256, 64, 1, 1, (2, 2), (0, 0)), "lds"), ((16, 57, 56, 256, 96, 1, 1, (2, 2), (0, 0)), "onehot_smfmac")):
        B, H, W, Cin, Cout, KH, KW, stride, pad = shape
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=5)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        name = dg.dg_conv_codes_kernel_name(case.lut, case.desc, variant)
        assert not name.startswith("codes_")
        Xc = torch.from_numpy(c.Ac).cuda()
        work = torch.zeros(B * H * W * Cin // 4, dtype=torch.uint8, device="cuda")
        got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, work=work, variant=variant)
        torch.cuda.synchronize()
        _assert_same(got.cpu().numpy(), oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad), f"unfused {shape}")
        if stride == (1, 1):
            assert name == case.kernel_name(variant)
            _assert_same(work.cpu().numpy().reshape(-1, Cin // 4), oracle.pack_codes(c.Ac.reshape(-1, Cin)), "work buffer")
        else:
            read = np.ascontiguousarray(c.Ac.reshape(B, H, W, Cin)[:, ::stride[0], ::stride[1], :]).reshape(-1, Cin)
            _assert_same(work.cpu().numpy()[:read.shape[0] * Cin // 4].reshape(-1, Cin // 4), oracle.pack_codes(read), "work buffer")
            if variant == "onehot_smfmac":
                assert name == "onehot_smfmac_ws_32xK"
        with pytest.raises(dg.DgError) as e:                                                  # needed and missing / too small
            dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, variant=variant)
        assert e.value.status == 1
        with pytest.raises(dg.DgError) as e:
            dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, work=work[:-1], variant=variant)
        assert e.value.status == 4


@pytest.mark.parametrize("plan,tile", [("1", "64x32"), ("2", "64x64"), ("1k2", "64x32_k2"), ("2k2", "64x64_k2"),
                                       ("1k4", "64x32_k4"), ("2k4", "64x64_k4")])
def test_tiled_kernel_on_unpacked_codes(plan, tile, monkeypatch):
    """The one-call entry points on the tiled kernel packing the codes itself (64 x 32 and 64 x 64 tiles, K unshared or
    shared by 2 or 4 wavefronts) -- on the sparse instruction where the output's channel axis is the contiguous one
    (convolutions, column-major GEMMs) unless the dense one's variant is named, else on the dense instruction:
    convolutions with windows, strides and padding, 64 to 320 channels, ragged M and N, garbage above bit 1 of the code
    bytes, scaled output; GEMMs in both output layouts; no work buffer."""
    monkeypatch.setenv("DG_ONEHOT_PLAN", plan)
    name, sparse_name = "codes_onehot_mfma_" + tile, "codes_onehot_smfmac_" + tile
    lw, la, entry = LEVELS["nonuniform_i8"]
    convs = [(2, 9, 7, 64, 36, 3, 3, (1, 1), (1, 1)), (1, 13, 11, 192, 70, 3, 3, (2, 2), (1, 1)), (3, 6, 5, 320, 64, 1, 1, (1, 1), (0, 0)),
             (1, 20, 17, 128, 130, 3, 2, (1, 2), (1, 0)), (2, 15, 15, 64, 100, 5, 5, (1, 1), (2, 2)), (1, 29, 29, 256, 70, 3, 3, (1, 1), (1, 1))]
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in convs:
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert dg.dg_conv_codes_kernel_name(case.lut, case.desc, "auto") == sparse_name
        assert dg.dg_conv_codes_kernel_name(case.lut, case.desc, "onehot_smfmac") == sparse_name
        assert dg.dg_conv_codes_kernel_name(case.lut, case.desc, "onehot_mfma") == name
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
        dirty = c.Ac | (np.random.default_rng(H + Cout).integers(0, 64, size=c.Ac.shape, dtype=np.uint8) << 2)
        Xc = torch.from_numpy(dirty).cuda()
        for variant in ("onehot_mfma", "onehot_smfmac", "auto"):
            got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, variant=variant)
            torch.cuda.synchronize()
            _assert_same(got.cpu().numpy(), acc, f"tiled conv on codes {(B, H, W, Cin, Cout, KH, KW, stride, pad)} {variant}")
        got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, scale=case.scale, variant="onehot_mfma")
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.scale_epilogue_nhwc(acc, c.scale))
        got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, scale=case.scale)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.scale_epilogue_nhwc(acc, c.scale))
    for (M, N, K) in [(70, 1000, 512), (64, 333, 576), (200, 64, 1280), (33, 5, 640)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K)
        case = GpuCase(inp, levels=(lw, la), entry=entry)
        assert dg.dg_gemm_codes_kernel_name(case.lut, M, N, K) == name
        Ac = torch.from_numpy(inp.Ac).cuda()
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K)
        torch.cuda.synchronize()
        _assert_same(got.cpu().numpy(), want, f"tiled gemm on codes {(M, N, K)} row-major")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, out=out, strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"tiled gemm on codes {(M, N, K)} column-major")
    # channels that are not whole 64-code chunks, or a wider tile: the packing kernel first
    c = wl.small_conv(1, 8, 8, 96, 32, 3, 3, (1, 1), (1, 1), seed=1)
    assert not dg.dg_conv_codes_kernel_name(GpuCase(c, levels=(lw, la), entry=entry).lut, GpuCase(c, levels=(lw, la), entry=entry).desc).startswith("codes_")


def test_gemm_from_unpacked_codes(monkeypatch):
    """dg_gemm_lut_codes against the oracle: small GEMMs where the split-K kernel packs the codes itself (row-major and
    column-major output, scaled output, one- and two-plane tables, ragged M and N, chunk widths of 1 and 2 words), and
    GEMMs with one to a few columns on the few-columns kernel, which does the same, and GEMMs it hands to the packing
    kernel first (K % 32 != 0, a tiled-kernel problem with K % 64 != 0, another variant)."""
    for table in ("nonuniform_i8", "extreme_i16"):
        lw, la, entry = LEVELS[table]
        for (M, N, K) in [(64, 196, 576), (70, 300, 96), (33, 250, 1024), (130, 77, 64), (5, 16, 3072), (1, 40, 32)]:
            monkeypatch.setenv("DG_ONEHOT_PLAN", "split")
            g = wl.make_inputs(wl.Workload(name="g", kind="gemm", M=M, N=N, K=K, scale=True, seed=M + N + K))
            case = GpuCase(g, levels=(lw, la), entry=entry)
            assert dg.dg_gemm_codes_kernel_name(case.lut, M, N, K).startswith("codes_onehot_mfma_")
            Ac = torch.from_numpy(g.Ac).cuda()
            want = oracle.gemm(g.Wc, g.Ac, lw, la)
            got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K)                       # no work buffer: must fuse
            torch.cuda.synchronize()
            _assert_same(got.cpu().numpy(), want, f"codes gemm {(M, N, K)} {table}")
            out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
            dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, out=out, strides=(1, M))
            torch.cuda.synchronize()
            _assert_same(out.cpu().numpy(), want.T.copy(), f"codes gemm {(M, N, K)} {table} column-major")
            got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, scale=case.scale)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), oracle.scale_epilogue_rows(want, g.scale)), "scaled codes gemm"
    monkeypatch.delenv("DG_ONEHOT_PLAN")
    lw, la, entry = LEVELS["nonuniform_i8"]
    # one or two columns: the few-columns kernel reads the codes as they are (AUTO for N <= 2, or asked for by name)
    for (M, N, K, variant) in [(200, 1, 2048, "auto"), (37, 2, 4096, "auto"), (64, 3, 1024, "smalln"), (130, 5, 8192, "smalln"),
                               (9, 7, 96, "smalln")]:
        g = wl.make_inputs(wl.Workload(name="g", kind="gemm", M=M, N=N, K=K, scale=True, seed=M + N + K))
        case = GpuCase(g, levels=(lw, la), entry=entry)
        assert dg.dg_gemm_codes_kernel_name(case.lut, M, N, K, variant) == "codes_smalln"
        Ac = torch.from_numpy(g.Ac | 0xA8).cuda()                                           # garbage above bit 1
        want = oracle.gemm(g.Wc, g.Ac, lw, la)
        got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, variant=variant)
        torch.cuda.synchronize()
        _assert_same(got.cpu().numpy(), want, f"codes gemm {(M, N, K)} few columns")
        got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, scale=case.scale, variant=variant)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.scale_epilogue_rows(want, g.scale)), "scaled codes gemm, few columns"
    for (M, N, K, variant) in [(17, 9, 20, "auto"), (256, 4096, 544, "auto"), (64, 196, 576, "perm")]:
        g = wl.small_gemm(M, N, K, seed=3)
        case = GpuCase(g, levels=(lw, la), entry=entry)
        name = dg.dg_gemm_codes_kernel_name(case.lut, M, N, K, variant)
        assert not name.startswith("codes_") and name == case.kernel_name(variant)
        Ac = torch.from_numpy(g.Ac).cuda()
        work = torch.zeros(N * K // 4, dtype=torch.uint8, device="cuda")
        got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, work=work, variant=variant)
        torch.cuda.synchronize()
        _assert_same(got.cpu().numpy(), oracle.gemm(g.Wc, g.Ac, lw, la), f"unfused gemm {(M, N, K)}")
        with pytest.raises(dg.DgError) as e:
            dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, variant=variant)
        assert e.value.status == 1


def test_random_convolution_shapes():
    """Seeded random convolution geometries (image, filter, stride, padding, channel counts, batch) through AUTO and
    every variant that accepts them: the oracle is the plain nested loop, so any disagreement is a kernel indexing bug."""
    rng = np.random.default_rng(2024)
    lw, la, entry = LEVELS["nonuniform_i8"]              # no zero activation level
    ran = {v: 0 for v in VARIANTS}
    for _ in range(40):
        KH, KW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        ph, pw = int(rng.integers(0, KH)), int(rng.integers(0, KW))
        H, W = int(rng.integers(KH, 24)), int(rng.integers(KW, 24))
        Cin = int(rng.choice([4, 8, 16, 32, 48, 64, 96, 128, 256]))
        Cout = int(rng.integers(1, 140))
        B = int(rng.integers(1, 5))
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, (sh, sw), (ph, pw), seed=int(rng.integers(1 << 30)))
        case = GpuCase(c, levels=(lw, la), entry=entry)
        want = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=(sh, sw), pad=(ph, pw))
        for variant in VARIANTS:
            got = run_or_unsupported(case, variant)
            if got is not None:
                ran[variant] += 1
                _assert_same(got, want, f"conv B={B} {H}x{W} Cin={Cin} Cout={Cout} {KH}x{KW} s=({sh},{sw}) p=({ph},{pw}) {variant}")
    assert ran["auto"] == 40 and ran["lds"] == 40 and ran["onehot_mfma"] >= 10 and ran["perm"] >= 10


def test_golden_tiny_conv_on_gpu(golden_dir):
    import json, os
    from test_oracle_pins import _tiny_conv_weights
    g = json.load(open(os.path.join(golden_dir, "tiny_conv.json")))
    Wc, Xc = _tiny_conv_weights(g), np.array(g["X"], dtype=np.uint8)
    for stride, key in (((1, 1), "Y_stride1"), ((2, 2), "Y_stride2")):
        inp = wl.Inputs(workload=wl._conv("tiny", 1, 3, 3, 4, 4, 3, 3, stride, (1, 1)), levels_w=np.array(g["levels_w"]),
                        levels_a=np.array(g["levels_a"]), Wc=Wc, Ac=Xc)
        for variant in VARIANTS:
            got = run_or_unsupported(GpuCase(inp), variant)
            if got is not None:
                _assert_same(got[0].transpose(2, 0, 1), np.array(g[key], dtype=np.int32), f"tiny conv {variant}")


@pytest.mark.parametrize("variant", VARIANTS)
def test_scale_epilogue(variant):
    # convolution (NHWC, scale per channel) and GEMM (scale per row)
    c = wl.small_conv(2, 13, 11, 64, 70, 3, 3, (1, 1), (1, 1), seed=5, scale=True)
    case = GpuCase(c)
    got = run_or_unsupported(case, variant, scale=True)
    if got is None:
        pytest.skip(f"{variant} unsupported")
    acc = oracle.conv2d(c.Wc, c.Ac, c.levels_w, c.levels_a, stride=(1, 1), pad=(1, 1))
    want = oracle.scale_epilogue_nhwc(acc, c.scale)
    assert got.dtype == np.float32
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=0)
    assert np.array_equal(got, want)          # one conversion and one multiply: expected to be identical

    g = wl.make_inputs(wl.Workload(name="g", kind="gemm", M=70, N=130, K=192, scale=True, seed=3))
    gc = GpuCase(g)
    gg = run_or_unsupported(gc, variant, scale=True)
    if gg is not None:
        want = oracle.scale_epilogue_rows(oracle.gemm(g.Wc, g.Ac, g.levels_w, g.levels_a), g.scale)
        np.testing.assert_allclose(gg, want, rtol=1e-6, atol=0)


@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_output_strides(variant):
    # write C transposed ([N][M]) through the stride arguments
    inp = wl.small_gemm(70, 130, 192, seed=21)
    case = GpuCase(inp)
    out = torch.full((130, 70), -7, dtype=torch.int32, device="cuda")
    try:
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, 70, 130, 192, out=out, variant=variant, strides=(1, 70))
    except dg.DgError as e:
        if e.status == 5:
            pytest.skip(f"{variant} unsupported")
        raise
    torch.cuda.synchronize()
    _assert_same(out.cpu().numpy(), oracle.gemm(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a).T.copy(), "strided")


def test_results_do_not_depend_on_code_statistics():
    # constant codes (every product the same table entry) and the skewed distribution
    for c, d in ((0, 3), (3, 3), (2, 1)):
        inp = wl.small_gemm(66, 140, 576, seed=1)
        inp.Wc[:] = c
        inp.Ac[:] = d
        for variant in VARIANTS:
            got = run_or_unsupported(GpuCase(inp), variant)
            if got is not None:
                assert np.all(got == 576 * int(inp.levels_w[c]) * int(inp.levels_a[d])), (c, d, variant)
    inp = wl.small_gemm(64, 300, 256, seed=2, dist="relu_skew")
    want = oracle.gemm(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a)
    for variant in VARIANTS:
        got = run_or_unsupported(GpuCase(inp), variant)
        if got is not None:
            _assert_same(got, want, f"skew {variant}")


@pytest.mark.parametrize("variant", VARIANTS)
def test_gemm_general_output_strides(variant):
    # neither stride is 1: every output lands in its own slot of a padded buffer, nothing else is touched
    M, N, K = 70, 130, 192
    inp = wl.small_gemm(M, N, K, seed=22)
    case = GpuCase(inp)
    scm, scn = 3 * N + 5, 3
    out = torch.full((M * scm,), -7, dtype=torch.int32, device="cuda")
    try:
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant=variant, strides=(scm, scn))
    except dg.DgError as e:
        if e.status == 5:
            pytest.skip(f"{variant} unsupported")
        raise
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = np.full(M * scm, -7, dtype=np.int32)
    ref = oracle.gemm(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a)
    idx = (np.arange(M)[:, None] * scm + np.arange(N)[None, :] * scn)
    want[idx.reshape(-1)] = ref.reshape(-1)
    _assert_same(got, want, f"general strides {variant}")


@pytest.mark.parametrize("variant", VARIANTS)
def test_degenerate_tables(variant):
    # all-zero table (range 0), a table with a single non-zero entry, and a constant non-zero table
    inp = wl.small_gemm(66, 140, 320, seed=31)
    for lw, la in (((0, 0, 0, 0), (1, 2, 3, 4)), ((0, 0, 5, 0), (0, -7, 0, 0)), ((3, 3, 3, 3), (-2, -2, -2, -2))):
        got = run_or_unsupported(GpuCase(inp, levels=(lw, la), entry=dg.DG_LUT_I8), variant)
        if got is not None:
            _assert_same(got, oracle.gemm(inp.Wc, inp.Ac, lw, la), f"degenerate {lw} {la} {variant}")


@pytest.mark.parametrize("variant", VARIANTS)
def test_long_reduction_near_the_int32_limit(variant):
    # K = 131072 with |entries| up to 127*127: |sum| can reach 2^31 -> rejected; with entries up to 16129 / 2 it fits
    K = 131072
    inp = wl.small_gemm(6, 10, K, seed=32)
    inp.Wc[0, :] = 0
    inp.Ac[0, :] = 0                      # output (0,0) is K * lw[0] * la[0]: the largest magnitude the table allows
    lw, la = (127, -128, 5, 0), (127, -128, 1, 0)
    with pytest.raises(dg.DgError) as e:
        GpuCase(inp, levels=(lw, la), entry=dg.DG_LUT_I16).run(variant)
    assert e.value.status in (3, 5)       # DG_ERR_RANGE (or UNSUPPORTED for a variant that rejects the shape first)
    lw, la = (63, -64, 5, 0), (127, -128, 1, 0)          # 131072 * 8192 = 2^30
    case = GpuCase(inp, levels=(lw, la), entry=dg.DG_LUT_I16)
    got = run_or_unsupported(case, variant)
    if got is not None:
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        assert want[0, 0] == K * 63 * 127
        _assert_same(got, want, f"long K {variant}")
    # an int8 table of full range (255) over the same K exercises the 16-bit-lane fold period
    lw, la = (127, -128, 5, 0), (1, 0, 1, 1)
    got = run_or_unsupported(GpuCase(inp, levels=(lw, la), entry=dg.DG_LUT_I8), variant)
    if got is not None:
        _assert_same(got, oracle.gemm(inp.Wc, inp.Ac, lw, la), f"long K int8 {variant}")


def test_empty_and_bad_shapes_launch_nothing():
    lut = dg.dg_build_lut((-2, -1, 0, 1), (0, 1, 2, 3))
    buf = torch.zeros(64, dtype=torch.uint8, device="cuda")
    out = torch.full((16,), 9, dtype=torch.int32, device="cuda")
    for M, N, K in ((0, 4, 4), (4, 0, 4), (4, 4, 0), (4, 4, 6), (-1, 4, 4)):
        with pytest.raises(dg.DgError) as e:
            dg.dg_gemm_lut(lut, buf, buf, M, N, K, out=out)
        assert e.value.status == 2
    torch.cuda.synchronize()
    assert bool((out == 9).all())


def test_quantize_pack_matches_oracle_quantiser_and_packing():
    rng = np.random.default_rng(40)
    cases = [(7, 20, 1.7, 0.3, -2), (196, 576, 0.9, -0.2, 0), (33, 4096, 3.0, 0.5, -2), (1, 4, 1.0, 0.0, 0)]
    for N, K, s, z, lo in cases:
        x = rng.normal(0.3, 1.2, size=(N, K)).astype(np.float32)
        # plant exact ties, huge values and non-finite values
        flat = x.reshape(-1)
        specials = np.array([0.5, -0.5, 1.5, 2.5, -1.5, 1e30, -1e30, np.inf, -np.inf, np.nan, 0.0, -0.0], np.float32)
        flat[: min(flat.size, specials.size)] = specials[: flat.size]
        got = dg.dg_quantize_pack_activations(torch.from_numpy(x).cuda(), N, K, s, z, lo).cpu().numpy()
        want = oracle.pack_codes(oracle.quantize_codes(x, s, z, lo, lo + 3))
        _assert_same(got.reshape(N, K // 4), want, f"quantize+pack {N}x{K}")
    # an unaligned source pointer takes the byte path
    x = rng.normal(0, 1, size=(9, 52)).astype(np.float32)
    base = torch.zeros(9 * 52 + 1, dtype=torch.float32, device="cuda")
    base[1:].copy_(torch.from_numpy(x.reshape(-1)))
    got = dg.dg_quantize_pack_activations(base[1:], 9, 52, 2.0, 0.5, -2).cpu().numpy()
    _assert_same(got.reshape(9, 13), oracle.pack_codes(oracle.quantize_codes(x, 2.0, 0.5, -2, 1)), "unaligned quantize")


def test_quantiser_is_not_fused_on_the_gpu():
    """The multiply and the add of Eq. 1 are two binary32 roundings on both sides (see the pin of the same name in
    test_oracle_pins.py): a compiler that contracts them into an FMA turns this code 2 into a 1."""
    s, x, z = float(np.float32(1 + 2.0 ** -23)), np.float32(0.5 - 2.0 ** -23), 1.0
    for count in (4, 16, 64, 4096 + 16 + 4):                   # byte path, vector path, both
        xs = np.full((1, count), x, np.float32)
        got = dg.dg_quantize_pack_activations(torch.from_numpy(xs).cuda(), 1, count, s, z, 0).cpu().numpy()
        assert np.array_equal(got.reshape(1, -1), oracle.pack_codes(oracle.quantize_codes(xs, s, z, 0, 3)))
        assert int(got[0]) == 0b10101010
    # the same decision inside the fused layer: sums of exactly 1 (one product of 1, the rest 0), scale = x
    Cin, Cout = 32, 8
    Wc = np.zeros((Cout, 1, 1, Cin), np.uint8)
    Xc = np.zeros((1, 4, 4, Cin), np.uint8)
    Wc[..., 0] = 1
    Xc[..., 0] = 1
    lut = dg.dg_build_lut((0, 1, 2, 3), (0, 1, 2, 3))
    Wp = dg.dg_pack_weights(torch.from_numpy(Wc).cuda(), Cout, Cin)
    Xp = dg.dg_pack_activations(torch.from_numpy(Xc).cuda(), 16, Cin)
    scale = torch.full((Cout,), float(x), dtype=torch.float32, device="cuda")
    got = dg.dg_conv2d_lut_requant(lut, Wp, Xp, dg.conv_desc(1, 4, 4, Cin, Cout, 1, 1), scale, s, z, 0).cpu().numpy()
    assert np.all(got == 0b10101010)


def test_dequantize_equals_the_scale_epilogue():
    # int32 sums -> separate dequantise stage == oracle epilogue == the kernels' fused epilogue, bit for bit
    rng = np.random.default_rng(77)
    for rows, C in ((7, 5), (196, 64), (33, 130), (1000, 256)):
        acc = rng.integers(-(1 << 30), 1 << 30, size=(rows, C)).astype(np.int32)     # beyond 2^24: conversion rounds
        acc[0, : min(C, 4)] = [0, -1, (1 << 24) + 1, -(1 << 24) - 3][: min(C, 4)]
        scale = rng.uniform(0.01, 0.1, size=C).astype(np.float32)
        got = dg.dg_dequantize(torch.from_numpy(acc).cuda(), rows, C, torch.from_numpy(scale).cuda()).cpu().numpy()
        assert np.array_equal(got, oracle.scale_epilogue_nhwc(acc.reshape(1, 1, rows, C), scale).reshape(rows, C))
    c = wl.small_conv(2, 13, 11, 64, 70, 3, 3, (1, 1), (1, 1), seed=5, scale=True)
    case = GpuCase(c)
    y = case.run("auto")
    fused = case.run("auto", scale=True)
    sep = dg.dg_dequantize(y, 2 * 13 * 11, 70, case.scale)
    torch.cuda.synchronize()
    assert torch.equal(sep.reshape(fused.shape), fused)
    with pytest.raises(dg.DgError) as e:
        dg.dg_dequantize(y, 0, 70, case.scale)
    assert e.value.status == 2


@pytest.mark.parametrize("plan", ["auto", "split", "1", "2", "4", "7", "2k2", "4k4"])
def test_fused_layer_equals_convolution_then_quantise_pack(plan, monkeypatch):
    """dg_conv2d_lut_requant against the oracle's convolution -> scale epilogue -> Eq. 1 quantiser -> packing, byte for
    byte, on every plan of the one-hot kernels (dense and sparse instruction); and against the library's own two-call
    path."""
    if plan != "auto":
        monkeypatch.setenv("DG_ONEHOT_PLAN", plan)
    rng = np.random.default_rng(31)
    for table, kernel in (("signed_unsigned", "onehot_mfma"), ("extreme_i16", "onehot_mfma"), ("nonuniform_i8", "onehot_smfmac"),
                          ("extreme_i16", "onehot_smfmac")):
        lw, la, entry = LEVELS[table]
        if table == "extreme_i16" and kernel == "onehot_smfmac" and plan != "auto":
            continue                                   # (its two-plane form has one tile)
        if table == "extreme_i16" and "k" in plan:
            continue
        if kernel == "onehot_smfmac" and plan.startswith("7"):
            continue                                   # (the sparse-instruction form has no 64 x 224 tile)
        for (B, H, W, Cin, Cout, KH, KW, stride, pad) in [(2, 24, 24, 32, 68, 3, 3, (1, 1), (1, 1)),
                                                          (1, 30, 30, 128, 40, 3, 3, (2, 2), (1, 1)),
                                                          (3, 16, 16, 64, 36, 1, 1, (1, 1), (0, 0)),
                                                          (1, 9, 9, 64, 128, 3, 3, (1, 1), (1, 1))]:
            c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout, scale=True)
            case = GpuCase(c, levels=(lw, la), entry=entry)
            acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
            y = oracle.scale_epilogue_nhwc(acc, c.scale)
            # a quantiser that spreads the outputs over all four codes, with exact ties among them
            qs = np.float32(3.0 / max(1e-6, float(np.percentile(np.abs(y), 90))))
            for qz, lo in ((np.float32(0.5), 0), (np.float32(0.0), -2)):
                codes = oracle.quantize_codes(y, float(qs), float(qz), lo, lo + 3)
                want = oracle.pack_codes(codes.reshape(-1, Cout))
                got = dg.dg_conv2d_lut_requant(case.lut, case.Wp, case.Ap, case.desc, case.scale, float(qs), float(qz), lo,
                                               variant=kernel)
                torch.cuda.synchronize()
                _assert_same(got.cpu().numpy().reshape(-1, Cout // 4), want, f"fused layer {(B, H, W, Cin, Cout)} {table} {plan}")
                yf = case.run(kernel, scale=True)
                two_calls = dg.dg_quantize_pack_activations(yf, yf.numel() // Cout, Cout, float(qs), float(qz), lo)
                torch.cuda.synchronize()
                assert torch.equal(got, two_calls)
    # what it declines: other variants, Cout % 4 != 0, a small output buffer
    c = wl.small_conv(1, 8, 8, 32, 6, 3, 3, (1, 1), (1, 1), seed=3, scale=True)
    case = GpuCase(c)
    with pytest.raises(dg.DgError) as e:
        dg.dg_conv2d_lut_requant(case.lut, case.Wp, case.Ap, case.desc, case.scale, 1.0, 0.0, 0)
    assert e.value.status == 2
    c = wl.small_conv(1, 8, 8, 32, 8, 3, 3, (1, 1), (1, 1), seed=3, scale=True)
    case = GpuCase(c)
    with pytest.raises(dg.DgError) as e:
        dg.dg_conv2d_lut_requant(case.lut, case.Wp, case.Ap, case.desc, case.scale, 1.0, 0.0, 0, variant="perm")
    assert e.value.status == 5
    with pytest.raises(dg.DgError) as e:
        dg.dg_conv2d_lut_requant(case.lut, case.Wp, case.Ap, case.desc, case.scale, 1.0, 0.0, 0,
                                 out=torch.empty(10, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 4


def test_quantize_pack_feeds_the_convolution():
    # fp32 NHWC input -> quantise+pack -> table convolution, against oracle quantiser -> oracle convolution
    rng = np.random.default_rng(41)
    B, H, W, Cin, Cout = 2, 12, 12, 64, 32
    x = np.abs(rng.normal(0, 1.0, size=(B, H, W, Cin))).astype(np.float32)
    c = wl.small_conv(B, H, W, Cin, Cout, 3, 3, (1, 1), (1, 1), seed=42)
    codes = oracle.quantize_codes(x, 1.5, 0.0, 0, 3)
    want = oracle.conv2d(c.Wc, codes, c.levels_w, c.levels_a, pad=(1, 1))
    lut = dg.dg_build_lut(c.levels_w, c.levels_a)
    Wp = dg.dg_pack_weights(torch.from_numpy(c.Wc).cuda(), Cout, 9 * Cin)
    Xp = dg.dg_quantize_pack_activations(torch.from_numpy(x).cuda(), B * H * W, Cin, 1.5, 0.0, 0)
    y = dg.dg_conv2d_lut(lut, Wp, Xp, dg.conv_desc(B, H, W, Cin, Cout, 3, 3, (1, 1), (1, 1)))
    torch.cuda.synchronize()
    _assert_same(y.cpu().numpy(), want, "quantize -> conv")


WIDE = {
    3: ([-4, -3, -2, -1, 0, 1, 2, 3], [5, 1, 2, 3, 4, 7, 6, 9]),        # no zero activation level: padding must still add 0
    4: (list(range(-8, 8)), [0, 3, 1, 7, 2, 9, 4, 15, 5, 6, 8, 10, 11, 12, 13, 14]),
}


@pytest.mark.parametrize("plan", ["auto", "lds", "split", "1", "2", "4", "7", "sparse"])
@pytest.mark.parametrize("bits", [3, 4])
def test_wide_codes_gemm_and_conv(bits, plan, monkeypatch):
    """Sec. 3.3 / Table 2: 64- and 256-entry tables.  They run on the LDS kernel (every shape) and on the one-hot
    matrix-core kernels (Cin % 16 == 0), whose every plan is forced in turn -- 4-bit codes also in the
    sparse-instruction form; the 2-bit-only kernels decline."""
    if plan == "sparse" and bits != 4:
        pytest.skip("the sparse-instruction form exists for 2- and 4-bit codes")
    lw, la = WIDE[bits]
    nlev = 1 << bits
    rng = np.random.default_rng(50 + bits)
    lut = dg.dg_build_lut_bits(bits, lw, la, dg.DG_LUT_I8)
    variant = plan if plan in ("auto", "lds") else ("onehot_smfmac" if plan == "sparse" else "onehot_mfma")
    if variant == "onehot_mfma":
        monkeypatch.setenv("DG_ONEHOT_PLAN", plan)
    for M, N, K in ((5, 7, 6), (64, 196, 576), (33, 130, 40), (70, 300, 64), (40, 1000, 96), (130, 257, 1024)):
        Wc, Ac = wl.draw_codes(rng, (M, K), nlev=nlev), wl.draw_codes(rng, (N, K), nlev=nlev)
        Wp = dg.dg_pack_codes_bits(torch.from_numpy(Wc).cuda(), M, K, bits)
        Ap = dg.dg_pack_codes_bits(torch.from_numpy(Ac).cuda(), N, K, bits)
        _assert_same(Ap.cpu().numpy().reshape(N, K // 2), oracle.pack_codes(Ac, bits), f"{bits}-bit pack")
        name = dg.dg_gemm_kernel_name(lut, M, N, K, variant)
        if K % 16 != 0:
            assert name == ("lds" if variant in ("auto", "lds") else "unsupported")
        else:
            assert name.startswith({"lds": "lds", "onehot_smfmac": "onehot_smfmac4"}.get(variant, "onehot_mfma"))
        if name == "unsupported":
            continue
        got = dg.dg_gemm_lut(lut, Wp, Ap, M, N, K, variant=variant)
        torch.cuda.synchronize()
        want = oracle.gemm(Wc, Ac, lw, la)
        _assert_same(got.cpu().numpy(), want, f"{bits}-bit gemm {(M, N, K)} {plan}")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")         # column-major output
        dg.dg_gemm_lut(lut, Wp, Ap, M, N, K, out=out, variant=variant, strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"{bits}-bit gemm {(M, N, K)} {plan} column-major")
        with pytest.raises(dg.DgError) as e:
            dg.dg_gemm_lut(lut, Wp, Ap, M, N, K, variant="perm")
        assert e.value.status == 5
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in [(2, 9, 7, 16, 12, 3, 3, (2, 1), (1, 1)),
                                                      (2, 20, 20, 32, 70, 3, 3, (1, 1), (1, 1)),
                                                      (1, 17, 15, 64, 40, 5, 5, (1, 1), (2, 2)),
                                                      (3, 12, 12, 128, 33, 1, 1, (1, 1), (0, 0))]:
        Wc = wl.draw_codes(rng, (Cout, KH, KW, Cin), nlev=nlev)
        Xc = wl.draw_codes(rng, (B, H, W, Cin), nlev=nlev)
        Wp = dg.dg_pack_codes_bits(torch.from_numpy(Wc).cuda(), Cout, KH * KW * Cin, bits)
        Xp = dg.dg_pack_codes_bits(torch.from_numpy(Xc).cuda(), B * H * W, Cin, bits)
        y = dg.dg_conv2d_lut(lut, Wp, Xp, dg.conv_desc(B, H, W, Cin, Cout, KH, KW, stride, pad), variant=variant)
        torch.cuda.synchronize()
        _assert_same(y.cpu().numpy(), oracle.conv2d(Wc, Xc, lw, la, stride=stride, pad=pad),
                     f"{bits}-bit conv {(B, H, W, Cin, Cout)} {plan}")
        if Cout % 4 == 0 and variant != "lds":
            # the fused layer takes these tables too: wide codes in, the next layer's 2-bit codes out
            scale = torch.from_numpy(np.linspace(0.5, 1.5, Cout, dtype=np.float32)).cuda()
            acc = oracle.conv2d(Wc, Xc, lw, la, stride=stride, pad=pad)
            yf = oracle.scale_epilogue_nhwc(acc, scale.cpu().numpy())
            qs = float(np.float32(3.0 / max(1e-6, float(np.percentile(np.abs(yf), 90)))))
            want = oracle.pack_codes(oracle.quantize_codes(yf, qs, 0.5, 0, 3).reshape(-1, Cout))
            got = dg.dg_conv2d_lut_requant(lut, Wp, Xp, dg.conv_desc(B, H, W, Cin, Cout, KH, KW, stride, pad), scale, qs, 0.5, 0,
                                           variant=variant)
            torch.cuda.synchronize()
            _assert_same(got.cpu().numpy().reshape(-1, Cout // 4), want, f"{bits}-bit fused layer {(B, H, W, Cin, Cout)} {plan}")


@pytest.mark.parametrize("variant", VARIANTS)
def test_non_separable_table(variant):
    # any 16 integers are a valid table (the table stores results, Sec. 5.3); the matrix-core comparison declines
    rng = np.random.default_rng(60)
    for lo, hi, entry in ((-3, 4, dg.DG_LUT_I8), (-100, 100, dg.DG_LUT_I8), (-3000, 3000, dg.DG_LUT_I16)):
        table = rng.integers(lo, hi, size=16)
        lut = dg.dg_build_lut_entries(table, entry)
        g = wl.small_gemm(70, 130, 192, seed=61)
        Wp = dg.dg_pack_weights(torch.from_numpy(g.Wc).cuda(), 70, 192)
        Ap = dg.dg_pack_activations(torch.from_numpy(g.Ac).cuda(), 130, 192)
        try:
            got = dg.dg_gemm_lut(lut, Wp, Ap, 70, 130, 192, variant=variant)
        except dg.DgError as e:
            assert e.status == 5 and variant not in ("auto", "lds")
            continue
        assert variant != "mfma_i8"
        torch.cuda.synchronize()
        _assert_same(got.cpu().numpy(), oracle.gemm_table(g.Wc, g.Ac, table), f"table {lo}..{hi} {variant}")
        c = wl.small_conv(2, 13, 11, 64, 24, 3, 3, (1, 1), (1, 1), seed=62)
        Wp = dg.dg_pack_weights(torch.from_numpy(c.Wc).cuda(), 24, 576)
        Xp = dg.dg_pack_activations(torch.from_numpy(c.Ac).cuda(), 2 * 13 * 11, 64)
        try:
            y = dg.dg_conv2d_lut(lut, Wp, Xp, dg.conv_desc(2, 13, 11, 64, 24, 3, 3, (1, 1), (1, 1)), variant=variant)
        except dg.DgError as e:
            assert e.status == 5 and variant not in ("auto", "lds")     # e.g. the small-N kernel takes no 3x3 filter
            continue
        torch.cuda.synchronize()
        _assert_same(y.cpu().numpy(), oracle.conv2d_table(c.Wc, c.Ac, table, pad=(1, 1)), f"table conv {variant}")


def test_f32_table():
    # binary32 products of floating-point levels, summed in binary32 in ascending k: expected to match bit for bit
    lw = np.array([-0.731, -0.204, 0.118, 0.655], np.float32)
    la = np.array([0.0, 0.391, 0.874, 1.62], np.float32)
    lut = dg.dg_build_lut_f32(lw, la)
    table = oracle.build_lut_f32(lw, la)
    assert np.array_equal(np.array(lut.entries(), np.float32), table)
    g = wl.small_gemm(33, 57, 320, seed=63)
    Wp = dg.dg_pack_weights(torch.from_numpy(g.Wc).cuda(), 33, 320)
    Ap = dg.dg_pack_activations(torch.from_numpy(g.Ac).cuda(), 57, 320)
    got = dg.dg_gemm_lut(lut, Wp, Ap, 33, 57, 320)
    torch.cuda.synchronize()
    want = oracle.gemm_table_f32(g.Wc, g.Ac, table)
    assert got.dtype == torch.float32 and dg.dg_gemm_kernel_name(lut, 33, 57, 320) == "lds_f32"
    np.testing.assert_allclose(got.cpu().numpy(), want, rtol=1e-6, atol=0)
    assert np.array_equal(got.cpu().numpy(), want)
    c = wl.small_conv(2, 9, 8, 16, 10, 3, 3, (1, 2), (1, 1), seed=64, scale=True)
    Wp = dg.dg_pack_weights(torch.from_numpy(c.Wc).cuda(), 10, 144)
    Xp = dg.dg_pack_activations(torch.from_numpy(c.Ac).cuda(), 2 * 9 * 8, 16)
    desc = dg.conv_desc(2, 9, 8, 16, 10, 3, 3, (1, 2), (1, 1))
    y = dg.dg_conv2d_lut(lut, Wp, Xp, desc)
    ys = dg.dg_conv2d_lut(lut, Wp, Xp, desc, scale=torch.from_numpy(c.scale).cuda())
    torch.cuda.synchronize()
    want = oracle.conv2d_table_f32(c.Wc, c.Ac, table, stride=(1, 2), pad=(1, 1))
    assert np.array_equal(y.cpu().numpy(), want)
    assert np.array_equal(ys.cpu().numpy(), want * c.scale[None, None, None, :])
    with pytest.raises(dg.DgError) as e:
        dg.dg_conv2d_lut(lut, Wp, Xp, desc, variant="perm")
    assert e.value.status == 5


def test_graph_replays_equal_eager_launches():
    """bench.py replays its steps from a HIP graph: a captured step (pack, then convolution; the fused layer; and the one-call path) must
    give, on every replay and with other work between the replays, what the same calls give launched one by one -- on a
    small layer (split-K kernel, LDS sums zeroed inside the kernel) and on one large enough for the sparse-instruction
    kernel."""
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in [(1, 28, 28, 64, 64, 3, 3, (1, 1), (1, 1)),
                                                      (16, 56, 56, 64, 128, 1, 1, (1, 1), (0, 0))]:
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=B + H + Cout, scale=True)
        case = GpuCase(c)
        assert case.kernel_name().startswith("onehot_mfma_splitk" if B == 1 else "onehot_smfmac_")
        dev = case.Wp.device
        codes = torch.from_numpy(c.Ac).to(dev)
        want = oracle.scale_epilogue_nhwc(oracle.conv2d(c.Wc, c.Ac, c.levels_w, c.levels_a, stride=stride, pad=pad), c.scale)
        Xp = torch.empty_like(case.Ap)
        y = torch.empty(want.shape, dtype=torch.float32, device=dev)
        q = torch.empty(B * want.shape[1] * want.shape[2] * Cout // 4, dtype=torch.uint8, device=dev)
        y1, work = torch.empty_like(y), torch.empty_like(case.Ap)         # the one-call path (bench.py's step)

        def step():
            dg.dg_pack_activations(codes, B * H * W, Cin, out=Xp)
            dg.dg_conv2d_lut(case.lut, case.Wp, Xp, case.desc, out=y, scale=case.scale)
            dg.dg_conv2d_lut_requant(case.lut, case.Wp, Xp, case.desc, case.scale, 8.0, 0.5, 0, out=q)
            dg.dg_conv2d_lut_codes(case.lut, case.Wp, codes, case.desc, work=work, out=y1, scale=case.scale)

        step()
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), want)
        q_eager = q.clone()
        side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for replay in range(4):
            Xp.zero_(), y.fill_(-1.0), q.fill_(255), y1.fill_(-2.0), work.fill_(7)       # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy(), want), f"replay {replay} of {(B, H, W, Cin, Cout)}"
            assert torch.equal(q, q_eager), f"replay {replay}: fused layer"
            assert torch.equal(Xp, case.Ap), f"replay {replay}: packed activations"
            assert np.array_equal(y1.cpu().numpy(), want), f"replay {replay}: one-call path"


def test_four_bit_auto_takes_the_sparse_kernel_on_large_layers():
    """AUTO's choice for 4-bit tables from 512 tiles of 64 x 128 up is the sparse-instruction kernel: a GEMM and an NHWC
    convolution of that size against the oracle (the forced-variant tests above only reach it on small shapes)."""
    lw, la = WIDE[4]
    lut = dg.dg_build_lut_bits(4, lw, la, dg.DG_LUT_I8)
    rng = np.random.default_rng(77)
    M, N, K = 130, 32770, 272                               # ragged in M and N; 3 x 257 tiles; one-word chunks
    Wc, Ac = wl.draw_codes(rng, (M, K), nlev=16), wl.draw_codes(rng, (N, K), nlev=16)
    Wp = dg.dg_pack_codes_bits(torch.from_numpy(Wc).cuda(), M, K, 4)
    Ap = dg.dg_pack_codes_bits(torch.from_numpy(Ac).cuda(), N, K, 4)
    assert dg.dg_gemm_kernel_name(lut, M, N, K) == "onehot_smfmac4_64x128"
    got = dg.dg_gemm_lut(lut, Wp, Ap, M, N, K)
    torch.cuda.synchronize()
    _assert_same(got.cpu().numpy(), oracle.gemm(Wc, Ac, lw, la), "4-bit gemm, AUTO")
    B, H, W, Cin, Cout = 16, 56, 56, 32, 96
    Wc = wl.draw_codes(rng, (Cout, 3, 3, Cin), nlev=16)
    Xc = wl.draw_codes(rng, (B, H, W, Cin), nlev=16)
    Wp = dg.dg_pack_codes_bits(torch.from_numpy(Wc).cuda(), Cout, 9 * Cin, 4)
    Xp = dg.dg_pack_codes_bits(torch.from_numpy(Xc).cuda(), B * H * W, Cin, 4)
    desc = dg.conv_desc(B, H, W, Cin, Cout, 3, 3, (1, 1), (1, 1))
    assert dg.dg_conv_kernel_name(lut, desc) == "onehot_smfmac4_64x128"
    y = dg.dg_conv2d_lut(lut, Wp, Xp, desc)
    torch.cuda.synchronize()
    acc = oracle.conv2d(Wc, Xc, lw, la, stride=(1, 1), pad=(1, 1))
    _assert_same(y.cpu().numpy(), acc, "4-bit conv, AUTO")
    scale = torch.from_numpy(np.linspace(0.5, 1.5, Cout, dtype=np.float32)).cuda()
    yf = oracle.scale_epilogue_nhwc(acc, scale.cpu().numpy())
    qs = float(np.float32(3.0 / max(1e-6, float(np.percentile(np.abs(yf), 90)))))
    want = oracle.pack_codes(oracle.quantize_codes(yf, qs, 0.5, 0, 3).reshape(-1, Cout))
    got = dg.dg_conv2d_lut_requant(lut, Wp, Xp, desc, scale, qs, 0.5, 0)
    torch.cuda.synchronize()
    _assert_same(got.cpu().numpy().reshape(-1, Cout // 4), want, "4-bit fused layer, AUTO (sparse-instruction kernel)")


@pytest.mark.parametrize("waves", [0, 3, 7, 100000, -3])
@pytest.mark.parametrize("K", [64, 128, 256, 512])
def test_stationary_weight_kernel(K, waves, monkeypatch):
    """The sparse-instruction kernel with stationary weight operands (K = 64, 128, 256, and 512 on packed activations; no
    filter window), forced on
    shapes with ragged M and N: runs of one, of an even and of an odd number of pixel blocks per wavefront (`waves`: 0 =
    the default count, 3 and 7 = long runs, 100000 = one block per wavefront); GEMM with column-major output (run as it
    is) and row-major output (run transposed), 1x1 convolution -- also with strides, equal and unequal, on odd image
    sizes -- with int32, scaled fp32 and re-quantised packed output."""
    monkeypatch.setenv("DG_ONEHOT_PLAN", "ws")
    if waves:
        monkeypatch.setenv("DG_WS_WAVES", str(abs(waves)))
    if waves < 0:       # (the form that packs codes itself: waiting for its stores whenever it waits for staged codes)
        monkeypatch.setenv("DG_WS_COUNT_STORES", "0")
    lw, la, entry = LEVELS["nonuniform_i8"]
    for (M, N) in [(70, 1000), (64, 333), (33, 64), (130, 2049), (5, 31)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K)
        case = GpuCase(inp, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == "onehot_smfmac_ws_32xK"
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), want, f"ws gemm {(M, N, K)} row-major")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant="onehot_smfmac", strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"ws gemm {(M, N, K)} column-major")
    for (B, H, W, Cout, stride) in [(3, 9, 7, 36, (1, 1)), (1, 31, 33, 64, (1, 1)), (2, 16, 16, 100, (1, 1)),
                                    (3, 19, 18, 36, (2, 2)), (2, 31, 33, 72, (3, 2)), (1, 9, 40, 64, (1, 2))]:
        c = wl.small_conv(B, H, W, K, Cout, 1, 1, stride, (0, 0), seed=H + K + Cout, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == "onehot_smfmac_ws_32xK"
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), acc, f"ws conv {(B, H, W, K, Cout, stride)}")
        y = oracle.scale_epilogue_nhwc(acc, c.scale)
        got = case.run("onehot_smfmac", scale=True).cpu().numpy()
        np.testing.assert_allclose(got, y, rtol=1e-6, atol=0)
        assert np.array_equal(got, y)
        qs = np.float32(3.0 / max(1e-6, float(np.percentile(np.abs(y), 90))))
        codes = oracle.quantize_codes(y, float(qs), 0.5, 0, 3)
        q = dg.dg_conv2d_lut_requant(case.lut, case.Wp, case.Ap, case.desc, case.scale, float(qs), 0.5, 0, variant="onehot_smfmac")
        torch.cuda.synchronize()
        _assert_same(q.cpu().numpy().reshape(-1, Cout // 4), oracle.pack_codes(codes.reshape(-1, Cout)), f"ws fused layer {(B, H, W, K, Cout)}")
    # a filter window, padding or another K is not its case: the tiled sparse-instruction kernel takes over
    c = wl.small_conv(1, 8, 8, 64, 32, 3, 3, (1, 1), (1, 1), seed=1)
    assert GpuCase(c, levels=(lw, la), entry=entry).kernel_name("onehot_smfmac") != "onehot_smfmac_ws_32xK"
    if K == 512:        # (on codes one per byte: the packing kernel first)
        c = wl.small_conv(1, 31, 33, K, 64, 1, 1, (1, 1), (0, 0), seed=3)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert not dg.dg_conv_codes_kernel_name(case.lut, case.desc, "onehot_smfmac").startswith("codes_onehot_smfmac_ws")
        return
    # on codes one per byte it packs them itself (no work buffer needed): convolutions, and GEMMs whose output has the
    # weight rows' axis contiguous (the other layout runs transposed, with the packing kernel first)
    for (B, H, W, Cout) in [(3, 9, 7, 36), (1, 31, 33, 64), (2, 16, 16, 100), (1, 1, 5, 8)]:
        c = wl.small_conv(B, H, W, K, Cout, 1, 1, (1, 1), (0, 0), seed=H + K + Cout + 1, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert dg.dg_conv_codes_kernel_name(case.lut, case.desc, "onehot_smfmac") == "codes_onehot_smfmac_ws_32xK"
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la)
        # (garbage above bit 1 of every code byte: the packing drops it, as the packing kernel does)
        dirty = c.Ac | (np.random.default_rng(H + Cout).integers(0, 64, size=c.Ac.shape, dtype=np.uint8) << 2)
        Xc = torch.from_numpy(dirty).cuda()
        got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, variant="onehot_smfmac")
        torch.cuda.synchronize()
        _assert_same(got.cpu().numpy(), acc, f"ws conv on codes {(B, H, W, K, Cout)}")
        got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, scale=case.scale, variant="onehot_smfmac")
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.scale_epilogue_nhwc(acc, c.scale))
    for (M, N) in [(70, 1000), (33, 64), (130, 2049)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K + 1)
        case = GpuCase(inp, levels=(lw, la), entry=entry)
        Ac = torch.from_numpy(inp.Ac).cuda()
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, out=out, strides=(1, M), variant="onehot_smfmac")
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"ws gemm on codes {(M, N, K)} column-major")
        assert dg.dg_gemm_codes_kernel_name(case.lut, M, N, K, "onehot_smfmac") == "onehot_smfmac_ws_32xK"     # row-major
        got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Ac, M, N, K, work=torch.empty_like(case.Ap), variant="onehot_smfmac")
        torch.cuda.synchronize()
        _assert_same(got.cpu().numpy(), want, f"ws gemm on codes {(M, N, K)} row-major")


@pytest.mark.parametrize("plan,name", [("12", "onehot_smfmac_staged_32x64"), ("12k2", "onehot_smfmac_staged_32x64_k2"),
                                       ("12k4", "onehot_smfmac_staged_32x64_k4"), ("14", "onehot_smfmac_staged_32x128"),
                                       ("14k2", "onehot_smfmac_staged_32x128_k2"), ("14k4", "onehot_smfmac_staged_32x128_k4"),
                                       ("16", "onehot_smfmac_staged_32x192"), ("17", "onehot_smfmac_staged_32x224"),
                                       ("24", "onehot_smfmac_staged_64x128")])
def test_staged_sparse_kernel(plan, name, monkeypatch):
    """The tiled sparse-instruction kernel whose operands go through LDS in 32-byte runs (Cin % 128 == 0), every tile
    shape forced: convolutions with a padded 3x3 window (taps outside the image at every border), a stride, one, two and
    three runs per tap, a single run in all (K = 128: shared tiles then leave wavefronts without a share), ragged M and N
    (tiles partly outside, fewer columns than a tile), scaled fp32 and re-quantised packed output; GEMMs in both output
    layouts (the row-major one runs transposed)."""
    monkeypatch.setenv("DG_ONEHOT_PLAN", plan)
    lw, la, entry = LEVELS["nonuniform_i8"]
    convs = [(2, 9, 7, 128, 36, 3, 3, (1, 1), (1, 1)), (1, 13, 11, 256, 70, 3, 3, (2, 2), (1, 1)),
             (3, 6, 5, 384, 64, 1, 1, (1, 1), (0, 0)), (1, 5, 4, 128, 33, 1, 1, (1, 1), (0, 0)),
             (1, 20, 17, 128, 130, 3, 2, (1, 2), (1, 0)), (2, 15, 15, 256, 100, 5, 5, (1, 1), (2, 2)),
             (1, 29, 29, 128, 70, 3, 3, (1, 1), (1, 1))]
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in convs:
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == name
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), acc, f"staged conv {(B, H, W, Cin, Cout, KH, KW, stride, pad)}")
        y = oracle.scale_epilogue_nhwc(acc, c.scale)
        got = case.run("onehot_smfmac", scale=True).cpu().numpy()
        assert np.array_equal(got, y)
        if Cout % 4 == 0:
            qs = np.float32(3.0 / max(1e-6, float(np.percentile(np.abs(y), 90))))
            codes = oracle.quantize_codes(y, float(qs), 0.5, 0, 3)
            q = dg.dg_conv2d_lut_requant(case.lut, case.Wp, case.Ap, case.desc, case.scale, float(qs), 0.5, 0, variant="onehot_smfmac")
            torch.cuda.synchronize()
            _assert_same(q.cpu().numpy().reshape(-1, Cout // 4), oracle.pack_codes(codes.reshape(-1, Cout)),
                         f"staged fused layer {(B, H, W, Cin, Cout)}")
    for (M, N, K) in [(70, 1000, 128), (64, 333, 512), (200, 64, 1280), (33, 5, 256)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K)
        case = GpuCase(inp, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == name
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), want, f"staged gemm {(M, N, K)} row-major")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant="onehot_smfmac", strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"staged gemm {(M, N, K)} column-major")
    # channels that are not whole 16-byte chunks: the direct-load kernel of the same tile; whole chunks but not whole
    # 32-byte runs: the staged kernel's two narrow unshared tiles only (test_staged_kernel_half_runs)
    c = wl.small_conv(1, 8, 8, 32, 32, 3, 3, (1, 1), (1, 1), seed=1)
    assert "staged" not in GpuCase(c, levels=(lw, la), entry=entry).kernel_name("onehot_smfmac")
    c = wl.small_conv(1, 8, 8, 64, 32, 3, 3, (1, 1), (1, 1), seed=1)
    assert ("staged" in GpuCase(c, levels=(lw, la), entry=entry).kernel_name("onehot_smfmac")) == (plan in ("12", "14"))
    # seeded random geometries: filter, stride, padding, image, channels, batch
    rng = np.random.default_rng(77 + len(plan))
    for _ in range(12):
        KH, KW = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, KH)), int(rng.integers(0, KW))
        H, W = int(rng.integers(KH, 20)), int(rng.integers(KW, 20))
        Cin, Cout, B = int(rng.choice([128, 256, 384])), int(rng.integers(1, 140)), int(rng.integers(1, 4))
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, (sh, sw), (ph, pw), seed=int(rng.integers(1 << 30)))
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == name
        want = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=(sh, sw), pad=(ph, pw))
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), want,
                     f"staged conv B={B} {H}x{W} Cin={Cin} Cout={Cout} {KH}x{KW} s=({sh},{sw}) p=({ph},{pw}) plan {plan}")


@pytest.mark.parametrize("bias", ["0", "1"])
@pytest.mark.parametrize("plan,name", [("12", "onehot_smfmac_staged_32x64"), ("14", "onehot_smfmac_staged_32x128")])
def test_staged_kernel_half_runs(plan, name, bias, monkeypatch):
    """The staged kernel on layers whose filter taps are an odd number of 64-position chunks (Cin = 64, 192, 320): the
    two chunks of a 32-byte run may then lie in different taps, and the last run of K may be half a run.  Padded windows,
    strides, ragged M and N, one chunk in all (K = 64), with the table as it is and raised; scaled output; GEMMs in both
    output layouts."""
    monkeypatch.setenv("DG_ONEHOT_PLAN", plan)
    monkeypatch.setenv("DG_STAGED_BIAS", bias)
    lw, la, entry = LEVELS["nonuniform_i8"]
    convs = [(2, 9, 7, 64, 36, 3, 3, (1, 1), (1, 1)), (1, 13, 11, 192, 70, 3, 3, (2, 2), (1, 1)),
             (3, 6, 5, 320, 64, 1, 1, (1, 1), (0, 0)), (1, 5, 4, 64, 33, 1, 1, (1, 1), (0, 0)),
             (1, 20, 17, 64, 130, 3, 2, (1, 2), (1, 0)), (2, 15, 15, 64, 100, 5, 5, (1, 1), (2, 2)),
             (1, 29, 29, 64, 70, 3, 3, (1, 1), (1, 1)), (1, 12, 12, 192, 40, 2, 2, (1, 1), (1, 1))]
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in convs:
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == name
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), acc, f"staged conv, half runs {(B, H, W, Cin, Cout, KH, KW, stride, pad)}")
        got = case.run("onehot_smfmac", scale=True).cpu().numpy()
        assert np.array_equal(got, oracle.scale_epilogue_nhwc(acc, c.scale))
    for (M, N, K) in [(70, 1000, 64), (64, 333, 192), (200, 64, 1216), (33, 5, 320)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K)
        case = GpuCase(inp, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == name
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), want, f"staged gemm, half runs {(M, N, K)} row-major")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant="onehot_smfmac", strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"staged gemm, half runs {(M, N, K)} column-major")
    rng = np.random.default_rng(177 + len(plan))
    for _ in range(12):
        KH, KW = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, KH)), int(rng.integers(0, KW))
        H, W = int(rng.integers(KH, 20)), int(rng.integers(KW, 20))
        Cin, Cout, B = int(rng.choice([64, 192, 320])), int(rng.integers(1, 140)), int(rng.integers(1, 4))
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, (sh, sw), (ph, pw), seed=int(rng.integers(1 << 30)))
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == name
        want = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=(sh, sw), pad=(ph, pw))
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), want,
                     f"staged conv, half runs B={B} {H}x{W} Cin={Cin} Cout={Cout} {KH}x{KW} s=({sh},{sw}) p=({ph},{pw}) plan {plan}")


@pytest.mark.parametrize("bias", ["1", "0"])
@pytest.mark.parametrize("levels", ["signed_unsigned", "twos_complement", "nonuniform_i8", "wide_i8", "all_positive"])
@pytest.mark.parametrize("plan", ["14k4", "17", "24"])
def test_staged_kernel_raised_table(plan, levels, bias, monkeypatch):
    """The staged kernel multiplies with the table raised to 0 ... max - min and starts every sum at minus that raise
    times the positions of K the pixel sees: tables with negative, with only positive entries (lowered), one too wide to
    raise (127 and -128), the raise switched off; padded and strided windows where border pixels see fewer taps, ragged
    tiles, K shared between wavefronts (one of them starts the sums), GEMMs in both layouts."""
    monkeypatch.setenv("DG_ONEHOT_PLAN", plan)
    monkeypatch.setenv("DG_STAGED_BIAS", bias)
    lw, la, entry = LEVELS[levels]
    for (B, H, W, Cin, Cout, KH, KW, stride, pad) in [(2, 9, 7, 128, 36, 3, 3, (1, 1), (1, 1)), (1, 11, 13, 256, 70, 5, 4, (2, 1), (4, 3)),
                                                      (1, 6, 6, 128, 64, 7, 7, (1, 1), (3, 3))]:
        c = wl.small_conv(B, H, W, Cin, Cout, KH, KW, stride, pad, seed=H + Cin + Cout + 5, scale=True)
        case = GpuCase(c, levels=(lw, la), entry=entry)
        assert "staged" in case.kernel_name("onehot_smfmac")
        acc = oracle.conv2d(c.Wc, c.Ac, lw, la, stride=stride, pad=pad)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), acc, f"raised table {levels} conv {(B, H, W, Cin, Cout, KH, KW, stride, pad)}")
        assert np.array_equal(case.run("onehot_smfmac", scale=True).cpu().numpy(), oracle.scale_epilogue_nhwc(acc, c.scale))
    for (M, N, K) in [(70, 300, 384), (33, 5, 128)]:
        inp = wl.small_gemm(M, N, K, seed=M + N + K + 9)
        case = GpuCase(inp, levels=(lw, la), entry=entry)
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), want, f"raised table {levels} gemm {(M, N, K)} row-major")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant="onehot_smfmac", strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"raised table {levels} gemm {(M, N, K)} column-major")


@pytest.mark.parametrize("waves", [0, 1, 3, 8])
@pytest.mark.parametrize("K", [256, 1280, 4096, 8192])
def test_few_columns_sparse_kernel(K, waves, monkeypatch):
    """The few-columns kernel on the sparse instruction (weights as the index operand), forced on shapes with ragged M
    and 1 to 40 columns (up to three passes of 16), any split of K over the wavefronts; row-major and column-major
    output, int32 and scaled fp32."""
    monkeypatch.setenv("DG_ONEHOT_PLAN", "fewn")
    if waves:
        monkeypatch.setenv("DG_FEWN_WAVES", str(waves))
    lw, la, entry = LEVELS["nonuniform_i8"]
    for (M, N) in [(70, 1), (33, 2), (8, 5), (130, 16), (64, 17), (300, 40)]:
        inp = wl.make_inputs(wl.Workload(name="g", kind="gemm", M=M, N=N, K=K, scale=True, seed=M + N + K))
        case = GpuCase(inp, levels=(lw, la), entry=entry)
        assert case.kernel_name("onehot_smfmac") == "onehot_smfmac_fewn_16"
        want = oracle.gemm(inp.Wc, inp.Ac, lw, la)
        _assert_same(case.run("onehot_smfmac").cpu().numpy(), want, f"fewn gemm {(M, N, K)}")
        out = torch.full((N, M), -7, dtype=torch.int32, device="cuda")
        dg.dg_gemm_lut(case.lut, case.Wp, case.Ap, M, N, K, out=out, variant="onehot_smfmac", strides=(1, M))
        torch.cuda.synchronize()
        _assert_same(out.cpu().numpy(), want.T.copy(), f"fewn gemm {(M, N, K)} column-major")
        got = case.run("onehot_smfmac", scale=True).cpu().numpy()
        ref = oracle.scale_epilogue_rows(want, inp.scale)
        np.testing.assert_allclose(got, ref, rtol=1e-6, atol=0)
        assert np.array_equal(got, ref)
    # K must be whole super-steps of 256 positions
    inp = wl.small_gemm(64, 4, 320, seed=2)
    assert GpuCase(inp, levels=(lw, la), entry=entry).kernel_name("onehot_smfmac") != "onehot_smfmac_fewn_16"
