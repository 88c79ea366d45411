"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (variant "auto"),
plus every other variant that accepts the shape.  Where the oracle finishes in seconds the whole output
is compared; otherwise a seeded sample of outputs (borders included) is computed one by one by the oracle."""
import numpy as np
import pytest

import oracle
from paper_2304_09049_amd import workloads as wl
from gpu_helpers import GpuCase, run_or_unsupported

pytestmark = pytest.mark.gpu

VARIANTS = ["auto", "perm", "lds", "mfma_i8", "smalln", "lut65k", "onehot_mfma", "onehot_smfmac"]
# every output compared, except on the 8192-cube GEMM (550 G multiply-adds for the oracle): there a seeded sample of
# more than 1 % of the 67 M outputs, with the first and last rows and columns (the last tiles of either axis) added
FULL = ["gemm_64x196x576", "resnet18_conv3x3_b1", "resnet50_conv1x1_b32", "vgg16_conv3x3_b16", "gemm_8192x1x8192_i16",
        "gemm_8192x16x8192_i16", "gemm_8192x256x8192_i16"]
SAMPLED = ["gemm_8192x8192x8192_i16"]
SAMPLE_FRACTION = 0.0105


def _border_heavy_positions(w, rng, count):
    """Flat NHWC output indices: a uniform sample plus every corner / some edge pixels of a few images."""
    total = w.N * w.M
    pos = [rng.integers(0, total, size=count)]
    if w.kind == "gemm":
        # output [M][N]: a sample of the first and last two rows and columns, and the four corner 40 x 40 blocks whole
        for m in (0, 1, w.M - 2, w.M - 1):
            pos.append(m * w.N + rng.integers(0, w.N, size=512))
        for n in (0, 1, w.N - 2, w.N - 1):
            pos.append(rng.integers(0, w.M, size=512) * w.N + n)
        edge = np.arange(40)
        for ms in (edge, w.M - 1 - edge):
            for ns in (edge, w.N - 1 - edge):
                pos.append((ms[:, None] * w.N + ns[None, :]).reshape(-1))
    if w.kind == "conv":
        OH = (w.H + 2 * w.pad[0] - w.KH) // w.stride[0] + 1
        OW = (w.W + 2 * w.pad[1] - w.KW) // w.stride[1] + 1
        for b in (0, w.B - 1):
            for oh in (0, 1, OH - 2, OH - 1):
                for ow in (0, 1, OW - 2, OW - 1):
                    px = (b * OH + oh) * OW + ow
                    pos.append(px * w.M + rng.integers(0, w.M, size=8))
    return np.unique(np.concatenate(pos))


def _one_call(case, inp):
    """The step bench.py times: dg_conv2d_lut_codes / dg_gemm_lut_codes on the unpacked codes (AUTO), with a work buffer
    for the problems whose packing is not fused into the kernel."""
    import torch
    from paper_2304_09049_amd import binding as dg
    Xc = torch.from_numpy(inp.Ac).cuda()
    w = inp.workload
    if w.kind == "conv":
        got = dg.dg_conv2d_lut_codes(case.lut, case.Wp, Xc, case.desc, work=torch.empty_like(case.Ap))
    else:
        got = dg.dg_gemm_lut_codes(case.lut, case.Wp, Xc, w.M, w.N, w.K, work=torch.empty_like(case.Ap))
    torch.cuda.synchronize()
    return got.cpu().numpy()


@pytest.mark.parametrize("name", FULL)
def test_full_output(name):
    w = wl.CONFIGS[name]
    inp = wl.make_inputs(w)
    case = GpuCase(inp)
    if w.kind == "conv":
        want = oracle.conv2d(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a, stride=w.stride, pad=w.pad)
    else:
        want = oracle.gemm(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a)
    ran = []
    for variant in VARIANTS:
        got = run_or_unsupported(case, variant)
        if got is None:
            continue
        ran.append(variant)
        assert np.array_equal(got, want), f"{name} {variant}: {np.count_nonzero(got != want)} outputs differ"
    assert "auto" in ran and "lds" in ran
    assert np.array_equal(_one_call(case, inp), want), f"{name}: packing + convolution / GEMM as one call"
    if w.scale:
        got = case.run("auto", scale=True).cpu().numpy()
        ref = oracle.scale_epilogue_nhwc(want, inp.scale)
        np.testing.assert_allclose(got, ref, rtol=1e-6, atol=0)


@pytest.mark.parametrize("name", SAMPLED)
def test_sampled_output(name):
    w = wl.CONFIGS[name]
    inp = wl.make_inputs(w)
    case = GpuCase(inp)
    rng = np.random.default_rng(123)
    count = int(np.ceil(SAMPLE_FRACTION * w.M * w.N))      # (8192-cube: 704 644 outputs, 5.8 G multiply-adds for the oracle)
    pos = _border_heavy_positions(w, rng, count)
    assert len(pos) >= 0.01 * w.M * w.N
    if w.kind == "conv":
        want = oracle.conv2d_sampled(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a, pos, stride=w.stride, pad=w.pad)
    else:
        ms, ns = pos // w.N, pos % w.N            # GEMM output is [M][N]
        want = oracle.gemm_sampled(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a, ms, ns)
    ran = []
    for variant in VARIANTS:
        if variant in ("lds", "lut65k") and w.ops > 2e11:
            continue                               # the plain kernels would take too long at this size
        got = run_or_unsupported(case, variant)
        if got is None:
            continue
        ran.append(variant)
        flat = got.reshape(-1)[pos]
        assert np.array_equal(flat, want), f"{name} {variant}: {np.count_nonzero(flat != want)} sampled outputs differ"
    assert "auto" in ran
    assert np.array_equal(_one_call(case, inp).reshape(-1)[pos], want), f"{name}: packing + convolution / GEMM as one call"


@pytest.mark.parametrize("name", ["vgg16_conv3x3_b16", "gemm_8192x8192x8192_i16"])
def test_sampled_output_two_plane_table(name):
    """The same full-size shapes under a table with entries beyond int8 (levels up to +-127, no zero activation
    level): AUTO's sparse-instruction two-plane kernel and the dense-instruction one, against sampled oracle outputs."""
    from paper_2304_09049_amd import binding as dg
    w = wl.CONFIGS[name]
    inp = wl.make_inputs(w)
    lw, la = (127, -128, 5, 3), (-128, 127, 1, 2)
    case = GpuCase(inp, levels=(lw, la), entry=dg.DG_LUT_I16)
    assert case.kernel_name("auto") == "onehot_smfmac_2p_32x128"
    assert case.kernel_name("onehot_mfma").startswith("onehot_mfma_2p_")
    rng = np.random.default_rng(321)
    pos = _border_heavy_positions(w, rng, int(min(200000, 3e9 // w.K)))
    if w.kind == "conv":
        want = oracle.conv2d_sampled(inp.Wc, inp.Ac, lw, la, pos, stride=w.stride, pad=w.pad)
    else:
        want = oracle.gemm_sampled(inp.Wc, inp.Ac, lw, la, pos // w.N, pos % w.N)
    for variant in ("auto", "onehot_mfma"):
        flat = case.run(variant).cpu().numpy().reshape(-1)[pos]
        assert np.array_equal(flat, want), f"{name} {variant}: {np.count_nonzero(flat != want)} sampled outputs differ"


NETWORK_LAYERS = [
    # (B, H, Cin, Cout, filter, stride), AUTO's kernel on packed codes, the one-call step's kernel
    ((32, 28, 320, 320, 3, 1), "onehot_smfmac_staged_32x128", "onehot_smfmac_staged_32x128"),       # taps of 2.5 runs
    ((32, 56, 256, 256, 3, 1), "onehot_smfmac_staged_32x224", "onehot_smfmac_staged_32x224"),
    ((32, 56, 256, 512, 1, 2), "onehot_smfmac_ws_32xK", "onehot_smfmac_ws_32xK"),                   # strided; the step packs the pixels read
    ((32, 28, 512, 512, 1, 1), "onehot_smfmac_ws_32xK", "onehot_smfmac_ws_32xK"),                   # K = 512
    ((8, 14, 1024, 256, 1, 1), "onehot_smfmac_staged_32x64_k4", "codes_onehot_smfmac_64x32_k4"),    # the tiled kernel packs
    ((1, 56, 256, 64, 1, 1), "onehot_mfma_splitk_s4", "codes_onehot_mfma_splitk_s4"),               # 64-position chunks
    ((8, 7, 512, 512, 3, 1), "onehot_mfma_splitk_s12", "onehot_mfma_splitk_s12"),
]


@pytest.mark.parametrize("shape,kernel,step_kernel", NETWORK_LAYERS)
def test_sampled_output_network_layers(shape, kernel, step_kernel):
    """Full-size layers of the networks bench.py --layers times, one per kernel and rule that the small parity cases
    reach only through forced plans: AUTO's kernel on packed codes and the one-call step on unpacked codes, against
    sampled oracle outputs (borders included)."""
    from paper_2304_09049_amd import binding as dg
    B, H, Cin, Cout, k, s = shape
    w = wl._conv("layer", B, H, H, Cin, Cout, k, k, (s, s), (k // 2, k // 2))
    inp = wl.make_inputs(w)
    case = GpuCase(inp)
    assert case.kernel_name("auto") == kernel
    assert dg.dg_conv_codes_kernel_name(case.lut, case.desc, "auto") == step_kernel
    rng = np.random.default_rng(B + H + Cin + Cout)
    pos = _border_heavy_positions(w, rng, int(min(60000, 2e8 // w.K)))
    want = oracle.conv2d_sampled(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a, pos, stride=w.stride, pad=w.pad)
    got = case.run("auto").cpu().numpy().reshape(-1)[pos]
    assert np.array_equal(got, want), f"{shape} {kernel}: {np.count_nonzero(got != want)} sampled outputs differ"
    got = _one_call(case, inp).reshape(-1)[pos]
    assert np.array_equal(got, want), f"{shape} {step_kernel}: {np.count_nonzero(got != want)} sampled outputs differ (one call)"
