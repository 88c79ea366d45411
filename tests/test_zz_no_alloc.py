"""The entry point that allocates nothing (dg_conv2d_lut_codes_static: packed activations staged in the library's static
device buffer) against dg_conv2d_lut_codes with a caller's work buffer, through the C ABI: two calls in a row, the
second on a smaller input, each bit-exact (int32) / equal (fp32 epilogue: the same kernels run on the same bytes)."""
import numpy as np
import pytest
import torch

from paper_2304_09049_amd import binding as dg
from paper_2304_09049_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _case(B, H, W, Cin, Cout, seed, scale):
    c = wl.small_conv(B, H, W, Cin, Cout, 3, 3, (1, 1), (1, 1), seed=seed, scale=scale)
    w = c.workload
    dev = torch.device("cuda:0")
    lut = dg.dg_build_lut(c.levels_w, c.levels_a)
    Wp = dg.dg_pack_weights(torch.from_numpy(c.Wc).to(dev), w.M, w.K)
    Xc = torch.from_numpy(c.Ac).to(dev)
    desc = dg.conv_desc(w.B, w.H, w.W, w.Cin, w.Cout, w.KH, w.KW, w.stride, w.pad)
    sc = torch.from_numpy(c.scale).to(dev) if scale else None
    return lut, Wp, Xc, desc, sc, w


def test_static_staging_matches_work_buffer_two_calls():
    # the first layer is one AUTO runs as two kernels (packing kernel into the staging buffer, then the convolution);
    # the second, smaller one is forced onto that path by naming a variant that never fuses the packing
    runs = [(_case(8, 28, 28, 96, 256, 11, False), "auto"), (_case(2, 14, 14, 96, 64, 12, True), "onehot_smfmac"),
            (_case(1, 9, 7, 32, 40, 13, False), "perm")]
    assert not dg.dg_conv_codes_kernel_name(runs[0][0][0], runs[0][0][3], "auto").startswith("codes_")
    for (lut, Wp, Xc, desc, sc, w), variant in runs:
        need = dg.dg_packed_activation_bytes(w.B * w.H * w.W, w.Cin)
        assert need <= dg.dg_static_work_bytes()
        dtype = torch.float32 if sc is not None else torch.int32
        # 3x3 filter, stride 1, pad 1: the output is as large as the input
        want = torch.empty((w.B, w.H, w.W, w.Cout), dtype=dtype, device=Xc.device)
        got = torch.full_like(want, 77)
        work = torch.empty(need, dtype=torch.uint8, device=Xc.device)
        dg.dg_conv2d_lut_codes(lut, Wp, Xc, desc, work=work, out=want, scale=sc, variant=variant)
        dg.dg_conv2d_lut_codes_static(lut, Wp, Xc, desc, out=got, scale=sc, variant=variant)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want.cpu().numpy()), (variant, w)


def test_static_staging_rejects_oversize():
    lut, Wp, Xc, desc, sc, w = _case(1, 8, 8, 32, 32, 14, False)
    big = dg.conv_desc(64, 112, 112, 64, 32, 3, 3, (1, 1), (1, 1))      # 12.8 MB of packed activations
    out = torch.empty(4, dtype=torch.int32, device=Xc.device)
    with pytest.raises(dg.DgError) as err:
        dg.dg_conv2d_lut_codes_static(lut, Wp, Xc, big, out=out)
    assert err.value.status == 4          # DG_ERR_BUFFER, before anything is launched
    torch.cuda.synchronize()
