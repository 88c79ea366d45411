"""Helpers for the GPU parity tests: run one seeded workload through the C ABI (pack kernels, then the
GEMM / convolution kernel) and hand back numpy arrays.  Nothing here computes expected values."""
import numpy as np
import torch

from paper_2304_09049_amd import binding as dg


def entry_type(inp) -> int:
    return dg.DG_LUT_I16 if inp.workload.lut_entry == "i16" else dg.DG_LUT_I8


class GpuCase:
    """Device-resident packed operands of one workload."""

    def __init__(self, inp, levels=None, entry=None):
        w = inp.workload
        self.inp, self.w = inp, w
        lw, la = (inp.levels_w, inp.levels_a) if levels is None else levels
        self.levels = (np.asarray(lw), np.asarray(la))
        self.lut = dg.dg_build_lut(lw, la, entry_type(inp) if entry is None else entry)
        dev = torch.device("cuda:0")
        Wc = torch.from_numpy(inp.Wc).to(dev)
        Ac = torch.from_numpy(inp.Ac).to(dev)
        self.Wp = dg.dg_pack_weights(Wc, w.M, w.K)
        if w.kind == "conv":
            self.Ap = dg.dg_pack_activations(Ac, w.B * w.H * w.W, w.Cin)
            self.desc = dg.conv_desc(w.B, w.H, w.W, w.Cin, w.Cout, w.KH, w.KW, w.stride, w.pad)
        else:
            self.Ap = dg.dg_pack_activations(Ac, w.N, w.K)
            self.desc = None
        self.scale = torch.from_numpy(inp.scale).to(dev) if inp.scale is not None else None
        torch.cuda.synchronize()

    def run(self, variant="auto", scale=False, out=None):
        s = self.scale if scale else None
        if self.w.kind == "conv":
            y = dg.dg_conv2d_lut(self.lut, self.Wp, self.Ap, self.desc, out=out, scale=s, variant=variant)
        else:
            y = dg.dg_gemm_lut(self.lut, self.Wp, self.Ap, self.w.M, self.w.N, self.w.K, out=out, scale=s,
                               variant=variant)
        torch.cuda.synchronize()
        return y

    def kernel_name(self, variant="auto") -> str:
        if self.w.kind == "conv":
            return dg.dg_conv_kernel_name(self.lut, self.desc, variant)
        return dg.dg_gemm_kernel_name(self.lut, self.w.M, self.w.N, self.w.K, variant)


def run_or_unsupported(case: GpuCase, variant, scale=False):
    """Result as numpy, or None when the variant declares the shape unsupported (status 5)."""
    try:
        return case.run(variant, scale=scale).cpu().numpy()
    except dg.DgError as e:
        if e.status == 5 and variant != "auto" and variant != "lds":
            return None
        raise
