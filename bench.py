#!/usr/bin/env python3
"""Benchmark of the 2-bit lookup-table convolution on one MI355X.

One "step" is one pass of the run-time hot path over one batch of synthetic codes already resident in
HBM: pack the activation codes four per byte, then the table convolution / GEMM with its epilogue.  A
step goes through the one-call entry points dg_conv2d_lut_codes / dg_gemm_lut_codes, which on small layers (the
headline one) run a single kernel that packs the codes in registers as it loads them, and on the others the
packing kernel followed by the convolution / GEMM kernel.  The two-call time
of the same work is reported beside it.  The table and the packed weights are built once, before the timed
region (the paper packs weights offline, Sec. 5.2).  Steps are replayed from a HIP graph so that the host's
launch cost does not cap a microsecond-scale kernel.

Prints ONE JSON line.  `value` = 2*M*N*K / time per step, in GOPS, for the headline workload: the ResNet50-style
1x1 bottleneck convolution at batch 32 (56x56x256 -> 64, M=64 N=100352 K=256), the largest ResNet-shaped layer of
the benchmark set.  (The ResNet18-style 3x3 layer at batch 1 -- 0.23 GOP, a 3.5 us kernel of which 1.6 us is the
launch -- and the 64x196x576 GEMM are in `sweep` with their launch floors: their roofline fraction measures launch
latency, not the kernel.)

`roofline` (headline) and every `sweep` row price the kernel's EFFECTIVE work -- 2*M*N*K table operations (one
lookup and one add per product) and the algorithmic bytes -- against the ceiling that binds the shape:
t_roof = max(bytes / 8 TB/s, 2MNK / 5 POPS), frac = t_roof / t_kernel.  The int8 multiply-accumulates the matrix
cores actually perform (4 per product when selecting with one-hot operands, 2 on the sparse instruction) are
reported apart as `mfma_pipe_frac`: pipe utilisation, not a roofline fraction.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# published MI355X peaks used for the roofline fractions
HBM_PEAK_GBS = 8000.0
INT8_MFMA_PEAK_TOPS = 5000.0
# VALU issue ceiling of the permute kernel: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions/s;
# the inner loop spends one permute (4 products) and half a three-operand add per 4 products, so at most
# 4 / 1.5 products per lane-instruction, 2 ops per product.
VALU_LANE_INSTR_PER_S = 256 * 4 * 16 * 2.4e9
PERM_ALU_PEAK_TOPS = VALU_LANE_INSTR_PER_S * (4 / 1.5) * 2 / 1e12

# HBM bytes per launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by what the same
# counter reads for a plain copy of known size.  The figures and the commands that produced them live in
# profiles/hbm_traffic_counters.txt; its lines "traffic <workload> <kernel> <fetch KiB> <write KiB>" (already scaled)
# are read here.  A (workload, kernel) pair that was not profiled reports null.
def load_measured_traffic():
    table = {}
    path = os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")
    if os.path.exists(path):
        with open(path) as f:
            for line in f:
                t = line.split()
                if len(t) == 5 and t[0] == "traffic":
                    table[(t[1], t[2])] = (float(t[3]), float(t[4]))
    return table


MEASURED_TRAFFIC_KIB = load_measured_traffic()


def measured_traffic(w, name):
    kib = MEASURED_TRAFFIC_KIB.get((w.name, name))
    return None if kib is None else int(round((kib[0] + kib[1]) * 1024))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default=None, help="name in workloads.CONFIGS (default: the headline conv)")
    ap.add_argument("--variant", default="auto", help="auto | perm | lds | mfma_i8 | smalln | lut65k | onehot_mfma | onehot_smfmac")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from the host instead of a HIP graph")
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-workload kernel sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--table-values", action="store_true",
                    help="also time the workload's kernel (AUTO and the comparison) with other tables of the same shape: "
                         "the matrix pipe's power draw, and with it the clock, follows the operands' values")
    ap.add_argument("--layers", default=None, metavar="BATCHES",
                    help="instead of the benchmark line: every quantised convolution of ResNet-18, ResNet-50 and VGG-16 "
                         "(224 x 224 inputs; the first layer, on 3 input channels, is not one) at these batch sizes, e.g. "
                         "1,8,32 -- per layer the one-call step from unpacked codes and AUTO's kernel on packed codes "
                         "against the two one-hot forms and the decode-and-multiply comparison; one JSON line")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also run one plain device-to-device copy of this many MiB (a known-size dispatch "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled)")
    return ap.parse_args()


class Runner:
    """Device-resident operands of one workload and the calls that make up a step."""

    def __init__(self, w, variant="auto"):
        import torch
        from paper_2304_09049_amd import binding as dg
        from paper_2304_09049_amd import workloads as wl
        self.torch, self.dg, self.w, self.variant = torch, dg, w, variant
        self.inp = inp = wl.make_inputs(w)
        dev = torch.device("cuda:0")
        entry = dg.DG_LUT_I16 if w.lut_entry == "i16" else dg.DG_LUT_I8
        self.lut = dg.dg_build_lut(inp.levels_w, inp.levels_a, entry)
        self.Wp = dg.dg_pack_weights(torch.from_numpy(inp.Wc).to(dev), w.M, w.K)      # offline
        self.codes = torch.from_numpy(inp.Ac).to(dev)                                  # resident input
        self.scale = torch.from_numpy(inp.scale).to(dev) if inp.scale is not None else None
        if w.kind == "conv":
            self.rows, self.rowk = w.B * w.H * w.W, w.Cin
            self.desc = dg.conv_desc(w.B, w.H, w.W, w.Cin, w.Cout, w.KH, w.KW, w.stride, w.pad)
            OH = dg.dg_conv_out_dim(w.H, w.KH, w.stride[0], w.pad[0])
            OW = dg.dg_conv_out_dim(w.W, w.KW, w.stride[1], w.pad[1])
            shape = (w.B, OH, OW, w.Cout)
        else:
            self.rows, self.rowk = w.N, w.K
            self.desc = None
            shape = (w.M, w.N)
        self.Ap = torch.empty(dg.dg_packed_activation_bytes(self.rows, self.rowk), dtype=torch.uint8, device=dev)
        self.out = torch.empty(shape, dtype=torch.float32 if self.scale is not None else torch.int32, device=dev)
        self.pack()
        torch.cuda.synchronize()

    def pack(self):
        self.dg.dg_pack_activations(self.codes, self.rows, self.rowk, out=self.Ap)

    def kernel(self, variant=None):
        v = self.variant if variant is None else variant
        if self.desc is not None:
            self.dg.dg_conv2d_lut(self.lut, self.Wp, self.Ap, self.desc, out=self.out, scale=self.scale, variant=v)
        else:
            self.dg.dg_gemm_lut(self.lut, self.Wp, self.Ap, self.w.M, self.w.N, self.w.K, out=self.out,
                                scale=self.scale, variant=v)

    def step(self):
        """The whole hot path on the resident codes, through the one-call entry points, which pack inside the kernel on
        small problems and run the packing kernel first on the others."""
        if self.desc is not None:
            self.dg.dg_conv2d_lut_codes(self.lut, self.Wp, self.codes, self.desc, work=self.Ap, out=self.out,
                                        scale=self.scale, variant=self.variant)
        else:
            self.dg.dg_gemm_lut_codes(self.lut, self.Wp, self.codes, self.w.M, self.w.N, self.w.K, work=self.Ap,
                                      out=self.out, scale=self.scale, variant=self.variant)

    def two_calls(self):
        self.pack()
        self.kernel()

    def step_kernel_name(self):
        """The convolution / GEMM kernel of a step ("codes_..." when it does the packing itself)."""
        if self.desc is not None:
            return self.dg.dg_conv_codes_kernel_name(self.lut, self.desc, self.variant)
        return self.dg.dg_gemm_codes_kernel_name(self.lut, self.w.M, self.w.N, self.w.K, self.variant)

    def make_cold_weights(self, total_bytes=640 << 20):
        """Copies of the packed weights that together exceed the 256 MB last-level cache."""
        n = max(2, total_bytes // max(1, self.Wp.numel()))
        self.cold = [self.Wp.clone() for _ in range(n)]
        self.turn = 0

    def kernel_cold(self, variant=None):
        """The kernel on the next copy of the weights: every launch streams them from HBM."""
        self.turn += 1
        keep, self.Wp = self.Wp, self.cold[self.turn % len(self.cold)]
        try:
            self.kernel(variant)
        finally:
            self.Wp = keep

    def kernel_name(self, variant=None):
        v = self.variant if variant is None else variant
        if self.desc is not None:
            return self.dg.dg_conv_kernel_name(self.lut, self.desc, v)
        return self.dg.dg_gemm_kernel_name(self.lut, self.w.M, self.w.N, self.w.K, v)


def time_calls(torch, fn, count, use_graph, chunk=500):
    """Milliseconds per call of `fn` over exactly `count` calls, between two events on torch's current stream."""
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if use_graph:
        per = min(chunk, count)
        while count % per:
            per -= 1
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            fn()                                   # make sure nothing lazy happens during capture
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(per):
                    fn()
        torch.cuda.synchronize()
        graph.replay()                             # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        # Untimed replays for about 30 ms, not waited for: capturing left the GPU idle and its clocks take that long to
        # settle again (a short run measured 10 % slower without).  The timed replays are queued behind them, so the
        # timed region starts on a busy GPU and holds exactly `count` back-to-back calls.
        start.record()
        graph.replay()
        end.record()
        torch.cuda.synchronize()
        for _ in range(int(min(2000, max(1, 30.0 / max(start.elapsed_time(end), 1e-3))))):
            graph.replay()
        start.record()
        for _ in range(count // per):
            graph.replay()
        end.record()
    else:
        torch.cuda.synchronize()
        start.record()
        for _ in range(count):
            fn()
        end.record()
    torch.cuda.synchronize()
    return start.elapsed_time(end) / count


def time_steady(torch, fn, use_graph):
    """Milliseconds per call once the clocks have settled: size the run to about 30 ms of GPU work from a first rough
    timing, run it once untimed, then time it (the first passes after an idle spell run up to 15 % slower)."""
    for _ in range(3):
        fn()
    rough = max(time_calls(torch, fn, 5, False), 1e-3)
    reps = int(min(2000, max(10, 30.0 / rough)))
    graph = use_graph and reps >= 100
    if graph:
        reps -= reps % 100
    time_calls(torch, fn, reps, graph, chunk=100)
    runs = sorted(time_calls(torch, fn, reps, graph, chunk=100) for _ in range(5))
    return runs[2]                                 # median of 5


def single_launch_us(torch, fn):
    """Median over 21 single launches of the time between two events around one launch from the host (what one call
    costs in isolation: launch latency included, nothing overlapped)."""
    torch.cuda.synchronize()
    out = []
    for _ in range(21):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        out.append(a.elapsed_time(b) * 1e3)
    return round(sorted(out)[10], 2)


def mfma_ops_factor(name):
    """int8 multiply-accumulates the matrix cores perform per effective operation: the one-hot kernel contracts over 4K
    (one operand byte per table column); on the sparse instruction, which skips the half of them that its index says
    are zero, over 2K (priced against the DENSE peak all the same); the decode-and-multiply comparison kernel over K;
    table kernels on the VALU issue none."""
    if name.startswith("onehot_mfma") or name.startswith("codes_onehot_mfma"):
        return 4
    if name.startswith("onehot_smfmac") or name.startswith("smfmac_"):
        return 2
    if name.startswith("mfma_i8"):
        return 1
    return None


def algorithmic_bytes(w, name):
    """Bytes a launch of kernel `name` has to move: the workload's packed operands and output; a kernel that reads the
    activation codes one per byte reads four times the packed activations."""
    packed = (w.B * w.H * w.W * w.Cin // 4) if w.kind == "conv" else w.N * w.K // 4
    extra = 3 * packed if name.startswith("codes_") else 0
    return w.algorithmic_bytes + extra


def roofline_object(w, ms, name):
    """Effective work of one launch of duration `ms` against the binding ceiling of the shape: the HBM time of the
    algorithmic bytes or the int8 matrix-core time of 2MNK operations, whichever is longer."""
    alg = algorithmic_bytes(w, name)
    t = ms * 1e-3
    t_hbm = alg / (HBM_PEAK_GBS * 1e9)
    t_mfma = w.ops / (INT8_MFMA_PEAK_TOPS * 1e12)
    f = mfma_ops_factor(name)
    common = {"traffic": measured_traffic(w, name), "kernel": name, "us": round(ms * 1e3, 3),
              "algorithmic_bytes": alg, "ops_2mnk": w.ops,
              "hbm_frac": round(t_hbm / t, 5), "int8_mfma_frac_effective": round(t_mfma / t, 5),
              "valu_lookup_frac": round(w.ops / (PERM_ALU_PEAK_TOPS * 1e12) / t, 5),
              # int8 multiply-accumulates performed on the matrix cores (pipe utilisation, not a roofline fraction)
              "mfma_pipe_frac": None if f is None else round(f * t_mfma / t, 5)}
    if t_hbm >= t_mfma:
        ach = alg / t / 1e9
        return {"bound": "hbm", "achieved": round(ach, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 5), **common}
    ach = w.ops / t / 1e12
    return {"bound": "mfma", "achieved": round(ach, 3), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": round(ach / INT8_MFMA_PEAK_TOPS, 5), **common,
            "note": "effective table operations (2MNK) against the dense int8 peak; selecting with one-hot operands "
                    "performs 4 (dense instruction) or 2 (sparse instruction) multiply-accumulates per product, so "
                    "0.25 / 0.5 is the most a table kernel can reach on this ceiling"}


def kernel_report(w, ms, name):
    """One sweep row: the launch's effective rates and its fraction of each ceiling."""
    r = roofline_object(w, ms, name)
    r["gops"] = round(w.ops / (ms * 1e-3) / 1e9, 1)
    r["algorithmic_GBps"] = round(algorithmic_bytes(w, name) / (ms * 1e-3) / 1e9, 1)
    return r


def launch_floor_us(torch, w, name, use_graph):
    """Duration of an empty kernel with the grid of the split-K one-hot kernel (the shape is in its name): what the
    launch alone costs.  None for other kernels."""
    from paper_2304_09049_amd import binding as dg
    if name.startswith("codes_"):
        name = name[len("codes_"):]
    prefix = "onehot_mfma_splitk_s"
    if not name.startswith(prefix):
        return None
    blocks, threads = -(-w.M // 32) * -(-w.N // 32), 64 * int(name[len(prefix):])
    fn = lambda: dg.dg_launch_empty(blocks, threads)
    for _ in range(3):
        fn()
    return round(time_calls(torch, fn, 2000, use_graph) * 1e3, 3)


def stage_kernels(torch, w):
    """The HBM-bound stages either side of the table kernel, on one large activation tensor: packing of codes, the
    fused fp32 quantise + pack, and the dequantise of int32 sums.  Bytes are algorithmic (input read once + output
    written once)."""
    from paper_2304_09049_amd import binding as dg
    rows, k = w.B * w.H * w.W, w.Cin
    count = rows * k
    dev = torch.device("cuda:0")
    # successive calls walk through enough distinct inputs (> 512 MB) that none is served by the 256 MB last-level cache
    n_codes, n_x = 1 + (512 << 20) // count, 1 + (512 << 20) // (4 * count)
    codes = [torch.randint(0, 4, (count,), dtype=torch.uint8, device=dev) for _ in range(n_codes)]
    xs = [torch.rand(count, dtype=torch.float32, device=dev) * 3.0 for _ in range(n_x)]
    out = torch.empty(count // 4, dtype=torch.uint8, device=dev)
    turn = [0]

    def pack():
        turn[0] += 1
        dg.dg_pack_activations(codes[turn[0] % n_codes], rows, k, out=out)

    def quantize_pack():
        turn[0] += 1
        dg.dg_quantize_pack_activations(xs[turn[0] % n_x], rows, k, 1.0, 0.0, 0, out=out)

    accs = [torch.randint(-1000, 1000, (count,), dtype=torch.int32, device=dev) for _ in range(n_x)]
    scale_c = torch.rand(k, dtype=torch.float32, device=dev)
    deq = torch.empty(count, dtype=torch.float32, device=dev)

    def dequantize():
        turn[0] += 1
        dg.dg_dequantize(accs[turn[0] % n_x], rows, k, scale_c, out=deq)

    report = []
    for name, fn, nbytes in (("pack_vec16_unrolled_kernel", pack, count + count // 4),
                             ("quantize_pack_vec16_kernel", quantize_pack, 4 * count + count // 4),
                             ("dequantize_kernel", dequantize, 8 * count)):
        for _ in range(3):
            fn()
        ms = time_calls(torch, fn, 200, True, chunk=100)
        gbs = nbytes / (ms * 1e-3) / 1e9
        report.append({"kernel": name, "codes": count, "us": round(ms * 1e3, 3), "algorithmic_GBps": round(gbs, 1),
                       "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)})
    return report


def wide_code_kernels(torch, w, use_graph):
    """Tables beyond the 16 int8 entries of the headline path, on the shape of workload `w` (a convolution): 2-bit codes
    with int16 entries (two int8 planes), and the 3- and 4-bit tables of Sec. 3.3 / Table 2; each on the one-hot
    matrix-core kernel AUTO picks (two planes and 4-bit codes: a sparse-instruction form, so also the dense one) and on
    the plain LDS kernel.  `mfma_pipe_frac` counts the multiply-accumulates performed, `int8_mfma_frac_effective` 2MNK."""
    from paper_2304_09049_amd import binding as dg
    dev = torch.device("cuda:0")
    report = []
    for bits in (2, 3, 4):
        nlev = 1 << bits
        if bits == 2:
            # 2-bit codes with entries up to 16384: beyond int8, so the one-hot kernel selects from two int8 planes
            lut = dg.dg_build_lut_bits(2, [127, -128, 5, 3], [-128, 127, 1, 2], dg.DG_LUT_I16)
        else:
            lut = dg.dg_build_lut_bits(bits, list(range(-(nlev // 2), nlev // 2)), list(range(nlev)), dg.DG_LUT_I8)
        gen = torch.Generator(device=dev).manual_seed(bits)
        Wc = torch.randint(0, nlev, (w.Cout, w.KH, w.KW, w.Cin), dtype=torch.uint8, device=dev, generator=gen)
        Xc = torch.randint(0, nlev, (w.B, w.H, w.W, w.Cin), dtype=torch.uint8, device=dev, generator=gen)
        Wp = dg.dg_pack_codes_bits(Wc, w.Cout, w.KH * w.KW * w.Cin, bits)
        Xp = dg.dg_pack_codes_bits(Xc, w.B * w.H * w.W, w.Cin, bits)
        desc = dg.conv_desc(w.B, w.H, w.W, w.Cin, w.Cout, w.KH, w.KW, w.stride, w.pad)
        out = dg.dg_conv2d_lut(lut, Wp, Xp, desc)
        for variant in ("auto", "onehot_mfma", "lds"):
            name = dg.dg_conv_kernel_name(lut, desc, variant)
            if variant == "onehot_mfma" and name == dg.dg_conv_kernel_name(lut, desc, "auto"):
                continue                                 # (already timed as AUTO's choice)
            fn = lambda v=variant: dg.dg_conv2d_lut(lut, Wp, Xp, desc, out=out, variant=v)
            ms = time_steady(torch, fn, use_graph)
            tops = w.ops / (ms * 1e-3) / 1e12
            # multiply-accumulates performed per effective operation: 2^bits when selecting with the dense instruction
            # (8 for the two planes of 2-bit codes), half of that with the sparse one
            factor = None
            if name.startswith("onehot_mfma"):
                factor = 8 if bits == 2 else nlev
            elif name.startswith("onehot_smfmac"):
                factor = 4 if bits == 2 else nlev // 2
            report.append({"bits": bits, "workload_shape": w.name, "variant": variant, "kernel": name,
                           "us": round(ms * 1e3, 3), "gops": round(tops * 1e3, 1),
                           "int8_mfma_frac_effective": round(tops / INT8_MFMA_PEAK_TOPS, 4),
                           "mfma_pipe_frac": None if factor is None else round(factor * tops / INT8_MFMA_PEAK_TOPS, 4)})
    return report


def fused_layers(torch, names, use_graph):
    """A whole layer -- table convolution, scale, re-quantise, pack -- as one kernel (dg_conv2d_lut_requant) against
    the same work as two calls (dg_conv2d_lut with the scale epilogue, then dg_quantize_pack_activations)."""
    from paper_2304_09049_amd import binding as dg
    from paper_2304_09049_amd import workloads as wl
    report = []
    for name in names:
        w = wl.CONFIGS[name]
        r = Runner(w, "auto")
        dev = r.Wp.device
        scale = r.scale if r.scale is not None else torch.rand(w.Cout, dtype=torch.float32, device=dev) * 0.09 + 0.01
        yf = torch.empty(r.out.shape, dtype=torch.float32, device=dev)
        packed = torch.empty(dg.dg_packed_activation_bytes(w.N, w.Cout), dtype=torch.uint8, device=dev)

        def two_calls():
            dg.dg_conv2d_lut(r.lut, r.Wp, r.Ap, r.desc, out=yf, scale=scale)
            dg.dg_quantize_pack_activations(yf, w.N, w.Cout, 0.05, 0.5, 0, out=packed)

        def fused():
            dg.dg_conv2d_lut_requant(r.lut, r.Wp, r.Ap, r.desc, scale, 0.05, 0.5, 0, out=packed)

        t2, t1 = time_steady(torch, two_calls, use_graph), time_steady(torch, fused, use_graph)
        report.append({"workload": name, "kernel": r.kernel_name(), "conv_then_quantize_pack_us": round(t2 * 1e3, 3),
                       "fused_layer_us": round(t1 * 1e3, 3), "fused_gops": round(w.ops / (t1 * 1e-3) / 1e9, 1)})
    return report


def cpu_baseline(w):
    """The CPU oracle, as it stands, on the host cores: the full headline workload, repeated."""
    import oracle
    from paper_2304_09049_amd import workloads as wl
    inp = wl.make_inputs(w)

    def once():
        if w.kind == "conv":
            return oracle.conv2d(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a, stride=w.stride, pad=w.pad)
        return oracle.gemm(inp.Wc, inp.Ac, inp.levels_w, inp.levels_a)

    cores = oracle.max_threads()
    once()
    reps, t0 = 0, time.perf_counter()
    while reps < 3 or time.perf_counter() - t0 < 5.0:
        once()
        reps += 1
    dt_all = (time.perf_counter() - t0) / reps
    oracle.set_threads(1)
    t0 = time.perf_counter()
    once()
    dt_one = time.perf_counter() - t0
    oracle.set_threads(cores)
    return {"value": round(w.ops / dt_all / 1e9, 3), "unit": "GOPS", "cores": cores, "kind": "oracle",
            "sample": f"the full {w.name} workload (M={w.M} N={w.N} K={w.K}), {reps} passes on {cores} threads",
            "single_thread_gops": round(w.ops / dt_one / 1e9, 3)}


def table_values(torch, r, use_graph):
    """The runner's kernel on the same codes with other level vectors: same instructions, different operand values."""
    import numpy as np
    dg, w = r.dg, r.w
    entry = dg.DG_LUT_I16 if w.lut_entry == "i16" else dg.DG_LUT_I8
    tables = [("as specified", tuple(int(x) for x in r.inp.levels_w), tuple(int(x) for x in r.inp.levels_a)),
              ("all zero", (0, 0, 0, 0), (0, 1, 2, 3)), ("0 ... 9", (0, 1, 2, 3), (0, 1, 2, 3)),
              ("-6 ... 3", (-2, -1, 0, 1), (0, 1, 2, 3)), ("2 ... 49", (1, 3, 5, 7), (2, 4, 6, 7)),
              ("-64 ... 64", (-8, -3, 3, 7), (-8, -3, 3, 7))]
    keep, out = r.lut, []
    for what, lw, la in tables:
        r.lut = dg.dg_build_lut(np.array(lw, np.int8), np.array(la, np.int8), entry)
        out.append({"entries": what, "levels_w": list(lw), "levels_a": list(la), "kernel": r.kernel_name("auto"),
                    "us": round(time_steady(torch, lambda: r.kernel("auto"), use_graph) * 1e3, 2),
                    "mfma_i8_us": round(time_steady(torch, lambda: r.kernel("mfma_i8"), use_graph) * 1e3, 2)})
    r.lut = keep
    return out


def network_layers():
    """(H, Cin, Cout, filter, stride, count) of the quantised convolutions of three ImageNet networks, H the input's side.
    ResNet-50 with the stride on the 3x3 convolution of a stage's first block; shortcuts are 1x1 with stride 2."""
    resnet50 = [(56, 64, 64, 1, 1, 1), (56, 64, 64, 3, 1, 3), (56, 64, 256, 1, 1, 4), (56, 256, 64, 1, 1, 2),
                (56, 256, 128, 1, 1, 1), (56, 128, 128, 3, 2, 1), (28, 128, 128, 3, 1, 3), (28, 128, 512, 1, 1, 4),
                (28, 512, 128, 1, 1, 3), (56, 256, 512, 1, 2, 1),
                (28, 512, 256, 1, 1, 1), (28, 256, 256, 3, 2, 1), (14, 256, 256, 3, 1, 5), (14, 256, 1024, 1, 1, 6),
                (14, 1024, 256, 1, 1, 5), (28, 512, 1024, 1, 2, 1),
                (14, 1024, 512, 1, 1, 1), (14, 512, 512, 3, 2, 1), (7, 512, 512, 3, 1, 2), (7, 512, 2048, 1, 1, 3),
                (7, 2048, 512, 1, 1, 2), (14, 1024, 2048, 1, 2, 1)]
    resnet18 = [(56, 64, 64, 3, 1, 4), (56, 64, 128, 3, 2, 1), (28, 128, 128, 3, 1, 3), (56, 64, 128, 1, 2, 1),
                (28, 128, 256, 3, 2, 1), (14, 256, 256, 3, 1, 3), (28, 128, 256, 1, 2, 1),
                (14, 256, 512, 3, 2, 1), (7, 512, 512, 3, 1, 3), (14, 256, 512, 1, 2, 1)]
    vgg16 = [(224, 64, 64, 3, 1, 1), (112, 64, 128, 3, 1, 1), (112, 128, 128, 3, 1, 1), (56, 128, 256, 3, 1, 1),
             (56, 256, 256, 3, 1, 2), (28, 256, 512, 3, 1, 1), (28, 512, 512, 3, 1, 2), (14, 512, 512, 3, 1, 3)]
    return {"resnet18": resnet18, "resnet50": resnet50, "vgg16": vgg16}


def layers(torch, batches, use_graph):
    """Every layer of network_layers() at every batch size: the one-call step (AUTO, from unpacked codes), and the
    kernels on packed codes -- AUTO, the dense and the sparse one-hot form each in its own plan, the comparison.  Totals
    per network and batch weigh each layer by its count."""
    from paper_2304_09049_amd import workloads as wl
    rows, totals, seen = [], [], {}
    for net, shapes in network_layers().items():
        for B in batches:
            tot = {"network": net, "batch": B, "layers": 0, "gop": 0.0, "step_us": 0.0, "auto_us": 0.0, "onehot_mfma_us": 0.0,
                   "onehot_smfmac_us": 0.0, "mfma_i8_us": 0.0}
            for (H, Cin, Cout, k, s, count) in shapes:
                key = (B, H, Cin, Cout, k, s)
                if key not in seen:
                    if B * H * H * Cin > (1 << 30):
                        continue                                   # (not at this batch: the codes alone exceed 1 GiB)
                    w = wl._conv(f"{H}x{H}x{Cin}_{Cout}_{k}x{k}s{s}_b{B}", B, H, H, Cin, Cout, k, k, (s, s), (k // 2, k // 2))
                    r = Runner(w, "auto")
                    row = {"layer": w.name, "gop": round(w.ops / 1e9, 3), "step_kernel": r.step_kernel_name(),
                           "step_us": round(time_steady(torch, r.step, use_graph) * 1e3, 2), "kernel": r.kernel_name("auto")}
                    for v in ("auto", "onehot_mfma", "onehot_smfmac", "mfma_i8"):
                        row[v + "_us"] = round(time_steady(torch, lambda: r.kernel(v), use_graph) * 1e3, 2)
                    seen[key] = row
                    rows.append(row)
                    del r
                row = seen[key]
                tot["layers"] += count
                tot["gop"] += count * row["gop"]
                for f in ("step_us", "auto_us", "onehot_mfma_us", "onehot_smfmac_us", "mfma_i8_us"):
                    tot[f] += count * row[f]
            for f in tot:
                if isinstance(tot[f], float):
                    tot[f] = round(tot[f], 2)
            tot["step_effective_tops"] = round(tot["gop"] / tot["step_us"] * 1e3, 1) if tot["step_us"] else None
            totals.append(tot)
    return {"layers": rows, "totals": totals}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this path has no multi-GPU leg (it would shard N with no "
              "collective); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2304_09049_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    use_graph = not args.no_graph
    if args.calibrate_copy > 0:
        src = torch.ones(args.calibrate_copy << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)             # an elementwise kernel: reads and writes exactly that many bytes
        torch.cuda.synchronize()
        del src, dst
    if args.layers:
        out = layers(torch, [int(b) for b in args.layers.split(",")], use_graph)
        out.update({"what": "quantised convolutions of three networks, per layer and in total (us)", "data": "synthetic",
                    "launch": "hip graph replay" if use_graph else "host launches"})
        print(json.dumps(out))
        return
    w = wl.CONFIGS[args.workload or wl.HEADLINE]
    r = Runner(w, args.variant)

    for _ in range(args.warmup):
        r.step()
    torch.cuda.synchronize()
    ms_step = time_calls(torch, r.step, args.steps, use_graph)
    ms_kernel = time_calls(torch, r.kernel, args.steps, use_graph)       # the convolution / GEMM kernel on packed input
    ms_pack = time_calls(torch, r.pack, args.steps, use_graph)
    ms_two = time_calls(torch, r.two_calls, args.steps, use_graph)
    name, step_name = r.kernel_name(), r.step_kernel_name()
    fused = step_name.startswith("codes_")        # the step is ONE kernel, which packs the codes as it loads them
    dom_name, ms_dom = (step_name, ms_step) if fused else (name, ms_kernel)

    line = {
        "metric": "effective GOPS (2*M*N*K/s), 2-bit LUT conv",
        "value": round(w.ops / (ms_step * 1e-3) / 1e9, 1),
        "unit": "GOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32",
        "dtype_note": "int32 accumulation of int8 table entries selected by 2-bit codes" +
                      ("; one fp32 multiply per output in the scale epilogue" if w.scale else ""),
        "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "variant": args.variant, "kernel": dom_name,
                   "step": ("dg_conv2d_lut_codes" if w.kind == "conv" else "dg_gemm_lut_codes") +
                           (": unpacked codes in, one kernel that packs them as it loads them" if fused else
                            ": packing kernel + " + ("convolution" if w.kind == "conv" else "GEMM") + " kernel"),
                   "launch": "hip graph replay" if use_graph else "host launches"},
        # the same work as two calls, and its parts, for comparison
        "two_call_step_us": round(ms_two * 1e3, 3),
        "kernel_only": kernel_report(w, ms_kernel, name),
        "pack_activations_us": round(ms_pack * 1e3, 3),
        "roofline": roofline_object(w, ms_dom, dom_name),
        "empty_launch_same_grid_us": launch_floor_us(torch, w, dom_name, use_graph),
        "paper_context": "up to 1.74x over QNNPACK INT8 on an Intel i7-9700K (speedup ratios only; no absolute figure)",
    }
    if w.act_dist != "uniform":
        # Sec. 5.3: a table kernel's latency does not depend on the codes -- the same shape with uniform codes
        import dataclasses
        ru = Runner(dataclasses.replace(w, act_dist="uniform", name=w.name + "_uniform_codes"), args.variant)
        ms_uniform = time_calls(torch, ru.kernel, args.steps, use_graph)
        line["code_distribution_check"] = {"codes_as_specified": w.act_dist, "kernel_us": round(ms_kernel * 1e3, 3),
                                           "kernel_us_uniform_codes": round(ms_uniform * 1e3, 3),
                                           "ratio": round(ms_uniform / ms_kernel, 4)}
        del ru

    if not args.no_sweep:
        sweep = []
        for wname, ww in wl.CONFIGS.items():
            rr = r if ww is w else Runner(ww, "auto")
            for variant in ("auto", "onehot_mfma", "onehot_smfmac", "perm", "mfma_i8", "lut65k", "lds"):
                if variant in ("lds", "lut65k") and ww.ops > 1e11:
                    continue
                try:
                    kname = rr.kernel_name(variant)
                    if kname == "unsupported":
                        continue
                    if variant != "auto" and kname == rr.kernel_name("auto"):
                        continue                     # (already timed as AUTO's choice)
                    fn = lambda v=variant, q=rr: q.kernel(v)
                    ms = time_steady(torch, fn, use_graph)
                    rep = kernel_report(ww, ms, kname)
                    rep.update({"workload": wname, "variant": variant})
                    if variant == "auto":
                        # the whole step on this shape (unpacked codes in, through the one-call entry point) beside its
                        # convolution / GEMM kernel alone
                        rep["step_kernel"] = rr.step_kernel_name()
                        rep["step_us"] = round(time_steady(torch, rr.step, use_graph) * 1e3, 3)
                    if ww.ops < 1e9:
                        # roofline time far below the launch overhead: also what one isolated launch costs
                        rep["single_launch_us"] = single_launch_us(torch, fn)
                    if variant == "auto" and ww.kind == "gemm" and ww.N <= 16 and ww.M * ww.K // 4 >= (8 << 20):
                        # weight-streaming shapes: also with the weights NOT resident in the last-level cache
                        rr.make_cold_weights()
                        cold = lambda q=rr: q.kernel_cold("auto")
                        ms_cold = time_steady(torch, cold, use_graph)
                        rep["us_weights_from_hbm"] = round(ms_cold * 1e3, 3)
                        rep["frac_hbm_weights_from_hbm"] = round(ww.algorithmic_bytes / (ms_cold * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                        rr.cold = None
                    sweep.append(rep)
                except Exception as e:                      # report, never hide
                    sweep.append({"workload": wname, "variant": variant, "error": str(e)})
            del rr
        line["sweep"] = sweep
        line["stage_kernels"] = stage_kernels(torch, wl.CONFIGS["resnet50_conv1x1_b32"])
        line["wide_codes"] = wide_code_kernels(torch, wl.CONFIGS["vgg16_conv3x3_b16"], use_graph)
        line["fused_layers"] = fused_layers(torch, ["resnet18_conv3x3_b1", "resnet50_conv1x1_b32", "vgg16_conv3x3_b16"],
                                            use_graph)

    if args.table_values:
        line["table_values"] = table_values(torch, r, use_graph)
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
