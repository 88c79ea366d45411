"""ctypes binding over the C ABI of ``libdeepgemm_hip.so`` (declared in ``include/deepgemm_hip.h``).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  torch is
used for device memory and streams, nothing else.  There is no CPU fallback: if the library has
not been built, loading fails with an explicit error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdeepgemm_hip.so")

DG_OK = 0
STATUS_NAMES = ("DG_OK", "DG_ERR_NULL", "DG_ERR_SHAPE", "DG_ERR_RANGE", "DG_ERR_BUFFER",
                "DG_ERR_UNSUPPORTED", "DG_ERR_HIP")
DG_LUT_I8, DG_LUT_I16, DG_LUT_F32 = 0, 1, 2
DG_KERNEL_AUTO, DG_KERNEL_PERM, DG_KERNEL_LDS, DG_KERNEL_MFMA_I8, DG_KERNEL_SMALLN, DG_KERNEL_LUT65K = 0, 1, 2, 3, 4, 5
DG_KERNEL_ONEHOT_MFMA = 6
DG_KERNEL_ONEHOT_SMFMAC = 7
KERNELS = {"auto": DG_KERNEL_AUTO, "perm": DG_KERNEL_PERM, "lds": DG_KERNEL_LDS,
           "mfma_i8": DG_KERNEL_MFMA_I8, "smalln": DG_KERNEL_SMALLN, "lut65k": DG_KERNEL_LUT65K,
           "onehot_mfma": DG_KERNEL_ONEHOT_MFMA, "onehot_smfmac": DG_KERNEL_ONEHOT_SMFMAC}

# every symbol include/deepgemm_hip.h declares
EXPORTS = (
    "dg_status_string", "dg_last_error", "dg_build_lut", "dg_build_lut_bits", "dg_lut_bits", "dg_lut_entries",
    "dg_lut_entries_all", "dg_lut_destroy", "dg_build_lut_entries", "dg_build_lut_f32", "dg_lut_entries_f32",
    "dg_packed_activation_bytes", "dg_packed_weight_bytes", "dg_packed_bytes_bits", "dg_pack_weights",
    "dg_pack_activations", "dg_pack_codes_bits", "dg_quantize_pack_activations",
    "dg_gemm_lut", "dg_conv_out_dim", "dg_conv2d_lut", "dg_gemm_kernel_name", "dg_conv_kernel_name",
    "dg_conv2d_lut_codes", "dg_conv_codes_kernel_name", "dg_gemm_lut_codes", "dg_gemm_codes_kernel_name",
    "dg_launch_empty", "dg_dequantize", "dg_conv2d_lut_requant",
    "dg_static_work_bytes", "dg_conv2d_lut_codes_static",
)


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "H", "W", "Cin", "Cout", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w")]


class DgError(RuntimeError):
    def __init__(self, status: int, detail: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else f"status {status}"
        super().__init__(f"{name}: {detail}")


_lib = None


def lib() -> ctypes.CDLL:
    """Load the library (once).  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2304_09049_amd.build` "
                          "(hipcc, gfx950).  This package has no CPU fallback.")
    L = ctypes.CDLL(LIB_PATH)
    c_i64, c_vp, c_sz, c_int = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    L.dg_status_string.argtypes, L.dg_status_string.restype = [c_int], ctypes.c_char_p
    L.dg_last_error.argtypes, L.dg_last_error.restype = [], ctypes.c_char_p
    L.dg_build_lut.argtypes, L.dg_build_lut.restype = [c_vp, c_vp, c_int, ctypes.POINTER(c_vp)], c_int
    L.dg_lut_entries.argtypes, L.dg_lut_entries.restype = [c_vp, c_vp], c_int
    L.dg_build_lut_entries.argtypes, L.dg_build_lut_entries.restype = [c_vp, c_int, ctypes.POINTER(c_vp)], c_int
    L.dg_build_lut_f32.argtypes, L.dg_build_lut_f32.restype = [c_vp, c_vp, ctypes.POINTER(c_vp)], c_int
    L.dg_lut_entries_f32.argtypes, L.dg_lut_entries_f32.restype = [c_vp, c_vp], c_int
    L.dg_build_lut_bits.argtypes = [ctypes.c_int32, c_vp, c_vp, c_int, ctypes.POINTER(c_vp)]
    L.dg_build_lut_bits.restype = c_int
    L.dg_lut_bits.argtypes, L.dg_lut_bits.restype = [c_vp], ctypes.c_int32
    L.dg_lut_entries_all.argtypes, L.dg_lut_entries_all.restype = [c_vp, c_vp, ctypes.c_int32], c_int
    L.dg_packed_bytes_bits.argtypes, L.dg_packed_bytes_bits.restype = [c_i64, c_i64, ctypes.c_int32], c_sz
    L.dg_pack_codes_bits.argtypes = [c_vp, c_i64, c_i64, ctypes.c_int32, c_vp, c_sz, c_vp]
    L.dg_pack_codes_bits.restype = c_int
    L.dg_lut_destroy.argtypes, L.dg_lut_destroy.restype = [c_vp], None
    L.dg_packed_activation_bytes.argtypes, L.dg_packed_activation_bytes.restype = [c_i64, c_i64], c_sz
    L.dg_packed_weight_bytes.argtypes, L.dg_packed_weight_bytes.restype = [c_i64, c_i64], c_sz
    for f in (L.dg_pack_weights, L.dg_pack_activations):
        f.argtypes, f.restype = [c_vp, c_i64, c_i64, c_vp, c_sz, c_vp], c_int
    L.dg_quantize_pack_activations.argtypes = [c_vp, c_i64, c_i64, ctypes.c_float, ctypes.c_float, ctypes.c_int32,
                                               c_vp, c_sz, c_vp]
    L.dg_quantize_pack_activations.restype = c_int
    L.dg_gemm_lut.argtypes = [c_vp, c_vp, c_vp, c_i64, c_i64, c_i64, c_vp, c_i64, c_i64, c_vp, c_vp, c_int, c_vp]
    L.dg_gemm_lut.restype = c_int
    L.dg_conv_out_dim.argtypes, L.dg_conv_out_dim.restype = [c_i64] * 4, c_i64
    L.dg_conv2d_lut.argtypes = [c_vp, c_vp, c_vp, ctypes.POINTER(ConvDesc), c_vp, c_vp, c_vp, c_int, c_vp]
    L.dg_conv2d_lut.restype = c_int
    L.dg_gemm_kernel_name.argtypes, L.dg_gemm_kernel_name.restype = [c_vp, c_i64, c_i64, c_i64, c_int], ctypes.c_char_p
    L.dg_conv_kernel_name.argtypes = [c_vp, ctypes.POINTER(ConvDesc), c_int]
    L.dg_conv_kernel_name.restype = ctypes.c_char_p
    L.dg_conv2d_lut_codes.argtypes = [c_vp, c_vp, c_vp, ctypes.POINTER(ConvDesc), c_vp, c_sz, c_vp, c_vp, c_vp, c_int, c_vp]
    L.dg_conv2d_lut_codes.restype = c_int
    L.dg_static_work_bytes.argtypes, L.dg_static_work_bytes.restype = [], c_sz
    L.dg_conv2d_lut_codes_static.argtypes = [c_vp, c_vp, c_vp, ctypes.POINTER(ConvDesc), c_vp, c_vp, c_vp, c_int, c_vp]
    L.dg_conv2d_lut_codes_static.restype = c_int
    L.dg_gemm_lut_codes.argtypes = [c_vp, c_vp, c_vp, c_i64, c_i64, c_i64, c_vp, c_sz, c_vp, c_i64, c_i64, c_vp, c_vp, c_int, c_vp]
    L.dg_gemm_lut_codes.restype = c_int
    L.dg_gemm_codes_kernel_name.argtypes = [c_vp, c_i64, c_i64, c_i64, c_int]
    L.dg_gemm_codes_kernel_name.restype = ctypes.c_char_p
    L.dg_conv_codes_kernel_name.argtypes = [c_vp, ctypes.POINTER(ConvDesc), c_int]
    L.dg_conv_codes_kernel_name.restype = ctypes.c_char_p
    L.dg_launch_empty.argtypes, L.dg_launch_empty.restype = [c_i64, c_int, c_vp], c_int
    L.dg_dequantize.argtypes, L.dg_dequantize.restype = [c_vp, c_i64, c_i64, c_vp, c_vp, c_vp], c_int
    L.dg_conv2d_lut_requant.argtypes = [c_vp, c_vp, c_vp, ctypes.POINTER(ConvDesc), c_vp, ctypes.c_float, ctypes.c_float,
                                        ctypes.c_int32, c_vp, ctypes.c_size_t, c_int, c_vp]
    L.dg_conv2d_lut_requant.restype = c_int
    _lib = L
    return L


def _check(status: int) -> None:
    if status != DG_OK:
        raise DgError(status, lib().dg_last_error().decode())


def _kernel(variant) -> int:
    return KERNELS[variant] if isinstance(variant, str) else int(variant)


def _stream_ptr(stream) -> ctypes.c_void_p:
    """hipStream_t of a torch stream (default: torch's current stream)."""
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev_ptr(t, dtype=None, name="tensor") -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


class Lut:
    """Owner of a ``dg_lut`` built by ``dg_build_lut``."""

    def __init__(self, levels_w: Sequence[int], levels_a: Sequence[int], entry: int = DG_LUT_I8, bits: int = 2,
                 entries: Optional[Sequence[int]] = None):
        self._h = None
        self.bits = bits
        self.is_f32 = entry == DG_LUT_F32
        handle = ctypes.c_void_p(0)
        if entries is not None:                       # a table given as such (any 16 integers)
            arr = (ctypes.c_int16 * 16)(*[int(v) for v in entries])
            _check(lib().dg_build_lut_entries(arr, int(entry), ctypes.byref(handle)))
            self._h = handle
            return
        if self.is_f32:                               # binary32 products of floating-point levels
            lwf = (ctypes.c_float * 4)(*[float(v) for v in levels_w])
            laf = (ctypes.c_float * 4)(*[float(v) for v in levels_a])
            _check(lib().dg_build_lut_f32(lwf, laf, ctypes.byref(handle)))
            self._h = handle
            return
        nlev = 1 << bits
        if len(levels_w) != nlev or len(levels_a) != nlev:
            raise ValueError(f"{bits}-bit codes need {nlev} levels per side")
        lw = (ctypes.c_int8 * nlev)(*[int(v) for v in levels_w])
        la = (ctypes.c_int8 * nlev)(*[int(v) for v in levels_a])
        if bits == 2:
            _check(lib().dg_build_lut(lw, la, int(entry), ctypes.byref(handle)))
        else:
            _check(lib().dg_build_lut_bits(bits, lw, la, int(entry), ctypes.byref(handle)))
        self._h = handle

    @property
    def handle(self) -> ctypes.c_void_p:
        return self._h

    def entries(self):
        if self.is_f32:
            outf = (ctypes.c_float * 16)()
            _check(lib().dg_lut_entries_f32(self._h, outf))
            return list(outf)
        count = 1 << (2 * self.bits)
        out = (ctypes.c_int16 * count)()
        if self.bits == 2:
            _check(lib().dg_lut_entries(self._h, out))
        else:
            _check(lib().dg_lut_entries_all(self._h, out, count))
        return list(out)

    def __del__(self):
        if getattr(self, "_h", None) is not None and _lib is not None:
            _lib.dg_lut_destroy(self._h)
            self._h = None


def dg_build_lut(levels_w, levels_a, entry: int = DG_LUT_I8) -> Lut:
    return Lut(levels_w, levels_a, entry)


def dg_build_lut_entries(entries, entry: int = DG_LUT_I16) -> Lut:
    return Lut((), (), entry, entries=entries)


def dg_build_lut_f32(levels_w, levels_a) -> Lut:
    return Lut(levels_w, levels_a, DG_LUT_F32)


def dg_build_lut_bits(bits: int, levels_w, levels_a, entry: int = DG_LUT_I8) -> Lut:
    return Lut(levels_w, levels_a, entry, bits=bits)


def dg_packed_bytes_bits(rows: int, K: int, bits: int) -> int:
    return int(lib().dg_packed_bytes_bits(rows, K, bits))


def dg_pack_codes_bits(codes, rows: int, K: int, bits: int, out=None, stream=None):
    """codes: uint8 device tensor with rows*K elements of `bits`-bit codes -> packed uint8 tensor (weights or activations)."""
    import torch
    if out is None:
        out = torch.empty(dg_packed_bytes_bits(rows, K, bits), dtype=torch.uint8, device=codes.device)
    _check(lib().dg_pack_codes_bits(_dev_ptr(codes, torch.uint8, "codes"), rows, K, bits,
                                    _dev_ptr(out, torch.uint8, "packed"), out.numel(), _stream_ptr(stream)))
    return out


def dg_packed_activation_bytes(rows: int, K: int) -> int:
    return int(lib().dg_packed_activation_bytes(rows, K))


def dg_packed_weight_bytes(M: int, K: int) -> int:
    return int(lib().dg_packed_weight_bytes(M, K))


def dg_conv_out_dim(size: int, k: int, stride: int, pad: int) -> int:
    return int(lib().dg_conv_out_dim(size, k, stride, pad))


def _pack(fn, size_fn, codes, rows: int, K: int, out, stream):
    import torch
    if out is None:
        out = torch.empty(size_fn(rows, K), dtype=torch.uint8, device=codes.device)
    _check(fn(_dev_ptr(codes, torch.uint8, "codes"), rows, K, _dev_ptr(out, torch.uint8, "packed"),
              out.numel(), _stream_ptr(stream)))
    return out


def dg_pack_weights(codes, M: int, K: int, out=None, stream=None):
    """codes: uint8 device tensor with M*K elements ([M][K], or [Cout][KH][KW][Cin]) -> packed uint8 tensor."""
    return _pack(lib().dg_pack_weights, dg_packed_weight_bytes, codes, M, K, out, stream)


def dg_pack_activations(codes, N: int, K: int, out=None, stream=None):
    """codes: uint8 device tensor with N*K elements ([N][K], or NHWC with N = B*H*W, K = C) -> packed uint8 tensor."""
    return _pack(lib().dg_pack_activations, dg_packed_activation_bytes, codes, N, K, out, stream)


def dg_quantize_pack_activations(x, N: int, K: int, scale: float, zero_point: float, lo: int, out=None, stream=None):
    """x: float32 device tensor with N*K elements -> packed 2-bit codes of clip(rint(scale*x + zero_point), lo, lo+3) - lo."""
    import torch
    if out is None:
        out = torch.empty(dg_packed_activation_bytes(N, K), dtype=torch.uint8, device=x.device)
    _check(lib().dg_quantize_pack_activations(_dev_ptr(x, torch.float32, "x"), N, K, scale, zero_point, lo,
                                              _dev_ptr(out, torch.uint8, "packed"), out.numel(), _stream_ptr(stream)))
    return out


def dg_gemm_lut(lut: Lut, Wp, Ap, M: int, N: int, K: int, out=None, scale=None, variant="auto",
                stream=None, strides: Optional[Sequence[int]] = None):
    """C[m][n] = sum_k LUT[4*Wc[m][k] + Ac[n][k]].  Returns int32 [M][N], or float32 when `scale` is given."""
    import torch
    as_float = scale is not None or lut.is_f32
    dtype = torch.float32 if as_float else torch.int32
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=Wp.device)
    scm, scn = (N, 1) if strides is None else strides
    c_int = _dev_ptr(out, torch.int32, "out") if not as_float else ctypes.c_void_p(0)
    c_f32 = _dev_ptr(out, torch.float32, "out") if as_float else ctypes.c_void_p(0)
    _check(lib().dg_gemm_lut(lut.handle, _dev_ptr(Wp, torch.uint8, "Wp"), _dev_ptr(Ap, torch.uint8, "Ap"),
                             M, N, K, c_int, scm, scn, _dev_ptr(scale, torch.float32, "scale"), c_f32,
                             _kernel(variant), _stream_ptr(stream)))
    return out


def dg_gemm_lut_codes(lut: Lut, Wp, Ac, M: int, N: int, K: int, work=None, out=None, scale=None, variant="auto",
                      stream=None, strides: Optional[Sequence[int]] = None):
    """Packing stage + GEMM as one call, from codes one per byte (`Ac`: uint8 [N][K]).  `work` is the packed-activation
    buffer the library uses when it does not fuse the packing into the kernel (may be None)."""
    import torch
    as_float = scale is not None or lut.is_f32
    dtype = torch.float32 if as_float else torch.int32
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=Wp.device)
    scm, scn = (N, 1) if strides is None else strides
    c_int = _dev_ptr(out, torch.int32, "out") if not as_float else ctypes.c_void_p(0)
    c_f32 = _dev_ptr(out, torch.float32, "out") if as_float else ctypes.c_void_p(0)
    _check(lib().dg_gemm_lut_codes(lut.handle, _dev_ptr(Wp, torch.uint8, "Wp"), _dev_ptr(Ac, torch.uint8, "Ac"), M, N, K,
                                   _dev_ptr(work, torch.uint8, "work"), 0 if work is None else work.numel(), c_int,
                                   scm, scn, _dev_ptr(scale, torch.float32, "scale"), c_f32, _kernel(variant),
                                   _stream_ptr(stream)))
    return out


def dg_gemm_codes_kernel_name(lut: Lut, M: int, N: int, K: int, variant="auto") -> str:
    return lib().dg_gemm_codes_kernel_name(lut.handle, M, N, K, _kernel(variant)).decode()


def conv_desc(B, H, W, Cin, Cout, KH, KW, stride=(1, 1), pad=(0, 0)) -> ConvDesc:
    return ConvDesc(B, H, W, Cin, Cout, KH, KW, stride[0], stride[1], pad[0], pad[1])


def dg_conv2d_lut(lut: Lut, Wp, Xp, desc: ConvDesc, out=None, scale=None, variant="auto", stream=None):
    """NHWC convolution by table lookup.  Returns [B][OH][OW][Cout], int32 or float32 (when `scale` is given)."""
    import torch
    OH = dg_conv_out_dim(desc.H, desc.KH, desc.stride_h, desc.pad_h)
    OW = dg_conv_out_dim(desc.W, desc.KW, desc.stride_w, desc.pad_w)
    as_float = scale is not None or lut.is_f32
    dtype = torch.float32 if as_float else torch.int32
    if out is None:
        out = torch.empty((desc.B, max(OH, 0), max(OW, 0), desc.Cout), dtype=dtype, device=Wp.device)
    y_int = _dev_ptr(out, torch.int32, "out") if not as_float else ctypes.c_void_p(0)
    y_f32 = _dev_ptr(out, torch.float32, "out") if as_float else ctypes.c_void_p(0)
    _check(lib().dg_conv2d_lut(lut.handle, _dev_ptr(Wp, torch.uint8, "Wp"), _dev_ptr(Xp, torch.uint8, "Xp"),
                               ctypes.byref(desc), y_int, _dev_ptr(scale, torch.float32, "scale"), y_f32,
                               _kernel(variant), _stream_ptr(stream)))
    return out


def dg_conv2d_lut_codes(lut: Lut, Wp, Xc, desc: ConvDesc, work=None, out=None, scale=None, variant="auto", stream=None):
    """Packing stage + NHWC convolution as one call, from codes one per byte (`Xc`: uint8 [B][H][W][Cin]).  `work` is
    the packed-activation buffer the library uses when it does not fuse the packing into the kernel (may be None)."""
    import torch
    OH = dg_conv_out_dim(desc.H, desc.KH, desc.stride_h, desc.pad_h)
    OW = dg_conv_out_dim(desc.W, desc.KW, desc.stride_w, desc.pad_w)
    as_float = scale is not None or lut.is_f32
    dtype = torch.float32 if as_float else torch.int32
    if out is None:
        out = torch.empty((desc.B, max(OH, 0), max(OW, 0), desc.Cout), dtype=dtype, device=Wp.device)
    y_int = _dev_ptr(out, torch.int32, "out") if not as_float else ctypes.c_void_p(0)
    y_f32 = _dev_ptr(out, torch.float32, "out") if as_float else ctypes.c_void_p(0)
    work_bytes = 0 if work is None else work.numel()
    _check(lib().dg_conv2d_lut_codes(lut.handle, _dev_ptr(Wp, torch.uint8, "Wp"), _dev_ptr(Xc, torch.uint8, "Xc"),
                                     ctypes.byref(desc), _dev_ptr(work, torch.uint8, "work"), work_bytes, y_int,
                                     _dev_ptr(scale, torch.float32, "scale"), y_f32, _kernel(variant), _stream_ptr(stream)))
    return out


def dg_static_work_bytes() -> int:
    return int(lib().dg_static_work_bytes())


def dg_conv2d_lut_codes_static(lut: Lut, Wp, Xc, desc: ConvDesc, out, scale=None, variant="auto", stream=None):
    """dg_conv2d_lut_codes with the library's own staging buffer; `out` is required (the call allocates nothing)."""
    import torch
    as_float = scale is not None or lut.is_f32
    y_int = _dev_ptr(out, torch.int32, "out") if not as_float else ctypes.c_void_p(0)
    y_f32 = _dev_ptr(out, torch.float32, "out") if as_float else ctypes.c_void_p(0)
    _check(lib().dg_conv2d_lut_codes_static(lut.handle, _dev_ptr(Wp, torch.uint8, "Wp"), _dev_ptr(Xc, torch.uint8, "Xc"),
                                            ctypes.byref(desc), y_int, _dev_ptr(scale, torch.float32, "scale"), y_f32,
                                            _kernel(variant), _stream_ptr(stream)))
    return out


def dg_conv_codes_kernel_name(lut: Lut, desc: ConvDesc, variant="auto") -> str:
    return lib().dg_conv_codes_kernel_name(lut.handle, ctypes.byref(desc), _kernel(variant)).decode()


def dg_gemm_kernel_name(lut: Lut, M: int, N: int, K: int, variant="auto") -> str:
    return lib().dg_gemm_kernel_name(lut.handle, M, N, K, _kernel(variant)).decode()


def dg_conv_kernel_name(lut: Lut, desc: ConvDesc, variant="auto") -> str:
    return lib().dg_conv_kernel_name(lut.handle, ctypes.byref(desc), _kernel(variant)).decode()


def dg_launch_empty(blocks: int, threads: int, stream=None) -> None:
    """A launch that does nothing: the cost of a grid of that shape (measurement aid)."""
    _check(lib().dg_launch_empty(blocks, threads, _stream_ptr(stream)))


def dg_dequantize(acc, rows: int, C: int, scale, out=None, stream=None):
    """acc: int32 device tensor [rows][C]; scale: float32 [C] -> float32 [rows][C] = float(acc) * scale[c]."""
    import torch
    if out is None:
        out = torch.empty(acc.shape, dtype=torch.float32, device=acc.device)
    _check(lib().dg_dequantize(_dev_ptr(acc, torch.int32, "acc"), rows, C, _dev_ptr(scale, torch.float32, "scale"),
                               _dev_ptr(out, torch.float32, "out"), _stream_ptr(stream)))
    return out


def dg_conv2d_lut_requant(lut: Lut, Wp, Xp, desc: ConvDesc, scale, q_scale: float, q_zero: float, lo: int, out=None,
                          variant="auto", stream=None):
    """One fused layer: table convolution, per-channel scale, re-quantisation and packing -> packed uint8 [B*OH*OW][Cout/4]."""
    import torch
    OH = dg_conv_out_dim(desc.H, desc.KH, desc.stride_h, desc.pad_h)
    OW = dg_conv_out_dim(desc.W, desc.KW, desc.stride_w, desc.pad_w)
    if out is None:
        out = torch.empty(dg_packed_activation_bytes(desc.B * OH * OW, desc.Cout), dtype=torch.uint8, device=Wp.device)
    _check(lib().dg_conv2d_lut_requant(lut.handle, _dev_ptr(Wp, torch.uint8, "Wp"), _dev_ptr(Xp, torch.uint8, "Xp"),
                                       ctypes.byref(desc), _dev_ptr(scale, torch.float32, "scale"), q_scale, q_zero, lo,
                                       _dev_ptr(out, torch.uint8, "packed"), out.numel(), _kernel(variant),
                                       _stream_ptr(stream)))
    return out
