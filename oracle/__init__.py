"""CPU oracle for the 2-bit lookup-table GEMM / convolution -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrappers over ``dg_oracle.c`` (the result, by explicit multiply of
decoded levels) and ``dg_lut_reference.c`` (the table method's steps on packed
bytes).  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import this package; the GPU library never does, and this package never imports
the GPU library.

Every function takes and returns numpy arrays.  Codes are ``uint8``, one per
element; levels are 4 integers per side (2-bit codes, the paper's kernels) or 8 /
16 (the 3- and 4-bit extension of Sec. 3.3).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SOURCES = ("dg_oracle.c", "dg_lut_reference.c")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle's C files with gcc into ``oracle/liboracle.so``."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    if not force and os.path.exists(_SO):
        newest = max(os.path.getmtime(s) for s in srcs)
        if os.path.getmtime(_SO) >= newest:
            return _SO
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", _SO] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.dgo_max_threads.restype = ctypes.c_int
        lib.dgo_set_threads.argtypes = [ctypes.c_int]
        lib.dgo_gemm.argtypes = [p, p, p, p, ctypes.c_int, i64, i64, i64, p]
        lib.dgo_gemm_sampled.argtypes = [p, p, p, p, ctypes.c_int, i64, i64, i64, p, p, i64, p]
        lib.dgo_conv_out_dim.argtypes = [i64] * 4
        lib.dgo_conv_out_dim.restype = i64
        lib.dgo_conv2d.argtypes = [p, p, p, p, ctypes.c_int] + [i64] * 11 + [p]
        lib.dgo_conv2d_sampled.argtypes = [p, p, p, p, ctypes.c_int] + [i64] * 11 + [p, i64, p]
        lib.dgo_scale_epilogue_nhwc.argtypes = [p, p, i64, i64, p]
        lib.dgo_scale_epilogue_nhwc.restype = None
        lib.dgo_scale_epilogue_rows.argtypes = [p, p, i64, i64, p]
        lib.dgo_scale_epilogue_rows.restype = None
        lib.dgo_quantize_codes.argtypes = [p, i64, ctypes.c_float, ctypes.c_float, ctypes.c_int32, ctypes.c_int32, p]
        lib.dgo_gemm_table.argtypes = [p, p, p, ctypes.c_int, i64, i64, i64, p]
        lib.dgo_conv2d_table.argtypes = [p, p, p, ctypes.c_int] + [i64] * 11 + [p]
        lib.dgo_build_lut_f32.argtypes = [p, p, p]
        lib.dgo_build_lut_f32.restype = None
        lib.dgo_gemm_table_f32.argtypes = [p, p, p, i64, i64, i64, p]
        lib.dgo_conv2d_table_f32.argtypes = [p, p, p] + [i64] * 11 + [p]
        lib.dgo_build_lut.argtypes = [p, p, ctypes.c_int, p]
        lib.dgo_build_lut.restype = None
        lib.dgo_pack_codes.argtypes = [p, i64, ctypes.c_int, p]
        lib.dgo_unpack_codes.argtypes = [p, i64, ctypes.c_int, p]
        lib.dgo_unpack_codes.restype = None
        lib.dgo_lut_gemm_packed.argtypes = [p, p, p, ctypes.c_int, i64, i64, i64, p]
        _lib = lib
    return _lib


class OracleError(ValueError):
    """Raised when the oracle rejects its input (bad code, overflow, bad shape)."""


_ERRORS = {1: "a code is greater than 3", 2: "a sum does not fit int32", 3: "bad shape or index"}


def _check(rc: int) -> None:
    if rc != 0:
        raise OracleError(_ERRORS.get(rc, f"error {rc}"))


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _codes(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.uint8)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise OracleError(f"expected shape {shape}, got {a.shape}")
    return a


def _levels(v) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.int32)
    if v.ndim != 1 or v.shape[0] not in (4, 8, 16):
        raise OracleError("a level table has 4, 8 or 16 entries (2-, 3- or 4-bit codes)")
    return v


def _both(levels_w, levels_a):
    lw, la = _levels(levels_w), _levels(levels_a)
    if lw.shape != la.shape:
        raise OracleError("both sides use the same code width")
    return lw, la, int(lw.shape[0])


def max_threads() -> int:
    return int(_load().dgo_max_threads())


def set_threads(n: int) -> None:
    _load().dgo_set_threads(int(n))


def gemm(Wc, Ac, levels_w, levels_a) -> np.ndarray:
    """C[m][n] = sum_k lw[Wc[m][k]] * la[Ac[n][k]]  (int32, [M][N])."""
    Wc, Ac = _codes(Wc), _codes(Ac)
    M, K = Wc.shape
    N, K2 = Ac.shape
    if K != K2:
        raise OracleError("reduction lengths differ")
    C = np.zeros((M, N), dtype=np.int32)
    lw, la, nlev = _both(levels_w, levels_a)
    _check(_load().dgo_gemm(_ptr(Wc), _ptr(Ac), _ptr(lw), _ptr(la), nlev, M, N, K, _ptr(C)))
    return C


def gemm_sampled(Wc, Ac, levels_w, levels_a, ms, ns) -> np.ndarray:
    """The GEMM result at positions (ms[i], ns[i]) only."""
    Wc, Ac = _codes(Wc), _codes(Ac)
    M, K = Wc.shape
    N, K2 = Ac.shape
    if K != K2:
        raise OracleError("reduction lengths differ")
    ms = np.ascontiguousarray(ms, dtype=np.int64)
    ns = np.ascontiguousarray(ns, dtype=np.int64)
    out = np.zeros(ms.shape[0], dtype=np.int32)
    lw, la, nlev = _both(levels_w, levels_a)
    _check(_load().dgo_gemm_sampled(_ptr(Wc), _ptr(Ac), _ptr(lw), _ptr(la), nlev, M, N, K,
                                    _ptr(ms), _ptr(ns), ms.shape[0], _ptr(out)))
    return out


def conv_out_dim(size: int, k: int, stride: int, pad: int) -> int:
    return int(_load().dgo_conv_out_dim(size, k, stride, pad))


def conv2d(Wc, Xc, levels_w, levels_a, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """Direct NHWC convolution.  Wc [Cout][KH][KW][Cin], Xc [B][H][W][Cin] -> int32 [B][OH][OW][Cout]."""
    Wc, Xc = _codes(Wc), _codes(Xc)
    Cout, KH, KW, Cin = Wc.shape
    B, H, W, Cin2 = Xc.shape
    if Cin != Cin2:
        raise OracleError("channel counts differ")
    sh, sw = stride
    ph, pw = pad
    OH, OW = conv_out_dim(H, KH, sh, ph), conv_out_dim(W, KW, sw, pw)
    Y = np.zeros((B, max(OH, 0), max(OW, 0), Cout), dtype=np.int32)
    lw, la, nlev = _both(levels_w, levels_a)
    _check(_load().dgo_conv2d(_ptr(Wc), _ptr(Xc), _ptr(lw), _ptr(la), nlev, B, H, W, Cin, Cout,
                              KH, KW, sh, sw, ph, pw, _ptr(Y)))
    return Y


def conv2d_sampled(Wc, Xc, levels_w, levels_a, positions, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """The convolution result at flat NHWC output indices ``positions`` only."""
    Wc, Xc = _codes(Wc), _codes(Xc)
    Cout, KH, KW, Cin = Wc.shape
    B, H, W, Cin2 = Xc.shape
    if Cin != Cin2:
        raise OracleError("channel counts differ")
    sh, sw = stride
    ph, pw = pad
    pos = np.ascontiguousarray(positions, dtype=np.int64)
    out = np.zeros(pos.shape[0], dtype=np.int32)
    lw, la, nlev = _both(levels_w, levels_a)
    _check(_load().dgo_conv2d_sampled(_ptr(Wc), _ptr(Xc), _ptr(lw), _ptr(la), nlev, B, H, W, Cin, Cout,
                                      KH, KW, sh, sw, ph, pw, _ptr(pos), pos.shape[0], _ptr(out)))
    return out


def scale_epilogue_nhwc(acc, scale) -> np.ndarray:
    """out[..., c] = float32(acc[..., c]) * scale[c]  (channels last)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    C = acc.shape[-1]
    if scale.shape != (C,):
        raise OracleError("one scale per channel")
    out = np.zeros(acc.shape, dtype=np.float32)
    _load().dgo_scale_epilogue_nhwc(_ptr(acc), _ptr(scale), acc.size // max(C, 1), C, _ptr(out))
    return out


def scale_epilogue_rows(acc, scale) -> np.ndarray:
    """out[m][n] = float32(acc[m][n]) * scale[m]  (GEMM result stored [M][N])."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    M, N = acc.shape
    if scale.shape != (M,):
        raise OracleError("one scale per row")
    out = np.zeros(acc.shape, dtype=np.float32)
    _load().dgo_scale_epilogue_rows(_ptr(acc), _ptr(scale), M, N, _ptr(out))
    return out


def quantize_codes(x, scale: float, zero_point: float, lo: int, hi: int) -> np.ndarray:
    """code = clip(rint(float32(scale * x) + zero_point), lo, hi) - lo, decided in float32 (Eq. 1); hi - lo must be 3."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.zeros(x.shape, dtype=np.uint8)
    _check(_load().dgo_quantize_codes(_ptr(x), x.size, float(np.float32(scale)), float(np.float32(zero_point)),
                                      int(lo), int(hi), _ptr(codes)))
    return codes


# ---- tables that are given as such: arbitrary integer entries, binary32 entries --------------------------------

def _nlev_of_table(table) -> int:
    n = {16: 4, 64: 8, 256: 16}.get(int(np.asarray(table).size))
    if n is None:
        raise OracleError("a table has 16, 64 or 256 entries")
    return n


def gemm_table(Wc, Ac, table) -> np.ndarray:
    """C[m][n] = sum_k table[nlev*Wc[m][k] + Ac[n][k]] for an arbitrary integer table (it need not be a product of levels)."""
    Wc, Ac = _codes(Wc), _codes(Ac)
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(-1)
    (M, K), N = Wc.shape, Ac.shape[0]
    C = np.zeros((M, N), dtype=np.int32)
    _check(_load().dgo_gemm_table(_ptr(Wc), _ptr(Ac), _ptr(table), _nlev_of_table(table), M, N, K, _ptr(C)))
    return C


def conv2d_table(Wc, Xc, table, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    Wc, Xc = _codes(Wc), _codes(Xc)
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(-1)
    Cout, KH, KW, Cin = Wc.shape
    B, H, W, _ = Xc.shape
    OH, OW = conv_out_dim(H, KH, stride[0], pad[0]), conv_out_dim(W, KW, stride[1], pad[1])
    Y = np.zeros((B, max(OH, 0), max(OW, 0), Cout), dtype=np.int32)
    _check(_load().dgo_conv2d_table(_ptr(Wc), _ptr(Xc), _ptr(table), _nlev_of_table(table), B, H, W, Cin, Cout,
                                    KH, KW, stride[0], stride[1], pad[0], pad[1], _ptr(Y)))
    return Y


def build_lut_f32(levels_w, levels_a) -> np.ndarray:
    """table[4*w + a] = float32(lw[w]) * float32(la[a]), one binary32 multiply each."""
    lw = np.ascontiguousarray(levels_w, dtype=np.float32)
    la = np.ascontiguousarray(levels_a, dtype=np.float32)
    if lw.shape != (4,) or la.shape != (4,):
        raise OracleError("binary32 tables are defined for 2-bit codes: 4 levels per side")
    table = np.zeros(16, dtype=np.float32)
    _load().dgo_build_lut_f32(_ptr(lw), _ptr(la), _ptr(table))
    return table


def gemm_table_f32(Wc, Ac, table) -> np.ndarray:
    """binary32 sum of table entries, one addition per k in ascending order, starting from +0."""
    Wc, Ac = _codes(Wc), _codes(Ac)
    table = np.ascontiguousarray(table, dtype=np.float32)
    (M, K), N = Wc.shape, Ac.shape[0]
    C = np.zeros((M, N), dtype=np.float32)
    _check(_load().dgo_gemm_table_f32(_ptr(Wc), _ptr(Ac), _ptr(table), M, N, K, _ptr(C)))
    return C


def conv2d_table_f32(Wc, Xc, table, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    Wc, Xc = _codes(Wc), _codes(Xc)
    table = np.ascontiguousarray(table, dtype=np.float32)
    Cout, KH, KW, Cin = Wc.shape
    B, H, W, _ = Xc.shape
    OH, OW = conv_out_dim(H, KH, stride[0], pad[0]), conv_out_dim(W, KW, stride[1], pad[1])
    Y = np.zeros((B, max(OH, 0), max(OW, 0), Cout), dtype=np.float32)
    _check(_load().dgo_conv2d_table_f32(_ptr(Wc), _ptr(Xc), _ptr(table), B, H, W, Cin, Cout, KH, KW,
                                        stride[0], stride[1], pad[0], pad[1], _ptr(Y)))
    return Y


# ---- the table method's own steps (dg_lut_reference.c) -----------------------------------

def build_lut(levels_w, levels_a) -> np.ndarray:
    """table[nlev*w + a] = lw[w] * la[a]  (int32, nlev*nlev entries: 16 for 2-bit codes, 64, 256)."""
    lw, la, nlev = _both(levels_w, levels_a)
    table = np.zeros(nlev * nlev, dtype=np.int32)
    _load().dgo_build_lut(_ptr(lw), _ptr(la), nlev, _ptr(table))
    return table


def codes_per_byte(bits: int) -> int:
    return 4 if bits == 2 else 2


def pack_codes(codes, bits: int = 2) -> np.ndarray:
    """Pack along the last axis: 2-bit codes four per byte (code k at bits 2*(k%4) of byte k//4); 3- and 4-bit
    codes two per byte in 4-bit slots (code k at bits 4*(k%2) of byte k//2)."""
    codes = _codes(codes)
    per = codes_per_byte(bits)
    if codes.shape[-1] % per != 0:
        raise OracleError(f"the packed axis must be a multiple of {per}")
    packed = np.zeros(codes.shape[:-1] + (codes.shape[-1] // per,), dtype=np.uint8)
    _check(_load().dgo_pack_codes(_ptr(codes), codes.size, bits, _ptr(packed)))
    return packed


def unpack_codes(packed, bits: int = 2) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    codes = np.zeros(packed.shape[:-1] + (packed.shape[-1] * codes_per_byte(bits),), dtype=np.uint8)
    _load().dgo_unpack_codes(_ptr(packed), codes.size, bits, _ptr(codes))
    return codes


def lut_gemm_packed(Wp, Ap, table, K: int, bits: int = 2) -> np.ndarray:
    """GEMM by table lookup on packed operands (Algorithm 1, one byte at a time)."""
    Wp = np.ascontiguousarray(Wp, dtype=np.uint8)
    Ap = np.ascontiguousarray(Ap, dtype=np.uint8)
    table = np.ascontiguousarray(table, dtype=np.int32)
    M, N = Wp.shape[0], Ap.shape[0]
    per = codes_per_byte(bits)
    if Wp.shape[1] * per != K or Ap.shape[1] * per != K or table.shape != (1 << (2 * bits),):
        raise OracleError("bad packed shapes")
    C = np.zeros((M, N), dtype=np.int32)
    _check(_load().dgo_lut_gemm_packed(_ptr(Wp), _ptr(Ap), _ptr(table), bits, M, N, K, _ptr(C)))
    return C
