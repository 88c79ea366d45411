"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol,
builds tables correctly and rejects bad arguments before anything is launched."""
import ctypes
import itertools
import json
import os
import re

import pytest

from paper_2304_09049_amd import binding as dg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "deepgemm_hip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dg_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = dg.lib()
    names = declared_symbols()
    assert set(names) == set(dg.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    L = dg.lib()
    for i, name in enumerate(dg.STATUS_NAMES):
        assert L.dg_status_string(i).decode() == name


def test_build_lut_brute_force_all_pairs():
    for lw, la in [((-2, -1, 0, 1), (0, 1, 2, 3)), ((0, 1, -2, -1), (3, 1, 0, 2)), ((-8, 7, 3, -5), (-7, 6, -8, 1))]:
        t = dg.dg_build_lut(lw, la, dg.DG_LUT_I8).entries()
        for w, a in itertools.product(range(4), range(4)):
            assert t[4 * w + a] == lw[w] * la[a]


def test_build_lut_matches_hand_written_table(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "lut16_signed_unsigned.json")))
    assert dg.dg_build_lut(g["levels_w"], g["levels_a"]).entries() == g["table"]


def test_build_lut_rejects_int8_overflow_and_accepts_int16():
    with pytest.raises(dg.DgError) as e:
        dg.dg_build_lut((127, 0, 0, 0), (2, 0, 0, 0), dg.DG_LUT_I8)
    assert e.value.status == 3          # DG_ERR_RANGE: 254 does not fit int8
    with pytest.raises(dg.DgError):
        dg.dg_build_lut((-128, 0, 0, 0), (-1, 0, 0, 0), dg.DG_LUT_I8)   # +128
    t = dg.dg_build_lut((127, -128, 0, 1), (-128, 127, 1, 0), dg.DG_LUT_I16).entries()
    assert t[0] == 127 * -128 and t[5] == -128 * 127 and t[4] == 16384
    dg.dg_build_lut((-128, 0, 0, 0), (1, 0, 0, 0), dg.DG_LUT_I8)        # -128 fits


def test_build_lut_null_arguments():
    L = dg.lib()
    h = ctypes.c_void_p(0)
    lw = (ctypes.c_int8 * 4)(1, 2, 3, 4)
    assert L.dg_build_lut(None, lw, 0, ctypes.byref(h)) == 1
    assert L.dg_build_lut(lw, lw, 0, None) == 1
    assert L.dg_build_lut(lw, lw, 7, ctypes.byref(h)) == 5
    assert b"NULL" in L.dg_last_error() or b"unknown" in L.dg_last_error()
    L.dg_lut_destroy(None)


def test_packed_sizes():
    assert dg.dg_packed_activation_bytes(196, 576) == 196 * 144
    assert dg.dg_packed_activation_bytes(3, 6) == 0           # K % 4 != 0
    assert dg.dg_packed_activation_bytes(-1, 8) == 0
    assert dg.dg_packed_weight_bytes(64, 576) >= 64 * 144


def test_conv_out_dim():
    assert dg.dg_conv_out_dim(56, 3, 1, 1) == 56
    assert dg.dg_conv_out_dim(56, 3, 2, 1) == 28
    assert dg.dg_conv_out_dim(8, 3, 2, 0) == 3
    assert dg.dg_conv_out_dim(224, 7, 2, 3) == 112
    assert dg.dg_conv_out_dim(2, 3, 1, 0) == 0


def test_gemm_argument_errors_are_caught_before_any_launch():
    L = dg.lib()
    lut = dg.dg_build_lut((-2, -1, 0, 1), (0, 1, 2, 3))
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    call = lambda *a: L.dg_gemm_lut(*a)
    assert call(None, fake, fake, 4, 4, 4, fake, 4, 1, None, None, 0, None) == 1       # NULL table
    assert call(lut.handle, None, fake, 4, 4, 4, fake, 4, 1, None, None, 0, None) == 1  # NULL operand
    assert call(lut.handle, fake, fake, 4, 4, 4, None, 4, 1, None, None, 0, None) == 1  # NULL output
    assert call(lut.handle, fake, fake, 4, 4, 4, fake, 4, 1, fake, None, 0, None) == 1  # scale but no fp32 out
    assert call(lut.handle, fake, fake, 0, 4, 4, fake, 4, 1, None, None, 0, None) == 2  # M = 0
    assert call(lut.handle, fake, fake, 4, 4, 6, fake, 4, 1, None, None, 0, None) == 2  # K % 4
    assert call(lut.handle, fake, fake, 4, 4, 4, fake, 0, 1, None, None, 0, None) == 2  # zero stride
    big = dg.dg_build_lut((127, -128, 0, 1), (-128, 127, 1, 0), dg.DG_LUT_I16)
    assert call(big.handle, fake, fake, 4, 4, 1 << 18, fake, 4, 1, None, None, 0, None) == 3   # 2^18 * 16384 = 2^32
    assert L.dg_last_error().decode() != ""


def test_conv_argument_errors_are_caught_before_any_launch():
    L = dg.lib()
    lut = dg.dg_build_lut((-2, -1, 0, 1), (0, 1, 2, 3))
    fake = ctypes.c_void_p(0x1000)

    def call(desc, w=fake, x=fake, y=fake, scale=None, yf=None):
        return L.dg_conv2d_lut(lut.handle, w, x, ctypes.byref(desc) if desc is not None else None, y, scale, yf, 0, None)

    good = dg.conv_desc(1, 8, 8, 8, 4, 3, 3, (1, 1), (1, 1))
    assert call(None) == 1
    assert call(good, w=None) == 1
    assert call(good, y=None) == 1
    assert call(dg.conv_desc(1, 8, 8, 6, 4, 3, 3)) == 2                    # Cin % 4
    assert call(dg.conv_desc(1, 2, 2, 8, 4, 3, 3)) == 2                    # filter larger than image
    assert call(dg.conv_desc(1, 8, 8, 8, 4, 3, 3, (0, 1))) == 2            # stride 0
    assert call(dg.conv_desc(1, 8, 8, 8, 4, 3, 3, (1, 1), (-1, 0))) == 2   # negative pad
    assert call(dg.conv_desc(0, 8, 8, 8, 4, 3, 3)) == 2                    # empty batch


def test_one_call_entry_points_check_their_arguments_before_any_launch():
    L = dg.lib()
    lut = dg.dg_build_lut((-2, -1, 0, 1), (0, 1, 2, 3))
    fake = ctypes.c_void_p(0x1000)
    g = lambda w, a, M, N, K, work, wb, c: L.dg_gemm_lut_codes(lut.handle, w, a, M, N, K, work, wb, c, N, 1, None, None, 0, None)
    assert g(None, fake, 4, 4, 8, fake, 100, fake) == 1                      # NULL operand
    assert g(fake, fake, 4, 4, 8, fake, 100, None) == 1                      # NULL output
    assert g(fake, fake, 4, 4, 6, fake, 100, fake) == 2                      # K % 4 != 0
    assert g(fake, fake, 4, 0, 8, fake, 100, fake) == 2
    assert g(fake, fake, 4, 4, 8, None, 0, fake) == 1                        # K % 32 != 0 is never fused: the work buffer is needed
    assert g(fake, fake, 4, 4, 8, fake, 7, fake) == 4                        # ... and must hold 4 * 8 / 4 bytes
    assert L.dg_gemm_lut_codes(None, fake, fake, 4, 4, 8, fake, 100, fake, 4, 1, None, None, 0, None) == 1
    desc = dg.conv_desc(1, 8, 8, 8, 4, 3, 3, (1, 1), (1, 1))
    c = lambda w, x, d, work, wb, y: L.dg_conv2d_lut_codes(lut.handle, w, x, ctypes.byref(d) if d is not None else None, work, wb,
                                                           y, None, None, 0, None)
    assert c(None, fake, desc, fake, 1000, fake) == 1
    assert c(fake, fake, None, fake, 1000, fake) == 1
    assert c(fake, fake, desc, fake, 1000, None) == 1
    assert c(fake, fake, dg.conv_desc(1, 8, 8, 6, 4, 3, 3), fake, 1000, fake) == 2     # Cin % 4 != 0
    assert c(fake, fake, desc, None, 0, fake) == 1                           # Cin = 8 is never fused: the work buffer is needed
    assert c(fake, fake, desc, fake, 8 * 8 * 8 // 4 - 1, fake) == 4


def test_pack_argument_errors():
    L = dg.lib()
    fake = ctypes.c_void_p(0x1000)
    assert L.dg_pack_activations(None, 4, 4, fake, 4, None) == 1
    assert L.dg_pack_activations(fake, 4, 6, fake, 100, None) == 2
    assert L.dg_pack_activations(fake, 0, 4, fake, 100, None) == 2
    assert L.dg_pack_weights(fake, 4, 8, fake, 7, None) == 4               # needs 8 bytes


def test_wide_tables_follow_table2():
    # Table 2 of the paper: b + b index bits, 2^(2b) entries
    for bits, n in ((3, 64), (4, 256)):
        lw = list(range(-(1 << (bits - 1)), 1 << (bits - 1)))
        la = list(range(1 << bits))
        t = dg.dg_build_lut_bits(bits, lw, la, dg.DG_LUT_I8)
        e = t.entries()
        assert len(e) == n and dg.lib().dg_lut_bits(t.handle) == bits
        for w, a in itertools.product(range(1 << bits), repeat=2):
            assert e[(w << bits) | a] == lw[w] * la[a]
    L = dg.lib()
    h = ctypes.c_void_p(0)
    lw = (ctypes.c_int8 * 32)(*range(32))
    assert L.dg_build_lut_bits(5, lw, lw, 0, ctypes.byref(h)) == 5
    assert L.dg_build_lut_bits(1, lw, lw, 0, ctypes.byref(h)) == 5
    assert dg.dg_packed_bytes_bits(10, 8, 4) == 40 and dg.dg_packed_bytes_bits(10, 8, 3) == 40
    assert dg.dg_packed_bytes_bits(10, 8, 2) == 20 and dg.dg_packed_bytes_bits(10, 7, 4) == 0


def test_tables_given_as_such():
    entries = [3, -7, 100, 0, 5, 5, -128, 127, 1, 2, 3, 4, -1, -2, -3, -4]
    assert dg.dg_build_lut_entries(entries, dg.DG_LUT_I8).entries() == entries
    with pytest.raises(dg.DgError) as e:
        dg.dg_build_lut_entries([200] + [0] * 15, dg.DG_LUT_I8)
    assert e.value.status == 3
    assert dg.dg_build_lut_entries([200] + [0] * 15, dg.DG_LUT_I16).entries()[0] == 200
    import numpy as np
    lw, la = np.array([0.1, -0.37, 1.5, 3.0e-3], np.float32), np.array([0.0, 0.7, 1.9, 2.25], np.float32)
    got = np.array(dg.dg_build_lut_f32(lw, la).entries(), dtype=np.float32)
    assert np.array_equal(got, (lw[:, None] * la[None, :]).astype(np.float32).reshape(-1))   # one float32 multiply each


def test_empty_launch_rejects_bad_grids_before_launching():
    L = dg.lib()
    assert L.dg_launch_empty(0, 64, None) == 2
    assert L.dg_launch_empty(10, 0, None) == 2
    assert L.dg_launch_empty(10, 100, None) == 2          # not a multiple of 64
    assert L.dg_launch_empty(10, 2048, None) == 2         # more than 1024 threads
    assert L.dg_launch_empty(1 << 40, 64, None) == 2


def test_kernel_names_need_no_gpu():
    # the plan functions are host code: small layers split K, large ones get a wave tile, wide entries two planes
    lut = dg.dg_build_lut((-2, -1, 0, 1), (0, 1, 2, 3))
    assert dg.dg_gemm_kernel_name(lut, 64, 196, 576).startswith("onehot_mfma_splitk_s")
    # large layers: the sparse instruction, operands staged through LDS where the taps are whole 32-byte runs
    assert dg.dg_gemm_kernel_name(lut, 8192, 8192, 8192) == "onehot_smfmac_staged_64x128"
    assert dg.dg_gemm_kernel_name(lut, 8192, 8192, 8192 + 64) == "onehot_smfmac_64x128"
    assert dg.dg_gemm_kernel_name(lut, 8192, 8192, 8192, "onehot_mfma") == "onehot_mfma_64x128"
    assert dg.dg_gemm_kernel_name(lut, 8192, 256, 8192) == "onehot_smfmac_staged_32x128_k4"      # wavefronts share tiles
    assert dg.dg_gemm_kernel_name(lut, 8192, 256, 8192 + 64) == "onehot_smfmac_64x64_k4"
    assert dg.dg_gemm_kernel_name(lut, 8192, 256, 8192, "onehot_mfma") == "onehot_mfma_64x64_k4"
    assert dg.dg_gemm_kernel_name(lut, 8192, 64, 8192) == "onehot_smfmac_staged_32x64_k4"
    assert dg.dg_gemm_kernel_name(lut, 8192, 64, 8192 + 64) == "onehot_mfma_64x32_k4"  # narrow shared tiles, direct loads: dense
    assert dg.dg_gemm_kernel_name(lut, 8192, 1, 8192) == "onehot_smfmac_fewn_16"       # 1 to 16 columns, long rows
    assert dg.dg_gemm_kernel_name(lut, 8192, 1, 8192 + 64) == "smalln"
    assert dg.dg_gemm_kernel_name(lut, 64, 196, 48).startswith("perm")        # Cin % 32 != 0, % 16 == 0
    assert dg.dg_gemm_kernel_name(lut, 5, 7, 12) == "lds"                      # Cin % 16 != 0
    # the comparison kernel has the same plans, and a 128 x 128 tile of its own for the largest problems
    assert dg.dg_gemm_kernel_name(lut, 64, 196, 576, "mfma_i8").startswith("mfma_i8_splitk_s")
    assert dg.dg_gemm_kernel_name(lut, 8192, 8192, 8192, "mfma_i8") == "mfma_i8_128x128"
    wide = dg.dg_build_lut((127, -128, 5, 0), (-128, 127, 1, 0), dg.DG_LUT_I16)
    assert dg.dg_gemm_kernel_name(wide, 8192, 8192, 8192) == "onehot_smfmac_2p_32x128"   # large layers: the sparse instruction
    assert dg.dg_gemm_kernel_name(wide, 8192, 8192, 8192, "onehot_mfma") == "onehot_mfma_2p_32x128"
    assert dg.dg_gemm_kernel_name(wide, 256, 1568, 2304).startswith("onehot_mfma_2p_")
    t4 = dg.dg_build_lut_bits(4, list(range(-8, 8)), list(range(16)), dg.DG_LUT_I8)
    assert dg.dg_gemm_kernel_name(t4, 256, 50176, 2304) == "onehot_smfmac4_64x128"      # large layers: the sparse instruction
    assert dg.dg_gemm_kernel_name(t4, 256, 50176, 2304, "onehot_mfma").startswith("onehot_mfma_64x")
    assert dg.dg_gemm_kernel_name(t4, 256, 1568, 2304).startswith("onehot_mfma_")
    assert dg.dg_gemm_kernel_name(t4, 256, 50176, 2304, "perm") == "unsupported"
    # packing + convolution in one call: fused into the split-K kernel on small layers only
    small = dg.conv_desc(1, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1))
    large = dg.conv_desc(16, 56, 56, 256, 256, 3, 3, (1, 1), (1, 1))
    assert dg.dg_conv_codes_kernel_name(lut, small) == "codes_onehot_mfma_splitk_s9"
    assert dg.dg_conv_codes_kernel_name(lut, small, "onehot_smfmac") == dg.dg_conv_kernel_name(lut, small, "onehot_smfmac")
    # (1568 pixel blocks x 8 channel blocks: 32 x 224 tiles leave the busiest SIMD 14 blocks, 64 x 128 tiles 16)
    assert dg.dg_conv_codes_kernel_name(lut, large) == dg.dg_conv_kernel_name(lut, large) == "onehot_smfmac_staged_32x224"
    assert dg.dg_gemm_codes_kernel_name(lut, 64, 196, 576) == "codes_onehot_mfma_splitk_s9"
    # K up to 512 split: the dense instruction walks K in chunks of 64 positions where 128 would cap the wavefronts per tile
    k256 = dg.conv_desc(1, 56, 56, 256, 64, 1, 1, (1, 1), (0, 0))
    assert dg.dg_conv_kernel_name(lut, k256) == "onehot_mfma_splitk_s4"
    assert dg.dg_conv_codes_kernel_name(lut, k256) == "codes_onehot_mfma_splitk_s4"
    assert dg.dg_conv_kernel_name(lut, k256, "mfma_i8") == "mfma_i8_splitk_s4"
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(1, 28, 28, 512, 128, 1, 1, (1, 1), (0, 0))) == "onehot_mfma_splitk_s8"
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(1, 14, 14, 1024, 256, 1, 1, (1, 1), (0, 0))) == "onehot_mfma_splitk_s8"
    # layers of a few microseconds on the tiled kernels: one call packs in the dense instruction's narrow tiles (up to
    # about 1e9 table operations, more where a strided 1x1 layer leaves most of the input unread), larger ones do not
    mid = dg.conv_desc(8, 14, 14, 1024, 256, 1, 1, (1, 1), (0, 0))
    assert dg.dg_conv_kernel_name(lut, mid) == "onehot_smfmac_staged_32x64_k4"
    assert dg.dg_conv_codes_kernel_name(lut, mid) == "codes_onehot_smfmac_64x32_k4"
    assert dg.dg_conv_codes_kernel_name(lut, mid, "onehot_mfma") == "codes_onehot_mfma_64x32_k4"
    strided = dg.conv_desc(32, 56, 56, 256, 128, 1, 1, (2, 2), (0, 0))
    assert dg.dg_conv_codes_kernel_name(lut, strided) == "codes_onehot_smfmac_64x32"
    big = dg.conv_desc(32, 14, 14, 1024, 256, 1, 1, (1, 1), (0, 0))
    assert dg.dg_conv_codes_kernel_name(lut, big) == dg.dg_conv_kernel_name(lut, big) == "onehot_smfmac_staged_32x64"
    # taps of an odd number of 64-position chunks: staged with a window and 192 channels or more, direct loads with 64
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(32, 28, 28, 320, 320, 3, 3, (1, 1), (1, 1))) == "onehot_smfmac_staged_32x128"
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(32, 28, 28, 192, 96, 3, 3, (1, 1), (1, 1))) == "onehot_smfmac_staged_32x64"
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(32, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1))) == "onehot_smfmac_64x64"
    # unshared 64 x 32 tiles: the sparse instruction where every SIMD has more than one (1568 here, 784 at batch 8 of 56 x 56)
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(1, 224, 224, 64, 64, 3, 3, (1, 1), (1, 1))) == "onehot_smfmac_64x32"
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(8, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1))) == "onehot_mfma_64x32"
    # K = 512 shared by four wavefronts would be one run each: not staged
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(8, 28, 28, 512, 128, 1, 1, (1, 1), (0, 0))) == "onehot_mfma_64x32_k4"
    assert dg.dg_conv_kernel_name(lut, dg.conv_desc(8, 14, 14, 1024, 256, 1, 1, (1, 1), (0, 0))) == "onehot_smfmac_staged_32x64_k4"
    assert dg.dg_gemm_codes_kernel_name(lut, 8192, 1, 8192) == "codes_smalln"
    # 256 row blocks would each pack the activations for themselves: two kernels unless the fused form is asked for by name
    assert dg.dg_gemm_codes_kernel_name(lut, 8192, 16, 8192) == dg.dg_gemm_kernel_name(lut, 8192, 16, 8192)
    assert dg.dg_gemm_codes_kernel_name(lut, 8192, 16, 8192, "onehot_mfma").startswith("codes_onehot_mfma_splitk_s")
    assert dg.dg_gemm_codes_kernel_name(lut, 8192, 8192, 8192) == "onehot_smfmac_staged_64x128"


def test_dequantize_argument_errors():
    L = dg.lib()
    fake = ctypes.c_void_p(0x1000)
    assert L.dg_dequantize(None, 4, 4, fake, fake, None) == 1
    assert L.dg_dequantize(fake, 4, 4, None, fake, None) == 1
    assert L.dg_dequantize(fake, 0, 4, fake, fake, None) == 2
    assert L.dg_dequantize(fake, 4, -1, fake, fake, None) == 2


def test_network_layer_tables_add_up():
    """bench.py --layers: the layer tables against the networks' published sizes.  Multiply-accumulates of all
    convolutions on a 224 x 224 input, less the first layer's (7x7x3 -> 64 at stride 2 on 112 x 112 outputs for the
    ResNets, 3x3x3 -> 64 on 224 x 224 for VGG-16), which is not quantised: ResNet-18 1.81 G less 0.118 G and the
    classifier, ResNet-50 4.09 G less 0.118 G, VGG-16 15.35 G less 0.087 G."""
    import bench
    nets = bench.network_layers()
    macs, count = {}, {}
    for net, shapes in nets.items():
        macs[net] = sum(n * ((H + 2 * (k // 2) - k) // s + 1) ** 2 * Cin * Cout * k * k for (H, Cin, Cout, k, s, n) in shapes)
        count[net] = sum(n for (*_, n) in shapes)
    assert count == {"resnet18": 19, "resnet50": 52, "vgg16": 12}
    assert abs(macs["resnet18"] / 1e9 - 1.69) < 0.01
    assert abs(macs["resnet50"] / 1e9 - 3.97) < 0.01
    assert abs(macs["vgg16"] / 1e9 - 15.26) < 0.01
