"""Do the pins bite?  Each case plants ONE plausible mistake in a private copy of the oracle's C source (a wrong sign,
a transposed operand, a dropped term, a wrong bound, a swapped loop order ...), rebuilds that copy on the CPU and runs
the pin suite against it: at least one pin must fail.  The unmodified copy must pass (control)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

F32_CONV_LOOPS = """                    for (int64_t kh = 0; kh < KH; ++kh) {
                        const int64_t ih = oh * sh - ph + kh;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            const int64_t iw = ow * sw - pw + kw;
                            if (iw < 0 || iw >= W) continue;
"""
F32_CONV_LOOPS_KW_FIRST = """                    for (int64_t kw = 0; kw < KW; ++kw) {
                        const int64_t iw = ow * sw - pw + kw;
                        if (iw < 0 || iw >= W) continue;
                        for (int64_t kh = 0; kh < KH; ++kh) {
                            const int64_t ih = oh * sh - ph + kh;
                            if (ih < 0 || ih >= H) continue;
"""

# (name, file, function the text is looked for in (None: whole file, first occurrence), original text, planted text)
MUTATIONS = [
    ("gemm_sign", "dg_oracle.c", None, "s += (int64_t)lw[w[k]] * (int64_t)la[a[k]];", "s -= (int64_t)lw[w[k]] * (int64_t)la[a[k]];"),
    ("gemm_levels_transposed", "dg_oracle.c", None, "s += (int64_t)lw[w[k]] * (int64_t)la[a[k]];",
     "s += (int64_t)lw[a[k]] * (int64_t)la[w[k]];"),
    ("gemm_drops_last_term", "dg_oracle.c", None, "for (int64_t k = 0; k < K; ++k) {", "for (int64_t k = 0; k < K - 1; ++k) {"),
    ("conv_pad_sign", "dg_oracle.c", "conv_point", "int64_t iw = ow * sw - pw + kw;", "int64_t iw = ow * sw + pw + kw;"),
    ("conv_strides_swapped", "dg_oracle.c", "conv_point", "int64_t ih = oh * sh - ph + kh;", "int64_t ih = oh * sw - ph + kh;"),
    ("conv_bound_off_by_one", "dg_oracle.c", "conv_point", "if (iw < 0 || iw >= W) continue;", "if (iw < 0 || iw > W - 2) continue;"),
    ("conv_filter_transposed", "dg_oracle.c", "conv_point", "Wc + ((co * KH + kh) * KW + kw) * Cin;",
     "Wc + ((co * KH + kw) * KW + kh) * Cin;"),
    ("conv_sign", "dg_oracle.c", "conv_point", "s += (int64_t)lw[w[ci]] * (int64_t)la[x[ci]];",
     "s -= (int64_t)lw[w[ci]] * (int64_t)la[x[ci]];"),
    ("epilogue_scale_index", "dg_oracle.c", "dgo_scale_epilogue_nhwc", "out[r * channels + c] = f * scale[c];",
     "out[r * channels + c] = f * scale[0];"),
    ("table_gemm_index_order", "dg_oracle.c", "dgo_gemm_table(", "s += table[nlev * w + a];", "s += table[nlev * a + w];"),
    ("table_conv_index_order", "dg_oracle.c", "dgo_conv2d_table(", "s += table[nlev * w + a];", "s += table[nlev * a + w];"),
    ("f32_table_index_order", "dg_oracle.c", "dgo_build_lut_f32", "table[4 * w + a] = p;", "table[4 * a + w] = p;"),
    ("f32_gemm_descending_k", "dg_oracle.c", "dgo_gemm_table_f32", "for (int64_t k = 0; k < K; ++k) {",
     "for (int64_t k = K - 1; k >= 0; --k) {"),
    ("f32_conv_kw_before_kh", "dg_oracle.c", "dgo_conv2d_table_f32", F32_CONV_LOOPS, F32_CONV_LOOPS_KW_FIRST),
    ("f32_conv_descending_ci", "dg_oracle.c", "dgo_conv2d_table_f32", "for (int64_t ci = 0; ci < Cin; ++ci) {",
     "for (int64_t ci = Cin - 1; ci >= 0; --ci) {"),
    ("f32_conv_descending_kh", "dg_oracle.c", "dgo_conv2d_table_f32", "for (int64_t kh = 0; kh < KH; ++kh) {",
     "for (int64_t kh = KH - 1; kh >= 0; --kh) {"),
    ("lut_index_order", "dg_lut_reference.c", "dgo_build_lut", "table[nlev * w + a] = lw[w] * la[a];",
     "table[nlev * a + w] = lw[w] * la[a];"),
    ("pack_slot_order", "dg_lut_reference.c", "dgo_pack_codes", "byte = (uint8_t)(byte | (c << (sb * i)));",
     "byte = (uint8_t)(byte | (c << (8 - sb - sb * i)));"),
    ("lookup_weight_code_low", "dg_lut_reference.c", "dgo_lut_gemm_packed", "sum += table[(w << bits) | a];",
     "sum += table[(a << bits) | w];"),
]


def _plant(text: str, function, old: str, new: str) -> str:
    start = 0 if function is None else text.index(function)
    at = text.index(old, start)               # ValueError: the oracle was edited and this case needs updating
    return text[:at] + new + text[at + len(old):]


def _run_pins(tmp, mutation):
    work = os.path.join(tmp, "tree")
    os.makedirs(os.path.join(work, "tests"))
    os.makedirs(os.path.join(work, "paper_2304_09049_amd"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(work, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(work, "tests", "golden"))
    for name in ("conftest.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", name), os.path.join(work, "tests", name))
    for name in ("__init__.py", "workloads.py"):
        shutil.copy(os.path.join(ROOT, "paper_2304_09049_amd", name), os.path.join(work, "paper_2304_09049_amd", name))
    if mutation is not None:
        _, fname, function, old, new = mutation
        path = os.path.join(work, "oracle", fname)
        with open(path) as f:
            text = f.read()
        with open(path, "w") as f:
            f.write(_plant(text, function, old, new))
    env = dict(os.environ, PYTHONPATH=work, PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                          cwd=work, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)


def test_control_unmodified_copy_passes(tmp_path):
    r = _run_pins(str(tmp_path), None)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("mutation", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_pin_fails_for_each_planted_mistake(tmp_path, mutation):
    r = _run_pins(str(tmp_path), mutation)
    assert r.returncode == 1, f"no pin failed for {mutation[0]} (pytest rc {r.returncode}):\n{r.stdout[-1500:]}"
    assert "failed" in r.stdout
