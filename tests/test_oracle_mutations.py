"""The pins have teeth: plausible mistakes planted in a *copy* of the oracle's
source (on the CPU, in a temp dir) must each be caught by the brute-force pin.

Each mutation is a textual edit of oracle/mdnn_oracle.c that still compiles:
a transposed filter index, a flipped kernel, a dropped pad, a wrong stride use,
a dropped channel stride, alpha applied per term, a wrong output index.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from test_oracle_pins import im2col_gemm

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "mdnn_oracle.c")

MUTATIONS = {
    "filter_ky_kx_transposed": ("filt[(((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o];",
                                "filt[(((size_t)c * Sk + kx) * Sk + ky) * (size_t)No + o];"),
    "kernel_flipped":          ("int iy = y * stride - pad + ky;\n                                if",
                                "int iy = y * stride - pad + (Sk - 1 - ky);\n                                if"),
    "pad_dropped_in_x":        ("int ix = x * stride - pad + kx;\n                                    if",
                                "int ix = x * stride + kx;\n                                    if"),
    "stride_on_tap":           ("int iy = y * stride - pad + ky;\n                                if",
                                "int iy = y - pad + ky * stride;\n                                if"),
    "input_row_stride_wrong":  ("in + (((size_t)c * Hi + iy) * Wi + ix) * (size_t)Nb;",
                                "in + (((size_t)c * Wi + iy) * Hi + ix) * (size_t)Nb;"),
    "filter_o_not_innermost":  ("filt[(((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o];",
                                "filt[(((size_t)o * Nc + c) * Sk + ky) * Sk + kx];"),
    "output_yx_swapped":       ("size_t base = (((size_t)o * Ho + y) * Wo + x) * (size_t)Nb;",
                                "size_t base = (((size_t)o * Wo + x) * Ho + y) * (size_t)Nb;"),
    "alpha_squared":           ("out[base + n] = (float)((double)alpha * S[n]);",
                                "out[base + n] = (float)((double)alpha * (double)alpha * S[n]);"),
    "apron_clamped_not_zero":  ("if (iy < 0 || iy >= Hi) continue;      /* zero apron */",
                                "if (iy < 0) iy = 0; if (iy >= Hi) iy = Hi - 1;"),
}


def _run(lib, inp, filt, stride, pad, alpha, out_shape):
    out = np.full(out_shape, np.nan, dtype=np.float32)
    Nc, Hi, Wi, Nb = inp.shape
    _, Sk, _, No = filt.shape
    i, f, p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
    lib.mdnn_oracle_conv_fprop.argtypes = [p, p, p, p, i, i, i, i, i, i, i, i, f, i]
    lib.mdnn_oracle_conv_fprop.restype = i
    rc = lib.mdnn_oracle_conv_fprop(inp.ctypes.data, filt.ctypes.data, out.ctypes.data, None,
                                    Nb, Wi, Hi, Nc, No, Sk, stride, pad, alpha, 1)
    assert rc == 0
    return out


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation anchor for {name} no longer in the oracle source"
    mutated = text.replace(old, new, 1)
    c = tmp_path / "mut.c"
    so = tmp_path / "mut.so"
    c.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    rng = np.random.default_rng(77)
    Nb, Nc, Hi, Wi, No, Sk, stride, pad, alpha = 3, 3, 9, 7, 4, 3, 2, 1, 0.75
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    filt = rng.uniform(-1, 1, size=(Nc, Sk, Sk, No)).astype(np.float32)
    want = im2col_gemm(inp, filt, stride, pad, alpha).astype(np.float32)
    got = _run(lib, inp, filt, stride, pad, alpha, want.shape)
    assert not np.allclose(got, want, rtol=1e-5, atol=1e-6, equal_nan=False), \
        f"the brute-force pin did not notice mutation {name}"


def test_unmutated_copy_passes(tmp_path):
    so = tmp_path / "same.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(so), SRC, "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    rng = np.random.default_rng(77)
    Nb, Nc, Hi, Wi, No, Sk, stride, pad, alpha = 3, 3, 9, 7, 4, 3, 2, 1, 0.75
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    filt = rng.uniform(-1, 1, size=(Nc, Sk, Sk, No)).astype(np.float32)
    want = im2col_gemm(inp, filt, stride, pad, alpha).astype(np.float32)
    got = _run(lib, inp, filt, stride, pad, alpha, want.shape)
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-7)
