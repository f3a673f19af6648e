"""CPU-only pins of the oracle's filter-gradient function (BPROP w.r.t. the weights).

The paper (arXiv 1501.06633, abstract and Section 3.5) only conjectures that
its approach carries over to BPROP and prints nothing to compare with, so the
function is pinned by what defines this gradient: it is the adjoint of the
(already pinned) forward map on the filter side -- with basis filters that
identity fixes every element on its own --, it equals a sum over output pixels
of patch x gradient outer products, it equals what the library's autograd
gives in float64, and delta inputs give a single known element.  Planted
mistakes in a copy of the source must be caught by the brute-force pin.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

CASES = [
    # Nb Nc Hi Wi No Sk stride pad
    (3, 2, 7, 6, 4, 3, 1, 1),
    (2, 3, 5, 7, 3, 1, 1, 0),
    (2, 2, 8, 8, 3, 3, 2, 0),
    (3, 3, 9, 7, 2, 5, 2, 2),
    (2, 1, 10, 11, 3, 4, 3, 1),
    (4, 2, 6, 6, 3, 3, 1, 2),
    (1, 2, 11, 11, 2, 11, 4, 0),   # one window: the gradient is an outer product
    (2, 3, 12, 9, 4, 3, 4, 1),
    (2, 2, 5, 5, 3, 3, 1, 4),      # pad > Sk - 1: some taps only ever see the apron
]


def outer_product_sum(inp, dout, Sk, stride, pad, alpha):
    """dfilt = alpha * sum over output pixels of (patch: Nc,Sk,Sk,Nb) . (gradient: No,Nb)^T; float64."""
    Nc, Hi, Wi, Nb = inp.shape
    No, Ho, Wo, _ = dout.shape
    big = np.zeros((Nc, Hi + 2 * pad, Wi + 2 * pad, Nb))
    big[:, pad:pad + Hi, pad:pad + Wi, :] = inp
    D = dout.astype(np.float64)
    acc = np.zeros((Nc, Sk, Sk, No))
    for y in range(Ho):
        for x in range(Wo):
            patch = big[:, y * stride:y * stride + Sk, x * stride:x * stride + Sk, :]
            acc += np.tensordot(patch, D[:, y, x, :], axes=([3], [1]))
    return alpha * acc


@pytest.mark.parametrize("Nb,Nc,Hi,Wi,No,Sk,stride,pad", CASES)
def test_matches_outer_product_sum(oracle_mod, Nb, Nc, Hi, Wi, No, Sk, stride, pad):
    rng = np.random.default_rng(600 + Nb + 7 * Sk + stride)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    dout = rng.uniform(-1, 1, size=(No, Ho, Wo, Nb)).astype(np.float32)
    got, absum = oracle_mod.conv_bprop_filter(inp, dout, Sk, stride, pad, 0.75)
    want = outer_product_sum(inp, dout, Sk, stride, pad, 0.75)
    assert got.shape == want.shape == (Nc, Sk, Sk, No)
    assert (np.abs(got.astype(np.float64) - want) <= 6e-8 * np.abs(want) + 1e-14 * absum + 1e-45).all()
    want_abs = outer_product_sum(np.abs(inp), np.abs(dout), Sk, stride, pad, 1.0)
    np.testing.assert_allclose(absum, want_abs, rtol=1e-12, atol=1e-300)


@pytest.mark.parametrize("Nb,Nc,Hi,Wi,No,Sk,stride,pad", CASES)
def test_is_the_adjoint_of_the_forward_oracle(oracle_mod, Nb, Nc, Hi, Wi, No, Sk, stride, pad):
    """<fprop(x, w), g> == <w, bprop_filter(x, g)> for integer data (both sides exact)."""
    rng = np.random.default_rng(700 + Nb + 3 * Sk + stride)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    x = rng.integers(-3, 4, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    g = rng.integers(-3, 4, size=(No, Ho, Wo, Nb)).astype(np.float32)
    w = rng.integers(-3, 4, size=(Nc, Sk, Sk, No)).astype(np.float32)
    y = oracle_mod.conv_fprop(x, w, stride, pad, 0.5, want_abs=False).astype(np.float64)
    dw = oracle_mod.conv_bprop_filter(x, g, Sk, stride, pad, 0.5, want_abs=False).astype(np.float64)
    assert float((y * g).sum()) == float((w * dw).sum())


def test_every_element_is_the_forward_response_to_a_basis_filter(oracle_mod):
    """With w = the basis filter e_k, <fprop(x, e_k), g> is element k of the gradient."""
    Nb, Nc, Hi, Wi, No, Sk, stride, pad = 2, 2, 7, 6, 3, 3, 2, 1
    rng = np.random.default_rng(31)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    x = rng.integers(-3, 4, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    g = rng.integers(-3, 4, size=(No, Ho, Wo, Nb)).astype(np.float32)
    dw = oracle_mod.conv_bprop_filter(x, g, Sk, stride, pad, 1.0, want_abs=False)
    for k in range(Nc * Sk * Sk * No):
        w = np.zeros(Nc * Sk * Sk * No, np.float32)
        w[k] = 1.0
        y = oracle_mod.conv_fprop(x, w.reshape(Nc, Sk, Sk, No), stride, pad, 1.0, want_abs=False)
        assert float((y.astype(np.float64) * g).sum()) == float(dw.reshape(-1)[k])


@pytest.mark.parametrize("Nb,Nc,Hi,Wi,No,Sk,stride,pad", CASES)
def test_matches_torch_autograd(oracle_mod, Nb, Nc, Hi, Wi, No, Sk, stride, pad):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(800 + Nb + 5 * Sk + stride)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    dout = rng.uniform(-1, 1, size=(No, Ho, Wo, Nb)).astype(np.float32)
    got = oracle_mod.conv_bprop_filter(inp, dout, Sk, stride, pad, 1.0, want_abs=False)
    x = torch.from_numpy(inp).permute(3, 0, 1, 2).double()               # (N, Nc, Hi, Wi)
    g = torch.from_numpy(dout).permute(3, 0, 1, 2).double()              # (N, No, Ho, Wo)
    w = torch.zeros(No, Nc, Sk, Sk, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.conv2d(x, w, stride=stride, padding=pad).backward(g)
    want = w.grad.permute(1, 2, 3, 0).numpy()                            # (Nc, Sk, Sk, No)
    np.testing.assert_allclose(got, want, rtol=3e-7, atol=1e-7)


def test_deltas_give_one_element(oracle_mod):
    Nb, Nc, Hi, Wi, No, Sk, stride, pad = 2, 3, 9, 8, 4, 3, 2, 1
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    for (c0, iy, ix, n0), (o0, y0, x0) in [((0, 0, 0, 0), (1, 0, 0)), ((2, 5, 4, 1), (3, 2, 2)),
                                           ((1, 8, 7, 0), (0, Ho - 1, Wo - 1)), ((1, 3, 3, 1), (2, 0, 0))]:
        inp = np.zeros((Nc, Hi, Wi, Nb), np.float32)
        inp[c0, iy, ix, n0] = 3.0
        dout = np.zeros((No, Ho, Wo, Nb), np.float32)
        dout[o0, y0, x0, n0] = 0.5
        got = oracle_mod.conv_bprop_filter(inp, dout, Sk, stride, pad, 2.0, want_abs=False)
        want = np.zeros_like(got)
        ky, kx = iy - (y0 * stride - pad), ix - (x0 * stride - pad)
        if 0 <= ky < Sk and 0 <= kx < Sk:
            want[c0, ky, kx, o0] = 3.0
        np.testing.assert_array_equal(got, want)
        # the same delta in another image of the batch never meets the gradient
        dout2 = np.zeros_like(dout)
        dout2[o0, y0, x0, 1 - n0] = 0.5
        assert not oracle_mod.conv_bprop_filter(inp, dout2, Sk, stride, pad, 2.0, want_abs=False).any()


def test_taps_that_only_see_the_apron_get_zero(oracle_mod):
    # 1x1 input, pad 1, one 3x3 window: only the centre tap ever meets the image
    inp = np.full((1, 1, 1, 2), 2.0, np.float32)
    dout = np.ones((2, 1, 1, 2), np.float32)
    got = oracle_mod.conv_bprop_filter(inp, dout, 3, 1, 1, 1.0, want_abs=False)
    want = np.zeros((1, 3, 3, 2), np.float32)
    want[0, 1, 1, :] = 4.0
    np.testing.assert_array_equal(got, want)


def test_points_agree_with_the_full_function(oracle_mod):
    Nb, Nc, Hi, Wi, No, Sk, stride, pad = 4, 3, 10, 9, 5, 3, 2, 1
    rng = np.random.default_rng(5)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    dout = rng.uniform(-1, 1, size=(No, Ho, Wo, Nb)).astype(np.float32)
    full, absum = oracle_mod.conv_bprop_filter(inp, dout, Sk, stride, pad, 1.5)
    idx = np.stack([rng.integers(0, Nc, 64), rng.integers(0, Sk, 64), rng.integers(0, Sk, 64),
                    rng.integers(0, No, 64)], axis=1).astype(np.int32)
    vals, ab = oracle_mod.conv_bprop_filter_points(inp, dout, idx, Sk, stride, pad, 1.5)
    np.testing.assert_array_equal(vals, full[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])
    np.testing.assert_array_equal(ab, absum[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])
    with pytest.raises(ValueError):
        oracle_mod.conv_bprop_filter_points(inp, dout, np.array([[Nc, 0, 0, 0]], np.int32), Sk, stride, pad, 1.0)


def test_rejects_mismatched_geometry(oracle_mod):
    with pytest.raises(ValueError):
        oracle_mod.conv_bprop_filter(np.zeros((1, 9, 9, 2), np.float32), np.zeros((2, 3, 3, 2), np.float32),
                                     3, 2, 0, 1.0)
    with pytest.raises(ValueError):
        oracle_mod.conv_bprop_filter(np.zeros((1, 9, 9, 2), np.float32), np.zeros((2, 4, 4, 3), np.float32),
                                     3, 2, 0, 1.0)


# ---- planted mistakes, in a copy of the source, on the CPU -------------------------------
SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "mdnn_oracle.c")
_ANCHOR = "int mdnn_oracle_conv_bprop_filter(const float* in"

MUTATIONS = {
    "tap_rows_cols_swapped":  ("size_t e = (((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o;",
                               "size_t e = (((size_t)c * Sk + kx) * Sk + ky) * (size_t)No + o;"),
    "filters_not_innermost":  ("size_t e = (((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o;",
                               "size_t e = (((size_t)o * Nc + c) * Sk + ky) * Sk + kx;"),
    "kernel_flipped":         ("int iy = y * stride - pad + ky;\n                        if (iy < 0 || iy >= Hi) continue;       /* zero apron */",
                               "int iy = y * stride - pad + (Sk - 1 - ky);\n                        if (iy < 0 || iy >= Hi) continue;"),
    "pad_dropped_in_x":       ("int ix = x * stride - pad + kx;\n                            if (ix < 0 || ix >= Wi) continue;\n                            const float* a",
                               "int ix = x * stride + kx;\n                            if (ix < 0 || ix >= Wi) continue;\n                            const float* a"),
    "stride_on_tap":          ("int iy = y * stride - pad + ky;\n                        if (iy < 0 || iy >= Hi) continue;       /* zero apron */",
                               "int iy = y - pad + ky * stride;\n                        if (iy < 0 || iy >= Hi) continue;"),
    "gradient_yx_swapped":    ("const float* g = dout + (((size_t)o * Ho + y) * Wo + x) * (size_t)Nb;\n                            for (int n = 0; n < Nb; ++n) {\n                                double p = (double)a[n] * (double)g[n];\n                                S += p;\n                                A += fabs(p);\n                            }\n                        }\n                    }\n                    size_t e",
                               "const float* g = dout + (((size_t)o * Wo + x) * Ho + y) * (size_t)Nb;\n                            for (int n = 0; n < Nb; ++n) {\n                                double p = (double)a[n] * (double)g[n];\n                                S += p;\n                                A += fabs(p);\n                            }\n                        }\n                    }\n                    size_t e"),
    "apron_clamped_not_zero": ("if (iy < 0 || iy >= Hi) continue;       /* zero apron */",
                               "if (iy < 0) iy = 0; if (iy >= Hi) iy = Hi - 1;"),
    "alpha_dropped":          ("dfilt[e] = (float)((double)alpha * S);", "dfilt[e] = (float)S;"),
    "batch_not_summed":       ("for (int n = 0; n < Nb; ++n) {\n                                double p = (double)a[n] * (double)g[n];\n                                S += p;\n                                A += fabs(p);\n                            }\n                        }\n                    }\n                    size_t e",
                               "for (int n = 0; n < 1; ++n) {\n                                double p = (double)a[n] * (double)g[n];\n                                S += p;\n                                A += fabs(p);\n                            }\n                        }\n                    }\n                    size_t e"),
}

_MUT_CASE = (3, 3, 9, 7, 4, 3, 2, 1, 0.75)    # Nb Nc Hi Wi No Sk stride pad alpha (Hi != Wi, Ho != Wo)


def _run_copy(so, inp, dout, Sk, stride, pad, alpha):
    lib = ctypes.CDLL(str(so))
    i, f, p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
    lib.mdnn_oracle_conv_bprop_filter.argtypes = [p, p, p, p, i, i, i, i, i, i, i, i, f, i]
    lib.mdnn_oracle_conv_bprop_filter.restype = i
    Nc, Hi, Wi, Nb = inp.shape
    No = dout.shape[0]
    out = np.full((Nc, Sk, Sk, No), np.nan, np.float32)
    assert lib.mdnn_oracle_conv_bprop_filter(inp.ctypes.data, dout.ctypes.data, out.ctypes.data, None,
                                             Nb, Wi, Hi, Nc, No, Sk, stride, pad, alpha, 1) == 0
    return out


def _mut_inputs(oracle_mod):
    Nb, Nc, Hi, Wi, No, Sk, stride, pad, alpha = _MUT_CASE
    rng = np.random.default_rng(78)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    assert Wo != Ho
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    dout = rng.uniform(-1, 1, size=(No, Ho, Wo, Nb)).astype(np.float32)
    return inp, dout, outer_product_sum(inp, dout, Sk, stride, pad, alpha).astype(np.float32)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, oracle_mod, name):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    head, body = text.split(_ANCHOR, 1)
    assert body.count(old) >= 1, f"mutation anchor for {name} no longer in the oracle source"
    c = tmp_path / "mut.c"
    so = tmp_path / "mut.so"
    c.write_text(head + _ANCHOR + body.replace(old, new, 1))
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    inp, dout, want = _mut_inputs(oracle_mod)
    got = _run_copy(so, inp, dout, _MUT_CASE[5], _MUT_CASE[6], _MUT_CASE[7], _MUT_CASE[8])
    assert not np.allclose(got, want, rtol=1e-5, atol=1e-6), f"the brute-force pin did not notice mutation {name}"


def test_unmutated_copy_passes(tmp_path, oracle_mod):
    so = tmp_path / "same.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(so), SRC, "-lm"], check=True)
    inp, dout, want = _mut_inputs(oracle_mod)
    got = _run_copy(so, inp, dout, _MUT_CASE[5], _MUT_CASE[6], _MUT_CASE[7], _MUT_CASE[8])
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=1e-6)
