"""CPU-only pins of the oracle's data-gradient function (BPROP w.r.t. the input).

The paper (arXiv 1501.06633, abstract and Section 3.5) only states the belief
that the same techniques carry over to BPROP, so there is nothing printed to
compare with; the function is pinned by what defines a gradient: it is the
adjoint of the (already pinned) forward map, it equals a scatter-add of every
forward term, it equals the library's transposed convolution in float64, and a
delta in dout reproduces the filter.
"""
import numpy as np
import pytest

CASES = [
    # Nb Nc Hi Wi No Sk stride pad
    (3, 2, 7, 6, 4, 3, 1, 1),
    (2, 3, 5, 7, 3, 1, 1, 0),
    (2, 2, 8, 8, 3, 3, 2, 0),      # (8-3) % 2 != 0: last input row/col never read -> gradient 0 there
    (3, 3, 9, 7, 2, 5, 2, 2),
    (2, 1, 10, 11, 3, 4, 3, 1),
    (4, 2, 6, 6, 3, 3, 1, 2),      # pad = Sk - 1
    (1, 2, 11, 11, 2, 11, 4, 0),   # one window
    (2, 3, 12, 9, 4, 3, 4, 1),     # stride larger than the filter: gaps in the gradient
    (2, 2, 5, 6, 3, 3, 1, 3),      # pad = Sk: the outermost windows lie wholly in the apron
    (3, 2, 4, 4, 2, 1, 1, 2),      # 1x1 filter with an apron of two
    (2, 2, 7, 7, 3, 2, 2, 3),      # strided, pad > Sk - 1
]


def scatter_add(dout, filt, in_hw, stride, pad, alpha):
    """Every forward term out[o,y,x,n] += in[c,y*s-p+ky,x*s-p+kx,n] * filt[c,ky,kx,o]
    gives din[c,y*s-p+ky,x*s-p+kx,n] += dout[o,y,x,n] * filt[c,ky,kx,o]; float64."""
    No, Ho, Wo, Nb = dout.shape
    Nc, Sk, _, _ = filt.shape
    Hi, Wi = in_hw
    big = np.zeros((Nc, Hi + 2 * pad, Wi + 2 * pad, Nb))
    F = filt.astype(np.float64)
    D = dout.astype(np.float64)
    for y in range(Ho):
        for x in range(Wo):
            # (Nc,Sk,Sk,No) . (No,Nb) -> (Nc,Sk,Sk,Nb)
            big[:, y * stride:y * stride + Sk, x * stride:x * stride + Sk, :] += np.tensordot(F, D[:, y, x, :], axes=([3], [0]))
    return alpha * big[:, pad:pad + Hi, pad:pad + Wi, :]


def ulps_f32(a, b):
    a = np.asarray(a, np.float32)
    b = np.asarray(b, np.float32)
    spacing = np.spacing(np.maximum(np.abs(a), np.abs(b)).astype(np.float32))
    return np.abs(a.astype(np.float64) - b.astype(np.float64)) / spacing


@pytest.mark.parametrize("Nb,Nc,Hi,Wi,No,Sk,stride,pad", CASES)
def test_matches_scatter_add(oracle_mod, Nb, Nc, Hi, Wi, No, Sk, stride, pad):
    rng = np.random.default_rng(300 + Nb + 7 * Sk + stride)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    dout = rng.uniform(-1, 1, size=(No, Ho, Wo, Nb)).astype(np.float32)
    filt = rng.uniform(-1, 1, size=(Nc, Sk, Sk, No)).astype(np.float32)
    got, absum = oracle_mod.conv_bprop_data(dout, filt, (Hi, Wi), stride, pad, 0.75)
    want = scatter_add(dout, filt, (Hi, Wi), stride, pad, 0.75)
    assert got.shape == want.shape == (Nc, Hi, Wi, Nb)
    # double sums in different orders, one fp32 rounding each: a few 1e-16 relative to the abs sum
    assert (np.abs(got.astype(np.float64) - want) <= 6e-8 * np.abs(want) + 1e-14 * absum + 1e-45).all()
    want_abs = scatter_add(np.abs(dout), np.abs(filt), (Hi, Wi), stride, pad, 1.0)
    np.testing.assert_allclose(absum, want_abs, rtol=1e-12, atol=1e-300)


@pytest.mark.parametrize("Nb,Nc,Hi,Wi,No,Sk,stride,pad", CASES)
def test_is_the_adjoint_of_the_forward_oracle(oracle_mod, Nb, Nc, Hi, Wi, No, Sk, stride, pad):
    """<fprop(x), g> == <x, bprop_data(g)> for integer data (both sides exact)."""
    rng = np.random.default_rng(400 + Nb + 3 * Sk + stride)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    x = rng.integers(-3, 4, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    g = rng.integers(-3, 4, size=(No, Ho, Wo, Nb)).astype(np.float32)
    filt = rng.integers(-3, 4, size=(Nc, Sk, Sk, No)).astype(np.float32)
    y = oracle_mod.conv_fprop(x, filt, stride, pad, 0.5, want_abs=False).astype(np.float64)
    dx = oracle_mod.conv_bprop_data(g, filt, (Hi, Wi), stride, pad, 0.5, want_abs=False).astype(np.float64)
    assert float((y * g).sum()) == float((x * dx).sum())


@pytest.mark.parametrize("Nb,Nc,Hi,Wi,No,Sk,stride,pad", CASES)
def test_matches_torch_transposed_convolution(oracle_mod, Nb, Nc, Hi, Wi, No, Sk, stride, pad):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(500 + Nb + 5 * Sk + stride)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    dout = rng.uniform(-1, 1, size=(No, Ho, Wo, Nb)).astype(np.float32)
    filt = rng.uniform(-1, 1, size=(Nc, Sk, Sk, No)).astype(np.float32)
    got = oracle_mod.conv_bprop_data(dout, filt, (Hi, Wi), stride, pad, 1.0, want_abs=False)
    g = torch.from_numpy(dout).permute(3, 0, 1, 2).double()              # (N, No, Ho, Wo)
    w = torch.from_numpy(filt).permute(3, 0, 1, 2).double()              # (No, Nc, Sk, Sk)
    oph = Hi - ((Ho - 1) * stride - 2 * pad + Sk)
    opw = Wi - ((Wo - 1) * stride - 2 * pad + Sk)
    want = torch.nn.functional.conv_transpose2d(g, w, stride=stride, padding=pad, output_padding=(oph, opw))
    want = want.permute(1, 2, 3, 0).numpy()                              # (Nc, Hi, Wi, N)
    assert want.shape == got.shape
    np.testing.assert_allclose(got, want, rtol=3e-7, atol=1e-7)


def test_delta_gradient_reproduces_the_filter(oracle_mod):
    Nb, Nc, Hi, Wi, No, Sk, stride, pad = 2, 3, 9, 8, 4, 3, 2, 1
    rng = np.random.default_rng(9)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    filt = rng.uniform(-1, 1, size=(Nc, Sk, Sk, No)).astype(np.float32)
    for (o0, y0, x0, n0) in [(0, 0, 0, 0), (3, Ho - 1, Wo - 1, 1), (2, 1, 2, 0)]:
        dout = np.zeros((No, Ho, Wo, Nb), np.float32)
        dout[o0, y0, x0, n0] = 1.0
        got = oracle_mod.conv_bprop_data(dout, filt, (Hi, Wi), stride, pad, 2.0, want_abs=False)
        want = np.zeros_like(got)
        for ky in range(Sk):
            for kx in range(Sk):
                iy, ix = y0 * stride - pad + ky, x0 * stride - pad + kx
                if 0 <= iy < Hi and 0 <= ix < Wi:
                    want[:, iy, ix, n0] = 2.0 * filt[:, ky, kx, o0]
        np.testing.assert_array_equal(got, want)


def test_unreached_input_pixels_get_zero(oracle_mod):
    # 8 wide, 3x3 stride 2 pad 0: windows cover columns 0..6, column 7 is never read
    dout = np.ones((2, 3, 3, 2), np.float32)
    filt = np.ones((1, 3, 3, 2), np.float32)
    got = oracle_mod.conv_bprop_data(dout, filt, (8, 8), 2, 0, 1.0, want_abs=False)
    assert not got[:, 7, :, :].any() and not got[:, :, 7, :].any()
    assert got[0, 0, 0, 0] == 2.0 and got[0, 2, 2, 0] == 8.0     # corner: 1 window x 2 filters; overlap of 4 windows


def test_rejects_mismatched_geometry(oracle_mod):
    with pytest.raises(ValueError):
        oracle_mod.conv_bprop_data(np.zeros((2, 3, 3, 2), np.float32), np.zeros((1, 3, 3, 2), np.float32),
                                   (9, 9), 2, 0, 1.0)


def test_points_agree_with_the_full_function(oracle_mod):
    Nb, Nc, Hi, Wi, No, Sk, stride, pad = 4, 3, 10, 9, 5, 3, 2, 1
    rng = np.random.default_rng(6)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    dout = rng.uniform(-1, 1, size=(No, Ho, Wo, Nb)).astype(np.float32)
    filt = rng.uniform(-1, 1, size=(Nc, Sk, Sk, No)).astype(np.float32)
    full, absum = oracle_mod.conv_bprop_data(dout, filt, (Hi, Wi), stride, pad, 1.5)
    idx = np.stack([rng.integers(0, Nc, 200), rng.integers(0, Hi, 200), rng.integers(0, Wi, 200),
                    rng.integers(0, Nb, 200)], axis=1).astype(np.int32)
    vals, ab = oracle_mod.conv_bprop_data_points(dout, filt, idx, (Hi, Wi), stride, pad, 1.5)
    np.testing.assert_array_equal(vals, full[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])
    np.testing.assert_array_equal(ab, absum[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])
    with pytest.raises(ValueError):
        oracle_mod.conv_bprop_data_points(dout, filt, np.array([[0, Hi, 0, 0]], np.int32), (Hi, Wi), stride, pad, 1.0)
