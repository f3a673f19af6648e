"""CPU-only pins of the oracle against things other than itself.

The paper (arXiv 1501.06633) prints no worked numeric example, so the oracle is
pinned by what the definition in Section 2 and the matrix statement in
Section 3 fix: brute-force patch-matrix x filter-matrix products on physically
padded images, the 1x1 special case that is a plain matrix product, delta
filters, (bi)linearity, a closed form for constant data, translation, an
independent library routine in float64, the shapes of Table 1 and hand-worked
values of the complexity formula.
"""
import os

import numpy as np
import pytest

from paper_1501_06633_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------
# independent brute force: Section 3's statement executed literally
# --------------------------------------------------------------------------
def im2col_gemm(inp, filt, stride, pad, alpha):
    """For every output coordinate build the Nb x (Sk^2 Nc) unrolled patch of a
    physically zero-padded image and multiply it by the (Sk^2 Nc) x No filter
    matrix, all in float64.  Returns float64 (No, Ho, Wo, Nb)."""
    Nc, Hi, Wi, Nb = inp.shape
    _, Sk, _, No = filt.shape
    big = np.zeros((Nc, Hi + 2 * pad, Wi + 2 * pad, Nb), dtype=np.float64)
    big[:, pad:pad + Hi, pad:pad + Wi, :] = inp
    tops = list(range(0, Hi + 2 * pad - Sk + 1, stride))     # windows that fit
    lefts = list(range(0, Wi + 2 * pad - Sk + 1, stride))
    F = filt.astype(np.float64).reshape(Nc * Sk * Sk, No)     # one column per filter
    out = np.empty((No, len(tops), len(lefts), Nb), dtype=np.float64)
    for yi, t in enumerate(tops):
        for xi, l in enumerate(lefts):
            patch = big[:, t:t + Sk, l:l + Sk, :].reshape(Nc * Sk * Sk, Nb).T   # Nb x K
            out[:, yi, xi, :] = alpha * (patch @ F).T
    return out


def rand_case(rng, Nb, Nc, Hi, Wi, No, Sk):
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    filt = rng.uniform(-1, 1, size=(Nc, Sk, Sk, No)).astype(np.float32)
    return inp, filt


def ulps_f32(a, b):
    a = np.asarray(a, np.float32)
    b = np.asarray(b, np.float32)
    spacing = np.spacing(np.maximum(np.abs(a), np.abs(b)).astype(np.float32))
    return np.abs(a.astype(np.float64) - b.astype(np.float64)) / spacing


SMALL = [
    # Nb Nc Hi Wi No Sk stride pad
    (3, 2, 7, 6, 4, 3, 1, 1),
    (2, 3, 5, 7, 3, 1, 1, 0),
    (1, 1, 6, 6, 1, 2, 2, 0),
    (3, 3, 7, 7, 2, 5, 1, 2),
    (2, 2, 7, 5, 4, 3, 2, 1),
    (3, 1, 7, 7, 3, 3, 3, 2),
    (2, 3, 6, 7, 2, 2, 3, 1),
    (5, 2, 4, 9, 3, 3, 1, 2),
    (4, 3, 9, 4, 5, 4, 2, 2),
    (1, 2, 3, 3, 2, 3, 1, 0),   # single output coordinate
    (2, 1, 5, 5, 1, 5, 1, 2),   # filter as large as the image
    (2, 2, 8, 8, 3, 3, 2, 0),   # (8-3) not divisible by 2: trailing row/col unused
]


@pytest.mark.parametrize("Nb,Nc,Hi,Wi,No,Sk,stride,pad", SMALL)
def test_matches_im2col_gemm(oracle_mod, Nb, Nc, Hi, Wi, No, Sk, stride, pad):
    rng = np.random.default_rng(1000 + Nb * 7 + Sk * 13 + stride * 3 + pad)
    inp, filt = rand_case(rng, Nb, Nc, Hi, Wi, No, Sk)
    alpha = 0.75
    got, absum = oracle_mod.conv_fprop(inp, filt, stride, pad, alpha)
    want = im2col_gemm(inp, filt, stride, pad, alpha)
    assert got.shape == want.shape
    # both sides accumulate in double and round once: at most 1 ulp apart
    assert ulps_f32(got, want.astype(np.float32)).max() <= 1.0
    # the tolerance scale: sum of |products| = the same product with |.| data
    want_abs = im2col_gemm(np.abs(inp), np.abs(filt), stride, pad, 1.0)
    np.testing.assert_allclose(absum, want_abs, rtol=1e-12, atol=0)


def test_one_by_one_is_matmul(oracle_mod):
    rng = np.random.default_rng(11)
    Nb, Nc, Hi, Wi, No = 5, 7, 4, 6, 9
    inp, filt = rand_case(rng, Nb, Nc, Hi, Wi, No, 1)
    alpha = -1.5
    got = oracle_mod.conv_fprop(inp, filt, 1, 0, alpha, want_abs=False)
    F = filt.astype(np.float64).reshape(Nc, No)
    X = inp.astype(np.float64).reshape(Nc, Hi * Wi * Nb)
    want = (alpha * (F.T @ X)).reshape(No, Hi, Wi, Nb)
    assert ulps_f32(got, want.astype(np.float32)).max() <= 1.0


@pytest.mark.parametrize("stride,pad,Sk", [(1, 1, 3), (2, 2, 5), (1, 0, 3), (3, 1, 4), (1, 3, 4)])
def test_delta_filter_reproduces_shifted_input(oracle_mod, stride, pad, Sk):
    rng = np.random.default_rng(5 + stride + pad)
    Nb, Nc, Hi, Wi, No = 3, 4, 9, 8, 5
    inp = rng.uniform(-1, 1, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)
    for (c0, ky0, kx0, o0) in [(0, 0, 0, 0), (Nc - 1, Sk - 1, 0, 2), (1, 1, Sk - 1, No - 1),
                               (2, Sk - 1, Sk - 1, 3)]:
        filt = np.zeros((Nc, Sk, Sk, No), dtype=np.float32)
        filt[c0, ky0, kx0, o0] = 1.0
        alpha = 2.0     # power of two: exact
        got, absum = oracle_mod.conv_fprop(inp, filt, stride, pad, alpha)
        want = np.zeros((No, Ho, Wo, Nb), dtype=np.float32)
        in_apron = 0
        for y in range(Ho):
            for x in range(Wo):
                iy, ix = y * stride - pad + ky0, x * stride - pad + kx0
                if 0 <= iy < Hi and 0 <= ix < Wi:
                    want[o0, y, x, :] = alpha * inp[c0, iy, ix, :]
                else:
                    in_apron += 1
        np.testing.assert_array_equal(got, want)
        if pad > 0:
            assert in_apron > 0                    # the apron case was exercised
        others = np.delete(got, o0, axis=0)
        assert not others.any()
        assert not np.delete(absum, o0, axis=0).any()


def test_alpha_linearity_and_zero(oracle_mod):
    rng = np.random.default_rng(21)
    inp, filt = rand_case(rng, 4, 3, 8, 7, 5, 3)
    base = oracle_mod.conv_fprop(inp, filt, 1, 1, 1.0, want_abs=False).astype(np.float64)
    for alpha in (2.0, -0.5, 0.25, 4.0):        # powers of two: exact scaling
        got = oracle_mod.conv_fprop(inp, filt, 1, 1, alpha, want_abs=False)
        np.testing.assert_array_equal(got.astype(np.float64), alpha * base)
    for alpha in (0.3, -1.7):
        got = oracle_mod.conv_fprop(inp, filt, 1, 1, alpha, want_abs=False)
        a32 = float(np.float32(alpha))          # alpha crosses the interface as fp32
        # base and got are each rounded once, the product once more: three half-ulps
        assert ulps_f32(got, (a32 * base).astype(np.float32)).max() <= 2.5
    z = oracle_mod.conv_fprop(inp, filt, 1, 1, 0.0, want_abs=False)
    assert not z.any()


def test_additivity_in_both_operands(oracle_mod):
    rng = np.random.default_rng(31)
    # multiples of 1/64 in [-1,1): sums and products are exact in float32/float64
    q = lambda shape: (rng.integers(-64, 64, size=shape) / 64.0).astype(np.float32)
    a1, a2 = q((3, 7, 8, 4)), q((3, 7, 8, 4))
    f1, f2 = q((3, 3, 3, 5)), q((3, 3, 3, 5))
    conv = lambda a, f: oracle_mod.conv_fprop(a, f, 2, 1, 1.0, want_abs=False)
    np.testing.assert_array_equal(conv(a1 + a2, f1), conv(a1, f1) + conv(a2, f1))
    np.testing.assert_array_equal(conv(a1, f1 + f2), conv(a1, f1) + conv(a1, f2))


@pytest.mark.parametrize("stride,pad,Sk,Hi,Wi", [(1, 1, 3, 6, 7), (2, 2, 5, 9, 8), (4, 0, 11, 27, 23),
                                                  (1, 2, 3, 5, 5), (3, 1, 3, 10, 7)])
def test_all_ones_closed_form(oracle_mod, stride, pad, Sk, Hi, Wi):
    Nb, Nc, No = 3, 5, 4
    inp = np.ones((Nc, Hi, Wi, Nb), dtype=np.float32)
    filt = np.ones((Nc, Sk, Sk, No), dtype=np.float32)
    alpha = 0.5
    got, absum = oracle_mod.conv_fprop(inp, filt, stride, pad, alpha)
    Wo, Ho = oracle_mod.out_dims(Wi, Hi, Sk, stride, pad)

    def taps(pos, extent):      # filter taps that land inside the image
        return sum(1 for k in range(Sk) if 0 <= pos * stride - pad + k < extent)

    for y in range(Ho):
        for x in range(Wo):
            v = alpha * Nc * taps(y, Hi) * taps(x, Wi)
            assert (got[:, y, x, :] == np.float32(v)).all()
            assert (absum[:, y, x, :] == Nc * taps(y, Hi) * taps(x, Wi)).all()
    if pad == 0:
        assert (got == np.float32(alpha * Nc * Sk * Sk)).all()


def test_translation_shifts_output(oracle_mod):
    rng = np.random.default_rng(41)
    Nb, Nc, Hi, Wi, No, Sk, stride, pad = 2, 3, 12, 14, 3, 3, 2, 1
    inp, filt = rand_case(rng, Nb, Nc, Hi, Wi, No, Sk)
    moved = np.zeros_like(inp)
    moved[:, stride:, 2 * stride:, :] = inp[:, :-stride, :-2 * stride, :]   # down 1, right 2 outputs
    a = oracle_mod.conv_fprop(inp, filt, stride, pad, 1.0, want_abs=False)
    b = oracle_mod.conv_fprop(moved, filt, stride, pad, 1.0, want_abs=False)
    # away from the borders the output moves by (1, 2) output pixels, bit for bit
    np.testing.assert_array_equal(b[:, 2:-1, 3:-1, :], a[:, 1:-2, 1:-3, :])


@pytest.mark.parametrize("name,scale", [("tiny", 1), ("conv1", 8), ("conv2", 4), ("conv3", 2)])
def test_matches_torch_conv2d_float64(oracle_mod, name, scale):
    """Library special case: the operation is conv2d on (N,C,H,W) views.  The
    named layers are shrunk (batch, channels and image divided) to run fast."""
    torch = pytest.importorskip("torch")
    L = W.LAYERS[name]
    small = W.custom(name + "_small", max(1, L.Nb // (4 * scale)), max(L.Sk, L.Hi // scale),
                     max(L.Sk, L.Wi // scale + 1), max(1, L.Nc // scale), max(1, L.No // (2 * scale)),
                     L.Sk, L.stride, L.pad, L.alpha, L.in_dist, L.filt_dist, L.seed)
    inp, filt = W.make_inputs(small)
    got, absum = oracle_mod.conv_fprop(inp, filt, small.stride, small.pad, small.alpha)
    x = torch.from_numpy(inp).permute(3, 0, 1, 2).double()
    w = torch.from_numpy(filt).permute(3, 0, 1, 2).double()
    want = small.alpha * torch.nn.functional.conv2d(x, w, stride=small.stride, padding=small.pad)
    want = want.permute(1, 2, 3, 0).numpy()
    assert got.shape == want.shape
    err = np.abs(got.astype(np.float64) - want)
    # one fp32 rounding of a double sum: half an ulp of |value|, plus double noise on the sum
    assert (err <= 6.0e-8 * np.abs(want) + 1e-13 * absum + 1e-45).all()
    want_abs = torch.nn.functional.conv2d(x.abs(), w.abs(), stride=small.stride,
                                          padding=small.pad).permute(1, 2, 3, 0).numpy()
    np.testing.assert_allclose(absum, want_abs, rtol=1e-11)


def test_exact_integer_data_is_order_independent(oracle_mod):
    """With small-integer data every partial sum is an exact integer, so the
    brute force (different summation order, physical padding) must agree bit
    for bit -- the same property the GPU parity tests rely on."""
    L = W.custom("ints", 4, 9, 10, 6, 5, 3, 2, 1, alpha=0.5)
    inp, filt = W.make_int_inputs(L)
    got = oracle_mod.conv_fprop(inp, filt, L.stride, L.pad, L.alpha, want_abs=False)
    want = im2col_gemm(inp, filt, L.stride, L.pad, L.alpha).astype(np.float32)
    np.testing.assert_array_equal(got, want)


def test_points_entry_matches_brute_force_and_full(oracle_mod):
    rng = np.random.default_rng(51)
    Nb, Nc, Hi, Wi, No, Sk, stride, pad = 4, 3, 9, 7, 5, 3, 2, 1
    inp, filt = rand_case(rng, Nb, Nc, Hi, Wi, No, Sk)
    alpha = 1.25
    full, fabs = oracle_mod.conv_fprop(inp, filt, stride, pad, alpha)
    brute = im2col_gemm(inp, filt, stride, pad, alpha)
    No_, Ho, Wo, _ = full.shape
    idx = np.stack([rng.integers(0, No_, 200), rng.integers(0, Ho, 200),
                    rng.integers(0, Wo, 200), rng.integers(0, Nb, 200)], axis=1).astype(np.int32)
    idx[0] = (0, 0, 0, 0)
    idx[1] = (No_ - 1, Ho - 1, Wo - 1, Nb - 1)
    vals, ab = oracle_mod.conv_fprop_points(inp, filt, idx, stride, pad, alpha)
    o, y, x, n = idx.T
    assert ulps_f32(vals, brute[o, y, x, n].astype(np.float32)).max() <= 1.0
    np.testing.assert_array_equal(vals, full[o, y, x, n])
    np.testing.assert_allclose(ab, fabs[o, y, x, n], rtol=1e-13)
    with pytest.raises(ValueError):
        oracle_mod.conv_fprop_points(inp, filt, np.array([[No_, 0, 0, 0]], np.int32), stride, pad, alpha)


def test_table1_output_sizes(oracle_mod):
    rows = 0
    with open(os.path.join(GOLDEN, "table1_shapes.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            _, _, Wi, _, Wo, _, Sk, stride, pad = line.split()
            Wi, Wo, Sk, stride, pad = map(int, (Wi, Wo, Sk, stride, pad))
            assert oracle_mod.out_dims(Wi, Wi, Sk, stride, pad) == (Wo, Wo), line
            rows += 1
    assert rows == 10


def test_out_dims_non_square_and_errors(oracle_mod):
    assert oracle_mod.out_dims(7, 5, 3, 1, 0) == (5, 3)          # (Wo, Ho)
    assert oracle_mod.out_dims(8, 8, 3, 2, 0) == (3, 3)          # floor: last column unused
    assert oracle_mod.out_dims(5, 5, 5, 1, 0) == (1, 1)
    assert oracle_mod.out_dims(227, 227, 11, 4, 0) == (55, 55)
    for bad in [(5, 5, 6, 1, 0), (0, 5, 1, 1, 0), (5, 5, 3, 0, 0), (5, 5, 3, 1, -1)]:
        with pytest.raises(ValueError):
            oracle_mod.out_dims(*bad)


def test_complexity_formula_values(oracle_mod):
    rows = 0
    with open(os.path.join(GOLDEN, "flops_values.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            Nb, Wo, Ho, Nc, No, Sk, C = map(int, line.split())
            assert oracle_mod.flops(Nb, Wo, Ho, Nc, No, Sk) == C, line
            rows += 1
    assert rows == 8
    # proportional to Nb and to No; the "+1" term is the alpha scale per output
    assert oracle_mod.flops(6, 3, 5, 7, 11, 2) == 3 * oracle_mod.flops(2, 3, 5, 7, 11, 2)
    assert oracle_mod.flops(2, 3, 5, 7, 22, 2) == 2 * oracle_mod.flops(2, 3, 5, 7, 11, 2)


def test_rejects_bad_arguments(oracle_mod):
    inp = np.zeros((2, 4, 4, 3), np.float32)
    filt = np.zeros((2, 5, 5, 2), np.float32)
    with pytest.raises(ValueError):
        oracle_mod.conv_fprop(inp, filt, 1, 0, 1.0)             # filter larger than image
    with pytest.raises(ValueError):
        oracle_mod.conv_fprop(inp, np.zeros((3, 3, 3, 2), np.float32), 1, 0, 1.0)   # channel mismatch
    with pytest.raises(ValueError):
        oracle_mod.conv_fprop(inp.astype(np.float64), filt, 1, 2, 1.0)


def test_thread_count_does_not_change_result(oracle_mod):
    L = W.custom("t", 4, 10, 9, 5, 6, 3, 1, 1)
    inp, filt = W.make_inputs(L)
    a = oracle_mod.conv_fprop(inp, filt, 1, 1, 1.0, want_abs=False, nthreads=1)
    b = oracle_mod.conv_fprop(inp, filt, 1, 1, 1.0, want_abs=False, nthreads=3)
    np.testing.assert_array_equal(a, b)
