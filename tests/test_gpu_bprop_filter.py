"""GPU parity of the filter gradient (BPROP w.r.t. the weights) against the
oracle, through the C ABI.  Same acceptance bound as the forward path: per
element |gpu - oracle| <= 1e-4 * |alpha| * A (A = sum of |products|), exactly 0
where A == 0, plus the 5e-6 regression bound; integer data bit for bit (every
partial sum is an integer below 2^24, so any summation order gives the same
fp32 result)."""
import sys

import numpy as np
import pytest

from paper_1501_06633_amd import workloads as W

pytestmark = pytest.mark.gpu

LOOSE, TIGHT = 1e-4, 5e-6


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1501_06633_amd import binding as B
    B.lib()
    import oracle
    oracle.build(force=False)
    return torch, B, oracle


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make_pair(layer, oracle, integer=False):
    """Seeded forward input and output gradient of the layer's shape."""
    Wo, Ho = oracle.out_dims(layer.Wi, layer.Hi, layer.Sk, layer.stride, layer.pad)
    rng = np.random.Generator(np.random.PCG64(layer.seed + 424243))
    shape = (layer.No, Ho, Wo, layer.Nb)
    if integer:
        inp, _ = W.make_int_inputs(layer)
        dout = rng.integers(-4, 5, size=shape).astype(np.float32)
    else:
        inp, _ = W.make_inputs(layer)
        dout = rng.standard_normal(size=shape, dtype=np.float32)
    return inp, dout


def run_gpu(env, layer, inp, dout, **kw):
    torch, B, _ = env
    out = B.mdnn_conv_bprop_filter(torch.from_numpy(inp).cuda(), torch.from_numpy(dout).cuda(),
                                   layer.Sk, layer.stride, layer.pad, layer.alpha, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check(got, want, absum, alpha, what):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    scale = abs(alpha) * absum
    zero = scale == 0
    assert (got[zero] == 0).all(), f"{what}: non-zero gradient where every product is zero"
    ratio = np.zeros_like(err)
    np.divide(err, scale, out=ratio, where=~zero)
    worst = float(ratio.max()) if ratio.size else 0.0
    say(f"    {what}: max |err|/(|alpha| A) = {worst:.3e} over {got.size} elements")
    assert np.isfinite(got).all()
    assert worst <= LOOSE and worst <= TIGHT, f"{what}: bound exceeded ({worst:.3e})"


@pytest.mark.parametrize("name", ["tiny", "conv1", "conv2", "conv3", "vgg"])
def test_layer_gradient_matches_oracle_everywhere(env, name):
    """The five benchmark layers at full size, every element of dfilt."""
    _, B, oracle = env
    L = W.LAYERS[name]
    say(f"[bprop-filter] layer={name} dims={L.dims()}")
    inp, dout = make_pair(L, oracle)
    got = run_gpu(env, L, inp, dout)
    want, absum = oracle.conv_bprop_filter(inp, dout, L.Sk, L.stride, L.pad, L.alpha)
    check(got, want, absum, L.alpha, name)


@pytest.mark.parametrize("name", ["conv1", "vgg"])
def test_layer_gradient_integer_bitwise(env, name):
    """Full-size contraction lengths (387200 and 200704 terms) with integer data: bit for bit."""
    _, B, oracle = env
    L = W.LAYERS[name]
    say(f"[bprop-filter-int] layer={name} dims={L.dims()}")
    inp, dout = make_pair(L, oracle, integer=True)
    got = run_gpu(env, L, inp, dout)
    want = oracle.conv_bprop_filter(inp, dout, L.Sk, L.stride, L.pad, L.alpha, want_abs=False)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("name", sorted(W.TABLE1))
def test_paper_table1_shapes_sampled(env, name):
    """The ten layer shapes of the paper's Table 1 at full size (minibatch 128): elements of dfilt
    sampled in every tile against the oracle's one-by-one evaluation.  K reaches
    9216 and No 1024 here (72 x 8 tiles), so the contraction is not cut at all for the largest."""
    _, B, oracle = env
    L, _ = W.TABLE1[name]
    st, need = B.mdnn_conv_bprop_filter_workspace(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    say(f"[bprop-filter-table1] layer={name} dims={L.dims()} ranges={need // (L.Nc * L.Sk * L.Sk * L.No * 4)}")
    inp, dout = make_pair(L, oracle)
    got = run_gpu(env, L, inp, dout)
    # dfilt seen as the K x No matrix the kernel tiles (128 rows by 128 / 96 / 64 / 32 columns): two
    # points in every 16 x 16 block, block corners included, so no tile goes without a sample
    K = L.Nc * L.Sk * L.Sk
    rc = W.stratified_points(K, L.No, 16, 16, 2, L.seed % 1000)
    k, o = rc[:, 0], rc[:, 1]
    idx = np.stack([k // (L.Sk * L.Sk), (k // L.Sk) % L.Sk, k % L.Sk, o], axis=1).astype(np.int32)
    say(f"    {idx.shape[0]} points")
    vals, absum = oracle.conv_bprop_filter_points(inp, dout, idx, L.Sk, L.stride, L.pad, L.alpha)
    c, ky, kx, o = idx.T
    check(got[c, ky, kx, o], vals, absum, L.alpha, name)


ODD = [
    # name             Nb  Hi  Wi  Nc  No  Sk st pad alpha
    ("ragged",         12, 11,  9,  5, 36, 3, 1, 1, 0.5),    # Nb % 4 == 0 only: 16-byte copies, per-lane walk
    ("scalar_path",     7, 10, 11,  3, 37, 3, 2, 1, 1.5),    # Nb odd: 4-byte copies
    ("scalar_nb1",      1, 23, 19,  6, 10, 5, 1, 2, 1.0),
    ("uniform_nb16",   16, 12, 10,  8, 24, 3, 2, 1, 0.5),    # Nb % 16 == 0: scalar walk over coordinates
    ("uniform_nb48",   48,  9,  7,  4, 20, 3, 1, 1, 1.0),
    ("stride3_nonsq",  20,  9, 14,  6, 40, 4, 3, 1, 0.25),
    ("stride_gt_sk",    8, 12,  9,  4,  8, 3, 4, 1, 1.0),
    ("one_by_one",     16,  6,  7, 40, 24, 1, 1, 0, -2.0),
    ("pad_gt_sk",       8,  5,  5,  3, 12, 3, 1, 4, 1.0),    # taps that only ever see the apron: exactly 0
    ("one_window",      4,  5,  5,  4,  8, 5, 1, 0, 1.0),    # a single output coordinate, one slab
    ("k_tiles",        32, 15, 13, 20, 200, 3, 1, 1, 1.0),   # K = 180 (two row tiles), two column tiles
    ("wide_k",         16,  8,  8, 40, 130, 5, 1, 2, 1.0),   # K = 1000, No just past one tile
    ("big_filter",     32, 24, 24,  3, 96, 11, 4, 0, 1.0),   # the first-layer shape in small
]


@pytest.mark.parametrize("case", ODD, ids=[c[0] for c in ODD])
def test_odd_shapes_integer_bitwise(env, case):
    _, B, oracle = env
    name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha = case
    L = W.custom(name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha, seed=W.SEED_BASE + 300 + len(name))
    say(f"[bprop-filter-odd] case={name} dims={L.dims()}")
    inp, dout = make_pair(L, oracle, integer=True)
    got = run_gpu(env, L, inp, dout)
    want = oracle.conv_bprop_filter(inp, dout, Sk, stride, pad, alpha, want_abs=False)
    np.testing.assert_array_equal(got, want)


def test_is_the_adjoint_of_the_gpu_forward(env):
    """<fprop(x, w), g> == <w, bprop_filter(x, g)> with both sides on the GPU, integer data (exact)."""
    torch, B, oracle = env
    L = W.custom("adjf", 16, 12, 10, 8, 24, 3, 2, 1, 0.5)
    x, w = W.make_int_inputs(L)
    _, g = make_pair(L, oracle, integer=True)
    d_x, d_w, d_g = (torch.from_numpy(a).cuda() for a in (x, w, g))
    y = B.mdnn_conv_fprop(d_x, d_w, L.stride, L.pad, L.alpha)
    dw = B.mdnn_conv_bprop_filter(d_x, d_g, L.Sk, L.stride, L.pad, L.alpha)
    torch.cuda.synchronize()
    assert float((y.double() * d_g.double()).sum()) == float((d_w.double() * dw.double()).sum())


def test_caller_workspace_overwrite_and_determinism(env):
    torch, B, oracle = env
    L = W.custom("wsf", 32, 20, 20, 12, 40, 3, 1, 1, 0.75)
    inp, dout = make_pair(L, oracle)
    st, need = B.mdnn_conv_bprop_filter_workspace(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    assert st == 0 and need >= L.Nc * L.Sk * L.Sk * L.No * 4
    ws = torch.full((need // 4 + 8,), float("nan"), device="cuda")          # garbage in, larger than needed
    dfilt = torch.full((L.Nc, L.Sk, L.Sk, L.No), float("nan"), device="cuda")
    d_in, d_g = torch.from_numpy(inp).cuda(), torch.from_numpy(dout).cuda()
    B.mdnn_conv_bprop_filter(d_in, d_g, L.Sk, L.stride, L.pad, L.alpha, dfilt=dfilt, workspace=ws)
    torch.cuda.synchronize()
    first = dfilt.cpu().numpy()
    want, absum = oracle.conv_bprop_filter(inp, dout, L.Sk, L.stride, L.pad, L.alpha)
    check(first, want, absum, L.alpha, "caller workspace")
    again = B.mdnn_conv_bprop_filter(d_in, d_g, L.Sk, L.stride, L.pad, L.alpha)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(again.cpu().numpy(), first)                # fixed summation order
    with pytest.raises(B.MdnnError):
        B.mdnn_conv_bprop_filter(d_in, d_g, L.Sk, L.stride, L.pad, L.alpha, workspace=ws[: need // 4 - 4])


def test_offsets_beyond_two_gib(env):
    """A forward input of 3.0 GiB: the patch gather of the filter gradient works with byte offsets
    above 2^31 and with apron origins that wrap around zero.  Sampled elements of dfilt, biased to
    the last channels and the border taps, against the oracle's one-by-one evaluation; integer
    data with a sparse gradient so that every partial sum stays exact."""
    torch, B, oracle = env
    Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha = 128, 64, 64, 1536, 8, 3, 1, 1, 1.0
    say(f"[bprop-filter-3gib] in bytes = {4 * Nb * Hi * Wi * Nc}")
    rng = np.random.default_rng(W.SEED_BASE + 78)
    inp = rng.integers(-2, 3, size=(Nc, Hi, Wi, Nb), dtype=np.int8).astype(np.float32)
    dout = (rng.integers(-2, 3, size=(No, Hi, Wi, Nb)) * (rng.random((No, Hi, Wi, Nb)) < 0.25)).astype(np.float32)
    d_in = torch.from_numpy(inp).cuda()
    got = B.mdnn_conv_bprop_filter(d_in, torch.from_numpy(dout).cuda(), Sk, stride, pad, alpha)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    del d_in
    npts = 1500
    idx = np.stack([rng.integers(0, Nc, npts), rng.integers(0, Sk, npts),
                    rng.integers(0, Sk, npts), rng.integers(0, No, npts)], axis=1).astype(np.int32)
    idx[:500, 0] = rng.integers(Nc - 40, Nc, 500)      # offsets above 2^31 ... 3 GiB
    idx[500:600, 0] = rng.integers(0, 2, 100)
    idx[0] = (0, 0, 0, 0)
    idx[1] = (Nc - 1, Sk - 1, Sk - 1, No - 1)
    vals, _ = oracle.conv_bprop_filter_points(inp, dout, idx, Sk, stride, pad, alpha)
    c, ky, kx, o = idx.T
    np.testing.assert_array_equal(got[c, ky, kx, o], vals)        # |sum| <= 4 * 524288 * 0.25 << 2^24: exact
    assert np.abs(vals).max() > 0
