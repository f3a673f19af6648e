"""GPU parity of the data gradient (BPROP w.r.t. the input) against the oracle,
through the C ABI.  Same acceptance bound as the forward path: per element
|gpu - oracle| <= 1e-4 * |alpha| * A (A = sum of |products|), exactly 0 where
A == 0, plus the 5e-6 regression bound; integer data bit for bit."""
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


def make_grad(layer, oracle, integer=False):
    """Seeded output gradient of the layer's forward shape, and its filters."""
    Wo, Ho = oracle.out_dims(layer.Wi, layer.Hi, layer.Sk, layer.stride, layer.pad)
    rng = np.random.Generator(np.random.PCG64(layer.seed + 31337))
    shape = (layer.No, Ho, Wo, layer.Nb)
    if integer:
        dout = rng.integers(-4, 5, size=shape).astype(np.float32)
        filt = rng.integers(-4, 5, size=(layer.Nc, layer.Sk, layer.Sk, layer.No)).astype(np.float32)
    else:
        dout = rng.standard_normal(size=shape, dtype=np.float32)
        _, filt = W.make_inputs(layer)
    return dout, filt


def run_gpu(env, layer, dout, filt):
    torch, B, _ = env
    out = B.mdnn_conv_bprop_data(torch.from_numpy(dout).cuda(), torch.from_numpy(filt).cuda(),
                                 (layer.Hi, layer.Wi), layer.stride, layer.pad, layer.alpha)
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


@pytest.mark.parametrize("name", ["tiny", "conv2", "conv3", "vgg"])
def test_layer_gradient_matches_oracle_everywhere(env, name):
    """Stride-1 layers at full size, every element of din."""
    _, B, oracle = env
    L = W.LAYERS[name]
    say(f"[bprop] layer={name} dims={L.dims()}")
    dout, filt = make_grad(L, oracle)
    got = run_gpu(env, L, dout, filt)
    want, absum = oracle.conv_bprop_data(dout, filt, (L.Hi, L.Wi), L.stride, L.pad, L.alpha)
    check(got, want, absum, L.alpha, name)


def test_strided_first_layer_gradient(env):
    """conv1 (stride 4, 11x11): the gradient goes through the residue-class path; whole tensor."""
    _, B, oracle = env
    L = W.LAYERS["conv1"]
    say(f"[bprop] layer=conv1 dims={L.dims()}")
    dout, filt = make_grad(L, oracle)
    got = run_gpu(env, L, dout, filt)
    want, absum = oracle.conv_bprop_data(dout, filt, (L.Hi, L.Wi), L.stride, L.pad, L.alpha)
    check(got, want, absum, L.alpha, "conv1")


@pytest.mark.parametrize("name", sorted(W.TABLE1))
def test_paper_table1_shapes_sampled(env, name):
    """The ten layer shapes of the paper's Table 1 at full size (minibatch 128): elements of din
    sampled in every tile against the oracle's one-by-one evaluation.  The two first layers
    (stride 4) go through the residue-class path."""
    _, B, oracle = env
    L, _ = W.TABLE1[name]
    say(f"[bprop-table1] layer={name} dims={L.dims()}")
    dout, filt = make_grad(L, oracle)
    got = run_gpu(env, L, dout, filt)
    # din seen as the Nc x (Hi*Wi*Nb) matrix the kernels tile: two points in every 16-row by
    # 64-column block, block corners included -- no tile or tail piece of any tile shape (the
    # narrowest is 32 rows by 128 columns; the strided layers pass through a gather that works
    # on 4-column groups) is left without a sample
    idx = W.output_points((L.Nc, L.Nb), L.Hi, L.Wi, 16, 64, 2, L.seed % 1000)
    say(f"    {idx.shape[0]} points")
    vals, absum = oracle.conv_bprop_data_points(dout, filt, idx, (L.Hi, L.Wi), L.stride, L.pad, L.alpha)
    c, iy, ix, n = idx.T
    check(got[c, iy, ix, n], vals, absum, L.alpha, name)


ODD = [
    # name             Nb  Hi  Wi  Nc  No  Sk st pad alpha
    ("ragged",         12, 11,  9,  5, 36, 3, 1, 1, 0.5),
    ("scalar_path",     7, 10, 11,  3, 37, 3, 2, 1, 1.5),    # Nb, No, Nc not multiples of 4
    ("stride2_unread",  8,  8,  8,  4, 12, 3, 2, 0, 1.0),    # last row / column never read: gradient 0
    ("stride3_nonsq",  20,  9, 14,  6, 40, 4, 3, 1, 0.25),
    ("stride_gt_sk",    8, 12,  9,  4,  8, 3, 4, 1, 1.0),    # gaps between windows
    ("one_by_one",     16,  6,  7, 40, 24, 1, 1, 0, -2.0),
    ("pad_max",         8,  6,  6,  3, 12, 3, 1, 2, 1.0),    # pad = Sk - 1
    ("one_window",      4,  5,  5,  4,  8, 5, 1, 0, 1.0),
    ("many_tiles",     32, 15, 13, 20, 200, 3, 1, 1, 1.0),
    ("s2_5x5_pad2",    16, 13, 11,  6, 20, 5, 2, 2, 1.0),    # T = 3, classes with 9 / 6 / 4 real taps
    ("s2_4x4",          8, 10, 12,  5, 16, 4, 2, 1, 0.5),    # T = 2, every class full
    ("s3_7x7_pad3",     8, 17, 15,  4, 12, 7, 3, 3, 1.0),
    ("s2_odd_batch",    5,  9,  9,  3, 10, 3, 2, 1, 1.0),    # 4-byte gather
    ("s5_3x3_pad2",     8, 14, 14,  4,  8, 3, 5, 2, 1.0),    # most classes have no tap at all
    ("s2_one_window",   4,  6,  6,  3,  8, 6, 2, 0, 1.0),
    ("pad_eq_sk",       8,  7,  9,  4, 12, 3, 1, 3, 1.0),    # stride 1, pad > Sk - 1: the general path with one class
    ("pad_gt_sk_1x1",   4,  5,  5,  3,  8, 1, 1, 2, 0.5),    # 1x1 filter with an apron of two
    ("s2_pad_gt_sk",    8,  8,  8,  4,  8, 2, 2, 3, 1.0),    # strided with pad > Sk - 1
]


@pytest.mark.parametrize("case", ODD, ids=[c[0] for c in ODD])
def test_odd_shapes_integer_bitwise(env, case):
    _, B, oracle = env
    name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha = case
    L = W.custom(name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha, seed=W.SEED_BASE + 200 + len(name))
    say(f"[bprop-odd] case={name} dims={L.dims()}")
    dout, filt = make_grad(L, oracle, integer=True)
    got = run_gpu(env, L, dout, filt)
    want = oracle.conv_bprop_data(dout, filt, (Hi, Wi), stride, pad, alpha, want_abs=False)
    np.testing.assert_array_equal(got, want)


def test_is_the_adjoint_of_the_gpu_forward(env):
    """<fprop(x), g> == <x, bprop_data(g)> with both sides on the GPU, integer data (exact)."""
    torch, B, oracle = env
    L = W.custom("adj", 16, 12, 10, 8, 24, 3, 2, 1, 0.5)
    x, filt = W.make_int_inputs(L)
    g, _ = make_grad(L, oracle, integer=True)
    d_x, d_f, d_g = (torch.from_numpy(a).cuda() for a in (x, filt, g))
    y = B.mdnn_conv_fprop(d_x, d_f, L.stride, L.pad, L.alpha)
    dx = B.mdnn_conv_bprop_data(d_g, d_f, (L.Hi, L.Wi), L.stride, L.pad, L.alpha)
    torch.cuda.synchronize()
    assert float((y.double() * d_g.double()).sum()) == float((d_x.double() * dx.double()).sum())


def test_caller_workspace_and_overwrite(env):
    torch, B, oracle = env
    L = W.custom("ws", 8, 9, 9, 4, 16, 3, 2, 1, 1.0)
    dout, filt = make_grad(L, oracle, integer=True)
    st, need = B.mdnn_conv_bprop_data_workspace(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    assert st == 0
    ws = torch.full((need // 4 + 8,), float("nan"), device="cuda")          # garbage in, larger than needed
    din = torch.full((L.Nc, L.Hi, L.Wi, L.Nb), float("nan"), device="cuda")
    B.mdnn_conv_bprop_data(torch.from_numpy(dout).cuda(), torch.from_numpy(filt).cuda(), (L.Hi, L.Wi),
                           L.stride, L.pad, L.alpha, din=din, workspace=ws)
    torch.cuda.synchronize()
    want = oracle.conv_bprop_data(dout, filt, (L.Hi, L.Wi), L.stride, L.pad, L.alpha, want_abs=False)
    np.testing.assert_array_equal(din.cpu().numpy(), want)


def test_result_beyond_two_gib(env):
    """A data gradient of 3.0 GiB: the stores of the forward kernel it runs on reach byte offsets
    above 2^31.  Sampled elements, biased to the last channels and the border, against the
    oracle's one-by-one evaluation; integer data, exact."""
    torch, B, oracle = env
    Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha = 128, 64, 64, 1536, 8, 3, 1, 1, 0.5
    say(f"[bprop-3gib] din bytes = {4 * Nb * Hi * Wi * Nc}")
    rng = np.random.default_rng(W.SEED_BASE + 79)
    dout = rng.integers(-3, 4, size=(No, Hi, Wi, Nb)).astype(np.float32)
    filt = rng.integers(-3, 4, size=(Nc, Sk, Sk, No)).astype(np.float32)
    got = B.mdnn_conv_bprop_data(torch.from_numpy(dout).cuda(), torch.from_numpy(filt).cuda(), (Hi, Wi),
                                 stride, pad, alpha)
    torch.cuda.synchronize()
    npts = 20000
    idx = np.stack([rng.integers(0, Nc, npts), rng.integers(0, Hi, npts),
                    rng.integers(0, Wi, npts), rng.integers(0, Nb, npts)], axis=1).astype(np.int32)
    idx[:5000, 0] = rng.integers(Nc - 40, Nc, 5000)
    idx[5000:6000, 1] = rng.choice([0, Hi - 1], 1000)
    idx[6000:7000, 2] = rng.choice([0, Wi - 1], 1000)
    idx[0] = (0, 0, 0, 0)
    idx[1] = (Nc - 1, Hi - 1, Wi - 1, Nb - 1)
    t = torch.from_numpy(idx.astype(np.int64)).cuda()
    sampled = got[t[:, 0], t[:, 1], t[:, 2], t[:, 3]].cpu().numpy()
    del got
    vals, _ = oracle.conv_bprop_data_points(dout, filt, idx, (Hi, Wi), stride, pad, alpha)
    np.testing.assert_array_equal(sampled, vals)
    assert np.abs(vals).max() > 0


# Stride-2 3x3 layers with 32 input channels: the residue-class problem has 4 * 32 = 128 filters of
# 2 x 2 taps and one 128-column tile per pixel of the (Ho + 1) x (Wo + 1) class grid at minibatch
# 128, so the tile count -- and with it the tail cut of the scattering kernel -- is (Ho + 1)(Wo + 1).
SCATTER_TAILS = [
    # Ho  Wo  what the plan of the class problem must contain
    (13, 19, dict(tiles=280, eighthed=24)),                     # eighths beside one round
    (12, 25, dict(tiles=338, thirded=82)),                      # thirds
    (14, 22, dict(tiles=345, quartered=64, eighthed=25)),       # a quarter and an eighth per unit
    (13, 27, dict(tiles=392, halved=128, eighthed=8)),          # a half and an eighth per unit
    (19, 26, dict(tiles=540, whole=512, eighthed=28)),          # eighths in front of two rounds
]


@pytest.mark.parametrize("Ho,Wo,want", SCATTER_TAILS, ids=[f"{c[2]['tiles']}_tiles" for c in SCATTER_TAILS])
def test_scattering_epilogue_in_every_tail_piece_bitwise(env, Ho, Wo, want):
    """The strided data gradient scatters straight from the accumulators into din; when the class
    problem's last round of tiles is cut, the half, third, quarter and eighth bodies do the
    scattering.  Integer data, whole tensor, bit for bit."""
    torch, B, oracle = env
    Nb, Nc, No, Sk, stride, pad, alpha = 128, 32, 4, 3, 2, 0, 0.5
    Hi, Wi = 2 * Ho + 1, 2 * Wo + 1
    assert oracle.out_dims(Wi, Hi, Sk, stride, pad) == (Wo, Ho)
    plan = B.mdnn_describe_launch(Nb, Wo, Ho, No, stride * stride * Nc, 2, 1, 1)    # the class problem, as the library plans it
    say(f"[bprop-scatter-tails] Ho={Ho} Wo={Wo} plan={plan}")
    for k, v in want.items():
        assert plan[k] == v, (k, plan)
    rng = np.random.default_rng(500 + Ho * Wo)
    dout = rng.integers(-4, 5, size=(No, Ho, Wo, Nb)).astype(np.float32)
    filt = rng.integers(-4, 5, size=(Nc, Sk, Sk, No)).astype(np.float32)
    got = B.mdnn_conv_bprop_data(torch.from_numpy(dout).cuda(), torch.from_numpy(filt).cuda(), (Hi, Wi), stride, pad, alpha)
    torch.cuda.synchronize()
    wanted = oracle.conv_bprop_data(dout, filt, (Hi, Wi), stride, pad, alpha, want_abs=False)
    np.testing.assert_array_equal(got.cpu().numpy(), wanted)
