"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.

Acceptance bound (per output):  |gpu - oracle| <= 1e-4 * |alpha| * A  where A
is the sum of |in * filt| over the taps of that output (the oracle returns it);
where A == 0 the GPU value must be exactly zero.  A much tighter regression
bound (TIGHT) is asserted as well: fp32 accumulation over K <= 2400 terms sits
near 1e-6 * A, and a silent drop to a reduced-precision matrix format (~1e-3
per product) would pass the loose bound at these K but not the tight one.
Integer-valued inputs must match bit for bit (every partial sum is exact in
fp32, so no summation order can change the result).
"""
import sys

import numpy as np
import pytest

from paper_1501_06633_amd import workloads as W

pytestmark = pytest.mark.gpu

LOOSE = 1e-4
TIGHT = 5e-6


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1501_06633_amd import binding as B
    B.lib()                                    # fail loudly if the HIP library is missing
    import oracle
    oracle.build(force=False)
    return torch, B, oracle


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def tile_points(B, L, shape, seed):
    """(o, y, x, n) rows covering the launch grid of layer L without a gap: at least two outputs --
    first and last element among them -- in every 16-row by half-tile-wide block of the No x M
    output, hence in every workgroup tile, in every piece a tile of the last round may be cut into
    (halves, 48- and 32-row thirds, quarters, column halves) and in the ragged tiles at the edges."""
    plan = B.mdnn_describe_launch(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    to, tm = map(int, plan["tile"].split("x"))
    No, Ho, Wo, Nb = shape
    idx = W.output_points((No, Nb), Ho, Wo, min(16, to), max(tm // 2, 4), 2, seed)
    # every block of the grid really holds a point
    m = (idx[:, 1].astype(np.int64) * Wo + idx[:, 2]) * Nb + idx[:, 3]
    blocks = set(zip((idx[:, 0] // min(16, to)).tolist(), (m // max(tm // 2, 4)).tolist()))
    assert len(blocks) == -(-No // min(16, to)) * -(-(Ho * Wo * Nb) // max(tm // 2, 4))
    return idx


def run_gpu(env, layer, inp, filt, variant=None):
    torch, B, _ = env
    d_in = torch.from_numpy(inp).cuda()
    d_f = torch.from_numpy(filt).cuda()
    out = B.mdnn_conv_fprop(d_in, d_f, layer.stride, layer.pad, layer.alpha, variant=variant)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check(got, want, absum, alpha, what):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    scale = abs(alpha) * absum
    zero = scale == 0
    assert (got[zero] == 0).all(), f"{what}: non-zero output where every product is zero"
    ratio = np.zeros_like(err)
    np.divide(err, scale, out=ratio, where=~zero)
    worst = float(ratio.max()) if ratio.size else 0.0
    say(f"    {what}: max |err|/(|alpha| A) = {worst:.3e} over {got.size} outputs")
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert worst <= LOOSE, f"{what}: acceptance bound exceeded ({worst:.3e})"
    assert worst <= TIGHT, f"{what}: fp32-accumulation regression bound exceeded ({worst:.3e})"
    return worst


# ---------------------------------------------------------------- full layers
@pytest.mark.parametrize("name", W.ORDER)
def test_layer_matches_oracle_everywhere(env, name):
    """All five layer shapes at full size, every output element, default variant
    (the launch configuration bench.py times)."""
    _, B, oracle = env
    L = W.LAYERS[name]
    say(f"[parity] layer={name} seed={L.seed} dims={L.dims()} "
        f"variant={B.mdnn_choose_variant(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)}")
    inp, filt = W.make_inputs(L)
    got = run_gpu(env, L, inp, filt)
    want, absum = oracle.conv_fprop(inp, filt, L.stride, L.pad, L.alpha)
    assert got.shape == want.shape
    check(got, want, absum, L.alpha, name)


@pytest.mark.parametrize("name", W.ORDER)
def test_layer_integer_data_bitwise(env, name):
    """Full-size layers with small-integer data: sampled outputs (plus all four
    corners of the output tensor) must equal the oracle bit for bit."""
    _, B, oracle = env
    L = W.LAYERS[name]
    say(f"[parity-int] layer={name} seed={L.seed + 7919}")
    inp, filt = W.make_int_inputs(L)
    got = run_gpu(env, L, inp, filt)
    No, Ho, Wo, Nb = got.shape
    rng = np.random.default_rng(L.seed)
    npts = 40000
    idx = np.stack([rng.integers(0, No, npts), rng.integers(0, Ho, npts),
                    rng.integers(0, Wo, npts), rng.integers(0, Nb, npts)], axis=1).astype(np.int32)
    idx[0] = (0, 0, 0, 0)
    idx[1] = (No - 1, Ho - 1, Wo - 1, Nb - 1)
    idx[2] = (No - 1, 0, Wo - 1, 0)
    idx[3] = (0, Ho - 1, 0, Nb - 1)
    vals, _ = oracle.conv_fprop_points(inp, filt, idx, L.stride, L.pad, L.alpha)
    o, y, x, n = idx.T
    np.testing.assert_array_equal(got[o, y, x, n], vals)
    assert np.abs(vals).max() > 0


@pytest.mark.parametrize("name", sorted(W.TABLE1))
def test_paper_table1_shapes_sampled(env, name):
    """The ten layer shapes of the paper's Table 1 at full size (minibatch 128):
    outputs sampled in every tile and tail piece of the launch (see tile_points)
    against the oracle's one-by-one evaluation, default variant.  Overfeat L4/L5
    have K = 4608 / 9216, more than one offset-table chunk."""
    _, B, oracle = env
    L, _ = W.TABLE1[name]
    say(f"[parity-table1] layer={name} seed={L.seed} plan="
        f"{B.mdnn_describe_launch(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)}")
    inp, filt = W.make_inputs(L)
    got = run_gpu(env, L, inp, filt)
    idx = tile_points(B, L, got.shape, L.seed % 1000)
    say(f"    {idx.shape[0]} points")
    vals, absum = oracle.conv_fprop_points(inp, filt, idx, L.stride, L.pad, L.alpha)
    o, y, x, n = idx.T
    check(got[o, y, x, n], vals, absum, L.alpha, name)


@pytest.mark.parametrize("name", list(W.VGG16))
def test_vgg16_shapes_sampled(env, name):
    """The nine distinct 3x3 shapes of a VGG-16 style network at minibatch 64, full size (tensors up
    to 0.8 GB, 12544 tiles): outputs sampled in every tile and tail piece of the launch (see
    tile_points; up to 200 000 of them) against the oracle's one-by-one evaluation, default
    variant -- the launch configuration `bench.py --vgg16` times."""
    torch, B, oracle = env
    L = W.VGG16[name]
    say(f"[parity-vgg16] layer={name} seed={L.seed} plan="
        f"{B.mdnn_describe_launch(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)}")
    inp, filt = W.make_inputs(L)
    d_in, d_f = torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda()
    out = B.mdnn_conv_fprop(d_in, d_f, L.stride, L.pad, L.alpha)
    torch.cuda.synchronize()
    idx = tile_points(B, L, tuple(out.shape), L.seed % 1000)
    say(f"    {idx.shape[0]} points")
    t = torch.from_numpy(idx.astype(np.int64)).cuda()
    got = out[t[:, 0], t[:, 1], t[:, 2], t[:, 3]].cpu().numpy()        # gather on the device: out is up to 0.8 GB
    assert bool(torch.isfinite(out).all())
    del out, d_in, d_f
    vals, absum = oracle.conv_fprop_points(inp, filt, idx, L.stride, L.pad, L.alpha)
    check(got, vals, absum, L.alpha, name)


def test_output_bound_first_layer_integer_bitwise(env):
    """The 3 -> 64 channel first layer of the VGG-16 style network at full size (K = 27: bound by
    writing its 822 MB output; 64 x 512 tiles, stores with the non-temporal hint): integer data,
    points in every tile, bit for bit."""
    torch, B, oracle = env
    L = W.VGG16["conv1_1"]
    plan = B.mdnn_describe_launch(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    say(f"[parity-first-layer] plan={plan}")
    assert plan["variant"] == "o64m512" and plan["tile"] == "64x512"
    inp, filt = W.make_int_inputs(L)
    out = B.mdnn_conv_fprop(torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda(), L.stride, L.pad, L.alpha)
    torch.cuda.synchronize()
    idx = tile_points(B, L, tuple(out.shape), 27)
    t = torch.from_numpy(idx.astype(np.int64)).cuda()
    got = out[t[:, 0], t[:, 1], t[:, 2], t[:, 3]].cpu().numpy()
    del out
    vals, _ = oracle.conv_fprop_points(inp, filt, idx, L.stride, L.pad, L.alpha)
    np.testing.assert_array_equal(got, vals)
    assert np.abs(vals).max() > 0


# ------------------------------------------------------- odd shapes, all variants
ODD = [
    # name              Nb  Hi  Wi  Nc  No  Sk st pad alpha
    ("ragged_vec",      12, 11,  9,  5, 36, 3, 1, 1, 0.5),     # tails in No, M and K
    ("ragged_scalar",    7, 10, 11,  3, 37, 3, 2, 1, 1.5),     # Nb, No not multiples of 4
    ("nb1_no1",          1,  9,  9,  2,  1, 3, 1, 0, 1.0),
    ("one_by_one",      16,  6,  7, 40, 24, 1, 1, 0, -2.0),    # plain matrix product
    ("big_filter",       8, 12, 12,  3, 16, 7, 2, 3, 1.0),
    ("filter_eq_image",  4,  5,  5,  4,  8, 5, 1, 0, 1.0),     # a single output coordinate
    ("wide_apron",       8,  6,  6,  3, 12, 3, 1, 2, 1.0),     # pad close to Sk: whole rows of taps in the apron
    ("stride3_nonsq",   20,  9, 14,  6, 40, 4, 3, 1, 0.25),
    ("k_odd",            8,  8,  8,  3, 32, 3, 1, 1, 1.0),     # K = 27: odd, one partial slab
    ("many_tiles",      32, 15, 13, 20, 200, 3, 1, 1, 1.0),    # several tiles both ways + tails
    ("long_k_chunked",   8,  6,  6, 520, 32, 3, 1, 1, 1.0),    # K = 4680 > one offset-table chunk
    ("odd_filters",     32, 15, 13, 20, 202, 3, 1, 1, 1.0),    # only No off the multiple of 4: 4-byte filter copies alone
    ("odd_batch",       30, 15, 13, 20, 200, 3, 1, 1, 0.5),    # only Nb: 4-byte patch copies and stores alone (M = 5850)
    ("odd_batch_strided", 6, 17, 16, 7, 136, 5, 2, 2, 1.0),    # the same with an apron and a stride; M = 384
]


@pytest.mark.parametrize("case", ODD, ids=[c[0] for c in ODD])
def test_odd_shapes_every_usable_variant(env, case):
    _, B, oracle = env
    name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha = case
    L = W.custom(name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha, seed=W.SEED_BASE + 100 + len(name))
    inp, filt = W.make_inputs(L)
    want, absum = oracle.conv_fprop(inp, filt, stride, pad, alpha)
    ran = 0
    for variant in [None] + B.mdnn_variant_names():
        try:          # a variant whose 16-byte copies this Nb or No rules out is refused
            B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad, variant)
        except B.MdnnError:
            assert variant is not None and (Nb % 4 or No % 4), variant
            continue
        say(f"[parity-odd] case={name} variant={variant} dims={L.dims()}")
        got = run_gpu(env, L, inp, filt, variant)
        check(got, want, absum, alpha, f"{name}/{variant}")
        ran += 1
    assert ran >= 2


def test_mid_size_all_variants_integer_bitwise(env):
    """One mid-size shape that spans many tiles of every variant, integer data,
    whole tensor compared bit for bit -- also a race detector for the LDS
    double buffering."""
    _, B, oracle = env
    L = W.custom("mid", 64, 14, 14, 48, 288, 3, 1, 1, 0.5)
    inp, filt = W.make_int_inputs(L)
    want = oracle.conv_fprop(inp, filt, L.stride, L.pad, L.alpha, want_abs=False)
    for variant in B.mdnn_variant_names():
        say(f"[parity-mid] variant={variant}")
        got = run_gpu(env, L, inp, filt, variant)
        np.testing.assert_array_equal(got, want, err_msg=variant)


# ------------------------------------------------- tail pieces (half / third / quarter / eighth tiles)
TAILS = [
    # name        Nb  Hi  Wi  Nc  No  Sk st pad alpha  pieces per cut tile with the deep-slab kernel, with the shallow-slab one
    ("halves",    128,  6, 91,  8, 128, 3, 1, 0, 1.0,  2, 2),      # 356 tiles: 100 left over -> halves
    ("quarters",  128, 10, 39,  8, 128, 3, 1, 0, 0.5,  4, 4),      # 296 tiles:  40 left over -> quarters
    ("quarters_ragged", 64, 11, 40, 6, 200, 3, 1, 1, 2.0, 4, (128, 0, 56, 0)),   # padded, ragged filter tile, 2 pixels per tile; 440 tiles
    ("thirds",    128, 14, 30,  8, 128, 3, 1, 0, 1.0,  3, (0, 0, 64, 16)),      # 336 tiles: 80 left over -> 48 + 48 + 32 rows; a quarter and an eighth per unit
    ("thirds_ragged", 64, 12, 28, 6, 200, 3, 1, 1, 2.0, 3, (0, 0, 64, 16)),     # 336 tiles, the second filter tile has 72 rows
    # 392 tiles, 136 left over: both kernels pair halves with eighths
    ("one_round_136", 128, 16, 30, 8, 128, 3, 1, 0, 0.5, (128, 0, 0, 8), (128, 0, 0, 8)),
    ("one_round_164", 128, 16, 32, 8, 128, 3, 1, 0, 0.5, 4, (128, 0, 36, 0)),   # 420 tiles: quarter chains; halves with quarters
    ("one_round_89", 128, 17, 25, 8, 128, 3, 1, 0, 0.5, 2, (0, 0, 64, 25)),   # 345 tiles: halves; quarters paired with eighths
    ("one_round_24", 128, 12, 30, 8, 128, 3, 1, 0, 2.0, 8, 4),                 # 280 tiles: eighths beside one round on the deep-slab kernel
    ("two_rounds_28", 128, 22, 29, 8, 128, 3, 1, 0, 1.0, 8, 8),                # 540 tiles: eighths in front of two rounds
    ("two_rounds_136", 128, 20, 38, 8, 128, 3, 1, 0, 0.5, (128, 0, 0, 8), 4),    # 648 tiles: halves with eighths; quarter chains
]


@pytest.mark.parametrize("case", TAILS, ids=[c[0] for c in TAILS])
@pytest.mark.parametrize("variant", ["o128m128", "o128m128k8"])
def test_tail_pieces_bitwise(env, case, variant):
    """Launches whose last partial round of tiles is cut into half, third, quarter or
    eighth tiles: the plan says so, and integer data must match the oracle bit for bit."""
    _, B, oracle = env
    name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha, want_deep, want_shallow = case
    want = want_deep if variant == "o128m128" else want_shallow
    plan = B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad, variant)
    say(f"[parity-tail] case={name} variant={variant} plan={plan}")
    if isinstance(want, tuple):          # (halved, thirded, quartered, eighthed): a mixture, all of it in front of the whole tiles
        assert plan["split"] == 0 and (plan["halved"], plan["thirded"], plan["quartered"], plan["eighthed"]) == want
        assert sum(want) == plan["tiles"] - plan["whole"] and plan["pieces_first"] == plan["pieces"]
    else:
        assert plan["split"] == want and plan["pieces"] == (plan["tiles"] - plan["whole"]) * want
    L = W.custom(name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha)
    inp, filt = W.make_int_inputs(L)
    want_out = oracle.conv_fprop(inp, filt, stride, pad, alpha, want_abs=False)
    got = run_gpu(env, L, inp, filt, variant)
    np.testing.assert_array_equal(got, want_out)


@pytest.mark.parametrize("variant,split,pieces", [("o96m256", 4, 256), ("o96m256:h", 2, 128)])
def test_tail_pieces_of_the_96_row_tile_bitwise(env, variant, split, pieces):
    """The 96x256 tile (eight waves of 48x64) is halved along the filters (48x256 on eight waves of
    48x32) and quartered along the columns as well (48x128): 320 tiles = one round + 64 tiles cut
    into 256 quarter pieces by the library's own plan, or into 128 halves when pinned."""
    _, B, oracle = env
    Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha = 128, 34, 22, 4, 96, 3, 1, 0, 1.0
    plan = B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad, variant)
    say(f"[parity-tail-96] plan={plan}")
    assert plan["tiles"] == 320 and plan["split"] == split and plan["pieces"] == pieces
    L = W.custom("tail_m", Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha)
    inp, filt = W.make_int_inputs(L)
    want = oracle.conv_fprop(inp, filt, stride, pad, alpha, want_abs=False)
    got = run_gpu(env, L, inp, filt, variant)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("variant,No,want_plan", [
    ("o128m128k8", 768, dict(tiles=588, whole=512, split=0, quartered=64, eighthed=12, pieces=352, pieces_first=352)),   # a pairing: all pieces in front
    ("o128m128k8:h", 768, dict(tiles=588, whole=512, split=2, pieces=152, pieces_first=152)),  # halves: all in front
    ("o128m128", 1280, dict(tiles=910, whole=768, split=0, halved=128, eighthed=14, pieces=368, pieces_first=368)),   # a pairing on the other kernel
    ("o128m128:q", 1280, dict(tiles=910, whole=768, split=4, pieces=568, pieces_first=256)),    # 256 in front, 312 behind
    # every tile in thirds (the cut pinned through the variant name): 48- and 32-row pieces only
    ("o128m128:T", 256, dict(tiles=182, whole=0, split=3, thirded=182, pieces=546, pieces_first=0)),
    # thirds of the last round with two rounds of whole tiles in front: the pieces go first
    ("o128m128:t", 1664, dict(tiles=1183, whole=1024, split=3, thirded=159, pieces=477, pieces_first=256)),
    # every tile in eighths (16-row pieces only), on both kernels; eighths in front of and behind four rounds
    ("o128m128:E", 256, dict(tiles=182, whole=0, split=8, eighthed=182, pieces=1456, pieces_first=0)),
    ("o128m128k8:E", 256, dict(tiles=182, whole=0, split=8, eighthed=182, pieces=1456, pieces_first=0)),
    ("o128m128k8:e", 1664, dict(tiles=1183, whole=1024, split=8, eighthed=159, pieces=1272, pieces_first=256)),
])
def test_pieces_before_and_after_the_whole_tiles_bitwise(env, variant, No, want_plan):
    """With two or more rounds of whole tiles, up to one piece per CU is launched before them and
    the rest after them; every piece and every tile must still be computed exactly once."""
    _, B, oracle = env
    Nb, Hi, Wi, Nc, Sk, stride, pad, alpha = 64, (14 if No == 768 else 13), 14, 8, 3, 1, 1, 0.5
    plan = B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad, variant)
    say(f"[parity-front-pieces] plan={plan}")
    for k, v in want_plan.items():
        assert plan[k] == v, (k, plan)
    L = W.custom("front_pieces", Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha)
    inp, filt = W.make_int_inputs(L)
    want = oracle.conv_fprop(inp, filt, stride, pad, alpha, want_abs=False)
    got = run_gpu(env, L, inp, filt, variant)
    np.testing.assert_array_equal(got, want)


def test_offsets_beyond_two_gib(env):
    """An input of 3.0 GiB (byte offsets above 2^31, close to the 4 GiB limit of the
    32-bit buffer offsets) and a padded geometry whose apron origins wrap around
    zero: sampled outputs, concentrated on the last channels and on the border,
    against the oracle's one-by-one evaluation."""
    torch, B, oracle = env
    Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha = 128, 64, 64, 1536, 8, 3, 1, 1, 1.0
    L = W.custom("big_in", Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha, seed=W.SEED_BASE + 77)
    say(f"[parity-3gib] in bytes = {4 * Nb * Hi * Wi * Nc}")
    rng = np.random.default_rng(L.seed)
    inp = rng.integers(-2, 3, size=(Nc, Hi, Wi, Nb), dtype=np.int8).astype(np.float32)
    filt = np.zeros((Nc, Sk, Sk, No), np.float32)
    filt[-64:] = rng.integers(-2, 3, size=(64, Sk, Sk, No)).astype(np.float32)    # only the last channels count:
    filt[:2] = rng.integers(-2, 3, size=(2, Sk, Sk, No)).astype(np.float32)       # offsets > 2^31, and the first two
    d_in = torch.from_numpy(inp).cuda()
    d_f = torch.from_numpy(filt).cuda()
    out = B.mdnn_conv_fprop(d_in, d_f, stride, pad, alpha)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    del d_in
    npts = 4000
    idx = np.stack([rng.integers(0, No, npts), rng.integers(0, Hi, npts),
                    rng.integers(0, Wi, npts), rng.integers(0, Nb, npts)], axis=1).astype(np.int32)
    idx[:400, 1] = rng.choice([0, Hi - 1], 400)       # top / bottom rows: taps in the apron
    idx[400:800, 2] = rng.choice([0, Wi - 1], 400)    # left / right columns
    idx[0] = (0, 0, 0, 0)
    idx[1] = (No - 1, Hi - 1, Wi - 1, Nb - 1)
    vals, _ = oracle.conv_fprop_points(inp, filt, idx, stride, pad, alpha)
    o, y, x, n = idx.T
    np.testing.assert_array_equal(got[o, y, x, n], vals)          # integer data: exact
    assert np.abs(vals).max() > 0


# ------------------------------------------------------------ semantic edge cases
def test_delta_filter_and_apron_zeros(env):
    _, B, _ = env
    L = W.custom("delta", 8, 9, 8, 4, 8, 3, 1, 1, 2.0)
    inp, _ = W.make_inputs(L)
    filt = np.zeros((L.Nc, L.Sk, L.Sk, L.No), np.float32)
    c0, ky0, kx0, o0 = 2, 0, 2, 5
    filt[c0, ky0, kx0, o0] = 1.0
    say("[parity-delta]")
    got = run_gpu(env, L, inp, filt)
    want = np.zeros_like(got)
    for y in range(got.shape[1]):
        for x in range(got.shape[2]):
            iy, ix = y - L.pad + ky0, x - L.pad + kx0
            if 0 <= iy < L.Hi and 0 <= ix < L.Wi:
                want[o0, y, x, :] = 2.0 * inp[c0, iy, ix, :]
    np.testing.assert_array_equal(got, want)


def test_alpha_zero_and_determinism(env):
    torch, B, _ = env
    L = W.LAYERS["tiny"]
    inp, filt = W.make_inputs(L)
    d_in, d_f = torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda()
    say("[parity-alpha0]")
    z = B.mdnn_conv_fprop(d_in, d_f, L.stride, L.pad, 0.0)
    a = B.mdnn_conv_fprop(d_in, d_f, L.stride, L.pad, 1.0)
    b = B.mdnn_conv_fprop(d_in, d_f, L.stride, L.pad, 1.0)
    torch.cuda.synchronize()
    assert not z.cpu().numpy().any()
    assert torch.equal(a, b)


def test_output_is_overwritten_not_accumulated(env):
    torch, B, oracle = env
    L = W.custom("ow", 8, 8, 8, 4, 16, 3, 1, 1, 1.0)
    inp, filt = W.make_int_inputs(L)
    d_in, d_f = torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda()
    out = torch.full((16, 8, 8, 8), float("nan"), device="cuda")
    say("[parity-overwrite]")
    B.mdnn_conv_fprop(d_in, d_f, 1, 1, 1.0, out=out)
    torch.cuda.synchronize()
    want = oracle.conv_fprop(inp, filt, 1, 1, 1.0, want_abs=False)
    np.testing.assert_array_equal(out.cpu().numpy(), want)


def test_runs_on_a_side_stream(env):
    torch, B, oracle = env
    L = W.custom("stream", 16, 10, 10, 8, 32, 3, 1, 1, 1.0)
    inp, filt = W.make_int_inputs(L)
    d_in, d_f = torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    say("[parity-stream]")
    with torch.cuda.stream(s):
        out = B.mdnn_conv_fprop(d_in, d_f, 1, 1, 1.0)
    s.synchronize()
    want = oracle.conv_fprop(inp, filt, 1, 1, 1.0, want_abs=False)
    np.testing.assert_array_equal(out.cpu().numpy(), want)


def test_mfma_probe_runs(env):
    torch, B, _ = env
    sink = torch.zeros(256 * 4 * 64, device="cuda")
    say("[probe]")
    flops = B.mdnn_mfma_peak_probe(sink, 256, 4, 100)
    torch.cuda.synchronize()
    assert flops == 256 * 4 * 100 * 4 * 4096
    assert torch.isfinite(sink).all() and float(sink.abs().sum()) > 0
