"""Host-only checks of the C ABI: the library loads without a GPU, exports
every function include/mdnn.h declares, and rejects bad arguments before
anything could be launched.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_1501_06633_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mdnn.h")

FAKE = 0x10000          # 16-byte aligned, never dereferenced: every call below fails validation first


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_1501_06633_amd import build
        build.build_lib()
    return B.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mdnn_[a-z_0-9]+)\s*\(", text)))


def test_exports_every_declared_symbol(L):
    names = declared_functions()
    assert {"mdnn_conv_fprop", "mdnn_conv_fprop_variant", "mdnn_out_dims", "mdnn_conv_flops",
            "mdnn_status_string", "mdnn_variant_count", "mdnn_variant_name",
            "mdnn_choose_variant", "mdnn_describe_launch", "mdnn_mfma_peak_probe",
            "mdnn_conv_bprop_data", "mdnn_conv_bprop_data_workspace", "mdnn_conv_bprop_data_static",
            "mdnn_conv_bprop_filter", "mdnn_conv_bprop_filter_workspace", "mdnn_sgemm_tn"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"libmdnn.so does not export {n}"


def test_out_dims_and_flops_match_the_paper(L):
    golden = os.path.join(ROOT, "tests", "golden")
    for line in open(os.path.join(golden, "table1_shapes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        _, _, Wi, _, Wo, _, Sk, stride, pad = line.split()
        st, wo, ho = B.mdnn_out_dims(int(Wi), int(Wi), int(Sk), int(stride), int(pad))
        assert (st, wo, ho) == (B.MDNN_OK, int(Wo), int(Wo)), line
    for line in open(os.path.join(golden, "flops_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        Nb, Wo, Ho, Nc, No, Sk, C = map(int, line.split())
        assert B.mdnn_conv_flops(Nb, Wo, Ho, Nc, No, Sk) == C, line
    assert B.mdnn_out_dims(7, 5, 3, 1, 0) == (B.MDNN_OK, 5, 3)
    assert B.mdnn_out_dims(8, 8, 3, 2, 0) == (B.MDNN_OK, 3, 3)
    assert B.mdnn_conv_flops(0, 1, 1, 1, 1, 1) == 0


def test_out_dims_errors(L):
    assert B.mdnn_out_dims(5, 5, 6, 1, 0)[0] == B.MDNN_EINVAL
    assert B.mdnn_out_dims(5, 5, 3, 0, 0)[0] == B.MDNN_EINVAL
    assert B.mdnn_out_dims(5, 5, 3, 1, -1)[0] == B.MDNN_EINVAL
    assert B.mdnn_out_dims(0, 5, 1, 1, 0)[0] == B.MDNN_EINVAL
    assert L.mdnn_out_dims(5, 5, 3, 1, 0, None, None) == B.MDNN_ENULL


GOOD = dict(Nb=8, Wi=32, Hi=32, Nc=16, No=32, Sk=3, stride=1, pad=1)


def call(in_ptr=FAKE, filt_ptr=FAKE, out_ptr=FAKE, alpha=1.0, variant=None, **kw):
    d = dict(GOOD)
    d.update(kw)
    return B.mdnn_conv_fprop_raw(in_ptr, filt_ptr, out_ptr, d["Nb"], d["Wi"], d["Hi"], d["Nc"], d["No"],
                                 d["Sk"], d["stride"], d["pad"], alpha, None, variant)


def test_null_pointers(L):
    assert call(in_ptr=None) == B.MDNN_ENULL
    assert call(filt_ptr=None) == B.MDNN_ENULL
    assert call(out_ptr=None) == B.MDNN_ENULL


@pytest.mark.parametrize("kw", [dict(Nb=0), dict(Wi=0), dict(Hi=-1), dict(Nc=0), dict(No=0), dict(Sk=0),
                                dict(stride=0), dict(pad=-1), dict(Sk=35), dict(Sk=35, Wi=40), dict(Sk=35, Hi=40),
                                dict(alpha=float("nan")), dict(alpha=float("inf"))])
def test_invalid_arguments(L, kw):
    assert call(**kw) == B.MDNN_EINVAL


def test_too_big(L):
    assert call(Nb=1024, Wi=1024, Hi=1024, Nc=1) == B.MDNN_ETOOBIG          # in = 4 GiB exactly
    assert call(Nb=128, Wi=2048, Hi=2048, Nc=1, No=4) == B.MDNN_ETOOBIG     # out = 8 GiB
    assert call(Nc=65536, Sk=3, No=4096) == B.MDNN_ETOOBIG                  # filt
    assert call(Nc=16384, Sk=4, No=2048, Hi=8, Wi=8, Nb=4) == B.MDNN_ETOOBIG   # filt = 2 GiB exactly
    assert call(Nb=2**20, Wi=2**20, Hi=2**20, Nc=2**20) == B.MDNN_ETOOBIG   # no wrap-around
    # a very wide, shallow filter matrix: 2^26 filters of one tap are only 256 MiB, but the rows past
    # the last one, which must read as zero, would have byte offsets that wrap back into the buffer
    assert call(Nb=1, Wi=2, Hi=2, Nc=1, Sk=1, pad=0, No=2**26) == B.MDNN_ETOOBIG
    assert B.mdnn_describe_launch(1, 2, 2, 1, 2**23, 1, 1, 0)["tiles"] > 0           # 2^23 filters fit


def test_misaligned(L):
    assert call(in_ptr=FAKE + 4) == B.MDNN_EALIGN
    assert call(filt_ptr=FAKE + 8) == B.MDNN_EALIGN
    assert call(out_ptr=FAKE + 1) == B.MDNN_EALIGN


def test_unknown_or_unusable_variant(L):
    assert call(variant="no_such_tile") == B.MDNN_EINVAL
    vec = [n for n in B.mdnn_variant_names() if n[-1] not in "sab"]
    assert call(variant=vec[0], Nb=6) == B.MDNN_EINVAL       # 16-byte variant needs Nb % 4 == 0
    # the tiles with one narrow operand: "a" copies filters 4 bytes at a time (any No), "b" patches (any Nb)
    assert call(variant="o128m128a", Nb=6) == B.MDNN_EINVAL and call(variant="o128m128b", No=6) == B.MDNN_EINVAL


def test_variant_registry_and_choice(L):
    names = B.mdnn_variant_names()
    assert len(names) == len(set(names)) >= 3
    assert L.mdnn_variant_name(-1) is None and L.mdnn_variant_name(len(names)) is None
    for shape in [(8, 32, 32, 16, 32, 3, 1, 1), (128, 227, 227, 3, 96, 11, 4, 0),
                  (128, 27, 27, 96, 256, 5, 1, 2), (64, 56, 56, 256, 256, 3, 1, 1),
                  (7, 9, 9, 3, 5, 3, 1, 1)]:
        assert B.mdnn_choose_variant(*shape) in names
    assert B.mdnn_choose_variant(7, 9, 9, 3, 5, 3, 1, 1).endswith("s")     # scalar-load variant
    assert B.mdnn_choose_variant(64, 56, 56, 256, 250, 3, 1, 1) == "o128m128k8a"  # only the filter count is off the multiple of 4
    assert B.mdnn_choose_variant(50, 56, 56, 256, 256, 3, 1, 1) == "o128m128k8b"  # only the minibatch is
    assert B.mdnn_choose_variant(50, 56, 56, 256, 250, 3, 1, 1) == "o128m128s"    # both
    assert B.mdnn_choose_variant(6, 9, 10, 5, 40, 3, 2, 1) == "o64m64s"           # a small layer: the only small tile it can take
    assert B.mdnn_choose_variant(8, 2, 2, 1, 1, 3, 1, 0) is None          # invalid geometry


def test_choice_between_the_two_128x128_tiles_follows_the_tile_count(L):
    """128 images per pixel, 256 filters: 2 * Hi * 16 tiles of 128x128.  The two-per-CU tile takes
    everything up to two rounds; the three-per-CU tile takes longer launches except (a) those whose
    whole tiles fill the 768 slots once and partly a second time with fewer than 256 pieces in
    front (measured at 73-82 %) and (b) launches of up to six rounds whose whole tiles fill their
    last wave of 768 exactly and that have tail pieces to place (the pieces then have no room)."""
    pick = lambda Hi: B.mdnn_choose_variant(128, 16, Hi, 256, 256, 3, 1, 1)
    plan = lambda Hi: B.mdnn_describe_launch(128, 16, Hi, 256, 256, 3, 1, 1, "o128m128k8")
    for Hi in (8, 12, 16):                                      # up to two rounds
        assert plan(Hi)["tiles"] <= 512 and pick(Hi) == "o128m128", Hi
    for Hi in (18, 20, 23, 24):                                 # 576 ... 768 tiles: two rounds and a tail, or 768 whole
        assert plan(Hi)["whole"] <= 768 and pick(Hi) == "o128m128k8", Hi
    for Hi in (26, 28):                                         # 832, 896 tiles: 768 whole ones and a tail
        assert plan(Hi)["whole"] == 768 and plan(Hi)["pieces"] > 0 and pick(Hi) == "o128m128", Hi
    for Hi in (31, 32):                                         # 992, 1024 tiles
        d = plan(Hi)
        assert 768 < d["whole"] < 1248 and d["pieces"] < 256 and pick(Hi) == "o128m128", Hi
    for Hi in (33, 34, 35, 36):                                 # 1056 ... 1152 tiles: 1024 whole + 256 or more pieces in front
        d = plan(Hi)
        assert d["whole"] == 1024 and d["pieces_first"] >= 256 and pick(Hi) == "o128m128k8", Hi
    for Hi in (39, 40, 48, 80):                                 # 1248 tiles and more
        assert pick(Hi) == "o128m128k8", Hi


def test_variant_choice_is_the_committed_one(L):
    """The heuristic's choice (variant and tail cut) for 72 named shapes -- the five benchmark layers,
    the paper's Table 1, a VGG-16 style network and a 48-shape grid -- equals the committed
    snapshot, so that an edit to the cost model is visible as a diff of named shapes.  After a
    deliberate change: python tests/golden/write_variant_choice.py."""
    import importlib.util
    path = os.path.join(ROOT, "tests", "golden", "write_variant_choice.py")
    spec = importlib.util.spec_from_file_location("write_variant_choice", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = open(os.path.join(ROOT, "tests", "golden", "variant_choice.txt")).read().splitlines()
    got = mod.text().splitlines()
    assert len(got) == len(want) == 1 + 5 + 10 + 9 + 48
    for g, w in zip(got, want):
        assert g == w


def test_long_k_keeps_the_resident_workgroups(L):
    """The offset table is capped per variant so that LDS use, and with it the number of
    workgroups per CU, does not depend on K."""
    for v, per_cu in (("o128m128k8", 3), ("o128m128", 2), ("o96m128", 3), ("o96m256", 2), ("o64m256", 2),
                      ("o32m128", 4)):
        short = B.mdnn_describe_launch(128, 14, 14, 64, 192, 3, 1, 1, v)
        long_ = B.mdnn_describe_launch(128, 14, 14, 1024, 192, 3, 1, 1, v)
        assert long_["lds_bytes"] * per_cu <= 160 * 1024, v
        assert long_["lds_bytes"] * (per_cu + 1) > 160 * 1024 or v.startswith("o32"), v
        assert long_["table_entries"] % long_["kslab"] == 0 and long_["table_entries"] < 9216
        assert short["table_entries"] == 576


def test_describe_launch(L):
    d = B.mdnn_describe_launch(64, 56, 56, 256, 256, 3, 1, 1)
    assert d["K"] == 2304 and d["M"] == 56 * 56 * 64
    assert d["variant"] in B.mdnn_variant_names()
    to, tm = map(int, d["tile"].split("x"))
    assert d["tiles"] == -(-256 // to) * -(-d["M"] // tm)
    assert d["whole"] + d["halved"] + d["thirded"] + d["quartered"] + d["eighthed"] == d["tiles"]
    assert d["pieces"] == 2 * d["halved"] + 3 * d["thirded"] + 4 * d["quartered"] + 8 * d["eighthed"]
    assert d["lds_bytes"] <= 160 * 1024 and d["table_entries"] % d["kslab"] == 0
    # a pinned variant, a plan with the tail cut in pieces, and the error paths
    d = B.mdnn_describe_launch(128, 91, 6, 8, 128, 3, 1, 0, "o128m128")
    assert (d["tiles"], d["whole"], d["split"], d["pieces"]) == (356, 256, 2, 200)
    with pytest.raises(B.MdnnError):
        B.mdnn_describe_launch(8, 2, 2, 1, 1, 3, 1, 0)
    with pytest.raises(B.MdnnError):
        B.mdnn_describe_launch(8, 9, 9, 1, 4, 3, 1, 0, "nope")


def test_how_the_last_round_is_cut(L):
    """128 images, 128 filters, 3x3 unpadded: Ho * Wo tiles of 128x128, R whole rounds of 256 and
    r left-over tiles.  Pieces of one size: eighths up to r = 32, quarters up to 64, halves up to
    128, quarters in chains up to 192, then whole tiles; thirds (the deep-slab kernel) for 65 ... 85
    when R is odd.  Pairings of two sizes per unit (three-per-unit kernel): a quarter and an eighth
    for 65 ... 96 unless R mod 3 = 0, a half and an eighth (to 160) or a quarter (to 192) when
    R mod 3 = 1; the two-per-unit kernel takes the half and the eighth at every R and, for two to
    eight rounds, the quarter and the eighth where it has no thirds.  R mod 3 = 0 up to eight rounds on that kernel: quarters only."""
    def cut(r, variant, R=1):
        d = B.mdnn_describe_launch(128, 2 + 1, 2 + (256 * R + r), 4, 128, 3, 1, 0, variant)
        assert d["tiles"] == 256 * R + r and d["whole"] + d["halved"] + d["thirded"] + d["quartered"] + d["eighthed"] == d["tiles"]
        assert d["whole"] == (d["tiles"] if d["pieces"] == 0 else 256 * R)
        return "".join(f"{d[k]}{k[0]}" for k in ("halved", "thirded", "quartered", "eighthed") if d[k]) or "w"
    for R in (1, 2, 3, 4, 5, 7, 10):
        for v in ("o128m128", "o128m128k8"):
            three, full = v == "o128m128k8", v == "o128m128k8" and R % 3 == 0
            assert cut(0, v, R) == "w" and cut(200, v, R) == "w" and cut(255, v, R) == "w"
            assert cut(40, v, R) == "40q" and cut(64, v, R) == "64q"
            assert cut(24, v, R) == ("24q" if full or (three and R == 1) else "24e"), (v, R)
            assert cut(32, v, R) == ("32q" if full or (three and R == 1) else "32e") and cut(33, v, R) == "33q"
            if three:
                assert cut(72, v, R) == ("72q" if full and R <= 8 else "72h" if full else "64q8e"), (v, R)
                assert cut(96, v, R) == ("96q" if full and R <= 8 else "96h" if full else "64q32e")
                assert cut(136, v, R) == ("128h8e" if R % 3 == 1 else "136q"), (v, R)
                assert cut(160, v, R) == ("128h32e" if R % 3 == 1 else "160q")
                assert cut(161, v, R) == ("128h33q" if R % 3 == 1 else "161q") and cut(192, v, R) == ("128h64q" if R % 3 == 1 else "192q")
                assert cut(100, v, R) == ("100q" if full and R <= 8 else "100h") and cut(128, v, R) == ("128q" if full and R <= 8 else "128h")
            else:
                pairs = 2 <= R <= 8       # a quarter and an eighth per unit where thirds are not taken
                assert cut(65, v, R) == ("65t" if R % 2 else "64q1e" if pairs else "65h")
                assert cut(85, v, R) == ("85t" if R % 2 else "64q21e" if pairs else "85h")
                assert cut(86, v, R) == ("64q22e" if pairs else "86h") and cut(96, v, R) == ("64q32e" if pairs else "96h")
                assert cut(97, v, R) == "97h" and cut(128, v, R) == "128h"
                assert cut(129, v, R) == "128h1e" and cut(160, v, R) == "128h32e"
                assert cut(161, v, R) == "161q" and cut(192, v, R) == "192q"
    # where the pieces go: pairings all in front, single sizes up to one per unit in front of two or more rounds
    d = B.mdnn_describe_launch(128, 2 + 1, 2 + 392, 4, 128, 3, 1, 0, "o128m128k8")
    assert (d["whole"], d["pieces"], d["pieces_first"]) == (256, 320, 320)
    d = B.mdnn_describe_launch(128, 2 + 1, 2 + 540, 4, 128, 3, 1, 0, "o128m128k8")
    assert (d["whole"], d["split"], d["eighthed"], d["pieces"], d["pieces_first"]) == (512, 8, 28, 224, 224)
    d = B.mdnn_describe_launch(128, 2 + 1, 2 + 648, 4, 128, 3, 1, 0, "o128m128k8")   # two rounds + 136: quarter chains
    assert (d["whole"], d["split"], d["quartered"], d["pieces_first"]) == (512, 4, 136, 256)
    d = B.mdnn_describe_launch(128, 2 + 1, 2 + 280, 4, 128, 3, 1, 0, "o128m128")     # one round: the pieces go behind
    assert (d["whole"], d["split"], d["eighthed"], d["pieces_first"]) == (256, 8, 24, 0)
    d = B.mdnn_describe_launch(128, 2 + 1, 2 + 136, 4, 128, 3, 1, 0, "o128m128k8")   # no whole round at all
    assert d["whole"] == 0 and d["split"] in (2, 4)
    assert L.mdnn_describe_launch(8, 9, 9, 1, 4, 3, 1, 0, None, None, 0) == B.MDNN_ENULL


def test_bprop_data_workspace_and_argument_checks(L):
    # stride 1: only the rearranged filter bank (Nc*Sk*Sk*No floats), rounded up to 256 bytes
    st, n = B.mdnn_conv_bprop_data_workspace(64, 56, 56, 256, 256, 3, 1, 1)
    assert st == B.MDNN_OK and n == 256 * 9 * 256 * 4
    # stride 4, 11x11: 16 residue classes with 3x3 sub-filters -> a bank of (96*9) x (16*3) floats;
    # the per-class results go straight into din and need no room
    st, n = B.mdnn_conv_bprop_data_workspace(128, 227, 227, 3, 96, 11, 4, 0)
    bank = 96 * 9 * 48 * 4
    assert st == B.MDNN_OK and n == ((bank + 255) // 256) * 256
    # stride 1 with pad > Sk - 1 goes the way of the strided layers: one class, the turned-over bank
    st, n = B.mdnn_conv_bprop_data_workspace(8, 8, 8, 2, 4, 3, 1, 3)
    assert st == B.MDNN_OK and n == 512                                 # the 288-byte bank rounded up to 256s
    assert B.mdnn_conv_bprop_data_workspace(8, 2, 2, 2, 4, 3, 1, 0)[0] == B.MDNN_EINVAL     # no output
    assert L.mdnn_conv_bprop_data_workspace(8, 8, 8, 2, 4, 3, 1, 1, None) == B.MDNN_ENULL
    args = (8, 8, 8, 2, 4, 3, 1, 1)
    need = B.mdnn_conv_bprop_data_workspace(*args)[1]
    call_b = lambda d=FAKE, f=FAKE, o=FAKE, w=FAKE, wb=need, a=1.0: L.mdnn_conv_bprop_data(d, f, o, w, wb, *args, a, None)
    assert call_b(d=None) == B.MDNN_ENULL and call_b(w=None) == B.MDNN_ENULL
    assert call_b(wb=need - 1) == B.MDNN_EINVAL
    assert call_b(a=float("nan")) == B.MDNN_EINVAL
    assert call_b(w=FAKE + 4) == B.MDNN_EALIGN


def test_static_data_gradient_argument_checks(L):
    """The allocation-free variant refuses everything the workspace call refuses, and whatever does
    not fit its static array, before it touches the GPU."""
    args = (8, 8, 8, 2, 4, 3, 1, 1)
    call_s = lambda d=FAKE, f=FAKE, o=FAKE, a=1.0, dims=args: L.mdnn_conv_bprop_data_static(d, f, o, *dims, a, None)
    assert call_s(d=None) == B.MDNN_ENULL and call_s(f=None) == B.MDNN_ENULL and call_s(o=None) == B.MDNN_ENULL
    assert call_s(a=float("nan")) == B.MDNN_EINVAL
    assert call_s(o=FAKE + 4) == B.MDNN_EALIGN
    assert call_s(dims=(8, 2, 2, 2, 4, 3, 1, 0)) == B.MDNN_EINVAL          # no output
    # the limit is the header's constant, in terms of mdnn_conv_bprop_data_workspace()
    header = open(HEADER).read()
    m = re.search(r"#define\s+MDNN_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", header)
    assert m and (int(m.group(1)) << int(m.group(2))) == B.MDNN_STATIC_SCRATCH_BYTES
    fits = (128, 12, 12, 1024, 1024, 3, 1, 1)        # bank of 36 MiB
    assert B.mdnn_conv_bprop_data_workspace(*fits)[1] <= B.MDNN_STATIC_SCRATCH_BYTES
    assert call_s(dims=fits, o=FAKE + 4) == B.MDNN_EALIGN                   # passed the size check
    assert call_s(dims=(128, 227, 227, 3, 96, 11, 4, 0), o=FAKE + 4) == B.MDNN_EALIGN    # a strided layer fits too
    for too_big in [(128, 12, 12, 1024, 1280, 3, 1, 1),                     # bank of 45 MiB
                    (16, 40, 40, 256, 512, 11, 4, 0)]:                      # 16 classes x 3x3 x 256 x 512: 72 MiB
        assert B.mdnn_conv_bprop_data_workspace(*too_big)[1] > B.MDNN_STATIC_SCRATCH_BYTES
        assert call_s(dims=too_big) == B.MDNN_ETOOBIG


def test_bprop_filter_workspace_and_argument_checks(L):
    # the workspace holds a whole number of K x No partial gradients, at least one
    for dims in [(64, 56, 56, 256, 256, 3, 1, 1), (128, 227, 227, 3, 96, 11, 4, 0), (8, 32, 32, 16, 32, 3, 1, 1),
                 (1, 5, 5, 2, 3, 5, 1, 0), (7, 10, 11, 3, 37, 3, 2, 1), (128, 12, 12, 1024, 1024, 3, 1, 1),
                 (128, 27, 27, 96, 256, 5, 1, 2)]:
        st, n = B.mdnn_conv_bprop_filter_workspace(*dims)
        Nb, Wi, Hi, Nc, No, Sk, stride, pad = dims
        one = Nc * Sk * Sk * No * 4
        assert st == B.MDNN_OK and n >= one and n % one == 0, dims
        _, wo, ho = B.mdnn_out_dims(Wi, Hi, Sk, stride, pad)
        ranges = n // one
        assert ranges <= max(1, (wo * ho * Nb + 15) // 16), dims       # never an empty range
        # the busiest of the 256 compute units gets at most 15 % more than an even share of the slabs
        slabs = -(-(wo * ho * Nb) // 16)
        for w in (128, 96, 64, 32):
            tiles = -(-(Nc * Sk * Sk) // 128) * -(-No // w)
            if tiles * slabs >= 256 * 64:
                busiest = -(-(tiles * ranges) // 256) * -(-slabs // ranges)
                if busiest <= 1.15 * tiles * slabs / 256:
                    break
        else:
            assert tiles * slabs < 256 * 64, dims
    # any pad is accepted (the data gradient needs pad <= Sk - 1, this one does not)
    assert B.mdnn_conv_bprop_filter_workspace(8, 5, 5, 3, 12, 3, 1, 4)[0] == B.MDNN_OK
    assert B.mdnn_conv_bprop_filter_workspace(8, 2, 2, 2, 4, 3, 1, 0)[0] == B.MDNN_EINVAL   # no output
    assert B.mdnn_conv_bprop_filter_workspace(1 << 12, 1 << 10, 1 << 10, 1, 4, 3, 1, 0)[0] == B.MDNN_ETOOBIG
    assert L.mdnn_conv_bprop_filter_workspace(8, 8, 8, 2, 4, 3, 1, 1, None) == B.MDNN_ENULL
    args = (8, 8, 8, 2, 4, 3, 1, 1)
    need = B.mdnn_conv_bprop_filter_workspace(*args)[1]
    call_f = lambda i=FAKE, d=FAKE, o=FAKE, w=FAKE, wb=need, a=1.0: L.mdnn_conv_bprop_filter(i, d, o, w, wb, *args, a, None)
    assert call_f(i=None) == B.MDNN_ENULL and call_f(d=None) == B.MDNN_ENULL
    assert call_f(o=None) == B.MDNN_ENULL and call_f(w=None) == B.MDNN_ENULL
    assert call_f(wb=need - 1) == B.MDNN_EINVAL
    assert call_f(a=float("inf")) == B.MDNN_EINVAL
    assert call_f(d=FAKE + 8) == B.MDNN_EALIGN


def test_sgemm_argument_checks(L):
    A, Bm, C = FAKE, FAKE + 4096, FAKE + 8192
    assert L.mdnn_sgemm_tn(None, Bm, C, 8, 8, 8, 1.0, None) == B.MDNN_ENULL
    assert L.mdnn_sgemm_tn(A, None, C, 8, 8, 8, 1.0, None) == B.MDNN_ENULL
    assert L.mdnn_sgemm_tn(A, Bm, None, 8, 8, 8, 1.0, None) == B.MDNN_ENULL
    for dims in [(0, 8, 8), (8, 0, 8), (8, 8, 0), (-1, 8, 8)]:
        assert L.mdnn_sgemm_tn(A, Bm, C, *dims, 1.0, None) == B.MDNN_EINVAL
    assert L.mdnn_sgemm_tn(A, Bm, C, 8, 8, 8, float("nan"), None) == B.MDNN_EINVAL
    assert L.mdnn_sgemm_tn(A + 4, Bm, C, 8, 8, 8, 1.0, None) == B.MDNN_EALIGN
    assert L.mdnn_sgemm_tn(A, Bm, C + 8, 8, 8, 8, 1.0, None) == B.MDNN_EALIGN
    assert L.mdnn_sgemm_tn(A, Bm, C, 8, 2**20, 2**10, 1.0, None) == B.MDNN_ETOOBIG    # b = 4 GiB
    assert L.mdnn_sgemm_tn(A, Bm, C, 2**16, 2**14, 8, 1.0, None) == B.MDNN_ETOOBIG    # c = 4 GiB
    assert L.mdnn_sgemm_tn(A, Bm, C, 2**15, 8, 2**14, 1.0, None) == B.MDNN_ETOOBIG    # a = 2 GiB


def test_status_strings(L):
    seen = {B.status_string(s) for s in range(6)}
    assert len(seen) == 6 and all(seen)
    assert B.status_string(99)


def test_probe_argument_checks(L):
    assert L.mdnn_mfma_peak_probe(None, 1, 1, 1, None, None) == B.MDNN_ENULL
    assert L.mdnn_mfma_peak_probe(FAKE, 0, 1, 1, None, None) == B.MDNN_EINVAL
    assert L.mdnn_mfma_peak_probe(FAKE, 1, 5, 1, None, None) == B.MDNN_EINVAL
    assert L.mdnn_mfma_peak_probe(FAKE, 1, 1, 0, None, None) == B.MDNN_EINVAL


def test_tensor_wrapper_refuses_cpu_tensors(L):
    torch = pytest.importorskip("torch")
    with pytest.raises(ValueError):
        B.mdnn_conv_fprop(torch.zeros(2, 4, 4, 4), torch.zeros(2, 3, 3, 4), 1, 1)
