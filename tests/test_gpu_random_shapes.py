"""Seeded random small shapes through all three entry points, integer data, bit for bit against
the oracle: batch sizes that take the 16-byte, the per-lane and the 4-byte copy paths, filter
counts around every tile width, strides 1-4, pads from 0 to Sk."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_bitwise(seed):
    import torch
    from paper_1501_06633_amd import binding as B
    import oracle

    rng = np.random.default_rng(seed)
    done = 0
    for it in range(120):
        Nb = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 20, 32, 48, 64]))
        Sk = int(rng.integers(1, 8))
        stride = int(rng.integers(1, 5))
        pad = int(rng.integers(0, Sk + 1))
        Hi = int(rng.integers(max(1, Sk - 2 * pad), 30))
        Wi = int(rng.integers(max(1, Sk - 2 * pad), 30))
        Nc = int(rng.integers(1, 24))
        No = int(rng.choice([1, 2, 3, 4, 8, 12, 31, 32, 33, 64, 65, 96, 97, 128, 130, 140]))
        alpha = float(rng.choice([1.0, 0.5, -2.0]))
        Wo, Ho = oracle.out_dims(Wi, Hi, Sk, stride, pad)
        x = rng.integers(-4, 5, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
        w = rng.integers(-4, 5, size=(Nc, Sk, Sk, No)).astype(np.float32)
        g = rng.integers(-4, 5, size=(No, Ho, Wo, Nb)).astype(np.float32)
        d_x, d_w, d_g = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(g).cuda()
        what = f"seed={seed} case={it} Nb={Nb} Hi={Hi} Wi={Wi} Nc={Nc} No={No} Sk={Sk} stride={stride} pad={pad} alpha={alpha}"
        print(what, flush=True)
        y = B.mdnn_conv_fprop(d_x, d_w, stride, pad, alpha)
        dw = B.mdnn_conv_bprop_filter(d_x, d_g, Sk, stride, pad, alpha)
        dx = B.mdnn_conv_bprop_data(d_g, d_w, (Hi, Wi), stride, pad, alpha)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y.cpu().numpy(), oracle.conv_fprop(x, w, stride, pad, alpha, want_abs=False), err_msg=what)
        np.testing.assert_array_equal(dw.cpu().numpy(), oracle.conv_bprop_filter(x, g, Sk, stride, pad, alpha, want_abs=False),
                                      err_msg=what)
        np.testing.assert_array_equal(dx.cpu().numpy(),
                                      oracle.conv_bprop_data(g, w, (Hi, Wi), stride, pad, alpha, want_abs=False), err_msg=what)
        done += 1
    assert done == 120


def test_long_contractions_every_variant_bitwise():
    """Forty seeded shapes with K = Nc*Sk*Sk between 700 and 7000 (beyond every variant's LDS
    table, so the contraction is walked in several table fills) on small images, through every
    tile variant: integer data, bit for bit against the oracle."""
    import torch
    from paper_1501_06633_amd import binding as B
    import oracle

    rng = np.random.default_rng(2025)
    runs = 0
    for it in range(40):
        Nb = int(rng.choice([4, 8, 12, 16, 32, 64]))
        Sk = int(rng.choice([1, 2, 3, 5]))
        stride = int(rng.integers(1, 3))
        pad = int(rng.integers(0, Sk))
        Hi = int(rng.integers(Sk, 9))
        Wi = int(rng.integers(Sk, 9))
        Nc = max(1, int(rng.integers(700, 7000)) // (Sk * Sk))
        No = int(rng.choice([4, 32, 36, 64, 96, 100, 128, 192, 260]))
        alpha = float(rng.choice([1.0, 0.5]))
        x = rng.integers(-4, 5, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
        w = rng.integers(-4, 5, size=(Nc, Sk, Sk, No)).astype(np.float32)
        want = oracle.conv_fprop(x, w, stride, pad, alpha, want_abs=False)
        d_x, d_w = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        what = f"case={it} Nb={Nb} Hi={Hi} Wi={Wi} Nc={Nc} No={No} Sk={Sk} stride={stride} pad={pad} alpha={alpha}"
        print(what, flush=True)
        for v in B.mdnn_variant_names():
            y = B.mdnn_conv_fprop(d_x, d_w, stride, pad, alpha, variant=v)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(y.cpu().numpy(), want, err_msg=f"{what} variant={v}")
            runs += 1
    assert runs == 40 * len(B.mdnn_variant_names())


def test_pinned_cuts_on_random_shapes_bitwise():
    """Thirty seeded mid-size shapes whose tiles are all cut, or whose last round is cut, in every way
    a kernel offers (halves, 48 + 48 + 32-row thirds, quarters, 16-row eighths, pairings of two sizes;
    pinned through the variant name):
    ragged filter counts, ragged column counts, pads and strides, integer data, bit for bit."""
    import torch
    from paper_1501_06633_amd import binding as B
    import oracle

    pinned = ["o128m128:H", "o128m128:T", "o128m128:Q", "o128m128:t", "o128m128k8:H", "o128m128k8:Q",
              "o96m256:H", "o96m256:h", "o96m256:Q", "o96m256:q",
              "o128m128a:H", "o128m128a:Q", "o128m128b:H", "o128m128b:Q", "o128m128k8a:Q", "o128m128k8a:h", "o128m128k8b:Q", "o128m128k8b:q", "o128m128s:H", "o128m128s:Q", "o128m128k8:m", "o128m128k8:n", "o128m128k8:p", "o128m128k8:E", "o128m128:e", "o64m256k8:H", "o64m256k8:Q", "o64m256k8:q", "o48m128:w", "o64m512:w"]
    rng = np.random.default_rng(4096)
    runs = paired = 0
    for it in range(30):
        Nb = int(rng.choice([4, 8, 16, 32, 64]))
        Sk = int(rng.choice([1, 3, 3, 5]))
        stride = int(rng.integers(1, 3))
        pad = int(rng.integers(0, Sk))
        Hi = int(rng.integers(max(Sk, 6), 20))
        Wi = int(rng.integers(max(Sk, 6), 20))
        Nc = int(rng.integers(1, 12))
        No = int(rng.choice([40, 100, 128, 132, 200, 256, 300]))
        alpha = float(rng.choice([1.0, 0.5]))
        x = rng.integers(-4, 5, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
        w = rng.integers(-4, 5, size=(Nc, Sk, Sk, No)).astype(np.float32)
        want = oracle.conv_fprop(x, w, stride, pad, alpha, want_abs=False)
        d_x, d_w = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        what = f"case={it} Nb={Nb} Hi={Hi} Wi={Wi} Nc={Nc} No={No} Sk={Sk} stride={stride} pad={pad} alpha={alpha}"
        print(what, flush=True)
        for v in pinned:
            pairing = {"m": (128, 192), "n": (128, 160), "p": (64, 96)}.get(v[-1]) if ":" in v else None
            if pairing:                   # a pairing of two piece sizes exists for a range of left-over tiles only
                r = B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad, v.split(":")[0])["tiles"] % 256
                if not pairing[0] < r <= pairing[1]:
                    runs += 1
                    continue
                paired += 1
            y = B.mdnn_conv_fprop(d_x, d_w, stride, pad, alpha, variant=v)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(y.cpu().numpy(), want, err_msg=f"{what} variant={v}")
            runs += 1
    assert runs == 30 * len(pinned) and paired >= 3


def test_default_plans_with_one_to_five_rounds_of_tiles_bitwise():
    """Sixty seeded shapes whose 128 x 128 tile count lies between one and five rounds of 256, with
    the variant and the tail cut left to the library: halves, thirds, quarters, eighths, chains and
    the pairings of two piece sizes all occur (asserted), filter tiles are ragged in a third of the
    shapes, and the forward result and the data gradient (the same kernels on the turned-over
    bank) must match the oracle bit for bit on integer data."""
    import torch
    from paper_1501_06633_amd import binding as B
    import oracle

    rng = np.random.default_rng(2718)
    seen = set()
    for it in range(60):
        Nb = int(rng.choice([32, 64, 128]))
        No = int(rng.choice([128, 128, 200, 256, 256, 384]))
        want_tiles = int(rng.integers(257, 1300))
        col_tiles = max(1, want_tiles // -(-No // 128))
        pixels = max(1, col_tiles * 128 // Nb)
        Ho = int(rng.integers(1, 24))
        Wo = max(1, pixels // Ho)
        Sk = int(rng.choice([1, 3]))
        pad = int(rng.integers(0, Sk))
        Hi, Wi = Ho + Sk - 1 - 2 * pad, Wo + Sk - 1 - 2 * pad
        if Hi < 1 or Wi < 1:
            Hi, Wi, pad = Ho + Sk - 1, Wo + Sk - 1, 0
        Nc = int(rng.integers(1, 5))
        alpha = float(rng.choice([1.0, 0.5]))
        plan = B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, 1, pad)
        cut = tuple(k for k in ("halved", "thirded", "quartered", "eighthed") if plan[k])
        seen.add((plan["variant"], cut, plan["pieces_first"] > 0, plan["pieces"] > plan["pieces_first"]))
        x = rng.integers(-4, 5, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
        w = rng.integers(-4, 5, size=(Nc, Sk, Sk, No)).astype(np.float32)
        g = rng.integers(-4, 5, size=(No, plan["M"] // Nb // (Wi + 2 * pad - Sk + 1), Wi + 2 * pad - Sk + 1, Nb)).astype(np.float32)
        what = f"case={it} Nb={Nb} Hi={Hi} Wi={Wi} Nc={Nc} No={No} Sk={Sk} pad={pad} alpha={alpha} plan={plan}"
        print(what, flush=True)
        d_x, d_w, d_g = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(g).cuda()
        y = B.mdnn_conv_fprop(d_x, d_w, 1, pad, alpha)
        dx = B.mdnn_conv_bprop_data(d_g, d_w, (Hi, Wi), 1, pad, alpha)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y.cpu().numpy(), oracle.conv_fprop(x, w, 1, pad, alpha, want_abs=False), err_msg=what)
        np.testing.assert_array_equal(dx.cpu().numpy(), oracle.conv_bprop_data(g, w, (Hi, Wi), 1, pad, alpha, want_abs=False),
                                      err_msg=what)
    cuts = {c for _, c, _, _ in seen}
    for need in [("halved",), ("quartered",), ("eighthed",), ("thirded",), ("halved", "eighthed"), ("halved", "quartered")]:
        assert need in cuts, (need, sorted(cuts))
    assert any(first and behind for _, _, first, behind in seen)      # pieces in front of and behind the whole tiles


def test_default_plans_with_sizes_off_the_multiple_of_four_bitwise():
    """Forty seeded shapes with one to four rounds of 128 x 128 tiles whose minibatch, filter count
    or both are no multiples of 4, under the library's own plan: the tiles with one or both
    operands in 4-byte copies, their half and quarter pieces and ragged filter tiles all occur
    (asserted); forward result and data gradient bit for bit on integer data."""
    import torch
    from paper_1501_06633_amd import binding as B
    import oracle

    rng = np.random.default_rng(31415)
    seen = set()
    for it in range(40):
        kind = it % 3                                       # 0: only No odd, 1: only Nb, 2: both
        Nb = int(rng.choice([32, 64]) if kind == 0 else rng.choice([6, 30, 50, 66]))
        No = int(rng.choice([128, 256]) if kind == 1 else rng.choice([130, 202, 250, 257]))
        want_tiles = int(rng.integers(257, 1100))
        col_tiles = max(1, want_tiles // -(-No // 128))
        pixels = max(1, col_tiles * 128 // Nb)
        Ho = int(rng.integers(1, 24))
        Wo = max(1, pixels // Ho)
        Sk = int(rng.choice([1, 3]))
        pad = int(rng.integers(0, Sk))
        Hi, Wi = Ho + Sk - 1 - 2 * pad, Wo + Sk - 1 - 2 * pad
        if Hi < 1 or Wi < 1:
            Hi, Wi, pad = Ho + Sk - 1, Wo + Sk - 1, 0
        Nc = int(rng.integers(1, 4))
        alpha = float(rng.choice([1.0, 0.5]))
        plan = B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, 1, pad)
        cut = tuple(k for k in ("halved", "thirded", "quartered", "eighthed") if plan[k])
        seen.add((plan["variant"], cut))
        Wo2 = Wi + 2 * pad - Sk + 1
        Ho2 = Hi + 2 * pad - Sk + 1
        x = rng.integers(-4, 5, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
        w = rng.integers(-4, 5, size=(Nc, Sk, Sk, No)).astype(np.float32)
        g = rng.integers(-4, 5, size=(No, Ho2, Wo2, Nb)).astype(np.float32)
        what = f"case={it} Nb={Nb} Hi={Hi} Wi={Wi} Nc={Nc} No={No} Sk={Sk} pad={pad} alpha={alpha} plan={plan}"
        print(what, flush=True)
        d_x, d_w, d_g = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(g).cuda()
        y = B.mdnn_conv_fprop(d_x, d_w, 1, pad, alpha)
        dx = B.mdnn_conv_bprop_data(d_g, d_w, (Hi, Wi), 1, pad, alpha)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y.cpu().numpy(), oracle.conv_fprop(x, w, 1, pad, alpha, want_abs=False), err_msg=what)
        np.testing.assert_array_equal(dx.cpu().numpy(), oracle.conv_bprop_data(g, w, (Hi, Wi), 1, pad, alpha, want_abs=False),
                                      err_msg=what)
    variants = {v for v, _ in seen}
    assert {"o128m128k8a", "o128m128k8b", "o128m128s"} <= variants or {"o128m128a", "o128m128b", "o128m128s"} <= variants, sorted(seen)
    assert any(c for v, c in seen if v[-1] in "ab") and any(c for v, c in seen if v == "o128m128s"), sorted(seen)


def test_mid_size_random_shapes_all_three_calls_bitwise():
    """Seventy seeded shapes with a hundred to a few thousand tiles -- minibatches 30, 32, 50, 64, 100
    and 128, 64 to 512 filters, 1x1 to 5x5, strides 1 and 2, pads up to Sk + 1 -- through the forward
    call and both gradients under the library's own plans (whatever tail cut, copy width and
    workspace split they take), integer data, bit for bit."""
    import torch
    from paper_1501_06633_amd import binding as B
    import oracle

    rng = np.random.default_rng(21)
    cuts = set()
    for it in range(70):
        Nb = int(rng.choice([32, 64, 128, 50, 30, 100]))
        Sk = int(rng.choice([1, 3, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 1, 2]))
        pad = int(rng.integers(0, Sk + 2))
        Hi, Wi = int(rng.integers(12, 44)), int(rng.integers(12, 44))
        Nc = int(rng.integers(1, 7))
        No = int(rng.choice([64, 96, 128, 192, 250, 256, 384, 512]))
        alpha = float(rng.choice([1.0, 0.5]))
        Wo, Ho = oracle.out_dims(Wi, Hi, Sk, stride, pad)
        x = rng.integers(-4, 5, size=(Nc, Hi, Wi, Nb)).astype(np.float32)
        w = rng.integers(-4, 5, size=(Nc, Sk, Sk, No)).astype(np.float32)
        g = rng.integers(-4, 5, size=(No, Ho, Wo, Nb)).astype(np.float32)
        d_x, d_w, d_g = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(g).cuda()
        plan = B.mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, stride, pad)
        what = (f"case={it} Nb={Nb} Hi={Hi} Wi={Wi} Nc={Nc} No={No} Sk={Sk} stride={stride} pad={pad} alpha={alpha} "
                f"variant={plan['variant']} tiles={plan['tiles']}")
        print(what, flush=True)
        cuts.add((plan["variant"], plan["halved"] > 0, plan["thirded"] > 0, plan["quartered"] > 0, plan["eighthed"] > 0))
        y = B.mdnn_conv_fprop(d_x, d_w, stride, pad, alpha)
        dw = B.mdnn_conv_bprop_filter(d_x, d_g, Sk, stride, pad, alpha)
        dx = B.mdnn_conv_bprop_data(d_g, d_w, (Hi, Wi), stride, pad, alpha)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y.cpu().numpy(), oracle.conv_fprop(x, w, stride, pad, alpha, want_abs=False), err_msg=what)
        np.testing.assert_array_equal(dw.cpu().numpy(), oracle.conv_bprop_filter(x, g, Sk, stride, pad, alpha, want_abs=False),
                                      err_msg=what)
        np.testing.assert_array_equal(dx.cpu().numpy(),
                                      oracle.conv_bprop_data(g, w, (Hi, Wi), stride, pad, alpha, want_abs=False), err_msg=what)
    assert len(cuts) >= 8, cuts          # the seed really spreads over kernels and cuts
