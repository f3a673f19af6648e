"""The allocation-free data-gradient entry point (mdnn_conv_bprop_data_static) against the
workspace entry point it is a variant of (mdnn_conv_bprop_data), through the C ABI: same kernels,
same plan, so the two results must be equal bit for bit; and against the oracle to the usual
bound.  Two calls in a row on the same GPU, the second with a smaller problem (the static array
still holds the first call's bank), then a strided layer (whose per-class results go straight
to the result tensor), then the size limit."""
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


def both_ways(env, L, seed):
    """din by the workspace call and by the static call, on the same seeded data."""
    torch, B, oracle = env
    Wo, Ho = oracle.out_dims(L.Wi, L.Hi, L.Sk, L.stride, L.pad)
    rng = np.random.Generator(np.random.PCG64(seed))
    dout = rng.standard_normal(size=(L.No, Ho, Wo, L.Nb), dtype=np.float32)
    _, filt = W.make_inputs(L)
    d_g, d_f = torch.from_numpy(dout).cuda(), torch.from_numpy(filt).cuda()
    ref = B.mdnn_conv_bprop_data(d_g, d_f, (L.Hi, L.Wi), L.stride, L.pad, L.alpha)
    din = torch.full((L.Nc, L.Hi, L.Wi, L.Nb), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.mdnn_conv_bprop_data_static(d_g, d_f, (L.Hi, L.Wi), L.stride, L.pad, L.alpha, din)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return dout, filt, ref.cpu().numpy(), din.cpu().numpy()


def check_oracle(env, L, dout, filt, got, what):
    _, _, oracle = env
    want, absum = oracle.conv_bprop_data(dout, filt, (L.Hi, L.Wi), L.stride, L.pad, L.alpha)
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    scale = abs(L.alpha) * absum
    zero = scale == 0
    assert (got[zero] == 0).all(), what
    ratio = np.zeros_like(err)
    np.divide(err, scale, out=ratio, where=~zero)
    worst = float(ratio.max())
    say(f"    {what}: max |err|/(|alpha| A) = {worst:.3e} over {got.size} elements")
    assert worst <= LOOSE and worst <= TIGHT, f"{what}: {worst:.3e}"


def test_two_calls_in_a_row_second_smaller(env):
    big = W.LAYERS["conv3"]                                    # bank 3.5 MB
    small = W.custom("small_after_big", 8, 9, 11, 12, 20, 3, 1, 1, 0.5, seed=W.SEED_BASE + 4242)
    for L, seed in ((big, 11), (small, 12)):
        say(f"[no-alloc] static data gradient, layer={L.name} dims={L.dims()}")
        dout, filt, ref, got = both_ways(env, L, seed)
        assert np.isfinite(got).all()
        assert np.array_equal(ref.view(np.uint32), got.view(np.uint32)), f"{L.name}: differs from the workspace call"
        check_oracle(env, L, dout, filt, got, L.name)


def test_strided_layer_results_in_static_array(env):
    """Stride 2: the residue-class filter bank lives in the static array and the results are
    scattered into din; then a smaller stride-1 call right after it."""
    strided = W.custom("static_strided", 16, 21, 19, 8, 24, 5, 2, 1, 1.0, seed=W.SEED_BASE + 4243)
    after = W.custom("static_after", 4, 7, 7, 4, 8, 3, 1, 0, 2.0, seed=W.SEED_BASE + 4244)
    for L, seed in ((strided, 13), (after, 14)):
        say(f"[no-alloc] static data gradient, layer={L.name} dims={L.dims()}")
        dout, filt, ref, got = both_ways(env, L, seed)
        assert np.array_equal(ref.view(np.uint32), got.view(np.uint32)), f"{L.name}: differs from the workspace call"
        check_oracle(env, L, dout, filt, got, L.name)


def test_limit_is_an_error_not_a_launch(env):
    """A problem whose workspace exceeds the static array is refused before anything is enqueued."""
    torch, B, _ = env
    L = W.custom("bank_45_mib", 128, 12, 12, 1024, 1280, 3, 1, 1)
    st, need = B.mdnn_conv_bprop_data_workspace(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    assert st == 0 and need > B.MDNN_STATIC_SCRATCH_BYTES
    tiny = torch.zeros(64, device="cuda")
    st = B.lib().mdnn_conv_bprop_data_static(tiny.data_ptr(), tiny.data_ptr(), tiny.data_ptr(),
                                             L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad, 1.0, None)
    assert st == B.MDNN_ETOOBIG
