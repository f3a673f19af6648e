"""GPU parity of the plain matrix product c = alpha * a^T b (the SGEMM the paper's
conclusion measures the convolution against; Section 3's product for a 1 x 1
filter), called through the C ABI, against the CPU oracle.

Bar: |gpu - oracle| <= 1e-4 * |alpha| * sum_k |a b| per element, and the fp32
regression bound 5e-6 as for the convolution; integer-valued operands bit for bit.
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


def run_gpu(env, a, b, alpha):
    torch, B, _ = env
    c = B.mdnn_sgemm_tn(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), alpha)
    torch.cuda.synchronize()
    return c.cpu().numpy()


def check(got, want, absum, alpha, what):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    scale = abs(alpha) * absum
    zero = scale == 0
    assert (got[zero] == 0).all(), f"{what}: non-zero where every product is zero"
    ratio = np.zeros_like(err)
    np.divide(err, scale, out=ratio, where=~zero)
    worst = float(ratio.max()) if ratio.size else 0.0
    say(f"    {what}: max |err|/(|alpha| A) = {worst:.3e} over {got.size} elements")
    assert np.isfinite(got).all()
    assert worst <= LOOSE, f"{what}: acceptance bound exceeded ({worst:.3e})"
    assert worst <= TIGHT, f"{what}: fp32-accumulation regression bound exceeded ({worst:.3e})"


# several tiles plus ragged tails in every dimension; K not a multiple of the slab; N or M not a
# multiple of 4 (the scalar-load variant); one row / one column / one term
SHAPES = [
    (256, 512, 128), (384, 1000, 333), (100, 260, 77), (96, 3072, 363), (33, 129, 65),
    (1, 1, 1), (1, 700, 50), (300, 1, 40), (7, 5, 3), (130, 258, 1), (64, 4096, 600),
    (512, 200, 4100),                       # K beyond one offset-table fill
]


@pytest.mark.parametrize("N,M,K", SHAPES)
def test_matches_oracle_everywhere(env, N, M, K):
    _, _, oracle = env
    say(f"[sgemm] N={N} M={M} K={K}")
    a, b = W.make_matrices(N, M, K, seed=N + M + K)
    alpha = 0.75
    got = run_gpu(env, a, b, alpha)
    want, absum = oracle.sgemm_tn(a, b, alpha)
    assert got.shape == want.shape
    check(got, want, absum, alpha, f"{N}x{M}x{K}")


@pytest.mark.parametrize("N,M,K", [(256, 1024, 512), (100, 260, 77), (97, 131, 300)])
def test_integer_operands_bitwise(env, N, M, K):
    _, _, oracle = env
    say(f"[sgemm int] N={N} M={M} K={K}")
    a, b = W.make_matrices(N, M, K, seed=5, integer=True)
    got = run_gpu(env, a, b, 1.0)
    want = oracle.sgemm_tn(a, b, 1.0, want_abs=False)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("N,M,K", [(4096, 4096, 4096), (4096, 16384, 2304)])
def test_bench_sizes_on_sampled_rows_and_columns(env, N, M, K):
    """The sizes bench.py --sgemm times: the oracle computes a random 48 x 64 sub-matrix
    (sampled columns of a and of b), which must match the same elements of the GPU result."""
    _, _, oracle = env
    say(f"[sgemm sampled] N={N} M={M} K={K}")
    a, b = W.make_matrices(N, M, K, seed=11)
    got = run_gpu(env, a, b, 1.0)
    rng = np.random.default_rng(N + M)
    rows = np.unique(np.concatenate([rng.integers(0, N, 44), [0, N - 1, 127, 128]]))
    cols = np.unique(np.concatenate([rng.integers(0, M, 60), [0, M - 1, 255, 256]]))
    want, absum = oracle.sgemm_tn(np.ascontiguousarray(a[:, rows]), np.ascontiguousarray(b[:, cols]), 1.0)
    check(got[np.ix_(rows, cols)], want, absum, 1.0, f"{N}x{M}x{K} sampled")
    assert np.isfinite(got).all()


def test_equals_the_1x1_convolution_bitwise(env):
    """Same kernel, same tiling: the product and the 1 x 1 convolution of the same data agree bit for bit."""
    torch, B, _ = env
    Nb, Hi, Wi, Nc, No = 64, 6, 5, 200, 96
    L = W.custom("one_by_one", Nb, Hi, Wi, Nc, No, 1, 1, 0)
    inp, filt = W.make_inputs(L)
    d_in, d_f = torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda()
    out = B.mdnn_conv_fprop(d_in, d_f, 1, 0, 1.0)
    c = B.mdnn_sgemm_tn(d_f.reshape(Nc, No), d_in.reshape(Nc, Hi * Wi * Nb), 1.0)
    torch.cuda.synchronize()
    # tile boundaries fall on the same flat columns, so the summation order is the same
    assert torch.equal(out.reshape(No, -1), c)


def test_argument_errors(env):
    torch, B, _ = env
    a = torch.zeros((8, 4), device="cuda")
    b = torch.zeros((8, 12), device="cuda")
    with pytest.raises(ValueError):
        B.mdnn_sgemm_tn(a, torch.zeros((9, 12), device="cuda"))
    with pytest.raises(ValueError):
        B.mdnn_sgemm_tn(a, b, c=torch.zeros((12, 4), device="cuda"))
    with pytest.raises(ValueError):
        B.mdnn_sgemm_tn(a.cpu(), b)
    c = B.mdnn_sgemm_tn(a, b)
    torch.cuda.synchronize()
    assert c.shape == (4, 12) and not c.any()
