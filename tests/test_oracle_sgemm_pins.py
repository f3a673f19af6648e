"""CPU-only pins of the oracle's plain matrix product c = alpha * a^T b.

The paper (arXiv 1501.06633, Sections 3 and 4) calibrates its convolution
against SGEMM: the per-coordinate patch x filter-matrix product is a matrix
multiply, and with a 1 x 1 filter the whole convolution is one.  The pins are
a hand-worked 2 x 2 x 3 case (chosen so that a transposed operand gives other
numbers), the library's float64 matmul, identity operands, the already pinned
forward-convolution oracle at Sk = 1, and planted mistakes in a copy of the
source.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest


def test_hand_worked_case(oracle_mod):
    # c[o][m] = sum_k a[k][o] * b[k][m]
    a = np.array([[1, 2], [3, 4]], np.float32)                 # K=2 x N=2
    b = np.array([[5, 6, 7], [8, 9, 10]], np.float32)          # K=2 x M=3
    c, ab = oracle_mod.sgemm_tn(a, b, 1.0)
    # row 0: 1*[5,6,7] + 3*[8,9,10]; row 1: 2*[5,6,7] + 4*[8,9,10]
    assert c.tolist() == [[29, 33, 37], [42, 48, 54]]
    assert ab.tolist() == [[29, 33, 37], [42, 48, 54]]
    # the untransposed product a.b would have been [[21,24,27],[47,54,61]]
    c2 = oracle_mod.sgemm_tn(a, -b, 0.5, want_abs=False)
    assert c2.tolist() == [[-14.5, -16.5, -18.5], [-21, -24, -27]]


@pytest.mark.parametrize("N,M,K", [(1, 1, 1), (3, 5, 7), (7, 3, 5), (5, 7, 3), (33, 130, 65), (96, 257, 19)])
def test_matches_float64_matmul(oracle_mod, N, M, K):
    rng = np.random.default_rng(N * 1000 + M * 10 + K)
    a = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    b = rng.uniform(-1, 1, (K, M)).astype(np.float32)
    c, ab = oracle_mod.sgemm_tn(a, b, 0.75)
    want = 0.75 * (a.astype(np.float64).T @ b.astype(np.float64))
    want_ab = np.abs(a.astype(np.float64)).T @ np.abs(b.astype(np.float64))
    # one rounding to fp32 of a float64 sum: half an ulp plus the float64 sum's own error
    np.testing.assert_allclose(c, want, rtol=2.0 ** -23, atol=1e-12)
    np.testing.assert_allclose(ab, want_ab, rtol=1e-12)
    assert np.array_equal(c, oracle_mod.sgemm_tn(a, b, 0.75, want_abs=False, nthreads=1))


def test_identity_operands(oracle_mod):
    rng = np.random.default_rng(5)
    b = rng.normal(size=(6, 11)).astype(np.float32)
    assert np.array_equal(oracle_mod.sgemm_tn(np.eye(6, dtype=np.float32), b, 1.0, want_abs=False), b)
    a = rng.normal(size=(6, 4)).astype(np.float32)
    assert np.array_equal(oracle_mod.sgemm_tn(a, np.eye(6, dtype=np.float32), 1.0, want_abs=False), a.T)
    # a rectangular "selector": row k of b lands in row perm[k] of c
    sel = np.zeros((3, 5), np.float32)
    sel[0, 4] = sel[1, 0] = sel[2, 2] = 1
    c = oracle_mod.sgemm_tn(sel, b[:3], 2.0, want_abs=False)
    assert np.array_equal(c[4], 2 * b[0]) and np.array_equal(c[0], 2 * b[1]) and np.array_equal(c[2], 2 * b[2])
    assert not c[1].any() and not c[3].any()


@pytest.mark.parametrize("Nb,Hi,Wi,Nc,No", [(4, 3, 5, 7, 6), (1, 1, 1, 9, 2), (8, 2, 2, 3, 5)])
def test_is_the_forward_convolution_with_a_1x1_filter(oracle_mod, Nb, Hi, Wi, Nc, No):
    rng = np.random.default_rng(Nb + Hi + Nc)
    inp = rng.uniform(-1, 1, (Nc, Hi, Wi, Nb)).astype(np.float32)
    filt = rng.uniform(-1, 1, (Nc, 1, 1, No)).astype(np.float32)
    out, ab = oracle_mod.conv_fprop(inp, filt, 1, 0, 1.25)
    c, ab2 = oracle_mod.sgemm_tn(filt.reshape(Nc, No), inp.reshape(Nc, Hi * Wi * Nb), 1.25)
    assert np.array_equal(out.reshape(No, -1), c)
    assert np.array_equal(ab.reshape(No, -1), ab2)


def test_exact_on_integers(oracle_mod):
    rng = np.random.default_rng(9)
    a = rng.integers(-8, 9, (40, 12)).astype(np.float32)
    b = rng.integers(-8, 9, (40, 21)).astype(np.float32)
    c = oracle_mod.sgemm_tn(a, b, 1.0, want_abs=False)
    assert np.array_equal(c.astype(np.int64), a.astype(np.int64).T @ b.astype(np.int64))


def test_rejects_bad_arguments(oracle_mod):
    a = np.zeros((3, 4), np.float32)
    with pytest.raises(ValueError):
        oracle_mod.sgemm_tn(a, np.zeros((4, 4), np.float32), 1.0)
    with pytest.raises(ValueError):
        oracle_mod.sgemm_tn(a.astype(np.float64), np.zeros((3, 4), np.float32), 1.0)
    with pytest.raises(ValueError):
        oracle_mod.sgemm_tn(a.T, np.zeros((4, 4), np.float32), 1.0)          # not contiguous


# ---- planted mistakes, in a copy of the source, on the CPU -------------------------------
SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "mdnn_oracle.c")
_ANCHOR = "int mdnn_oracle_sgemm_tn(const float* a"

MUTATIONS = {
    "a_not_transposed": ("a[(size_t)k * N + o]", "a[(size_t)o * K + k]"),
    "b_transposed":     ("b[(size_t)k * M + m]", "b[(size_t)m * K + k]"),
    "c_transposed":     ("c[(size_t)o * M + m] =", "c[(size_t)m * N + o] ="),
    "alpha_dropped":    ("(float)((double)alpha * s)", "(float)s"),
    "last_k_dropped":   ("for (int k = 0; k < K; ++k)", "for (int k = 0; k < K - 1; ++k)"),
    "float_products":   ("double p = (double)a[(size_t)k * N + o] * (double)b[(size_t)k * M + m];",
                         "float pf = a[(size_t)k * N + o] * b[(size_t)k * M + m]; double p = pf;"),
}


def _run_copy(so, a, b, alpha):
    lib = ctypes.CDLL(str(so))
    i, f, p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
    lib.mdnn_oracle_sgemm_tn.argtypes = [p, p, p, p, i, i, i, f, i]
    lib.mdnn_oracle_sgemm_tn.restype = i
    K, N = a.shape
    M = b.shape[1]
    c = np.full((N, M), np.nan, np.float32)
    assert lib.mdnn_oracle_sgemm_tn(a.ctypes.data, b.ctypes.data, c.ctypes.data, None, N, M, K, alpha, 1) == 0
    return c


def _mut_inputs():
    rng = np.random.default_rng(31)
    # square on purpose: the transposed-operand mutations then stay inside the buffers
    a = rng.uniform(-1, 1, (6, 6)).astype(np.float32)
    b = rng.uniform(-1, 1, (6, 6)).astype(np.float32)
    return a, b, 0.75 * (a.astype(np.float64).T @ b.astype(np.float64))


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    head, body = text.split(_ANCHOR, 1)
    assert body.count(old) >= 1, f"mutation anchor for {name} no longer in the oracle source"
    c = tmp_path / "mut.c"
    so = tmp_path / "mut.so"
    c.write_text(head + _ANCHOR + body.replace(old, new, 1))
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    a, b, want = _mut_inputs()
    got = _run_copy(so, a, b, 0.75)
    # the float64 pin's own bar: one fp32 rounding of the exact sum
    assert not np.allclose(got, want, rtol=2.0 ** -23, atol=1e-12), f"the matmul pin did not notice mutation {name}"


def test_unmutated_copy_passes(tmp_path):
    so = tmp_path / "same.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(so), SRC, "-lm"], check=True)
    a, b, want = _mut_inputs()
    np.testing.assert_allclose(_run_copy(so, a, b, 0.75), want, rtol=2.0 ** -23, atol=1e-12)
