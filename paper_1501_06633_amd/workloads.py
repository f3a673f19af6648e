"""Seeded synthetic layer workloads: shapes and input tensors only.

This module holds none of the convolution's arithmetic (not even the output
size): it names layer geometries and draws input / filter values.  Both the
GPU parity tests and the CPU oracle's tests take their data from here so that
the two sides see the same bytes.

The five named layers follow the usual AlexNet / VGG layer geometries (image
-like dense first layer, post-ReLU-like half-zero activations afterwards,
small zero-mean Gaussian weights); they stand in for trained networks, which
are not needed to time or check a convolution.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np

SEED_BASE = 150106633


@dataclass(frozen=True)
class Layer:
    name: str
    Nb: int
    Hi: int
    Wi: int
    Nc: int
    No: int
    Sk: int
    stride: int
    pad: int
    alpha: float
    in_dist: str      # "uniform_pm1" | "uniform01" | "uniform01_relu"
    filt_dist: str    # "uniform_pm1" | "normal_0p01"
    seed: int

    def dims(self) -> dict:
        d = asdict(self)
        return {k: d[k] for k in ("Nb", "Hi", "Wi", "Nc", "No", "Sk", "stride", "pad", "alpha")}


LAYERS = {
    "tiny":  Layer("tiny",    8,  32,  32,  16,  32,  3, 1, 1, 1.0, "uniform_pm1",    "uniform_pm1", SEED_BASE + 0),
    "conv1": Layer("conv1", 128, 227, 227,   3,  96, 11, 4, 0, 1.0, "uniform01",      "normal_0p01", SEED_BASE + 1),
    "conv2": Layer("conv2", 128,  27,  27,  96, 256,  5, 1, 2, 1.0, "uniform01_relu", "normal_0p01", SEED_BASE + 2),
    "conv3": Layer("conv3", 128,  13,  13, 256, 384,  3, 1, 1, 1.0, "uniform01_relu", "normal_0p01", SEED_BASE + 3),
    "vgg":   Layer("vgg",    64,  56,  56, 256, 256,  3, 1, 1, 0.5, "uniform01_relu", "normal_0p01", SEED_BASE + 4),
}
ORDER = ("tiny", "conv1", "conv2", "conv3", "vgg")


# The ten layer shapes of the paper's Table 1 (FPROP, minibatch 128).  Input size,
# channels, output size, filter count and filter size are the paper's; it prints
# neither stride nor pad, the values here are the ones that map the printed input
# size to the printed output size under the floor formula (customary AlexNet-v2 /
# OverFeat-fast definitions).  `paper_ce` is the paper's maxDNN computational
# efficiency on a GTX 980 (Table 1, last column): context for a table, never a target.
TABLE1 = {}
for _i, (_name, _wi, _nc, _no, _sk, _st, _pad, _ce) in enumerate([
        ("alexnet_v2.conv1", 224,    3,   64, 11, 4, 2, 93.4),
        ("alexnet_v2.conv2",  27,   64,  192,  5, 1, 2, 95.5),
        ("alexnet_v2.conv3",  13,  192,  384,  3, 1, 1, 95.1),
        ("alexnet_v2.conv4",  13,  384,  256,  3, 1, 1, 95.0),
        ("alexnet_v2.conv5",  13,  256,  256,  3, 1, 1, 94.6),
        ("overfeat.L1",      231,    3,   96, 11, 4, 0, 70.3),
        ("overfeat.L2",       24,   96,  256,  5, 1, 0, 95.6),
        ("overfeat.L3",       12,  256,  512,  3, 1, 1, 94.4),
        ("overfeat.L4",       12,  512, 1024,  3, 1, 1, 96.2),
        ("overfeat.L5",       12, 1024, 1024,  3, 1, 1, 96.3)]):
    TABLE1[_name] = (Layer(_name, 128, _wi, _wi, _nc, _no, _sk, _st, _pad, 1.0,
                           "uniform01" if _nc == 3 else "uniform01_relu", "normal_0p01",
                           SEED_BASE + 50 + _i), _ce)


# The nine distinct 3x3 convolution shapes of a VGG-16 style network at minibatch 64 (the `vgg`
# benchmark layer is its 256 -> 256 layer at 56 x 56): a third workload, synthetic data only.
VGG16 = {}
for _i, (_name, _hw, _nc, _no) in enumerate([
        ("conv1_1", 224,   3,  64), ("conv1_2", 224,  64,  64),
        ("conv2_1", 112,  64, 128), ("conv2_2", 112, 128, 128),
        ("conv3_1",  56, 128, 256), ("conv3_2",  56, 256, 256),
        ("conv4_1",  28, 256, 512), ("conv4_2",  28, 512, 512),
        ("conv5_1",  14, 512, 512)]):
    VGG16[_name] = Layer("vgg16." + _name, 64, _hw, _hw, _nc, _no, 3, 1, 1, 1.0,
                         "uniform01", "normal_0p01", SEED_BASE + 80 + _i)


def custom(name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha=1.0,
           in_dist="uniform_pm1", filt_dist="uniform_pm1", seed=SEED_BASE + 1000) -> Layer:
    return Layer(name, Nb, Hi, Wi, Nc, No, Sk, stride, pad, alpha, in_dist, filt_dist, seed)


def make_inputs(layer: Layer):
    """Return (inp, filt): float32, C-contiguous, shapes (Nc,Hi,Wi,Nb) and
    (Nc,Sk,Sk,No).  Draw order: input values, zero mask (if any), filters."""
    rng = np.random.Generator(np.random.PCG64(layer.seed))
    ishape = (layer.Nc, layer.Hi, layer.Wi, layer.Nb)
    fshape = (layer.Nc, layer.Sk, layer.Sk, layer.No)
    if layer.in_dist == "uniform_pm1":
        inp = rng.uniform(-1.0, 1.0, size=ishape).astype(np.float32)
    elif layer.in_dist == "uniform01":
        inp = rng.random(size=ishape, dtype=np.float32)
    elif layer.in_dist == "uniform01_relu":
        inp = rng.random(size=ishape, dtype=np.float32)
        keep = rng.integers(0, 2, size=ishape, dtype=np.uint8)
        inp *= keep
    else:
        raise ValueError(layer.in_dist)
    if layer.filt_dist == "uniform_pm1":
        filt = rng.uniform(-1.0, 1.0, size=fshape).astype(np.float32)
    elif layer.filt_dist == "normal_0p01":
        filt = (rng.standard_normal(size=fshape, dtype=np.float32) * np.float32(0.01))
    else:
        raise ValueError(layer.filt_dist)
    return np.ascontiguousarray(inp), np.ascontiguousarray(filt)


def make_int_inputs(layer: Layer, lo=-4, hi=4):
    """Small-integer valued float32 tensors of the layer's shape: every partial
    sum stays below 2**24, so any summation order gives the same fp32 result."""
    rng = np.random.Generator(np.random.PCG64(layer.seed + 7919))
    ishape = (layer.Nc, layer.Hi, layer.Wi, layer.Nb)
    fshape = (layer.Nc, layer.Sk, layer.Sk, layer.No)
    inp = rng.integers(lo, hi + 1, size=ishape).astype(np.float32)
    filt = rng.integers(lo, hi + 1, size=fshape).astype(np.float32)
    return inp, filt


def make_matrices(N, M, K, seed, integer=False):
    """Operands of the plain matrix product c (N x M) = alpha * a^T b: a (K,N), b (K,M), float32.
    b is drawn like an activation (uniform in [-1, 1)), a like a filter matrix (normal, sigma 0.01);
    with ``integer`` both hold small integers so that every fp32 partial sum is exact."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + seed))
    if integer:
        b = rng.integers(-4, 5, size=(K, M)).astype(np.float32)
        a = rng.integers(-4, 5, size=(K, N)).astype(np.float32)
    else:
        b = rng.uniform(-1.0, 1.0, size=(K, M)).astype(np.float32)
        a = rng.standard_normal(size=(K, N), dtype=np.float32) * np.float32(0.01)
    return np.ascontiguousarray(a), np.ascontiguousarray(b)


def stratified_points(rows, cols, tile_rows, tile_cols, per_tile, seed):
    """Sample positions (row, col) of a rows x cols matrix so that every tile_rows x tile_cols tile of
    its tiling (ragged last tiles included) holds at least ``per_tile`` (>= 2) of them: the tile's
    first and last element, then uniform draws inside the tile.  Tiles are those of the coarsest
    launch grid; a test that wants every piece of a cut tile covered passes the piece's size.
    Returns an int64 array (npts, 2).  Index bookkeeping only: none of the method's arithmetic."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 7000 + seed))
    r0 = np.arange(0, rows, tile_rows, dtype=np.int64)
    c0 = np.arange(0, cols, tile_cols, dtype=np.int64)
    R0, C0 = np.meshgrid(r0, c0, indexing="ij")
    R0, C0 = R0.ravel(), C0.ravel()
    R1 = np.minimum(R0 + tile_rows, rows)          # exclusive ends
    C1 = np.minimum(C0 + tile_cols, cols)
    pts = [np.stack([R0, C0], axis=1), np.stack([R1 - 1, C1 - 1], axis=1)]
    for _ in range(max(0, per_tile - 2)):
        r = R0 + (rng.random(R0.size) * (R1 - R0)).astype(np.int64)
        c = C0 + (rng.random(C0.size) * (C1 - C0)).astype(np.int64)
        pts.append(np.stack([r, c], axis=1))
    return np.concatenate(pts, axis=0)


def output_points(layer_or_dims, Ho, Wo, tile_rows, tile_cols, per_tile, seed):
    """``stratified_points`` over the output seen as the No x (Ho*Wo*Nb) matrix the kernels tile,
    returned as (o, y, x, n) rows (int32) for the oracle's point-wise entry."""
    No, Nb = layer_or_dims
    rc = stratified_points(No, Ho * Wo * Nb, tile_rows, tile_cols, per_tile, seed)
    o, m = rc[:, 0], rc[:, 1]
    pix, n = m // Nb, m % Nb
    return np.stack([o, pix // Wo, pix % Wo, n], axis=1).astype(np.int32)
