"""Writes tests/golden/variant_choice.txt: the tile variant and tail cut the library's heuristic picks
for a fixed set of layer shapes.  The file is a snapshot of the product's own choice -- not an
expected value of the convolution -- kept so that an edit to the cost model shows up as a diff of
named shapes (tests/test_api_host.py compares against it).  Run after a deliberate change:

    python tests/golden/write_variant_choice.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from paper_1501_06633_amd import binding as B          # noqa: E402
from paper_1501_06633_amd import workloads as W        # noqa: E402


def shapes():
    """name -> (Nb, Wi, Hi, Nc, No, Sk, stride, pad): the five benchmark layers, the paper's ten
    Table 1 shapes, the nine VGG-16 style shapes, and a 48-shape grid of 3x3 layers (minibatch
    16 ... 128, 7x7 ... 56x56 pixels, 96 ... 512 channels)."""
    out = {}
    for name, L in W.LAYERS.items():
        out[name] = (L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    for name, (L, _) in W.TABLE1.items():
        out[name] = (L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    for name, L in W.VGG16.items():
        out["vgg16." + name] = (L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    for nb in (16, 32, 64, 128):
        for hw in (7, 14, 28, 56):
            for nc, no in ((96, 256), (256, 384), (512, 512)):
                out[f"grid.nb{nb}.{hw}x{hw}.{nc}to{no}"] = (nb, hw, hw, nc, no, 3, 1, 1)
    return out


def line(name, dims):
    d = B.mdnn_describe_launch(*dims)
    return (f"{name} {' '.join(map(str, dims))} {d['variant']} tiles={d['tiles']} whole={d['whole']} "
            f"halved={d['halved']} thirded={d['thirded']} quartered={d['quartered']} eighthed={d['eighthed']} first={d['pieces_first']}")


def text():
    rows = ["# name Nb Wi Hi Nc No Sk stride pad -> variant and tail cut chosen by the library (a snapshot, see the script)"]
    rows += [line(n, d) for n, d in shapes().items()]
    return "\n".join(rows) + "\n"


if __name__ == "__main__":
    with open(os.path.join(HERE, "variant_choice.txt"), "w") as f:
        f.write(text())
    print(text())
