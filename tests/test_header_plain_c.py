"""The boundary is a C ABI: include/mdnn.h must compile as plain C99, and a C
program linked against libmdnn.so must be able to call the host-only entry
points (no GPU is touched: only argument checks and the pure host functions)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include <stdio.h>
#include <string.h>
#include "mdnn.h"

int main(void)
{
    int Wo = 0, Ho = 0;
    size_t bytes = 0;
    char text[512];
    if (mdnn_out_dims(227, 227, 11, 4, 0, &Wo, &Ho) != MDNN_OK || Wo != 55 || Ho != 55) return 1;
    /* Section 2: 2 Nb Wo Ho (Nc Sk^2 + 1) No */
    if (mdnn_conv_flops(128, 55, 55, 3, 96, 11) != 2ull * 128 * 55 * 55 * (3 * 121 + 1) * 96) return 2;
    if (mdnn_conv_fprop(NULL, NULL, NULL, 8, 8, 8, 2, 4, 3, 1, 1, 1.0f, NULL) != MDNN_ENULL) return 3;
    if (mdnn_sgemm_tn(NULL, NULL, NULL, 8, 8, 8, 1.0f, NULL) != MDNN_ENULL) return 4;
    if (mdnn_conv_bprop_data_workspace(8, 8, 8, 2, 4, 3, 1, 1, &bytes) != MDNN_OK || bytes == 0) return 5;
    if (mdnn_conv_bprop_filter_workspace(8, 8, 8, 2, 4, 3, 1, 1, &bytes) != MDNN_OK || bytes == 0) return 6;
    if (mdnn_describe_launch(64, 56, 56, 256, 256, 3, 1, 1, NULL, text, sizeof text) != MDNN_OK) return 7;
    if (!strstr(text, "variant=") || mdnn_variant_count() < 3 || !mdnn_variant_name(0)) return 8;
    if (!mdnn_status_string(MDNN_ETOOBIG)[0]) return 9;
    puts(text);
    return 0;
}
"""


def test_header_compiles_as_c99_and_links(tmp_path):
    from paper_1501_06633_amd import binding as B
    lib = B.library_path() if hasattr(B, "library_path") else os.path.join(ROOT, "paper_1501_06633_amd", "libmdnn.so")
    if not os.path.exists(lib):
        pytest.skip("libmdnn.so not built")
    src = tmp_path / "use_mdnn.c"
    exe = tmp_path / "use_mdnn"
    src.write_text(PROGRAM)
    libdir = os.path.dirname(lib)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           "-o", str(exe), str(src), "-L", libdir, "-lmdnn", f"-Wl,-rpath,{libdir}"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    run = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=60)
    assert run.returncode == 0, f"exit {run.returncode}: {run.stdout}"
    assert "variant=o128m128k8" in run.stdout
