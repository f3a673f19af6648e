"""The host side of the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer.

Every translation unit of the library is compiled for the host only (no device code: nothing is
launched here) with the sanitizers on, linked with a C++ driver, and the driver walks the planning
arithmetic -- 64-bit size checks, division magic numbers, the tile-variant cost model, the tail
cuts, both workspace plans -- over benchmark shapes, a grid of sizes, every variant with every
pinned cut, and extreme arguments (INT_MAX, 1, sizes that overflow 32 bits), and every argument
error path of every entry point.  Any out-of-bounds access, signed overflow, bad shift or invalid
conversion in that arithmetic stops the driver."""
import os
import re
import subprocess
import textwrap

from paper_1501_06633_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = textwrap.dedent(r"""
    #include <climits>
    #include <cstdio>
    #include <cstdint>
    #include <cstring>
    #include "mdnn.h"
    static long calls = 0, ok = 0;
    static void plan_all(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int s, int p) {
        char text[512];
        int Wo = 0, Ho = 0;
        size_t bytes = 0;
        calls++;
        if (mdnn_out_dims(Wi, Hi, Sk, s, p, &Wo, &Ho) == MDNN_OK) (void)mdnn_conv_flops(Nb, Wo, Ho, Nc, No, Sk);
        (void)mdnn_choose_variant(Nb, Wi, Hi, Nc, No, Sk, s, p);
        if (mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, s, p, nullptr, text, sizeof text) == MDNN_OK) ok++;
        const char cuts[] = "whtqemnpHTQE";
        for (int v = 0; v < mdnn_variant_count(); ++v) {
            char name[48];
            (void)mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, s, p, mdnn_variant_name(v), text, sizeof text);
            for (const char* c = cuts; *c; ++c) {
                std::snprintf(name, sizeof name, "%s:%c", mdnn_variant_name(v), *c);
                (void)mdnn_describe_launch(Nb, Wi, Hi, Nc, No, Sk, s, p, name, text, 40);   // short buffer too
            }
        }
        (void)mdnn_conv_bprop_data_workspace(Nb, Wi, Hi, Nc, No, Sk, s, p, &bytes);
        (void)mdnn_conv_bprop_filter_workspace(Nb, Wi, Hi, Nc, No, Sk, s, p, &bytes);
        // calls that fail validation before anything could be launched: misaligned pointers
        float* bad = reinterpret_cast<float*>(uintptr_t(0x10004));
        float* good = reinterpret_cast<float*>(uintptr_t(0x10000));
        (void)mdnn_conv_fprop(bad, good, good, Nb, Wi, Hi, Nc, No, Sk, s, p, 1.0f, nullptr);
        (void)mdnn_conv_bprop_data(good, good, bad, good, SIZE_MAX, Nb, Wi, Hi, Nc, No, Sk, s, p, 1.0f, nullptr);
        (void)mdnn_conv_bprop_data_static(good, bad, good, Nb, Wi, Hi, Nc, No, Sk, s, p, 1.0f, nullptr);
        (void)mdnn_conv_bprop_filter(good, good, good, bad, SIZE_MAX, Nb, Wi, Hi, Nc, No, Sk, s, p, 1.0f, nullptr);
    }
    int main() {
        // benchmark layers, the paper's Table 1, VGG-16 style shapes
        const int named[][8] = {
            {8, 32, 32, 16, 32, 3, 1, 1}, {128, 227, 227, 3, 96, 11, 4, 0}, {128, 27, 27, 96, 256, 5, 1, 2},
            {128, 13, 13, 256, 384, 3, 1, 1}, {64, 56, 56, 256, 256, 3, 1, 1}, {128, 224, 224, 3, 64, 11, 4, 2},
            {128, 13, 13, 384, 256, 3, 1, 1}, {128, 231, 231, 3, 96, 11, 4, 0}, {128, 24, 24, 96, 256, 5, 1, 0},
            {128, 12, 12, 1024, 1024, 3, 1, 1}, {64, 224, 224, 3, 64, 3, 1, 1}, {64, 14, 14, 512, 512, 3, 1, 1},
            {50, 56, 56, 256, 256, 3, 1, 1}, {64, 56, 56, 256, 250, 3, 1, 1}, {7, 10, 11, 3, 37, 3, 2, 1}};
        for (const auto& d : named) plan_all(d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7]);
        // a grid: minibatch x image x channels, and tile counts through every tail regime
        const int nbs[] = {1, 4, 16, 128}, hws[] = {1, 7, 28, 112}, chans[] = {1, 3, 96, 513};
        for (int nb : nbs) for (int hw : hws) for (int nc : chans) for (int no : chans)
            for (int sk = 1; sk <= 5; sk += 2) for (int s = 1; s <= 4; s += 3)
                plan_all(nb, hw, hw + 1, nc, no, sk, s, sk / 2);
        for (int r = 0; r < 256; r += 5) plan_all(128, 3, 2 + 256 + r, 4, 128, 3, 1, 0);
        // extremes: every combination must be rejected or planned without undefined behaviour
        const int ext[] = {INT_MIN, -1, 0, 1, 2, 3, 65535, 65536, 1 << 20, 1 << 26, 1 << 30, INT_MAX};
        for (int a : ext) for (int b : ext) {
            plan_all(a, b, b, 1, 1, 1, 1, 0);
            plan_all(1, a, b, 1, 1, 1, 1, 0);
            plan_all(1, 4, 4, a, b, 1, 1, 0);
            plan_all(2, 8, 8, 2, 2, a, b, 0);
            plan_all(2, 8, 8, 2, 2, 3, a, b);
            plan_all(4, a, 3, 2, b, 3, 1, 1);
        }
        // plain matrix product and probe argument checks
        float* good = reinterpret_cast<float*>(uintptr_t(0x10000));
        for (int a : ext) for (int b : ext) (void)mdnn_sgemm_tn(good, good, reinterpret_cast<float*>(uintptr_t(0x10004)), a, b, 8, 1.0f, nullptr);
        uint64_t fl = 0;
        for (int a : ext) (void)mdnn_mfma_peak_probe(nullptr, a, a, a, &fl, nullptr);
        for (int st = -2; st < 9; ++st) if (!mdnn_status_string((mdnn_status)st)) return 3;
        (void)mdnn_variant_name(-1); (void)mdnn_variant_name(INT_MAX);
        std::printf("sanitized api calls=%ld planned=%ld\n", calls, ok);
        return (ok > 500) ? 0 : 2;
    }
""")


def test_host_api_clean_under_asan_ubsan(tmp_path):
    hipcc = build.hipcc()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    common = [hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17", *san,
              "-I", os.path.join(ROOT, "include"), "-I", build.CSRC, "-Wno-unused-command-line-argument"]
    drv = tmp_path / "driver.cpp"
    drv.write_text(DRIVER)
    objs = []
    for src in build.SOURCES + [str(drv)]:
        obj = tmp_path / (os.path.splitext(os.path.basename(src))[0] + ".o")
        res = subprocess.run([*common, "-c", "-o", str(obj), src], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout[-3000:]
        objs.append(str(obj))
    # A host-only object still refers to the device code of its unit by name; there is none here
    # (nothing is launched), so give the linker an empty stand-in for each.
    undefined = subprocess.run(["nm", "-u", *objs], stdout=subprocess.PIPE, text=True, check=True).stdout
    names = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", undefined)))
    stand_in = tmp_path / "no_device_code.c"
    stand_in.write_text("".join(f"const char {n}[8] = {{0}};\n" for n in names))
    exe = tmp_path / "driver"
    res = subprocess.run([hipcc, "--cuda-host-only", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                          "-Wno-unused-command-line-argument", "-Wno-option-ignored", "-o", str(exe), *objs,
                          "-x", "c", str(stand_in)],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "sanitized api calls=" in res.stdout and "runtime error" not in res.stdout
