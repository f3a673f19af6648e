"""Static checks on the gfx950 code hipcc generates from our own kernel source
(compiled to assembly here, no GPU needed): the contraction really runs on the
FP32 matrix cores -- a tolerance alone cannot tell a reduced-precision matrix
format from fp32 at K ~ 2300 -- operands really go global -> LDS directly,
nothing spills, and none of the instruction forms this project must avoid
(packed-FP32 VALU ops, scalar-cache writes) appears.
"""
import os
import re

import pytest

from paper_1501_06633_amd import build, lds_hazard_check

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def unit_asm(source):
    """gfx950 assembly of one translation unit, as the library build left it (built now if stale)."""
    path = build.device_asm_path(source)
    if build.stale() or not os.path.exists(path):
        build.build_lib(force=True)
    return open(path).read()


@pytest.fixture(scope="module")
def asm():
    """All translation units that instantiate the convolution kernel."""
    units = [s for s in build.KERNEL_SOURCES if "conv_variants_" in s]
    assert len(units) >= 7
    return "\n".join(unit_asm(s) for s in units)


@pytest.fixture(scope="module")
def asm_filter_grad():
    return unit_asm([f for f in build.KERNEL_SOURCES if f.endswith("bprop_filter.hip")][0])


def mnemonics(text):
    ops = set()
    for line in text.splitlines():
        line = line.split(";")[0].strip()
        if not line or line.startswith(".") or line.endswith(":"):
            continue
        ops.add(line.split()[0])
    return ops


def test_contraction_is_fp32_mfma_only(asm):
    ops = mnemonics(asm)
    mfma = {o for o in ops if o.startswith(("v_mfma", "v_smfmac"))}
    # no bf16 / f16 / xf32 / i8 / f8 / sparse forms: the two FP32 shapes only
    assert mfma == {"v_mfma_f32_32x32x2_f32", "v_mfma_f32_16x16x4_f32"}, mfma
    assert asm.count("v_mfma_f32_32x32x2_f32") > 1000    # every variant carries the unrolled loop
    assert asm.count("v_mfma_f32_16x16x4_f32") > 100     # the 48-row tiles


def test_operands_go_global_to_lds_directly(asm):
    assert re.search(r"buffer_load_dwordx4 .* lds", asm)
    assert re.search(r"buffer_load_dword .* lds", asm)   # the scalar-copy variant
    assert "ds_read_b128" in asm or "ds_read_b64" in asm


def test_no_forbidden_instruction_forms(asm):
    ops = mnemonics(asm)
    assert not {o for o in ops if o.startswith(("v_pk_add_f32", "v_pk_mul_f32", "v_pk_fma_f32"))}
    assert not {o for o in ops if o.startswith(("s_store", "s_buffer_store", "s_atomic", "s_buffer_atomic",
                                                "s_dcache_wb", "s_dcache_inv", "s_scratch_store"))}


def test_no_spills_and_register_budget(asm):
    spills = [int(x) for x in re.findall(r"\.vgpr_spill_count:\s+(\d+)", asm)]
    sspills = [int(x) for x in re.findall(r"\.sgpr_spill_count:\s+(\d+)", asm)]
    scratch = [int(x) for x in re.findall(r"\.private_segment_fixed_size:\s+(\d+)", asm)]
    assert spills and not any(spills) and not any(scratch)          # nothing ever goes to scratch memory
    names = re.findall(r"\.name:\s+(\S+)", asm)
    # Scalar registers parked in vector-register lanes: tolerated in the 4-byte-copy kernels
    # (template argument VW = 1, 14 or 41), which carry ten to sixteen copies per thread and slab,
    # each with an LDS address of its own in a scalar register; elsewhere only a
    # few, and only outside every loop (the kernels that carry all piece bodies park a value or two
    # across a whole tile).
    parked = {k: v for k, v in zip(names, sspills) if v and not re.search(r"Li(1|14|41)ELi2ELi32EEE", k)}
    assert all(v <= 4 for v in parked.values()), parked
    for name in parked:
        body = asm[asm.index(name + ":"):asm.index(".size\t" + name)].splitlines()
        label_at = {m.group(1): i for i, l in enumerate(body) if (m := re.match(r"(\.LBB[0-9_]+):", l))}
        loops = [(label_at[m.group(1)], i) for i, l in enumerate(body)
                 if (m := re.search(r"s_c?branch\w*\s+(\.LBB[0-9_]+)", l)) and label_at.get(m.group(1), i) < i]
        for i, l in enumerate(body):
            if "v_writelane" in l or "v_readlane" in l:
                assert not any(a <= i <= b for a, b in loops), (name, l)
    vgprs = dict(zip(names, map(int, re.findall(r"\.vgpr_count:\s+(\d+)", asm))))
    # the 128x128 kernels must leave room for three waves per SIMD (512 / 3 = 170 registers)
    main = [v for k, v in vgprs.items() if "Li2ELi2ELi2ELi2E" in k]
    assert main and max(main) <= 168, vgprs


def test_filter_gradient_kernels(asm_filter_grad):
    """The same static checks on the filter-gradient kernels."""
    text = asm_filter_grad
    ops = mnemonics(text)
    assert {o for o in ops if o.startswith(("v_mfma", "v_smfmac"))} == {"v_mfma_f32_32x32x2_f32"}
    assert re.search(r"buffer_load_dwordx4 .* lds", text) and re.search(r"buffer_load_dword .* lds", text)
    assert "ds_read_b128" in text
    assert not {o for o in ops if o.startswith(("v_pk_add_f32", "v_pk_mul_f32", "v_pk_fma_f32"))}
    assert not {o for o in ops if o.startswith(("s_store", "s_buffer_store", "s_atomic", "s_buffer_atomic",
                                                "s_dcache_wb", "s_dcache_inv", "s_scratch_store"))}
    assert not any(int(x) for x in re.findall(r"\.vgpr_spill_count:\s+(\d+)", text))
    assert not any(int(x) for x in re.findall(r"\.private_segment_fixed_size:\s+(\d+)", text))
    vgprs = dict(zip(re.findall(r"\.name:\s+(\S+)", text), map(int, re.findall(r"\.vgpr_count:\s+(\d+)", text))))
    # three workgroups per compute unit are planned for: the 16-byte-copy kernels must fit 512 / 3 registers
    vec = [v for k, v in vgprs.items() if "conv_bprop_filter_kernelILi4E" in k]
    assert len(vec) == 8 and max(vec) <= 168, vgprs


def test_no_register_is_touched_while_an_lds_read_into_it_is_in_flight(asm, asm_filter_grad):
    """The hand-counted LDS waits hold on every path of every kernel (see lds_hazard_check)."""
    n, bad = lds_hazard_check.check(asm)
    assert n >= 13 and not bad, bad[:5]
    n, bad = lds_hazard_check.check(asm_filter_grad)
    assert n >= 12 and not bad, bad[:5]


_GOOD = """
k:
\tds_read_b32 v1, v9
\tds_read_b32 v2, v9 offset:4
\ts_waitcnt lgkmcnt(1)
\tv_add_f32 v3, v1, v1
\ts_cbranch_scc1 .LBB0_2
\tds_read_b32 v1, v9 offset:8
.LBB0_2:
\ts_waitcnt lgkmcnt(0)
\tv_add_f32 v3, v2, v1
\ts_endpgm
"""


def test_the_checker_itself():
    n, bad = lds_hazard_check.check(_GOOD)
    assert n == 1 and not bad
    # a copy before the wait that makes the value valid
    n, bad = lds_hazard_check.check(_GOOD.replace("\ts_waitcnt lgkmcnt(1)\n", "\tv_mov_b32 v4, v1\n\ts_waitcnt lgkmcnt(1)\n"))
    assert bad and bad[0][3] == [1]
    # waiting for too few: the second read is still in flight when v2 is used
    n, bad = lds_hazard_check.check(_GOOD.replace("lgkmcnt(0)", "lgkmcnt(1)"))
    assert any(2 in b[3] for b in bad)
    # only one path is wrong: the read issued on the fall-through path is not waited for
    n, bad = lds_hazard_check.check(_GOOD.replace(".LBB0_2:\n\ts_waitcnt lgkmcnt(0)", ".LBB0_2:\n\ts_waitcnt lgkmcnt(1)\n\tv_mov_b32 v5, v2"))
    assert bad and all(b[3] == [1] or b[3] == [2] for b in bad)
    # reusing the destination register for something else while the read is in flight
    n, bad = lds_hazard_check.check(_GOOD.replace("\ts_waitcnt lgkmcnt(1)\n", "\tv_mov_b32 v2, 0\n\ts_waitcnt lgkmcnt(1)\n"))
    assert bad and bad[0][3] == [2]
