"""Build-time checks that need no GPU: the register guard of the build (every kernel without scratch memory,
spills or accumulation registers) and the public header as plain C99."""
import os
import subprocess

import pytest

from paper_2409_12210_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

REMARKS = """
route.hip:12:1: remark: Function Name: good_kernel [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     TotalSGPRs: 40 [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     VGPRs: 200 [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     AGPRs: 0 [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     Dynamic Stack: False [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     Occupancy [waves/SIMD]: 2 [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     SGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
route.hip:12:1: remark:     LDS Size [bytes/block]: 776 [-Rpass-analysis=kernel-resource-usage]
route.hip:90:1: remark: Function Name: spilling_kernel [-Rpass-analysis=kernel-resource-usage]
route.hip:90:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]
route.hip:90:1: remark:     AGPRs: 0 [-Rpass-analysis=kernel-resource-usage]
route.hip:90:1: remark:     ScratchSize [bytes/lane]: 300 [-Rpass-analysis=kernel-resource-usage]
route.hip:90:1: remark:     VGPRs Spill: 76 [-Rpass-analysis=kernel-resource-usage]
route.hip:99:1: remark: Function Name: agpr_kernel [-Rpass-analysis=kernel-resource-usage]
route.hip:99:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]
route.hip:99:1: remark:     AGPRs: 124 [-Rpass-analysis=kernel-resource-usage]
route.hip:99:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
route.hip:99:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
"""


def test_resource_guard_flags_scratch_spills_and_accumulation_registers():
    res = B.parse_resource_remarks(REMARKS)
    assert set(res) == {"good_kernel", "spilling_kernel", "agpr_kernel"}
    assert res["good_kernel"] == dict(sgprs=40, vgprs=200, agprs=0, scratch=0, occupancy=2, sgpr_spill=0,
                                      vgpr_spill=0, lds=776)
    bad = B.resource_violations(res)
    assert len(bad) == 2
    assert any("spilling_kernel" in b and "300" in b and "76" in b for b in bad)
    assert any("agpr_kernel" in b and "124" in b for b in bad)
    assert B.resource_violations({"good_kernel": res["good_kernel"]}) == []


def test_every_built_kernel_is_within_the_register_budget():
    if not os.path.exists(B.RESOURCES) or not os.path.exists(B.LIB):
        B.build(verbose=False)
    rows = [l.split() for l in open(B.RESOURCES) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 60                                   # every instantiation of every kernel is listed
    names = " ".join(r[0] for r in rows)
    for k in ("router_stream_kernel", "router_kernel", "router_token_kernel", "scatter_kernel", "combine_kernel",
              "bwd_gate_rows_kernel", "gg_bf16_kernel", "gg_bf16_skinny_kernel", "gg_f32_kernel", "plan_bwd_kernel",
              "route_scan_kernel"):
        assert k in names, k
    for name, vgprs, agprs, scratch, spill, occupancy, lds in rows:
        assert int(scratch) == 0 and int(spill) == 0 and int(agprs) == 0, name
        assert 0 < int(vgprs) <= 256 and int(lds) <= 160 * 1024, name


def test_public_header_is_plain_c99(tmp_path):
    src = tmp_path / "use_header.c"
    src.write_text('#include "modse.h"\n'
                   "int main(void) {\n"
                   "  modse_desc d; modse_routing r; modse_gate_ext g; size_t n = 0;\n"
                   "  (void)r; (void)g; d.d_ff = 0;\n"
                   "  return (int)modse_workspace_size(&d, 0, MODSE_WS_FWD, &n) + MODSE_N_STAGES\n"
                   "         + (int)MODSE_ROUTE_STATIC_SCRATCH_BYTES * 0;\n"
                   "}\n")
    obj = tmp_path / "use_header.o"
    r = subprocess.run(["gcc", "-std=c99", "-pedantic-errors", "-Wall", "-Wextra", "-Werror", "-I",
                        os.path.join(ROOT, "include"), "-c", str(src), "-o", str(obj)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
