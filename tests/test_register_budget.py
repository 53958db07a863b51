"""The scoring kernel's design rests on a whole column living in registers with 16 waves
per compute unit: at most 128 vector registers per lane and nothing spilled.  The
compiler's own resource report (-Rpass-analysis=kernel-resource-usage, written beside the
objects by the build) is parsed here; no GPU is needed."""
import os

import pytest

from paper_2605_17879_amd import build as hip_build

SOURCES = ("score.hip", "score_z.hip")


def _report(src):
    path = hip_build.resource_file(src)
    source = os.path.join(hip_build.CSRC, "score.hip")
    if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(source):
        hip_build.build()                       # (the build writes the reports)
    with open(path) as f:
        return hip_build.parse_resources(f.read())


@pytest.mark.parametrize("src", SOURCES)
def test_every_scoring_instantiation_is_within_the_register_budget(src):
    res = _report(src)
    tilings = {k: hip_build.tiling_of(k) for k in res if hip_build.tiling_of(k)}
    want_z = 1 if src == "score_z.hip" else 0
    # six tilings of whole batches (exact fit and ragged) and those of the per-column route
    batch = {(64, 1, 10), (64, 4, 10), (256, 4, 11), (256, 16, 11), (512, 16, 12), (1024, 16, 12)}
    column = {(64, 1, 10), (64, 4, 10), (256, 4, 11), (1024, 4, 12), (1024, 8, 12), (1024, 16, 12)}
    seen_batch = {t[:3] for t in tilings.values() if t[4] == 0 and t[5] == want_z}
    seen_column = {t[:3] for t in tilings.values() if t[4] == 1 and t[5] == want_z}
    assert seen_batch == batch and seen_column == column, (seen_batch, seen_column)
    assert hip_build.check_register_budget(res) == []
    for name, t in tilings.items():
        r = res[name]
        assert r["VGPRs"] + r["AGPRs"] <= hip_build.VGPR_BUDGET, name
        assert r["Occupancy [waves/SIMD]"] >= 4, name
        assert r["LDS Size [bytes/block]"] == 0, name          # all of its LDS is dynamic (sized by the launcher)
        if t[3] and t[0] >= 256 and not t[4]:                  # exact-fit batch tilings: nothing in scratch memory
            assert r["VGPRs Spill"] == 0 and r["ScratchSize [bytes/lane]"] == 0, (name, r)


def test_the_parser_reads_the_compiler_remarks():
    text = """x.hip:1:1: remark: Function Name: _ZN1_12score_kernelILi1024ELi16ELi12ELb1ELb0ELb0EEEv13gd_score_args [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     VGPRs: 129 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     AGPRs: 0 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     ScratchSize [bytes/lane]: 16 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     Dynamic Stack: False [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     Occupancy [waves/SIMD]: 3 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     VGPRs Spill: 4 [-Rpass-analysis=kernel-resource-usage]
"""
    res = hip_build.parse_resources(text)
    (name, r), = res.items()
    assert hip_build.tiling_of(name) == (1024, 16, 12, 1, 0, 0)
    assert r == {"VGPRs": 129, "AGPRs": 0, "ScratchSize [bytes/lane]": 16, "Dynamic Stack": False,
                 "Occupancy [waves/SIMD]": 3, "VGPRs Spill": 4}
    bad = hip_build.check_register_budget(res)
    assert len(bad) == 3, bad
