"""What the compiler says about the kernels of the last build (hipcc's kernel-resource-usage
remarks, kept by the build beside the objects): no attention kernel touches scratch memory, and
the selection kernels that are planned for several workgroups per compute unit fit their
register budget. Host-only: reads a text file the build wrote."""
import os
import subprocess

import pytest

from paper_2605_15508_amd import build


@pytest.fixture(scope="module")
def resources():
    if not os.path.exists(build.RESOURCES) or build.needs_build():
        build.build(force=True)
    return build.kernel_resources()


def demangle(sym):
    try:
        return subprocess.run(["c++filt", sym], capture_output=True, text=True, check=True).stdout.strip()
    except (OSError, subprocess.CalledProcessError):
        return sym


def test_every_attention_kernel_runs_without_scratch(resources):
    attn = {k: v for k, v in resources.items() if "attn_split_kernel" in k or "attn_combine_kernel" in k
            or "attn_probsum_kernel" in k}
    assert len(attn) >= 20                      # the instantiated variants are all there
    bad = {demangle(k): v["ScratchSize"] for k, v in attn.items() if v["ScratchSize"] != 0}
    assert not bad, bad


def test_the_logits_dump_at_head_size_128_has_no_four_tile_form(resources):
    # planned with two query tiles at most: its four-tile form would spill about a hundred registers
    assert not [k for k in resources if "attn_split_kernelILi128ELi4ELb0ELb1E" in k]


def test_selection_kernels_fit_the_occupancy_they_are_planned_for(resources):
    for k, v in resources.items():
        if "select_rowpass_kernelILi256" in k:
            assert v["VGPRs"] <= 96 and v["ScratchSize"] == 0, demangle(k)        # five workgroups per CU or more
        if "select_write_kernel" in k:
            assert v["VGPRs"] <= 128 and v["ScratchSize"] == 0, demangle(k)       # four workgroups per CU
