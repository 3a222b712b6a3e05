"""Registers, scratch and LDS of the built kernels, as the compiler reported them at build time
(paper_2401_04658_amd/_build/kernel_resources.json, written by build.py from -Rpass-analysis=kernel-resource-usage).

The block kernels keep a d x d fp32 state in registers and sit at the register limit of their occupancy.  A change
anywhere in such a kernel can tip the allocator into spilling inside the block loop; a spilled value is reloaded
through the vector memory counter, behind the tile loads in flight, and the kernel loses a third of its speed without
failing any parity test.  These checks catch that at build time, on the CPU."""
import json
import os
import re

import pytest

from paper_2401_04658_amd import build

LDS_PER_CU = 160 * 1024


@pytest.fixture(scope="module")
def resources():
    if not os.path.exists(build.RESOURCES):
        build.build()
    with open(build.RESOURCES) as f:
        return json.load(f)


def family(name):
    m = re.search(r"\d+([a-z0-9_]+?_kernel|mfma_peak_kernel)", name)
    return m.group(1) if m else name


def test_every_kernel_is_reported(resources):
    fams = {family(k) for k in resources}
    for f in ("scan_bf16_half_kernel", "scan_wide_kernel", "chunk_state_bf16_kernel", "scan_bf16_kernel", "scan_f32_kernel",
              "decode_kernel", "tail_bf16_kernel", "left_product_bf16_kernel", "norm_rows_kernel", "state_scan_kernel",
              "recur_kernel", "varlen_map_kernel"):
        assert f in fams, f
    for k, v in resources.items():
        for key in ("VGPRs", "ScratchSize", "Occupancy", "LDS"):
            assert isinstance(v.get(key), int), (k, key)


def test_no_kernel_has_a_dynamic_stack_or_more_lds_than_a_compute_unit(resources):
    for k, v in resources.items():
        assert v["Dynamic_Stack"] == "False", k
        assert v["LDS"] <= LDS_PER_CU, (k, v["LDS"])
        assert v["SGPRs_Spill"] == 0, k


# bytes of scratch per lane: a handful of loop-invariant values that the allocator parks outside the block loop (read
# back in the rare ragged-block path or after the loop) is what the kernels have today; a spill inside the loop shows
# up as hundreds of bytes
SCRATCH_LIMIT = {
    "scan_bf16_half_kernel": 32, "scan_wide_kernel": 32, "chunk_state_bf16_kernel": 0, "scan_bf16_kernel": 0,
    "scan_f32_kernel": 0, "decode_kernel": 0, "tail_bf16_kernel": 0, "left_product_bf16_kernel": 0,
    "norm_rows_kernel": 0,
}


def test_the_block_kernels_do_not_spill_in_their_loops(resources):
    seen = set()
    for k, v in resources.items():
        f = family(k)
        if f in SCRATCH_LIMIT:
            seen.add(f)
            assert v["ScratchSize"] <= SCRATCH_LIMIT[f], (k, v["ScratchSize"], v["VGPRs"])
    assert seen == set(SCRATCH_LIMIT)


def test_occupancy_the_kernels_are_designed_for(resources):
    """Two waves per SIMD for every MFMA scan kernel that carries a state slice (their LDS reads and conversions are
    covered by the other wave); three for the head_dim 96 kernel outside its twin form; the streaming kernels more."""
    for k, v in resources.items():
        f = family(k)
        if f in ("scan_bf16_half_kernel", "scan_wide_kernel", "chunk_state_bf16_kernel", "tail_bf16_kernel"):
            assert v["Occupancy"] >= 2, (k, v["Occupancy"])
        if f == "scan_wide_kernel" and "Li96E" in k and not k.split("Li96E")[1].startswith("Lb1ELb0ELb0ELb1E"):
            assert v["Occupancy"] >= 3, (k, v["Occupancy"])
        if f in ("decode_kernel", "norm_rows_kernel"):
            assert v["Occupancy"] >= 4, (k, v["Occupancy"])
