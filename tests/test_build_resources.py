"""Host-side guard on what the compiler made of the hot kernels: the register-resident kernels
must not spill (a spill inside their passes costs more than any tuning gains: every reload waits on
the same counter as the row loads), and no kernel may ask for more LDS than a CU has.  Reads the
table that the in-tree build writes from the compiler's resource-usage remarks."""
import os

import pytest

from paper_2402_14160_amd import build

LDS_PER_CU = 160 * 1024


@pytest.fixture(scope="module")
def resources():
    if not os.path.exists(build.RESOURCES):
        build.build()
    return build.kernel_resources()


def _kernels(table, fragment):
    found = {k: v for k, v in table.items() if fragment in k}
    assert found, fragment
    return found


def test_every_kernel_fits_the_cu(resources):
    assert len(resources) >= 30
    for name, use in resources.items():
        assert use["LDS Size"] <= LDS_PER_CU, name
        assert use["VGPRs"] <= 256, name
        assert use["Occupancy"] >= 1, name


@pytest.mark.parametrize("fragment", [
    "tree_attn_bf16_w32_kernel", "tree_attn_bf16_kernel", "tree_attn_f32_kernel", "tree_attn_merge_kernel",
    "lse_kernel",
    "rrs_group_kernelILi512ELi16ELi0E",    # both rows in registers, next rows staged
    "rrs_group_kernelILi256ELi8ELi0E",
    "rrs_group_kernelILi512ELi0ELi0E",     # streaming variant
    "rrs_path_kernelILi512ELi16ELi0E", "rrs_path_kernelILi256ELi8ELi0E",
    "rrs_final_kernel", "sbs_select_kernel", "filter_kv",
])
def test_resident_kernels_do_not_spill(resources, fragment):
    for name, use in _kernels(resources, fragment).items():
        assert use["ScratchSize"] == 0, (name, use)


@pytest.mark.parametrize("fragment,limit", [
    ("rrs_group_kernelILi512ELi25ELi18E", 96),   # 50k vocabularies: 7 draft chunks + the target row in registers
    ("rrs_path_kernelILi512ELi25ELi18E", 96),
    ("gumbel_topk_kernel", 64),                  # held to 64 / 128 registers for two workgroups per CU
    ("prob_filter_kernel", 128),
])
def test_known_spills_stay_small(resources, fragment, limit):
    """Bytes of scratch per lane of the kernels that are known to spill a little outside their
    inner passes: a bound, so that a change that makes them spill in earnest is seen."""
    for name, use in _kernels(resources, fragment).items():
        assert use["ScratchSize"] <= limit, (name, use)
