"""Every attention kernel must fit its registers: a spill to scratch memory is the failure that the paper's
Section 7 describes for its 128x128 tile (register pressure serialising the second GEMM).  CPU only: compiles the
kernels for gfx950 and reads the compiler's resource report."""
import pytest

from paper_2312_11918_amd import build


@pytest.fixture(scope="module")
def kernels():
    return build.resource_usage()


def test_every_instantiation_is_reported(kernels):
    names = {k["name"] for k in kernels}
    # 2 element types x (3 head dimensions x 4 mask/partial-tile combinations of the 128-row shape
    #                    + 2 head dimensions x with and without the causal mask of the 256-row shape)
    assert len(names) == 2 * (3 * 4 + 2 * 2), sorted(names)


def test_no_kernel_uses_scratch_memory(kernels):
    bad = [(k["name"], k["scratch_bytes_per_lane"]) for k in kernels if k["scratch_bytes_per_lane"] != 0]
    assert not bad, f"kernels that spill to scratch: {bad}"


def test_register_and_lds_budgets_match_the_launch_shapes(kernels):
    for k in kernels:
        total = k["vgprs"] + k["agprs"]
        one_per_simd = "d=256" in k["name"]
        if one_per_simd:
            assert total <= 512, k
            assert k["lds_bytes_per_workgroup"] <= 160 * 1024, k
        else:
            # two wavefronts share a SIMD's 512 registers per lane
            assert total <= 256 and k["waves_per_simd"] >= 2, k
            per_cu = k["lds_bytes_per_workgroup"] * (2 if "4 wavefronts" in k["name"] else 1)
            assert per_cu <= 160 * 1024, k
