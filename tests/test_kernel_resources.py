"""What the compiler made of the GEMM kernel: all 256 accumulator registers of a wavefront in the AGPR half of
its register file, one wavefront per SIMD, and nothing spilled to scratch memory in any instantiation (a spill
inside the K loop costs far more than the few registers it saves; outside it, it still means the loop's
register budget was exceeded somewhere).  Compiles the device code; no GPU needed."""
import pytest

from paper_2402_14800_amd import build


@pytest.fixture(scope="module")
def gemm_usage():
    return build.kernel_resource_usage("gemm_bf16_packed.hip")


def test_packed_gemm_instantiations_do_not_spill(gemm_usage):
    gemms = {n: u for n, u in gemm_usage.items() if "gemm_packed_kernel" in n}
    assert len(gemms) >= 5                       # dense store / SwiGLU, grouped store / SwiGLU / row-scaled fp32
    for name, u in gemms.items():
        assert u["ScratchSize"] == 0, (name, u)
        assert u["VGPRs Spill"] == 0 and u["SGPRs Spill"] == 0, (name, u)
        assert u["AGPRs"] == 256 and u["VGPRs"] <= 256, (name, u)
        assert u["Occupancy"] == 1, (name, u)


def test_pack_kernel_is_light(gemm_usage):
    pack = [u for n, u in gemm_usage.items() if "pack_kernel" in n]
    assert pack and all(u["ScratchSize"] == 0 for u in pack)


def test_table_scorer_keeps_three_wavefronts_per_simd_without_spilling():
    """The look-up scorer is planned as one resident round of workgroups, three per CU: every instantiation has to
    fit three wavefronts per SIMD with its per-subset look-up addresses in registers, not in scratch memory."""
    usage = build.kernel_resource_usage("enumerate.hip")
    luts = {n: u for n, u in usage.items() if "score_lut_kernel" in n}
    assert len(luts) >= 7
    for name, u in luts.items():
        assert u["ScratchSize"] == 0 and u["VGPRs Spill"] == 0, (name, u)
        assert u["Occupancy"] >= 3, (name, u)
