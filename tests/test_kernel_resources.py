"""What the compiler reports for the gfx950 kernels (no GPU needed: hipcc cross-compiles): none of them uses scratch
memory - so no launch makes the runtime allocate a scratch buffer, which the entry point that allocates nothing relies
on - every kernel fits the register file without spills, and the attention kernel's LDS fits a CU."""
import pytest

from paper_2602_14516_amd import build


@pytest.fixture(scope="module")
def resources():
    return build.kernel_resources()


def test_no_kernel_uses_scratch_memory_or_spills_vector_registers(resources):
    assert len(resources) >= 10, sorted(resources)
    for name, r in resources.items():
        assert r["ScratchSize [bytes/lane]"] == 0, (name, r)
        assert r["VGPRs Spill"] == 0, (name, r)
        assert r["VGPRs"] + r["AGPRs"] <= 256, (name, r)


def test_attention_kernels_keep_two_waves_per_simd_and_fit_the_lds(resources):
    attn = {n: r for n, r in resources.items() if "attn_kernel" in n}
    assert len(attn) == 4, sorted(attn)                       # d = 64 / 128 x bf16 / 8-bit cache
    for name, r in attn.items():
        assert r["Occupancy [waves/SIMD]"] >= 2, (name, r)    # 8 waves of one workgroup on 4 SIMDs
        assert r["LDS Size [bytes/block]"] <= 160 * 1024, (name, r)
