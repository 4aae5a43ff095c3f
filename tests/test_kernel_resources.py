"""The hot kernels must not use scratch memory: a register spill inside a GEMM or attention kernel costs far more than
its instruction count suggests (every reload waits for all outstanding memory operations), and nothing else in the
test suite would notice one.  Reads the per-kernel resource reports that the build keeps beside the object files
(hipcc -Rpass-analysis=kernel-resource-usage); no GPU needed."""
import json
import os

import pytest

from paper_2602_07306_amd import build as B

# kernel name fragment -> sources that instantiate it
HOT = {
    "gemm_mfma_kernel": ["kernels_gemm_mfma_store.hip", "kernels_gemm_mfma_residual.hip", "kernels_gemm_mfma_swiglu.hip",
                         "kernels_gemm_mfma_qkv_a.hip", "kernels_gemm_mfma_qkv_b.hip", "kernels_gemm_mfma_qkv_c.hip",
                         "kernels_gemm_mfma_qkv_d.hip"],
    "gemm_dl_kernel": ["kernels_gemm_mfma_store.hip", "kernels_gemm_mfma_residual.hip", "kernels_gemm_mfma_swiglu.hip",
                       "kernels_gemm_mfma_qkv_a.hip"],
    "gemm_skinny_kernel": ["kernels_gemm_skinny.hip"],
    "gemm_gemv_kernel": ["kernels_gemm_skinny.hip"],
    "attn_prefill_lds_kernel": ["kernels_attn_prefill_mfma.hip"],
    "attn_decode": ["kernels_attn_decode.hip"],
}


def load(src):
    path = B.resources_path(src)
    if not os.path.exists(path):
        pytest.skip("%s is missing: run `python -m paper_2602_07306_amd.build`" % path)
    return json.load(open(path))


@pytest.mark.parametrize("fragment", sorted(HOT))
def test_hot_kernels_use_no_scratch_memory(fragment):
    seen = 0
    for src in HOT[fragment]:
        for name, res in load(src).items():
            if fragment not in name:
                continue
            seen += 1
            assert res["ScratchSize"] == 0 and res["VGPRs Spill"] == 0, (src, name, res)
    assert seen > 0, "no kernel named *%s* in %s" % (fragment, HOT[fragment])


def test_the_big_gemm_tile_keeps_its_accumulators_in_accumulation_registers():
    """256 x 256 tile, four wavefronts: 256 accumulators per lane, which only fit beside the staging registers when
    they live in AGPRs."""
    res = load("kernels_gemm_mfma_swiglu.hip")
    big = [r for n, r in res.items() if "gemm_mfma_kernelILi256ELi256ELi2ELi2ELi64" in n]
    assert big and all(r["AGPRs"] == 256 for r in big), big
