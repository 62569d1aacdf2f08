"""GPU parity of every selectable GEMM kernel variant (lora_set_tuning) against the CPU oracle: the
automatic choice reaches only some of them at a given shape, the others stay reachable for tuning and must
compute the same result.  Small workloads with a ragged last tile, packed and single calls."""
import pytest

from gpu_util import run_and_check
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl

pytestmark = pytest.mark.gpu

FUSED_VARIANTS = sorted(B.FUSED_VARIANTS.values())
SPLIT_VARIANTS = sorted(B.SPLIT_VARIANTS.values())

@pytest.mark.parametrize("variant", FUSED_VARIANTS)
def test_fused_variant_decode_and_prefill(variant):
    tuning = {B.LORA_TUNE_FUSED_VARIANT: variant}
    run_and_check(wl.config2(shrink=8, n_tokens=300), path=B.LORA_PATH_FUSED, tuning=tuning)
    run_and_check(wl.config3(shrink=8, n_req=6, len_div=8), path=B.LORA_PATH_FUSED, tuning=tuning, packed=True)


@pytest.mark.parametrize("variant", SPLIT_VARIANTS)
def test_split_variant_decode(variant):
    tuning = {B.LORA_TUNE_SPLIT_VARIANT: variant}
    run_and_check(wl.config2(shrink=8, n_tokens=300), path=B.LORA_PATH_SPLITK, tuning=tuning)
    run_and_check(wl.config4(shrink=8), path=B.LORA_PATH_SPLITK, split_k=3, tuning=tuning, packed=True)


@pytest.mark.parametrize("variant", [6, 7])
def test_whole_line_split_variants_short_k_ranges(variant):
    # 16 splits of a 512-wide K leave every workgroup fewer K tiles than the ring has stages
    tuning = {B.LORA_TUNE_SPLIT_VARIANT: variant}
    run_and_check(wl.config1(), path=B.LORA_PATH_SPLITK, split_k=16, tuning=tuning)
    run_and_check(wl.config1(), path=B.LORA_PATH_SPLITK, split_k=2, tuning=tuning)


@pytest.mark.parametrize("mode", [B.LORA_INLINE_SHRINK_OFF, B.LORA_INLINE_SHRINK_ON])
@pytest.mark.parametrize("variant", [8, 9, 10, 11])
def test_shrink_inside_the_fused_launch(mode, variant):
    # fused path up to 1024 tokens: the shrink by the first workgroups of the GEMM launch, or as a launch of its own;
    # two steps in a row (the launch leaves its counters at zero for the next one)
    tuning = {B.LORA_TUNE_INLINE_SHRINK: mode, B.LORA_TUNE_FUSED_VARIANT: variant}
    run_and_check(wl.config2(shrink=8, n_tokens=300), path=B.LORA_PATH_FUSED, tuning=tuning, packed=True)
    run_and_check(wl.config4(shrink=8), path=B.LORA_PATH_FUSED, tuning=tuning, packed=True)
    run_and_check(wl.qwen_decode(shrink=4, n_tokens=200), path=B.LORA_PATH_FUSED, tuning=tuning)
