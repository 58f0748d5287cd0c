"""Shape sweep with the same kernels (the axes of the paper's efficiency figure and ablations):
multi-head attention without grouping (Llama-2 style, one query head per KV head), a group of 5
(Qwen-2.5 style 40 query / 8 KV heads), hash widths r = 32 / 64 / 256 (hash-bit ablation), token
budgets 0.4 % and 3.13 %, and a 256K-token cache.  Every case: bulk key encode, a decode step in
both launch forms and the dense baseline, each against the oracle at the bar of the other GPU tests.
"""
import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(400)]

from paper_2506_02572_amd import synth
from tests.test_gpu_full_configs import run_workload

@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def test_mha_32_kv_heads(torch_mod):
    run_workload(torch_mod, synth.SWEEP["mha32_32k"], {0}, True)


def test_group_of_5_ragged_batch(torch_mod):
    run_workload(torch_mod, synth.SWEEP["g5_40q8kv_32k"], {0}, True)


def test_group_of_16(torch_mod):
    run_workload(torch_mod, synth.SWEEP["g16_128q8kv_32k"], {0}, True)


def test_hash_bits_64_and_32(torch_mod):
    run_workload(torch_mod, synth.SWEEP["r64_32k"], {0}, True)
    run_workload(torch_mod, synth.SWEEP["r32_32k"], {0}, True)


def test_hash_bits_256_group_of_8(torch_mod):
    run_workload(torch_mod, synth.SWEEP["r256_g8_ragged"], {0}, True)


def test_budgets_0p4_and_3p13_percent(torch_mod):
    run_workload(torch_mod, synth.SWEEP["budget0p4_32k"], {0}, True, dense=False)
    run_workload(torch_mod, synth.SWEEP["budget3p13_32k"], {0}, True, dense=False)


def test_context_256k_with_append(torch_mod):
    run_workload(torch_mod, synth.SWEEP["ctx256k"], {0, 1}, True)


def test_batch_8_at_32k_the_papers_headline_shape(torch_mod):
    run_workload(torch_mod, synth.SWEEP["b8_32k"], {0}, True)
