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

W = synth.Workload


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def test_mha_32_kv_heads(torch_mod):
    run_workload(torch_mod, W("mha_32kv_16k", 1, 32, 32, 128, 128, (16384,), (256,), 4, 8.0), {0}, True)


def test_group_of_5_ragged_batch(torch_mod):
    run_workload(torch_mod, W("g5_40q8kv", 2, 40, 8, 128, 128, (20000, 12345), (400, 192), 4, 8.0), {0}, True)


def test_hash_bits_64_and_32(torch_mod):
    # no single-launch kernel for these widths: the step runs as three launches
    run_workload(torch_mod, W("r64_32k", 1, 32, 8, 128, 64, (32768,), (512,), 4, 8.0), {0}, False)
    run_workload(torch_mod, W("r32_16k", 1, 32, 8, 128, 32, (16384,), (256,), 0, 1.0), {0}, False)


def test_hash_bits_256_group_of_8(torch_mod):
    run_workload(torch_mod, W("r256_g8", 2, 64, 8, 128, 256, (24000, 9000), (384, 128), 8, 16.0), {0}, True)


def test_budgets_0p4_and_3p13_percent(torch_mod):
    run_workload(torch_mod, W("budget_0p4", 1, 32, 8, 128, 128, (32768,), (128,), 4, 8.0), {0}, True, dense=False)
    run_workload(torch_mod, W("budget_3p13", 1, 32, 8, 128, 128, (32768,), (1024,), 4, 8.0), {0}, True, dense=False)


def test_context_256k_with_append(torch_mod):
    w = W("ctx_256k", 1, 32, 8, 128, 128, (262144,), (4096,), 4, 8.0, append_steps=2)
    run_workload(torch_mod, w, {0, 1}, True)
