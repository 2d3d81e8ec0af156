"""`-m gpu`: the HIP library against the CPU oracle, through the C ABI, on the same seeded inputs."""
import sys

import numpy as np
import pytest

from tests.parity import run_parity, assert_close
from workloads import make_workload, table_values

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2208_05321_amd import load_library
    load_library()          # fail loudly if the HIP library is not built
    return torch


@pytest.mark.parametrize("warm", [True, False])
def test_config1_full(torch_cuda, warm):
    log(f"config 1, warm={warm}")
    w = make_workload("c1")
    tot = run_parity(w, w.num_batches, warm=warm)
    assert 0.5 < tot["hit_ids"] / tot["ids"] < 0.95


@pytest.mark.parametrize("name,scale,ratio,batches", [
    ("c2", 0.1, 0.015, 12), ("c3", 0.03, 0.03, 8), ("c4", 0.01, 0.03, 8), ("c5", 0.05, 0.015, 6),
])
def test_scaled_configs(torch_cuda, name, scale, ratio, batches):
    log(f"{name} at scale {scale}")
    w = make_workload(name, scale=scale, cache_ratio=ratio)
    tot = run_parity(w, batches, warm=True, deep_every=3, values_every=3, log=log)
    assert tot["miss"] > 0 and tot["evict"] > 0


def test_cold_start_scaled_c2(torch_cuda):
    w = make_workload("c2", scale=0.05, cache_ratio=0.05)
    tot = run_parity(w, 8, warm=False, deep_every=2, values_every=2, log=log)
    assert tot["evict"] > 0


@pytest.mark.parametrize("staging_rows", [1, 7, 100000])
def test_results_independent_of_staging_buffer(torch_cuda, staging_rows):
    """The transmitter's buffer bound changes the number of rounds, never the result (Section 4.3)."""
    w = make_workload("c2", scale=0.004, cache_ratio=0.05)
    run_parity(w, 6, warm=True, staging_rows=staging_rows)


@pytest.mark.parametrize("staging_rows", [0, 5])
def test_staged_block_transmitter(torch_cuda, staging_rows):
    """The paper's gather -> bulk copy -> scatter transmitter gives the same results as the direct one."""
    w = make_workload("c2", scale=0.02, cache_ratio=0.04)
    run_parity(w, 6, warm=True, staged=True, staging_rows=staging_rows)
    run_parity(w, 4, warm=False, staged=True, staging_rows=staging_rows)
