"""Seeded sweep of irregular shapes through sdllm_block_step (all three cache states) against the
oracle: head counts and group sizes, prompt lengths that leave ragged tiles on either side of the
block, blocks in the middle of the generation, retention ratios, pooling windows and the ranking
variants, in combinations the hand-picked cases of test_gpu_parity.py do not list."""
import numpy as np
import pytest

from paper_2508_02558_amd import binding as B
from paper_2508_02558_amd import workloads as wl
from tests.test_gpu_parity import _run_block

pytestmark = pytest.mark.gpu


def _random_case(seed):
    rng = np.random.default_rng(5000 + seed)
    group = int(rng.choice([1, 1, 2, 3, 4, 7, 8]))
    n_kv = int(rng.integers(1, 4))
    gen_blocks = int(rng.integers(2, 5))
    w = wl.WORKLOADS["llada8b_layer"].scaled(
        batch=int(rng.integers(1, 4)), n_q_heads=group * n_kv, n_kv_heads=n_kv,
        prompt=int(rng.integers(0, 700)), gen=32 * gen_blocks,
        retention=float(rng.choice([0.1, 0.25, 0.5, 0.5, 0.7, 0.9])), pool_kernel=int(rng.choice([1, 3, 3, 5, 7])))
    block_index = int(rng.integers(0, gen_blocks))
    modes = {}
    if rng.random() < 0.3:
        modes.update(select_mode=B.SDLLM_JOINT, k_rounding=B.SDLLM_FLOOR)
    if rng.random() < 0.3:
        modes.update(score_mode=B.SDLLM_LOGIT_MEAN)
    if rng.random() < 0.2:
        modes.update(pool_mode=B.SDLLM_AVG_POOL)
    if rng.random() < 0.2 and "select_mode" not in modes:
        modes.update(evict_scope=B.SDLLM_EVICT_PREFIX_ONLY)
    return w, block_index, modes


@pytest.mark.parametrize("seed", range(16))
def test_random_shape_block(seed):
    w, block_index, modes = _random_case(seed)
    _run_block(w, layer=seed, block_index=block_index, n_steps=3, **modes)


def _random_long_case(seed):
    """Shapes whose ranked segments take the two-launch selection (more than 8192 candidates): a long prompt,
    sometimes a long suffix as well, a block anywhere in the generation, every ranking variant."""
    rng = np.random.default_rng(9000 + seed)
    group = int(rng.choice([1, 2, 7]))
    prompt = int(rng.integers(8193, 45000))
    gen_blocks = int(rng.choice([2, 3, 300, 400]))          # the long generations give a long suffix too
    w = wl.WORKLOADS["llada8b_layer"].scaled(
        batch=int(rng.integers(1, 3)), n_q_heads=group, n_kv_heads=1, prompt=prompt, gen=32 * gen_blocks,
        retention=float(rng.choice([0.05, 0.25, 0.5, 0.8])), pool_kernel=int(rng.choice([1, 3, 3, 5, 9])))
    block_index = int(rng.integers(0, min(gen_blocks, 40)))
    modes = {}
    if rng.random() < 0.3:
        modes.update(select_mode=B.SDLLM_JOINT, k_rounding=B.SDLLM_FLOOR)
    if rng.random() < 0.3:
        modes.update(score_mode=B.SDLLM_LOGIT_MEAN)
    if rng.random() < 0.2:
        modes.update(pool_mode=B.SDLLM_AVG_POOL)
    if rng.random() < 0.2 and "select_mode" not in modes:
        modes.update(evict_scope=B.SDLLM_EVICT_PREFIX_ONLY)
    return w, block_index, modes


@pytest.mark.parametrize("seed", range(8))
def test_random_long_segment_block(seed):
    w, block_index, modes = _random_long_case(seed)
    _run_block(w, layer=seed, block_index=block_index, n_steps=3, **modes)
