"""The 3B- and 8B-shaped workloads at their full sizes against the oracle.

``*_every_unit_*``: every unit at every step of the workload (256 for the 8B shape, 128 for the 3B shape) for the
selection, the miss count, the load list and the residency maps (bit-exact), and every unit's attention output
on 16 evenly spaced steps plus the last; on the first layer
of the stack in the launch configuration ``bench.py`` times (one stream, ``nosa_decode_step``, the plain
attention kernel at its default split count) and on the last layer in the library's default order (gather on
the side stream, two attention launches around it).  ``*_sampled_units`` keeps the older check (default order,
sampled units re-run as one-unit oracle problems, size-independent properties over all units)."""
import pytest

from nosa_inputs import CONFIGS
from pipeline import run_fullsize_all_units, run_fullsize_sampled

pytestmark = pytest.mark.gpu



def _attention_steps(steps):
    return sorted(set(range(0, steps, steps // 16)) | {steps - 1})


@pytest.mark.parametrize("layer_index,mode", [(0, "fused"), (31, "overlap")])
def test_8b_shaped_every_unit_every_step(layer_index, mode):
    """batch 64, 32 q / 8 KV heads, d128, 32768 tokens, K = 64, Kq = 8, bf16: 512 units, 8 GiB host pool."""
    w = CONFIGS["8b"]
    assert layer_index < w.layers
    r = run_fullsize_all_units(w, seed=0, layer_index=layer_index, steps=w.steps, attention_steps=_attention_steps(w.steps),
                               mode=mode)
    print("8b all units", layer_index, mode, r, flush=True)


@pytest.mark.parametrize("layer_index,mode", [(0, "fused"), (27, "overlap")])
def test_3b_shaped_every_unit_every_step(layer_index, mode):
    """batch 32, 24 q / 4 KV heads (group 6), d128, 16384 tokens, AR(1) queries: 128 units, 4 attention splits."""
    w = CONFIGS["3b"]
    assert layer_index < w.layers
    r = run_fullsize_all_units(w, seed=0, layer_index=layer_index, steps=w.steps, attention_steps=_attention_steps(w.steps),
                               mode=mode)
    print("3b all units", layer_index, mode, r, flush=True)


def test_8b_shaped_larger_pool_importance_ranked_victims():
    """The 8B shape with a pool of C = 96 slots for K = 64 selected blocks and victim_policy 1 (a miss overwrites
    the least important block outside the selection): every unit, 24 steps, one-stream order."""
    w = CONFIGS["8b"].replace(gpu_slots=96, victim_policy=1)
    r = run_fullsize_all_units(w, seed=0, layer_index=1, steps=24, attention_steps=[0, 11, 23], mode="fused")
    print("8b C=96 policy 1", r, flush=True)


def test_8b_shaped_full_size_sampled_units():
    run_fullsize_sampled(CONFIGS["8b"], seed=0, steps=5, n_samples=10)


def test_3b_shaped_full_size_sampled_units():
    run_fullsize_sampled(CONFIGS["3b"], seed=0, steps=6, n_samples=8)
