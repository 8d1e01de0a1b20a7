"""The 3B- and 8B-shaped workloads at their full sizes, in the launch configuration bench.py times,
checked on sampled units against the oracle and on all units via size-independent properties."""
import pytest

from nosa_inputs import CONFIGS
from pipeline import run_fullsize_sampled

pytestmark = pytest.mark.gpu


def test_8b_shaped_full_size_sampled_units():
    """batch 64, 32 q / 8 KV heads, d128, 32768 tokens, K = 64, Kq = 8, bf16: 512 units, 8 GiB host pool."""
    run_fullsize_sampled(CONFIGS["8b"], seed=0, steps=5, n_samples=10)


def test_3b_shaped_full_size_sampled_units():
    """batch 32, 24 q / 4 KV heads (group 6), d128, 16384 tokens, AR(1) queries."""
    run_fullsize_sampled(CONFIGS["3b"], seed=0, steps=6, n_samples=8)
