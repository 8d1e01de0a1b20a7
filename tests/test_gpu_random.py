"""Seeded random shapes through the same parity harness as the hand-picked cases: decode steps
(fixed context), growing context and sparse prefill, each against the oracle.  The draw covers
head dims, GQA groups, budgets (K, Kq, Ns, Nw), pool capacities beyond K, ragged tails, pooling
windows that differ from the blocks, both victim policies, both dtypes and all query structures.
A case the library declines by design (an unsupported group size) counts as skipped.
"""
import numpy as np
import pytest

from helpers import small_workload
from nosa_inputs import random_residency
from pipeline import run_growing, run_parity, run_prefill_parity

pytestmark = pytest.mark.gpu

POOLS = [(64, 64), (64, 64), (64, 64), (32, 16), (16, 32), (32, 32)]


def _budget(rng, big):
    ns = int(rng.choice([1, 1, 2]))
    nw = int(rng.integers(1, 17 if big else 5))
    kq = int(rng.integers(0, 17 if big else 5))
    ke = int(rng.integers(0, 30 if big else 6))
    return ns, nw, kq, ke


def _run(fn, *a, **kw):
    import paper_2510_13602_amd as nosa
    try:
        return fn(*a, **kw)
    except nosa.NosaError as e:
        if "unsupported" in str(e):
            pytest.skip(str(e))
        raise


@pytest.mark.parametrize("case", range(16))
def test_random_decode_steps(case):
    rng = np.random.default_rng(1000 + case)
    d, hkv = int(rng.choice([64, 128])), int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 3, 4, 6, 8]))
    ns, nw, kq, ke = _budget(rng, rng.random() < 0.3)
    K = ns + nw + kq + ke
    nblk = int(rng.integers(max(1, K // 2), 4 * K + 8))
    tail = int(rng.integers(0, 64)) * int(rng.random() < 0.7)
    T = max(1, 64 * nblk + tail - 64 * int(tail > 0))
    C = K + int(rng.integers(0, K + 1)) * int(rng.random() < 0.5)
    pool = POOLS[int(rng.integers(0, len(POOLS)))]
    w = small_workload(batch=int(rng.choice([1, 2, 3])), n_q_heads=g * hkv, n_kv_heads=hkv, head_dim=d, context=T,
                       k_blocks=K, kq_blocks=kq, sink_blocks=ns, window_blocks=nw, gpu_slots=C,
                       dtype=str(rng.choice(["bf16", "bf16", "fp32"])),
                       structure=str(rng.choice(["planted", "key_offset", "heavy", "ar1", "drift"])),
                       pool_kernel=pool[0], pool_stride=pool[1], victim_policy=int(rng.random() < 0.4))
    seed = int(rng.integers(0, 1 << 30))
    res = random_residency(w, seed, 0, w.max_blocks) if rng.random() < 0.4 else None
    _run(run_parity, w, seed, steps=int(rng.integers(2, 6)), overlap=bool(rng.random() < 0.6), residency=res)


@pytest.mark.parametrize("case", range(8))
def test_random_ragged_batches(case):
    """Every batch element at its own token count, empty and one-token sequences included."""
    rng = np.random.default_rng(1500 + case)
    d, hkv, g = int(rng.choice([64, 128])), int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 4, 8]))
    ns, nw, kq, ke = _budget(rng, False)
    K = ns + nw + kq + ke
    T = 64 * int(rng.integers(K, 4 * K + 8))
    B = int(rng.integers(2, 6))
    C = K + int(rng.integers(0, K + 1)) * int(rng.random() < 0.5)
    pool = POOLS[int(rng.integers(0, len(POOLS)))]
    w = small_workload(batch=B, n_q_heads=g * hkv, n_kv_heads=hkv, head_dim=d, context=T, k_blocks=K, kq_blocks=kq,
                       sink_blocks=ns, window_blocks=nw, gpu_slots=C, dtype=str(rng.choice(["bf16", "fp32"])),
                       structure=str(rng.choice(["planted", "key_offset", "ar1"])), pool_kernel=pool[0], pool_stride=pool[1],
                       victim_policy=int(rng.random() < 0.4))
    n_tok = rng.integers(0, T + 1, size=B).astype(np.int32)
    n_tok[rng.integers(0, B)] = T
    n_tok[rng.integers(0, B)] = int(rng.choice([0, 1, 63, 64, 65]))
    _run(run_parity, w, int(rng.integers(0, 1 << 30)), steps=3, overlap=bool(rng.random() < 0.6), poison=False, n_tokens=n_tok)


@pytest.mark.parametrize("case", range(8))
def test_random_growing_context(case):
    rng = np.random.default_rng(2000 + case)
    d, hkv, g = int(rng.choice([64, 128])), int(rng.choice([1, 2])), int(rng.choice([1, 2, 4, 8]))
    ns, nw, kq, ke = _budget(rng, False)
    K = ns + nw + kq + ke
    T = 64 * int(rng.integers(K, 3 * K + 4)) + int(rng.integers(0, 64))
    steps = int(rng.integers(20, 150))
    C = K + int(rng.integers(0, K + 1)) * int(rng.random() < 0.5)
    pool = POOLS[int(rng.integers(0, len(POOLS)))]
    w = small_workload(batch=int(rng.choice([1, 2])), n_q_heads=g * hkv, n_kv_heads=hkv, head_dim=d, context=T, k_blocks=K,
                       kq_blocks=kq, sink_blocks=ns, window_blocks=nw, gpu_slots=C, dtype=str(rng.choice(["bf16", "fp32"])),
                       generated=steps + 1, structure=str(rng.choice(["planted", "key_offset", "drift"])),
                       pool_kernel=pool[0], pool_stride=pool[1], victim_policy=int(rng.random() < 0.3))
    _run(run_growing, w, int(rng.integers(0, 1 << 30)), steps)


@pytest.mark.parametrize("case", range(16))
def test_random_prefill(case):
    rng = np.random.default_rng(3000 + case)
    d, hkv = int(rng.choice([64, 128])), int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16]))
    big = rng.random() < 0.4
    ns, nw, kq, ke = _budget(rng, big)
    K = ns + nw + kq + ke
    p0 = 64 * int(rng.integers(0, 100 if big else 24)) * int(rng.random() < 0.8)
    lq = 64 * int(rng.integers(1, 7))
    n_blocks = max(K, (p0 + lq) // 64 + int(rng.integers(0, 3)))
    pool = POOLS[int(rng.integers(0, len(POOLS)))]
    w = small_workload(batch=int(rng.choice([1, 2, 3])), n_q_heads=g * hkv, n_kv_heads=hkv, head_dim=d, context=p0 + lq,
                       k_blocks=K, kq_blocks=kq, sink_blocks=ns, window_blocks=nw, gpu_slots=n_blocks, dtype="bf16",
                       structure=str(rng.choice(["planted", "key_offset", "heavy"])), generated=n_blocks * 64 - (p0 + lq),
                       pool_kernel=pool[0], pool_stride=pool[1])
    _run(run_prefill_parity, w, seed=int(rng.integers(0, 1 << 30)), p0=p0, lq=lq)
