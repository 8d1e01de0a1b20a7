"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every
symbol that include/nosa.h declares, and validates parameter sets on the host."""
import ctypes
import os
import re

import pytest

import paper_2510_13602_amd as nosa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "nosa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nosa_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = nosa.load_library()
    names = _declared()
    assert {"nosa_block_score", "nosa_select", "nosa_fetch", "nosa_sparse_decode"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/nosa.h but not exported"
    assert sorted(nosa.EXPORTS) == names


def _good(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, k_blocks=64, kq_blocks=8, sink_blocks=1,
                window_blocks=16, gpu_slots=64, max_blocks=512, n_sub_max=512, dtype="bf16")
    base.update(kw)
    return nosa.make_params(**base)


def test_params_struct_matches_header_layout():
    assert ctypes.sizeof(nosa.Params) == 17 * 4
    nosa.validate_params(_good())
    nosa.validate_params(_good(n_q_heads=10))           # bf16: any group of 1..16 heads
    nosa.validate_params(_good(n_q_heads=14))
    assert nosa.load_library().nosa_workspace_bytes(_good()) >= 4 * 2 * 16 * 4 * 130 * 4


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=96), nosa.binding.NOSA_ESHAPE),
    (dict(block_size=32), nosa.binding.NOSA_ESHAPE),
    (dict(n_q_heads=7), nosa.binding.NOSA_EINVAL),
    (dict(n_q_heads=10, dtype="fp32"), nosa.binding.NOSA_ESHAPE),   # group 5: bf16 only (matrix-core kernel)
    (dict(n_q_heads=34), nosa.binding.NOSA_ESHAPE),          # group 17: more heads than one matrix-core tile
    (dict(kq_blocks=60), nosa.binding.NOSA_ESHAPE),          # sink + window + kq > K
    (dict(gpu_slots=32), nosa.binding.NOSA_ESHAPE),          # C < K
    (dict(window_blocks=0), nosa.binding.NOSA_EINVAL),
    (dict(dtype=7), nosa.binding.NOSA_EINVAL),
    (dict(victim_policy=2), nosa.binding.NOSA_EINVAL),
    (dict(k_blocks=512, gpu_slots=512), nosa.binding.NOSA_ESHAPE),
    (dict(max_blocks=100000), nosa.binding.NOSA_ESHAPE),
    (dict(n_sub_max=513), nosa.binding.NOSA_EINVAL),
    (dict(pool_kernel=128), nosa.binding.NOSA_EINVAL),
    (dict(batch=0), nosa.binding.NOSA_EINVAL),
    (dict(softmax_scale=float("nan")), nosa.binding.NOSA_EINVAL),
])
def test_validation_rejects(kw, code):
    with pytest.raises(nosa.NosaError) as e:
        nosa.validate_params(_good(**kw))
    assert e.value.code == code
    assert nosa.load_library().nosa_workspace_bytes(_good(**kw)) == 0


def test_null_arguments_are_errors_not_crashes():
    lib = nosa.load_library()
    assert lib.nosa_validate_params(None, None, 0) == nosa.binding.NOSA_EINVAL
    assert lib.nosa_create(None, None, None) == nosa.binding.NOSA_EINVAL
    assert lib.nosa_destroy(None) == 0
    assert lib.nosa_block_score(None, None, None, None, None, None, None) == nosa.binding.NOSA_EINVAL
    assert lib.nosa_select(None, *([None] * 9)) == nosa.binding.NOSA_EINVAL
    assert lib.nosa_fetch(None, *([None] * 8)) == nosa.binding.NOSA_EINVAL
    assert lib.nosa_sparse_decode(None, *([None] * 10)) == nosa.binding.NOSA_EINVAL
    assert lib.nosa_prefill_select(None, None, None, None, 0, 64, None, None, None, None, None) == nosa.binding.NOSA_EINVAL
    assert lib.nosa_prefill_attend(None, None, None, None, None, None, None, 0, 64, None, None) == nosa.binding.NOSA_EINVAL
    assert b"NULL" in lib.nosa_last_error(None)


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(nosa.NosaError):
        nosa.Nosa(_good())


def test_bench_refuses_more_than_one_gpu():
    """The path runs on one GPU; the benchmark says so instead of pretending to scale."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)
