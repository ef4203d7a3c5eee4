"""CPU-side checks of the boundary: the C-ABI library loads and exports every
function include/rapid.h declares; host-side planning entry points behave."""
import ctypes
import os
import re

import pytest

from paper_2502_20330_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rapid.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rapid_[a-z_]+)\s*\(", text)))


def test_header_declares_the_two_operations():
    names = declared_functions()
    assert "rapid_verify_attn" in names and "rapid_accept" in names


def test_library_loads_and_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("librapid.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in rapid.h but not exported"
    assert sorted(binding.EXPORTS) == declared_functions()


def test_strerror_and_shape_checks_need_no_gpu():
    lib = binding.load_library()
    assert lib.rapid_strerror(0) == b"ok"
    assert b"support" in lib.rapid_strerror(-3)
    s = binding.AttnShape()
    s.batch, s.q_max, s.n_q_heads, s.n_kv_heads, s.head_dim, s.max_ctx = 1, 9, 32, 8, 128, 131072
    s.gamma, s.softmax_scale = 8, 0.088
    s.kv_batch_stride, s.kv_token_stride, s.kv_head_stride = 131072 * 1024, 1024, 128
    chunk = lib.rapid_verify_attn_chunk(None, ctypes.byref(s))
    assert chunk > 0 and chunk % 128 == 0
    nsplit = -(-s.max_ctx // chunk)
    need = lib.rapid_verify_attn_workspace_bytes(None, ctypes.byref(s))
    assert need >= 1 * 8 * nsplit * 36 * 130 * 4
    s.head_dim = 96
    assert lib.rapid_verify_attn_chunk(None, ctypes.byref(s)) == -3
    assert lib.rapid_verify_attn_workspace_bytes(None, ctypes.byref(s)) == 0
    s.head_dim, s.softmax_scale = 128, 0.0
    assert lib.rapid_verify_attn_chunk(None, ctypes.byref(s)) == -1
    assert lib.rapid_accept_workspace_bytes(None, 1, 8, 128256) > 0
    assert lib.rapid_accept_workspace_bytes(None, 0, 8, 128256) == 0


def test_product_path_has_no_cpu_fallback():
    """Without a GPU the binding refuses to construct instead of computing elsewhere."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(binding.RapidError):
        binding.Rapid(0)


def test_product_code_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_20330_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "rapid_oracle" not in text, f


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU program: any other --gpus value ends with a message and a non-zero status."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
