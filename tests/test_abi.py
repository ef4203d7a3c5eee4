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


def _shape(batch, q_max, hq, hkv, d, max_ctx, token_major=True, page=0, hint=0):
    s = binding.AttnShape()
    s.batch, s.q_max, s.n_q_heads, s.n_kv_heads, s.head_dim, s.max_ctx = batch, q_max, hq, hkv, d, max_ctx
    s.gamma, s.softmax_scale = q_max - 1, d ** -0.5
    if page:
        s.page_size, s.max_pages = page, -(-max_ctx // page)
        s.kv_page_stride, s.kv_token_stride, s.kv_head_stride = page * hkv * d, hkv * d, d
    elif token_major:
        s.kv_batch_stride, s.kv_token_stride, s.kv_head_stride = max_ctx * hkv * d, hkv * d, d
    else:
        s.kv_batch_stride, s.kv_token_stride, s.kv_head_stride = max_ctx * hkv * d, d, max_ctx * d
    s.ctx_sum_hint = hint
    return s


def test_split_planning_on_the_named_workloads_needs_no_gpu():
    """Host-side planning (no context: 256 compute units assumed): tokens per KV split for the benchmark shapes,
    the row cap, the 32-bit span limits and the chunk of the output head."""
    lib = binding.load_library()
    chunk = lambda s: lib.rapid_verify_attn_chunk(None, ctypes.byref(s))
    # one workgroup per compute unit for sequences of equal length: 8 kv heads x 32 splits
    assert chunk(_shape(1, 9, 32, 8, 128, 131072)) == 4096                      # configs 3 and 5
    assert chunk(_shape(1, 9, 64, 8, 128, 131072)) == 4096
    assert chunk(_shape(1, 9, 32, 8, 128, 32768)) == 1024                       # config 2
    assert chunk(_shape(1, 11, 28, 4, 128, 131072)) == 2048                     # 4 kv heads x 64 splits
    assert chunk(_shape(1, 1, 32, 8, 128, 8192)) == 256                         # drafter decode: the minimum
    assert chunk(_shape(1, 5, 4, 1, 64, 2048)) == 256
    # a ragged batch whose total the caller knows is planned for two rounds of workgroups
    ragged = chunk(_shape(8, 9, 32, 8, 128, 131072, page=16, hint=560858))
    plain = chunk(_shape(8, 9, 32, 8, 128, 131072, page=16))
    assert ragged % 128 == 0 and plain % 128 == 0 and ragged < plain
    assert 8 * (560858 // ragged + 8) <= 2 * 256 + 8 * 8
    # an explicit split is rounded up to whole tiles of 128 tokens
    s = _shape(1, 9, 32, 8, 128, 131072)
    s.chunk_tokens = 1000
    assert chunk(s) == 1024
    # rows per kv head: (gamma + 1) * group <= 96
    assert chunk(_shape(1, 11, 64, 8, 128, 131072)) > 0                         # 88 rows
    assert chunk(_shape(1, 12, 64, 8, 128, 131072)) == 4096                     # 96 rows
    assert chunk(_shape(1, 13, 64, 8, 128, 131072)) == -3                       # 104 rows
    # offsets inside one sequence (or page) are 32-bit: 2^21 tokens x 2 KiB per token do not fit
    assert chunk(_shape(1, 9, 32, 8, 128, 1 << 21)) == -3
    assert chunk(_shape(1, 9, 32, 8, 128, 1 << 21, token_major=False)) > 0     # 256 B per token do
    assert chunk(_shape(1, 9, 32, 8, 128, 1 << 21, page=16)) > 0               # and pages are small
    # the workspace grows with the number of splits and rows
    ws = lambda s: lib.rapid_verify_attn_workspace_bytes(None, ctypes.byref(s))
    assert ws(_shape(1, 9, 64, 8, 128, 131072)) > ws(_shape(1, 9, 32, 8, 128, 131072)) > 0
    assert ws(_shape(2, 9, 32, 8, 128, 131072)) >= ws(_shape(1, 9, 32, 8, 128, 131072))
    # output head: one chunk per workgroup, whole rounds of 256 workgroups, at most 512 entries, any row count
    for vocab, want in ((128256, 512), (152064, 304), (32000, 128), (16, 16), (1000, 16)):
        for rows in (1, 9, 72, 96):
            ch = lib.rapid_lm_head_chunk(None, vocab, rows)
            assert ch == want, (vocab, rows, ch)
            assert lib.rapid_lm_head_stat_chunks(None, vocab, rows) == -(-vocab // ch)
    assert lib.rapid_lm_head_chunk(None, 128256, 97) == 0 and lib.rapid_lm_head_chunk(None, 0, 9) == 0


def test_split_planning_invariants_on_random_shapes():
    """Seeded random shapes: an accepted shape gets whole tiles of 128 tokens per split, a workspace that holds
    the partials of every (sequence, kv head, split, packed row) and grows with nothing but those counts; a
    refused shape gets an error code from the chunk query and 0 bytes from the workspace query."""
    import random
    lib = binding.load_library()
    rng = random.Random(20330)
    seen_ok = seen_bad = 0
    for _ in range(400):
        d = rng.choice([64, 128, 128, 128, 96])
        hkv = rng.choice([1, 2, 3, 4, 8])
        group = rng.choice([1, 2, 4, 7, 8])
        q_max = rng.randint(1, 14)
        batch = rng.choice([1, 1, 2, 8])
        max_ctx = rng.choice([1, 100, 4096, 33000, 131072, 1 << 20])
        layout = rng.choice(["token", "head", "paged"])
        page = rng.choice([16, 64, 24]) if layout == "paged" else 0
        s = _shape(batch, q_max, hkv * group, hkv, d, max_ctx, token_major=layout != "head", page=page)
        s.chunk_tokens = rng.choice([0, 0, 0, 1000, 128, 5000])
        chunk = lib.rapid_verify_attn_chunk(None, ctypes.byref(s))
        ws = lib.rapid_verify_attn_workspace_bytes(None, ctypes.byref(s))
        rows = q_max * group
        legal = d in (64, 128) and rows <= 96 and page in (0, 16, 64) and q_max <= max_ctx
        if chunk <= 0:
            seen_bad += 1
            assert ws == 0 and chunk in (-1, -3), (chunk, ws)
            assert not legal or max_ctx >= 1 << 20, "a legal shape was refused"   # (2^20 tokens x 2 KiB overflow 32 bits)
            continue
        seen_ok += 1
        assert legal
        assert chunk % 128 == 0
        if s.chunk_tokens:
            assert chunk == -(-s.chunk_tokens // 128) * 128
        nsplit = -(-max_ctx // chunk)
        need = batch * hkv * nsplit * (-(-rows // 16) * 16) * (d + 2) * 4
        assert need <= ws <= need + 2 * 256, (ws, need)
    assert seen_ok > 100 and seen_bad > 30


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
