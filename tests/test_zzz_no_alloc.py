"""GPU test of the allocation-free entry point rapid_verify_attn_static (collected last on purpose).

It must give what rapid_verify_attn gives for the same inputs: both run the same kernels, so the
comparison is bit for bit, which is inside the attention tolerance by construction; the second, smaller
call runs with whatever the first one left in the library's static scratch array, and is also checked
against the float64 oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2502_20330_amd import binding
from paper_2502_20330_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _inputs(cfg, layer):
    import gpu_util as gu
    inp = wl.gen_attn_inputs(cfg, layer=layer)
    s = inp.seqs
    dev = dict(q=gu.bf16_to_dev(inp.q), k=gu.bf16_to_dev(inp.k), v=gu.bf16_to_dev(inp.v),
               ctx=torch.from_numpy(s.ctx_lens).cuda(), gam=torch.from_numpy(s.gammas).cuda(),
               pt=torch.from_numpy(s.page_table).cuda() if s.page_table is not None else None)
    return inp, dev


def _both(r, cfg, inp, dev):
    s = inp.seqs
    kw = dict(gammas=dev["gam"], page_table=dev["pt"], max_ctx=s.max_ctx, softmax_scale=cfg.softmax_scale)
    lse_a = torch.zeros((cfg.batch, cfg.n_q_heads, cfg.q_max), dtype=torch.float32, device="cuda")
    lse_b = torch.zeros_like(lse_a)
    want = r.rapid_verify_attn(dev["q"], dev["k"], dev["v"], dev["ctx"], lse_out=lse_a, **kw)
    out = torch.full_like(dev["q"], float("nan"))
    torch.cuda.synchronize()
    # number of allocations torch has ever made (frees by the garbage collector do not move it)
    allocations = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]
    before = allocations()
    got = r.rapid_verify_attn_static(dev["q"], dev["k"], dev["v"], dev["ctx"], out=out, lse_out=lse_b, **kw)
    torch.cuda.synchronize()
    assert allocations() == before
    assert got.data_ptr() == out.data_ptr()
    return want, got, lse_a, lse_b


def test_static_scratch_entry_point_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    import gpu_util as gu
    r = gu.rapid()
    # first call: a ragged, paged batch of three sequences with several splits each
    big = wl.scaled(wl.CONFIGS["ragged_paged"], name="static_big", batch=3, ctx=(9000, 40000))
    inp1, dev1 = _inputs(big, layer=11)
    want1, got1, la1, lb1 = _both(r, big, inp1, dev1)
    assert torch.equal(want1.view(torch.int16), got1.view(torch.int16))
    assert torch.equal(la1, lb1)
    # second call right after it: smaller (one short sequence, fewer rows, contiguous cache)
    small = wl.scaled(wl.CONFIGS["llama8b_32k"], name="static_small", ctx=(1500, 1500), gamma_choices=(3,))
    inp2, dev2 = _inputs(small, layer=12)
    want2, got2, la2, lb2 = _both(r, small, inp2, dev2)
    assert torch.equal(want2.view(torch.int16), got2.view(torch.int16))
    assert torch.equal(la2, lb2)
    s = inp2.seqs
    bs, ts, hs, ps = wl.kv_strides(small, s)
    ref = oracle.verify_attn(inp2.q, inp2.k, inp2.v, s.ctx_lens, oracle.KVLayout(bs, ts, hs), Hkv=small.n_kv_heads,
                             scale=small.softmax_scale, gammas=s.gammas)
    gu.assert_attn_close(gu.bf16_to_host(got2), ref, "static entry point, second call")


def test_static_scratch_entry_point_refuses_shapes_beyond_its_limit():
    import gpu_util as gu
    r = gu.rapid()
    q = torch.zeros((64, 9, 32, 128), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((64, 16, 8, 128), dtype=torch.bfloat16, device="cuda")
    ctx = torch.full((64,), 16, dtype=torch.int32, device="cuda")
    shape = r.attn_shape(q, kv, 131072, chunk_tokens=2048)     # 64 splits per (sequence, head)
    shape.kv_batch_stride = 131072 * 8 * 128                # host-side description of a large cache; never launched
    need = r.lib.rapid_verify_attn_workspace_bytes(r._ctx, ctypes.byref(shape))
    assert need > binding.STATIC_SCRATCH_BYTES
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = r.lib.rapid_verify_attn_static(r._ctx, ctypes.byref(shape), P(q), P(kv), P(kv), P(ctx), None, None, P(q),
                                        None, None)
    assert rc == binding.RAPID_ETOOLARGE
    assert b"scratch" in r.lib.rapid_strerror(rc)
