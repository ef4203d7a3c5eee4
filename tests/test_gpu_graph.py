"""A whole validation round recorded into a HIP graph and replayed: the library changes no function
attribute and allocates nothing on its launch paths, so every entry point can be captured.  Each replay
(with ordinary eager work and synchronisations in between) must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

from paper_2502_20330_amd import workloads as wl

pytestmark = pytest.mark.gpu

gu = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global gu
    import gpu_util
    gu = gpu_util
    yield


def test_captured_round_replays_identically():
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=4, ctx=(300, 4000), vocab=8192, name="graph_round")
    inp = wl.gen_attn_inputs(cfg)
    s = inp.seqs
    acc = wl.gen_accept_inputs(cfg, seqs=s)
    r = gu.rapid()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    q, k, v = gu.bf16_to_dev(inp.q), gu.bf16_to_dev(inp.k), gu.bf16_to_dev(inp.v)
    rng = np.random.default_rng(5)
    kn = gu.bf16_to_dev(wl.f32_to_bf16_bits(rng.standard_normal((cfg.batch, cfg.q_max, cfg.n_kv_heads, cfg.head_dim),
                                                                 dtype=np.float32)))
    vn = gu.bf16_to_dev(wl.f32_to_bf16_bits(rng.standard_normal((cfg.batch, cfg.q_max, cfg.n_kv_heads, cfg.head_dim),
                                                                 dtype=np.float32)))
    ctx, gam, pt = dev(s.ctx_lens), dev(s.gammas), dev(s.page_table)
    zt, zd, tok, u = dev(acc.target_logits), dev(acc.draft_logits), dev(acc.draft_tokens), dev(acc.uniforms)
    h, w = wl.gen_lm_head_inputs(5, 1024, 3000)
    hd, wd = gu.bf16_to_dev(h), gu.bf16_to_dev(w)

    out = torch.empty_like(q)
    lens = torch.empty_like(ctx)
    # zeros: ratio entries at positions k >= gamma_b are never written by the library
    outs = (torch.zeros(cfg.batch, dtype=torch.int32, device="cuda"),
            torch.zeros(cfg.batch, cfg.q_max, dtype=torch.int32, device="cuda"),
            torch.zeros(cfg.batch, cfg.gamma_max, dtype=torch.float32, device="cuda"))
    logits = torch.empty(5, 3000, dtype=torch.float32, device="cuda")
    stats = torch.empty(5, r.lib.rapid_lm_head_stat_chunks(r._ctx, 3000, 5), 2, dtype=torch.float32, device="cuda")

    def round_():
        r.rapid_kv_append(k, v, kn, vn, ctx, gammas=gam, page_table=pt, max_ctx=s.max_ctx)
        r.rapid_verify_attn(q, k, v, ctx, gammas=gam, page_table=pt, max_ctx=s.max_ctx,
                            softmax_scale=cfg.softmax_scale, out=out)
        r.rapid_lm_head(hd, wd, logits=logits, stats=stats)
        r.rapid_accept(zt, zd, tok, cfg.eta, u, gammas=gam, outs=outs)
        lens.copy_(ctx)
        r.rapid_kv_commit(lens, outs[0], gammas=gam)

    round_()                                             # eager: also sizes the binding's workspace
    torch.cuda.synchronize()
    want = [t.clone() for t in (out, lens, logits, stats, *outs)]

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            round_()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        for t in (out, lens, logits, stats, *outs):      # eager work between replays: scrub the outputs
            t.fill_(0) if t.dtype != torch.bfloat16 else t.zero_()
        scratch = torch.randn(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lens", "logits", "stats", "n_accepted", "tokens", "ratio"),
                              (out, lens, logits, stats, *outs), want):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager round"
        assert torch.isfinite(scratch)
