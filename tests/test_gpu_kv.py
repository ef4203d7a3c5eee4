"""GPU parity: rapid_kv_append / rapid_kv_commit (C ABI) against the oracle, bit for bit (byte copies
and integer arithmetic), and one whole validation round: append -> verify attention -> accept -> commit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_20330_amd import workloads as wl

pytestmark = pytest.mark.gpu

gu = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global gu
    import gpu_util
    gu = gpu_util
    yield


def new_rows(cfg, seed):
    rng = np.random.default_rng(seed)
    shape = (cfg.batch, cfg.q_max, cfg.n_kv_heads, cfg.head_dim)
    return (wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)),
            wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)))


def append_case(cfg, head_major=False):
    inp = wl.gen_attn_inputs(cfg)
    s = inp.seqs
    kn, vn = new_rows(cfg, 77)
    k_ref, v_ref = inp.k.copy(), inp.v.copy()
    bs, ts, hs, ps = wl.kv_strides(cfg, s)
    lay = oracle.KVLayout(bs, ts, hs, cfg.page_size if cfg.paged else 0, ps,
                          s.page_table.shape[1] if s.page_table is not None else 0)
    oracle.kv_append(k_ref, v_ref, kn, vn, s.ctx_lens, lay, gammas=s.gammas, page_table=s.page_table)
    assert not np.array_equal(k_ref, inp.k)
    k, v = gu.bf16_to_dev(inp.k), gu.bf16_to_dev(inp.v)
    if head_major:
        k = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        v = v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    pt = torch.from_numpy(s.page_table).cuda() if s.page_table is not None else None
    gu.rapid().rapid_kv_append(k, v, gu.bf16_to_dev(kn), gu.bf16_to_dev(vn), torch.from_numpy(s.ctx_lens).cuda(),
                               gammas=torch.from_numpy(s.gammas).cuda(), page_table=pt, max_ctx=s.max_ctx)
    torch.cuda.synchronize()
    to_bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(to_bits(k), k_ref) and np.array_equal(to_bits(v), v_ref)
    return inp, kn, vn, k, v, k_ref, v_ref, lay


def test_append_contiguous_ragged_batch():
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=5, ctx=(40, 900), paged=False, name="kv_ragged")
    append_case(cfg)
    append_case(cfg, head_major=True)


def test_append_paged_16_and_64():
    for page in (16, 64):
        cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=4, ctx=(30, 700), page_size=page, name=f"kv_paged{page}")
        append_case(cfg)
        append_case(cfg, head_major=True)


def test_append_head_dim_64_gamma_0():
    cfg = wl.scaled(wl.CONFIGS["tiny"], batch=3, ctx=(1, 300), gamma_choices=(0,), name="kv_g0")
    append_case(cfg)


def test_commit_matches_oracle():
    rng = np.random.default_rng(4)
    B = 1000
    gam = rng.integers(0, 9, B).astype(np.int32)
    n = (rng.random(B) * (gam + 1)).astype(np.int32)
    ctx = (gam + 1 + rng.integers(0, 100000, B)).astype(np.int32)
    ref = oracle.kv_commit(ctx, n, gammas=gam)
    got = gu.rapid().rapid_kv_commit(torch.from_numpy(ctx.copy()).cuda(), torch.from_numpy(n).cuda(),
                                     gammas=torch.from_numpy(gam).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), ref)
    got2 = gu.rapid().rapid_kv_commit(torch.tensor([100, 50], dtype=torch.int32, device="cuda"),
                                      torch.tensor([8, 0], dtype=torch.int32, device="cuda"), 8)
    assert got2.cpu().tolist() == [100, 42]


def test_whole_validation_round_on_device():
    """append -> rapid_verify_attn -> rapid_accept -> rapid_kv_commit with lengths, gammas and accepted counts
    never leaving the device; attention against the oracle on the oracle-appended cache, lengths against the
    oracle's commit rule."""
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=4, ctx=(300, 3000), vocab=4099, name="kv_round")
    inp, kn, vn, k, v, k_ref, v_ref, lay = append_case(cfg)
    s = inp.seqs
    ctx = torch.from_numpy(s.ctx_lens.copy()).cuda()
    gam = torch.from_numpy(s.gammas).cuda()
    pt = torch.from_numpy(s.page_table).cuda()
    out = gu.rapid().rapid_verify_attn(gu.bf16_to_dev(inp.q), k, v, ctx, gammas=gam, page_table=pt,
                                       max_ctx=s.max_ctx, softmax_scale=cfg.softmax_scale)
    ref = oracle.verify_attn(inp.q, k_ref, v_ref, s.ctx_lens, lay, Hkv=cfg.n_kv_heads, scale=cfg.softmax_scale,
                             gammas=s.gammas, page_table=s.page_table)
    gu.assert_attn_close(gu.bf16_to_host(out), ref, "attention on the appended cache")
    acc = wl.gen_accept_inputs(cfg, seqs=s)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    n_acc, toks, _ = gu.rapid().rapid_accept(dev(acc.target_logits), dev(acc.draft_logits), dev(acc.draft_tokens),
                                             cfg.eta, dev(acc.uniforms), gammas=gam)
    gu.rapid().rapid_kv_commit(ctx, n_acc, gammas=gam)
    torch.cuda.synchronize()
    ref_acc = oracle.accept(acc.target_logits, acc.draft_logits, acc.draft_tokens, acc.uniforms, eta=cfg.eta,
                            temperature=cfg.temperature, tail_alpha=cfg.tail_alpha, gammas=s.gammas)
    res = gu.compare_accept((n_acc.cpu().numpy(), toks.cpu().numpy(), None), ref_acc, s.gammas, cfg.gamma_max)
    assert res["n_mismatch"] == 0 and res["token_mismatch"] == 0, res
    if res["exempt_sequences"] == 0:
        assert np.array_equal(ctx.cpu().numpy(), oracle.kv_commit(s.ctx_lens, ref_acc.n_accepted, gammas=s.gammas))
    assert np.array_equal(ctx.cpu().numpy(), oracle.kv_commit(s.ctx_lens, n_acc.cpu().numpy(), gammas=s.gammas))


def test_paged_commit_lists_released_pages():
    """rapid_kv_commit_pages against the oracle, bit for bit: lengths, released page ids, counts; several page
    sizes, per-sequence gammas, every accepted count."""
    rng = np.random.default_rng(5)
    for page in (16, 32, 128):
        B, gmax = 37, 10
        gam = rng.integers(0, gmax + 1, size=B).astype(np.int32)
        n = np.array([rng.integers(0, g + 1) for g in gam], dtype=np.int32)
        ctx = np.array([rng.integers(g + 1, 5000) for g in gam], dtype=np.int32)
        max_pages = -(-5000 // page) + 1
        table = np.stack([rng.permutation(4000)[:max_pages] for _ in range(B)]).astype(np.int32)
        cap = (gmax + 1 + page - 2) // page + 1
        want_len, want_rel, want_cnt = oracle.kv_commit_pages(ctx, n, table, page, cap, gammas=gam)
        lens = torch.from_numpy(ctx.copy()).cuda()
        rel, cnt = gu.rapid().rapid_kv_commit_pages(lens, torch.from_numpy(n).cuda(), torch.from_numpy(table).cuda(),
                                                    page_size=page, q_max=gmax + 1, max_ctx=5000,
                                                    gammas=torch.from_numpy(gam).cuda(), n_pages=4000)
        torch.cuda.synchronize()
        assert np.array_equal(lens.cpu().numpy(), want_len)
        assert np.array_equal(cnt.cpu().numpy(), want_cnt)
        assert np.array_equal(rel.cpu().numpy(), want_rel)
        assert want_cnt.max() >= 1                      # the case is exercised


def test_page_ids_outside_the_pool_are_clamped():
    """Page-table entries are device data: with the pool size stated in the shape, entries outside [0, n_pages)
    are clamped before they are used as addresses (the result then reads some valid page; it must not fault)."""
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], name="bad_pages", batch=2, ctx=(300, 900))
    inp = wl.gen_attn_inputs(cfg, layer=2)
    s = inp.seqs
    bad = s.page_table.copy()
    bad[0, 3] = 1 << 30
    bad[1, 0] = -5
    q, k, v = gu.bf16_to_dev(inp.q), gu.bf16_to_dev(inp.k), gu.bf16_to_dev(inp.v)
    out = gu.rapid().rapid_verify_attn(q, k, v, torch.from_numpy(s.ctx_lens).cuda(), gammas=torch.from_numpy(s.gammas).cuda(),
                                       page_table=torch.from_numpy(bad).cuda(), max_ctx=s.max_ctx)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
