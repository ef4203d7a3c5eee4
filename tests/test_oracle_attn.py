"""Pins for the float64 attention oracle: it is checked against things that are
not itself -- a dense masked-softmax written with torch library ops, closed
forms, and invariants of causal GQA attention."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2502_20330_amd import workloads as wl


def rand_bits(rng, shape, scale=1.0):
    return wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32) * np.float32(scale))


def contiguous_layout(Lmax, Hkv, d):
    return oracle.KVLayout(batch_stride=Lmax * Hkv * d, token_stride=Hkv * d, head_stride=d)


def dense_reference(q, k, v, ctx_lens, gammas, Hkv, scale):
    """[R x L] score matrix, -inf mask, torch.softmax, matmul; float64."""
    qf = torch.from_numpy(wl.bf16_bits_to_f32(q)).double()
    kf = torch.from_numpy(wl.bf16_bits_to_f32(k)).double()
    vf = torch.from_numpy(wl.bf16_bits_to_f32(v)).double()
    B, Qmax, Hq, d = qf.shape
    G = Hq // Hkv
    out = torch.zeros(B, Qmax, Hq, d, dtype=torch.float64)
    lse = torch.zeros(B, Hq, Qmax, dtype=torch.float64)
    for b in range(B):
        L, Q = int(ctx_lens[b]), int(gammas[b]) + 1
        for h in range(Hq):
            K = kf[b, :L, h // G]                      # [L, d]
            Vv = vf[b, :L, h // G]
            S = scale * qf[b, :Q, h] @ K.T             # [Q, L]
            pos = torch.arange(L)[None, :]
            lim = (L - Q + torch.arange(Q))[:, None]
            S = S.masked_fill(pos > lim, float("-inf"))
            out[b, :Q, h] = torch.softmax(S, dim=-1) @ Vv
            lse[b, h, :Q] = torch.logsumexp(S, dim=-1)
    return out.numpy(), lse.numpy()


@pytest.mark.parametrize("B,Hq,Hkv,d,Lmax,gam", [
    (1, 4, 1, 8, 17, [3]),
    (2, 4, 2, 64, 64, [4, 2]),
    (3, 6, 3, 16, 33, [0, 5, 1]),
])
def test_matches_dense_torch(B, Hq, Hkv, d, Lmax, gam):
    rng = np.random.default_rng(11)
    Qmax = max(gam) + 1
    q = rand_bits(rng, (B, Qmax, Hq, d))
    k = rand_bits(rng, (B, Lmax, Hkv, d))
    v = rand_bits(rng, (B, Lmax, Hkv, d))
    ctx = np.array([Lmax - 3 * b for b in range(B)], dtype=np.int32)
    gammas = np.array(gam, dtype=np.int32)
    scale = 1.0 / math.sqrt(d)
    out, lse = oracle.verify_attn(q, k, v, ctx, contiguous_layout(Lmax, Hkv, d), Hkv=Hkv,
                                  scale=scale, gammas=gammas, want_lse=True)
    ref, ref_lse = dense_reference(q, k, v, ctx, gammas, Hkv, scale)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12, atol=1e-13)
    # padded query rows are zero
    for b in range(B):
        assert np.all(out[b, gam[b] + 1:] == 0.0)


def test_identical_keys_give_mean_of_visible_values():
    rng = np.random.default_rng(3)
    B, Hq, Hkv, d, L, g = 1, 2, 1, 16, 40, 3
    q = rand_bits(rng, (B, g + 1, Hq, d))
    krow = rand_bits(rng, (1, 1, Hkv, d))
    k = np.broadcast_to(krow, (B, L, Hkv, d)).copy()
    v = rand_bits(rng, (B, L, Hkv, d))
    out = oracle.verify_attn(q, k, v, [L], contiguous_layout(L, Hkv, d), Hkv=Hkv, scale=0.3)
    vf = wl.bf16_bits_to_f32(v).astype(np.float64)
    for i in range(g + 1):
        nvis = L - (g + 1) + i + 1
        want = vf[0, :nvis, 0].mean(axis=0)
        for h in range(Hq):
            np.testing.assert_allclose(out[0, i, h], want, rtol=1e-13, atol=1e-15)


def test_constant_values_pass_through():
    rng = np.random.default_rng(4)
    B, Hq, Hkv, d, L, g = 1, 4, 2, 8, 25, 2
    q = rand_bits(rng, (B, g + 1, Hq, d))
    k = rand_bits(rng, (B, L, Hkv, d))
    vrow = rand_bits(rng, (1, 1, Hkv, d))
    v = np.broadcast_to(vrow, (B, L, Hkv, d)).copy()
    out = oracle.verify_attn(q, k, v, [L], contiguous_layout(L, Hkv, d), Hkv=Hkv, scale=0.5)
    vf = wl.bf16_bits_to_f32(vrow).astype(np.float64)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, :, h], np.broadcast_to(vf[0, 0, h // 2], (g + 1, d)),
                                   rtol=1e-14)


def test_dominant_key_selects_its_value():
    rng = np.random.default_rng(5)
    d, L, g = 8, 50, 1
    q = wl.f32_to_bf16_bits(np.full((1, g + 1, 1, d), 4.0, dtype=np.float32))
    k = rand_bits(rng, (1, L, 1, d), 0.01)
    k[0, 7, 0] = wl.f32_to_bf16_bits(np.full(d, 8.0, dtype=np.float32))   # score 256*scale
    v = rand_bits(rng, (1, L, 1, d))
    out = oracle.verify_attn(q, k, v, [L], contiguous_layout(L, 1, d), Hkv=1, scale=1.0)
    want = wl.bf16_bits_to_f32(v)[0, 7, 0].astype(np.float64)
    np.testing.assert_allclose(out[0, 0, 0], want, atol=1e-60)
    np.testing.assert_allclose(out[0, 1, 0], want, atol=1e-60)


def test_no_context_row0_is_first_value_and_rows_are_prefix_softmax():
    rng = np.random.default_rng(6)
    d, g = 16, 4
    L = g + 1
    q = rand_bits(rng, (1, L, 1, d))
    k = rand_bits(rng, (1, L, 1, d))
    v = rand_bits(rng, (1, L, 1, d))
    scale = 0.25
    out = oracle.verify_attn(q, k, v, [L], contiguous_layout(L, 1, d), Hkv=1, scale=scale)
    qf, kf, vf = (wl.bf16_bits_to_f32(a).astype(np.float64) for a in (q, k, v))
    np.testing.assert_array_equal(out[0, 0, 0], vf[0, 0, 0])
    for i in range(L):
        s = scale * kf[0, : i + 1, 0] @ qf[0, i, 0]
        w = np.exp(s - s.max())
        w /= w.sum()
        np.testing.assert_allclose(out[0, i, 0], w @ vf[0, : i + 1, 0], rtol=1e-13, atol=1e-15)


def test_causality_later_verify_positions_do_not_leak():
    rng = np.random.default_rng(7)
    Hq, Hkv, d, L, g = 2, 1, 8, 30, 4
    q = rand_bits(rng, (1, g + 1, Hq, d))
    k = rand_bits(rng, (1, L, Hkv, d))
    v = rand_bits(rng, (1, L, Hkv, d))
    lay = contiguous_layout(L, Hkv, d)
    base = oracle.verify_attn(q, k, v, [L], lay, Hkv=Hkv, scale=0.4)
    j = 3                                  # verify position 3 = cache row L-Q+3
    k2, v2 = k.copy(), v.copy()
    k2[0, L - (g + 1) + j] = rand_bits(rng, (Hkv, d))
    v2[0, L - (g + 1) + j] = rand_bits(rng, (Hkv, d))
    pert = oracle.verify_attn(q, k2, v2, [L], lay, Hkv=Hkv, scale=0.4)
    assert np.array_equal(base[0, :j], pert[0, :j])          # bit-identical
    assert not np.array_equal(base[0, j:], pert[0, j:])


def test_rows_beyond_ctx_len_are_ignored():
    rng = np.random.default_rng(8)
    Hq, Hkv, d, Lmax, L, g = 2, 2, 8, 40, 29, 2
    q = rand_bits(rng, (1, g + 1, Hq, d))
    k = rand_bits(rng, (1, Lmax, Hkv, d))
    v = rand_bits(rng, (1, Lmax, Hkv, d))
    lay = contiguous_layout(Lmax, Hkv, d)
    a = oracle.verify_attn(q, k, v, [L], lay, Hkv=Hkv, scale=0.4)
    k[0, L:] = 0x7FC0
    v[0, L:] = 0x7FC0                      # NaN bits in the unused tail
    b = oracle.verify_attn(q, k, v, [L], lay, Hkv=Hkv, scale=0.4)
    assert np.array_equal(a, b)


def test_permuting_context_keys_changes_nothing_but_rounding():
    rng = np.random.default_rng(9)
    Hq, Hkv, d, L, g = 4, 2, 16, 48, 3
    q = rand_bits(rng, (1, g + 1, Hq, d))
    k = rand_bits(rng, (1, L, Hkv, d))
    v = rand_bits(rng, (1, L, Hkv, d))
    lay = contiguous_layout(L, Hkv, d)
    a = oracle.verify_attn(q, k, v, [L], lay, Hkv=Hkv, scale=0.3)
    nctx = L - (g + 1)
    perm = np.concatenate([rng.permutation(nctx), np.arange(nctx, L)])
    b = oracle.verify_attn(q, k[:, perm], v[:, perm], [L], lay, Hkv=Hkv, scale=0.3)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_split_merge_formula_reproduces_whole():
    """out = sum_s e^{lse_s - lse} out_s: merging oracle results of disjoint
    key ranges with their log-sum-exps gives the oracle result of the union."""
    rng = np.random.default_rng(10)
    d, L = 16, 60
    q = rand_bits(rng, (1, 1, 1, d))
    k = rand_bits(rng, (1, L, 1, d))
    v = rand_bits(rng, (1, L, 1, d))
    whole, lse = oracle.verify_attn(q, k, v, [L], contiguous_layout(L, 1, d), Hkv=1, scale=0.5,
                                    gamma=0, want_lse=True)
    parts = []
    for lo, hi in [(0, 13), (13, 41), (41, 60)]:
        kk, vv = k[:, lo:hi].copy(), v[:, lo:hi].copy()
        o, l = oracle.verify_attn(q, kk, vv, [hi - lo], contiguous_layout(hi - lo, 1, d), Hkv=1,
                                  scale=0.5, gamma=0, want_lse=True)
        parts.append((o[0, 0, 0], l[0, 0, 0]))
    m = max(l for _, l in parts)
    num = sum(np.exp(l - m) * o for o, l in parts)
    den = sum(np.exp(l - m) for _, l in parts)
    np.testing.assert_allclose(whole[0, 0, 0], num / den, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse[0, 0, 0], m + np.log(den), rtol=1e-13)


def test_gqa_heads_of_a_group_share_kv_and_groups_do_not():
    rng = np.random.default_rng(12)
    Hq, Hkv, d, L, g = 4, 2, 8, 20, 1
    qrow = rand_bits(rng, (1, g + 1, 1, d))
    q = np.broadcast_to(qrow, (1, g + 1, Hq, d)).copy()
    k = rand_bits(rng, (1, L, Hkv, d))
    v = rand_bits(rng, (1, L, Hkv, d))
    out = oracle.verify_attn(q, k, v, [L], contiguous_layout(L, Hkv, d), Hkv=Hkv, scale=0.5)
    assert np.array_equal(out[0, :, 0], out[0, :, 1])
    assert np.array_equal(out[0, :, 2], out[0, :, 3])
    assert not np.array_equal(out[0, :, 1], out[0, :, 2])


def test_paged_cache_equals_contiguous():
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=3, n_q_heads=4, n_kv_heads=2, head_dim=16,
                    ctx=(20, 70), gamma_choices=(1, 2, 3), vocab=32)
    inp = wl.gen_attn_inputs(cfg)
    s = inp.seqs
    bs, ts, hs, ps = wl.kv_strides(cfg, s)
    lay = oracle.KVLayout(bs, ts, hs, cfg.page_size, ps, s.page_table.shape[1])
    paged = oracle.verify_attn(inp.q, inp.k, inp.v, s.ctx_lens, lay, Hkv=cfg.n_kv_heads, scale=0.25,
                               gammas=s.gammas, page_table=s.page_table)
    # gather pages into a contiguous cache by hand
    Lmax = s.max_ctx
    kc = np.zeros((cfg.batch, Lmax, cfg.n_kv_heads, cfg.head_dim), dtype=np.uint16)
    vc = np.zeros_like(kc)
    for b in range(cfg.batch):
        for j in range(s.ctx_lens[b]):
            pg = s.page_table[b, j // cfg.page_size]
            kc[b, j] = inp.k[pg, j % cfg.page_size]
            vc[b, j] = inp.v[pg, j % cfg.page_size]
    cont = oracle.verify_attn(inp.q, kc, vc, s.ctx_lens, contiguous_layout(Lmax, cfg.n_kv_heads, cfg.head_dim),
                              Hkv=cfg.n_kv_heads, scale=0.25, gammas=s.gammas)
    assert np.array_equal(paged, cont)


def test_scale_is_applied_to_scores():
    """Doubling the scale equals doubling q (exact in bf16)."""
    rng = np.random.default_rng(13)
    d, L = 8, 12
    q = rand_bits(rng, (1, 2, 1, d))
    k = rand_bits(rng, (1, L, 1, d))
    v = rand_bits(rng, (1, L, 1, d))
    q2 = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(q) * np.float32(2.0))
    lay = contiguous_layout(L, 1, d)
    a = oracle.verify_attn(q, k, v, [L], lay, Hkv=1, scale=0.5)
    b = oracle.verify_attn(q2, k, v, [L], lay, Hkv=1, scale=0.25)
    np.testing.assert_allclose(a, b, rtol=1e-14)


def test_invalid_arguments_are_rejected():
    rng = np.random.default_rng(14)
    q = rand_bits(rng, (1, 3, 2, 8))
    k = rand_bits(rng, (1, 10, 1, 8))
    with pytest.raises(ValueError):
        oracle.verify_attn(q, k, k, [2], contiguous_layout(10, 1, 8), Hkv=1, scale=1.0)  # ctx < gamma+1
