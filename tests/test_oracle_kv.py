"""Pins of the oracle's cache bookkeeping (CPU only): numpy indexing on a plain [B, L, Hkv, d] array,
the paged = contiguous equivalence through the attention oracle, and a token-by-token simulation of
the index updates of Alg. 1 for the commit rule."""
import numpy as np
import pytest

import oracle


def rand_u16(rng, shape):
    return rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)


def test_append_matches_numpy_indexing_and_touches_nothing_else():
    rng = np.random.default_rng(0)
    B, L, Hkv, d, Qmax = 3, 40, 2, 8, 5
    k = rand_u16(rng, (B, L, Hkv, d)); v = rand_u16(rng, (B, L, Hkv, d))
    kn = rand_u16(rng, (B, Qmax, Hkv, d)); vn = rand_u16(rng, (B, Qmax, Hkv, d))
    ctx = np.array([40, 17, 5], dtype=np.int32)
    gam = np.array([4, 2, 0], dtype=np.int32)
    k_ref, v_ref = k.copy(), v.copy()
    for b in range(B):
        Q = gam[b] + 1
        k_ref[b, ctx[b] - Q:ctx[b]] = kn[b, :Q]
        v_ref[b, ctx[b] - Q:ctx[b]] = vn[b, :Q]
    oracle.kv_append(k, v, kn, vn, ctx, oracle.KVLayout(L * Hkv * d, Hkv * d, d), gammas=gam)
    assert np.array_equal(k, k_ref) and np.array_equal(v, v_ref)


def test_append_head_major_strides():
    rng = np.random.default_rng(1)
    B, L, Hkv, d, Q = 2, 12, 3, 4, 3
    k = rand_u16(rng, (B, Hkv, L, d)); v = rand_u16(rng, (B, Hkv, L, d))
    kn = rand_u16(rng, (B, Q, Hkv, d)); vn = rand_u16(rng, (B, Q, Hkv, d))
    ctx = np.array([12, 7], dtype=np.int32)
    k_ref, v_ref = k.copy(), v.copy()
    for b in range(B):
        k_ref[b, :, ctx[b] - Q:ctx[b]] = kn[b].transpose(1, 0, 2)
        v_ref[b, :, ctx[b] - Q:ctx[b]] = vn[b].transpose(1, 0, 2)
    oracle.kv_append(k, v, kn, vn, ctx, oracle.KVLayout(Hkv * L * d, d, L * d), gamma=Q - 1)
    assert np.array_equal(k, k_ref) and np.array_equal(v, v_ref)


def test_append_paged_lands_where_the_page_table_says():
    rng = np.random.default_rng(2)
    B, Hkv, d, Q, page, npages = 2, 2, 4, 4, 4, 9
    pool_k = rand_u16(rng, (npages, page, Hkv, d)); pool_v = rand_u16(rng, (npages, page, Hkv, d))
    kn = rand_u16(rng, (B, Q, Hkv, d)); vn = rand_u16(rng, (B, Q, Hkv, d))
    pt = np.array([[5, 2, 7, 0], [1, 8, 3, 4]], dtype=np.int32)
    ctx = np.array([14, 6], dtype=np.int32)            # both appends cross a page boundary
    k_ref, v_ref = pool_k.copy(), pool_v.copy()
    for b in range(B):
        for i in range(Q):
            t = ctx[b] - Q + i
            k_ref[pt[b, t // page], t % page] = kn[b, i]
            v_ref[pt[b, t // page], t % page] = vn[b, i]
    lay = oracle.KVLayout(0, Hkv * d, d, page, page * Hkv * d, pt.shape[1])
    oracle.kv_append(pool_k, pool_v, kn, vn, ctx, lay, gamma=Q - 1, page_table=pt)
    assert np.array_equal(pool_k, k_ref) and np.array_equal(pool_v, v_ref)


def test_commit_rule_against_token_by_token_simulation_of_alg1():
    """Simulate the sequence bookkeeping of Alg. 1 with explicit token lists: every accepted draft
    extends the sequence, then one token is drawn; the cache holds keys/values for every token except
    the newest one.  The closed form of the oracle must give the same cache length."""
    rng = np.random.default_rng(3)
    for _ in range(200):
        prefix = int(rng.integers(1, 50))               # tokens generated so far (cache holds prefix-1 of them)
        gamma = int(rng.integers(0, 9))
        n = int(rng.integers(0, gamma + 1))
        seq = list(range(prefix))
        cache = seq[:-1]                                 # the newest token has no K/V yet
        drafts = [100 + k for k in range(gamma)]
        # verification: the newest token and all drafts enter the cache
        cache_during = cache + [seq[-1]] + drafts
        ctx_during = len(cache_during)
        for k in range(n):                               # "x_j <- x'_j ; i <- j + 1"
            seq.append(drafts[k])
        seq.append(999)                                  # residual / bonus draw, "i <- i + 1"
        cache_after = seq[:-1]
        got = oracle.kv_commit(np.array([ctx_during]), np.array([n]), gamma=gamma)
        assert got[0] == len(cache_after)
        assert cache_during[:got[0]] == cache_after      # and what stays is a prefix of what was there


def test_commit_per_sequence_gammas_and_bad_input():
    out = oracle.kv_commit(np.array([100, 50, 9]), np.array([8, 0, 2]), gammas=np.array([8, 4, 2]))
    assert out.tolist() == [100, 46, 9]
    with pytest.raises(ValueError):
        oracle.kv_commit(np.array([100]), np.array([5]), gamma=4)


def test_paged_commit_releases_exactly_the_pages_nothing_kept_lives_in():
    """Pin of the page bookkeeping by explicit sets: simulate every token's page-table slot, collect the slots
    that hold a token before the commit and none after it; the oracle must list the page ids of exactly those
    slots, in slot order, and never a slot that still holds a kept token."""
    rng = np.random.default_rng(11)
    for _ in range(300):
        page = int(rng.choice([1, 2, 4, 16, 32]))
        gamma = int(rng.integers(0, 11))
        n = int(rng.integers(0, gamma + 1))
        l_old = int(rng.integers(gamma + 1, 200))
        max_pages = -(-200 // page) + 2
        table = rng.permutation(1000)[:max_pages].astype(np.int32)[None]
        cap = (gamma + 1 + page - 2) // page + 1
        new, rel, cnt = oracle.kv_commit_pages(np.array([l_old]), np.array([n]), table, page, cap, gamma=gamma)
        l_new = l_old - (gamma + 1) + (1 + n)
        assert new[0] == l_new
        slots_before = {t // page for t in range(l_old)}
        slots_after = {t // page for t in range(l_new)}
        want = sorted(slots_before - slots_after)
        assert rel[0, :cnt[0]].tolist() == [int(table[0, j]) for j in want]
        assert np.all(rel[0, cnt[0]:] == -1)
        assert cnt[0] <= cap


def test_paged_commit_hand_cases():
    table = np.arange(100, 120, dtype=np.int32)[None]          # slot j -> page 100 + j
    # 16-token pages, 40 tokens incl. 9 verification positions (tokens 31..39), 2 drafts accepted -> 34 tokens:
    # slots 0..2 were in use (tokens 0..39), slots 0..2 are still needed (tokens 32, 33 live in slot 2): nothing freed
    new, rel, cnt = oracle.kv_commit_pages(np.array([40]), np.array([2]), table, 16, 2, gamma=8)
    assert new.tolist() == [34] and cnt.tolist() == [0] and rel.tolist() == [[-1, -1]]
    # nothing accepted -> 32 tokens = exactly two pages: slot 2 is freed
    new, rel, cnt = oracle.kv_commit_pages(np.array([40]), np.array([0]), table, 16, 2, gamma=8)
    assert new.tolist() == [32] and cnt.tolist() == [1] and rel.tolist() == [[102, -1]]
    # 4-token pages: tokens 31..39 sit in slots 7, 8, 9; keep 32 -> slots 8 and 9 go
    new, rel, cnt = oracle.kv_commit_pages(np.array([40]), np.array([0]), table, 4, 4, gamma=8)
    assert cnt.tolist() == [2] and rel[0, :2].tolist() == [108, 109]
    # everything accepted: nothing to free
    new, rel, cnt = oracle.kv_commit_pages(np.array([40]), np.array([8]), table, 4, 4, gamma=8)
    assert new.tolist() == [40] and cnt.tolist() == [0]
