"""Pins of the oracle's output head and chunk statistics (CPU only).  None of them calls the
oracle to check itself: library matmul / logsumexp, closed forms and hand cases."""
import numpy as np
import pytest
from scipy.special import logsumexp

import oracle
from paper_2502_20330_amd import workloads as wl


def bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def widen(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def test_lm_head_equals_library_matmul_on_non_square_shapes():
    rng = np.random.default_rng(5)
    for rows, hidden, vocab in [(1, 64, 7), (3, 96, 50), (9, 256, 33), (16, 32, 129)]:
        h, w = bf16(rng.standard_normal((rows, hidden))), bf16(rng.standard_normal((vocab, hidden)))
        z = oracle.lm_head(h, w)
        ref = widen(h) @ widen(w).T
        assert z.shape == (rows, vocab)
        np.testing.assert_allclose(z, ref, rtol=1e-12, atol=1e-12)


def test_lm_head_one_hot_rows_pick_hidden_entries():
    """W row v = e_{pi(v)} -> z[r][v] = h[r][pi(v)] exactly (catches a transposed or mis-strided operand)."""
    rng = np.random.default_rng(6)
    rows, hidden, vocab = 4, 48, 20
    pi = rng.integers(0, hidden, size=vocab)
    w = np.zeros((vocab, hidden), dtype=np.float32)
    w[np.arange(vocab), pi] = 1.0
    h = bf16(rng.standard_normal((rows, hidden)))
    z = oracle.lm_head(h, bf16(w))
    assert np.array_equal(z, widen(h)[:, pi])


def test_lm_head_hand_case():
    h = bf16([[1.0, 2.0, -1.0], [0.5, 0.0, 4.0]])
    w = bf16([[1.0, 1.0, 1.0], [2.0, -1.0, 0.0], [0.0, 0.0, 0.25], [-3.0, 0.5, 1.0]])
    z = oracle.lm_head(h, w)
    assert np.array_equal(z, np.array([[2.0, 0.0, -0.25, -3.0], [4.5, 1.0, 1.0, 2.5]]))


def test_lm_head_is_linear_in_h():
    rng = np.random.default_rng(7)
    h1, h2 = bf16(rng.integers(-8, 8, (2, 40))), bf16(rng.integers(-8, 8, (2, 40)))      # exactly representable
    w = bf16(rng.integers(-4, 4, (11, 40)))
    hs = bf16(widen(h1) + widen(h2))
    assert np.array_equal(oracle.lm_head(hs, w), oracle.lm_head(h1, w) + oracle.lm_head(h2, w))


@pytest.mark.parametrize("T", [1.0, 0.1, 2.5])
def test_chunk_stats_against_library_logsumexp(T):
    rng = np.random.default_rng(8)
    z = rng.standard_normal((3, 1000)) * 4
    chunk = 128                                      # 7 full blocks and a short one
    cmax, csum = oracle.chunk_stats(z, chunk, T)
    assert cmax.shape == (3, 8)
    for c in range(8):
        blk = z[:, c * chunk:(c + 1) * chunk]
        np.testing.assert_array_equal(cmax[:, c], blk.max(axis=1))
        np.testing.assert_allclose(np.log(csum[:, c]) + cmax[:, c] / T, logsumexp(blk / T, axis=1), rtol=1e-12)
    # the blocks recombine to the row's log-normaliser of softmax(z/T)
    M = cmax.max(axis=1, keepdims=True)
    total = np.log((csum * np.exp((cmax - M) / T)).sum(axis=1)) + M[:, 0] / T
    np.testing.assert_allclose(total, logsumexp(z / T, axis=1), rtol=1e-12)


def test_chunk_stats_constant_row_closed_form():
    z = np.full((1, 10), 3.0)
    cmax, csum = oracle.chunk_stats(z, 4, 0.5)
    assert np.array_equal(cmax, [[3.0, 3.0, 3.0]]) and np.array_equal(csum, [[4.0, 4.0, 2.0]])
