"""Pins of the oracle's chunk selection (CPU only): library cosine / argsort, hand cases, ties."""
import numpy as np

import oracle
from paper_2502_20330_amd import workloads as wl


def test_similarity_equals_library_cosine_and_selection_equals_argsort():
    emb, q = wl.gen_retrieval_inputs(200)
    sim, sel, margin = oracle.retrieve(emb, q, 10, 0.3)
    e64, q64 = emb.astype(np.float64), q.astype(np.float64)
    ref = (e64 @ q64) / (np.linalg.norm(e64, axis=1) * np.linalg.norm(q64))
    np.testing.assert_allclose(sim, ref, rtol=1e-12, atol=1e-14)
    order = np.argsort(-ref, kind="stable")[:10]
    expect = np.sort(order[ref[order] >= 0.3])
    assert np.array_equal(sel, expect)
    assert 0 < len(sel) <= 10 and margin > 0
    assert np.all(np.diff(sel) > 0)                     # document order


def test_hand_case_threshold_and_top_k():
    q = np.array([1.0, 0.0], dtype=np.float32)
    emb = np.array([[1, 0], [0, 1], [1, 1], [-1, 0], [3, 4], [2, 0]], dtype=np.float32)
    # cosines: 1, 0, 0.7071, -1, 0.6, 1
    sim, sel, _ = oracle.retrieve(emb, q, 3, 0.3)
    np.testing.assert_allclose(sim, [1, 0, 2 ** -0.5, -1, 0.6, 1], rtol=1e-12)
    assert sel.tolist() == [0, 2, 5]                    # top 3: chunks 0, 5 (tie, both in), 2
    _, sel, _ = oracle.retrieve(emb, q, 5, 0.65)
    assert sel.tolist() == [0, 2, 5]                    # 0.6 and below are filtered although k allows them
    _, sel, _ = oracle.retrieve(emb, q, 1, 0.3)
    assert sel.tolist() == [0]                          # equal similarities: the lower index wins
    _, sel, _ = oracle.retrieve(emb, q, 6, -2.0)
    assert sel.tolist() == [0, 1, 2, 3, 4, 5]
    _, sel, _ = oracle.retrieve(emb, q, 4, 2.0)
    assert sel.tolist() == []


def test_margin_is_the_smallest_distance_to_a_decision_boundary():
    """Same hand case (cosines 1, 0, 0.7071, -1, 0.6, 1).  The margin is the smaller of (a) the gap between
    the k-th and the (k+1)-th similarity in rank order and (b) the smallest |similarity - threshold|."""
    q = np.array([1.0, 0.0], dtype=np.float32)
    emb = np.array([[1, 0], [0, 1], [1, 1], [-1, 0], [3, 4], [2, 0]], dtype=np.float32)
    r2 = 2 ** -0.5
    # k = 3: ranks 1, 1, .7071 | .6 -> gap .1071; nearest similarity to the threshold 0.3 is 0 or 0.6 (0.3 away)
    assert abs(oracle.retrieve(emb, q, 3, 0.3)[2] - (r2 - 0.6)) < 1e-12
    # k = 2: the k-th and (k+1)-th values are 1 (chunk 5) and .7071 -> gap .2929 < .3
    assert abs(oracle.retrieve(emb, q, 2, 0.3)[2] - (1.0 - r2)) < 1e-12
    # k = 1: the two best are equal -> gap 0
    assert oracle.retrieve(emb, q, 1, 0.3)[2] == 0.0
    # threshold close to a similarity decides: |0.6 - 0.58| = 0.02 < every rank gap
    assert abs(oracle.retrieve(emb, q, 3, 0.58)[2] - (0.6 - 0.58)) < 1e-9
    # k = n: no rank boundary, only the threshold counts: nearest is 0.7071 - 0.65
    assert abs(oracle.retrieve(emb, q, 6, 0.65)[2] - (0.65 - 0.6)) < 1e-9


def test_scaling_a_chunk_does_not_change_its_similarity_and_zero_vectors_score_zero():
    emb, q = wl.gen_retrieval_inputs(50, dim=64)
    a, _, _ = oracle.retrieve(emb, q, 5, 0.3)
    emb2 = emb.copy()
    emb2[7] *= 8.0                                       # exact in binary floating point
    emb2[9] = 0.0
    b, _, _ = oracle.retrieve(emb2, 4.0 * q, 5, 0.3)
    assert abs(a[7] - b[7]) < 1e-15 and b[9] == 0.0
    np.testing.assert_allclose(np.delete(a, [9]), np.delete(b, [9]), rtol=1e-12)


def test_budget_rule():
    assert oracle.retrieval_top_k(131072) == 10             # 1/24 of 128K = 5461 tokens -> 10 whole chunks
    assert oracle.retrieval_top_k(32768) == 8               # floor of 4096 tokens
    assert oracle.retrieval_top_k(1 << 20) == 85
