"""Pins for the float64 accept/resample oracle (Alg. 1 validation loop).

None of these call the oracle to check itself: they use a separately written
textbook speculative sampler (eta = 0), library softmax / finite differences
(Eq. new_target, Eq. delta, Proposition 1), the analytically derived output
law (Appendix B's bookkeeping with the clamp of Alg. 1's residual), hand-worked
inverse-CDF cases and degenerate inputs."""
import json
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax
from scipy.stats import chisquare

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- helpers
def np_distributions(z, zq, eta, T, alpha):
    """Eq. new_target + tail rule with library softmax (independent of the C code)."""
    p = sp_softmax(np.asarray(z, dtype=np.float64) / T)
    q = sp_softmax(np.asarray(zq, dtype=np.float64) / T)
    ph = sp_softmax(np.asarray(z, dtype=np.float64) / T + eta * (q - p))
    tail = ph < alpha * ph.max()
    ph = np.where(tail, p, ph)
    return p, q, ph


def output_law(p, q, ph):
    """Law of the token emitted at one position: accepted with probability
    min(q, ph) per token, otherwise drawn from norm(max(p-ph, p-q, 0))."""
    acc = np.minimum(q, ph)
    beta = acc.sum()
    w = np.maximum(np.maximum(p - ph, p - q), 0.0)
    if w.sum() <= 0:
        w = p
    return acc + (1.0 - beta) * w / w.sum(), beta


def sample_tokens(rng, q, n):
    return rng.choice(len(q), size=n, p=q).astype(np.int32)


def textbook_sd(z, zq, tokens, uniforms, T):
    """Sec. 2.1, Eq. 1-2, written directly: accept iff r <= min(1, p/q), on the
    first reject draw from norm(max(p-q, 0)), all accepted -> draw from p."""
    g = len(tokens)
    out = []
    for k in range(g):
        p = sp_softmax(z[k].astype(np.float64) / T)
        q = sp_softmax(zq[k].astype(np.float64) / T)
        x = tokens[k]
        if float(uniforms[k]) <= min(1.0, p[x] / q[x]):
            out.append(int(x))
            continue
        w = np.maximum(p - q, 0.0)
        return k, out + [cdf_pick(w, float(uniforms[g]))]
    p = sp_softmax(z[g].astype(np.float64) / T)
    return g, out + [cdf_pick(p, float(uniforms[g]))]


def cdf_pick(w, u):
    c = np.cumsum(w)               # index order, like the oracle
    t = u * c[-1]
    return int(np.searchsorted(c, t, side="right"))


# ---------------------------------------------------------------- Eq. new_target / delta
@pytest.mark.parametrize("T,eta", [(1.0, 0.5), (0.1, 5.0), (2.0, 20.0), (0.1, 50.0)])
def test_distributions_match_library_softmax_forms(T, eta):
    rng = np.random.default_rng(0)
    V = 50
    z, zq = rng.normal(0, 3, V), rng.normal(0, 3, V)
    p, q, ph = oracle.distributions(z, zq, eta=eta, temperature=T, tail_alpha=0.0)
    # form 1 (Eq. new_target): softmax(z/T + eta (q - p)); form 2 (Eq. delta): softmax(zh/T)
    rp, rq = sp_softmax(z / T), sp_softmax(zq / T)
    form1 = sp_softmax(z / T + eta * (rq - rp))
    form2 = sp_softmax((z + eta * T * (rq - rp)) / T)
    np.testing.assert_allclose(p, rp, rtol=1e-12)
    np.testing.assert_allclose(q, rq, rtol=1e-12)
    np.testing.assert_allclose(ph, form1, rtol=1e-11, atol=1e-300)
    np.testing.assert_allclose(form1, form2, rtol=1e-11, atol=1e-300)
    assert abs(ph.sum() - 1.0) < 1e-12                 # tail_alpha = 0: still a distribution
    assert np.all(np.isfinite(ph))


def test_proposition1_gradient_and_one_step():
    """d/dz [T^2 KL(q || softmax(z/T))] = T (p - q) by central differences, and
    one descent step of size eta on z reproduces the oracle's p_hat."""
    rng = np.random.default_rng(1)
    V, T, eta = 12, 0.7, 3.0
    z, zq = rng.normal(0, 2, V), rng.normal(0, 2, V)
    q = sp_softmax(zq / T)

    def loss(zz):
        pp = sp_softmax(zz / T)
        return T * T * np.sum(q * (np.log(q) - np.log(pp)))

    h = 1e-6
    grad = np.array([(loss(z + h * np.eye(V)[i]) - loss(z - h * np.eye(V)[i])) / (2 * h) for i in range(V)])
    p, q_o, ph = oracle.distributions(z, zq, eta=eta, temperature=T, tail_alpha=0.0)
    np.testing.assert_allclose(grad, T * (p - q_o), atol=1e-8)
    np.testing.assert_allclose(ph, sp_softmax((z - eta * grad) / T), atol=1e-7)
    # the shift moves mass toward the drafter: KL(q || p_hat) < KL(q || p)
    assert np.sum(q * np.log(q / ph)) < np.sum(q * np.log(q / p))


def test_tail_rule_replaces_only_entries_below_a_tenth_of_the_max():
    z = np.array([3.0, 2.5, 0.0, -1.0, -4.0])
    zq = np.array([0.0, 3.0, 2.0, -1.0, -2.0])
    eta, T = 2.0, 1.0
    p, q, raw = oracle.distributions(z, zq, eta=eta, temperature=T, tail_alpha=0.0)
    _, _, ph = oracle.distributions(z, zq, eta=eta, temperature=T, tail_alpha=0.1)
    tail = raw < 0.1 * raw.max()
    assert tail.any() and not tail.all()
    np.testing.assert_array_equal(ph[tail], p[tail])
    np.testing.assert_array_equal(ph[~tail], raw[~tail])
    rp, rq, rph = np_distributions(z, zq, eta, T, 0.1)
    np.testing.assert_allclose(ph, rph, rtol=1e-12)
    assert abs(ph.sum() - 1.0) > 1e-6                  # not renormalised


def test_eta_zero_makes_phat_equal_p():
    rng = np.random.default_rng(2)
    z, zq = rng.normal(0, 3, 33), rng.normal(0, 3, 33)
    p, q, ph = oracle.distributions(z, zq, eta=0.0, temperature=0.5, tail_alpha=0.1)
    np.testing.assert_array_equal(ph, p)


def test_phat_stays_near_p_for_moderate_eta():
    rng = np.random.default_rng(3)
    z, zq = rng.normal(0, 4, 1000), rng.normal(0, 4, 1000)
    prev = 0.0
    for eta in (0.1, 1.0, 5.0):
        p, q, ph = oracle.distributions(z, zq, eta=eta, tail_alpha=0.0)
        l1 = np.abs(ph - p).sum()
        assert prev <= l1 <= 2.0 * (np.exp(eta) - 1.0)   # |zh - z| <= eta elementwise
        prev = l1


# ---------------------------------------------------------------- inverse CDF convention
def test_inverse_cdf_hand_cases():
    # one sequence, gamma = 0: the only token is a draw from p = softmax(z)
    z = np.log(np.array([0.1, 0.2, 0.3, 0.4]))[None, None, :].astype(np.float32)
    zd = np.zeros((1, 0, 4), dtype=np.float32)
    edges = [(0.0, 0), (0.05, 0), (0.15, 1), (0.29, 1), (0.31, 2), (0.59, 2), (0.61, 3), (0.999, 3)]
    for u, want in edges:
        r = oracle.accept(z, zd, np.zeros((1, 0), np.int32), np.array([[u]], np.float32), eta=0.0)
        assert r.n_accepted[0] == 0 and r.out_tokens[0, 0] == want, (u, r.out_tokens)
    # a zero-weight token is never drawn, not even by u = 0 (strict > on the running sum)
    z0 = np.array([[[-np.inf, 0.0, 0.0]]], dtype=np.float32)
    r = oracle.accept(z0, np.zeros((1, 0, 3), np.float32), np.zeros((1, 0), np.int32),
                      np.array([[0.0]], np.float32), eta=0.0)
    assert r.out_tokens[0, 0] == 1


# ---------------------------------------------------------------- eta = 0: textbook SD
def test_eta_zero_equals_textbook_speculative_sampling():
    rng = np.random.default_rng(4)
    B, g, V, T = 400, 3, 11, 0.8
    zt = rng.normal(0, 2, (B, g + 1, V)).astype(np.float32)
    zd = (zt[:, :g] + rng.normal(0, 1.5, (B, g, V))).astype(np.float32)
    tok = np.stack([[sample_tokens(rng, sp_softmax(zd[b, k].astype(np.float64) / T), 1)[0]
                     for k in range(g)] for b in range(B)]).astype(np.int32)
    u = rng.random((B, g + 1)).astype(np.float32)
    r = oracle.accept(zt, zd, tok, u, eta=0.0, temperature=T)
    ns = []
    for b in range(B):
        n, toks = textbook_sd(zt[b], zd[b], tok[b], u[b], T)
        ns.append(n)
        assert r.n_accepted[b] == n
        assert list(r.out_tokens[b, : n + 1]) == toks
        assert np.all(r.out_tokens[b, n + 1:] == -1)
    assert 0 < np.mean(ns) < g                        # both branches exercised


def test_identical_logits_accept_everything_and_bonus_follows_p():
    rng = np.random.default_rng(5)
    B, g, V = 20000, 2, 6
    z1 = rng.normal(0, 1.5, (g + 1, V)).astype(np.float32)
    zt = np.broadcast_to(z1, (B, g + 1, V)).copy()
    zd = zt[:, :g].copy()
    tok = rng.integers(0, V, (B, g)).astype(np.int32)   # any token: ratio is 1
    u = rng.random((B, g + 1)).astype(np.float32)
    for eta in (0.0, 7.0):
        r = oracle.accept(zt, zd, tok, u, eta=eta)
        assert np.all(r.n_accepted == g)
        np.testing.assert_array_equal(r.out_tokens[:, :g], tok)
        np.testing.assert_allclose(r.ratio, 1.0, rtol=1e-12)
        counts = np.bincount(r.out_tokens[:, g], minlength=V)
        pg = sp_softmax(z1[g].astype(np.float64))
        assert chisquare(counts, pg * B).pvalue > 1e-4


def test_one_hot_drafter_on_targets_argmax_is_always_accepted_for_large_eta():
    rng = np.random.default_rng(6)
    V = 64
    z = rng.normal(0, 1, (1, 2, V)).astype(np.float32)
    x = int(np.argmax(z[0, 0]))
    zq = np.zeros((1, 1, V), np.float32)
    zq[0, 0, x] = 100.0
    for u0 in (0.0, 0.5, 0.99):
        r = oracle.accept(z, zq, np.array([[x]], np.int32), np.array([[u0, 0.3]], np.float32), eta=50.0)
        assert r.n_accepted[0] == 1 and r.out_tokens[0, 0] == x
        assert r.ratio[0, 0] > 0.99


# ---------------------------------------------------------------- output law
def run_trials(z, zq, eta, T, alpha, B, seed):
    """B independent one-position trials on fixed logits; returns the emitted first token."""
    rng = np.random.default_rng(seed)
    V = len(z)
    zt = np.broadcast_to(np.stack([z, z]).astype(np.float32), (B, 2, V)).copy()
    zd = np.broadcast_to(np.asarray(zq, np.float32)[None, None, :], (B, 1, V)).copy()
    q = sp_softmax(np.asarray(zq, np.float32).astype(np.float64) / T)
    tok = sample_tokens(rng, q, B)[:, None]
    u = rng.random((B, 2)).astype(np.float32)
    r = oracle.accept(zt, zd, tok, u, eta=eta, temperature=T, tail_alpha=alpha)
    return r, tok


def test_eta_zero_reproduces_the_target_distribution_chi_square():
    """The guarantee of Sec. 2.1: with eta = 0 the emitted token follows p exactly."""
    z = np.array([2.0, 1.0, 0.0, -1.0, 0.5, -0.3, 1.2, -2.0])
    zq = np.array([0.0, 2.0, 1.0, -1.0, -0.5, 0.8, 0.1, 0.4])
    B = 1_000_000
    r, _ = run_trials(z, zq, 0.0, 1.0, 0.1, B, seed=7)
    counts = np.bincount(r.out_tokens[:, 0], minlength=len(z))
    p = sp_softmax(z.astype(np.float32).astype(np.float64))
    assert chisquare(counts, p * B).pvalue > 1e-4
    # and the acceptance rate is sum(min(p, q))
    q = sp_softmax(zq.astype(np.float32).astype(np.float64))
    assert abs(r.n_accepted.mean() - np.minimum(p, q).sum()) < 4 * 0.5 / np.sqrt(B)


@pytest.mark.parametrize("eta,T,alpha", [(2.0, 1.0, 0.1), (5.0, 0.5, 0.1), (1.0, 1.0, 0.0), (20.0, 1.0, 0.1)])
def test_general_eta_follows_the_derived_law_chi_square(eta, T, alpha):
    """For eta > 0 the emitted token follows min(q, ph) + (1-beta) w / W (Appendix B's
    accounting with the residual clamped at 0 as in Alg. 1), which is NOT p in general."""
    z = np.array([2.0, 1.0, 0.0, -1.0, 0.5, -0.3, 1.2, -2.0])
    zq = np.array([0.0, 2.0, 1.0, -1.0, -0.5, 0.8, 0.1, 0.4])
    B = 1_000_000
    r, _ = run_trials(z, zq, eta, T, alpha, B, seed=8)
    p, q, ph = np_distributions(z.astype(np.float32), zq.astype(np.float32), eta, T, alpha)
    law, beta = output_law(p, q, ph)
    counts = np.bincount(r.out_tokens[:, 0], minlength=len(z))
    keep = law > 0
    assert counts[~keep].sum() == 0
    assert chisquare(counts[keep], law[keep] / law[keep].sum() * B).pvalue > 1e-4
    assert abs(r.n_accepted.mean() - beta) < 4 * 0.5 / np.sqrt(B)
    if eta >= 2.0 and alpha > 0:
        # the law differs from p by far more than sampling noise: a sampler that
        # "fixed" the residual to hit p would fail the chi-square above
        assert np.abs(law - p).max() > 0.05


def test_where_p_dominates_min_q_phat_the_law_is_p():
    """Appendix B's argument is valid when p >= min(q, ph) everywhere; then the
    emitted token follows p also for eta > 0."""
    z = np.array([1.0, 0.5, 0.0, -0.5])
    zq = z.copy()
    zq[0] += 0.02                                      # nearly identical drafter
    p, q, ph = np_distributions(z, zq, 1.0, 1.0, 0.0)
    law, _ = output_law(p, q, ph)
    if np.all(p >= np.minimum(q, ph) - 1e-15):
        np.testing.assert_allclose(law, p, atol=1e-12)
    # eta = 0 always satisfies it
    p, q, ph = np_distributions(z, np.array([0.0, 2.0, 1.0, -1.0]), 0.0, 1.0, 0.1)
    law, _ = output_law(p, q, ph)
    np.testing.assert_allclose(law, p, atol=1e-12)


def test_law_by_quadrature_over_the_two_uniforms():
    """Deterministic version of the chi-square: integrate the oracle's output over a
    midpoint grid of (r, u_draw) for every draft token, weight by q."""
    z = np.array([1.0, 0.2, -0.7], dtype=np.float32)
    zq = np.array([-0.5, 1.1, 0.3], dtype=np.float32)
    eta, n = 1.5, 256
    p, q, ph = np_distributions(z, zq, eta, 1.0, 0.1)
    law, _ = output_law(p, q, ph)
    grid = ((np.arange(n) + 0.5) / n).astype(np.float32)
    ua, ud = np.meshgrid(grid, grid, indexing="ij")
    u = np.stack([ua.ravel(), ud.ravel()], axis=1)
    est = np.zeros(3)
    for x in range(3):
        B = u.shape[0]
        zt = np.broadcast_to(np.stack([z, z]), (B, 2, 3)).copy()
        zd = np.broadcast_to(zq[None, None], (B, 1, 3)).copy()
        r = oracle.accept(zt, zd, np.full((B, 1), x, np.int32), u, eta=eta)
        est += q[x] * np.bincount(r.out_tokens[:, 0], minlength=3) / B
    np.testing.assert_allclose(est, law, atol=2.5 / n)


def test_multi_position_stop_law():
    """gamma = 3: P(n = k) = prod_{j<k} beta_j (1 - beta_k); the token at the stop
    position follows w_k / W_k; after 3 accepts the bonus follows p_3."""
    rng = np.random.default_rng(9)
    g, V, B, eta = 3, 5, 400_000, 1.0
    z = rng.normal(0, 1.5, (g + 1, V)).astype(np.float32)
    zq = (z[:g] + rng.normal(0, 1.0, (g, V))).astype(np.float32)
    zt = np.broadcast_to(z, (B, g + 1, V)).copy()
    zd = np.broadcast_to(zq, (B, g, V)).copy()
    dists = [np_distributions(z[k], zq[k], eta, 1.0, 0.1) for k in range(g)]
    tok = np.stack([sample_tokens(rng, dists[k][1], B) for k in range(g)], axis=1)
    u = rng.random((B, g + 1)).astype(np.float32)
    r = oracle.accept(zt, zd, tok, u, eta=eta)
    betas = [np.minimum(d[1], d[2]).sum() for d in dists]
    pn = [np.prod(betas[:k]) * (1 - betas[k]) for k in range(g)] + [np.prod(betas)]
    assert chisquare(np.bincount(r.n_accepted, minlength=g + 1), np.array(pn) * B).pvalue > 1e-4
    for k in range(g + 1):
        sel = r.n_accepted == k
        if k < g:
            p, q, ph = dists[k]
            w = np.maximum(np.maximum(p - ph, p - q), 0)
        else:
            w = sp_softmax(z[g].astype(np.float64))
        w = w / w.sum()
        counts = np.bincount(r.out_tokens[sel, k], minlength=V)
        keep = w > 1e-12
        assert counts[~keep].sum() == 0
        assert chisquare(counts[keep], w[keep] / w[keep].sum() * sel.sum()).pvalue > 1e-4
        # accepted prefix is the drafts, the rest is -1
        np.testing.assert_array_equal(r.out_tokens[sel, :k], tok[sel, :k])
        assert np.all(r.out_tokens[sel, k + 1:] == -1)


def test_accept_test_uses_phat_not_p():
    """A token the drafter likes and the target does not: rejected at eta = 0 for
    this uniform, accepted once the shift moves p_hat toward q."""
    z = np.array([[[2.0, 0.0, -1.0], [0.0, 0.0, 0.0]]], dtype=np.float32)
    zq = np.array([[[0.0, 2.0, -1.0]]], dtype=np.float32)
    tok = np.array([[1]], np.int32)
    p, q, _ = np_distributions(z[0, 0], zq[0, 0], 0.0, 1.0, 0.1)
    u = np.array([[min(0.9, 2.0 * p[1] / q[1]), 0.5]], np.float32)       # above p/q
    assert oracle.accept(z, zq, tok, u, eta=0.0).n_accepted[0] == 0
    r = oracle.accept(z, zq, tok, u, eta=5.0)
    _, _, ph = np_distributions(z[0, 0], zq[0, 0], 5.0, 1.0, 0.1)
    assert ph[1] / q[1] > u[0, 0]
    assert r.n_accepted[0] == 1
    np.testing.assert_allclose(r.ratio[0, 0], ph[1] / q[1], rtol=1e-12)


def test_per_sequence_gamma_and_unused_rows():
    rng = np.random.default_rng(10)
    B, gmax, V = 6, 4, 9
    zt = rng.normal(0, 2, (B, gmax + 1, V)).astype(np.float32)
    zd = zt[:, :gmax].copy()                           # identical: all accepted
    tok = rng.integers(0, V, (B, gmax)).astype(np.int32)
    u = rng.random((B, gmax + 1)).astype(np.float32)
    gam = np.array([0, 1, 2, 3, 4, 2], np.int32)
    r = oracle.accept(zt, zd, tok, u, eta=1.0, gammas=gam)
    np.testing.assert_array_equal(r.n_accepted, gam)
    for b in range(B):
        g = gam[b]
        want = cdf_pick(sp_softmax(zt[b, g].astype(np.float64)), float(u[b, gmax]))
        assert r.out_tokens[b, g] == want              # bonus from target row gamma_b
        assert np.all(r.out_tokens[b, g + 1:] == -1)


def test_extreme_settings_stay_finite():
    rng = np.random.default_rng(11)
    V = 2000
    z = rng.normal(0, 4, V)
    zq = z + rng.normal(0, 1, V)
    for T, eta in [(0.1, 50.0), (0.1, 0.0), (1.0, 50.0)]:
        p, q, ph = oracle.distributions(z, zq, eta=eta, temperature=T, tail_alpha=0.0)
        for a in (p, q, ph):
            assert np.all(np.isfinite(a)) and abs(a.sum() - 1) < 1e-12


def test_invalid_arguments_are_rejected():
    z = np.zeros((1, 2, 4), np.float32)
    zd = np.zeros((1, 1, 4), np.float32)
    u = np.zeros((1, 2), np.float32)
    with pytest.raises(ValueError):
        oracle.accept(z, zd, np.array([[4]], np.int32), u, eta=1.0)        # token out of range
    with pytest.raises(ValueError):
        oracle.accept(z, zd, np.array([[0]], np.int32), u, eta=1.0, temperature=0.0)
    with pytest.raises(ValueError):
        oracle.accept(z, zd, np.array([[0]], np.int32), u, eta=-1.0)


# ---------------------------------------------------------------- stored worked example
def test_worked_example_fixture():
    """V = 4 example (z = [2,1,0,-1], z_q = [0,2,1,-1], T = 1, eta = 2): the stored
    oracle output agrees with library-softmax arithmetic, and the oracle still
    reproduces it."""
    with open(os.path.join(GOLDEN, "accept_v4_example.json")) as f:
        gold = json.load(f)
    z, zq = np.array(gold["z"]), np.array(gold["zq"])
    p, q, ph = np_distributions(z, zq, gold["eta"], gold["T"], gold["tail_alpha"])
    np.testing.assert_allclose(gold["p"], p, rtol=1e-12)
    np.testing.assert_allclose(gold["p_hat"], ph, rtol=1e-12)
    law, beta = output_law(p, q, ph)
    np.testing.assert_allclose(gold["beta"], beta, rtol=1e-12)
    np.testing.assert_allclose(gold["law"], law, rtol=1e-12)
    o = oracle.distributions(z, zq, eta=gold["eta"], temperature=gold["T"], tail_alpha=gold["tail_alpha"])
    np.testing.assert_allclose(o[2], gold["p_hat"], rtol=1e-14)
    # the law is visibly not p here (softmax([2,1,0,-1])[0] = 0.6439...)
    assert abs(p[0] - 0.6439142598879722) < 1e-15 and abs(law[0] - p[0]) > 0.3
    for case in gold["cases"]:
        r = oracle.accept(np.array([[z, z]], np.float32), np.array([[zq]], np.float32),
                          np.array([[case["draft"]]], np.int32),
                          np.array([[case["r"], case["u"]]], np.float32), eta=gold["eta"])
        assert int(r.n_accepted[0]) == case["n_accepted"]
        assert int(r.out_tokens[0, 0]) == case["token"]


# ---------------------------------------------------------------- the margins the GPU comparison relies on
def test_accept_margin_hand_cases():
    """accept_margin = |min(1, rho) - r| (Alg. 1 accept test).  eta = 0, V = 2: p = (1/4, 3/4), q = (1/2, 1/2),
    so rho(token 0) = 1/2 and rho(token 1) = 3/2 (clamped to 1).  The uniform is placed a known distance
    from the threshold on either side; the margin must be that distance, and the decision must follow the
    side."""
    z = np.log(np.array([[1.0, 3.0], [1.0, 3.0]], dtype=np.float64)).astype(np.float32)[None]    # [1, 2, 2]
    zq = np.zeros((1, 1, 2), dtype=np.float32)
    p0 = float(sp_softmax(z[0, 0].astype(np.float64))[0])            # 0.25 up to the rounding of ln 3 to fp32
    for tok, thr in ((0, 2.0 * p0), (1, 1.0)):
        for delta in (+5e-6, -5e-6, +0.2, -0.3):
            u = np.float32(thr + delta)
            if not (0.0 <= u < 1.0):
                continue
            r = oracle.accept(z, zq, np.array([[tok]], np.int32), np.array([[u, 0.5]], np.float32), eta=0.0,
                              tail_alpha=0.0)
            want = abs(thr - float(u))
            assert abs(r.accept_margin[0, 0] - want) < 1e-12, (tok, delta, r.accept_margin, want)
            assert int(r.n_accepted[0]) == (1 if float(u) <= thr else 0)
            assert abs(r.ratio[0, 0] - (2.0 * p0 if tok == 0 else 2.0 * (1.0 - p0))) < 1e-12


def test_draw_margin_hand_cases():
    """draw_margin = distance of u to the nearer edge of the drawn token's interval of the NORMALISED
    cumulative distribution.  Residual at eta = 0 with p = (1/8, 2/8, 5/8), q = (.8, .1, .1): weights
    (0, .15, .525), W = .675, interval edges 0 | 0 | 2/9 | 1.  Bonus draw from p: edges 0 | 1/8 | 3/8 | 1."""
    z = np.log(np.array([1.0, 2.0, 5.0]))
    zq = np.log(np.array([0.8, 0.1, 0.1]))
    zt = np.stack([z, z]).astype(np.float32)[None]
    zd = zq.astype(np.float32)[None, None]
    p = sp_softmax(zt[0, 0].astype(np.float64))
    q = sp_softmax(zd[0, 0].astype(np.float64))
    w = np.maximum(p - q, 0.0)
    edges = np.concatenate([[0.0], np.cumsum(w) / w.sum()])
    assert abs(edges[2] - 2.0 / 9.0) < 1e-6
    # token 0 is drafted and rejected with r = 0.9 (rho = p0/q0 = 0.156)
    for u, tok in ((0.2, 1), (0.1, 1), (0.23, 2), (0.9, 2), (0.0, 1)):
        uf = np.float32(u)
        r = oracle.accept(zt, zd, np.array([[0]], np.int32), np.array([[0.9, uf]], np.float32), eta=0.0,
                          tail_alpha=0.0)
        assert r.n_accepted[0] == 0 and r.out_tokens[0, 0] == tok, (u, r.out_tokens)
        want = min(float(uf) - edges[tok], edges[tok + 1] - float(uf))
        assert abs(r.draw_margin[0] - want) < 1e-12, (u, r.draw_margin, want)
    # bonus row (draft accepted with r = 0): draw from p
    pe = np.concatenate([[0.0], np.cumsum(p)])
    for u, tok in ((0.05, 0), (0.124, 0), (0.126, 1), (0.37, 1), (0.38, 2), (0.99, 2)):
        uf = np.float32(u)
        r = oracle.accept(zt, zd, np.array([[2]], np.int32), np.array([[0.0, uf]], np.float32), eta=0.0,
                          tail_alpha=0.0)
        assert r.n_accepted[0] == 1 and r.out_tokens[0, 1] == tok, (u, r.out_tokens)
        want = min(float(uf) - pe[tok], pe[tok + 1] - float(uf))
        assert abs(r.draw_margin[0] - want) < 1e-12, (u, r.draw_margin, want)


def test_draw_margin_is_zero_when_the_target_rounds_up_to_the_total():
    """A uniform of exactly 1 (outside the [0, 1) contract) makes u * W equal W, no running sum exceeds
    it, and the draw falls back to the last entry with weight; the margin of that case is 0."""
    zt = np.log(np.array([[1.0, 2.0, 5.0, 1e-30], [1.0, 2.0, 5.0, 1e-30]])).astype(np.float32)[None]
    zd = np.zeros((1, 1, 4), dtype=np.float32)
    r = oracle.accept(zt, zd, np.array([[0]], np.int32), np.array([[0.0, 1.0]], np.float32), eta=0.0, tail_alpha=0.0)
    assert r.n_accepted[0] == 1 and r.draw_margin[0] == 0.0
    assert r.out_tokens[0, 1] == 3                       # the last entry whose weight is positive


# ---------------------------------------------------------------- the greedy limit T -> 0
def test_greedy_limit_equals_small_temperature_runs():
    """The T -> 0 rule is pinned against the general oracle at small temperatures.  The ratio of Alg. 1 behaves
    like exp((target gap - drafter gap) / T), so wherever the two gaps differ by more than 0.5 (or are both 0)
    T = 0.05 and 0.03 already sit in the limit: ratios are e^(+-10) and beyond, far from any uniform in
    [0.01, 0.99].  (Much smaller T would underflow q(x') to 0 in float64, which the general oracle treats as
    'accept'.)  Sequences with a closer call, or whose deciding row has a runner-up within 0.5 of the maximum,
    are left out; the gaps are computed here from the logits.  Drafts are the drafter's arg-max for two thirds
    of the sequences and arbitrary tokens for the rest; eta = 0, 5 and 50.  Prefix lengths are compared for
    all of them; the emitted token only where the rejected draft was the drafter's arg-max (what a greedy
    drafter proposes): for other ids the literal limit of the residual depends on the runner-up gaps and the
    greedy rule emits the target's arg-max instead (a stated deviation for inputs of probability 0)."""
    rng = np.random.default_rng(21)
    B, g, V = 300, 5, 200
    zt = rng.normal(0, 3, (B, g + 1, V)).astype(np.float32)
    zd = (zt[:, :g] + rng.normal(0, 2.0, (B, g, V))).astype(np.float32)
    tok = np.argmax(zd, -1).astype(np.int32)
    tok[::3] = rng.integers(0, V, size=tok[::3].shape)
    u = (rng.random((B, g + 1)) * 0.98 + 0.01).astype(np.float32)
    lim = oracle.accept_greedy(zt, zd, tok, u)
    z64, zd64 = zt.astype(np.float64), zd.astype(np.float64)
    idx = tok[..., None].astype(np.int64)
    gap_t = np.take_along_axis(z64[:, :g], idx, -1)[..., 0] - z64[:, :g].max(-1)
    gap_d = np.take_along_axis(zd64, idx, -1)[..., 0] - zd64.max(-1)
    diff = gap_t - gap_d
    top2 = np.sort(z64, -1)[..., -1] - np.sort(z64, -1)[..., -2]                       # [B, g+1]
    all_argmax = np.all(gap_d == 0, axis=1)                                            # the drafter's own arg-max everywhere
    n = lim.n_accepted
    stop_is_argmax = np.array([n[b] == g or gap_d[b, n[b]] == 0 for b in range(B)])
    for T, eta in ((0.05, 0.0), (0.03, 0.0), (0.03, 5.0), (0.005, 50.0)):
        # in the limit when the gap difference outweighs the mixing term (which moves scores by up to 2 eta) and
        # any uniform: (2 eta + ln 100) T, with margin
        need = max(0.5, 1.5 * (2 * eta + 4.6) * T)
        clear = np.all((np.abs(diff) > need) | ((gap_t == 0) & (gap_d == 0)), axis=1) & (top2[np.arange(B), n] > need)
        if T < 0.03:
            clear &= all_argmax                      # q(x') of an arbitrary id underflows to 0 at this temperature
        assert clear.sum() >= 40 and 0 < n[clear].mean() < g, (T, eta, clear.sum())
        gen = oracle.accept(zt, zd, tok, u, eta=eta, temperature=T, tail_alpha=0.1)
        np.testing.assert_array_equal(gen.n_accepted[clear], n[clear])
        sel = clear & stop_is_argmax
        assert sel.sum() >= 30
        np.testing.assert_array_equal(gen.out_tokens[sel], lim.out_tokens[sel])
    assert len(set(n[(np.arange(B) % 3 == 0) & np.all(np.abs(diff) > 0.5, axis=1)].tolist())) >= 2   # arbitrary ids: both outcomes


def test_greedy_limit_hand_cases():
    z = np.array([[[1.0, 5.0, 2.0], [0.0, 0.0, 9.0], [4.0, 4.0, 1.0]]], dtype=np.float32)     # arg-max 1, 2, 0 (tie -> lowest)
    zq = np.array([[[0.0, 3.0, 1.0], [7.0, 1.0, 6.5]]], dtype=np.float32)                       # arg-max 1, 0
    u = np.array([[0.5, 0.5, 0.123]], dtype=np.float32)
    # drafts (1, 0): position 0 agrees with the target; position 1 is the drafter's arg-max but not the target's
    r = oracle.accept_greedy(z, zq, np.array([[1, 0]], np.int32), u)
    assert r.n_accepted.tolist() == [1] and r.out_tokens.tolist() == [[1, 2, -1]]
    assert r.ratio[0].tolist() == [1.0, 0.0]
    # drafts (1, 2): both are the target's arg-max -> all accepted, bonus = arg-max of row 2 with the tie broken low;
    # token 2 at position 1 is not the drafter's arg-max: its gap (-0.5) is below the target's (0) -> ratio infinite
    r = oracle.accept_greedy(z, zq, np.array([[1, 2]], np.int32), u)
    assert r.n_accepted.tolist() == [2] and r.out_tokens.tolist() == [[1, 2, 0]]
    assert r.ratio[0, 0] == 1.0 and np.isinf(r.ratio[0, 1])
    # a token that is nobody's arg-max: target gap 1 - 5 = -4, drafter gap 0 - 3 = -3 -> rejected; 2: gaps -3, -2 -> rejected
    r = oracle.accept_greedy(z, zq, np.array([[0, 2]], np.int32), u)
    assert r.n_accepted.tolist() == [0] and r.out_tokens.tolist() == [[1, -1, -1]]
    # equal gaps (-3 and -3): the limit of the ratio is 1 -> accepted
    zq2 = zq.copy(); zq2[0, 0] = [0.0, 5.0, 2.0]
    r = oracle.accept_greedy(z, zq2, np.array([[2, 2]], np.int32), u)
    assert r.ratio[0, 0] == 1.0 and r.n_accepted.tolist() == [2]
    # a uniform of exactly 0 passes even a ratio of 0 (the literal r <= min(1, ratio))
    # (position 1 then holds the target's arg-max, so everything is accepted and the bonus row decides the last token)
    r = oracle.accept_greedy(z, zq, np.array([[0, 2]], np.int32), np.array([[0.0, 0.5, 0.1]], np.float32))
    assert r.n_accepted.tolist() == [2] and r.out_tokens.tolist() == [[0, 2, 0]]
    r = oracle.accept_greedy(z, zq, np.array([[0, 0]], np.int32), np.array([[0.0, 0.5, 0.1]], np.float32))
    assert r.n_accepted.tolist() == [1] and r.out_tokens.tolist() == [[0, 2, -1]]


def test_greedy_limit_identical_logits_and_gammas():
    rng = np.random.default_rng(4)
    zt = rng.normal(0, 3, (6, 5, 50)).astype(np.float32)
    tok = np.argmax(zt[:, :4], -1).astype(np.int32)
    gam = np.array([4, 2, 0, 4, 1, 3], dtype=np.int32)
    r = oracle.accept_greedy(zt, zt[:, :4].copy(), tok, rng.random((6, 5)).astype(np.float32), gammas=gam)
    assert r.n_accepted.tolist() == gam.tolist()
    for b in range(6):
        g = int(gam[b])
        assert r.out_tokens[b, :g].tolist() == tok[b, :g].tolist()
        assert r.out_tokens[b, g] == int(np.argmax(zt[b, g])) and np.all(r.out_tokens[b, g + 1:] == -1)
