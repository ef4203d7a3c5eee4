"""GPU parity: rapid_accept (C ABI, gfx950 kernels) against the float64 oracle.
Accepted-prefix length and emitted tokens must match bit for bit, except
sequences whose decisive accept test lies within 1e-5 of its uniform, or whose
draw lands within 1e-10 (normalised) of a CDF edge.  All inputs are seeded, so the
number of such sequences is a constant of each test and is asserted exactly (0
unless a test says otherwise)."""
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


def check(cfg, acc, what, *, eta=None, temperature=None, tail_alpha=None, use_gammas=True, exempt=0):
    eta = cfg.eta if eta is None else eta
    temperature = cfg.temperature if temperature is None else temperature
    tail_alpha = cfg.tail_alpha if tail_alpha is None else tail_alpha
    gpu, ref = gu.run_accept_case(acc, eta=eta, temperature=temperature, tail_alpha=tail_alpha, use_gammas=use_gammas)
    st = gu.compare_accept(gpu, ref, acc.gammas if use_gammas else None, cfg.gamma_max)
    print(f"[{what}] {st} mean_accepted={ref.n_accepted.mean():.2f}")
    assert st["n_mismatch"] == 0 and st["token_mismatch"] == 0, st
    assert st["exempt_sequences"] == exempt, st
    assert st["max_ratio_rel_err"] < 1e-4, st
    # shape of the token rows: accepted drafts, one drawn token in [0, V), then -1
    n, tok, _ = gpu
    for b in range(len(n)):
        assert 0 <= tok[b, n[b]] < cfg.vocab
        assert np.all(tok[b, n[b] + 1:] == -1)
        np.testing.assert_array_equal(tok[b, :n[b]], acc.draft_tokens[b, :n[b]])
    return gpu, ref, st


def test_tiny_config():
    cfg = wl.CONFIGS["tiny"]
    check(cfg, wl.gen_accept_inputs(cfg), "tiny")


def test_tiny_many_sequences_all_branches():
    cfg = wl.scaled(wl.CONFIGS["tiny"], draft_noise_std=1.5, gamma_choices=(0, 1, 2, 3, 4))
    acc = wl.gen_accept_inputs(cfg, batch=256)
    gpu, ref, st = check(cfg, acc, "tiny x256")
    assert len(set(ref.n_accepted.tolist())) >= 4           # rejects at several positions and full accepts


@pytest.mark.parametrize("V", [1, 2, 3, 5, 1023, 1024, 1025, 4099, 50257])
def test_vocab_sizes_and_unaligned_rows(V):
    cfg = wl.scaled(wl.CONFIGS["tiny"], vocab=V, draft_noise_std=1.0, gamma_choices=(3,))
    check(cfg, wl.gen_accept_inputs(cfg, batch=16), f"V={V}")


@pytest.mark.parametrize("eta,T,alpha", [(0.0, 1.0, 0.1), (1.0, 1.0, 0.0), (5.0, 1.0, 0.1), (20.0, 1.0, 0.1),
                                         (50.0, 1.0, 0.1), (5.0, 0.1, 0.1), (50.0, 0.1, 0.1), (2.0, 2.0, 0.3)])
def test_eta_temperature_tail_sweep(eta, T, alpha):
    cfg = wl.scaled(wl.CONFIGS["tiny"], vocab=32000, logit_std=2.0, draft_noise_std=0.7, temperature=T,
                    gamma_choices=(5,))
    check(cfg, wl.gen_accept_inputs(cfg, batch=48), f"eta={eta} T={T} alpha={alpha}", eta=eta, temperature=T,
          tail_alpha=alpha)


def test_identical_logits_accept_everything():
    cfg = wl.scaled(wl.CONFIGS["tiny"], draft_noise_std=0.0, gamma_choices=(4,))
    acc = wl.gen_accept_inputs(cfg, batch=32)
    gpu, ref, _ = check(cfg, acc, "identical logits", eta=3.0)
    assert np.all(gpu[0] == 4) and np.allclose(gpu[2], 1.0, rtol=1e-5)


def test_eta_zero_is_plain_speculative_sampling():
    cfg = wl.scaled(wl.CONFIGS["tiny"], draft_noise_std=1.0, gamma_choices=(4,))
    acc = wl.gen_accept_inputs(cfg, batch=64)
    gpu, ref, _ = check(cfg, acc, "eta=0", eta=0.0)
    # ratio is p(x)/q(x) computed independently here from the logits
    zt, zd = acc.target_logits.astype(np.float64), acc.draft_logits.astype(np.float64)
    lp = zt - np.log(np.exp(zt - zt.max(-1, keepdims=True)).sum(-1, keepdims=True)) - zt.max(-1, keepdims=True)
    lq = zd - np.log(np.exp(zd - zd.max(-1, keepdims=True)).sum(-1, keepdims=True)) - zd.max(-1, keepdims=True)
    idx = acc.draft_tokens[..., None].astype(np.int64)
    want = np.exp(np.take_along_axis(lp[:, :4], idx, -1) - np.take_along_axis(lq, idx, -1))[..., 0]
    np.testing.assert_allclose(gpu[2], want, rtol=1e-4)


def test_out_of_range_draft_token_is_rejected():
    cfg = wl.scaled(wl.CONFIGS["tiny"], draft_noise_std=0.0, gamma_choices=(4,))
    acc = wl.gen_accept_inputs(cfg, batch=2)
    acc.draft_tokens[0, 2] = cfg.vocab            # invalid id at position 2 of sequence 0
    acc.draft_tokens[1, 0] = -7
    dev = lambda a: torch.from_numpy(a).cuda()
    n, tok, _ = gu.rapid().rapid_accept(dev(acc.target_logits), dev(acc.draft_logits), dev(acc.draft_tokens), 1.0,
                                        dev(acc.uniforms))
    torch.cuda.synchronize()
    assert n.tolist() == [2, 0]
    assert 0 <= tok[0, 2] < cfg.vocab and 0 <= tok[1, 0] < cfg.vocab
    # the status block at the head of the workspace counts the positions rejected for that reason
    bad_ids, _ = gu.rapid().accept_status()
    assert bad_ids == 2
    gu.rapid().rapid_accept(dev(acc.target_logits), dev(acc.draft_logits),
                            dev(np.clip(acc.draft_tokens, 0, cfg.vocab - 1)), 1.0, dev(acc.uniforms))
    assert gu.rapid().accept_status()[0] == 0               # per call, not cumulative


def test_gamma_zero_only_draws_the_bonus():
    cfg = wl.scaled(wl.CONFIGS["tiny"], gamma_choices=(0,))
    acc = wl.gen_accept_inputs(cfg, batch=8)
    gpu, ref, _ = check(cfg, acc, "gamma=0")
    assert np.all(gpu[0] == 0)


def test_repeat_calls_are_identical():
    cfg = wl.CONFIGS["llama8b_32k"]
    acc = wl.gen_accept_inputs(cfg)
    dev = lambda a: torch.from_numpy(a).cuda()
    args = (dev(acc.target_logits), dev(acc.draft_logits), dev(acc.draft_tokens), cfg.eta, dev(acc.uniforms))
    a = [t.clone() for t in gu.rapid().rapid_accept(*args)]
    b = [t.clone() for t in gu.rapid().rapid_accept(*args)]
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(a, b))


@pytest.mark.parametrize("slice_entries", [4096, 8192, 16384])
def test_every_slice_size_and_the_give_up_path(slice_entries):
    """The row pass at each of its slice sizes against the oracle, and again with the bound of the
    inter-workgroup waits forced to zero from the host: every exchange then takes the path in which a
    workgroup computes the other workgroups' publications itself.  That path must be taken (counted in the
    status block) and must reproduce the normal run bit for bit, accept ratios included."""
    from paper_2502_20330_amd import binding
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=3, gamma_choices=(2, 5), draft_noise_std=1.5, name="giveup")
    acc = wl.gen_accept_inputs(cfg, salt=11)
    r = gu.rapid()
    try:
        r.set_option(binding.OPT_ACCEPT_SLICE, slice_entries)
        gpu, ref, st = check(cfg, acc, f"slice {slice_entries}")
        assert r.accept_status()[1] == 0 or True             # waits that time out on a busy box are legal
        r.set_option(binding.OPT_ACCEPT_WAIT_US, 0)
        gpu0, _ = gu.run_accept_case(acc, eta=cfg.eta)
        giveups = r.accept_status()[1]
        # bounds of the order of an exchange's own latency: some waits succeed, others give up, in one call
        mixed = []
        for wait_us in (1, 2, 4):
            r.set_option(binding.OPT_ACCEPT_WAIT_US, wait_us)
            mixed.append((wait_us, gu.run_accept_case(acc, eta=cfg.eta)[0], r.accept_status()[1]))
    finally:
        r.set_option(binding.OPT_ACCEPT_WAIT_US, 100)
        r.set_option(binding.OPT_ACCEPT_SLICE, 0)
    assert giveups > 0
    print(f"[slice {slice_entries}] give-ups: bound 0 -> {giveups}; " + ", ".join(f"{w} us -> {g}" for w, _, g in mixed))
    for _, other, _ in [(0, gpu0, giveups)] + mixed:
        np.testing.assert_array_equal(gpu[0], other[0])
        np.testing.assert_array_equal(gpu[1], other[1])
        assert np.array_equal(gpu[2].view(np.int32), other[2].view(np.int32))


def test_workspace_needs_no_clearing_and_a_captured_graph_replays():
    """The exchange words of a call are recognised by the call's tags, not by a cleared workspace.  So:
    (a) a workspace filled with arbitrary bits, or still holding another call's publications, gives
    the oracle's results; (b) a HIP graph that captured one call -- its launch arguments frozen, only
    the counter in the workspace moves -- gives the oracle's results on every replay, with other inputs
    each time and eager calls on the same workspace in between."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], vocab=128256, batch=4, gamma_choices=(1, 3, 4), draft_noise_std=1.5,
                    name="graph")
    r = gu.rapid()
    cases = [wl.gen_accept_inputs(cfg, salt=s) for s in (21, 22, 23, 24)]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ref = [gu.oracle.accept(c.target_logits, c.draft_logits, c.draft_tokens, c.uniforms,
                            eta=float(np.float32(cfg.eta)), temperature=float(np.float32(cfg.temperature)),
                            tail_alpha=float(np.float32(cfg.tail_alpha)), gammas=c.gammas) for c in cases]

    def agree(out, i, what):
        torch.cuda.synchronize()
        got = tuple(t.cpu().numpy() for t in out)
        st = gu.compare_accept(got, ref[i], cases[i].gammas, cfg.gamma_max)
        assert st["n_mismatch"] == 0 and st["token_mismatch"] == 0 and st["exempt_sequences"] == 0, (what, st)

    # (a) dirty workspace: random bytes, then all ones, then all zeros, before a call each
    zt, zd, tok, gam, u = (dev(x) for x in (cases[0].target_logits, cases[0].draft_logits, cases[0].draft_tokens,
                                            cases[0].gammas, cases[0].uniforms))
    r.rapid_accept(zt, zd, tok, cfg.eta, u, gammas=gam)       # sizes the workspace
    for fill in ("random", 255, 0):
        if fill == "random":
            r._ws_accept.copy_(torch.randint(0, 256, r._ws_accept.shape, dtype=torch.uint8, device="cuda",
                                              generator=torch.Generator("cuda").manual_seed(5)))
        else:
            r._ws_accept.fill_(fill)
        agree(r.rapid_accept(zt, zd, tok, cfg.eta, u, gammas=gam), 0, f"workspace filled with {fill}")
        assert r.accept_status() == (0, 0) or r.accept_status()[0] == 0

    # (b) one captured call, replayed over changing inputs
    outs = (torch.empty(cfg.batch, dtype=torch.int32, device="cuda"),
            torch.empty(cfg.batch, cfg.gamma_max + 1, dtype=torch.int32, device="cuda"),
            torch.empty(cfg.batch, cfg.gamma_max, dtype=torch.float32, device="cuda"))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        r.rapid_accept(zt, zd, tok, cfg.eta, u, gammas=gam, outs=outs)
    for i in (1, 2, 0, 3, 3):
        c = cases[i]
        for dst, src in ((zt, c.target_logits), (zd, c.draft_logits), (tok, c.draft_tokens), (gam, c.gammas),
                         (u, c.uniforms)):
            dst.copy_(dev(src))
        for o in outs:
            o.fill_(-7)
        graph.replay()
        agree(outs, i, f"replay with inputs {i}")
        agree(r.rapid_accept(zt, zd, tok, cfg.eta, u, gammas=gam), i, f"eager call after replay {i}")


def test_option_values_are_validated():
    from paper_2502_20330_amd import binding
    r = gu.rapid()
    for opt, val in ((binding.OPT_ACCEPT_SLICE, 1000), (binding.OPT_ACCEPT_WAIT_US, -1), (99, 0)):
        with pytest.raises(binding.RapidError) as e:
            r.set_option(opt, val)
        assert e.value.status == -1


# ---------------------------------------------------------------- the greedy limit (temperature 0)
@pytest.mark.parametrize("V,batch,gch", [(8192, 64, (0, 1, 4)), (128256, 8, (8,)), (50257, 16, (3, 10)), (7, 32, (2,))])
def test_greedy_limit(V, batch, gch):
    """temperature = 0: prefix lengths, tokens and the limits of the ratios (0, 1, infinity) against the
    oracle's statement of the T -> 0 limit, bit for bit.  Two thirds of the sequences draft the drafter's
    arg-max (what a greedy drafter does), the rest arbitrary ids; some logits are tied on purpose."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], vocab=V, batch=batch, gamma_choices=gch, draft_noise_std=1.5, name=f"greedy_V{V}")
    acc = wl.gen_accept_inputs(cfg, salt=5)
    g = cfg.gamma_max
    if g > 0:
        acc.draft_tokens[:] = np.argmax(acc.draft_logits, -1).astype(np.int32)
        rng = np.random.default_rng(9)
        acc.draft_tokens[::3] = rng.integers(0, V, size=acc.draft_tokens[::3].shape)
        acc.target_logits[1, 0, : min(V, 5)] = acc.target_logits[1, 0].max() + 1.0      # a five-way tie for the maximum
    gpu, ref = gu.run_accept_case(acc, eta=cfg.eta, temperature=0.0)
    np.testing.assert_array_equal(gpu[0], ref.n_accepted)
    np.testing.assert_array_equal(gpu[1], ref.out_tokens)
    if g > 0:
        for b in range(batch):
            gb = int(acc.gammas[b])
            np.testing.assert_array_equal(gpu[2][b, :gb].astype(np.float64), ref.ratio[b, :gb])
        assert len(set(ref.n_accepted.tolist())) >= 2


def test_greedy_limit_counts_out_of_range_ids_and_rejects_row_statistics():
    from paper_2502_20330_amd import binding
    cfg = wl.scaled(wl.CONFIGS["tiny"], draft_noise_std=0.0, gamma_choices=(4,))
    acc = wl.gen_accept_inputs(cfg, batch=2)
    acc.draft_tokens[:] = np.argmax(acc.draft_logits, -1).astype(np.int32)
    acc.draft_tokens[0, 2] = cfg.vocab
    dev = lambda a: torch.from_numpy(a).cuda()
    n, tok, _ = gu.rapid().rapid_accept(dev(acc.target_logits), dev(acc.draft_logits), dev(acc.draft_tokens), 1.0,
                                        dev(acc.uniforms), temperature=0.0)
    torch.cuda.synchronize()
    assert n.tolist() == [2, 4] and gu.rapid().accept_status()[0] == 1
    st = torch.zeros((2 * 5, 3, 2), device="cuda")
    with pytest.raises(binding.RapidError) as e:
        gu.rapid().rapid_accept(dev(acc.target_logits), dev(acc.draft_logits), dev(acc.draft_tokens), 1.0,
                                dev(acc.uniforms), temperature=0.0, target_stats=st)
    assert e.value.status == -1


def test_bad_arguments_return_error_codes():
    from paper_2502_20330_amd import binding
    z = torch.zeros(1, 2, 8, device="cuda")
    zd = torch.zeros(1, 1, 8, device="cuda")
    t = torch.zeros(1, 1, dtype=torch.int32, device="cuda")
    u = torch.zeros(1, 2, device="cuda")
    for kw in (dict(eta=-1.0), dict(eta=1.0, temperature=-0.5), dict(eta=1.0, tail_alpha=-0.5)):
        eta = kw.pop("eta")
        with pytest.raises(binding.RapidError) as e:
            gu.rapid().rapid_accept(z, zd, t, eta, u, **kw)
        assert e.value.status == -1


# ---------------------------------------------------------------- full benchmark sizes
def test_llama_vocab_full_size():
    """Configs 2/3/5: one sequence, gamma = 8, V = 128256, eta = 1 (and 5's eta sweep)."""
    cfg = wl.CONFIGS["llama8b_32k"]
    acc = wl.gen_accept_inputs(cfg)
    for eta in (1.0, 0.25, 0.5):
        check(cfg, acc, f"V=128256 B=1 eta={eta}", eta=eta)


def test_llama_vocab_many_sequences():
    """Same recipe, 64 seeded sequences with gamma in {4,6,8}: statistics of the exemptions."""
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"])
    acc = wl.gen_accept_inputs(cfg, batch=64, salt=1)
    gpu, ref, st = check(cfg, acc, "V=128256 B=64")
    assert 0 < ref.n_accepted.mean() < acc.gammas.mean()        # both outcomes occur


@pytest.mark.parametrize("eta,T", [(5.0, 1.0), (20.0, 1.0), (50.0, 1.0), (10.0, 0.1)])
def test_paper_settings_gamma_10_llama_vocab(eta, T):
    """gamma = 10 with the eta values the paper searches (5..20 self-speculation, 40..50 upward) and the low
    temperature 0.1 of its robustness study, at the LLaMA vocabulary size, 8 sequences."""
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=8, gamma_choices=(10,), temperature=T, name=f"g10_eta{eta}_T{T}")
    acc = wl.gen_accept_inputs(cfg)
    check(cfg, acc, f"gamma=10 eta={eta} T={T}", eta=eta, temperature=T)


@pytest.mark.parametrize("V,batch,gch,T", [(300000, 3, (2, 3), 1.0), (1 << 22, 2, (1, 2), 1.0), ((1 << 22) - 5, 1, (1,), 0.0),
                                          (600001, 2, (3,), 0.0)])
def test_vocabularies_of_more_than_64_slices(V, batch, gch, T):
    """More than 64 slices per row (up to the largest vocabulary the header allows, 2^22): the loops that walk
    the slices of a row 64 at a time -- polls, combines, the prefix over slice totals with its carry -- run
    more than once; also in the greedy limit."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], vocab=V, batch=batch, gamma_choices=gch, draft_noise_std=1.0, logit_std=4.0,
                    temperature=T if T > 0 else 1.0, name=f"V{V}")
    acc = wl.gen_accept_inputs(cfg, salt=V % 97)
    check(cfg, acc, f"V={V} T={T}", temperature=T)


def test_more_than_64_drafted_positions():
    """gamma = 70 (one kv-head group of one query head allows up to 95): the per-lane read of the accept flags
    and the row loops run over more than one wave's worth of positions; rejects placed late so that n > 64 occurs."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], vocab=4099, batch=6, gamma_choices=(70, 66, 3), draft_noise_std=0.05,
                    name="gamma70")
    acc = wl.gen_accept_inputs(cfg, salt=5)
    gpu, ref, _ = check(cfg, acc, "gamma=70", eta=0.5)
    assert ref.n_accepted.max() > 64


def test_nan_and_inf_logits_do_not_hang_or_write_out_of_range():
    """Behaviour on NaN / infinite logits is unspecified, but every call must return and every emitted
    token must be a vocabulary index or -1."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], vocab=5000, gamma_choices=(3,))
    acc = wl.gen_accept_inputs(cfg, batch=6)
    zt, zd = acc.target_logits.copy(), acc.draft_logits.copy()
    zt[0, 1, 17] = np.nan
    zd[1, 0, :] = np.nan
    zt[2, :, :] = np.nan
    zt[3, 2, 99] = np.inf
    zd[4, 1, 5] = -np.inf
    zt[5, :, :] = -np.inf
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    n, tok, _ = gu.rapid().rapid_accept(dev(zt), dev(zd), dev(acc.draft_tokens), 1.0, dev(acc.uniforms))
    torch.cuda.synchronize()
    n, tok = n.cpu().numpy(), tok.cpu().numpy()
    assert np.all((n >= 0) & (n <= 3))
    assert np.all((tok >= -1) & (tok < cfg.vocab))
