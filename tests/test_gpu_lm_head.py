"""GPU parity: rapid_lm_head (C ABI, gfx950 kernel) against the float64 oracle, element by element,
and the statistics it hands to rapid_accept_prestats.

Tolerances.  Logits: bf16 x bf16 products are exact in fp32; the kernel adds `hidden` of them in fp32
(MFMA accumulators, four K quarters added at the end), so the error is a few ulps of the largest partial
sum: |gpu - ref| <= 5e-5 + 1e-5 |ref| for |z| up to ~25 and hidden up to 8192 (measured: below 8e-6; printed).
Statistics: the chunk maximum must equal the maximum of the GPU's own logits bit for bit; the chunk sum is
an fp32 sum of at most 512 exponentials, relative error <= 2e-5 against the float64 sum over the oracle's logits
shifted by the GPU maximum."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_20330_amd import binding
from paper_2502_20330_amd import workloads as wl

pytestmark = pytest.mark.gpu

ATOL, RTOL = 5e-5, 1e-5

gu = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global gu
    import gpu_util
    gu = gpu_util
    yield


def run(rows, hidden, vocab, T=1.0, salt=0, what=""):
    h, w = wl.gen_lm_head_inputs(rows, hidden, vocab, salt=salt)
    hd, wd = gu.bf16_to_dev(h), gu.bf16_to_dev(w)
    logits, stats = gu.rapid().rapid_lm_head(hd, wd, temperature=T)
    torch.cuda.synchronize()
    z = logits.cpu().numpy().astype(np.float64)
    st = stats.cpu().numpy().astype(np.float64)
    ref = oracle.lm_head(h, w)
    err = np.abs(z - ref)
    assert np.all(np.isfinite(z))
    worst = np.unravel_index(np.argmax(err - RTOL * np.abs(ref)), err.shape)
    assert np.all(err <= ATOL + RTOL * np.abs(ref)), \
        f"{what}: max abs err {err.max():.3e} at {worst}: got {z[worst]:.6f} ref {ref[worst]:.6f}"
    CH = gu.rapid().lm_head_chunk(vocab, rows)              # chunk the library chose for this vocabulary and row count
    assert CH % 16 == 0 and 16 <= CH <= 512
    nch = (vocab + CH - 1) // CH
    assert st.shape == (rows, nch, 2)
    # chunk maxima: exactly the maxima of the logits the kernel wrote
    pad = np.full((rows, nch * CH), -np.inf)
    pad[:, :vocab] = z
    assert np.array_equal(st[:, :, 0], pad.reshape(rows, nch, CH).max(axis=2)), what + ": chunk maxima"
    # chunk sums against the oracle's definition on the oracle's logits, re-based to the GPU maximum
    cmax, csum = oracle.chunk_stats(ref, CH, T)
    ref_sum = csum * np.exp((cmax - st[:, :, 0]) / T)
    np.testing.assert_allclose(st[:, :, 1], ref_sum, rtol=2e-5 + 2 * ATOL / T, err_msg=what + ": chunk sums")
    print(f"[{what}] rows={rows} hidden={hidden} vocab={vocab} T={T}: max_abs={err.max():.3e} "
          f"max|ref|={np.abs(ref).max():.2f}")
    return z, st, (hd, wd)


@pytest.mark.parametrize("vocab", [16, 17, 500, 512, 513, 1000, 1024, 1537, 4103, 8192, 8193, 131072 + 16, 152064])
def test_vocabulary_edges(vocab):
    run(9, 1024, vocab, what=f"vocab{vocab}")


@pytest.mark.parametrize("rows", [1, 2, 5, 9, 11, 16, 17, 31, 32, 33, 48, 55, 64, 72, 80, 81, 96])
def test_row_counts(rows):
    """One to six blocks of 16 rows of h over one pass of the weights (a batch of verification steps)."""
    run(rows, 2048, 3000, salt=rows, what=f"rows{rows}")


@pytest.mark.parametrize("rows,hidden,vocab", [(72, 3584, 5000), (40, 1536, 777), (96, 4096, 16), (20, 512, 8193)])
def test_many_rows_on_other_widths_and_vocabulary_edges(rows, hidden, vocab):
    run(rows, hidden, vocab, salt=rows + hidden, what=f"rows{rows}_hidden{hidden}_vocab{vocab}")


@pytest.mark.parametrize("hidden", [128, 256, 384, 512, 1024, 1408, 1536, 2304, 3072, 3584, 4096, 5120, 8192])
def test_hidden_sizes(hidden):
    run(9, hidden, 2500, salt=hidden, what=f"hidden{hidden}")


@pytest.mark.parametrize("T", [0.1, 0.7, 2.0])
def test_temperature_in_statistics(T):
    run(4, 1024, 2000, T=T, what=f"T{T}")


@pytest.mark.parametrize("rows,vocab,ldz,first", [(3, 777, 1000, 0), (3, 776, 1000, 0), (19, 776, 1001, 0),
                                                  (3, 776, 1000, 1), (40, 2048, 2052, 2)])
def test_strided_logits_rows_and_no_stats(rows, vocab, ldz, first):
    """Row strides that are / are not a multiple of four floats and row starts that are / are not 16-byte
    aligned (the kernel stores four logits at a time only where it may); nothing outside [0, vocab) of a
    row is written."""
    h, w = wl.gen_lm_head_inputs(rows, 1024, vocab, salt=3)
    hd, wd = gu.bf16_to_dev(h), gu.bf16_to_dev(w)
    big = torch.full((rows * ldz + 8,), 7.0, dtype=torch.float32, device="cuda")
    view = big[first:first + rows * ldz].view(rows, ldz)[:, :vocab]
    gu.rapid().rapid_lm_head(hd, wd, want_stats=False, logits=view)
    torch.cuda.synchronize()
    ref = oracle.lm_head(h, w)
    flat = big.cpu().numpy().astype(np.float64)
    got = flat[first:first + rows * ldz].reshape(rows, ldz)
    assert np.all(np.abs(got[:, :vocab] - ref) <= ATOL + RTOL * np.abs(ref))
    assert np.all(got[:, vocab:] == 7.0), "elements past the vocabulary must not be written"
    assert np.all(flat[:first] == 7.0) and np.all(flat[first + rows * ldz:] == 7.0)


def test_repeat_calls_are_bitwise_identical():
    h, w = wl.gen_lm_head_inputs(9, 4096, 5000, salt=9)
    hd, wd = gu.bf16_to_dev(h), gu.bf16_to_dev(w)
    a, sa = gu.rapid().rapid_lm_head(hd, wd)
    a, sa = a.clone(), sa.clone()
    b, sb = gu.rapid().rapid_lm_head(hd, wd)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(sa, sb)


def test_bad_arguments_return_error_codes():
    r = gu.rapid()
    h = torch.zeros(97, 1024, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(64, 1024, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.RapidError) as e:
        r.rapid_lm_head(h, w, want_stats=False)
    assert e.value.status == binding.RAPID_EUNSUPPORTED                      # 97 rows
    with pytest.raises(binding.RapidError) as e:
        r.rapid_lm_head(h[:4, :1000].contiguous(), w[:, :1000].contiguous())
    assert e.value.status == binding.RAPID_EUNSUPPORTED                      # hidden not a multiple of 128
    with pytest.raises(binding.RapidError) as e:
        r.rapid_lm_head(h[:4], w, temperature=0.0)
    assert e.value.status == binding.RAPID_EINVAL


def test_full_size_head_and_accept_with_its_statistics():
    """LLaMA-3.1-8B head shape: 9 verification rows x 4096 hidden x 128256 entries.  Every logit against the
    oracle; then the acceptance pass fed with the kernel's logits and statistics against (a) the same pass
    forming its own statistics and (b) the oracle's accept on the very same logits."""
    cfg = wl.CONFIGS["llama8b_128k_step"]
    g, V = cfg.gamma_max, cfg.vocab
    z, st, _ = run(g + 1, 4096, V, what="llama8b head")
    zt = torch.from_numpy(z.astype(np.float32)).cuda().reshape(1, g + 1, V)
    acc = wl.gen_accept_inputs(cfg)
    # drafter logits: the same kernel, one row per drafter step, on hidden states that are the target's plus
    # noise (so that drafts are accepted at a realistic rate); input construction only
    h, w = wl.gen_lm_head_inputs(g + 1, 4096, V)
    noise = np.random.default_rng(11).standard_normal((g, 4096)).astype(np.float32) * 0.25
    hq = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(h[:g]) + noise)
    zq, stq = gu.rapid().rapid_lm_head(gu.bf16_to_dev(hq), gu.bf16_to_dev(w))
    zq_ref = oracle.lm_head(hq, w)
    assert np.all(np.abs(zq.cpu().numpy() - zq_ref) <= ATOL + RTOL * np.abs(zq_ref))
    # draft tokens: the drafter's own samples from softmax(zq), by the library's draw at gamma = 0
    toks = []
    u0 = torch.from_numpy(acc.uniforms[:, :g].copy()).cuda()
    for k in range(g):
        _, t, _ = gu.rapid().rapid_accept(zq[k].reshape(1, 1, V), torch.empty(1, 0, V, device="cuda"),
                                          torch.empty(1, 0, dtype=torch.int32, device="cuda"), 0.0,
                                          u0[:, k:k + 1].contiguous(), want_ratio=False)
        toks.append(t[0, 0])
    tok = torch.stack(toks).reshape(1, g).to(torch.int32)
    u = torch.from_numpy(acc.uniforms).cuda()
    zq3 = zq.reshape(1, g, V)
    accepted = []
    for eta in (0.0, 1.0, 5.0):
        a = gu.rapid().rapid_accept(zt, zq3, tok, eta, u)
        b = gu.rapid().rapid_accept(zt, zq3, tok, eta, u, target_stats=st_dev(st), draft_stats=stq)
        torch.cuda.synchronize()
        ref = oracle.accept(zt.cpu().numpy(), zq3.cpu().numpy(), tok.cpu().numpy(), acc.uniforms,
                            eta=eta, temperature=1.0, tail_alpha=0.1)
        for name, got in (("own statistics", a), ("head statistics", b)):
            res = gu.compare_accept(tuple(x.cpu().numpy() if x is not None else None for x in got), ref, None, g)
            assert res["n_mismatch"] == 0 and res["token_mismatch"] == 0, f"eta={eta} {name}: {res}"
            assert res["max_ratio_rel_err"] < 1e-4, f"eta={eta} {name}: {res}"
        print(f"[head+accept eta={eta}] n_accepted={int(b[0][0])} tokens={b[1][0].tolist()}")
        accepted.append(int(b[0][0]))
    assert max(accepted) > 0, "the correlated drafter should get some drafts accepted"


def test_batched_head_feeds_the_batched_accept():
    """The ragged batch of the benchmark (8 sequences, gamma in {4, 6, 8}: 72 row slots): one pass over the
    LLaMA-sized weights gives all target logits and their statistics, which rapid_accept_prestats consumes;
    every logit against the oracle, and the accept results against the oracle's accept on the same logits."""
    cfg = wl.CONFIGS["ragged_paged"]
    seqs = wl.gen_sequences(cfg)
    B, g, V = cfg.batch, cfg.gamma_max, cfg.vocab
    rows = B * (g + 1)
    z, st, _ = run(rows, 4096, V, what="batched head")
    zt = z.astype(np.float32).reshape(B, g + 1, V)
    rng = np.random.default_rng(17)
    zd = (zt[:, :g] + rng.standard_normal((B, g, V)).astype(np.float32)).astype(np.float32)
    tok = np.argmax(zd.astype(np.float64) + rng.gumbel(size=zd.shape), -1).astype(np.int32)
    u = rng.random((B, g + 1)).astype(np.float32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    got = gu.rapid().rapid_accept(dev(zt), dev(zd), dev(tok), cfg.eta, dev(u), gammas=dev(seqs.gammas),
                                  target_stats=st_dev(st))
    torch.cuda.synchronize()
    ref = oracle.accept(zt, zd, tok, u, eta=cfg.eta, gammas=seqs.gammas)
    res = gu.compare_accept(tuple(x.cpu().numpy() for x in got), ref, seqs.gammas, g)
    assert res["n_mismatch"] == 0 and res["token_mismatch"] == 0 and res["exempt_sequences"] == 0, res
    assert res["max_ratio_rel_err"] < 1e-4, res


@pytest.mark.parametrize("V,chunk", [(20000, 16), (20000, 48), (5000, 16), (128256, 512), (4097, 4097)])
@pytest.mark.parametrize("sides", ["both", "target", "draft"])
def test_accept_with_statistics_over_any_partition(V, chunk, sides):
    """rapid_accept_prestats takes the (max, sum exp) pairs of any partition of the vocabulary: here partitions
    of 1 to 1250 chunks per row (more chunks than a workgroup has threads included), written by the oracle's
    chunk statistics from the logits, for both rows, the target rows only and the draft rows only; a batch with
    different draft counts; against the oracle's accept on the same logits."""
    B, g, T = 3, 5, 0.7
    rng = np.random.default_rng(V + chunk)
    zt = (rng.standard_normal((B, g + 1, V)) * 3).astype(np.float32)
    zd = (zt[:, :g] + rng.standard_normal((B, g, V))).astype(np.float32)
    tok = np.argmax(zd.astype(np.float64) / T + rng.gumbel(size=zd.shape), -1).astype(np.int32)
    u = rng.random((B, g + 1)).astype(np.float32)
    gammas = np.array([5, 2, 0], dtype=np.int32)

    def stats(z):
        cmax, csum = oracle.chunk_stats(z.reshape(-1, V).astype(np.float64), chunk, T)
        return st_dev(np.stack([cmax, csum], -1))

    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    kw = {}
    if sides in ("both", "target"):
        kw["target_stats"] = stats(zt)
    if sides in ("both", "draft"):
        kw["draft_stats"] = stats(zd)
    got = gu.rapid().rapid_accept(dev(zt), dev(zd), dev(tok), 2.0, dev(u), gammas=dev(gammas), temperature=T, **kw)
    torch.cuda.synchronize()
    ref = oracle.accept(zt, zd, tok, u, eta=2.0, temperature=T, gammas=gammas)
    res = gu.compare_accept(tuple(x.cpu().numpy() for x in got), ref, gammas, g)
    assert res["n_mismatch"] == 0 and res["token_mismatch"] == 0 and res["exempt_sequences"] == 0, res
    assert res["max_ratio_rel_err"] < 1e-4, res


def st_dev(st):
    return torch.from_numpy(st.astype(np.float32)).cuda().contiguous()
