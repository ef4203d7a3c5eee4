"""GPU parity: rapid_verify_attn (C ABI, gfx950 kernels) against the float64 oracle,
element by element, on seeded inputs that span several tiles, several KV splits
and ragged tails.  Tolerance: |gpu - ref| <= 2e-2 + 1e-2*|ref| (bf16 in, fp32
accumulate, bf16 out); max abs / max rel errors are printed."""
import math

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


def check(cfg, inp=None, what="", **kw):
    inp = inp or wl.gen_attn_inputs(cfg)
    got, ref, lse, ref_lse = gu.run_attn_case(cfg, inp, **kw)
    s = inp.seqs
    e_abs, e_rel = gu.assert_attn_close(got, ref, what or cfg.name)
    for b in range(cfg.batch):
        Q = int(s.gammas[b]) + 1
        assert np.all(got[b, Q:] == 0.0), "padded query rows must be zero"
        np.testing.assert_allclose(lse[b, :, :Q], ref_lse[b, :, :Q], rtol=2e-3, atol=2e-3)
    print(f"[{what or cfg.name}] max_abs={e_abs:.3e} max_rel={e_rel:.3e}")
    return got, ref


def test_tiny_config():
    check(wl.CONFIGS["tiny"])


@pytest.mark.parametrize("L", [5, 6, 31, 32, 33, 37, 127, 128, 129, 160, 511, 512, 513, 1000])
def test_tile_and_split_edges(L):
    cfg = wl.scaled(wl.CONFIGS["tiny"], ctx=(L, L), name=f"edge_L{L}")
    check(cfg, chunk_tokens=128)


@pytest.mark.parametrize("chunk", [0, 128, 256, 640, 4096])
def test_split_count_does_not_change_result(chunk):
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], ctx=(4133, 4133), name=f"l8b_4133_chunk{chunk}")
    check(cfg, chunk_tokens=chunk)


def test_peaked_softmax_unscaled_keys():
    # K not pre-scaled: scores have std ~1 after 1/sqrt(d), softmax is far from uniform
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], ctx=(3000, 3000), k_scale=1.0, name="peaked")
    got, ref = check(cfg)
    assert np.abs(ref).max() > 0.1


def test_sharp_softmax_large_scale():
    cfg = wl.scaled(wl.CONFIGS["tiny"], ctx=(700, 700), name="sharp")
    check(cfg, scale=1.0)            # scores N(0, 64): one key dominates most rows


def test_needle_key():
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], ctx=(2500, 2500), name="needle")
    inp = wl.gen_attn_inputs(cfg)
    qf = wl.bf16_bits_to_f32(inp.q)
    # key 1234 of kv head 3 is aligned with query (pos 2, head 13): score +~20 after scaling
    qv = qf[0, 2, 13]
    target = qv * np.float32(20.0 * math.sqrt(128) / float(qv @ qv))
    inp.k[0, 1234, 3] = wl.f32_to_bf16_bits(target)
    got, ref = check(cfg, inp)
    vf = wl.bf16_bits_to_f32(inp.v)[0, 1234, 3]
    assert np.abs(ref[0, 2, 13] - vf).max() < 0.1


@pytest.mark.parametrize("hq,hkv,gam", [(64, 8, 8), (8, 8, 8), (16, 8, 4), (24, 8, 2), (8, 1, 9), (4, 4, 0), (32, 8, 10),
                                        (56, 8, 10), (28, 4, 8), (28, 4, 10)])
def test_group_sizes_and_gammas(hq, hkv, gam):
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], n_q_heads=hq, n_kv_heads=hkv, gamma_choices=(gam,),
                    ctx=(1300, 1300), name=f"g{hq // hkv}_gamma{gam}")
    check(cfg, chunk_tokens=512)


@pytest.mark.parametrize("L", [12, 40, 129, 300, 1023, 1024, 1025, 2500, 4133])
@pytest.mark.parametrize("gam,group", [(10, 8), (8, 8), (11, 8), (9, 7)])
def test_wide_row_counts_two_row_teams(L, gam, group):
    """65..96 packed rows run on the eight-wave kernel (two row teams per KV ring).  gamma = 10 with group
    size 8 is the paper's setting for its 70B / 72B targets (88 rows).  Lengths from fewer tokens than one
    tile per token quarter up to several splits, so that whole quarters of a split are empty."""
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], n_q_heads=2 * group, n_kv_heads=2, gamma_choices=(gam,),
                    ctx=(L, L), name=f"wide_g{group}_gamma{gam}_L{L}")
    check(cfg, chunk_tokens=1024 if L > 1024 else 0)


def test_wide_row_counts_layouts_and_ragged_batches():
    base = dict(n_q_heads=16, n_kv_heads=2, name="wide_layouts")
    # ragged batch, per-sequence gamma (some sequences have far fewer rows than the kernel is sized for)
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=3, ctx=(700, 5000), gamma_choices=(10, 3), **base)
    inp = wl.gen_attn_inputs(cfg, layer=3)
    check(cfg, inp, chunk_tokens=640)
    check(cfg, inp, chunk_tokens=640, head_major=True, what="wide head-major")
    # paged cache, head_dim 64, peaked softmax (unscaled keys)
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=2, ctx=(900, 3000), gamma_choices=(10,), paged=True, k_scale=1.0, **base)
    check(cfg, chunk_tokens=512, what="wide paged peaked")
    cfg = wl.scaled(wl.CONFIGS["tiny"], n_q_heads=24, n_kv_heads=3, ctx=(3000, 3000), gamma_choices=(10,), name="wide_d64")
    check(cfg, chunk_tokens=1024)
    # five row blocks (teams of 3 + 2 blocks): paged, ragged with per-sequence gamma, head-major pages, head_dim 64
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=3, ctx=(600, 4000), gamma_choices=(8, 2), paged=True, **base)
    inp = wl.gen_attn_inputs(cfg, layer=5)
    check(cfg, inp, chunk_tokens=512, what="3+2 paged ragged")
    check(cfg, inp, chunk_tokens=512, head_major=True, what="3+2 paged head-major")
    cfg = wl.scaled(wl.CONFIGS["tiny"], n_q_heads=21, n_kv_heads=3, ctx=(2900, 2900), gamma_choices=(10,), name="wide_d64_77rows")
    check(cfg, chunk_tokens=1024)
    cfg = wl.scaled(wl.CONFIGS["tiny"], n_q_heads=21, n_kv_heads=3, batch=2, ctx=(100, 1500), gamma_choices=(10, 9), paged=True,
                    name="wide_d64_77rows_paged")
    check(cfg, chunk_tokens=256)


def test_head_dim_64_multi_split():
    cfg = wl.scaled(wl.CONFIGS["tiny"], n_q_heads=16, n_kv_heads=4, ctx=(5000, 5000), name="d64")
    check(cfg, chunk_tokens=1024)


def test_ragged_batch_contiguous():
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], paged=False, batch=5, ctx=(200, 3000), name="ragged_contig")
    check(cfg, chunk_tokens=512)


def test_ragged_batch_paged():
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=6, ctx=(100, 3500), name="ragged_paged_small")
    inp = wl.gen_attn_inputs(cfg)
    assert len(set(inp.seqs.gammas.tolist())) > 1
    check(cfg, inp, chunk_tokens=512)


def test_paged_page_size_64():
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=3, ctx=(900, 2000), page_size=64, name="paged64")
    check(cfg, chunk_tokens=256)


def test_head_major_cache_strides():
    """Same data in a [B, Hkv, L, d] cache: only the strides differ."""
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], ctx=(1500, 1500), name="head_major")
    inp = wl.gen_attn_inputs(cfg)
    q, k, v = (gu.bf16_to_dev(x) for x in (inp.q, inp.k, inp.v))
    ctx = torch.from_numpy(inp.seqs.ctx_lens).cuda()
    base = gu.rapid().rapid_verify_attn(q, k, v, ctx, softmax_scale=cfg.softmax_scale)
    kh = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    vh = v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert kh.stride() != k.stride()
    alt = gu.rapid().rapid_verify_attn(q, kh, vh, ctx, softmax_scale=cfg.softmax_scale)
    torch.cuda.synchronize()
    assert torch.equal(base, alt)


@pytest.mark.parametrize("head_major", [False, True])
def test_k_and_v_rows_interleaved_in_one_allocation(head_major):
    """K and V of a (token, head) next to each other in one tensor, [B, Hkv, L, 2, d] or [B, L, Hkv, 2, d]: the
    same entry point through its strides (v = k + d elements).  Contiguous and paged, narrow and wide row
    counts, several splits; against the oracle."""
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=2, ctx=(900, 5000), n_q_heads=8, n_kv_heads=2, name="kv_interleaved")
    check(cfg, chunk_tokens=1024, head_major=head_major, kv_interleaved=True)
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=2, ctx=(300, 3000), n_q_heads=16, n_kv_heads=2, gamma_choices=(8, 3),
                    paged=True, name="kv_interleaved_paged_wide")
    check(cfg, chunk_tokens=512, head_major=head_major, kv_interleaved=True)
    cfg = wl.scaled(wl.CONFIGS["tiny"], ctx=(2000, 2000), n_q_heads=8, n_kv_heads=4, name="kv_interleaved_d64")
    check(cfg, chunk_tokens=0, head_major=head_major, kv_interleaved=True)


@pytest.mark.parametrize("L", [1919, 1920, 1921, 2048, 2175, 2176, 2177, 4095, 4097, 6015, 6016, 6017, 6271, 6273, 8192])
def test_head_major_uneven_split_pairs(L):
    """[B, Hkv, L, d] cache with one workgroup per compute unit or fewer: the library then
    rotates heads over dispatch slots and gives the two splits of a pair 2048 +- 128
    tokens.  Context lengths sit on and around every boundary that this produces."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], ctx=(L, L), n_q_heads=8, n_kv_heads=2, name=f"hm_pairs_L{L}")
    check(cfg, chunk_tokens=2048, head_major=True)


def test_head_major_uneven_split_pairs_ragged_batch():
    """Same, three sequences of different lengths under one max_ctx: some splits of the
    shorter sequences are empty and the merge must count the non-empty ones per head."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], batch=3, ctx=(1800, 10500), n_q_heads=16, n_kv_heads=4, head_dim=128,
                    name="hm_pairs_ragged")
    inp = wl.gen_attn_inputs(cfg)
    assert len(set(inp.seqs.ctx_lens.tolist())) == 3
    check(cfg, inp, chunk_tokens=2048, head_major=True)


def test_cache_rows_past_ctx_len_are_never_used():
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], ctx=(1111, 1111), name="tail_nan")
    inp = wl.gen_attn_inputs(cfg)
    q, k, v = (gu.bf16_to_dev(x) for x in (inp.q, inp.k, inp.v))
    pad = torch.full((1, 300, 8, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    k2, v2 = torch.cat([k, pad], 1), torch.cat([v, pad], 1)
    ctx = torch.from_numpy(inp.seqs.ctx_lens).cuda()
    a = gu.rapid().rapid_verify_attn(q, k, v, ctx, softmax_scale=cfg.softmax_scale, chunk_tokens=512)
    b = gu.rapid().rapid_verify_attn(q, k2, v2, ctx, softmax_scale=cfg.softmax_scale, chunk_tokens=512)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.isfinite(b.float()).all()


def test_repeat_calls_are_bitwise_identical():
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], ctx=(6000, 6000), name="determinism")
    inp = wl.gen_attn_inputs(cfg)
    q, k, v = (gu.bf16_to_dev(x) for x in (inp.q, inp.k, inp.v))
    ctx = torch.from_numpy(inp.seqs.ctx_lens).cuda()
    outs = [gu.rapid().rapid_verify_attn(q, k, v, ctx, softmax_scale=cfg.softmax_scale).clone() for _ in range(3)]
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_bad_arguments_return_error_codes():
    from paper_2502_20330_amd import binding
    r = gu.rapid()
    q = torch.zeros(1, 2, 4, 128, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, 64, 1, 128, dtype=torch.bfloat16, device="cuda")
    ctx = torch.tensor([64], dtype=torch.int32, device="cuda")
    with pytest.raises(binding.RapidError) as e:       # head_dim 96
        r.rapid_verify_attn(q[..., :96].contiguous(), k[..., :96].contiguous(), k[..., :96].contiguous(), ctx)
    assert e.value.status == -3
    q104 = torch.zeros(1, 13, 8, 128, dtype=torch.bfloat16, device="cuda")   # 13*8 = 104 packed rows > 96
    with pytest.raises(binding.RapidError) as e:
        r.rapid_verify_attn(q104, k, k, ctx)
    assert e.value.status == -3
    with pytest.raises(binding.RapidError) as e:       # scale <= 0
        r.rapid_verify_attn(q, k, k, ctx, softmax_scale=0.0)
    assert e.value.status == -1
    with pytest.raises(binding.RapidError) as e:       # misaligned cache pointer
        flat = torch.zeros(64 * 128 + 8, dtype=torch.bfloat16, device="cuda")
        r.rapid_verify_attn(q, flat[1:1 + 64 * 128].view(1, 64, 1, 128), flat[1:1 + 64 * 128].view(1, 64, 1, 128), ctx)
    assert e.value.status == -2


# ---------------------------------------------------------------- full benchmark sizes
def test_llama8b_32k_full_size():
    """Config 2 at its real size, every output element against the oracle."""
    check(wl.CONFIGS["llama8b_32k"])


def test_llama8b_128k_layers_full_size():
    """Config 3 shape (L = 131072) in the launch configuration the benchmark times:
    two of the 32 layers (first and last seed), every output element."""
    cfg = wl.CONFIGS["llama8b_128k_step"]
    for layer in (0, cfg.layers - 1):
        inp = wl.gen_attn_inputs(cfg, layer=layer)
        check(cfg, inp, what=f"{cfg.name}[layer {layer}]")


@pytest.mark.parametrize("layer", [0, 10, 21, 31])
def test_llama8b_128k_head_major_full_size(layer):
    """Config 3 shape with the cache in [B, Hkv, L, d] memory order, exactly the launch configuration the
    benchmark times by default (one workgroup per compute unit, rotated heads, uneven split pairs): four of
    the 32 layers including the first and the last, every output element against the oracle."""
    cfg = wl.CONFIGS["llama8b_128k_step"]
    inp = wl.gen_attn_inputs(cfg, layer=layer)
    check(cfg, inp, what=f"{cfg.name}[layer {layer}, head-major]", head_major=True)


def test_ragged_paged_full_size():
    """Config 4 at its real size: 8 sequences of 16K-128K tokens, gamma in {4,6,8}, 16-token
    pages with a seeded random page table; every output element against the oracle."""
    cfg = wl.CONFIGS["ragged_paged"]
    inp = wl.gen_attn_inputs(cfg)
    assert inp.seqs.ctx_lens.min() >= 16384 and inp.seqs.ctx_lens.max() <= 131072
    check(cfg, inp, what=f"{cfg.name} sum_ctx={int(inp.seqs.ctx_lens.sum())}")


def test_ragged_paged_head_major_pages():
    """Pages stored [n_pages, Hkv, 16, d] (each (page, head) 4 KiB contiguous), small sizes."""
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=4, ctx=(500, 5000), name="paged_head_major")
    inp = wl.gen_attn_inputs(cfg)
    s = inp.seqs
    q, k, v = (gu.bf16_to_dev(x) for x in (inp.q, inp.k, inp.v))
    kh = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    vh = v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    args = dict(gammas=torch.from_numpy(s.gammas).cuda(), page_table=torch.from_numpy(s.page_table).cuda(),
                max_ctx=s.max_ctx, softmax_scale=cfg.softmax_scale, chunk_tokens=512)
    ctx = torch.from_numpy(s.ctx_lens).cuda()
    a = gu.rapid().rapid_verify_attn(q, k, v, ctx, **args).clone()
    b = gu.rapid().rapid_verify_attn(q, kh, vh, ctx, **args)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_llama70b_128k_layer_full_size():
    """Config 5 shape (64 query heads, group 8 -> 72 packed rows), one layer."""
    cfg = wl.CONFIGS["llama70b_128k_step"]
    check(cfg, wl.gen_attn_inputs(cfg, layer=0), what=f"{cfg.name}[layer 0]")


@pytest.mark.parametrize("head_major", [False, True])
def test_paper_setting_gamma_10_group_8_at_128k_full_size(head_major):
    """gamma = 10 (Sec. 3, implementation details) on the 70B / 72B head shape (64 query / 8 kv heads):
    88 packed rows, 128K tokens, one layer, both cache orders, in the launch configuration of the benchmark."""
    cfg = wl.scaled(wl.CONFIGS["llama70b_128k_step"], gamma_choices=(10,), name="llama70b_gamma10_128k")
    check(cfg, wl.gen_attn_inputs(cfg, layer=1), what=f"{cfg.name}[head_major={head_major}]", head_major=head_major)


@pytest.mark.parametrize("paged", [False, True])
def test_caches_beyond_4_gib(paged):
    """A cache allocation of 5.4 GB per tensor: sequence and page bases lie past 2^32 bytes, so every base has
    to be formed in 64 bits (only offsets inside one sequence or page may be 32-bit).  The sequences themselves
    are short, so the host fills and the oracle reads only the tokens in use: contiguous, 40 sequences with
    room for 131072 tokens each; paged, a pool of 163840 pages of 16 tokens of which the table uses the last ones."""
    rng = np.random.default_rng(77)
    B, Hq, Hkv, d, Q = 40, 8, 4, 128, 3
    lens = rng.integers(300, 1000, size=B).astype(np.int32)
    lens[-1] = 999
    cap = 131072
    tok = Hkv * d
    n_used = 1008                                             # tokens per sequence that exist on the host
    kh = wl._normal_bf16(rng, (B, n_used, Hkv, d))
    vh = wl._normal_bf16(rng, (B, n_used, Hkv, d))
    qh = wl._normal_bf16(rng, (B, Q, Hq, d))
    q = gu.bf16_to_dev(qh)
    ctx = torch.from_numpy(lens).cuda()
    if not paged:
        k = torch.empty((B, cap, Hkv, d), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        assert k.numel() * 2 > (1 << 32)
        k[:, :n_used] = gu.bf16_to_dev(kh)
        v[:, :n_used] = gu.bf16_to_dev(vh)
        out = gu.rapid().rapid_verify_attn(q, k, v, ctx, gamma=Q - 1, max_ctx=n_used, softmax_scale=0.2)
        pt_host = None
        lay = gu.oracle.KVLayout(n_used * tok, tok, d, 0, 0, 0)
        kk, vv = kh, vh
    else:
        page, n_pages = 16, B * cap // 16
        per_seq = n_used // page                              # 63 pages per sequence
        k = torch.empty((n_pages, page, Hkv, d), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        # sequence b uses the pages n_pages - 1 - (b * per_seq + j): the top of the pool, bases past 4 GiB
        pt_host = (n_pages - 1 - (np.arange(B)[:, None] * per_seq + np.arange(per_seq)[None, :])).astype(np.int32)
        assert int(pt_host.min()) * page * tok * 2 > (1 << 32)
        idx = torch.from_numpy(pt_host.reshape(-1).astype(np.int64)).cuda()
        k[idx] = gu.bf16_to_dev(kh).reshape(B * per_seq, page, Hkv, d)
        v[idx] = gu.bf16_to_dev(vh).reshape(B * per_seq, page, Hkv, d)
        out = gu.rapid().rapid_verify_attn(q, k, v, ctx, gamma=Q - 1, page_table=torch.from_numpy(pt_host).cuda(),
                                           max_ctx=n_used, softmax_scale=0.2)
        # the oracle sees a compact pool holding the same pages in table order
        kk = kh.reshape(B * per_seq, page, Hkv, d)
        vv = vh.reshape(B * per_seq, page, Hkv, d)
        pt_compact = np.arange(B * per_seq, dtype=np.int32).reshape(B, per_seq)
        lay = gu.oracle.KVLayout(0, tok, d, page, page * tok, per_seq)
    torch.cuda.synchronize()
    ref = gu.oracle.verify_attn(qh, kk, vv, lens, lay, Hkv=Hkv, scale=0.2, gammas=None,
                             page_table=None if not paged else pt_compact, gamma=Q - 1)
    ref = ref[0] if isinstance(ref, tuple) else ref
    gu.assert_attn_close(gu.bf16_to_host(out), ref, what=f"cache beyond 4 GiB, paged={paged}")
    del k, v
    torch.cuda.empty_cache()


def test_hbm_read_probe_runs_and_checks_arguments():
    """The measurement aid streams a buffer without touching it and rejects sizes it cannot split."""
    from paper_2502_20330_amd import binding
    r = gu.rapid()
    buf = torch.arange(3 * 16384 * 50 + 100, dtype=torch.uint8, device="cuda")
    before = buf.clone()
    n = r.rapid_hbm_read_probe(buf)
    torch.cuda.synchronize()
    assert n == 3 * 16384 * 50 and torch.equal(buf, before)
    assert r.rapid_hbm_read_probe(buf, 16384) == 16384           # fewer blocks than waves
    torch.cuda.synchronize()
    import ctypes
    bad = r.lib.rapid_hbm_read_probe(r._ctx, ctypes.c_void_p(buf.data_ptr()), 1000, None, None)
    assert bad == binding.RAPID_EINVAL
    # Every 16 KiB block is looked at by some wave, also with uneven shares per workgroup pair: the kernel
    # writes `sink` when the XOR of the words a lane inspects (word `lane` of each block) is one constant,
    # so a buffer of zeros with that constant planted in one block must set it.
    magic = 0x9E3779B9
    for skew in (0, 3, 16):
        r.set_option(binding.OPT_PROBE_SKEW, skew)
        for nblock in (150, 5000):
            z = torch.zeros(nblock * 16384 // 4, dtype=torch.int32, device="cuda")
            sink = torch.zeros(1, dtype=torch.int32, device="cuda")
            rng = np.random.default_rng(nblock + skew)
            picks = [0, nblock - 1] + [int(x) for x in rng.integers(0, nblock, 24)]
            for blk in picks:
                lane = int(rng.integers(0, 64))
                z[blk * 4096 + lane] = magic - (1 << 32)
                sink.zero_()
                rc = r.lib.rapid_hbm_read_probe(r._ctx, ctypes.c_void_p(z.data_ptr()), nblock * 16384,
                                                ctypes.c_void_p(sink.data_ptr()), None)
                assert rc == 0
                torch.cuda.synchronize()
                assert int(sink.item()) & 0xFFFFFFFF == magic, (skew, nblock, blk, lane)
                z[blk * 4096 + lane] = 0
    r.set_option(binding.OPT_PROBE_SKEW, 0)
    assert r.lib.rapid_set_option(r._ctx, binding.OPT_PROBE_SKEW, 17) == binding.RAPID_EINVAL


@pytest.mark.parametrize("name", ["drafter_decode_8k", "drafter_decode_16k_b8"])
def test_drafter_decode_step_full_size(name):
    """The drafter's decode step on the retrieved context (Sec. 2.2): one query position per
    sequence (gamma = 0, 4 packed rows per kv head), 8K tokens / a ragged batch of 4K-16K tokens,
    two layers, in both cache orders; every output element against the oracle."""
    cfg = wl.CONFIGS[name]
    for layer in (0, cfg.layers - 1):
        inp = wl.gen_attn_inputs(cfg, layer=layer)
        assert int(inp.seqs.gammas.max()) == 0
        check(cfg, inp, what=f"{name}[layer {layer}]")
        check(cfg, inp, what=f"{name}[layer {layer}, head-major]", head_major=True)


def test_paper_gamma_10_at_32k():
    """The paper's own setting of gamma = 10 drafts per round (Sec. 3, implementation details): 11 query
    positions x 4 heads = 44 packed rows per kv head, LLaMA-3.1-8B shape at 32K tokens, both cache orders."""
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], gamma_choices=(10,), name="gamma10_32k")
    inp = wl.gen_attn_inputs(cfg)
    check(cfg, inp)
    check(cfg, inp, head_major=True, what="gamma10_32k head-major")


def test_ctx_sum_hint_changes_the_plan_not_the_result():
    """A ragged batch with and without the caller's sum-of-lengths hint: different KV splits, both within
    tolerance of the oracle."""
    cfg = wl.scaled(wl.CONFIGS["ragged_paged"], batch=6, ctx=(200, 20000), paged=False, name="hint")
    inp = wl.gen_attn_inputs(cfg)
    s = inp.seqs
    q, k, v = (gu.bf16_to_dev(x) for x in (inp.q, inp.k, inp.v))
    ctx, gam = torch.from_numpy(s.ctx_lens).cuda(), torch.from_numpy(s.gammas).cuda()
    r = gu.rapid()
    hint = int(s.ctx_lens.astype(np.int64).sum())
    plain = r.attn_shape(q, k, s.max_ctx)
    hinted = r.attn_shape(q, k, s.max_ctx, ctx_sum_hint=hint)
    assert r.verify_attn_chunk(hinted) < r.verify_attn_chunk(plain)
    import oracle
    bs, ts, hs, ps = wl.kv_strides(cfg, s)
    ref = oracle.verify_attn(inp.q, inp.k, inp.v, s.ctx_lens, oracle.KVLayout(bs, ts, hs), Hkv=cfg.n_kv_heads,
                             scale=cfg.softmax_scale, gammas=s.gammas)
    for h in (0, hint):
        out = r.rapid_verify_attn(q, k, v, ctx, gammas=gam, max_ctx=s.max_ctx, softmax_scale=cfg.softmax_scale,
                                  ctx_sum_hint=h)
        torch.cuda.synchronize()
        gu.assert_attn_close(gu.bf16_to_host(out), ref, f"hint={h}")


def test_out_of_range_device_values_are_clamped():
    """ctx_lens and gammas are device data the host cannot validate: values outside their ranges are clamped
    (gamma_b to [0, Qmax-1], ctx_lens[b] to max_ctx) instead of steering any access out of bounds, and a
    sequence of length 0 yields zeros.  The valid sequences of the same batch are unaffected."""
    cfg = wl.scaled(wl.CONFIGS["llama8b_32k"], batch=4, ctx=(900, 900), gamma_choices=(3,), name="clamp")
    inp = wl.gen_attn_inputs(cfg)
    s = inp.seqs
    q, k, v = (gu.bf16_to_dev(x) for x in (inp.q, inp.k, inp.v))
    bad_ctx = np.array([900, 900, 900 + 5000, 0], dtype=np.int32)
    bad_gam = np.array([3, 99, -7, 3], dtype=np.int32)
    out = gu.rapid().rapid_verify_attn(q, k, v, torch.from_numpy(bad_ctx).cuda(), gammas=torch.from_numpy(bad_gam).cuda(),
                                       max_ctx=900, softmax_scale=cfg.softmax_scale)
    torch.cuda.synchronize()
    got = gu.bf16_to_host(out)
    assert np.all(np.isfinite(got))
    import oracle
    bs, ts, hs, ps = wl.kv_strides(cfg, s)
    eff_ctx = np.array([900, 900, 900, 900], dtype=np.int32)
    eff_gam = np.array([3, cfg.q_max - 1, 0, 3], dtype=np.int32)
    ref = oracle.verify_attn(inp.q, inp.k, inp.v, eff_ctx, oracle.KVLayout(bs, ts, hs), Hkv=cfg.n_kv_heads,
                             scale=cfg.softmax_scale, gammas=eff_gam)
    gu.assert_attn_close(got[:3], ref[:3], "clamped sequences")
    assert np.all(got[3] == 0.0)
