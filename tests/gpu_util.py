"""Helpers shared by the GPU parity tests: upload seeded inputs, call the C-ABI
binding, run the float64 oracle on the same inputs, compare."""
import numpy as np
import torch

import oracle
from paper_2502_20330_amd import binding
from paper_2502_20330_amd import workloads as wl

ATOL, RTOL = 2e-2, 1e-2          # |gpu - ref| <= ATOL + RTOL*|ref| (bf16 in, fp32 accumulate, bf16 out)
ACCEPT_TIE = 1e-5                # |min(1, ratio) - u| below this: accept decision may differ
# Normalised CDF-edge margin below which the drawn token may differ.  The device forms the draw weights
# of the one row it draws from entirely in float64 (exponentials, normalisers, running sums), as the
# oracle does; the two differ by summation order and by the last bits of the exponential only:
# <= V * 2^-52 ~ 3e-11 at V = 128256 in the worst case, ~1e-13 typically.  1e-10 is orders of magnitude
# below the width of any token's interval that a float32 uniform can resolve, so no token is exempt by
# construction; every seeded test asserts that the exemption was not used at all.
DRAW_TIE = 1e-10

_rapid = None


def rapid():
    global _rapid
    if _rapid is None:
        _rapid = binding.Rapid(0)
    return _rapid


def bf16_to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_host(t: torch.Tensor) -> np.ndarray:
    return wl.bf16_bits_to_f32(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)


def run_attn_case(cfg, inp, *, chunk_tokens=0, scale=None, want_lse=True, head_major=False, kv_interleaved=False):
    """Runs GPU and oracle on one AttnInputs; returns (gpu_out f64, ref f64, gpu_lse, ref_lse).
    head_major: the GPU sees the same cache re-stored in [B, Hkv, L, d] memory order.
    kv_interleaved: K and V in ONE allocation [B, Hkv, L, 2, d] (or [B, L, Hkv, 2, d]): the K row and the V row
    of a (token, head) are adjacent, v = k + d elements, and both are addressed with the same strides."""
    s = inp.seqs
    scale = cfg.softmax_scale if scale is None else scale
    q, k, v = bf16_to_dev(inp.q), bf16_to_dev(inp.k), bf16_to_dev(inp.v)
    if kv_interleaved:
        kv = torch.stack([k, v], dim=3)                                     # [B or pages, tokens, Hkv, 2, d]
        if head_major:
            kv = kv.permute(0, 2, 1, 3, 4).contiguous().permute(0, 2, 1, 3, 4)
        k, v = kv[:, :, :, 0, :], kv[:, :, :, 1, :]
        assert k.stride() == v.stride() and v.data_ptr() - k.data_ptr() == 2 * cfg.head_dim
    elif head_major:
        k = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        v = v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    ctx = torch.from_numpy(s.ctx_lens).cuda()
    gam = torch.from_numpy(s.gammas).cuda()
    pt = torch.from_numpy(s.page_table).cuda() if s.page_table is not None else None
    lse = torch.full((cfg.batch, cfg.n_q_heads, cfg.q_max), float("nan"), dtype=torch.float32, device="cuda")
    out = rapid().rapid_verify_attn(q, k, v, ctx, gammas=gam, page_table=pt, max_ctx=s.max_ctx,
                                    softmax_scale=scale, chunk_tokens=chunk_tokens,
                                    lse_out=lse if want_lse else None)
    torch.cuda.synchronize()
    bs, ts, hs, ps = wl.kv_strides(cfg, s)
    lay = oracle.KVLayout(bs, ts, hs, cfg.page_size if cfg.paged else 0, ps,
                          s.page_table.shape[1] if s.page_table is not None else 0)
    ref, ref_lse = oracle.verify_attn(inp.q, inp.k, inp.v, s.ctx_lens, lay, Hkv=cfg.n_kv_heads, scale=scale,
                                      gammas=s.gammas, page_table=s.page_table, want_lse=True)
    return bf16_to_host(out), ref, lse.cpu().numpy().astype(np.float64), ref_lse


def assert_attn_close(got, ref, what=""):
    err = np.abs(got - ref)
    bound = ATOL + RTOL * np.abs(ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    rel = err / np.maximum(np.abs(ref), 1e-30)
    big = np.abs(ref) > 1e-2
    msg = (f"{what}: max abs err {err.max():.3e}, max rel err (|ref|>1e-2) "
           f"{rel[big].max() if big.any() else 0:.3e}, worst at {worst}: got {got[worst]:.6f} ref {ref[worst]:.6f}")
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    assert np.all(err <= bound), msg
    # the same bound with its absolute part scaled to the size of the outputs, so
    # that near-uniform attention (|out| ~ 1e-2) is not passed by atol alone
    tight = ATOL * min(1.0, float(np.abs(ref).max())) + RTOL * np.abs(ref)
    assert np.all(err <= tight), "scaled-atol check, " + msg
    return err.max(), (rel[big].max() if big.any() else 0.0)


def run_accept_case(acc, *, eta, temperature=1.0, tail_alpha=0.1, use_gammas=True):
    """Runs GPU and oracle accept on AcceptInputs; returns (gpu tuple on host, oracle result)."""
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    gam = acc.gammas if use_gammas else None
    n, toks, ratio = rapid().rapid_accept(dev(acc.target_logits), dev(acc.draft_logits), dev(acc.draft_tokens),
                                          float(eta), dev(acc.uniforms),
                                          gammas=dev(gam) if gam is not None else None,
                                          temperature=float(temperature), tail_alpha=float(tail_alpha))
    torch.cuda.synchronize()
    if temperature == 0:                 # the greedy limit has its own statement in the oracle
        ref = oracle.accept_greedy(acc.target_logits, acc.draft_logits, acc.draft_tokens, acc.uniforms, gammas=gam)
    else:
        ref = oracle.accept(acc.target_logits, acc.draft_logits, acc.draft_tokens, acc.uniforms,
                            eta=float(np.float32(eta)), temperature=float(np.float32(temperature)),
                            tail_alpha=float(np.float32(tail_alpha)), gammas=gam)
    return (n.cpu().numpy(), toks.cpu().numpy(), ratio.cpu().numpy() if ratio is not None else None), ref


def compare_accept(gpu, ref, gammas, gmax):
    """Bit-exact comparison of accepted-prefix length and emitted tokens, exempting
    (and counting) sequences whose decisive accept test or draw is a near-tie in
    the oracle's float64 margins.  Returns a dict of counts."""
    n_g, tok_g, ratio_g = gpu
    B = len(n_g)
    stats = dict(sequences=B, n_mismatch=0, token_mismatch=0, accept_near_ties=0, draw_near_ties=0,
                 exempt_sequences=0, max_ratio_rel_err=0.0)
    for b in range(B):
        g = int(gammas[b]) if gammas is not None else gmax
        near_accept = bool(np.any(ref.accept_margin[b, :g] <= ACCEPT_TIE))
        near_draw = bool(ref.draw_margin[b] <= DRAW_TIE)
        stats["accept_near_ties"] += int(np.sum(ref.accept_margin[b, :g] <= ACCEPT_TIE))
        stats["draw_near_ties"] += int(near_draw)
        if ratio_g is not None and g > 0:
            r, rr = ratio_g[b, :g].astype(np.float64), ref.ratio[b, :g]
            assert np.array_equal(np.isinf(r), np.isinf(rr)), "infinite ratios must agree"
            ok = np.isfinite(rr) & (rr > 1e-30)
            if ok.any():
                stats["max_ratio_rel_err"] = max(stats["max_ratio_rel_err"],
                                                 float(np.max(np.abs(r[ok] - rr[ok]) / rr[ok])))
        same_n = int(n_g[b]) == int(ref.n_accepted[b])
        same_tok = np.array_equal(tok_g[b], ref.out_tokens[b])
        if same_n and same_tok:
            continue
        if (not same_n and near_accept) or (same_n and near_draw):
            stats["exempt_sequences"] += 1
            continue
        if not same_n:
            stats["n_mismatch"] += 1
        else:
            stats["token_mismatch"] += 1
    return stats
