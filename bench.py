#!/usr/bin/env python3
"""Benchmark of the RAPID verification step on one MI355X.

One step = the whole hot path over one batch of synthetic input: verify attention
of all layers of the workload (each layer has its own bf16 KV cache resident in
HBM) followed by one accept/resample pass over the full vocabulary.

Default workload: the Llama-3-8B-shaped full verify step at 128K context,
gamma = 8 (32 layers, 32 query / 8 kv heads, head_dim 128, vocabulary 128256),
the configuration the headline metric is quoted on.  Prints ONE JSON line:
`value` is the effective KV GB/s of the whole step, `verify_step_us` its latency and
`hbm_frac_of_peak` the fraction of the 8 TB/s HBM peak (the three parts of the metric).
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X published HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_128k_step")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = the workload's)")
    ap.add_argument("--chunk-tokens", type=int, default=0, help="KV split size override (0 = library's choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=8, help="layers of attention the oracle is timed on")
    ap.add_argument("--kv-layout", choices=["head-major", "token-major", "head-major-kv-interleaved"], default="head-major",
                    help="KV cache memory order: [B,Hkv,L,d] (default, the layout the library prefers) or "
                         "[B,L,Hkv,d]; paged: [pages,Hkv,page,d] or [pages,page,Hkv,d]; head-major-kv-interleaved: K and V "
                         "in one tensor [B,Hkv,L,2,d] / [pages,Hkv,page,2,d], the two rows of a (token, head) adjacent")
    ap.add_argument("--with-lm-head", action="store_true",
                    help="also run the target's output head (hidden x vocab bf16 weights) inside every step and feed "
                         "its logits and row statistics to the accept pass (batch 1 workloads)")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the short extra measurements of the other 128K configurations (the `also` object)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for rocprofv3 byte counters)")
    return ap.parse_args()


TRAFFIC_SOURCES = {"verify_attn": "verify_attn.hip", "rapid_accept": "accept.hip", "rapid_lm_head": "lm_head.hip"}


def source_sha256(kernel_key: str) -> str:
    """Hash of the kernel source a traffic figure belongs to."""
    path = os.path.join(ROOT, "paper_2502_20330_amd", "csrc", TRAFFIC_SOURCES[kernel_key])
    return hashlib.sha256(open(path, "rb").read()).hexdigest()[:16]


def profile_traffic(kernel_key: str):
    """HBM bytes per launch of a kernel from the committed rocprofv3 counter summary (profiles/*.txt, a line
    `traffic_bytes_per_launch[<key>]: N`), or None.  The summary also records the hash of the kernel source
    it was taken with (`source_sha256[<key>]: H`); a figure whose source has changed since is stale and is
    not reported."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    pat = re.compile(r"traffic_bytes_per_launch\[" + re.escape(kernel_key) + r"\]:\s*([0-9.eE+]+)")
    hpat = re.compile(r"source_sha256\[" + re.escape(kernel_key) + r"\]:\s*([0-9a-f]+)")
    for name in sorted(os.listdir(pdir)):
        if name.endswith((".txt", ".md")):
            text = open(os.path.join(pdir, name)).read()
            m, h = pat.search(text), hpat.search(text)
            if m:
                return float(m.group(1)) if h and h.group(1) == source_sha256(kernel_key) else None
    return None


def also_workload(r, cfg, n_layers, head_major, steps=5, warmup=2):
    """A short measurement of another workload (`n_layers` of its attention layers over rotating caches of at
    least 1 GiB, and its accept pass): per-layer attention time, effective KV GB/s, fraction of peak."""
    import numpy as np
    import torch

    from paper_2502_20330_amd import workloads as wl
    dev = r.device
    lib = r.lib
    seqs = wl.gen_sequences(cfg)
    B, Q, Hq, Hkv, d = cfg.batch, cfg.q_max, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    ctx_lens = torch.from_numpy(seqs.ctx_lens).to(dev)
    gammas = torch.from_numpy(seqs.gammas).to(dev)
    page_table = torch.from_numpy(seqs.page_table).to(dev) if cfg.paged else None
    kv_shape = (seqs.n_pages, cfg.page_size, Hkv, d) if cfg.paged else (B, seqs.max_ctx, Hkv, d)

    def kv_randn(g):
        if head_major:
            return torch.randn((kv_shape[0], Hkv, kv_shape[1], d), dtype=torch.bfloat16, device=dev,
                               generator=g).permute(0, 2, 1, 3)
        return torch.randn(kv_shape, dtype=torch.bfloat16, device=dev, generator=g)

    tokens_alloc = (seqs.n_pages * cfg.page_size) if cfg.paged else B * seqs.max_ctx
    nbuf = max(n_layers, -(-(1 << 30) // (tokens_alloc * cfg.kv_bytes_per_token())))
    nbuf = -(-nbuf // n_layers) * n_layers
    ks, vs, qs = [], [], []
    for layer in range(nbuf):
        g = torch.Generator(device=dev)
        g.manual_seed(1000 * wl.SEED_QKV + layer)
        k = kv_randn(g)
        if cfg.k_scale != 1.0:
            k.mul_(cfg.k_scale)
        ks.append(k)
        vs.append(kv_randn(g))
        qs.append(torch.randn((B, Q, Hq, d), dtype=torch.bfloat16, device=dev, generator=g))
    out = torch.empty_like(qs[0])
    g = torch.Generator(device=dev)
    g.manual_seed(wl.SEED_LOGITS)
    gmax, V = cfg.gamma_max, cfg.vocab
    zt = torch.randn((B, gmax + 1, V), device=dev, generator=g) * cfg.logit_std
    zd = (zt[:, :gmax] + torch.randn((B, gmax, V), device=dev, generator=g) * cfg.draft_noise_std).contiguous()
    gumbel = -torch.log(-torch.log(torch.rand((B, gmax, V), device=dev, generator=g).clamp_min(1e-20)))
    draft_tokens = torch.argmax(zd / cfg.temperature + gumbel, dim=-1).to(torch.int32)
    del gumbel
    uniforms = torch.rand((B, gmax + 1), device=dev, generator=g)
    n_acc = torch.empty(B, dtype=torch.int32, device=dev)
    out_tok = torch.empty((B, gmax + 1), dtype=torch.int32, device=dev)
    tokens = int(seqs.ctx_lens.astype(np.int64).sum())
    shape = r.attn_shape(qs[0], ks[0], seqs.max_ctx, page_table=page_table, softmax_scale=cfg.softmax_scale,
                         ctx_sum_hint=tokens)
    ws = torch.empty(max(lib.rapid_verify_attn_workspace_bytes(r._ctx, ctypes.byref(shape)), 256),
                     dtype=torch.uint8, device=dev)
    # a workspace of its own: the accept pass keeps a call counter in it from one call to the next
    ws_a = torch.empty(max(lib.rapid_accept_workspace_bytes(r._ctx, B, gmax, V), 256), dtype=torch.uint8, device=dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    P = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else None
    attn_args = [(r._ctx, ctypes.byref(shape), P(qs[l]), P(ks[l]), P(vs[l]), P(ctx_lens), P(gammas), P(page_table),
                  P(out), None, P(ws), ws.numel(), stream) for l in range(nbuf)]
    acc_args = (r._ctx, B, gmax, V, P(zt), P(zd), P(draft_tokens), P(gammas), float(cfg.eta), float(cfg.temperature),
                float(cfg.tail_alpha), P(uniforms), P(n_acc), P(out_tok), None, P(ws_a), ws_a.numel(), stream)

    def check(rc):
        if rc != 0:
            raise RuntimeError(f"librapid status {rc}: {lib.rapid_strerror(rc).decode()}")

    # As in the main measurement, all steps are enqueued back to back and the host waits once at the end, so
    # that no step starts on an idle device.  These workloads have short steps (0.4-0.8 ms), and the device needs
    # several milliseconds of load before its clocks settle: the step count is therefore chosen by time, about
    # 20 ms of untimed steps and at least 10 ms of timed ones, from the duration of a first step.
    def one_step(it, e):
        first = (it * n_layers) % nbuf
        e[0].record()
        for a in attn_args[first:first + n_layers]:
            check(lib.rapid_verify_attn(*a))
        e[1].record()
        check(lib.rapid_accept(*acc_args))
        e[2].record()

    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    one_step(0, e)
    torch.cuda.synchronize()
    first_ms = max(e[0].elapsed_time(e[2]), 1e-3)
    warmup = max(warmup, min(200, int(20.0 / first_ms) + 1))
    steps = max(steps, min(100, int(10.0 / first_ms) + 1))
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(warmup + steps)]
    for it in range(warmup + steps):
        one_step(it + 1, evs[it])
    torch.cuda.synchronize()
    attn_ms = sum(e[0].elapsed_time(e[1]) for e in evs[warmup:])
    acc_ms = sum(e[1].elapsed_time(e[2]) for e in evs[warmup:])
    per_layer_us = attn_ms / (steps * n_layers) * 1e3
    kv_bytes_layer = tokens * cfg.kv_bytes_per_token()
    gbps = kv_bytes_layer / (per_layer_us * 1e-6) / 1e9
    logit_bytes = int(sum((2 * int(gb) + 1) * V * 4 for gb in seqs.gammas))
    acc_us = acc_ms / steps * 1e3
    del ks, vs, qs, attn_args
    torch.cuda.empty_cache()
    return {"layers_timed": n_layers, "layers_of_the_workload": cfg.layers, "steps": steps, "batch": B,
            "ctx_tokens": tokens, "packed_rows": Q * (Hq // Hkv), "kv_bytes_per_layer": kv_bytes_layer,
            "rotating_cache_bytes": nbuf * tokens_alloc * cfg.kv_bytes_per_token(),
            "attention_per_layer_us": round(per_layer_us, 2), "attention_gbps": round(gbps, 1),
            "attention_frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "accept_us": round(acc_us, 2), "accept_logit_bytes": logit_bytes,
            "accept_gbps": round(logit_bytes / (acc_us * 1e-6) / 1e9, 1),
            "accept_frac_of_peak": round(logit_bytes / (acc_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}


def accept_batches(r, cfg, batches=(1, 8, 64), iters=10):
    """The accept pass of `cfg` (its vocabulary, gamma, eta, temperature) on batches of several sizes: time per
    call and logit bytes per second.  The logits rotate over up to eight buffers so that no call finds them in
    the Infinity Cache; every sequence has its drafter's own arg-max as drafted tokens."""
    import torch

    from paper_2502_20330_amd import workloads as wl
    dev = r.device
    lib = r.lib
    gmax, V = cfg.gamma_max, cfg.vocab
    out = {}
    for B in batches:
        g = torch.Generator(device=dev)
        g.manual_seed(wl.SEED_LOGITS + B)
        logit_bytes = B * (2 * gmax + 1) * V * 4
        nbuf = max(1, min(8, (600 << 20) // logit_bytes))
        bufs = []
        for _ in range(nbuf):
            zt = torch.randn((B, gmax + 1, V), device=dev, generator=g) * cfg.logit_std
            zd = (zt[:, :gmax] + torch.randn((B, gmax, V), device=dev, generator=g) * (cfg.draft_noise_std or 1.0)).contiguous()
            bufs.append((zt, zd, torch.argmax(zd, dim=-1).to(torch.int32)))
        u = torch.rand((B, gmax + 1), device=dev, generator=g)
        n_acc = torch.empty(B, dtype=torch.int32, device=dev)
        out_tok = torch.empty((B, gmax + 1), dtype=torch.int32, device=dev)
        ws = torch.empty(max(lib.rapid_accept_workspace_bytes(r._ctx, B, gmax, V), 256), dtype=torch.uint8, device=dev)
        stream = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
        P = lambda t: ctypes.c_void_p(t.data_ptr())
        calls = [(r._ctx, B, gmax, V, P(zt), P(zd), P(tok), None, float(cfg.eta), float(cfg.temperature),
                  float(cfg.tail_alpha), P(u), P(n_acc), P(out_tok), None, P(ws), ws.numel(), stream)
                 for zt, zd, tok in bufs]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(3 + iters):
            if i == 3:
                e0.record()
            rc = lib.rapid_accept(*calls[i % nbuf])
            if rc != 0:
                raise RuntimeError(f"librapid status {rc}: {lib.rapid_strerror(rc).decode()}")
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / iters * 1e3
        gbps = logit_bytes / (us * 1e-6) / 1e9
        out[str(B)] = {"accept_us": round(us, 2), "logit_bytes": logit_bytes, "gbps": round(gbps, 1),
                       "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4)}
        del bufs, calls
        torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2502_20330_amd import binding
    from paper_2502_20330_amd import workloads as wl

    cfg = wl.CONFIGS[args.workload]
    layers = args.layers or cfg.layers
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    r = binding.Rapid(0)
    lib = r.lib

    # ---------------------------------------------------------------- synthetic inputs, resident in HBM
    seqs = wl.gen_sequences(cfg)
    B, Q, Hq, Hkv, d = cfg.batch, cfg.q_max, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    ctx_lens = torch.from_numpy(seqs.ctx_lens).to(dev)
    gammas = torch.from_numpy(seqs.gammas).to(dev)
    page_table = torch.from_numpy(seqs.page_table).to(dev) if cfg.paged else None
    # logical shape is always [B or pages, tokens, Hkv, d]; the memory order is the layout's
    kv_shape = (seqs.n_pages, cfg.page_size, Hkv, d) if cfg.paged else (B, seqs.max_ctx, Hkv, d)
    head_major = args.kv_layout != "token-major"
    interleaved = args.kv_layout == "head-major-kv-interleaved"   # K and V rows of a (token, head) adjacent, one tensor

    def kv_randn(g):
        if head_major:
            t = torch.randn((kv_shape[0], Hkv, kv_shape[1], d), dtype=torch.bfloat16, device=dev, generator=g)
            return t.permute(0, 2, 1, 3)
        return torch.randn(kv_shape, dtype=torch.bfloat16, device=dev, generator=g)

    def kv_pair(g):
        """(k, v) of one layer, logical shape kv_shape each."""
        if interleaved:
            t = torch.randn((kv_shape[0], Hkv, kv_shape[1], 2, d), dtype=torch.bfloat16, device=dev, generator=g)
            if cfg.k_scale != 1.0:
                t[:, :, :, 0, :].mul_(cfg.k_scale)
            t = t.permute(0, 2, 1, 3, 4)
            return t[:, :, :, 0, :], t[:, :, :, 1, :]
        k = kv_randn(g)
        if cfg.k_scale != 1.0:
            k.mul_(cfg.k_scale)
        return k, kv_randn(g)

    # Distinct cache buffers: at least one per layer, and enough of them (>= 1 GiB together) that no
    # launch finds its cache in the 256 MB Infinity Cache left there by an earlier one.
    tokens_alloc = (seqs.n_pages * cfg.page_size) if cfg.paged else B * seqs.max_ctx
    kv_alloc_layer = tokens_alloc * cfg.kv_bytes_per_token()
    nbuf = max(layers, -(-(1 << 30) // kv_alloc_layer))
    nbuf = -(-nbuf // layers) * layers                      # whole steps
    ks, vs, qs = [], [], []
    for layer in range(nbuf):
        g = torch.Generator(device=dev)
        g.manual_seed(1000 * wl.SEED_QKV + layer)
        k, v = kv_pair(g)
        ks.append(k)
        vs.append(v)
        qs.append(torch.randn((B, Q, Hq, d), dtype=torch.bfloat16, device=dev, generator=g))
    outs = [torch.empty_like(qs[0]) for _ in range(2)]
    g = torch.Generator(device=dev)
    g.manual_seed(wl.SEED_LOGITS)
    gmax, V = cfg.gamma_max, cfg.vocab
    zt = torch.randn((B, gmax + 1, V), device=dev, generator=g) * cfg.logit_std
    if cfg.draft_noise_std is None:
        zd = torch.randn((B, gmax, V), device=dev, generator=g) * cfg.logit_std
    else:
        zd = (zt[:, :gmax] + torch.randn((B, gmax, V), device=dev, generator=g) * cfg.draft_noise_std).contiguous()
    # drafter's own samples (Gumbel-max) and the uniforms of the accept tests / the draw
    gumbel = -torch.log(-torch.log(torch.rand((B, gmax, V), device=dev, generator=g).clamp_min(1e-20)))
    draft_tokens = torch.argmax(zd / cfg.temperature + gumbel, dim=-1).to(torch.int32)
    del gumbel
    uniforms = torch.rand((B, gmax + 1), device=dev, generator=g)
    head = None
    if args.with_lm_head:
        if B * (gmax + 1) > 96:
            print("bench.py: --with-lm-head handles at most 96 verification rows", file=sys.stderr)
            sys.exit(2)
        g2 = torch.Generator(device=dev)
        g2.manual_seed(wl.SEED_LM_HEAD)
        hid = cfg.hidden
        h_t = torch.randn((B * (gmax + 1), hid), device=dev, generator=g2).to(torch.bfloat16)
        w_t = (torch.randn((V, hid), device=dev, generator=g2) * (cfg.logit_std / math.sqrt(hid))).to(torch.bfloat16)
        zt, st_t = r.rapid_lm_head(h_t, w_t, temperature=cfg.temperature)      # the step overwrites both
        zt = zt.reshape(B, gmax + 1, V)
        if cfg.draft_noise_std is not None and gmax > 0:
            zd = (zt[:, :gmax] + torch.randn((B, gmax, V), device=dev, generator=g2) * cfg.draft_noise_std).contiguous()
            gumbel = -torch.log(-torch.log(torch.rand((B, gmax, V), device=dev, generator=g2).clamp_min(1e-20)))
            draft_tokens = torch.argmax(zd / cfg.temperature + gumbel, dim=-1).to(torch.int32)
            del gumbel
        head = (h_t, w_t, st_t)
    n_acc = torch.empty(B, dtype=torch.int32, device=dev)
    out_tok = torch.empty((B, gmax + 1), dtype=torch.int32, device=dev)
    ratio = torch.empty((B, gmax), dtype=torch.float32, device=dev)

    # ---------------------------------------------------------------- prepared C-ABI calls
    shape = r.attn_shape(qs[0], ks[0], seqs.max_ctx, page_table=page_table, softmax_scale=cfg.softmax_scale,
                         chunk_tokens=args.chunk_tokens, ctx_sum_hint=int(seqs.ctx_lens.astype(np.int64).sum()))
    chunk = r.verify_attn_chunk(shape)
    ws_attn = lib.rapid_verify_attn_workspace_bytes(r._ctx, ctypes.byref(shape))
    ws_acc = lib.rapid_accept_workspace_bytes(r._ctx, B, gmax, V)
    ws = torch.empty(max(ws_attn, 256), dtype=torch.uint8, device=dev)
    ws_a = torch.empty(max(ws_acc, 256), dtype=torch.uint8, device=dev)      # the accept pass's own (it keeps state)
    stream = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    P = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else None
    attn_args = [(r._ctx, ctypes.byref(shape), P(qs[l]), P(ks[l]), P(vs[l]), P(ctx_lens), P(gammas), P(page_table),
                  P(outs[l & 1]), None, P(ws), ws.numel(), stream) for l in range(nbuf)]
    acc_args = (r._ctx, B, gmax, V, P(zt), P(zd), P(draft_tokens), P(gammas), float(cfg.eta),
                float(cfg.temperature), float(cfg.tail_alpha), P(uniforms), P(n_acc), P(out_tok), P(ratio),
                P(ws_a), ws_a.numel(), stream)

    if head:
        head_args = (r._ctx, B * (gmax + 1), cfg.hidden, V, P(head[0]), P(head[1]), float(cfg.temperature),
                     P(zt), V, P(head[2]), stream)
        acc_pre_args = acc_args[:12] + (P(head[2]), head[2].shape[1], None, 0) + acc_args[12:]

    def check(rc):
        if rc != 0:
            raise RuntimeError(f"librapid status {rc}: {lib.rapid_strerror(rc).decode()}")

    step_no = [0]

    def step(ev=None):
        first = (step_no[0] * layers) % nbuf
        step_no[0] += 1
        if ev:
            ev[0].record()
        for a in attn_args[first:first + layers]:
            check(lib.rapid_verify_attn(*a))
        if ev:
            ev[1].record()
        if head:
            check(lib.rapid_lm_head(*head_args))
            if ev:
                ev[3].record()
            check(lib.rapid_accept_prestats(*acc_pre_args))
        else:
            check(lib.rapid_accept(*acc_args))
        if ev:
            ev[2].record()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                                  # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst
    # Clock pre-warm, before the W warm-up steps: after a pause the device needs 10-15 ms of load before its
    # clocks settle (the first steps of a cold run read about 5 % slow), and W steps of a small workload are
    # far shorter than that.  One step is timed to size it, then about 20 ms more of untimed steps follow.
    pw = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    pw[0].record()
    step()
    pw[1].record()
    torch.cuda.synchronize()
    prewarm_steps = 1 + min(300, int(20.0 / max(pw[0].elapsed_time(pw[1]), 1e-3)))
    for _ in range(prewarm_steps - 1):
        step()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t_begin = torch.cuda.Event(enable_timing=True)
    t_end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_begin.record()
    for s in range(args.steps):
        step(evs[s])
    t_end.record()
    torch.cuda.synchronize()
    total_ms = t_begin.elapsed_time(t_end)
    ms_per_step = total_ms / args.steps
    attn_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps      # all layers of one step
    head_ms = sum(e[1].elapsed_time(e[3]) for e in evs) / args.steps if head else 0.0
    acc_ms = sum(e[3 if head else 1].elapsed_time(e[2]) for e in evs) / args.steps

    # measured ceiling: 2 GiB streamed with no arithmetic, in launches as large as one attention call's
    # cache traffic (so launch and ramp-up cost weigh the same), never the same bytes twice in a row
    scratch = torch.empty(1 << 31, dtype=torch.uint8, device=dev)
    per_launch = max(1 << 24, min(1 << 30, (int(seqs.ctx_lens.astype(np.int64).sum()) * cfg.kv_bytes_per_token())
                                  // 16384 * 16384))
    pieces = [scratch[o:o + per_launch] for o in range(0, (1 << 31) - per_launch + 1, per_launch)]

    def probe(skew):
        r.set_option(binding.OPT_PROBE_SKEW, skew)
        for pc in pieces[:2]:
            r.rapid_hbm_read_probe(pc)
        torch.cuda.synchronize()
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        probe_bytes = sum(r.rapid_hbm_read_probe(pc) for _ in range(5) for pc in pieces)
        p1.record()
        torch.cuda.synchronize()
        r.set_option(binding.OPT_PROBE_SKEW, 0)
        return probe_bytes / (p0.elapsed_time(p1) * 1e-3) / 1e9

    stream_gbps = probe(0)
    # the same read with the uneven shares the attention kernel gives a pair of KV splits (3/32 of a share)
    stream_uneven_gbps = probe(3)
    del scratch, pieces

    tokens = int(seqs.ctx_lens.astype(np.int64).sum())
    kv_bytes_layer = tokens * cfg.kv_bytes_per_token()                    # algorithmic: K and V read once
    kv_bytes_step = kv_bytes_layer * layers
    logit_bytes = int(sum((2 * int(gb) + 1) * V * 4 for gb in seqs.gammas))
    value = kv_bytes_step / (ms_per_step * 1e-3) / 1e9
    attn_launch_ms = attn_ms / layers
    attn_gbps = kv_bytes_layer / (attn_launch_ms * 1e-3) / 1e9
    acc_gbps = logit_bytes / (acc_ms * 1e-3) / 1e9

    # the committed counter summary covers the default launch configuration only
    profiled = (cfg.name == "llama8b_128k_step" and head_major and not interleaved and not args.chunk_tokens
                and layers == cfg.layers)
    result = {
        "metric": "verify-step \u00b5s + effective KV GB/s (% HBM peak) at 128K ctx, gamma=8",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "clock_prewarm_steps": prewarm_steps,
        "ms_per_step": round(ms_per_step, 4), "verify_step_us": round(ms_per_step * 1e3, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "layers": layers, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": d, "ctx_tokens": tokens, "gamma": gmax, "vocab": V, "eta": cfg.eta,
                   "kv_layout": (("[pages,Hkv,16,2,d] (K and V rows adjacent)" if interleaved
                                  else "[pages,Hkv,16,d]" if head_major else "[pages,16,Hkv,d]") if cfg.paged
                                 else ("[B,Hkv,L,2,d] (K and V rows adjacent)" if interleaved
                                       else "[B,Hkv,L,d]" if head_major else "[B,L,Hkv,d]")), "chunk_tokens": chunk,
                   "kv_bytes_per_step": kv_bytes_step},
        "hbm_frac_of_peak": round(value / HBM_PEAK_GBPS, 4),
        "breakdown_us": {"attention_all_layers": round(attn_ms * 1e3, 1),
                         "attention_per_layer": round(attn_launch_ms * 1e3, 2), "accept": round(acc_ms * 1e3, 2)},
        "roofline": {"bound": "hbm", "kernel": "rapid_verify_attn (verify_attn_split + verify_attn_merge, one call = one layer)",
                     "achieved": round(attn_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": kv_bytes_layer,
                     "traffic": profile_traffic("verify_attn") if profiled else None,
                     "stream_read_probe_gbps": round(stream_gbps, 1) if stream_gbps else None,
                     "stream_read_probe_uneven_gbps": round(stream_uneven_gbps, 1) if stream_uneven_gbps else None,
                     "frac_of_stream_read_probe": round(attn_gbps / max(stream_gbps, stream_uneven_gbps), 4)
                     if stream_gbps else None},
        "roofline_accept": {"bound": "hbm", "kernel": "rapid_accept (all kernels of one call)",
                            "achieved": round(acc_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": round(acc_gbps / HBM_PEAK_GBPS, 4), "algorithmic_bytes_per_launch": logit_bytes,
                            "traffic": profile_traffic("rapid_accept") if profiled and not head else None},
    }

    if head:
        w_bytes = V * cfg.hidden * 2
        result["config"]["lm_head"] = {"hidden": cfg.hidden, "rows": B * (gmax + 1), "weight_bytes": w_bytes}
        result["breakdown_us"]["lm_head"] = round(head_ms * 1e3, 2)
        result["roofline_lm_head"] = {"bound": "hbm", "kernel": "rapid_lm_head (lm_head_stream)",
                                      "achieved": round(w_bytes / (head_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                                      "unit": "GB/s", "frac": round(w_bytes / (head_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                      "algorithmic_bytes_per_launch": w_bytes,
                                      "traffic": profile_traffic("rapid_lm_head") if cfg.name == "llama8b_128k_step" else None}

    # ---------------------------------------------------------------- the other 128K configurations, briefly
    if cfg.name == "llama8b_128k_step" and not args.no_also and not head:
        del ks, vs, qs, attn_args
        torch.cuda.empty_cache()
        result["also"] = {name: also_workload(r, wl.CONFIGS[name], n_layers, head_major)
                          for name, n_layers in (("ragged_paged", 1), ("llama70b_128k_step", 8))}
        result["also"]["accept_by_batch"] = accept_batches(r, cfg)
        also_mode = True
    else:
        also_mode = False

    # ---------------------------------------------------------------- oracle on the host cores (baseline only)
    if not args.no_cpu_baseline:
        import oracle
        nl = max(1, min(args.cpu_layers, layers))
        to_bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        bs, ts, hs, ps = wl.kv_strides(cfg, seqs)
        lay = oracle.KVLayout(bs, ts, hs, cfg.page_size if cfg.paged else 0, ps,
                              seqs.page_table.shape[1] if cfg.paged else 0)
        if also_mode:                   # the caches were released for the extra workloads: same seeds again
            ks, vs, qs = [], [], []
            for layer in range(nl):
                g = torch.Generator(device=dev)
                g.manual_seed(1000 * wl.SEED_QKV + layer)
                k = kv_randn(g)
                if cfg.k_scale != 1.0:
                    k.mul_(cfg.k_scale)
                ks.append(k)
                vs.append(kv_randn(g))
                qs.append(torch.randn((B, Q, Hq, d), dtype=torch.bfloat16, device=dev, generator=g))
            attn_args = [(r._ctx, ctypes.byref(shape), P(qs[l]), P(ks[l]), P(vs[l]), P(ctx_lens), P(gammas), P(page_table),
                          P(outs[l & 1]), None, P(ws), ws.numel(), stream) for l in range(nl)]
        host = [(to_bits(qs[l]), to_bits(ks[l]), to_bits(vs[l])) for l in range(nl)]
        acc_host = (zt.cpu().numpy(), zd.cpu().numpy(), draft_tokens.cpu().numpy(), uniforms.cpu().numpy())
        worst = 0.0
        t0 = time.perf_counter()
        refs = [oracle.verify_attn(q, k, v, seqs.ctx_lens, lay, Hkv=Hkv, scale=cfg.softmax_scale,
                                   gammas=seqs.gammas, page_table=seqs.page_table) for q, k, v in host]
        ref_acc = oracle.accept(*acc_host[:3], acc_host[3], eta=cfg.eta, temperature=cfg.temperature,
                                tail_alpha=cfg.tail_alpha, gammas=seqs.gammas)
        cpu_s = time.perf_counter() - t0
        for l in range(nl):             # parity of the timed launch configuration, for the record
            check(lib.rapid_verify_attn(*attn_args[l]))
            torch.cuda.synchronize()
            got = wl.bf16_bits_to_f32(to_bits(outs[l & 1])).astype(np.float64)
            worst = max(worst, float(np.max(np.abs(got - refs[l]) - 1e-2 * np.abs(refs[l]))))
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        result["cpu_baseline"] = {
            "value": round(kv_bytes_layer * nl / cpu_s / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{nl} of {layers} layers of verify attention (all heads, all {Q} positions, "
                      f"{tokens} tokens) + the accept pass, float64, {cpu_s:.1f} s",
            "gpu_vs_oracle_max_abs_err_minus_1e-2_rel": round(worst, 6),
            "accept_matches_oracle": bool(np.array_equal(out_tok.cpu().numpy(), ref_acc.out_tokens)),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
