"""Seeded synthetic inputs shaped like the paper's long-context workloads.

This module is the one piece shared by the GPU tests, the benchmark and the
oracle tests.  It draws random numbers and lays them out; it holds none of the
method's arithmetic (no softmax, no attention, no accept rule) and imports
neither the GPU binding nor the oracle.

The paper evaluates on LongBench v2 / InfiniteBench with LLaMA-3.1 and Qwen2.5
models at ~120K-token contexts (Sec. 3); none of that data exists here.  The
inputs below reproduce only shapes and rough statistics: context 2K-128K
tokens, GQA 4/1, 32/8 and 64/8 heads, head_dim 64/128, vocabulary 8192 or
128256, gamma 4-8, draft logits = target logits + noise so that acceptance
lands in the paper's 60-85 % band.

bf16 tensors travel as uint16 bit patterns on the host (numpy has no bf16).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np

# seeds of the independent random streams
SEED_QKV, SEED_UNIFORM, SEED_LOGITS, SEED_PAGES, SEED_DRAFT = 0, 1, 2, 3, 4


@dataclass(frozen=True)
class VerifyConfig:
    name: str
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx: Tuple[int, int]                 # (lo, hi) inclusive range of context lengths
    gamma_choices: Tuple[int, ...]       # per-sequence gamma drawn from these
    vocab: int
    eta: float
    logit_std: float
    draft_noise_std: Optional[float]     # None: draft logits independent of the target's
    k_scale: float = 1.0                 # K is multiplied by this before rounding to bf16
    paged: bool = False
    page_size: int = 16
    temperature: float = 1.0
    tail_alpha: float = 0.1
    etas: Tuple[float, ...] = field(default=())
    hidden: int = 4096                   # model width (rows of the output head)

    @property
    def gamma_max(self) -> int:
        return max(self.gamma_choices)

    @property
    def q_max(self) -> int:
        return self.gamma_max + 1

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    def kv_bytes_per_token(self) -> int:
        """K and V bytes of one context token of one layer (bf16)."""
        return 2 * self.n_kv_heads * self.head_dim * 2


CONFIGS = {
    # the five workloads the benchmark definition names, in its order
    "tiny": VerifyConfig("tiny", 1, 1, 4, 1, 64, (2048, 2048), (4,), 8192, 0.5, 3.0, None),
    "llama8b_32k": VerifyConfig("llama8b_32k", 1, 1, 32, 8, 128, (32768, 32768), (8,), 128256,
                                1.0, 4.0, 1.0, k_scale=1.0 / math.sqrt(128)),
    "llama8b_128k_step": VerifyConfig("llama8b_128k_step", 32, 1, 32, 8, 128, (131072, 131072),
                                      (8,), 128256, 1.0, 4.0, 1.0, k_scale=1.0 / math.sqrt(128)),
    "ragged_paged": VerifyConfig("ragged_paged", 1, 8, 32, 8, 128, (16384, 131072), (4, 6, 8),
                                 128256, 1.0, 4.0, 1.0, k_scale=1.0 / math.sqrt(128), paged=True),
    "llama70b_128k_step": VerifyConfig("llama70b_128k_step", 80, 1, 64, 8, 128, (131072, 131072),
                                       (8,), 128256, 0.5, 4.0, 1.0, k_scale=1.0 / math.sqrt(128),
                                       etas=(0.25, 0.5, 1.0), hidden=8192),
    # the paper's other model family at its small size (Qwen2.5-7B shape: 28 layers, 28 query / 4 kv heads,
    # width 3584, vocabulary 152064), gamma = 10 as in the paper's runs
    "qwen7b_128k_step": VerifyConfig("qwen7b_128k_step", 28, 1, 28, 4, 128, (131072, 131072), (10,), 152064,
                                     5.0, 4.0, 1.0, k_scale=1.0 / math.sqrt(128), hidden=3584),
    # next rows: the drafter's own decode step on the retrieved context (Sec. 2.2: the drafter works on
    # the shortened context, one position per step): the same two calls at gamma = 0, where the accept
    # call reduces to drawing the next token from softmax(z / T)
    "drafter_decode_8k": VerifyConfig("drafter_decode_8k", 32, 1, 32, 8, 128, (8192, 8192), (0,), 128256,
                                      0.0, 4.0, 1.0, k_scale=1.0 / math.sqrt(128)),
    "drafter_decode_16k_b8": VerifyConfig("drafter_decode_16k_b8", 32, 8, 32, 8, 128, (4096, 16384), (0,), 128256,
                                          0.0, 4.0, 1.0, k_scale=1.0 / math.sqrt(128)),
}


def scaled(cfg: VerifyConfig, **kw) -> VerifyConfig:
    """A copy of a config with some fields replaced (smaller test sizes)."""
    return replace(cfg, **kw)


# ---------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, scale: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24                      # bounded temporaries
    for s in range(0, n, step):
        e = min(n, s + step)
        x = rng.standard_normal(e - s, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        out[s:e] = f32_to_bf16_bits(x)
    return out.reshape(shape)


# ---------------------------------------------------------------- sequences
@dataclass
class Sequences:
    ctx_lens: np.ndarray                # int32 [B], counts the gamma_b+1 verify positions
    gammas: np.ndarray                  # int32 [B]
    page_table: Optional[np.ndarray]    # int32 [B, max_pages] or None
    n_pages: int                        # pages in the pool (paged) or 0
    max_ctx: int                        # row capacity of a contiguous cache


def gen_sequences(cfg: VerifyConfig) -> Sequences:
    rng = np.random.default_rng(SEED_PAGES)
    lo, hi = cfg.ctx
    ctx = rng.integers(lo, hi + 1, size=cfg.batch).astype(np.int32)
    gam = rng.choice(np.asarray(cfg.gamma_choices, dtype=np.int32), size=cfg.batch).astype(np.int32)
    ctx = np.maximum(ctx, gam + 1)
    if not cfg.paged:
        return Sequences(ctx, gam, None, 0, int(ctx.max()))
    ps = cfg.page_size
    need = (ctx.astype(np.int64) + ps - 1) // ps
    n_pages = int(need.sum()) + 7       # a few pages nobody owns
    perm = rng.permutation(n_pages).astype(np.int32)
    max_pages = int(need.max())
    table = np.full((cfg.batch, max_pages), -1, dtype=np.int32)
    pos = 0
    for b in range(cfg.batch):
        table[b, : need[b]] = perm[pos: pos + need[b]]
        pos += int(need[b])
    return Sequences(ctx, gam, table, n_pages, int(ctx.max()))


# ---------------------------------------------------------------- attention inputs
@dataclass
class AttnInputs:
    q: np.ndarray                       # uint16 [B, Qmax, Hq, d]
    k: np.ndarray                       # uint16 [B, Lmax, Hkv, d] or [n_pages, page, Hkv, d]
    v: np.ndarray
    seqs: Sequences


def gen_attn_inputs(cfg: VerifyConfig, layer: int = 0, seqs: Optional[Sequences] = None) -> AttnInputs:
    """Q, K, V ~ N(0,1) (K times cfg.k_scale), rounded to bf16, seeded per layer."""
    seqs = seqs or gen_sequences(cfg)
    rng = np.random.default_rng([SEED_QKV, layer])
    q = _normal_bf16(rng, (cfg.batch, cfg.q_max, cfg.n_q_heads, cfg.head_dim))
    if cfg.paged:
        shape = (seqs.n_pages, cfg.page_size, cfg.n_kv_heads, cfg.head_dim)
    else:
        shape = (cfg.batch, seqs.max_ctx, cfg.n_kv_heads, cfg.head_dim)
    k = _normal_bf16(rng, shape, cfg.k_scale)
    v = _normal_bf16(rng, shape)
    return AttnInputs(q, k, v, seqs)


def kv_strides(cfg: VerifyConfig, seqs: Sequences):
    """(batch_stride, token_stride, head_stride, page_stride) in elements."""
    tok = cfg.n_kv_heads * cfg.head_dim
    if cfg.paged:
        return 0, tok, cfg.head_dim, cfg.page_size * tok
    return seqs.max_ctx * tok, tok, cfg.head_dim, 0


# ---------------------------------------------------------------- accept inputs
@dataclass
class AcceptInputs:
    target_logits: np.ndarray           # float32 [B, gmax+1, V]
    draft_logits: np.ndarray            # float32 [B, gmax, V]
    draft_tokens: np.ndarray            # int32 [B, gmax]
    uniforms: np.ndarray                # float32 [B, gmax+1] in [0, 1)
    gammas: np.ndarray                  # int32 [B]


def gen_accept_inputs(cfg: VerifyConfig, seqs: Optional[Sequences] = None, batch: Optional[int] = None,
                      salt: int = 0) -> AcceptInputs:
    """Target logits N(0, std^2); draft logits = target + N(0, noise^2) (or independent).

    Draft tokens are drawn from the drafter's own distribution at temperature T
    with the Gumbel-max rule (argmax of logits/T + Gumbel noise), which needs no
    normalisation."""
    B = cfg.batch if batch is None else batch
    gmax, V = cfg.gamma_max, cfg.vocab
    rng = np.random.default_rng([SEED_LOGITS, salt])
    zt = rng.standard_normal((B, gmax + 1, V), dtype=np.float32) * np.float32(cfg.logit_std)
    if cfg.draft_noise_std is None:
        zd = rng.standard_normal((B, gmax, V), dtype=np.float32) * np.float32(cfg.logit_std)
    else:
        zd = zt[:, :gmax, :] + rng.standard_normal((B, gmax, V), dtype=np.float32) * np.float32(cfg.draft_noise_std)
    drng = np.random.default_rng([SEED_DRAFT, salt])
    tok = np.empty((B, gmax), dtype=np.int32)
    for b in range(B):
        gumbel = drng.gumbel(size=(gmax, V))
        tok[b] = np.argmax(zd[b].astype(np.float64) / cfg.temperature + gumbel, axis=-1)
    urng = np.random.default_rng([SEED_UNIFORM, salt])
    u = urng.random((B, gmax + 1), dtype=np.float32)
    if seqs is not None and batch is None:
        gam = seqs.gammas.copy()
    else:
        g2 = np.random.default_rng([SEED_PAGES, salt, 1])
        gam = g2.choice(np.asarray(cfg.gamma_choices, dtype=np.int32), size=B).astype(np.int32)
    return AcceptInputs(zt, zd, tok, u, gam)


# ---------------------------------------------------------------- output head
SEED_LM_HEAD = 5


def gen_lm_head_inputs(rows: int, hidden: int, vocab: int, *, logit_std: float = 4.0, salt: int = 0):
    """Final hidden states and output embedding as bf16 bit patterns: h ~ N(0, 1) [rows, hidden],
    W ~ N(0, logit_std^2 / hidden) [vocab, hidden], so that the logits h W^T have standard deviation
    logit_std like the synthetic logits of the accept workloads."""
    rng = np.random.default_rng([SEED_LM_HEAD, salt])
    h = _normal_bf16(rng, (rows, hidden))
    w = _normal_bf16(rng, (vocab, hidden), scale=logit_std / math.sqrt(hidden))
    return h, w


# ---------------------------------------------------------------- retrieval
SEED_RETRIEVAL = 6


def gen_retrieval_inputs(n_chunks: int, dim: int = 1024, *, relevant: int = 12, salt: int = 0):
    """Synthetic stand-in for sentence embeddings of the context's 512-token chunks and of the query (the
    paper embeds with BGE-M3, dense dimension 1024; no model or text is available here): unit-scale Gaussian
    chunk vectors, of which `relevant` share a component with the query so that their cosine similarities
    spread over roughly 0.15..0.8 and straddle the 0.3 threshold; the rest sit near 0."""
    rng = np.random.default_rng([SEED_RETRIEVAL, salt])
    query = rng.standard_normal(dim).astype(np.float32)
    emb = rng.standard_normal((n_chunks, dim)).astype(np.float32)
    idx = rng.choice(n_chunks, size=min(relevant, n_chunks), replace=False)
    mix = np.linspace(0.15, 0.8, num=len(idx)).astype(np.float32)
    for i, a in zip(idx, mix):
        emb[i] = a * query + np.sqrt(1.0 - a * a) * emb[i]
    emb *= rng.uniform(0.5, 2.0, size=(n_chunks, 1)).astype(np.float32)      # norms vary: cosine, not dot
    return emb, query
