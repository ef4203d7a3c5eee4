"""ctypes front end of the float64 CPU oracle (``rapid_oracle.c``).

TEST INFRASTRUCTURE.  Only ``tests/``, the smoke check and the CPU-baseline leg
of the benchmark may import this package; the GPU library never does, and this
package never imports the GPU library.  It holds no arithmetic of its own:
every number comes out of the C file, which is the thing to read against the
paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rapid_oracle.c")
# RAPID_ORACLE_LIB: load this shared object instead of the in-tree build (the mutation check of the
# test suite runs the pins against deliberately broken copies of the source to show that they bite)
_LIB = os.environ.get("RAPID_ORACLE_LIB") or os.path.join(_HERE, "librapid_oracle.so")
_lib = None


def compile_source(src: str, out: str) -> str:
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o", out, src, "-lm"],
                   check=True)
    return out


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (float64, OpenMP over independent units)."""
    if os.environ.get("RAPID_ORACLE_LIB"):
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


class _Layout(ctypes.Structure):
    _fields_ = [("batch_stride", ctypes.c_int64), ("token_stride", ctypes.c_int64),
                ("head_stride", ctypes.c_int64), ("page_size", ctypes.c_int32),
                ("page_stride", ctypes.c_int64), ("max_pages", ctypes.c_int32)]


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_verify_attn.restype = ctypes.c_int
        lib.oracle_accept.restype = ctypes.c_int
        lib.oracle_distributions.restype = None
        lib.oracle_lm_head.restype = ctypes.c_int
        lib.oracle_kv_append.restype = ctypes.c_int
        lib.oracle_retrieve.restype = ctypes.c_int
        lib.oracle_kv_commit.restype = ctypes.c_int
        lib.oracle_chunk_stats.restype = ctypes.c_int
        lib.oracle_kv_commit_pages.restype = ctypes.c_int
        lib.oracle_accept_greedy.restype = ctypes.c_int
        lib.oracle_retrieval_top_k.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a, ctype):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctype))


@dataclass
class KVLayout:
    """Element strides of a KV cache (see ``oracle_kv_layout`` in the C file)."""
    batch_stride: int
    token_stride: int
    head_stride: int
    page_size: int = 0
    page_stride: int = 0
    max_pages: int = 0


def verify_attn(q, k, v, ctx_lens, layout: KVLayout, *, Hkv, scale, gamma=None,
                gammas=None, page_table=None, want_lse=False):
    """q: uint16 (bf16 bits) [B,Qmax,Hq,d]; k, v: uint16 flat or shaped caches.

    Returns out float64 [B,Qmax,Hq,d] (and lse float64 [B,Hq,Qmax])."""
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    B, Qmax, Hq, d = q.shape
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    assert ctx_lens.shape == (B,)
    if gammas is not None:
        gammas = np.ascontiguousarray(gammas, dtype=np.int32)
        g = 0
    else:
        g = Qmax - 1 if gamma is None else int(gamma)
    if page_table is not None:
        page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    lay = _Layout(layout.batch_stride, layout.token_stride, layout.head_stride,
                  layout.page_size, layout.page_stride, layout.max_pages)
    out = np.empty((B, Qmax, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq, Qmax), dtype=np.float64) if want_lse else None
    rc = lib.oracle_verify_attn(
        ctypes.c_int(B), ctypes.c_int(Qmax), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        ctypes.c_int(d), ctypes.c_double(scale),
        _ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16),
        ctypes.byref(lay), _ptr(page_table, ctypes.c_int32),
        _ptr(ctx_lens, ctypes.c_int32), _ptr(gammas, ctypes.c_int32), ctypes.c_int(g),
        _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_verify_attn: invalid argument (rc={rc})")
    return (out, lse) if want_lse else out


@dataclass
class AcceptResult:
    n_accepted: np.ndarray      # int32 [B]
    out_tokens: np.ndarray      # int32 [B, gmax+1]
    ratio: np.ndarray           # float64 [B, gmax]
    accept_margin: np.ndarray   # float64 [B, gmax]
    draw_margin: np.ndarray     # float64 [B]


def accept(target_logits, draft_logits, draft_tokens, uniforms, *, eta, temperature=1.0,
           tail_alpha=0.1, gammas=None) -> AcceptResult:
    lib = _load()
    zt = np.ascontiguousarray(target_logits, dtype=np.float32)
    zd = np.ascontiguousarray(draft_logits, dtype=np.float32)
    B, g1, V = zt.shape
    gmax = g1 - 1
    assert zd.shape == (B, gmax, V), (zd.shape, (B, gmax, V))
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, gmax)
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    assert u.shape == (B, gmax + 1)
    if gammas is not None:
        gammas = np.ascontiguousarray(gammas, dtype=np.int32)
    n_acc = np.empty((B,), dtype=np.int32)
    out_tok = np.empty((B, gmax + 1), dtype=np.int32)
    ratio = np.full((B, gmax), np.nan, dtype=np.float64)
    amargin = np.full((B, gmax), np.inf, dtype=np.float64)
    dmargin = np.zeros((B,), dtype=np.float64)
    rc = lib.oracle_accept(
        ctypes.c_int(B), ctypes.c_int(gmax), ctypes.c_int64(V),
        _ptr(zt, ctypes.c_float), _ptr(zd, ctypes.c_float), _ptr(tok, ctypes.c_int32),
        _ptr(gammas, ctypes.c_int32), ctypes.c_double(eta), ctypes.c_double(temperature),
        ctypes.c_double(tail_alpha), _ptr(u, ctypes.c_float),
        _ptr(n_acc, ctypes.c_int32), _ptr(out_tok, ctypes.c_int32),
        _ptr(ratio, ctypes.c_double), _ptr(amargin, ctypes.c_double),
        _ptr(dmargin, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_accept: invalid argument (rc={rc})")
    return AcceptResult(n_acc, out_tok, ratio, amargin, dmargin)


def accept_greedy(target_logits, draft_logits, draft_tokens, uniforms, *, gammas=None) -> AcceptResult:
    """The T -> 0 limit of :func:`accept` (see ``oracle_accept_greedy``); draw_margin is 1 (no uniform is used)."""
    lib = _load()
    zt = np.ascontiguousarray(target_logits, dtype=np.float32)
    zd = np.ascontiguousarray(draft_logits, dtype=np.float32)
    B, g1, V = zt.shape
    gmax = g1 - 1
    assert zd.shape == (B, gmax, V)
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, gmax)
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    assert u.shape == (B, gmax + 1)
    if gammas is not None:
        gammas = np.ascontiguousarray(gammas, dtype=np.int32)
    n_acc = np.empty((B,), dtype=np.int32)
    out_tok = np.empty((B, gmax + 1), dtype=np.int32)
    ratio = np.full((B, gmax), np.nan, dtype=np.float64)
    amargin = np.full((B, gmax), np.inf, dtype=np.float64)
    rc = lib.oracle_accept_greedy(ctypes.c_int(B), ctypes.c_int(gmax), ctypes.c_int64(V), _ptr(zt, ctypes.c_float),
                                  _ptr(zd, ctypes.c_float), _ptr(tok, ctypes.c_int32), _ptr(gammas, ctypes.c_int32),
                                  _ptr(u, ctypes.c_float), _ptr(n_acc, ctypes.c_int32), _ptr(out_tok, ctypes.c_int32),
                                  _ptr(ratio, ctypes.c_double), _ptr(amargin, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_accept_greedy: invalid argument (rc={rc})")
    return AcceptResult(n_acc, out_tok, ratio, amargin, np.ones((B,), dtype=np.float64))


def distributions(z, zq, *, eta, temperature=1.0, tail_alpha=0.1):
    """(p, q, p_hat) of one position, float64 [V] each."""
    lib = _load()
    z = np.ascontiguousarray(z, dtype=np.float64)
    zq = np.ascontiguousarray(zq, dtype=np.float64)
    V = z.shape[0]
    p = np.empty(V); q = np.empty(V); ph = np.empty(V)
    lib.oracle_distributions(ctypes.c_int64(V), _ptr(z, ctypes.c_double),
                             _ptr(zq, ctypes.c_double), ctypes.c_double(eta),
                             ctypes.c_double(temperature), ctypes.c_double(tail_alpha),
                             _ptr(p, ctypes.c_double), _ptr(q, ctypes.c_double),
                             _ptr(ph, ctypes.c_double))
    return p, q, ph


def lm_head(h_bits, w_bits):
    """z = h W^T in float64 from bf16 bit patterns: h uint16 [rows, hidden], w uint16 [vocab, hidden]."""
    lib = _load()
    h = np.ascontiguousarray(h_bits, dtype=np.uint16)
    w = np.ascontiguousarray(w_bits, dtype=np.uint16)
    rows, hidden = h.shape
    vocab, hidden_w = w.shape
    if hidden_w != hidden:
        raise ValueError("hidden sizes differ")
    z = np.empty((rows, vocab), dtype=np.float64)
    rc = lib.oracle_lm_head(ctypes.c_int(rows), ctypes.c_int64(hidden), ctypes.c_int64(vocab),
                            _ptr(h, ctypes.c_uint16), _ptr(w, ctypes.c_uint16), _ptr(z, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_lm_head: invalid argument (rc={rc})")
    return z


def chunk_stats(z, chunk: int, temperature: float = 1.0):
    """Per block of `chunk` vocabulary entries: (max z, sum exp((z - max)/T)), float64 [rows, nch] each."""
    lib = _load()
    z = np.ascontiguousarray(z, dtype=np.float64)
    rows, vocab = z.shape
    nch = (vocab + chunk - 1) // chunk
    cmax = np.empty((rows, nch)); csum = np.empty((rows, nch))
    rc = lib.oracle_chunk_stats(ctypes.c_int(rows), ctypes.c_int64(vocab), ctypes.c_int64(chunk),
                                ctypes.c_double(temperature), _ptr(z, ctypes.c_double),
                                _ptr(cmax, ctypes.c_double), _ptr(csum, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_chunk_stats: invalid argument (rc={rc})")
    return cmax, csum


def _c_layout(layout: KVLayout) -> _Layout:
    return _Layout(layout.batch_stride, layout.token_stride, layout.head_stride, layout.page_size,
                   layout.page_stride, layout.max_pages)


def kv_append(k_cache, v_cache, k_new, v_new, ctx_lens, layout: KVLayout, *, gamma=None, gammas=None,
              page_table=None):
    """Writes rows 0..gamma_b of k_new/v_new (uint16 [B, Qmax, Hkv, d]) into the caches IN PLACE as the
    last gamma_b+1 tokens of every sequence (ctx_lens counts them)."""
    lib = _load()
    for a in (k_cache, v_cache):
        if a.dtype != np.uint16 or not a.flags.c_contiguous or not a.flags.writeable:
            raise ValueError("caches must be writable C-contiguous uint16 arrays")
    k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
    v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    B, Qmax, Hkv, d = k_new.shape
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    gammas = None if gammas is None else np.ascontiguousarray(gammas, dtype=np.int32)
    page_table = None if page_table is None else np.ascontiguousarray(page_table, dtype=np.int32)
    lay = _c_layout(layout)
    rc = lib.oracle_kv_append(ctypes.c_int(B), ctypes.c_int(Qmax), ctypes.c_int(Hkv), ctypes.c_int(d),
                              _ptr(k_new, ctypes.c_uint16), _ptr(v_new, ctypes.c_uint16),
                              _ptr(ctx_lens, ctypes.c_int32), _ptr(gammas, ctypes.c_int32),
                              ctypes.c_int(0 if gamma is None else gamma), ctypes.byref(lay),
                              _ptr(page_table, ctypes.c_int32),
                              _ptr(k_cache, ctypes.c_uint16), _ptr(v_cache, ctypes.c_uint16))
    if rc != 0:
        raise ValueError(f"oracle_kv_append: invalid argument (rc={rc})")


def kv_commit(ctx_lens, n_accepted, *, gamma=None, gammas=None):
    """Context lengths after a validation round that accepted n_accepted[b] drafts (new int32 array)."""
    lib = _load()
    out = np.array(ctx_lens, dtype=np.int32, copy=True)
    n_accepted = np.ascontiguousarray(n_accepted, dtype=np.int32)
    gammas = None if gammas is None else np.ascontiguousarray(gammas, dtype=np.int32)
    rc = lib.oracle_kv_commit(ctypes.c_int(len(out)), _ptr(gammas, ctypes.c_int32),
                              ctypes.c_int(0 if gamma is None else gamma),
                              _ptr(n_accepted, ctypes.c_int32), _ptr(out, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_kv_commit: invalid argument (rc={rc})")
    return out


def kv_commit_pages(ctx_lens, n_accepted, page_table, page_size: int, cap: int, *, gamma=None, gammas=None):
    """Paged commit: returns (new ctx_lens, released int32 [B, cap] page ids then -1, n_released int32 [B])."""
    lib = _load()
    out = np.array(ctx_lens, dtype=np.int32, copy=True)
    n_accepted = np.ascontiguousarray(n_accepted, dtype=np.int32)
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    gammas = None if gammas is None else np.ascontiguousarray(gammas, dtype=np.int32)
    B = len(out)
    rel = np.empty((B, cap), dtype=np.int32)
    cnt = np.empty(B, dtype=np.int32)
    rc = lib.oracle_kv_commit_pages(ctypes.c_int(B), _ptr(gammas, ctypes.c_int32),
                                    ctypes.c_int(0 if gamma is None else gamma), _ptr(n_accepted, ctypes.c_int32),
                                    _ptr(page_table, ctypes.c_int32), ctypes.c_int(page_table.shape[1]),
                                    ctypes.c_int(page_size), _ptr(out, ctypes.c_int32), _ptr(rel, ctypes.c_int32),
                                    ctypes.c_int(cap), _ptr(cnt, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_kv_commit_pages: invalid argument (rc={rc})")
    return out, rel, cnt


def retrieve(emb, query, top_k: int, threshold: float):
    """Chunk selection: returns (sim float64 [n], selected int32 [count] in document order, margin)."""
    lib = _load()
    emb = np.ascontiguousarray(emb, dtype=np.float32)
    query = np.ascontiguousarray(query, dtype=np.float32)
    n, dim = emb.shape
    sim = np.empty(n, dtype=np.float64)
    sel = np.empty(max(top_k, 1), dtype=np.int32)
    cnt = ctypes.c_int32(0)
    mg = ctypes.c_double(0.0)
    rc = lib.oracle_retrieve(ctypes.c_int(n), ctypes.c_int(dim), _ptr(emb, ctypes.c_float),
                             _ptr(query, ctypes.c_float), ctypes.c_int(top_k), ctypes.c_double(threshold),
                             _ptr(sim, ctypes.c_double), _ptr(sel, ctypes.c_int32), ctypes.byref(cnt),
                             ctypes.byref(mg))
    if rc != 0:
        raise ValueError(f"oracle_retrieve: invalid argument (rc={rc})")
    return sim, sel[:cnt.value].copy(), mg.value


def retrieval_top_k(ctx_tokens: int, chunk_tokens: int = 512) -> int:
    """Chunks the drafter's context may hold ("RAG Setup", Sec. 3): the retrieval context is at least 4096
    tokens and otherwise 1/24 of the input, counted in whole chunks."""
    return int(_load().oracle_retrieval_top_k(ctypes.c_int64(ctx_tokens), ctypes.c_int(chunk_tokens)))
