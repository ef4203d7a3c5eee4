"""ctypes binding of librapid.so: argument marshalling only.

Every step of the verification path runs in the library's gfx950 kernels; torch
supplies device memory and the stream.  There is no CPU fallback: if the library
has not been built, importing works but the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librapid.so")

RAPID_OK = 0
RAPID_EINVAL, RAPID_EALIGN, RAPID_EUNSUPPORTED, RAPID_EWORKSPACE, RAPID_EHIP, RAPID_ETOOLARGE = -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 32 << 20
OPT_ACCEPT_WAIT_US, OPT_ACCEPT_SLICE, OPT_PROBE_SKEW = 1, 2, 3
EXPORTS = ["rapid_create", "rapid_destroy", "rapid_strerror", "rapid_last_hip_error", "rapid_set_option",
           "rapid_verify_attn_chunk", "rapid_verify_attn_workspace_bytes", "rapid_verify_attn",
           "rapid_verify_attn_static",
           "rapid_accept_workspace_bytes", "rapid_accept", "rapid_accept_prestats",
           "rapid_lm_head_chunk", "rapid_lm_head_stat_chunks", "rapid_lm_head", "rapid_kv_append", "rapid_kv_commit",
           "rapid_kv_commit_pages",
           "rapid_retrieve", "rapid_hbm_read_probe"]


class RapidError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"librapid: {message} (status {status})")
        self.status = status


class AttnShape(ctypes.Structure):
    """Mirror of ``rapid_attn_shape`` in include/rapid.h."""
    _fields_ = [("batch", ctypes.c_int32), ("q_max", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("max_ctx", ctypes.c_int32),
                ("gamma", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("kv_batch_stride", ctypes.c_int64), ("kv_token_stride", ctypes.c_int64),
                ("kv_head_stride", ctypes.c_int64), ("kv_page_stride", ctypes.c_int64),
                ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
                ("chunk_tokens", ctypes.c_int32), ("n_pages", ctypes.c_int32),
                ("ctx_sum_hint", ctypes.c_int64)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load librapid.so and declare the C signatures.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RapidError(-100, f"{LIB_PATH} not found: build it with "
                               "`python -m paper_2502_20330_amd.build` (there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    lib.rapid_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int]
    lib.rapid_create.restype = ctypes.c_int
    lib.rapid_destroy.argtypes = [ctypes.c_void_p]
    lib.rapid_destroy.restype = None
    lib.rapid_strerror.argtypes = [ctypes.c_int]
    lib.rapid_strerror.restype = ctypes.c_char_p
    lib.rapid_last_hip_error.argtypes = [ctypes.c_void_p]
    lib.rapid_last_hip_error.restype = ctypes.c_int
    lib.rapid_set_option.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64]
    lib.rapid_set_option.restype = ctypes.c_int
    lib.rapid_verify_attn_chunk.argtypes = [ctypes.c_void_p, ctypes.POINTER(AttnShape)]
    lib.rapid_verify_attn_chunk.restype = ctypes.c_int
    lib.rapid_verify_attn_workspace_bytes.argtypes = [ctypes.c_void_p, ctypes.POINTER(AttnShape)]
    lib.rapid_verify_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.rapid_verify_attn.argtypes = [ctypes.c_void_p, ctypes.POINTER(AttnShape), vp, vp, vp, i32p, i32p, i32p,
                                      vp, f32p, vp, ctypes.c_size_t, vp]
    lib.rapid_verify_attn.restype = ctypes.c_int
    lib.rapid_verify_attn_static.argtypes = [ctypes.c_void_p, ctypes.POINTER(AttnShape), vp, vp, vp, i32p, i32p, i32p,
                                             vp, f32p, vp]
    lib.rapid_verify_attn_static.restype = ctypes.c_int
    lib.rapid_accept_workspace_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.rapid_accept_workspace_bytes.restype = ctypes.c_size_t
    lib.rapid_accept.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, f32p, f32p, i32p, i32p,
                                 ctypes.c_float, ctypes.c_float, ctypes.c_float, f32p, i32p, i32p, f32p,
                                 vp, ctypes.c_size_t, vp]
    lib.rapid_accept.restype = ctypes.c_int
    lib.rapid_accept_prestats.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, f32p, f32p, i32p, i32p,
                                          ctypes.c_float, ctypes.c_float, ctypes.c_float, f32p,
                                          f32p, ctypes.c_int, f32p, ctypes.c_int, i32p, i32p, f32p,
                                          vp, ctypes.c_size_t, vp]
    lib.rapid_accept_prestats.restype = ctypes.c_int
    lib.rapid_lm_head_chunk.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
    lib.rapid_lm_head_chunk.restype = ctypes.c_int
    lib.rapid_lm_head_stat_chunks.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
    lib.rapid_lm_head_stat_chunks.restype = ctypes.c_int
    lib.rapid_lm_head.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp, ctypes.c_float,
                                  f32p, ctypes.c_int64, f32p, vp]
    lib.rapid_lm_head.restype = ctypes.c_int
    lib.rapid_kv_append.argtypes = [ctypes.c_void_p, ctypes.POINTER(AttnShape), vp, vp, i32p, i32p, i32p, vp, vp, vp]
    lib.rapid_kv_append.restype = ctypes.c_int
    lib.rapid_kv_commit.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, i32p, i32p, i32p, vp]
    lib.rapid_kv_commit.restype = ctypes.c_int
    lib.rapid_kv_commit_pages.argtypes = [ctypes.c_void_p, ctypes.POINTER(AttnShape), i32p, i32p, i32p, i32p, i32p,
                                          ctypes.c_int, i32p, vp]
    lib.rapid_kv_commit_pages.restype = ctypes.c_int
    lib.rapid_retrieve.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, f32p, f32p, ctypes.c_int, ctypes.c_float,
                                   f32p, i32p, i32p, vp]
    lib.rapid_retrieve.restype = ctypes.c_int
    lib.rapid_hbm_read_probe.argtypes = [ctypes.c_void_p, vp, ctypes.c_size_t, vp, vp]
    lib.rapid_hbm_read_probe.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(lib, status: int, ctx=None):
    if status != RAPID_OK:
        msg = lib.rapid_strerror(status).decode()
        if ctx is not None and status == -5:
            msg += f" (hip error {lib.rapid_last_hip_error(ctx)})"
        raise RapidError(status, msg)


def _dptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


class Rapid:
    """One library context on one GPU plus a grow-only workspace tensor."""

    def __init__(self, device: int = 0):
        if not torch.cuda.is_available():
            raise RapidError(-101, "no GPU visible: the verification path has no CPU implementation")
        self.lib = load_library()
        self.device = torch.device("cuda", device)
        self._ctx = ctypes.c_void_p()
        torch.cuda.set_device(self.device)
        _check(self.lib, self.lib.rapid_create(ctypes.byref(self._ctx), device))
        self._ws: Optional[torch.Tensor] = None
        self._ws_accept: Optional[torch.Tensor] = None
        self._sink: Optional[torch.Tensor] = None

    def close(self):
        if self._ctx:
            self.lib.rapid_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, option: int, value: int):
        _check(self.lib, self.lib.rapid_set_option(self._ctx, int(option), int(value)))

    def accept_status(self):
        """(rejected out-of-range draft ids, exchange waits that gave up) of the last rapid_accept call that
        used this object's workspace; synchronises."""
        torch.cuda.synchronize(self.device)
        w = self._ws_accept[:8].view(torch.int32).cpu()
        return int(w[0]), int(w[1])

    def _workspace(self, nbytes: int) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        return self._ws

    def _accept_workspace(self, nbytes: int) -> torch.Tensor:
        # its own buffer: the accept pass keeps a call counter in it from one call to the next
        if self._ws_accept is None or self._ws_accept.numel() < nbytes:
            self._ws_accept = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        return self._ws_accept

    # ------------------------------------------------------------------ attention
    def attn_shape(self, q, k_cache, ctx_max: int, *, gamma: Optional[int] = None, page_table=None,
                   softmax_scale: Optional[float] = None, chunk_tokens: int = 0,
                   ctx_sum_hint: int = 0) -> AttnShape:
        B, Qmax, Hq, d = q.shape
        s = AttnShape()
        s.batch, s.q_max, s.n_q_heads, s.head_dim = B, Qmax, Hq, d
        s.n_kv_heads = k_cache.shape[2]
        s.max_ctx = int(ctx_max)
        s.gamma = Qmax - 1 if gamma is None else int(gamma)
        s.softmax_scale = float(softmax_scale) if softmax_scale is not None else d ** -0.5
        st = k_cache.stride()
        if k_cache.stride(3) != 1:
            raise RapidError(-1, "head_dim must be the contiguous dimension of the KV cache")
        if page_table is None:
            s.kv_batch_stride, s.kv_token_stride, s.kv_head_stride = st[0], st[1], st[2]
            s.kv_page_stride, s.page_size, s.max_pages = 0, 0, 0
        else:
            s.kv_page_stride, s.kv_token_stride, s.kv_head_stride = st[0], st[1], st[2]
            s.kv_batch_stride = 0
            s.page_size, s.max_pages = k_cache.shape[1], page_table.shape[1]
        s.chunk_tokens = int(chunk_tokens)
        s.n_pages = 0 if page_table is None else int(k_cache.shape[0])
        s.ctx_sum_hint = int(ctx_sum_hint)
        return s

    def verify_attn_chunk(self, shape: AttnShape) -> int:
        c = self.lib.rapid_verify_attn_chunk(self._ctx, ctypes.byref(shape))
        if c < 0:
            _check(self.lib, c)
        return c

    def rapid_verify_attn(self, q, k_cache, v_cache, ctx_lens, gamma: Optional[int] = None, *, gammas=None,
                          page_table=None, max_ctx: Optional[int] = None, softmax_scale: Optional[float] = None,
                          chunk_tokens: int = 0, out=None, lse_out=None, shape: Optional[AttnShape] = None,
                          ctx_sum_hint: int = 0):
        """q bf16 [B,Qmax,Hq,d]; k_cache/v_cache bf16 [B,Lmax,Hkv,d] (any batch/token/head strides)
        or paged [n_pages,page,Hkv,d] with page_table int32 [B,max_pages]; ctx_lens int32 [B]
        (device).  ``max_ctx`` is a host upper bound of ctx_lens (default: the cache capacity).
        Returns out bf16 [B,Qmax,Hq,d]; fills lse_out fp32 [B,Hq,Qmax] if given."""
        assert q.dtype == torch.bfloat16 and k_cache.dtype == torch.bfloat16 and v_cache.dtype == torch.bfloat16
        assert q.is_contiguous() and ctx_lens.dtype == torch.int32
        assert k_cache.stride() == v_cache.stride() and k_cache.shape == v_cache.shape
        if shape is None:
            if max_ctx is None:
                max_ctx = k_cache.shape[1] if page_table is None else page_table.shape[1] * k_cache.shape[1]
            shape = self.attn_shape(q, k_cache, max_ctx, gamma=gamma, page_table=page_table,
                                    softmax_scale=softmax_scale, chunk_tokens=chunk_tokens,
                                    ctx_sum_hint=ctx_sum_hint)
        if out is None:
            out = torch.empty_like(q)
        need = self.lib.rapid_verify_attn_workspace_bytes(self._ctx, ctypes.byref(shape))
        ws = self._workspace(need)
        rc = self.lib.rapid_verify_attn(self._ctx, ctypes.byref(shape), _dptr(q), _dptr(k_cache), _dptr(v_cache),
                                        _dptr(ctx_lens), _dptr(gammas), _dptr(page_table), _dptr(out),
                                        _dptr(lse_out), _dptr(ws), ws.numel(), _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)
        return out

    def rapid_verify_attn_static(self, q, k_cache, v_cache, ctx_lens, gamma: Optional[int] = None, *, gammas=None,
                                 page_table=None, max_ctx: Optional[int] = None,
                                 softmax_scale: Optional[float] = None, chunk_tokens: int = 0, out, lse_out=None,
                                 ctx_sum_hint: int = 0):
        """The allocation-free form of :meth:`rapid_verify_attn`: the caller passes `out`, the split partials go
        to the library's static device array, and neither this method nor the library allocates anything."""
        if max_ctx is None:
            max_ctx = k_cache.shape[1] if page_table is None else page_table.shape[1] * k_cache.shape[1]
        shape = self.attn_shape(q, k_cache, max_ctx, gamma=gamma, page_table=page_table, softmax_scale=softmax_scale,
                                chunk_tokens=chunk_tokens, ctx_sum_hint=ctx_sum_hint)
        rc = self.lib.rapid_verify_attn_static(self._ctx, ctypes.byref(shape), _dptr(q), _dptr(k_cache),
                                               _dptr(v_cache), _dptr(ctx_lens), _dptr(gammas), _dptr(page_table),
                                               _dptr(out), _dptr(lse_out), _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)
        return out

    # ------------------------------------------------------------------ accept
    def rapid_accept(self, target_logits, draft_logits, draft_tokens, eta: float, uniforms, *, gammas=None,
                     temperature: float = 1.0, tail_alpha: float = 0.1, want_ratio: bool = True, outs=None,
                     target_stats=None, draft_stats=None):
        """target_logits fp32 [B,g+1,V], draft_logits fp32 [B,g,V], draft_tokens int32 [B,g],
        uniforms fp32 [B,g+1].  Returns (n_accepted int32 [B], out_tokens int32 [B,g+1], ratio fp32 [B,g] or None).
        target_stats / draft_stats: optional fp32 [rows, chunks, 2] row statistics (see rapid_lm_head); with
        either one the call goes to rapid_accept_prestats."""
        B, g1, V = target_logits.shape
        g = g1 - 1
        assert target_logits.dtype == torch.float32 and target_logits.is_contiguous()
        assert draft_logits.dtype == torch.float32 and draft_logits.is_contiguous() and draft_logits.shape == (B, g, V)
        assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, g) and draft_tokens.is_contiguous()
        assert uniforms.dtype == torch.float32 and uniforms.shape == (B, g + 1) and uniforms.is_contiguous()
        if outs is None:
            n_acc = torch.empty(B, dtype=torch.int32, device=self.device)
            toks = torch.empty(B, g + 1, dtype=torch.int32, device=self.device)
            ratio = torch.zeros(B, max(g, 1), dtype=torch.float32, device=self.device)[:, :g] if want_ratio else None
            if ratio is not None:
                ratio = ratio.contiguous()
        else:
            n_acc, toks, ratio = outs
        need = self.lib.rapid_accept_workspace_bytes(self._ctx, B, g, V)
        ws = self._accept_workspace(need)
        if target_stats is None and draft_stats is None:
            rc = self.lib.rapid_accept(self._ctx, B, g, V, _dptr(target_logits), _dptr(draft_logits),
                                       _dptr(draft_tokens), _dptr(gammas), float(eta), float(temperature),
                                       float(tail_alpha), _dptr(uniforms), _dptr(n_acc), _dptr(toks), _dptr(ratio),
                                       _dptr(ws), ws.numel(), _stream_ptr(self.device))
        else:
            for st, rows in ((target_stats, B * (g + 1)), (draft_stats, B * g)):
                assert st is None or (st.dtype == torch.float32 and st.is_contiguous() and st.dim() == 3
                                      and st.shape[0] == rows and st.shape[2] == 2)
            rc = self.lib.rapid_accept_prestats(
                self._ctx, B, g, V, _dptr(target_logits), _dptr(draft_logits), _dptr(draft_tokens), _dptr(gammas),
                float(eta), float(temperature), float(tail_alpha), _dptr(uniforms),
                _dptr(target_stats), 0 if target_stats is None else target_stats.shape[1],
                _dptr(draft_stats), 0 if draft_stats is None else draft_stats.shape[1],
                _dptr(n_acc), _dptr(toks), _dptr(ratio), _dptr(ws), ws.numel(), _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)
        return n_acc, toks, ratio

    # ------------------------------------------------------------------ cache bookkeeping
    def rapid_kv_append(self, k_cache, v_cache, k_new, v_new, ctx_lens, gamma: Optional[int] = None, *, gammas=None,
                        page_table=None, max_ctx: Optional[int] = None):
        """Writes rows 0..gamma_b of k_new/v_new (bf16 [B,Qmax,Hkv,d]) into the caches in place as the last
        gamma_b+1 tokens of every sequence (ctx_lens counts them).  Cache layout as for rapid_verify_attn."""
        B, Qmax, Hkv, d = k_new.shape
        assert k_new.is_contiguous() and v_new.is_contiguous() and v_new.shape == k_new.shape
        assert k_new.dtype == torch.bfloat16 and k_cache.dtype == torch.bfloat16
        q_like = k_new                                         # only sizes are read from it
        ctx_max = max_ctx if max_ctx is not None else (k_cache.shape[1] if page_table is None else
                                                       page_table.shape[1] * k_cache.shape[1])
        shape = self.attn_shape(q_like, k_cache, ctx_max, gamma=gamma if gamma is not None else Qmax - 1,
                                page_table=page_table)
        rc = self.lib.rapid_kv_append(self._ctx, ctypes.byref(shape), _dptr(k_new), _dptr(v_new), _dptr(ctx_lens),
                                      _dptr(gammas), _dptr(page_table), _dptr(k_cache), _dptr(v_cache),
                                      _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)

    def rapid_kv_commit(self, ctx_lens, n_accepted, gamma: int = 0, *, gammas=None):
        """ctx_lens[b] <- ctx_lens[b] - (gamma_b+1) + 1 + n_accepted[b], in place on the device."""
        assert ctx_lens.dtype == torch.int32 and n_accepted.dtype == torch.int32
        rc = self.lib.rapid_kv_commit(self._ctx, ctx_lens.numel(), int(gamma), _dptr(gammas), _dptr(n_accepted),
                                      _dptr(ctx_lens), _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)
        return ctx_lens

    def rapid_kv_commit_pages(self, ctx_lens, n_accepted, page_table, *, page_size: int, q_max: int, max_ctx: int,
                              gamma: Optional[int] = None, gammas=None, n_pages: int = 0):
        """The length update of :meth:`rapid_kv_commit` for a paged cache plus the page ids that can be handed
        back to the allocator.  Returns (released int32 [B, cap] (page ids, then -1), n_released int32 [B])."""
        B = ctx_lens.numel()
        s = AttnShape()
        s.batch, s.q_max, s.n_q_heads, s.n_kv_heads, s.head_dim = B, q_max, 1, 1, 128
        s.max_ctx, s.gamma, s.softmax_scale = int(max_ctx), (q_max - 1 if gamma is None else int(gamma)), 1.0
        s.kv_token_stride, s.kv_head_stride, s.kv_page_stride = 128, 128, 128 * page_size
        s.page_size, s.max_pages, s.n_pages = int(page_size), page_table.shape[1], int(n_pages)
        cap = (q_max + page_size - 2) // page_size + 1
        rel = torch.empty((B, cap), dtype=torch.int32, device=self.device)
        cnt = torch.empty(B, dtype=torch.int32, device=self.device)
        rc = self.lib.rapid_kv_commit_pages(self._ctx, ctypes.byref(s), _dptr(gammas), _dptr(n_accepted),
                                            _dptr(page_table), _dptr(ctx_lens), _dptr(rel), cap, _dptr(cnt),
                                            _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)
        return rel, cnt

    # ------------------------------------------------------------------ retrieval
    def rapid_retrieve(self, chunk_emb, query_emb, top_k: int, threshold: float = 0.3):
        """chunk_emb fp32 [n, dim], query_emb fp32 [dim] -> (similarity fp32 [n], selected int32 [top_k]
        (document order, then -1), n_selected int32 [1]); all on the device."""
        n, dim = chunk_emb.shape
        assert chunk_emb.dtype == torch.float32 and chunk_emb.is_contiguous()
        assert query_emb.dtype == torch.float32 and query_emb.is_contiguous() and query_emb.shape == (dim,)
        sim = torch.empty(n, dtype=torch.float32, device=self.device)
        sel = torch.empty(max(int(top_k), 1), dtype=torch.int32, device=self.device)
        cnt = torch.empty(1, dtype=torch.int32, device=self.device)
        rc = self.lib.rapid_retrieve(self._ctx, n, dim, _dptr(chunk_emb), _dptr(query_emb), int(top_k),
                                     float(threshold), _dptr(sim), _dptr(sel), _dptr(cnt), _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)
        return sim, sel, cnt

    # ------------------------------------------------------------------ output head
    def lm_head_chunk(self, vocab: int, n_rows: int = 1) -> int:
        """Vocabulary entries per statistics chunk that rapid_lm_head uses for this vocabulary and row count."""
        return self.lib.rapid_lm_head_chunk(self._ctx, int(vocab), int(n_rows))

    def rapid_lm_head(self, h, w, *, temperature: float = 1.0, want_stats: bool = True, logits=None, stats=None):
        """h bf16 [rows, hidden], w bf16 [vocab, hidden] -> (logits fp32 [rows, vocab],
        stats fp32 [rows, chunks, 2] or None); chunk size: :meth:`lm_head_chunk`."""
        rows, hidden = h.shape
        vocab = w.shape[0]
        assert h.dtype == torch.bfloat16 and w.dtype == torch.bfloat16 and h.is_contiguous() and w.is_contiguous()
        assert w.shape[1] == hidden
        if logits is None:
            logits = torch.empty(rows, vocab, dtype=torch.float32, device=self.device)
        assert logits.dtype == torch.float32 and logits.stride(-1) == 1 and logits.shape == (rows, vocab)
        if want_stats and stats is None:
            stats = torch.empty(rows, self.lib.rapid_lm_head_stat_chunks(self._ctx, vocab, rows), 2, dtype=torch.float32,
                                device=self.device)
        rc = self.lib.rapid_lm_head(self._ctx, rows, hidden, vocab, _dptr(h), _dptr(w), float(temperature),
                                    _dptr(logits), logits.stride(0) if rows > 1 else vocab,
                                    _dptr(stats) if want_stats else None, _stream_ptr(self.device))
        _check(self.lib, rc, self._ctx)
        return logits, (stats if want_stats else None)

    # ------------------------------------------------------------------ measurement aid
    def rapid_hbm_read_probe(self, buf: torch.Tensor, nbytes: Optional[int] = None):
        """Streams the first `nbytes` bytes (default: all, rounded down to 16 KiB) of a dense tensor's
        memory through the attention kernel's load path; for timing only."""
        total = buf.numel() * buf.element_size()
        nbytes = (total if nbytes is None else nbytes) // 16384 * 16384
        if self._sink is None:
            self._sink = torch.zeros(1, dtype=torch.int32, device=self.device)
        _check(self.lib, self.lib.rapid_hbm_read_probe(self._ctx, _dptr(buf), nbytes, _dptr(self._sink),
                                                       _stream_ptr(self.device)), self._ctx)
        return nbytes


_default: dict = {}

def _get(device: int = 0) -> Rapid:
    if device not in _default:
        _default[device] = Rapid(device)
    return _default[device]


def rapid_verify_attn(q, k_cache, v_cache, ctx_lens, gamma=None, **kw):
    """Module-level form of :meth:`Rapid.rapid_verify_attn` on the tensors' device."""
    return _get(q.device.index or 0).rapid_verify_attn(q, k_cache, v_cache, ctx_lens, gamma, **kw)


def rapid_lm_head(h, w, **kw):
    """Module-level form of :meth:`Rapid.rapid_lm_head` on the tensors' device."""
    return _get(h.device.index or 0).rapid_lm_head(h, w, **kw)


def rapid_accept(target_logits, draft_logits, draft_tokens, eta, uniforms, **kw):
    """Module-level form of :meth:`Rapid.rapid_accept` on the tensors' device."""
    return _get(target_logits.device.index or 0).rapid_accept(target_logits, draft_logits, draft_tokens, eta,
                                                              uniforms, **kw)
