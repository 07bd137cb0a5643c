"""Python-side marshalling for libspec.so: packed weights, contexts, and the single-kernel calls."""
from __future__ import annotations

import atexit
import ctypes as C
import weakref
from typing import Callable, List, Optional

import numpy as np
import torch

from . import (ALGO_AR, ALGO_PEARL, ALGO_SD, PAGE_TOKENS, SPEC_MAX_TOKENS, Config, ModelDesc, Weights, check,
               load_library)


def _ptr(t: torch.Tensor) -> int:
    return t.data_ptr()


def _stream_ptr(s) -> int:
    return 0 if s is None else int(s.cuda_stream)


class PackedModel:
    """Device weights of one decoder in the library's layouts (projections panel-packed)."""

    def __init__(self, shape):
        self.shape = shape
        self.tok_embed = None
        self.final_norm = None
        self.lm_head = None
        self.layers: List[dict] = []
        self._keep = []

    def prefix(self, n_layers: int, shape) -> "PackedModel":
        """A model that shares the first n_layers layers, embedding, final norm and LM head."""
        m = PackedModel(shape)
        m.tok_embed, m.final_norm, m.lm_head = self.tok_embed, self.final_norm, self.lm_head
        m.layers = self.layers[:n_layers]
        return m

    def desc(self) -> ModelDesc:
        s = self.shape
        return ModelDesc(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab,
                         s.rope_theta, s.rms_eps)

    def c_weights(self) -> Weights:
        n = len(self.layers)
        arr = lambda key: (C.c_void_p * n)(*[_ptr(l[key]) for l in self.layers])
        w = Weights()
        w.tok_embed, w.final_norm, w.lm_head = _ptr(self.tok_embed), _ptr(self.final_norm), _ptr(self.lm_head)
        self._arrays = {k: arr(k) for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gateup", "w_down")}
        for k, v in self._arrays.items():
            setattr(w, k, C.cast(v, C.POINTER(C.c_void_p)))
        return w

    def nbytes(self) -> int:
        seen, total = set(), 0
        ts = [self.tok_embed, self.final_norm, self.lm_head] + [t for l in self.layers for t in l.values()]
        for t in ts:
            if t.data_ptr() not in seen:
                seen.add(t.data_ptr())
                total += t.numel() * t.element_size()
        return total


def _pack_into(dst: torch.Tensor, src: torch.Tensor, panel_start: int, panel_step: int):
    lib = load_library()
    assert src.dtype == torch.bfloat16 and src.is_contiguous() and src.is_cuda
    N, K = src.shape
    check(lib.spec_pack_weight(_ptr(dst), _ptr(src), N, K, panel_start, panel_step,
                               _stream_ptr(torch.cuda.current_stream())))


def pack_matrices(mats: List[torch.Tensor], interleave: bool = False) -> torch.Tensor:
    """Pack row-major bf16 matrices [N_i][K] into one panel-packed buffer (concatenated or interleaved)."""
    lib = load_library()
    K = mats[0].shape[1]
    total = sum(lib.spec_packed_bytes(m.shape[0], K) for m in mats)
    dst = torch.empty(total // 2, dtype=torch.bfloat16, device=mats[0].device)
    if interleave:
        assert all(m.shape == mats[0].shape for m in mats)
        for i, m in enumerate(mats):
            _pack_into(dst, m, i, len(mats))
    else:
        start = 0
        for m in mats:
            _pack_into(dst, m, start, 1)
            start += m.shape[0] // 16
    return dst


def pack_model(shape, get: Callable[[Optional[int], str], torch.Tensor], device="cuda") -> PackedModel:
    """Build a PackedModel.  get(layer or None, name) returns the row-major bf16 tensor on `device`;
    each source is dropped as soon as it is packed, so peak memory is the packed model plus one layer."""
    pm = PackedModel(shape)
    pm.tok_embed = get(None, "tok_embed").contiguous()
    pm.final_norm = get(None, "final_norm").contiguous()
    pm.lm_head = pack_matrices([get(None, "lm_head")])
    for l in range(shape.n_layers):
        lay = {"attn_norm": get(l, "attn_norm").contiguous(), "ffn_norm": get(l, "ffn_norm").contiguous()}
        lay["wqkv"] = pack_matrices([get(l, "wq"), get(l, "wk"), get(l, "wv")])
        lay["wo"] = pack_matrices([get(l, "wo")])
        lay["w_gateup"] = pack_matrices([get(l, "w_gate"), get(l, "w_up")], interleave=True)
        lay["w_down"] = pack_matrices([get(l, "w_down")])
        pm.layers.append(lay)
    torch.cuda.synchronize()
    return pm


def pack_from_dict(shape, w: dict, device="cuda") -> PackedModel:
    """Pack generator weights given as a dict of (CPU or GPU) tensors; values are cast to bf16."""
    def get(layer, name):
        t = w[name] if layer is None else w["layers"][layer][name]
        return t.to(device=device, dtype=torch.bfloat16).contiguous()
    return pack_model(shape, get, device)


_live_contexts = weakref.WeakSet()


@atexit.register
def _close_live_contexts():
    """No program leaves with live HIP objects of this library: contexts still open at interpreter exit are freed
    (graphs, events, device memory, then the streams made for them), and the device is drained before the runtime's
    own teardown starts."""
    for ctx in list(_live_contexts):
        try:
            ctx.close()
        except Exception:
            pass
    try:
        if torch.cuda.is_initialized():
            torch.cuda.synchronize()
    except Exception:
        pass


class SpecContext:
    """One target/draft pair with its caches: the calls of include/spec.h as methods."""

    def __init__(self, target: PackedModel, draft: PackedModel, gamma_max: int, max_seq: int,
                 temperature: float = 1.0, logit_scale: float = 1.0, stream_target=None, stream_draft=None,
                 on_close=None):
        """on_close: called after the context is freed (e.g. to destroy streams made for it)."""
        self.lib = load_library()
        self._on_close = on_close
        self.target, self.draft = target, draft
        self.stream_target = stream_target or torch.cuda.Stream()
        self.stream_draft = stream_draft or torch.cuda.Stream()
        self.vocab = target.shape.vocab
        cfg = Config(gamma_max, max_seq, PAGE_TOKENS, temperature, logit_scale,
                     _stream_ptr(self.stream_target), _stream_ptr(self.stream_draft))
        td, dd = target.desc(), draft.desc()
        tw, dw = target.c_weights(), draft.c_weights()
        self._ctx = C.c_void_p()
        torch.cuda.synchronize()
        check(self.lib.spec_init(C.byref(cfg), C.byref(td), C.byref(tw), C.byref(dd), C.byref(dw),
                                 C.byref(self._ctx)))
        self.gamma_max = gamma_max
        _live_contexts.add(self)

    def close(self):
        if getattr(self, "_ctx", None):
            self.lib.spec_free(self._ctx)
            self._ctx = None
            if self._on_close:
                self._on_close()
                self._on_close = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the six calls -------------------------------------------------------------------
    def prefill(self, prompt, which_mask: int = 3):
        arr = np.ascontiguousarray(np.asarray(prompt, dtype=np.int32))
        check(self.lib.spec_prefill(self._ctx, arr.ctypes.data_as(C.POINTER(C.c_int32)), len(arr), which_mask))

    def draft_step(self, u: float, want_token: bool = False):
        out = C.c_int32(-1)
        check(self.lib.spec_draft_step(self._ctx, float(u), C.byref(out) if want_token else None))
        return out.value if want_token else None

    def verify(self, tokens=None, n_tokens: Optional[int] = None, want_logits: bool = False):
        if tokens is not None:
            arr = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
            n = len(arr)
            tp = arr.ctypes.data_as(C.POINTER(C.c_int32))
        else:
            n, tp = int(n_tokens), None
        logits = np.empty((n, self.vocab), dtype=np.float32) if want_logits else None
        lp = logits.ctypes.data_as(C.POINTER(C.c_float)) if want_logits else None
        check(self.lib.spec_verify(self._ctx, tp, n, lp))
        return logits

    def verify_guess(self, guess=None, n_guess: int = 0, want_logits: bool = False):
        """Target forward over the frontier and guessed continuations (pre-verify of several draft tokens).  `guess`:
        the caller's tokens, or None for up to n_guess tokens of the library's own pool.  Returns (guesses fed, logits
        [fed + 1, vocab] or None)."""
        if guess is not None:
            arr = np.ascontiguousarray(np.asarray(guess, dtype=np.int32))
            n, gp = len(arr), arr.ctypes.data_as(C.POINTER(C.c_int32))
        else:
            n, gp = int(n_guess), None
        logits = np.empty((n + 1, self.vocab), dtype=np.float32) if want_logits else None
        lp = logits.ctypes.data_as(C.POINTER(C.c_float)) if want_logits else None
        fed = C.c_int(-1)
        check(self.lib.spec_verify_guess(self._ctx, gp, n, C.byref(fed), lp))
        return fed.value, (logits[:fed.value + 1] if want_logits else None)

    def pending_rows(self) -> int:
        return check(self.lib.spec_pending_rows(self._ctx))

    def accept(self, kind: int, r=(), u_resample: float = 0.5, force_mask: int = -1):
        r = np.ascontiguousarray(np.asarray(r, dtype=np.float32))
        n_acc, n_out, mode, keep = C.c_int(), C.c_int(), C.c_int(), C.c_int()
        toks = (C.c_int32 * (SPEC_MAX_TOKENS + 1))()
        check(self.lib.spec_accept(self._ctx, kind, r.ctypes.data_as(C.POINTER(C.c_float)), len(r), float(u_resample),
                                   int(force_mask), C.byref(n_acc), toks, C.byref(n_out), C.byref(mode),
                                   C.byref(keep)))
        return {"n_accepted": n_acc.value, "tokens": [toks[i] for i in range(n_out.value)],
                "next_mode": mode.value, "keep_len": keep.value}

    def rollback_kv(self, which: int, new_len: int):
        check(self.lib.spec_rollback_kv(self._ctx, which, new_len))

    def drop_drafts(self):
        check(self.lib.spec_drop_drafts(self._ctx))

    def rewind(self, committed_len: int):
        check(self.lib.spec_rewind(self._ctx, committed_len))

    def kv_len(self, which: int) -> int:
        return check(self.lib.spec_kv_len(self._ctx, which))

    def committed_len(self) -> int:
        return check(self.lib.spec_committed_len(self._ctx))

    def free_pages(self, which: int) -> int:
        return check(self.lib.spec_kv_free_pages(self._ctx, which))

    def forward_count(self, which: int) -> int:
        return int(self.lib.spec_forward_count(self._ctx, which))

    # ---- loops ---------------------------------------------------------------------------
    def generate(self, algo: int, gamma: int, n_generate: int, uniforms, force_bits=None, max_steps: int = 0):
        """Run AR / SD / PEARL for n_generate tokens.  `uniforms` has .draft [T,g], .accept [T,g+1], .resample [T]."""
        f32 = lambda a: np.ascontiguousarray(np.asarray(a, dtype=np.float32))
        ud, ra, ur = f32(uniforms.draft), f32(uniforms.accept), f32(uniforms.resample)
        g = max(gamma, 1)
        # a step commits at least one token, except the draft-only steps of algo 3 (at most every other step)
        need = max_steps if max_steps > 0 else n_generate * (2 if algo == 3 else 1)
        if algo != ALGO_AR:
            assert ud.shape == (ud.shape[0], g) and ra.shape == (ra.shape[0], g + 1)
            assert ud.shape[0] >= need and ra.shape[0] >= need
        assert ur.shape[0] >= need
        fb = None
        if force_bits is not None:
            fb = np.ascontiguousarray(np.asarray(force_bits, dtype=np.uint8))
            assert fb.shape[0] >= need and fb.shape[1] == g + 1
        n_out = min(n_generate, need * (g + 1))
        out = np.empty(n_out, dtype=np.int32)
        stats = np.zeros(8, dtype=np.float64)
        pf = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
        check(self.lib.spec_generate(self._ctx, algo, gamma, n_out, int(max_steps), pf(ud), pf(ra), pf(ur),
                                     fb.ctypes.data_as(C.POINTER(C.c_uint8)) if fb is not None else None,
                                     out.ctypes.data_as(C.POINTER(C.c_int32)),
                                     stats.ctypes.data_as(C.POINTER(C.c_double))))
        keys = ["steps", "committed", "draft_forwards", "target_forwards", "accepted", "tested", "post_steps", "seconds"]
        st = dict(zip(keys, stats.tolist()))
        return out[:min(n_out, int(st["committed"]))].tolist(), st

    def calibrate_gamma(self, n_iter: int = 8, cap: int = 16, concurrent: bool = False):
        """(gamma, seconds per target forward, seconds per draft forward): gamma = round(c) of Section 4.4.1."""
        g, tp, tq = C.c_int(), C.c_double(), C.c_double()
        check(self.lib.spec_calibrate_gamma(self._ctx, int(n_iter), int(cap), 1 if concurrent else 0, C.byref(g),
                                            C.byref(tp), C.byref(tq)))
        return g.value, tp.value, tq.value

    def set_option(self, option: int, value: int):
        check(self.lib.spec_set_option(self._ctx, option, value))

    def get_option(self, option: int) -> int:
        v = C.c_int()
        check(self.lib.spec_get_option(self._ctx, option, C.byref(v)))
        return v.value

    # ---- profiling -----------------------------------------------------------------------
    def set_profile(self, flags: int):
        check(self.lib.spec_set_profile(self._ctx, flags))

    def profile_read(self):
        ms, n, b = C.c_double(), C.c_longlong(), C.c_double()
        check(self.lib.spec_profile_read(self._ctx, C.byref(ms), C.byref(n), C.byref(b)))
        return ms.value, n.value, b.value


# ---- single kernels -------------------------------------------------------------------------
def gemm(x: torch.Tensor, w_packed: torch.Tensor, N: int, partials_only: bool = False) -> Optional[torch.Tensor]:
    """y[M][N] fp32 = x[M][K] (bf16) * W^T, W panel-packed; runs on torch's current stream."""
    lib = load_library()
    assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.is_cuda
    M, K = x.shape
    nb = lib.spec_gemm_workspace_bytes(M, N, K)
    if nb == 0:
        check(-1)
    work = torch.empty(nb // 4, dtype=torch.float32, device=x.device)
    st = _stream_ptr(torch.cuda.current_stream())
    if partials_only:
        check(lib.spec_gemm_partials(_ptr(x), _ptr(w_packed), M, N, K, _ptr(work), st))
        return None
    y = torch.empty((M, N), dtype=torch.float32, device=x.device)
    check(lib.spec_gemm(_ptr(y), _ptr(x), _ptr(w_packed), M, N, K, _ptr(work), st))
    return y


def dense_gemm(x: torch.Tensor, w_packed: torch.Tensor, N: int, epilogue: int = 0,
               y: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The prompt-sized matrix-core projection, on torch's current stream.

    epilogue 0: returns y[M][N] fp32 = x W^T; 1: adds x W^T into the given y; 2: returns z[M][N/2] bf16 =
    silu(gate) * up for a gate/up matrix with interleaved 16-row panels."""
    lib = load_library()
    assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.is_cuda
    M, K = x.shape
    st = _stream_ptr(torch.cuda.current_stream())
    if epilogue == 2:
        z = torch.empty((M, N // 2), dtype=torch.bfloat16, device=x.device)
        check(lib.spec_dense_gemm(None, _ptr(z), _ptr(x), _ptr(w_packed), M, N, K, 2, st))
        return z
    if epilogue == 1:
        assert y is not None and y.dtype == torch.float32 and y.is_contiguous() and tuple(y.shape) == (M, N)
    else:
        y = torch.empty((M, N), dtype=torch.float32, device=x.device)
    check(lib.spec_dense_gemm(_ptr(y), None, _ptr(x), _ptr(w_packed), M, N, K, epilogue, st))
    return y


def sample_row(logits: torch.Tensor, temperature: float, logit_scale: float, u: float):
    lib = load_library()
    assert logits.dtype == torch.float32 and logits.is_contiguous() and logits.dim() == 1
    q = torch.empty_like(logits)
    tok = torch.empty(1, dtype=torch.int32, device=logits.device)
    check(lib.spec_sample_row(_ptr(logits), logits.numel(), float(temperature), float(logit_scale), float(u), _ptr(q),
                              _ptr(tok), _stream_ptr(torch.cuda.current_stream())))
    return q, int(tok.item())


def accept_rows(p_logits: torch.Tensor, q_rows: Optional[torch.Tensor], x, r, temperature: float, logit_scale: float,
                u_resample: float):
    lib = load_library()
    assert p_logits.dtype == torch.float32 and p_logits.is_contiguous()
    n_rows, V = p_logits.shape
    n_test = len(x)
    xd = torch.tensor(list(x), dtype=torch.int32, device=p_logits.device) if n_test else None
    rr = np.ascontiguousarray(np.asarray(r, dtype=np.float32))
    res = (C.c_int32 * 2)()
    check(lib.spec_accept_rows(_ptr(p_logits), n_rows, _ptr(q_rows) if n_test else None, _ptr(xd) if n_test else None,
                               n_test, V, float(temperature), float(logit_scale),
                               rr.ctypes.data_as(C.POINTER(C.c_float)), float(u_resample), res,
                               _stream_ptr(torch.cuda.current_stream())))
    return res[0], res[1]


def accept_rows_static(p_logits: torch.Tensor, q_rows: Optional[torch.Tensor], x: Optional[torch.Tensor], r,
                       temperature: float, logit_scale: float, u_resample: float, result: torch.Tensor):
    """spec_accept_rows_static on torch's current stream: allocates nothing (x and result are the caller's device
    tensors: int32 [n_test] and int32 [2]); asynchronous."""
    lib = load_library()
    assert p_logits.dtype == torch.float32 and p_logits.is_contiguous()
    assert result.dtype == torch.int32 and result.numel() >= 2 and result.is_cuda
    n_rows, V = p_logits.shape
    n_test = 0 if x is None else int(x.numel())
    rr = np.ascontiguousarray(np.asarray(r, dtype=np.float32))
    check(lib.spec_accept_rows_static(_ptr(p_logits), n_rows, _ptr(q_rows) if n_test else None,
                                      _ptr(x) if n_test else None, n_test, V, float(temperature), float(logit_scale),
                                      rr.ctypes.data_as(C.POINTER(C.c_float)), float(u_resample), _ptr(result),
                                      _stream_ptr(torch.cuda.current_stream())))


def read_probe(buf: torch.Tensor):
    lib = load_library()
    out = torch.zeros(4, dtype=torch.int32, device=buf.device)
    check(lib.spec_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(out),
                              _stream_ptr(torch.cuda.current_stream())))
