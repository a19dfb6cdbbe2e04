"""ctypes front end of the C oracle (see neox_block_oracle.c for what each
routine computes and which passage of the paper it follows).

Test infrastructure only.  All arrays are numpy; fp16 tensors are passed as
their bit patterns.  KV caches here are in the canonical layout
[n_heads, capacity, head_dim] per sequence.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_U16P = C.POINTER(C.c_uint16)


class _Shape(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("rotary_dims", C.c_int32), ("ffn", C.c_int32),
                ("rope_base", C.c_double), ("ln_eps", C.c_double)]


_LAYER_FIELDS = ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "w_qkv", "b_qkv",
                 "w_dense", "b_dense", "w_up", "b_up", "w_down", "b_down")


class _Layer(C.Structure):
    _fields_ = [(n, _U16P) for n in _LAYER_FIELDS]


_TAP_FIELDS = ("y1", "y2", "q", "attn", "a", "m", "g", "k_new", "v_new")


class _Taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _TAP_FIELDS]


def _u16(a: np.ndarray):
    assert a.dtype == np.float16 and a.flags.c_contiguous
    return a.view(np.uint16).ctypes.data_as(_U16P)


class Oracle:
    """One compiled variant of the oracle ('f64' or 'f32')."""

    def __init__(self, variant: str = "f64"):
        _build.build()
        self.lib = C.CDLL(_build.lib_path(variant))
        self.real = {8: np.float64, 4: np.float32}[self.lib.orc_sizeof_real()]
        self._creal = {8: C.c_double, 4: C.c_float}[self.lib.orc_sizeof_real()]
        L = self.lib
        L.orc_half_to_real.restype = self._creal
        L.orc_half_to_real.argtypes = [C.c_uint16]
        L.orc_real_to_half.restype = C.c_uint16
        L.orc_real_to_half.argtypes = [self._creal]
        L.orc_gelu.restype = self._creal
        L.orc_gelu.argtypes = [self._creal]
        L.orc_block_decode.restype = C.c_int
        L.orc_block_decode_flags.restype = C.c_int

    # -- helpers ---------------------------------------------------------
    def _r(self, a):
        return np.ascontiguousarray(a, dtype=self.real)

    def _rp(self, a):
        return a.ctypes.data_as(C.c_void_p)

    @staticmethod
    def shape_struct(shape) -> _Shape:
        return _Shape(shape.hidden, shape.n_heads, shape.head_dim, shape.rotary_dims,
                      shape.ffn, float(shape.rope_base), float(shape.ln_eps))

    # -- conversions -----------------------------------------------------
    def half_to_real(self, a: np.ndarray) -> np.ndarray:
        a = np.ascontiguousarray(a, dtype=np.float16)
        out = np.empty(a.shape, dtype=self.real)
        self.lib.orc_half_to_real_n(_u16(a), self._rp(out), C.c_int64(a.size))
        return out

    def real_to_half(self, a) -> np.ndarray:
        a = self._r(a)
        out = np.empty(a.shape, dtype=np.float16)
        self.lib.orc_real_to_half_n(self._rp(a), _u16(out), C.c_int64(a.size))
        return out

    # -- steps -----------------------------------------------------------
    def layernorm(self, x, gamma=None, beta=None, eps=1e-5):
        x = self._r(x)
        y = np.empty_like(x)
        self.lib.orc_layernorm(self._rp(x), _u16(gamma) if gamma is not None else None,
                               _u16(beta) if beta is not None else None,
                               C.c_int(x.size), C.c_double(eps), self._rp(y))
        return y

    def gemv(self, W, b, v):
        v = self._r(v)
        rows, cols = W.shape
        assert v.size == cols
        out = np.empty(rows, dtype=self.real)
        self.lib.orc_gemv(_u16(W), _u16(b) if b is not None else None, self._rp(v),
                          C.c_int(rows), C.c_int(cols), self._rp(out))
        return out

    def rope(self, u, r, pos, base=10000.0):
        u = self._r(u).copy()
        self.lib.orc_rope(self._rp(u), C.c_int(r), C.c_int(pos), C.c_double(base))
        return u

    def attention_head(self, q, Kh, Vh, n_pos, return_probs=False):
        q = self._r(q)
        d = q.size
        assert Kh.shape[1] == d and Vh.shape[1] == d and Kh.shape[0] >= n_pos
        o = np.empty(d, dtype=self.real)
        p = np.empty(n_pos, dtype=self.real) if return_probs else None
        self.lib.orc_attention_head(self._rp(q), _u16(Kh), _u16(Vh), C.c_int(n_pos), C.c_int(d),
                                    self._rp(o), self._rp(p) if p is not None else None)
        return (o, p) if return_probs else o

    def gelu(self, z):
        z = self._r(z)
        out = np.empty_like(z)
        self.lib.orc_gelu_n(self._rp(z), self._rp(out), C.c_int64(z.size))
        return out

    # -- the block -------------------------------------------------------
    def gelu_tanh(self, z):
        z = self._r(z)
        out = np.empty_like(z)
        self.lib.orc_gelu_tanh_n(self._rp(z), self._rp(out), C.c_int64(z.size))
        return out

    def block_decode(self, shape, w: dict, K: np.ndarray, V: np.ndarray, pos: int, x,
                     taps: bool = False, flags: int | None = None):
        """One sequence.  K, V: fp16 [n_heads, capacity, head_dim], updated in
        place at row `pos`.  x: [hidden] (any float dtype; used as given).
        Returns the unrounded block output (and a dict of intermediates)."""
        assert K.dtype == np.float16 and K.flags.c_contiguous and V.flags.c_contiguous
        H, cap, d = K.shape
        assert (H, d) == (shape.n_heads, shape.head_dim) and V.shape == K.shape
        x = self._r(x).reshape(-1)
        assert x.size == shape.hidden
        lay = _Layer(*[_u16(w[n]) for n in _LAYER_FIELDS])
        sh = self.shape_struct(shape)
        out = np.empty(shape.hidden, dtype=self.real)
        tp, tap_arrays = None, {}
        if taps:
            sizes = {n: shape.hidden for n in _TAP_FIELDS}
            sizes["m"] = shape.ffn
            tap_arrays = {n: np.empty(sizes[n], dtype=self.real) for n in _TAP_FIELDS}
            tp = C.byref(_Taps(*[self._rp(tap_arrays[n]) for n in _TAP_FIELDS]))
        if flags is None:
            flags = int(getattr(shape, "flags", 0))      # 1: tanh GELU, 2: sequential residual
        rc = self.lib.orc_block_decode_flags(C.byref(sh), C.byref(lay), _u16(K), _u16(V),
                                             C.c_int(cap), C.c_int(pos), self._rp(x), self._rp(out), tp,
                                             C.c_int(flags))
        if rc != 0:
            raise ValueError("orc_block_decode: bad argument")
        return (out, tap_arrays) if taps else out

    def block_decode_f16(self, shape, w, K, V, pos, x_f16):
        """The block at its fp16 boundary: fp16 x in, fp16-rounded output."""
        return self.real_to_half(self.block_decode(shape, w, K, V, pos, self.half_to_real(x_f16)))

    def stack_decode(self, shape, layers, Ks, Vs, pos: int, x_f16, per_layer=None, taps_per_layer=None):
        """L blocks in sequence for one sequence.  The residual stream between
        blocks stays unrounded (`real`); fp16 only at entry and exit.
        per_layer (optional list) receives every layer's unrounded output,
        taps_per_layer (optional list) every layer's dict of intermediates."""
        x = self.half_to_real(np.asarray(x_f16).reshape(-1))
        for l, w in enumerate(layers):
            if taps_per_layer is not None:
                x, t = self.block_decode(shape, w, Ks[l], Vs[l], pos, x, taps=True)
                taps_per_layer.append(t)
            else:
                x = self.block_decode(shape, w, Ks[l], Vs[l], pos, x)
            if per_layer is not None:
                per_layer.append(x.copy())
        return self.real_to_half(x), x

    # -- prompt processing (paper Sec. 4.2 "Prefill Phase" names it without a
    #    formula: what it computes is the stack applied to every prompt token
    #    with causal attention, which is one decode step per token, in order) ---
    def prefill(self, shape, layers, Ks, Vs, pos0: int, X_f16):
        """X_f16: fp16 [T, hidden] prompt rows for positions pos0 .. pos0 + T - 1 of
        one sequence whose first pos0 rows are cached.  Ks, Vs are updated in
        place.  Returns (fp16 [T, hidden] outputs, unrounded [T, hidden])."""
        X = np.asarray(X_f16)
        out16, out = [], []
        for t in range(X.shape[0]):
            o16, o = self.stack_decode(shape, layers, Ks, Vs, pos0 + t, X[t])
            out16.append(o16)
            out.append(o)
        return np.stack(out16), np.stack(out)

    def lm_head_logits(self, shape, head: dict, x, eps=None):
        x = self._r(x).reshape(-1)
        vocab = head["w_lm"].shape[0]
        logits = np.empty(vocab, dtype=self.real)
        self.lib.orc_lm_head(_u16(head["lnf_g"]), _u16(head["lnf_b"]), _u16(head["w_lm"]),
                             self._rp(x), C.c_int(shape.hidden), C.c_int(vocab),
                             C.c_double(shape.ln_eps if eps is None else eps), self._rp(logits))
        return logits

    # -- greedy generation (the steps either side of the stack: paper Sec. 2.3
    #    replays one graph per generated token; Sec. 3 compares generated tokens
    #    with the baseline's and does not name the picking rule: argmax here) --
    def next_token(self, shape, head: dict, hidden_f16):
        """Final LayerNorm + LM head on the stack's fp16 output, then the index of
        the largest logit (the lowest index among equal maxima)."""
        logits = self.lm_head_logits(shape, head, self.half_to_real(np.asarray(hidden_f16).reshape(-1)))
        return int(np.argmax(logits)), logits

    def generate(self, shape, layers, Ks, Vs, head: dict, embed: np.ndarray, tokens, pos: int,
                 n_steps: int, trace: list | None = None):
        """n_steps greedy decode steps for one sequence.  tokens[pos] is the token
        whose K/V rows are appended at row `pos`; each step embeds it (fp16 table
        row), runs the stack, and picks tokens[pos + 1].  Ks, Vs are updated in
        place.  Returns the token list extended by n_steps entries; `trace`
        (optional) receives (hidden_f16, logits) of every step."""
        tokens = list(tokens)
        assert len(tokens) == pos + 1
        for _ in range(n_steps):
            x = np.ascontiguousarray(embed[tokens[pos]])
            hidden16, _ = self.stack_decode(shape, layers, Ks, Vs, pos, x)
            tok, logits = self.next_token(shape, head, hidden16)
            if trace is not None:
                trace.append((hidden16.copy(), logits))
            tokens.append(tok)
            pos += 1
        return tokens


_cache = {}


def load(variant: str = "f64") -> Oracle:
    if variant not in _cache:
        _cache[variant] = Oracle(variant)
    return _cache[variant]
