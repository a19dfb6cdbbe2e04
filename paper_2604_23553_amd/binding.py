"""ctypes binding of libcfpp.so: same names as include/cfpp.h, argument
marshalling only.  Device pointers are passed as integers (tensor.data_ptr())
or as objects with a data_ptr() method; streams as integers
(torch.cuda.current_stream().cuda_stream) or None for the default stream.

There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import contextlib
import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))

OPT_MODE, OPT_GRID, OPT_THREADS = 1, 2, 3
LAYER_TENSORS = ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "w_qkv", "b_qkv",
                 "w_dense", "b_dense", "w_up", "b_up", "w_down", "b_down")


class CfppError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__(f"{where}: status {status} ({detail})")
        self.status = status


class Config(C.Structure):
    """Mirror of `cfpp_config`."""
    _fields_ = [("hidden", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("rotary_dims", C.c_int32), ("ffn", C.c_int32), ("n_layers", C.c_int32),
                ("max_seq", C.c_int32), ("max_batch", C.c_int32),
                ("rope_base", C.c_float), ("ln_eps", C.c_float), ("flags", C.c_int32)]

    @classmethod
    def from_shape(cls, shape, max_seq: int, max_batch: int = 1, n_layers: int | None = None):
        return cls(shape.hidden, shape.n_heads, shape.head_dim, shape.rotary_dims, shape.ffn,
                   shape.n_layers if n_layers is None else n_layers, max_seq, max_batch,
                   float(shape.rope_base), float(shape.ln_eps), int(getattr(shape, "flags", 0)))


class _LayerSrc(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_TENSORS]


OPT_PROFILE_SKIP, OPT_EPOCH_LIMIT = 100, 101          # profiling library only
MODE_AUTO = -1

_LIBS = {"product": "libcfpp.so", "profile": "libcfpp_profile.so"}
_loaded = {}
_active = "product"


def library_path(kind: str = "product") -> str:
    """Path of the in-tree library: the product, or the profiling build of the same sources."""
    return os.path.join(_PKG, _LIBS[kind])


def _load(kind: str) -> C.CDLL:
    if kind not in _loaded:
        path = library_path(kind)
        if not os.path.exists(path):
            raise FileNotFoundError(
                f"{path} is missing: build the HIP library with "
                "`python -m paper_2604_23553_amd.build` (there is no fallback path)")
        L = C.CDLL(path)
        L.cfpp_status_string.restype = C.c_char_p
        L.cfpp_last_error.restype = C.c_char_p
        for n in ("cfpp_packed_layer_bytes", "cfpp_kv_layer_bytes", "cfpp_workspace_bytes"):
            getattr(L, n).restype = C.c_size_t
            getattr(L, n).argtypes = [C.POINTER(Config)]
        L.cfpp_prefill_scratch_bytes.restype = C.c_size_t
        L.cfpp_prefill_scratch_bytes.argtypes = [C.POINTER(Config), C.c_int32]
        L.cfpp_destroy.restype = None
        L.cfpp_destroy.argtypes = [C.c_void_p]
        _loaded[kind] = L
    return _loaded[kind]


def lib() -> C.CDLL:
    """The library the calls below go to: the product (libcfpp.so) unless a
    `with profile_build():` block is active."""
    return _load(_active)


@contextlib.contextmanager
def profile_build():
    """Routes the calls made inside the block to libcfpp_profile.so (tracer, skip
    bits, test taps, calibration kernels: include/cfpp_profile.h).  A context
    created inside the block must be used and destroyed inside it."""
    global _active
    before = _active
    _active = "profile"
    try:
        yield _load("profile")
    finally:
        _active = before


def _ptr(t) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if hasattr(t, "data_ptr"):
        t = t.data_ptr()
    return C.c_void_p(int(t))


def _check(st: int, where: str):
    if st != 0:
        L = lib()
        raise CfppError(st, where, f"{L.cfpp_status_string(st).decode()}: {L.cfpp_last_error().decode()}")


def cfpp_validate_config(cfg: Config) -> int:
    """Returns the status code (0 = supported); does not raise."""
    return int(lib().cfpp_validate_config(C.byref(cfg)))


def cfpp_packed_layer_bytes(cfg: Config) -> int:
    return int(lib().cfpp_packed_layer_bytes(C.byref(cfg)))


def cfpp_kv_layer_bytes(cfg: Config) -> int:
    return int(lib().cfpp_kv_layer_bytes(C.byref(cfg)))


def cfpp_workspace_bytes(cfg: Config) -> int:
    return int(lib().cfpp_workspace_bytes(C.byref(cfg)))


def cfpp_algorithmic_bytes(cfg: Config, pos_host, n_layers: int) -> int:
    pos = (C.c_int32 * len(pos_host))(*[int(p) for p in pos_host])
    out = C.c_uint64(0)
    _check(lib().cfpp_algorithmic_bytes(C.byref(cfg), pos, C.c_int32(len(pos_host)),
                                        C.c_int32(n_layers), C.byref(out)), "cfpp_algorithmic_bytes")
    return int(out.value)


def cfpp_pack_layer(cfg: Config, src: dict, packed_dst, stream=None):
    s = _LayerSrc(*[_ptr(src[n]) for n in LAYER_TENSORS])
    _check(lib().cfpp_pack_layer(C.byref(cfg), C.byref(s), _ptr(packed_dst), _ptr(stream)),
           "cfpp_pack_layer")


def cfpp_kv_import(cfg: Config, k_src, v_src, src_capacity: int, n_pos: int, b: int, kv_layer,
                   stream=None):
    _check(lib().cfpp_kv_import(C.byref(cfg), _ptr(k_src), _ptr(v_src), C.c_int32(src_capacity),
                                C.c_int32(n_pos), C.c_int32(b), _ptr(kv_layer), _ptr(stream)),
           "cfpp_kv_import")


def cfpp_kv_export(cfg: Config, kv_layer, b: int, pos_begin: int, n_pos: int, dst_capacity: int,
                   k_dst, v_dst, stream=None):
    _check(lib().cfpp_kv_export(C.byref(cfg), _ptr(kv_layer), C.c_int32(b), C.c_int32(pos_begin),
                                C.c_int32(n_pos), C.c_int32(dst_capacity), _ptr(k_dst), _ptr(v_dst),
                                _ptr(stream)), "cfpp_kv_export")


def cfpp_create(cfg: Config, workspace, workspace_bytes: int) -> int:
    """Returns the opaque context handle (an integer)."""
    ctx = C.c_void_p(0)
    _check(lib().cfpp_create(C.byref(cfg), _ptr(workspace), C.c_size_t(workspace_bytes),
                             C.byref(ctx)), "cfpp_create")
    return int(ctx.value)


def cfpp_destroy(ctx: int):
    lib().cfpp_destroy(C.c_void_p(ctx))


def cfpp_set_option(ctx: int, option: int, value: int):
    _check(lib().cfpp_set_option(C.c_void_p(ctx), C.c_int32(option), C.c_int64(value)),
           "cfpp_set_option")


def cfpp_get_option(ctx: int, option: int) -> int:
    v = C.c_int64(0)
    _check(lib().cfpp_get_option(C.c_void_p(ctx), C.c_int32(option), C.byref(v)), "cfpp_get_option")
    return int(v.value)


def cfpp_block_decode(ctx: int, packed_layer, kv_layer, x, pos_dev, batch: int, out, stream=None):
    _check(lib().cfpp_block_decode(C.c_void_p(ctx), _ptr(packed_layer), _ptr(kv_layer), _ptr(x),
                                   _ptr(pos_dev), C.c_int32(batch), _ptr(out), _ptr(stream)),
           "cfpp_block_decode")


def _ptr_array(items):
    return (C.c_void_p * len(items))(*[_ptr(t).value or 0 for t in items])


def cfpp_stack_decode(ctx: int, packed_layers, kv_layers, x, pos_dev, batch: int, out, stream=None):
    _check(lib().cfpp_stack_decode(C.c_void_p(ctx), _ptr_array(packed_layers), _ptr_array(kv_layers),
                                   _ptr(x), _ptr(pos_dev), C.c_int32(batch), _ptr(out), _ptr(stream)),
           "cfpp_stack_decode")


def cfpp_stack_prefill(ctx: int, packed_layers, kv_layers, x, pos0: int, n_tokens: int, b: int, out, stream=None):
    _check(lib().cfpp_stack_prefill(C.c_void_p(ctx), _ptr_array(packed_layers), _ptr_array(kv_layers),
                                    _ptr(x), C.c_int32(pos0), C.c_int32(n_tokens), C.c_int32(b), _ptr(out),
                                    _ptr(stream)),
           "cfpp_stack_prefill")


def cfpp_prefill_scratch_bytes(cfg: Config, rows: int) -> int:
    return int(lib().cfpp_prefill_scratch_bytes(C.byref(cfg), C.c_int32(rows)))


def cfpp_stack_prefill_gemm(ctx: int, packed_layers, kv_layers, x, pos0: int, n_tokens: int, b: int, out, scratch,
                            scratch_bytes: int, rows: int, stream=None):
    _check(lib().cfpp_stack_prefill_gemm(C.c_void_p(ctx), _ptr_array(packed_layers), _ptr_array(kv_layers),
                                         _ptr(x), C.c_int32(pos0), C.c_int32(n_tokens), C.c_int32(b), _ptr(out),
                                         _ptr(scratch), C.c_size_t(scratch_bytes), C.c_int32(rows), _ptr(stream)),
           "cfpp_stack_prefill_gemm")


def cfpp_stack_capture(ctx: int, packed_layers, kv_layers, x, pos_dev, batch: int, out, stream):
    _check(lib().cfpp_stack_capture(C.c_void_p(ctx), _ptr_array(packed_layers), _ptr_array(kv_layers),
                                    _ptr(x), _ptr(pos_dev), C.c_int32(batch), _ptr(out), _ptr(stream)),
           "cfpp_stack_capture")


def cfpp_stack_replay(ctx: int, stream):
    _check(lib().cfpp_stack_replay(C.c_void_p(ctx), _ptr(stream)), "cfpp_stack_replay")


class Lm(C.Structure):
    """cfpp_lm: device pointers of the embedding table, final LayerNorm and LM head."""
    _fields_ = [("embed", C.c_void_p), ("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p), ("w_lm", C.c_void_p),
                ("vocab", C.c_int32)]

    @classmethod
    def of(cls, embed, lnf_g, lnf_b, w_lm, vocab: int):
        return cls(_ptr(embed).value, _ptr(lnf_g).value, _ptr(lnf_b).value, _ptr(w_lm).value, int(vocab))


def cfpp_lm_embed(ctx: int, lm: Lm, tokens_dev, pos_dev, x, stream=None):
    _check(lib().cfpp_lm_embed(C.c_void_p(ctx), C.byref(lm), _ptr(tokens_dev), _ptr(pos_dev), _ptr(x),
                               _ptr(stream)), "cfpp_lm_embed")


def cfpp_lm_next(ctx: int, lm: Lm, hidden, tokens_dev, pos_dev, logits_dev=None, stream=None):
    _check(lib().cfpp_lm_next(C.c_void_p(ctx), C.byref(lm), _ptr(hidden), _ptr(tokens_dev), _ptr(pos_dev),
                              _ptr(logits_dev), _ptr(stream)), "cfpp_lm_next")


def cfpp_generate_capture(ctx: int, packed_layers, kv_layers, lm: Lm, tokens_dev, pos_dev, x_buf, hidden_buf,
                          stream):
    _check(lib().cfpp_generate_capture(C.c_void_p(ctx), _ptr_array(packed_layers), _ptr_array(kv_layers),
                                       C.byref(lm), _ptr(tokens_dev), _ptr(pos_dev), _ptr(x_buf),
                                       _ptr(hidden_buf), _ptr(stream)), "cfpp_generate_capture")


def cfpp_device_error(ctx: int, stream=None):
    """Synchronises the stream; raises CfppError if a kernel flagged an error."""
    _check(lib().cfpp_device_error(C.c_void_p(ctx), _ptr(stream)), "cfpp_device_error")


def cfpp_block_decode_static(cfg: Config, packed_layer, kv_layer, x, pos_dev, batch: int, out, stream=None):
    _check(lib().cfpp_block_decode_static(C.byref(cfg), _ptr(packed_layer), _ptr(kv_layer), _ptr(x),
                                          _ptr(pos_dev), C.c_int32(batch), _ptr(out), _ptr(stream)),
           "cfpp_block_decode_static")


# ---- profiling library only (inside `with profile_build():`) -------------------
def cfpp_debug_read(ctx: int, which: int, count: int, stream=None):
    import numpy as np
    out = np.empty(count, dtype=np.float32)
    _check(lib().cfpp_debug_read(C.c_void_p(ctx), C.c_int32(which),
                                 out.ctypes.data_as(C.POINTER(C.c_float)), C.c_size_t(count),
                                 _ptr(stream)), "cfpp_debug_read")
    return out


def cfpp_stream_read(src, nbytes: int, sink, grid: int, threads: int, unroll: int, stream=None):
    _check(lib().cfpp_stream_read(_ptr(src), C.c_size_t(nbytes), _ptr(sink), C.c_int32(grid),
                                  C.c_int32(threads), C.c_int32(unroll), _ptr(stream)), "cfpp_stream_read")


def cfpp_stream_copy(src, dst, nbytes: int, grid: int, threads: int, stream=None):
    _check(lib().cfpp_stream_copy(_ptr(src), _ptr(dst), C.c_size_t(nbytes), C.c_int32(grid),
                                  C.c_int32(threads), _ptr(stream)), "cfpp_stream_copy")
