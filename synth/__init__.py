"""Seeded synthetic inputs for GPT-NeoX/Pythia-shaped decode blocks.

This module only draws random numbers and lays them out in the canonical
GPT-NeoX tensor shapes.  It holds none of the decode arithmetic and is the
only code shared by the CPU oracle's tests and the HIP path's tests/bench.

Recipe (the synthetic stand-in for trained Pythia checkpoints and prompts,
which are not available offline): every tensor is drawn in fp32 from its own
(seed, layer, tensor-id) stream and rounded once to fp16 (round to nearest
even); both sides consume those same fp16 values.

    weights, biases  ~ N(0, 0.02)
    LN gamma         = 1 + N(0, 0.02),  LN beta ~ N(0, 0.02)
    x                ~ N(0, 1)
    cached K, V      ~ N(0, 1) for positions < S; NaN (tests) or 0 (bench) after
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, asdict

import numpy as np

MASTER_SEED = 23553

# tensor ids (second key of the per-tensor stream)
_TID = {
    "ln1_g": 1, "ln1_b": 2, "ln2_g": 3, "ln2_b": 4,
    "w_qkv": 5, "b_qkv": 6, "w_dense": 7, "b_dense": 8,
    "w_up": 9, "b_up": 10, "w_down": 11, "b_down": 12,
    "k_cache": 13, "v_cache": 14, "x": 15,
    "lnf_g": 16, "lnf_b": 17, "w_lm": 18, "seq_lens": 19, "embed": 20,
}
LAYER_TENSORS = ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "w_qkv", "b_qkv",
                 "w_dense", "b_dense", "w_up", "b_up", "w_down", "b_down")


FLAG_TANH_GELU = 1               # GELU by its tanh approximation instead of erf
FLAG_SEQUENTIAL_RESIDUAL = 2     # x1 = x + attention; out = x1 + MLP(LN2(x1)) instead of the parallel form


@dataclass(frozen=True)
class ModelShape:
    """Shape of one GPT-NeoX decoder block (names follow the model family)."""
    hidden: int
    n_heads: int
    head_dim: int
    rotary_dims: int
    ffn: int
    n_layers: int = 1
    rope_base: float = 10000.0
    ln_eps: float = 1e-5
    name: str = ""
    flags: int = 0          # FLAG_* bits: which reading of the block is meant (0 = GPT-NeoX / Pythia)

    def __post_init__(self):
        assert self.hidden == self.n_heads * self.head_dim

    def as_dict(self):
        return asdict(self)


# The five workload shapes the benchmarks and parity tests use.
SMALL_BLOCK = ModelShape(512, 8, 64, 16, 2048, 1, name="neox-h512")
PYTHIA_2_8B = ModelShape(2560, 32, 80, 20, 10240, 32, name="pythia-2.8b-shape")
PYTHIA_6_9B = ModelShape(4096, 32, 128, 32, 16384, 32, name="pythia-6.9b-shape")
VOCAB = 50304


def _rng(seed: int, layer: int, name: str) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(layer), _TID[name]])


def _normal_f16(rng, shape, std=1.0, mean=0.0) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return a.astype(np.float16)


def layer_tensor(shape: ModelShape, seed: int, layer: int, name: str) -> np.ndarray:
    h, f = shape.hidden, shape.ffn
    dims = {
        "ln1_g": (h,), "ln1_b": (h,), "ln2_g": (h,), "ln2_b": (h,),
        "w_qkv": (3 * h, h), "b_qkv": (3 * h,),
        "w_dense": (h, h), "b_dense": (h,),
        "w_up": (f, h), "b_up": (f,),
        "w_down": (h, f), "b_down": (h,),
    }[name]
    mean = 1.0 if name in ("ln1_g", "ln2_g") else 0.0
    return _normal_f16(_rng(seed, layer, name), dims, 0.02, mean)


def layer_weights(shape: ModelShape, seed: int = MASTER_SEED, layer: int = 0) -> dict:
    """The 12 canonical fp16 tensors of one block.

    w_qkv rows are ordered (head, {q,k,v}, dim): row (3*n + c)*head_dim + i.
    """
    return {n: layer_tensor(shape, seed, layer, n) for n in LAYER_TENSORS}


def kv_cache(shape: ModelShape, seed: int, layer: int, n_cached, capacity: int,
             batch: int = 1, poison: bool = True):
    """K, V as fp16 [batch, n_heads, capacity, head_dim]; positions < n_cached[b]
    are N(0,1), later slots are NaN (poison=True) or zero."""
    n_cached = np.broadcast_to(np.asarray(n_cached, dtype=np.int64), (batch,))
    assert int(n_cached.max(initial=0)) <= capacity
    fill = np.float16(np.nan) if poison else np.float16(0)
    out = []
    for name in ("k_cache", "v_cache"):
        rng = _rng(seed, layer, name)
        c = np.full((batch, shape.n_heads, capacity, shape.head_dim), fill, dtype=np.float16)
        for b in range(batch):
            s = int(n_cached[b])
            if s:
                c[b, :, :s, :] = _normal_f16(rng, (shape.n_heads, s, shape.head_dim))
        out.append(c)
    return out[0], out[1]


def x_input(shape: ModelShape, seed: int = MASTER_SEED, batch: int = 1) -> np.ndarray:
    return _normal_f16(_rng(seed, 0, "x"), (batch, shape.hidden))


def lm_head(shape: ModelShape, seed: int = MASTER_SEED, vocab: int = VOCAB) -> dict:
    """Final LayerNorm parameters and an untied random LM head [vocab, hidden]."""
    return {
        "lnf_g": _normal_f16(_rng(seed, 0, "lnf_g"), (shape.hidden,), 0.02, 1.0),
        "lnf_b": _normal_f16(_rng(seed, 0, "lnf_b"), (shape.hidden,), 0.02),
        "w_lm": _normal_f16(_rng(seed, 0, "w_lm"), (vocab, shape.hidden), 0.02),
    }


def embedding(shape: ModelShape, seed: int = MASTER_SEED, vocab: int = VOCAB) -> np.ndarray:
    """Random token embedding table [vocab, hidden], rows ~ N(0, 1) like the block input x."""
    return _normal_f16(_rng(seed, 0, "embed"), (vocab, shape.hidden))


def seq_lens(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """Per-sequence cached lengths, uniform in [lo, hi] inclusive."""
    return _rng(seed, 0, "seq_lens").integers(lo, hi + 1, size=batch).astype(np.int32)


def stack_weights(shape: ModelShape, seed: int = MASTER_SEED, workers: int = 8):
    """All layers' weights; layers are generated in parallel threads (numpy's
    generators release the GIL) but each tensor's values depend only on
    (seed, layer, name)."""
    with ThreadPoolExecutor(max_workers=workers) as ex:
        return list(ex.map(lambda l: layer_weights(shape, seed, l), range(shape.n_layers)))
