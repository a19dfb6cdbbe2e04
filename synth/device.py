"""Seeded synthetic inputs generated on the GPU (torch's device generator), for
workloads whose tensors are too large to draw on the host in a benchmark's time
budget (a 32-layer 6.9B-shaped stack is 13 GB).  Same laws as the numpy
generators of this package: weights and biases ~ N(0, 0.02), LayerNorm gamma =
1 + N(0, 0.02), beta ~ N(0, 0.02), cached K/V ~ N(0, 1), every value rounded once
to fp16.  The streams differ from the numpy ones (another generator), so these
tensors serve timing only; parity tests use the numpy generators, whose values
the CPU oracle sees too.  No arithmetic of the decode path lives here."""
import torch

from . import LAYER_TENSORS, MASTER_SEED


def _gen(device, seed, layer):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(layer)) & 0x7FFFFFFFFFFF)
    return g


def layer_tensors(shape, seed: int = MASTER_SEED, layer: int = 0, device="cuda:0") -> dict:
    """The 12 canonical fp16 tensors of one block, on `device`."""
    h, f = shape.hidden, shape.ffn
    dims = {"ln1_g": (h,), "ln1_b": (h,), "ln2_g": (h,), "ln2_b": (h,), "w_qkv": (3 * h, h), "b_qkv": (3 * h,),
            "w_dense": (h, h), "b_dense": (h,), "w_up": (f, h), "b_up": (f,), "w_down": (h, f), "b_down": (h,)}
    g = _gen(device, seed, layer)
    out = {}
    for n in LAYER_TENSORS:
        t = torch.randn(dims[n], generator=g, device=device, dtype=torch.float32) * 0.02
        if n in ("ln1_g", "ln2_g"):
            t = t + 1.0
        out[n] = t.to(torch.float16)
    return out


def fill_kv(kv_bytes: torch.Tensor, seed: int = MASTER_SEED, layer: int = 0):
    """Every slot of a layer's cache (any layout: a flat uint8 tensor of fp16 values) ~ N(0, 1)."""
    g = _gen(kv_bytes.device, seed + 7, layer)
    v = kv_bytes.view(torch.float16)
    v.copy_(torch.randn(v.shape, generator=g, device=kv_bytes.device, dtype=torch.float32).to(torch.float16))
