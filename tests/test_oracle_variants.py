"""Pins of the two alternative readings the oracle offers behind flags: the
tanh form of GELU (the paper says "accelerated GELU", Sec. 2.2, without naming
the flavour) and the sequential residual (Sec. 2.2 lists the chain as output
projection with residual -> post-attention LayerNorm -> MLP with residual).
CPU only."""
import dataclasses
import math

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import synth
from tests import bruteforce
from tests.test_oracle_block import tiny_case, f16


def test_tanh_gelu_closed_form_and_library(orc):
    z = np.linspace(-8, 8, 4001)
    got = orc.gelu_tanh(z)
    want = np.array([0.5 * t * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (t + 0.044715 * t ** 3))) for t in z])
    assert np.abs(got - want).max() < 1e-15
    torch = pytest.importorskip("torch")
    lib = torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy()
    assert np.abs(got - lib).max() < 1e-12
    assert orc.gelu_tanh(np.zeros(1))[0] == 0.0
    assert np.abs(orc.gelu_tanh(z) - orc.gelu_tanh(-z) - z).max() < 1e-12     # odd part is z/2, as for erf
    # an approximation of the erf form, not the same function
    d = np.abs(got - orc.gelu(z))
    assert 1e-4 < d.max() < 1e-3


@settings(max_examples=20, deadline=None)
@given(seed=st.integers(0, 10_000), H=st.integers(1, 3), S=st.integers(0, 4), flags=st.sampled_from([1, 2, 3]))
def test_variants_match_pure_python_brute_force(orc, seed, H, S, flags):
    shape, w, K, V, x = tiny_case(seed, h_per=4, H=H, r=2, f=8 * H, S=S)
    shape = dataclasses.replace(shape, flags=flags)
    wl = {k: v.astype(np.float64).tolist() for k, v in w.items()}
    want, _, _ = bruteforce.block(shape, wl, K.astype(np.float64).tolist(), V.astype(np.float64).tolist(), S,
                                  x.astype(np.float64).tolist(), lambda t: float(np.float16(t)))
    got = orc.block_decode(shape, w, K, V, S, x.astype(np.float64))
    assert np.abs(got - np.array(want)).max() < 1e-9 * max(1.0, np.abs(want).max())


def test_sequential_form_reduces_to_parallel_without_attention_branch_and_differs_with_it(orc):
    shape, w, K, V, x = tiny_case(5, h_per=8, H=2, r=2, f=32, S=4)
    seq = dataclasses.replace(shape, flags=synth.FLAG_SEQUENTIAL_RESIDUAL)
    xr = x.astype(np.float64)
    z = lambda k: np.zeros_like(w[k])
    w0 = dict(w, w_dense=z("w_dense"), b_dense=z("b_dense"))          # attention branch == 0
    a = orc.block_decode(shape, w0, K.copy(), V.copy(), 4, xr)
    b = orc.block_decode(seq, w0, K.copy(), V.copy(), 4, xr)
    assert np.array_equal(a, b)
    # with the attention branch a constant c: the sequential block equals the
    # parallel block evaluated on x + c with the attention branch switched off
    c = f16(np.linspace(-1, 1, 16))
    wc = dict(w0, b_dense=c)
    got = orc.block_decode(seq, wc, K.copy(), V.copy(), 4, xr)
    x1 = xr + c.astype(np.float64)
    y2 = orc.layernorm(x1, w["ln2_g"], w["ln2_b"], shape.ln_eps)
    g = orc.gemv(w["w_down"], w["b_down"], orc.gelu(orc.gemv(w["w_up"], w["b_up"], y2)))
    assert np.abs(got - (x1 + g)).max() < 1e-12
    par = orc.block_decode(shape, wc, K.copy(), V.copy(), 4, xr)
    assert np.abs(got - par).max() > 1e-3                              # the two readings do differ


def test_variants_match_independent_gpt_neox_layer(orc):
    """transformers' GPTNeoXLayer with use_parallel_residual=False and the tanh
    activation is an independent implementation of both variants at once."""
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    from transformers.models.gpt_neox import modeling_gpt_neox as m
    sh = dataclasses.replace(synth.SMALL_BLOCK, flags=3)
    try:
        cfg = tr.GPTNeoXConfig(hidden_size=sh.hidden, num_attention_heads=sh.n_heads,
                               intermediate_size=sh.ffn, num_hidden_layers=1, vocab_size=128,
                               max_position_embeddings=4096, use_parallel_residual=False,
                               hidden_act="gelu_pytorch_tanh")
        cfg._attn_implementation = "eager"
        layer = m.GPTNeoXLayer(cfg, 0).double().eval()
        rot = m.GPTNeoXRotaryEmbedding(cfg).double()
        cache = tr.DynamicCache()
    except Exception as e:  # API drift in the installed library
        pytest.skip(f"transformers API not as expected: {e}")
    w = synth.layer_weights(sh, 98, 0)
    t = lambda a: torch.from_numpy(a.astype(np.float64))
    layer.load_state_dict({
        "input_layernorm.weight": t(w["ln1_g"]), "input_layernorm.bias": t(w["ln1_b"]),
        "post_attention_layernorm.weight": t(w["ln2_g"]), "post_attention_layernorm.bias": t(w["ln2_b"]),
        "attention.query_key_value.weight": t(w["w_qkv"]), "attention.query_key_value.bias": t(w["b_qkv"]),
        "attention.dense.weight": t(w["w_dense"]), "attention.dense.bias": t(w["b_dense"]),
        "mlp.dense_h_to_4h.weight": t(w["w_up"]), "mlp.dense_h_to_4h.bias": t(w["b_up"]),
        "mlp.dense_4h_to_h.weight": t(w["w_down"]), "mlp.dense_4h_to_h.bias": t(w["b_down"]),
    }, strict=True)
    S = 29
    K, V = synth.kv_cache(sh, 98, 0, S, S + 1)
    x = synth.x_input(sh, 98)
    cache.update(t(K[:, :, :S]), t(V[:, :, :S]), 0)
    pos_ids = torch.tensor([[S]])
    hs = t(x)[None]
    with torch.no_grad():
        out = layer(hs, attention_mask=None, position_ids=pos_ids, layer_past=cache,
                    position_embeddings=rot(hs, pos_ids))
    out = (out[0] if isinstance(out, tuple) else out).reshape(-1).numpy()
    got = orc.block_decode(sh, w, K[0].copy(), V[0].copy(), S, x[0].astype(np.float64))
    assert np.abs(got - out).max() < 2e-5
    assert np.linalg.norm(got - out) / np.linalg.norm(out) < 2e-6
