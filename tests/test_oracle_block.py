"""Block-level pins for the oracle: the residual form, the QKV row convention,
the KV append, brute force on tiny shapes, an independent third-party
implementation of the same architecture, and the paper's printed shape facts."""
import json
import math
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import synth
from tests import bruteforce

HERE = os.path.dirname(os.path.abspath(__file__))


def f16(a):
    return np.asarray(a, dtype=np.float16)


def tiny_case(seed, h_per=4, H=2, r=2, f=16, S=3, std=0.5):
    shape = synth.ModelShape(H * h_per, H, h_per, r, f)
    rng = np.random.default_rng(seed)
    h = shape.hidden
    w = {
        "ln1_g": f16(1 + 0.1 * rng.standard_normal(h)), "ln1_b": f16(0.1 * rng.standard_normal(h)),
        "ln2_g": f16(1 + 0.1 * rng.standard_normal(h)), "ln2_b": f16(0.1 * rng.standard_normal(h)),
        "w_qkv": f16(std * rng.standard_normal((3 * h, h))), "b_qkv": f16(std * rng.standard_normal(3 * h)),
        "w_dense": f16(std * rng.standard_normal((h, h))), "b_dense": f16(std * rng.standard_normal(h)),
        "w_up": f16(std * rng.standard_normal((f, h))), "b_up": f16(std * rng.standard_normal(f)),
        "w_down": f16(std * rng.standard_normal((h, f))), "b_down": f16(std * rng.standard_normal(h)),
    }
    K = np.full((H, S + 1, h_per), np.nan, dtype=np.float16)
    V = np.full((H, S + 1, h_per), np.nan, dtype=np.float16)
    K[:, :S] = f16(rng.standard_normal((H, S, h_per)))
    V[:, :S] = f16(rng.standard_normal((H, S, h_per)))
    x = f16(rng.standard_normal(h))
    return shape, w, K, V, x


@settings(max_examples=25, deadline=None)
@given(seed=st.integers(0, 10_000), H=st.integers(1, 3), dq=st.integers(1, 3),
       S=st.integers(0, 5), rq=st.integers(0, 2))
def test_block_matches_pure_python_brute_force(orc, seed, H, dq, S, rq):
    d = 4 * dq
    r = min(d, 2 * rq)
    shape, w, K, V, x = tiny_case(seed, h_per=d, H=H, r=r, f=4 * H * d, S=S)
    wl = {k: v.astype(np.float64).tolist() for k, v in w.items()}
    rh = lambda t: float(np.float16(t))
    want, k_new, v_new = bruteforce.block(shape, wl, K.astype(np.float64).tolist(),
                                          V.astype(np.float64).tolist(), S,
                                          x.astype(np.float64).tolist(), rh)
    got = orc.block_decode(shape, w, K, V, S, x.astype(np.float64))
    assert np.abs(got - np.array(want)).max() < 1e-9 * max(1.0, np.abs(want).max())
    # appended rows: equal to the brute force's fp16 k, v up to one fp16 ulp at
    # rounding ties (the two sides sum in different orders)
    assert np.abs(K[:, S].astype(np.float64) - np.array(k_new)).max() <= 2.0 ** -10 * np.abs(k_new).max() + 1e-12
    assert np.abs(V[:, S].astype(np.float64) - np.array(v_new)).max() <= 2.0 ** -10 * np.abs(v_new).max() + 1e-12


def test_block_matches_independent_gpt_neox_layer(orc):
    """transformers' GPTNeoXLayer (random init, float64, eager attention) loaded
    with the same tensors is an independent implementation of the architecture:
    it pins the per-head interleaved QKV rows, half-split partial rotary, the
    parallel residual, eps, the dense bias and the erf GELU together."""
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    from transformers.models.gpt_neox import modeling_gpt_neox as m
    sh = synth.SMALL_BLOCK
    try:
        cfg = tr.GPTNeoXConfig(hidden_size=sh.hidden, num_attention_heads=sh.n_heads,
                               intermediate_size=sh.ffn, num_hidden_layers=1, vocab_size=128,
                               max_position_embeddings=4096)
        cfg._attn_implementation = "eager"
        layer = m.GPTNeoXLayer(cfg, 0).double().eval()
        rot = m.GPTNeoXRotaryEmbedding(cfg).double()
        cache = tr.DynamicCache()
    except Exception as e:  # API drift in the installed library
        pytest.skip(f"transformers API not as expected: {e}")
    assert cfg.use_parallel_residual and cfg.hidden_act == "gelu" and cfg.layer_norm_eps == 1e-5
    w = synth.layer_weights(sh, 99, 0)
    t = lambda a: torch.from_numpy(a.astype(np.float64))
    layer.load_state_dict({
        "input_layernorm.weight": t(w["ln1_g"]), "input_layernorm.bias": t(w["ln1_b"]),
        "post_attention_layernorm.weight": t(w["ln2_g"]), "post_attention_layernorm.bias": t(w["ln2_b"]),
        "attention.query_key_value.weight": t(w["w_qkv"]), "attention.query_key_value.bias": t(w["b_qkv"]),
        "attention.dense.weight": t(w["w_dense"]), "attention.dense.bias": t(w["b_dense"]),
        "mlp.dense_h_to_4h.weight": t(w["w_up"]), "mlp.dense_h_to_4h.bias": t(w["b_up"]),
        "mlp.dense_4h_to_h.weight": t(w["w_down"]), "mlp.dense_4h_to_h.bias": t(w["b_down"]),
    }, strict=True)
    S = 37
    K, V = synth.kv_cache(sh, 99, 0, S, S + 1)
    x = synth.x_input(sh, 99)
    cache.update(t(K[:, :, :S]), t(V[:, :, :S]), 0)
    pos_ids = torch.tensor([[S]])
    hs = t(x)[None]
    with torch.no_grad():
        out = layer(hs, attention_mask=None, position_ids=pos_ids, layer_past=cache,
                    position_embeddings=rot(hs, pos_ids))
    out = (out[0] if isinstance(out, tuple) else out).reshape(-1).numpy()
    Ko, Vo = K[0].copy(), V[0].copy()
    got, taps = orc.block_decode(sh, w, Ko, Vo, S, x[0].astype(np.float64), taps=True)
    # the only difference: the library keeps the new token's k, v unrounded
    assert np.abs(got - out).max() < 2e-5
    assert np.linalg.norm(got - out) / np.linalg.norm(out) < 2e-6
    # its cache now holds the (unrounded) new k, v: ours are their fp16 roundings
    k_lib = cache.layers[0].keys[0, :, S].numpy() if hasattr(cache, "layers") else None
    if k_lib is not None:
        # (equal except where different summation orders straddle a rounding boundary)
        diff = Ko[:, S] != k_lib.astype(np.float16)
        assert diff.mean() < 0.01
        assert np.abs(Ko[:, S].astype(np.float64) - k_lib).max() <= 2.0 ** -11 * np.abs(k_lib).max()


def test_residual_form_is_parallel(orc):
    shape, w, K, V, x = tiny_case(3, h_per=8, H=2, r=2, f=32, S=4)
    xr = x.astype(np.float64)
    z = lambda k: np.zeros_like(w[k])
    # both output matrices zero, biases zero -> out == x exactly
    w0 = dict(w, w_dense=z("w_dense"), w_down=z("w_down"), b_dense=z("b_dense"), b_down=z("b_down"))
    assert np.array_equal(orc.block_decode(shape, w0, K.copy(), V.copy(), 4, xr), xr)
    # only the two biases -> out = x + c1 + c2
    c1, c2 = f16(np.full(16, 0.5)), f16(np.full(16, -0.125))
    w1 = dict(w0, b_dense=c1, b_down=c2)
    assert np.array_equal(orc.block_decode(shape, w1, K.copy(), V.copy(), 4, xr), xr + 0.375)
    # parallel form: the MLP branch must not see the attention branch.  With
    # W_dense = 0 the attention branch is the constant b_dense = c; (out - c)
    # would change with c if LN2 read x + attention (the sequential form).
    outs = []
    for c in (0.0, 3.0):
        wc = dict(w, w_dense=z("w_dense"), b_dense=f16(np.full(16, c)))
        # vary c non-uniformly so LayerNorm cannot absorb it
        wc["b_dense"][::2] = 0
        outs.append(orc.block_decode(shape, wc, K.copy(), V.copy(), 4, xr) - wc["b_dense"].astype(np.float64))
    assert np.abs(outs[0] - outs[1]).max() < 1e-12


def test_qkv_rows_are_interleaved_per_head(orc):
    """Row (3n + c) * d + i of W_qkv feeds q/k/v (c = 0/1/2) of head n, dim i."""
    H, d, S = 3, 8, 2
    shape, w, K, V, x = tiny_case(5, h_per=d, H=H, r=0, f=16, S=S)
    for c, n, i in [(1, 2, 5), (2, 1, 3), (1, 0, 0), (2, 2, 7)]:
        wq = dict(w, w_qkv=np.zeros_like(w["w_qkv"]), b_qkv=np.zeros_like(w["b_qkv"]))
        wq["b_qkv"][(3 * n + c) * d + i] = 1.5
        Kc, Vc = K.copy(), V.copy()
        orc.block_decode(shape, wq, Kc, Vc, S, x.astype(np.float64))
        tgt, other = (Kc, Vc) if c == 1 else (Vc, Kc)
        want = np.zeros((H, d))
        want[n, i] = 1.5
        assert np.array_equal(tgt[:, S].astype(np.float64), want)
        assert np.array_equal(other[:, S].astype(np.float64), np.zeros((H, d)))
    # c = 0 (q): a huge q component on dim i of head n selects the cached key with
    # the largest K[n, t, i]; the tap shows it in (head, dim) order
    wq = dict(w, w_qkv=np.zeros_like(w["w_qkv"]), b_qkv=np.zeros_like(w["b_qkv"]))
    wq["b_qkv"][(3 * 1 + 0) * d + 4] = 2.0
    _, taps = orc.block_decode(shape, wq, K.copy(), V.copy(), S, x.astype(np.float64), taps=True)
    want = np.zeros(H * d)
    want[1 * d + 4] = 2.0
    assert np.array_equal(taps["q"], want)


def test_kv_append_writes_only_row_pos(orc):
    sh = synth.SMALL_BLOCK
    w = synth.layer_weights(sh, 5, 0)
    K, V = synth.kv_cache(sh, 5, 0, 20, 24)
    K, V = K[0], V[0]
    K0, V0 = K.copy(), V.copy()
    x = synth.x_input(sh, 5)[0]
    _, taps = orc.block_decode(sh, w, K, V, 20, x.astype(np.float64), taps=True)
    for new, old in ((K, K0), (V, V0)):
        mask = np.ones(24, bool)
        mask[20] = False
        assert np.array_equal(new[:, mask].view(np.uint16), old[:, mask].view(np.uint16))
        assert not np.isnan(new[:, 20]).any()
    # the appended k is RoPE(W_k y1 + b_k) rounded once to fp16: recompute with numpy
    y1 = taps["y1"]
    qkv = w["w_qkv"].astype(np.float64) @ y1 + w["b_qkv"].astype(np.float64)
    qkv = qkv.reshape(sh.n_heads, 3, sh.head_dim)
    assert np.array_equal(V[:, 20], qkv[:, 2].astype(np.float16))
    k = np.stack([orc.rope(qkv[n, 1], sh.rotary_dims, 20) for n in range(sh.n_heads)])
    assert np.array_equal(K[:, 20], k.astype(np.float16))


def test_rejects_bad_position(orc):
    shape, w, K, V, x = tiny_case(1)
    with pytest.raises(ValueError):
        orc.block_decode(shape, w, K, V, K.shape[1], x.astype(np.float64))


def test_f32_and_f64_variants_agree(orc, orc32):
    sh = synth.SMALL_BLOCK
    w = synth.layer_weights(sh, 11, 0)
    K, V = synth.kv_cache(sh, 11, 0, 128, 129)
    x = synth.x_input(sh, 11)[0]
    a = orc.block_decode(sh, w, K[0].copy(), V[0].copy(), 128, x.astype(np.float64))
    b = orc32.block_decode(sh, w, K[0].copy(), V[0].copy(), 128, x.astype(np.float32))
    assert np.abs(a - b).max() < 2e-5


def test_stack_composes_blocks_and_keeps_residual_unrounded(orc):
    sh = synth.ModelShape(64, 4, 16, 4, 256, n_layers=3)
    layers = synth.stack_weights(sh, 3)
    kv = [synth.kv_cache(sh, 3, l, 5, 6) for l in range(3)]
    Ks, Vs = [k[0][0].copy() for k in kv], [k[1][0].copy() for k in kv]
    x = synth.x_input(sh, 3)[0]
    per = []
    out16, out = orc.stack_decode(sh, layers, Ks, Vs, 5, x, per_layer=per)
    cur = x.astype(np.float64)
    for l in range(3):
        cur = orc.block_decode(sh, layers[l], kv[l][0][0].copy(), kv[l][1][0].copy(), 5, cur)
        assert np.array_equal(cur, per[l])
    assert np.array_equal(out16, cur.astype(np.float16))


def test_lm_head_and_argmax_tie_break(orc):
    sh = synth.ModelShape(64, 4, 16, 4, 256)
    head = synth.lm_head(sh, 4, vocab=300)
    x = np.random.default_rng(4).standard_normal(64)
    z = orc.layernorm(x, head["lnf_g"], head["lnf_b"], sh.ln_eps)
    want = head["w_lm"].astype(np.float64) @ z
    got = orc.lm_head_logits(sh, head, x)
    assert np.abs(got - want).max() < 1e-13
    head["w_lm"][200] = head["w_lm"][17]        # duplicate row -> tie, lowest index wins
    lg = orc.lm_head_logits(sh, head, x)
    lg[[17, 200]] = lg.max() + 1
    assert int(np.argmax(lg)) == 17


def test_paper_shape_facts():
    """The sizes the paper prints for Pythia-2.8B follow from the shape we use."""
    facts = json.load(open(os.path.join(HERE, "golden", "paper_shape_facts.json")))
    sh = synth.PYTHIA_2_8B
    assert round(sh.hidden * sh.ffn / 1e6, 1) == facts["mlp_down_params_millions"]
    assert sh.ffn * 2 / 1024 == facts["mlp_intermediate_kb"]
    assert round(2 * sh.ffn * 2 * sh.n_layers / 1e6, 2) == facts["intermediate_traffic_mb_per_step"]
    # ~2 flops per parameter per token, LM head included, plus attention at short context
    params = sh.n_layers * 12 * sh.hidden ** 2 + synth.VOCAB * sh.hidden
    assert abs(2 * params * 16 / 1e9 - facts["decode_gflop_per_16_tokens"]) / facts["decode_gflop_per_16_tokens"] < 0.05
