"""Pins of the oracle's prompt processing (paper Sec. 4.2 "Prefill Phase": the
stack applied to every prompt token with causal attention).  The oracle takes
one decode step per token; here the same prompt goes through the textbook
matrix form of a causal GPT-NeoX layer - all tokens at once, a masked
[T, pos0 + T] score matrix per head - written with numpy in float64.  CPU only."""
import numpy as np
from scipy.special import erf

import synth


def _ln(X, g, b, eps):
    mu = X.mean(axis=1, keepdims=True)
    var = ((X - mu) ** 2).mean(axis=1, keepdims=True)
    return (X - mu) / np.sqrt(var + eps) * g + b


def _rope(U, positions, r, base):
    """U: [T, H, d]; rotates dims (i, i + r/2), i < r/2, of every head by positions[t] * base^(-2i/r)."""
    out = U.copy()
    half = r // 2
    theta = base ** (-2.0 * np.arange(half) / r)
    ang = positions[:, None] * theta[None, :]                      # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = U[:, :, :half], U[:, :, half:r]
    out[:, :, :half] = lo * c - hi * s
    out[:, :, half:r] = hi * c + lo * s
    return out


def causal_layer(sh, w, K_cache, V_cache, pos0, X):
    """One parallel-residual layer over T tokens at once.  K_cache, V_cache: fp16
    [H, cap, d] with pos0 rows cached; rows pos0.. are written (rounded to fp16)."""
    f64 = lambda a: np.asarray(a).astype(np.float64)
    T, h = X.shape
    H, d, r = sh.n_heads, sh.head_dim, sh.rotary_dims
    Y1 = _ln(X, f64(w["ln1_g"]), f64(w["ln1_b"]), sh.ln_eps)
    Y2 = _ln(X, f64(w["ln2_g"]), f64(w["ln2_b"]), sh.ln_eps)
    qkv = (Y1 @ f64(w["w_qkv"]).T + f64(w["b_qkv"])).reshape(T, H, 3, d)
    pos = np.arange(pos0, pos0 + T, dtype=np.float64)
    q = _rope(qkv[:, :, 0], pos, r, sh.rope_base)
    k = _rope(qkv[:, :, 1], pos, r, sh.rope_base)
    v = qkv[:, :, 2]
    K_cache[:, pos0:pos0 + T] = k.transpose(1, 0, 2).astype(np.float16)
    V_cache[:, pos0:pos0 + T] = v.transpose(1, 0, 2).astype(np.float16)
    Kall, Vall = f64(K_cache[:, :pos0 + T]), f64(V_cache[:, :pos0 + T])        # [H, n, d]
    scores = np.einsum("thd,hnd->htn", q, Kall) / np.sqrt(d)                     # [H, T, n]
    mask = np.arange(pos0 + T)[None, :] > (pos0 + np.arange(T))[:, None]         # later positions
    scores = np.where(mask[None], -np.inf, scores)
    p = np.exp(scores - scores.max(axis=2, keepdims=True))
    p /= p.sum(axis=2, keepdims=True)
    o = np.einsum("htn,hnd->thd", p, Vall).reshape(T, h)
    a = o @ f64(w["w_dense"]).T + f64(w["b_dense"])
    z = Y2 @ f64(w["w_up"]).T + f64(w["b_up"])
    m = 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))
    g = m @ f64(w["w_down"]).T + f64(w["b_down"])
    return X + a + g


def _setup(seed, pos0, T, L=3):
    sh = synth.ModelShape(48, 3, 16, 4, 96, n_layers=L)
    layers = synth.stack_weights(sh, seed)
    cap = pos0 + T + 2
    kv = [synth.kv_cache(sh, seed, l, pos0, cap) for l in range(L)]
    Ks, Vs = [k[0][0].copy() for k in kv], [k[1][0].copy() for k in kv]
    X = synth.x_input(sh, seed, batch=T)
    return sh, layers, Ks, Vs, X


def test_prefill_equals_the_matrix_form_of_a_causal_stack(orc):
    for seed, pos0, T in ((3, 0, 7), (5, 6, 11)):
        sh, layers, Ks, Vs, X = _setup(seed, pos0, T)
        Km, Vm = [k.copy() for k in Ks], [v.copy() for v in Vs]
        out16, out = orc.prefill(sh, layers, Ks, Vs, pos0, X)
        Xm = X.astype(np.float64)
        for l, w in enumerate(layers):
            Xm = causal_layer(sh, w, Km[l], Vm[l], pos0, Xm)
        assert np.abs(out - Xm).max() < 1e-9
        assert np.mean(out16 == Xm.astype(np.float16)) > 0.99      # (a value on a rounding boundary may fall either way)
        for l in range(sh.n_layers):
            n = pos0 + T
            assert np.array_equal(Ks[l][:, :n].view(np.uint16), Km[l][:, :n].view(np.uint16))
            assert np.array_equal(Vs[l][:, :n].view(np.uint16), Vm[l][:, :n].view(np.uint16))


def test_prefill_is_causal_and_continues_like_decode(orc):
    sh, layers, Ks, Vs, X = _setup(9, 4, 9)
    Ks2, Vs2 = [k.copy() for k in Ks], [v.copy() for v in Vs]
    out16, _ = orc.prefill(sh, layers, Ks, Vs, 4, X)
    # a later token does not change an earlier output
    X2 = X.copy()
    X2[6] = -X2[6]
    out16b, _ = orc.prefill(sh, layers, Ks2, Vs2, 4, X2)
    assert np.array_equal(out16[:6].view(np.uint16), out16b[:6].view(np.uint16))
    assert not np.array_equal(out16[6:].view(np.uint16), out16b[6:].view(np.uint16))
    # the prompt in two pieces is the prompt in one
    sh, layers, Ks3, Vs3, X = _setup(9, 4, 9)
    a16, _ = orc.prefill(sh, layers, Ks3, Vs3, 4, X[:5])
    b16, _ = orc.prefill(sh, layers, Ks3, Vs3, 9, X[5:])
    assert np.array_equal(np.concatenate([a16, b16]).view(np.uint16), out16.view(np.uint16))
