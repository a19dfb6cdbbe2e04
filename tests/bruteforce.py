"""A second, independent statement of the decode block in pure-Python float
loops (math module only, no numpy arithmetic), for tiny shapes.  It exists to
pin the C oracle; it is written from the block's definition (paper Sec. 2.2 and
the GPT-NeoX conventions), not from the C source."""
import math


def layernorm(x, g, b, eps):
    n = len(x)
    mu = math.fsum(x) / n
    var = math.fsum((v - mu) ** 2 for v in x) / n
    return [(v - mu) / math.sqrt(var + eps) * g[i] + b[i] for i, v in enumerate(x)]


def matvec(W, bias, v):
    return [math.fsum(W[r][c] * v[c] for c in range(len(v))) + bias[r] for r in range(len(W))]


def rope(u, r, pos, base):
    u = list(u)
    half = r // 2
    for i in range(half):
        ang = pos * base ** (-2.0 * i / r)
        a, b = u[i], u[i + half]
        u[i] = a * math.cos(ang) - b * math.sin(ang)
        u[i + half] = b * math.cos(ang) + a * math.sin(ang)
    return u


def block(shape, w, K, V, pos, x, round_half):
    """w: dict of nested lists (floats); K, V: [H][cap][d] nested lists, rows < pos
    valid; round_half: callable float -> float (fp16 rounding of appended k, v).
    Returns (out list, k_new [H][d], v_new [H][d])."""
    h, H, d, r, f = shape.hidden, shape.n_heads, shape.head_dim, shape.rotary_dims, shape.ffn
    y1 = layernorm(x, w["ln1_g"], w["ln1_b"], shape.ln_eps)
    y2 = layernorm(x, w["ln2_g"], w["ln2_b"], shape.ln_eps)
    qkv = matvec(w["w_qkv"], w["b_qkv"], y1)
    attn, k_new, v_new = [], [], []
    for n in range(H):
        q = rope(qkv[(3 * n) * d:(3 * n + 1) * d], r, pos, shape.rope_base)
        k = rope(qkv[(3 * n + 1) * d:(3 * n + 2) * d], r, pos, shape.rope_base)
        v = qkv[(3 * n + 2) * d:(3 * n + 3) * d]
        k = [round_half(t) for t in k]
        v = [round_half(t) for t in v]
        k_new.append(k)
        v_new.append(v)
        keys = [K[n][t] for t in range(pos)] + [k]
        vals = [V[n][t] for t in range(pos)] + [v]
        s = [math.fsum(q[i] * kt[i] for i in range(d)) / math.sqrt(d) for kt in keys]
        mx = max(s)
        e = [math.exp(t - mx) for t in s]
        den = math.fsum(e)
        attn += [math.fsum(e[t] / den * vals[t][i] for t in range(len(vals))) for i in range(d)]
    a = matvec(w["w_dense"], w["b_dense"], attn)
    flags = getattr(shape, "flags", 0)
    if flags & 2:       # sequential reading: the post-attention LayerNorm sees x + attention
        x1 = [x[i] + a[i] for i in range(h)]
        y2 = layernorm(x1, w["ln2_g"], w["ln2_b"], shape.ln_eps)
    up = matvec(w["w_up"], w["b_up"], y2)
    if flags & 1:       # tanh form of GELU
        m = [0.5 * z * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3))) for z in up]
    else:
        m = [0.5 * z * (1.0 + math.erf(z / math.sqrt(2.0))) for z in up]
    g = matvec(w["w_down"], w["b_down"], m)
    if flags & 2:
        return [x1[i] + g[i] for i in range(h)], k_new, v_new
    return [x[i] + a[i] + g[i] for i in range(h)], k_new, v_new
