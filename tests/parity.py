"""Shared comparison helpers for the GPU parity tests."""
import numpy as np

# tolerance on the fp16 block output, as stated for this build's north star
MAX_ABS = 2e-2
REL_L2 = 5e-3
U32 = 2.0 ** -24          # unit roundoff of fp32


def errors(got, want):
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    assert got.shape == want.shape
    assert np.isfinite(got).all(), "non-finite values in the GPU output"
    return float(np.abs(got - want).max()), float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def assert_block_close(got, want, what=""):
    ma, rl = errors(got, want)
    assert ma <= MAX_ABS and rl <= REL_L2, f"{what}: max-abs {ma:.3e} (<= {MAX_ABS}), rel-L2 {rl:.3e} (<= {REL_L2})"
    return ma, rl


# ---- appended K/V rows ---------------------------------------------------------
# An appended element is fp16(v) of a value v the kernel evaluates in fp32:
#     v = sum_j W_ij y_j + b_i      (K: followed by the rotation of a pair)
# with y the LayerNorm of the layer input.  When the layer input is the same bits
# on both sides (a single block, layer 0 of a stack, a teacher-forced layer) the
# kernel's v differs from the exact value e only by fp32 evaluation error, for
# which the standard bound of a depth-n summation holds:
#     |v - e| <= n u A_i,   u = 2^-24,   A_i = sum_j |W_ij| |terms_j| + |b_i|.
# The longest chain of dependent fp32 operations any launch mode has behind one
# element: K/64 fused multiply-adds per lane (8 per 512-column unit), the two
# accumulators joined, 6 levels of the lane reduction, up to 8 wavefront slots
# added in order (or the matrix-core path's K-partials through LDS), the bias or
# the LayerNorm completion (3 operations), the rotation (2), and the LayerNorm of
# y itself (two reductions of log2(h) levels, the reciprocal root, the affine
# part: under 32 operations per element, which enter through A).  n = K/64 + 64
# covers all of them.  So the GPU's fp16 value g must be the rounding of SOME
# value within delta = n u A_i of e:
#     |g - e| <= ulp16(|e| + delta) / 2 + delta.
# No fraction of differing elements is asked for: an element either is a correct
# rounding under this bound or it is not.
def rounding_bound(A, K):
    return (K / 64.0 + 64.0) * U32 * np.asarray(A, dtype=np.float64)


def ulp16(v):
    """Spacing of binary16 at |v| (2^-24 in the subnormal range)."""
    v = np.abs(np.asarray(v, dtype=np.float64))
    _, ex = np.frexp(np.maximum(v, 2.0 ** -24))          # v in [2^(ex-1), 2^ex)
    return np.ldexp(1.0, np.maximum(ex - 1 - 10, -24))


def qkv_abs_sums(shape, w, x_real):
    """A_i for every row of the QKV projection, [3h] in canonical row order: dominates the
    sum of absolute terms of both forms the kernels evaluate, W (gamma (x - mu) inv + beta) + b
    and inv (W (gamma x) - mu W gamma) + (W beta + b)."""
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    x = f64(x_real).ravel()
    mu = x.mean()
    inv = 1.0 / np.sqrt(((x - mu) ** 2).mean() + shape.ln_eps)
    g, b = np.abs(f64(w["ln1_g"])), np.abs(f64(w["ln1_b"]))
    terms = g * np.abs(x - mu) * inv + g * abs(mu) * inv + b
    return np.abs(w["w_qkv"].astype(np.float32)) @ terms.astype(np.float32) + np.abs(f64(w["b_qkv"]))


def appended_rows_reference(shape, w, x_real, taps):
    """(k_exact, v_exact, A_k, A_v), each [H, d]: the oracle's unrounded new K (rotated)
    and V rows, and the abs-sums their rounding bound is built from (a rotated element
    mixes the two rows of its pair)."""
    H, d, r = shape.n_heads, shape.head_dim, shape.rotary_dims
    A = qkv_abs_sums(shape, w, x_real).reshape(H, 3, d)
    Ak, Av = A[:, 1].copy(), A[:, 2].copy()
    half = r // 2
    if half:
        pair = Ak[:, :half] + Ak[:, half:r]
        Ak[:, :half] = pair
        Ak[:, half:r] = pair
    return (np.asarray(taps["k_new"], dtype=np.float64).reshape(H, d),
            np.asarray(taps["v_new"], dtype=np.float64).reshape(H, d), Ak, Av)


def assert_appended_row(got16, exact, A, K, what=""):
    """got16: the kernel's fp16 row [H, d]; exact: the oracle's unrounded values."""
    g = np.asarray(got16, dtype=np.float16).astype(np.float64)
    e = np.asarray(exact, dtype=np.float64)
    assert g.shape == e.shape and np.isfinite(g).all(), what
    delta = rounding_bound(A, K)
    allowed = 0.5 * ulp16(np.abs(e) + delta) + delta
    over = np.abs(g - e) - allowed
    assert (over <= 0).all(), (f"{what}: {int((over > 0).sum())} appended values are not a rounding of the exact value "
                               f"within the fp32 evaluation bound (worst by {over.max():.3e})")


def assert_appended_rows(got_k16, got_v16, shape, w, x_real, taps, what=""):
    ke, ve, Ak, Av = appended_rows_reference(shape, w, x_real, taps)
    assert_appended_row(got_k16, ke, Ak, shape.hidden, f"{what} appended K")
    assert_appended_row(got_v16, ve, Av, shape.hidden, f"{what} appended V")


def assert_drifted_rows_close(got16, want16, what=""):
    """Appended rows of a layer whose input already differs between the two sides (layers
    behind the first of a stack): the residual stream's drift - which includes legitimate
    one-step differences of earlier appended rows, fed back through the attention with the
    new token's softmax weight - reaches them through the projection, so they are held to
    the tolerance of the block output, not to the rounding bound."""
    return assert_block_close(np.asarray(got16, dtype=np.float16), np.asarray(want16, dtype=np.float16), what)
