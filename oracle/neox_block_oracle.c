/*
 * CPU oracle for one GPT-NeoX / Pythia decoder block, single-token decode.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * definition-level implementation used only by the tests, the smoke check and
 * the benchmark's CPU-baseline leg.  It shares no code with the HIP library
 * and nothing in the HIP library calls it.
 *
 * What it computes (paper Sec. 2.2, the fused region: pre-attention LayerNorm,
 * QKV projection with per-head interleaved rows and KV-cache update, partial
 * rotary embedding on the first 25% of every head, decode attention over the
 * cache, output projection, post-attention LayerNorm, MLP up / GELU / down,
 * residual), in the residual form GPT-NeoX defines (both branches read the
 * block input):
 *
 *     out = x + Dense(Attn(LN1(x))) + Down(GELU(Up(LN2(x))))
 *
 * Fusion does not change the function, so every step is the textbook
 * definition written out.  Inputs are fp16 bit patterns (weights, biases, LN
 * parameters, KV cache) that are upcast exactly; all arithmetic is done in
 * `real` (double by default, float with -DORACLE_REAL=float); values are
 * rounded to fp16 only where the method stores fp16: the K/V rows appended to
 * the cache, and the block output (by the caller, through orc_real_to_half).
 *
 * Readings of points the paper leaves open (each is pinned by a CPU test):
 *   - LayerNorm: eps inside the square root, biased variance, two passes.
 *   - QKV row order: row (3*head + c)*head_dim + i, c = 0:q 1:k 2:v.
 *   - The attention output projection has a bias (GPT-NeoX does).
 *   - RoPE: half-split pairing (i, i + r/2) inside the rotary slice,
 *     theta_i = base^(-2i/r), angle = pos * theta_i, applied to q and k.
 *   - Softmax scale 1/sqrt(head_dim); no mask (every cached t <= pos).
 *   - GELU is the exact erf form.
 * The other readings of two of these points are available behind flags of
 * orc_block_decode_flags (they change nothing unless set):
 *   - ORC_TANH_GELU: the tanh approximation of GELU (the paper only says
 *     "accelerated GELU", Sec. 2.2, without naming the flavour);
 *   - ORC_SEQUENTIAL_RESIDUAL: the chain read literally in the order Sec. 2.2
 *     lists it - output projection with residual, then the post-attention
 *     LayerNorm on that sum, then the MLP with residual:
 *         x1 = x + Dense(Attn(LN1(x)));  out = x1 + Down(GELU(Up(LN2(x1))))
 *   - Cached K rows are already rotated.
 *
 * Loops over output rows / heads carry an OpenMP pragma; that only spreads
 * independent outputs over cores and changes no arithmetic or order inside
 * one output.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

typedef struct {
    int32_t hidden, n_heads, head_dim, rotary_dims, ffn;
    double rope_base, ln_eps;
} orc_shape;

/* canonical fp16 tensors of one block, as raw bit patterns */
typedef struct {
    const uint16_t *ln1_g, *ln1_b, *ln2_g, *ln2_b;
    const uint16_t *w_qkv, *b_qkv;     /* [3h, h], [3h] */
    const uint16_t *w_dense, *b_dense; /* [h, h],  [h]  */
    const uint16_t *w_up, *b_up;       /* [f, h],  [f]  */
    const uint16_t *w_down, *b_down;   /* [h, f],  [h]  */
} orc_layer;

/* optional taps on the intermediates (any pointer may be NULL) */
typedef struct {
    real *y1, *y2;     /* [h] LayerNorm outputs                   */
    real *q;           /* [h] rotated queries, (head, dim) order  */
    real *attn;        /* [h] concatenated per-head attention out */
    real *a;           /* [h] output projection                   */
    real *m;           /* [f] GELU(up)                            */
    real *g;           /* [h] down projection                     */
    real *k_new, *v_new; /* [h] the new token's K (rotated) and V rows before they are rounded to fp16 */
} orc_taps;

int orc_sizeof_real(void) { return (int)sizeof(real); }

/* ---- fp16 <-> real ---------------------------------------------------- */

/* exact upcast of an IEEE binary16 bit pattern */
real orc_half_to_real(uint16_t hbits)
{
    int sign = (hbits >> 15) & 1;
    int e = (hbits >> 10) & 0x1f;
    int mant = hbits & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)mant, -24);
    else if (e == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp((double)(mant + 1024), e - 25);
    return (real)(sign ? -v : v);
}

/* round to nearest even into binary16 (one rounding, from the real value) */
uint16_t orc_real_to_half(real rv)
{
    double v = (double)rv;
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v)) return 0x7e00u;
    if (a >= 65520.0) return sign | 0x7c00u;   /* midpoint 65504|65536 ties to even = inf */
    if (a < ldexp(1.0, -25)) return sign;      /* below half the smallest subnormal */
    int e;
    (void)frexp(a, &e);                        /* a = f * 2^e, f in [0.5, 1) */
    e -= 1;                                    /* a in [2^e, 2^(e+1)) */
    if (e < -14) {                             /* subnormal: multiples of 2^-24 */
        double r = rint(ldexp(a, 24));         /* may reach 1024 = smallest normal */
        return sign | (uint16_t)r;
    }
    double r = rint(ldexp(a, 10 - e));         /* in [1024, 2048] */
    if (r >= 2048.0) { r = 1024.0; e += 1; }
    if (e + 15 >= 31) return sign | 0x7c00u;
    return sign | (uint16_t)(((e + 15) << 10) | ((int)r - 1024));
}

void orc_half_to_real_n(const uint16_t *src, real *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = orc_half_to_real(src[i]);
}

void orc_real_to_half_n(const real *src, uint16_t *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = orc_real_to_half(src[i]);
}

/* ---- steps ------------------------------------------------------------ */

/* LayerNorm with affine: y_i = (x_i - mu) / sqrt(var + eps) * gamma_i + beta_i,
 * mu = mean(x), var = mean((x - mu)^2).  gamma/beta NULL -> no affine. */
void orc_layernorm(const real *x, const uint16_t *gamma, const uint16_t *beta,
                   int n, double eps, real *y)
{
    real mu = 0;
    for (int i = 0; i < n; ++i) mu += x[i];
    mu /= (real)n;
    real var = 0;
    for (int i = 0; i < n; ++i) var += (x[i] - mu) * (x[i] - mu);
    var /= (real)n;
    real inv = (real)1 / (real)sqrt((double)var + eps);
    for (int i = 0; i < n; ++i) {
        real t = (x[i] - mu) * inv;
        if (gamma) t = t * orc_half_to_real(gamma[i]);
        if (beta) t = t + orc_half_to_real(beta[i]);
        y[i] = t;
    }
}

/* out = W v + b, W row-major [rows, cols] fp16, b may be NULL */
void orc_gemv(const uint16_t *W, const uint16_t *b, const real *v,
              int rows, int cols, real *out)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const uint16_t *w = W + (int64_t)r * cols;
        real acc = 0;
        for (int c = 0; c < cols; ++c) acc += orc_half_to_real(w[c]) * v[c];
        if (b) acc += orc_half_to_real(b[r]);
        out[r] = acc;
    }
}

/* partial rotary embedding on one head vector u[head_dim], in place:
 * only u[0 .. r) is touched; pairs are (i, i + r/2). */
void orc_rope(real *u, int r, int pos, double base)
{
    int half = r / 2;
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)r);
        double phi = (double)pos * theta;
        real c = (real)cos(phi), s = (real)sin(phi);
        real a = u[i], b = u[i + half];
        u[i] = a * c - b * s;
        u[i + half] = b * c + a * s;
    }
}

/* softmax(q.K^T / sqrt(d)) V for one head over positions 0 .. n_pos-1.
 * Kh, Vh: [capacity, d] fp16 (only the first n_pos rows are read).
 * p_out (optional, [n_pos]) receives the softmax probabilities. */
void orc_attention_head(const real *q, const uint16_t *Kh, const uint16_t *Vh,
                        int n_pos, int d, real *o, real *p_out)
{
    real *s = (real *)malloc(sizeof(real) * (size_t)n_pos);
    real scale = (real)1 / (real)sqrt((double)d);
    real mx = -INFINITY;
    for (int t = 0; t < n_pos; ++t) {
        real acc = 0;
        for (int i = 0; i < d; ++i) acc += q[i] * orc_half_to_real(Kh[(int64_t)t * d + i]);
        s[t] = acc * scale;
        if (s[t] > mx) mx = s[t];
    }
    real den = 0;
    for (int t = 0; t < n_pos; ++t) { s[t] = (real)exp((double)(s[t] - mx)); den += s[t]; }
    for (int t = 0; t < n_pos; ++t) s[t] /= den;
    for (int i = 0; i < d; ++i) {
        real acc = 0;
        for (int t = 0; t < n_pos; ++t) acc += s[t] * orc_half_to_real(Vh[(int64_t)t * d + i]);
        o[i] = acc;
    }
    if (p_out) memcpy(p_out, s, sizeof(real) * (size_t)n_pos);
    free(s);
}

/* exact GELU: z/2 * (1 + erf(z / sqrt 2)) */
real orc_gelu(real z)
{
    return (real)(0.5 * (double)z * (1.0 + erf((double)z * 0.70710678118654752440)));
}

void orc_gelu_n(const real *z, real *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_gelu(z[i]);
}

/* tanh form: z/2 * (1 + tanh(sqrt(2/pi) * (z + 0.044715 z^3))) */
real orc_gelu_tanh(real z)
{
    const double t = (double)z;
    return (real)(0.5 * t * (1.0 + tanh(0.79788456080286535588 * (t + 0.044715 * t * t * t))));
}

void orc_gelu_tanh_n(const real *z, real *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_gelu_tanh(z[i]);
}

/* ---- the block -------------------------------------------------------- */

/*
 * One decode step of one block for one sequence.
 *   K, V : [n_heads, capacity, head_dim] fp16, positions 0..pos-1 valid on
 *          entry; row `pos` of every head is written (fp16-rounded k, v).
 *   x    : [hidden] block input;  out: [hidden] block output, NOT rounded.
 * Returns 0, or -1 on a bad argument.
 */
enum { ORC_TANH_GELU = 1, ORC_SEQUENTIAL_RESIDUAL = 2 };

int orc_block_decode_flags(const orc_shape *sh, const orc_layer *w,
                           uint16_t *K, uint16_t *V, int capacity, int pos,
                           const real *x, real *out, const orc_taps *taps, int flags)
{
    const int h = sh->hidden, H = sh->n_heads, d = sh->head_dim;
    const int r = sh->rotary_dims, f = sh->ffn;
    if (h != H * d || r < 0 || r > d || (r & 1) || pos < 0 || pos >= capacity) return -1;

    real *y1 = malloc(sizeof(real) * h), *y2 = malloc(sizeof(real) * h);
    real *qkv = malloc(sizeof(real) * 3 * h), *attn = malloc(sizeof(real) * h);
    real *a = malloc(sizeof(real) * h), *up = malloc(sizeof(real) * f);
    real *m = malloc(sizeof(real) * f), *g = malloc(sizeof(real) * h);
    real *qrot = malloc(sizeof(real) * h);

    /* 1. both LayerNorms read the block input (sequential form: the second one later) */
    orc_layernorm(x, w->ln1_g, w->ln1_b, h, sh->ln_eps, y1);
    if (!(flags & ORC_SEQUENTIAL_RESIDUAL)) orc_layernorm(x, w->ln2_g, w->ln2_b, h, sh->ln_eps, y2);

    /* 2. fused QKV projection, rows (head, {q,k,v}, dim) */
    orc_gemv(w->w_qkv, w->b_qkv, y1, 3 * h, h, qkv);

    /* 3-5. per head: rotate q and k, append k and v (fp16), attend */
#pragma omp parallel for schedule(static)
    for (int n = 0; n < H; ++n) {
        real *qn = qkv + (int64_t)(3 * n + 0) * d;
        real *kn = qkv + (int64_t)(3 * n + 1) * d;
        real *vn = qkv + (int64_t)(3 * n + 2) * d;
        orc_rope(qn, r, pos, sh->rope_base);
        orc_rope(kn, r, pos, sh->rope_base);
        uint16_t *Kn = K + (int64_t)n * capacity * d;
        uint16_t *Vn = V + (int64_t)n * capacity * d;
        if (taps && taps->k_new) memcpy(taps->k_new + (int64_t)n * d, kn, sizeof(real) * d);
        if (taps && taps->v_new) memcpy(taps->v_new + (int64_t)n * d, vn, sizeof(real) * d);
        for (int i = 0; i < d; ++i) {
            Kn[(int64_t)pos * d + i] = orc_real_to_half(kn[i]);
            Vn[(int64_t)pos * d + i] = orc_real_to_half(vn[i]);
        }
        memcpy(qrot + (int64_t)n * d, qn, sizeof(real) * d);
        orc_attention_head(qn, Kn, Vn, pos + 1, d, attn + (int64_t)n * d, NULL);
    }

    /* 6. output projection */
    orc_gemv(w->w_dense, w->b_dense, attn, h, h, a);

    /* sequential form: the attention branch joins the residual first, and the
       post-attention LayerNorm reads that sum */
    real *x1 = NULL;
    if (flags & ORC_SEQUENTIAL_RESIDUAL) {
        x1 = malloc(sizeof(real) * h);
        for (int i = 0; i < h; ++i) x1[i] = x[i] + a[i];
        orc_layernorm(x1, w->ln2_g, w->ln2_b, h, sh->ln_eps, y2);
    }

    /* 7-8. MLP */
    orc_gemv(w->w_up, w->b_up, y2, f, h, up);
    if (flags & ORC_TANH_GELU) orc_gelu_tanh_n(up, m, f);
    else orc_gelu_n(up, m, f);
    orc_gemv(w->w_down, w->b_down, m, h, f, g);

    /* 9. residual */
    if (x1) {
        for (int i = 0; i < h; ++i) out[i] = x1[i] + g[i];
        free(x1);
    } else {
        for (int i = 0; i < h; ++i) out[i] = x[i] + a[i] + g[i];
    }

    if (taps) {
        if (taps->y1) memcpy(taps->y1, y1, sizeof(real) * h);
        if (taps->y2) memcpy(taps->y2, y2, sizeof(real) * h);
        if (taps->q) memcpy(taps->q, qrot, sizeof(real) * h);
        if (taps->attn) memcpy(taps->attn, attn, sizeof(real) * h);
        if (taps->a) memcpy(taps->a, a, sizeof(real) * h);
        if (taps->m) memcpy(taps->m, m, sizeof(real) * f);
        if (taps->g) memcpy(taps->g, g, sizeof(real) * h);
    }
    free(y1); free(y2); free(qkv); free(attn); free(a); free(up); free(m); free(g); free(qrot);
    return 0;
}

int orc_block_decode(const orc_shape *sh, const orc_layer *w,
                     uint16_t *K, uint16_t *V, int capacity, int pos,
                     const real *x, real *out, const orc_taps *taps)
{
    return orc_block_decode_flags(sh, w, K, V, capacity, pos, x, out, taps, 0);
}

/* final LayerNorm + bias-free LM head: logits = W_lm LN(x) */
void orc_lm_head(const uint16_t *lnf_g, const uint16_t *lnf_b, const uint16_t *w_lm,
                 const real *x, int hidden, int vocab, double eps, real *logits)
{
    real *z = malloc(sizeof(real) * hidden);
    orc_layernorm(x, lnf_g, lnf_b, hidden, eps, z);
    orc_gemv(w_lm, NULL, z, vocab, hidden, logits);
    free(z);
}
