// Host side of the C ABI declared in include/cfpp.h: argument checks, layout
// arithmetic, context bookkeeping, launch-shape selection, graph capture.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "cfpp.h"
#ifdef CFPP_PROFILE
#include "cfpp_profile.h"
#endif
#include "lm_params.h"
#include "batched_params.h"
#include "prefill_params.h"
#include "decode_params.h"

using namespace cfpp;

// ---- errors -----------------------------------------------------------------
static thread_local char g_err[512] = "";

static cfpp_status fail(cfpp_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

// keeps the calling thread's error text over a probe whose refusal is not the caller's error
struct g_err_hold {
    char saved[sizeof g_err];
    g_err_hold() { std::memcpy(saved, g_err, sizeof g_err); }
    ~g_err_hold() { std::memcpy(g_err, saved, sizeof g_err); }
};

#define HIP_OK(call)                                                                  \
    do {                                                                              \
        hipError_t e_ = (call);                                                       \
        if (e_ != hipSuccess)                                                         \
            return fail(CFPP_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));    \
    } while (0)

extern "C" const char *cfpp_status_string(cfpp_status s)
{
    switch (s) {
    case CFPP_OK: return "ok";
    case CFPP_EINVAL: return "invalid argument";
    case CFPP_EUNSUPPORTED: return "unsupported configuration";
    case CFPP_ENOMEM: return "buffer too small";
    case CFPP_EHIP: return "HIP runtime error";
    case CFPP_ESTATE: return "call out of order";
    case CFPP_EDEVICE: return "device-side error";
    }
    return "unknown status";
}

extern "C" const char *cfpp_last_error(void) { return g_err; }

// ---- config -------------------------------------------------------------------
static bool aligned16(const void *p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" cfpp_status cfpp_validate_config(const cfpp_config *c)
{
    if (!c) return fail(CFPP_EINVAL, "config is NULL");
    if (c->hidden <= 0 || c->n_heads <= 0 || c->head_dim <= 0 || c->ffn <= 0 || c->n_layers <= 0 ||
        c->max_seq <= 0 || c->max_batch <= 0 || c->rotary_dims < 0)
        return fail(CFPP_EINVAL, "config has a non-positive dimension");
    if ((long long)c->n_heads * c->head_dim != c->hidden)
        return fail(CFPP_EINVAL, "hidden (%d) != n_heads (%d) * head_dim (%d)", c->hidden, c->n_heads,
                    c->head_dim);
    if ((c->rotary_dims & 1) || c->rotary_dims > c->head_dim)
        return fail(CFPP_EINVAL, "rotary_dims (%d) must be even and <= head_dim", c->rotary_dims);
    if (c->flags & ~(CFPP_FLAG_TANH_GELU | CFPP_FLAG_SEQUENTIAL_RESIDUAL))
        return fail(CFPP_EINVAL, "unknown bits in flags (0x%x)", c->flags);
    if (!(c->ln_eps >= 0.f) || !(c->rope_base > 0.f))
        return fail(CFPP_EINVAL, "ln_eps must be >= 0 and rope_base > 0");
    if (c->head_dim != 64 && c->head_dim != 80 && c->head_dim != 128)
        return fail(CFPP_EUNSUPPORTED, "head_dim %d: only 64, 80 and 128 have kernels", c->head_dim);
    if ((c->hidden % 8) || (c->ffn % 8))
        return fail(CFPP_EUNSUPPORTED, "hidden and ffn must be multiples of 8");
    if (c->hidden > 8192) return fail(CFPP_EUNSUPPORTED, "hidden %d > 8192", c->hidden);
    if (c->ffn > 32768) return fail(CFPP_EUNSUPPORTED, "ffn %d > 32768", c->ffn);
    if (c->n_layers > kMaxLayers) return fail(CFPP_EUNSUPPORTED, "n_layers %d > %d", c->n_layers, kMaxLayers);
    if (c->max_seq > (1 << 20)) return fail(CFPP_EUNSUPPORTED, "max_seq %d > 2^20", c->max_seq);
    if (c->max_batch > 64) return fail(CFPP_EUNSUPPORTED, "max_batch %d > 64", c->max_batch);
    return CFPP_OK;
}

static Dims dims_of(const cfpp_config &c)
{
    Dims m;
    m.h = c.hidden; m.H = c.n_heads; m.d = c.head_dim; m.r = c.rotary_dims; m.f = c.ffn;
    m.max_seq = c.max_seq; m.max_batch = c.max_batch; m.ln_eps = c.ln_eps;
    m.flags = c.flags;
    return m;
}

extern "C" size_t cfpp_packed_layer_bytes(const cfpp_config *c)
{
    if (cfpp_validate_config(c) != CFPP_OK) return 0;
    return packed_layout(c->hidden, c->ffn).total * sizeof(__half);
}

extern "C" size_t cfpp_kv_layer_bytes(const cfpp_config *c)
{
    if (cfpp_validate_config(c) != CFPP_OK) return 0;
    return kv_layer_elems(dims_of(*c)) * sizeof(__half);
}

extern "C" size_t cfpp_workspace_bytes(const cfpp_config *c)
{
    if (cfpp_validate_config(c) != CFPP_OK) return 0;
    return workspace_layout(dims_of(*c)).total;
}

extern "C" size_t cfpp_prefill_scratch_bytes(const cfpp_config *c, int32_t rows)
{
    if (cfpp_validate_config(c) != CFPP_OK || rows <= 0 || rows > kPfMaxRows || rows % kPfTile != 0) return 0;
    return pf_layout(dims_of(*c), rows).total;
}

extern "C" cfpp_status cfpp_algorithmic_bytes(const cfpp_config *c, const int32_t *pos_host,
                                              int32_t batch, int32_t n_layers, uint64_t *bytes)
{
    cfpp_status st = cfpp_validate_config(c);
    if (st != CFPP_OK) return st;
    if (!pos_host || !bytes || batch <= 0 || batch > c->max_batch || n_layers <= 0)
        return fail(CFPP_EINVAL, "bad pos/batch/n_layers/bytes argument");
    const uint64_t h = c->hidden, f = c->ffn;
    const uint64_t params = 3 * h * h + h * h + 2 * h * f + (3 * h + h + f + h) + 4 * h;  // 12h^2+13h when f = 4h
    uint64_t per_layer = params * 2;
    for (int b = 0; b < batch; ++b) {
        if (pos_host[b] < 0 || pos_host[b] >= c->max_seq) return fail(CFPP_EINVAL, "pos[%d] out of range", b);
        per_layer += (uint64_t)pos_host[b] * 2 * h * 2;   // cached K and V rows read
        per_layer += 2 * h * 2;                           // new K and V rows written
    }
    *bytes = per_layer * (uint64_t)n_layers + (uint64_t)batch * h * 2 * 2;  // x read, out written
    return CFPP_OK;
}

// ---- data preparation ------------------------------------------------------------
extern "C" cfpp_status cfpp_pack_layer(const cfpp_config *c, const cfpp_layer_src *src, void *packed_dst,
                                       cfpp_stream stream)
{
    cfpp_status st = cfpp_validate_config(c);
    if (st != CFPP_OK) return st;
    if (!src) return fail(CFPP_EINVAL, "src is NULL");
    const void *p[12] = {src->ln1_g, src->ln1_b, src->ln2_g, src->ln2_b, src->w_qkv, src->b_qkv,
                         src->w_dense, src->b_dense, src->w_up, src->b_up, src->w_down, src->b_down};
    for (int i = 0; i < 12; ++i)
        if (!aligned16(p[i])) return fail(CFPP_EINVAL, "source tensor %d is NULL or not 16-byte aligned", i);
    if (!aligned16(packed_dst)) return fail(CFPP_EINVAL, "packed_dst is NULL or not 16-byte aligned");
    const Dims dm = dims_of(*c);
    HIP_OK(launch_pack_layer(dm, packed_layout(dm.h, dm.f), p, static_cast<__half *>(packed_dst),
                             static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_kv_import(const cfpp_config *c, const void *k_src, const void *v_src,
                                      int32_t src_capacity, int32_t n_pos, int32_t b, void *kv_layer,
                                      cfpp_stream stream)
{
    cfpp_status st = cfpp_validate_config(c);
    if (st != CFPP_OK) return st;
    if (!aligned16(k_src) || !aligned16(v_src) || !aligned16(kv_layer))
        return fail(CFPP_EINVAL, "NULL or misaligned pointer");
    if (n_pos < 0 || n_pos > src_capacity || n_pos > c->max_seq || b < 0 || b >= c->max_batch)
        return fail(CFPP_EINVAL, "n_pos/b out of range");
    HIP_OK(launch_kv_import(dims_of(*c), static_cast<const __half *>(k_src), static_cast<const __half *>(v_src),
                            src_capacity, n_pos, b, static_cast<__half *>(kv_layer),
                            static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_kv_export(const cfpp_config *c, const void *kv_layer, int32_t b,
                                      int32_t pos_begin, int32_t n_pos, int32_t dst_capacity, void *k_dst,
                                      void *v_dst, cfpp_stream stream)
{
    cfpp_status st = cfpp_validate_config(c);
    if (st != CFPP_OK) return st;
    if (!aligned16(k_dst) || !aligned16(v_dst) || !aligned16(kv_layer))
        return fail(CFPP_EINVAL, "NULL or misaligned pointer");
    if (n_pos < 0 || pos_begin < 0 || (long long)pos_begin + n_pos > c->max_seq || n_pos > dst_capacity ||
        b < 0 || b >= c->max_batch)
        return fail(CFPP_EINVAL, "position range or b out of range");
    HIP_OK(launch_kv_export(dims_of(*c), static_cast<const __half *>(kv_layer), b, pos_begin, n_pos,
                            dst_capacity, static_cast<__half *>(k_dst), static_cast<__half *>(v_dst),
                            static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}

// ---- context -----------------------------------------------------------------------
static const unsigned long long kEpochLimit = 0xF0000000ull;   // re-zero the epoch counter beyond this many epochs
struct cfpp_ctx {
    cfpp_config cfg;
    Dims dm;
    PackedLayout lay;
    WorkspaceLayout wl;
    char *ws;
    int n_cu;
    int mode, grid, threads, debug;
    unsigned long long epochs_used, epoch_limit;   // tagged-word epochs handed out since the last zeroing; re-zero beyond the limit
    size_t lds_limit;
    bool prepared, lm_prepared;
    hipGraph_t graph;
    hipGraphExec_t exec;
    unsigned long long graph_epochs;   // tagged-word epochs one replay of the captured graph uses up
    int fused_grid, fused_threads;     // launch shape the whole-stack kernel was last found to fit
    bool fused_ok;
    int last_batch;
};

extern "C" cfpp_status cfpp_create(const cfpp_config *c, void *workspace, size_t workspace_bytes,
                                   cfpp_ctx **out_ctx)
{
    cfpp_status st = cfpp_validate_config(c);
    if (st != CFPP_OK) return st;
    if (!out_ctx) return fail(CFPP_EINVAL, "out_ctx is NULL");
    *out_ctx = nullptr;
    if (!aligned16(workspace)) return fail(CFPP_EINVAL, "workspace is NULL or not 16-byte aligned");
    const Dims dm = dims_of(*c);
    const WorkspaceLayout wl = workspace_layout(dm);
    if (workspace_bytes < wl.total)
        return fail(CFPP_ENOMEM, "workspace has %zu bytes, needs %zu", workspace_bytes, wl.total);

    int dev = 0;
    HIP_OK(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_OK(hipGetDeviceProperties(&prop, dev));

    cfpp_ctx *ctx = new (std::nothrow) cfpp_ctx();
    if (!ctx) return fail(CFPP_ENOMEM, "out of host memory");
    ctx->cfg = *c;
    ctx->dm = dm;
    ctx->lay = packed_layout(dm.h, dm.f);
    ctx->wl = wl;
    ctx->ws = static_cast<char *>(workspace);
    ctx->n_cu = prop.multiProcessorCount;
    ctx->mode = CFPP_MODE_AUTO;
    ctx->grid = 0;
    ctx->threads = 512;
    ctx->debug = 0;
    ctx->epochs_used = 0;
    ctx->epoch_limit = kEpochLimit;
    ctx->lds_limit = prop.sharedMemPerBlock > 0 ? (size_t)prop.sharedMemPerBlock : 65536;
    ctx->prepared = false;
    ctx->lm_prepared = false;
    ctx->graph = nullptr;
    ctx->exec = nullptr;
    ctx->graph_epochs = 0;
    ctx->fused_grid = 0; ctx->fused_threads = 0; ctx->fused_ok = false;
    ctx->last_batch = 1;

    // barrier words, error flag and per-head arrival counters start at zero
    hipError_t e = hipMemset(ctx->ws + wl.sync, 0, wl.layer_ptrs - wl.sync);
    if (e == hipSuccess) e = hipMemset(ctx->ws + wl.tagged, 0, wl.rope - wl.tagged);
    // rotary table in double on the host: angle = pos * base^(-2j/r)
    std::vector<float> tab;
    const int half = dm.r / 2;
    if (e == hipSuccess && half > 0) {
        tab.resize((size_t)dm.max_seq * half * 2);
        for (int j = 0; j < half; ++j) {
            const double theta = std::pow((double)c->rope_base, -2.0 * j / (double)dm.r);
            for (int t = 0; t < dm.max_seq; ++t) {
                const double a = (double)t * theta;
                tab[((size_t)t * half + j) * 2 + 0] = (float)std::cos(a);
                tab[((size_t)t * half + j) * 2 + 1] = (float)std::sin(a);
            }
        }
        e = hipMemcpy(ctx->ws + wl.rope, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        delete ctx;
        return fail(CFPP_EHIP, "workspace initialisation failed: %s", hipGetErrorString(e));
    }
    *out_ctx = ctx;
    return CFPP_OK;
}

extern "C" void cfpp_destroy(cfpp_ctx *ctx)
{
    if (!ctx) return;
    if (ctx->exec) (void)hipGraphExecDestroy(ctx->exec);
    if (ctx->graph) (void)hipGraphDestroy(ctx->graph);
    delete ctx;
}

// Barrier words, error flag, arrival counters, the epoch counter and the tagged
// words back to zero (waits for the device; never inside a stream capture).
static cfpp_status reset_sync_words(cfpp_ctx *ctx)
{
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemset(ctx->ws + ctx->wl.sync, 0, ctx->wl.layer_ptrs - ctx->wl.sync));
    HIP_OK(hipMemset(ctx->ws + ctx->wl.tagged, 0, ctx->wl.rope - ctx->wl.tagged));
    HIP_OK(hipDeviceSynchronize());
    ctx->epochs_used = 0;
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_set_option(cfpp_ctx *ctx, int32_t option, int64_t value)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    switch (option) {
    case CFPP_OPT_MODE:
        if (value == 3) return fail(CFPP_EUNSUPPORTED, "launch mode 3 (the wave-specialised stream kernel) has been retired");
        if (value < CFPP_MODE_AUTO || value > 2) return fail(CFPP_EINVAL, "mode must be -1 (auto), 0, 1 or 2");
        ctx->mode = (int)value;
        return CFPP_OK;
    case CFPP_OPT_GRID:
        if (value < 0 || value > kMaxGrid) return fail(CFPP_EINVAL, "grid must be in [0, %d]", kMaxGrid);
        ctx->grid = (int)value;
        return CFPP_OK;
    case CFPP_OPT_THREADS:
        if (value != 256 && value != 512) return fail(CFPP_EINVAL, "threads must be 256 or 512");
        ctx->threads = (int)value;
        return CFPP_OK;
#ifdef CFPP_PROFILE
    case CFPP_OPT_PROFILE_SKIP:
        ctx->debug = (int)value;
        return CFPP_OK;
    case CFPP_OPT_EPOCH_LIMIT:
        if (value < 1 || value > 0xffffffffll) return fail(CFPP_EINVAL, "epoch limit outside [1, 2^32)");
        ctx->epoch_limit = (unsigned long long)value;
        return CFPP_OK;
#endif
    }
    return fail(CFPP_EINVAL, "unknown option %d", option);
}

extern "C" cfpp_status cfpp_get_option(const cfpp_ctx *ctx, int32_t option, int64_t *value)
{
    if (!ctx || !value) return fail(CFPP_EINVAL, "NULL argument");
    switch (option) {
    case CFPP_OPT_MODE: *value = ctx->mode; return CFPP_OK;
    case CFPP_OPT_GRID: *value = ctx->grid ? ctx->grid : ctx->n_cu; return CFPP_OK;
    case CFPP_OPT_THREADS: *value = ctx->threads; return CFPP_OK;
    }
    return fail(CFPP_EINVAL, "unknown option %d", option);
}

// ---- launch shape ---------------------------------------------------------------------
static int ceil_div(int a, int b) { return (a + b - 1) / b; }

// K-slices per row for a GEMV where a workgroup owns `nrows` rows of `nchunk`
// chunks and has `nw` wavefronts: minimise rounds * (chunks per slice + fixed
// cost of finishing a unit).
static int pick_slices(int nrows, int nchunk, int nw)
{
    int best = 1;
    double best_cost = 1e30;
    for (int nsl = 1; nsl <= nchunk; ++nsl) {
        const int cps = ceil_div(nchunk, nsl);
        if (ceil_div(nchunk, cps) != nsl) continue;       // same slicing as a smaller nsl
        const int rounds = ceil_div(nrows * nsl, nw);
        const double cost = rounds * (cps + 0.5);
        if (cost < best_cost - 1e-9) { best_cost = cost; best = nsl; }
    }
    return best;
}

struct Shape {
    int grid, threads;
    int rows_qkv, rows_up, rows_h, nsl_down, nsl_dense;
    int f_a, rows_up_a, rows_up_b;   // whole-stack kernel: the MLP intermediate in two halves
    unsigned lds_floats;
};

static cfpp_status launch_shape(const cfpp_ctx *ctx, Shape *sh)
{
    const Dims &dm = ctx->dm;
    sh->grid = ctx->grid ? ctx->grid : ctx->n_cu;
    sh->threads = ctx->threads;
    const int nw = sh->threads / 64, G = sh->grid;
    sh->rows_qkv = (ceil_div(3 * dm.h, G) + 1) & ~1;
    sh->rows_up = ceil_div(dm.f, G);
    sh->rows_h = ceil_div(dm.h, G);
    sh->f_a = ceil_div(ceil_div(dm.f, kChunk), 2) * kChunk;       // the first half, in whole 512-column units
    if (sh->f_a > dm.f) sh->f_a = dm.f;
    sh->rows_up_a = ceil_div(sh->f_a, G);
    sh->rows_up_b = ceil_div(dm.f - sh->f_a, G);
    const int nch_h = ceil_div(dm.h, kChunk), nch_f = ceil_div(dm.f, kChunk);
    sh->nsl_down = pick_slices(sh->rows_h, nch_f, nw);
    sh->nsl_dense = pick_slices(sh->rows_h, nch_h, nw);
    const size_t a = 2 * (size_t)nch_h * kChunk + (size_t)(sh->rows_qkv + sh->rows_up) * nw + 16;
    const size_t b = (size_t)nch_f * kChunk + (size_t)sh->rows_h * nw + (size_t)nw * (dm.d + 2) + 4 + 2 * (size_t)dm.d;
    const size_t c = (size_t)nch_h * kChunk + (size_t)sh->rows_h * nw;
    size_t m = a > b ? a : b;
    m = m > c ? m : c;
    m = (m + 63) / 64 * 64;
    if (m * 4 > 160 * 1024) return fail(CFPP_EUNSUPPORTED, "needs %zu bytes of LDS (> 160 KiB)", m * 4);
    if ((size_t)dm.h > (size_t)32 * sh->threads)    // the LayerNorm keeps 32 values per thread
        return fail(CFPP_EUNSUPPORTED, "hidden %d needs more than 32 values per thread at %d threads", dm.h,
                    sh->threads);
    if ((size_t)dm.f > (size_t)32 * sh->threads)    // the MLP intermediate is staged with 32 values per thread
        return fail(CFPP_EUNSUPPORTED, "ffn %d needs more than 32 values per thread at %d threads", dm.f,
                    sh->threads);
    sh->lds_floats = (unsigned)m;
    return CFPP_OK;
}

// Launches that need more than the default 64 KiB of dynamic LDS must raise the
// kernels' limit first (once, outside any stream capture).
static cfpp_status prepare(cfpp_ctx *ctx)
{
    if (ctx->prepared) return CFPP_OK;
    HIP_OK(prepare_kernels(160 * 1024));
    HIP_OK(prepare_fused_kernels(160 * 1024));
    HIP_OK(prepare_bat_kernels(160 * 1024));
    ctx->prepared = true;
    return CFPP_OK;
}

static StepParams make_params(const cfpp_ctx *ctx, const Shape &sh, int b, const void *x,
                              const int32_t *pos_dev, void *out, int n_layers)
{
    const Dims &dm = ctx->dm;
    const WorkspaceLayout &wl = ctx->wl;
    StepParams P;
    P.dm = dm;
    P.lay = ctx->lay;
    P.sync = reinterpret_cast<unsigned *>(ctx->ws + wl.sync);
    P.seg_cnt = reinterpret_cast<unsigned *>(ctx->ws + wl.seg_cnt) + (size_t)b * dm.H;
    P.rope = reinterpret_cast<const float2 *>(ctx->ws + wl.rope);
    P.xres = reinterpret_cast<float *>(ctx->ws + wl.xres) + (size_t)b * 2 * dm.h;
    P.q = reinterpret_cast<float *>(ctx->ws + wl.q) + (size_t)b * dm.h;
    P.m = reinterpret_cast<float *>(ctx->ws + wl.m) + (size_t)b * dm.f;
    P.g = reinterpret_cast<float *>(ctx->ws + wl.g) + (size_t)b * dm.h;
    P.o = reinterpret_cast<float *>(ctx->ws + wl.o) + (size_t)b * dm.h;
    P.part = reinterpret_cast<float *>(ctx->ws + wl.part) + (size_t)b * dm.H * wl.part_slots * (dm.d + 2);
    P.part_slots = wl.part_slots;
    P.tagged = reinterpret_cast<float *>(ctx->ws + wl.tagged);
    P.pos = pos_dev + b;
    P.b = b;
    P.x_in = static_cast<const __half *>(x) + (size_t)b * dm.h;
    P.out = static_cast<__half *>(out) + (size_t)b * dm.h;
    P.n_layers = n_layers;
    P.parts = kPartAll;
    P.attn_g0 = 0;
    P.attn_G = 0;
    P.attn_bstep = 1;
    P.rows_qkv = sh.rows_qkv; P.rows_up = sh.rows_up; P.rows_h = sh.rows_h;
    P.f_a = sh.f_a; P.rows_up_a = sh.rows_up_a; P.rows_up_b = sh.rows_up_b;
    P.nsl_down = sh.nsl_down; P.nsl_dense = sh.nsl_dense;
    P.lds_floats = sh.lds_floats;
    P.debug = ctx->debug;
    P.trace = reinterpret_cast<unsigned long long *>(ctx->ws + wl.trace);
    P.w_single = nullptr;
    P.kv_single = nullptr;
    return P;
}

// One block with the phase kernels (or, persistent = true, with the persistent kernel that runs
// the same phases behind grid barriers).  Parallel residual: one pass.  Sequential
// residual: two passes over the same kernels - the attention half (LayerNorm,
// QKV, attention, output projection, x1 = x + a) and the MLP half (LayerNorm of
// x1, up, down, out = x1 + g) - as two consecutive slots of the fp32 residual
// ping-pong; P.n_layers counts slots.
static hipError_t launch_block_phases(const StepParams &P, const __half *w, __half *kv, int l, int grid,
                                      int threads, hipStream_t s, bool persistent = false)
{
    auto launch = persistent ? launch_block_persistent : launch_phases;
    if (!(P.dm.flags & kFlagSequentialResidual)) return launch(P, w, kv, l, grid, threads, s);
    StepParams Q = P;
    Q.parts = kPartQkv | kPartAttention | kPartDense;
    hipError_t e = launch(Q, w, kv, 2 * l, grid, threads, s);
    if (e != hipSuccess) return e;
    Q.parts = kPartUp | kPartDown;
    return launch(Q, w, kv, 2 * l + 1, grid, threads, s);
}

// Launch mode 0 with several sequences: the projections of a layer run once for
// groups of up to kBatMax sequences (weights streamed once per group, matrix
// cores), the attention per sequence in between.
static bool batched_path_shape(const cfpp_ctx *ctx, const Shape &sh)
{
    return !(ctx->dm.flags & kFlagSequentialResidual) && bat_supported(ctx->dm, sh.grid, sh.threads);
}
static bool batched_path(const cfpp_ctx *ctx, const Shape &sh, int batch)
{
    return batch > 1 && batched_path_shape(ctx, sh);
}

// kv_seq < 0: row i of x / pos / out is sequence i with its own cache (a decode step of
// `batch` sequences).  kv_seq >= 0: the rows are consecutive positions of sequence kv_seq
// (a group of prompt tokens): they use the workspace rows 0.. but all append to, and attend
// over, that one cache - the rows of the group are in the cache before its attention runs,
// so a token sees the tokens before it.
static cfpp_status launch_batched_layer(const cfpp_ctx *ctx, const Shape &sh, const __half *w, __half *kv, int l,
                                        int n_layers, const void *x, const int32_t *pos_dev, int batch, void *out,
                                        hipStream_t s, int kv_seq = -1)
{
    const Dims &dm = ctx->dm;
    const WorkspaceLayout &wl = ctx->wl;
    for (int b0 = 0; b0 < batch; b0 += kBatMax) {
        BatParams B;
        std::memset(&B, 0, sizeof B);
        B.dm = dm; B.lay = ctx->lay; B.w = w; B.kv = kv;
        B.pos = pos_dev + b0;
        B.nb = batch - b0 < kBatMax ? batch - b0 : kBatMax;
        B.b0 = b0; B.layer = l; B.n_layers = n_layers;
        B.kv_b0 = kv_seq < 0 ? b0 : kv_seq;
        B.kv_bstep = kv_seq < 0 ? 1 : 0;
        B.x_in = static_cast<const __half *>(x) + (size_t)b0 * dm.h;
        B.out = static_cast<__half *>(out) + (size_t)b0 * dm.h;
        B.xres = reinterpret_cast<float *>(ctx->ws + wl.xres) + (size_t)b0 * 2 * dm.h;
        B.q = reinterpret_cast<float *>(ctx->ws + wl.q) + (size_t)b0 * dm.h;
        B.m = reinterpret_cast<float *>(ctx->ws + wl.m) + (size_t)b0 * dm.f;
        B.o = reinterpret_cast<float *>(ctx->ws + wl.o) + (size_t)b0 * dm.h;
        B.rope = reinterpret_cast<const float2 *>(ctx->ws + wl.rope);
        B.sync = reinterpret_cast<unsigned *>(ctx->ws + wl.sync);
        HIP_OK(launch_bat_qkv_up(B, sh.grid, s));
        if (sh.grid >= B.nb) {
            StepParams P = make_params(ctx, sh, b0, x, pos_dev, out, n_layers);
            if (kv_seq >= 0) { P.b = kv_seq; P.attn_bstep = 0; }
            HIP_OK(launch_attention_batched(P, B.nb, w, kv, sh.grid, sh.threads, s));
        } else {
            for (int b = b0; b < b0 + B.nb; ++b) {
                StepParams P = make_params(ctx, sh, b, x, pos_dev, out, n_layers);
                if (kv_seq >= 0) P.b = kv_seq;
                HIP_OK(launch_attention_only(P, w, kv, sh.grid, sh.threads, s));
            }
        }
        HIP_OK(launch_bat_out(B, sh.grid, s));
    }
    return CFPP_OK;
}

static cfpp_status check_persistent(const cfpp_ctx *ctx, const Shape &sh)
{
    int per_cu = 0;
    HIP_OK(persistent_occupancy(ctx->dm.d, sh.threads, (size_t)sh.lds_floats * 4, &per_cu));
    if ((long long)per_cu * ctx->n_cu < sh.grid)
        return fail(CFPP_EUNSUPPORTED,
                    "persistent mode needs all %d workgroups resident, device fits %d x %d", sh.grid,
                    per_cu, ctx->n_cu);
    return CFPP_OK;
}

// Mode 2 (whole stack, hand-overs hidden behind streaming): shape limits and residency.
// The answer depends on the launch shape only and is remembered for the last one asked.
static cfpp_status check_fused(cfpp_ctx *ctx, const Shape &sh, const StepParams &P)
{
    if (ctx->fused_grid == sh.grid && ctx->fused_threads == sh.threads && ctx->fused_ok) return CFPP_OK;
    if (!fused_supported(ctx->dm, P, sh.grid, sh.threads))
        return fail(CFPP_EUNSUPPORTED,
                    "mode 2 needs grid >= n_heads, at most 64 rows of the hidden-size matrices per workgroup, "
                    "hidden <= 4096, hidden and ffn multiples of 512 and head_dim 64, 80 or 128; use mode 0 for "
                    "this shape");
    const size_t lds = fused_lds_bytes(ctx->dm, P, sh.threads);
    if (lds > 160 * 1024) return fail(CFPP_EUNSUPPORTED, "mode 2 needs %zu bytes of LDS (> 160 KiB)", lds);
    int per_cu = 0;
    HIP_OK(fused_occupancy(ctx->dm.d, sh.threads, lds, &per_cu));
    if ((long long)per_cu * ctx->n_cu < sh.grid)
        return fail(CFPP_EUNSUPPORTED, "mode 2 needs all %d workgroups resident, device fits %d x %d", sh.grid,
                    per_cu, ctx->n_cu);
    ctx->fused_grid = sh.grid; ctx->fused_threads = sh.threads; ctx->fused_ok = true;
    return CFPP_OK;
}

static cfpp_status check_io(const cfpp_ctx *ctx, const void *x, const int32_t *pos_dev, int32_t batch,
                            const void *out)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    if (!aligned16(x) || !aligned16(out)) return fail(CFPP_EINVAL, "x or out is NULL or not 16-byte aligned");
    if (!pos_dev || (reinterpret_cast<uintptr_t>(pos_dev) & 3u)) return fail(CFPP_EINVAL, "pos_dev is NULL or misaligned");
    if (batch <= 0 || batch > ctx->cfg.max_batch)
        return fail(CFPP_EINVAL, "batch %d outside [1, max_batch = %d]", batch, ctx->cfg.max_batch);
    const char *xb = static_cast<const char *>(x), *ob = static_cast<const char *>(out);
    const size_t n = (size_t)batch * ctx->dm.h * 2;
    if (xb < ob + n && ob < xb + n) return fail(CFPP_EINVAL, "out overlaps x");
    return CFPP_OK;
}

// The launch mode a call runs in.  An explicit mode is checked and refused when
// the shape has no kernel in it; CFPP_MODE_AUTO takes the fastest mode that
// supports the call and never refuses: several sequences -> the batched
// projections (mode 0); the whole-stack kernel where its shape limits and the
// residency check allow it (a step of several layers always, a block on its own - or
// a one-layer stack - from hidden 2048 on: below that a block is a handful of
// dependent hand-overs with nothing to stream behind them and the three phase
// kernels are quicker); else the phase kernels.
static cfpp_status resolve_mode(cfpp_ctx *ctx, const Shape &sh, const StepParams &P, int batch, bool stack,
                                int *mode_out)
{
    int mode = ctx->mode;
    if (mode == CFPP_MODE_AUTO) {
        mode = 0;
        const bool one_by_one = batch == 1 || !batched_path_shape(ctx, sh);
        if (one_by_one && ((stack && ctx->cfg.n_layers > 1) || ctx->dm.h >= 2048)) {
            g_err_hold hold;                               // a refusal here is not the caller's error
            if (check_fused(ctx, sh, P) == CFPP_OK) mode = 2;
        }
        *mode_out = mode;
        return CFPP_OK;
    }
    *mode_out = mode;
    if (mode == 2) return check_fused(ctx, sh, P);
    if (mode == 1) return check_persistent(ctx, sh);
    return CFPP_OK;
}

// Tagged-word epochs: every launch of the whole-stack kernel uses up n_layers + 1
// values of a 32-bit counter that lives in the workspace.  Long before it could
// wrap (and a stale word compare equal to a live tag) the counter and the tagged
// region are zeroed again, between launches, never inside a graph.
static cfpp_status account_epochs(cfpp_ctx *ctx, unsigned long long need)
{
    if (ctx->epochs_used + need > ctx->epoch_limit) {
        cfpp_status st = reset_sync_words(ctx);
        if (st != CFPP_OK) return st;
    }
    ctx->epochs_used += need;
    return CFPP_OK;
}

static bool capturing(hipStream_t s)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cs) != hipSuccess) { (void)hipGetLastError(); return false; }
    return cs != hipStreamCaptureStatusNone;
}

// phases_only: run the phase kernels (launch mode 0) whatever the context's mode says
static cfpp_status block_decode(cfpp_ctx *ctx, const void *packed_layer, void *kv_layer, const void *x,
                                const int32_t *pos_dev, int32_t batch, void *out, cfpp_stream stream,
                                bool phases_only)
{
    cfpp_status st = check_io(ctx, x, pos_dev, batch, out);
    if (st != CFPP_OK) return st;
    if (!aligned16(packed_layer) || !aligned16(kv_layer))
        return fail(CFPP_EINVAL, "packed_layer or kv_layer is NULL or not 16-byte aligned");
    Shape sh;
    if ((st = launch_shape(ctx, &sh)) != CFPP_OK) return st;
    if ((st = prepare(ctx)) != CFPP_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool seq = ctx->dm.flags & kFlagSequentialResidual;
    int mode = 0;
    if (!phases_only &&
        (st = resolve_mode(ctx, sh, make_params(ctx, sh, 0, x, pos_dev, out, 1), batch, false, &mode)) != CFPP_OK)
        return st;
    const __half *w = static_cast<const __half *>(packed_layer);
    __half *kv = static_cast<__half *>(kv_layer);
    ctx->last_batch = batch;
    if (mode == 0 && batched_path(ctx, sh, batch)) return launch_batched_layer(ctx, sh, w, kv, 0, 1, x, pos_dev, batch, out, s);
    if (mode == 2 && !capturing(s) && (st = account_epochs(ctx, 2ull * batch)) != CFPP_OK) return st;
    for (int b = 0; b < batch; ++b) {
        StepParams P = make_params(ctx, sh, b, x, pos_dev, out, mode != 2 && seq ? 2 : 1);
        if (mode == 0 || mode == 1) {
            HIP_OK(launch_block_phases(P, w, kv, 0, sh.grid, sh.threads, s, mode == 1));
        } else {
            P.w_single = w;
            P.kv_single = kv;
            HIP_OK(launch_stack_fused(P, nullptr, sh.grid, sh.threads, s));
        }
    }
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_block_decode(cfpp_ctx *ctx, const void *packed_layer, void *kv_layer,
                                         const void *x, const int32_t *pos_dev, int32_t batch, void *out,
                                         cfpp_stream stream)
{
    return block_decode(ctx, packed_layer, kv_layer, x, pos_dev, batch, out, stream, false);
}

// store_table: also enqueue the copy of the pointer table into the workspace
// (the whole-stack kernel reads it from device memory).  Capture stores it
// ahead of the captured region, so a replay is the decode kernels alone.
// epochs: receives the tagged-word epochs the enqueued launches use up.
static cfpp_status enqueue_stack(cfpp_ctx *ctx, const void *const *packed_layers, void *const *kv_layers,
                                 const void *x, const int32_t *pos_dev, int32_t batch, void *out,
                                 hipStream_t s, bool store_table, bool launch, unsigned long long *epochs = nullptr)
{
    cfpp_status st = check_io(ctx, x, pos_dev, batch, out);
    if (st != CFPP_OK) return st;
    if (!packed_layers || !kv_layers) return fail(CFPP_EINVAL, "layer pointer arrays are NULL");
    const int L = ctx->cfg.n_layers;
    for (int l = 0; l < L; ++l)
        if (!aligned16(packed_layers[l]) || !aligned16(kv_layers[l]))
            return fail(CFPP_EINVAL, "layer %d: NULL or misaligned pointer", l);
    Shape sh;
    if ((st = launch_shape(ctx, &sh)) != CFPP_OK) return st;
    int mode = 0;
    if ((st = resolve_mode(ctx, sh, make_params(ctx, sh, 0, x, pos_dev, out, L), batch, true, &mode)) != CFPP_OK)
        return st;
    LayerPtrs ptrs;
    std::memset(&ptrs, 0, sizeof ptrs);
    for (int l = 0; l < L; ++l) {
        ptrs.w[l] = static_cast<const __half *>(packed_layers[l]);
        ptrs.kv[l] = static_cast<__half *>(kv_layers[l]);
    }
    LayerPtrs *dev_ptrs = reinterpret_cast<LayerPtrs *>(ctx->ws + ctx->wl.layer_ptrs);
    if (store_table && mode == 2) HIP_OK(launch_store_layer_ptrs(ptrs, dev_ptrs, L, s));
    if (epochs) *epochs = mode == 2 ? (unsigned long long)(L + 1) * batch : 0;
    if (!launch) return CFPP_OK;
    ctx->last_batch = batch;
    if (mode == 0 && batched_path(ctx, sh, batch)) {
        for (int l = 0; l < L; ++l)
            if ((st = launch_batched_layer(ctx, sh, ptrs.w[l], ptrs.kv[l], l, L, x, pos_dev, batch, out, s)) != CFPP_OK)
                return st;
        return CFPP_OK;
    }
    const int slots = (ctx->dm.flags & kFlagSequentialResidual) ? 2 : 1;   // residual slots per block, phase kernels
    for (int b = 0; b < batch; ++b) {
        const StepParams P = make_params(ctx, sh, b, x, pos_dev, out, mode != 2 ? L * slots : L);
        if (mode == 2) {
            HIP_OK(launch_stack_fused(P, dev_ptrs, sh.grid, sh.threads, s));
        } else {
            for (int l = 0; l < L; ++l)
                HIP_OK(launch_block_phases(P, ptrs.w[l], ptrs.kv[l], l, sh.grid, sh.threads, s, mode == 1));
        }
    }
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_stack_decode(cfpp_ctx *ctx, const void *const *packed_layers,
                                         void *const *kv_layers, const void *x, const int32_t *pos_dev,
                                         int32_t batch, void *out, cfpp_stream stream)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    cfpp_status st = prepare(ctx);
    if (st != CFPP_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!capturing(s)) {
        // (worst case: every sequence through the whole-stack kernel)
        if ((st = account_epochs(ctx, (unsigned long long)(ctx->cfg.n_layers + 1) * (batch > 0 ? batch : 1))) != CFPP_OK)
            return st;
    }
    return enqueue_stack(ctx, packed_layers, kv_layers, x, pos_dev, batch, out, s, true, true);
}

// Prompt processing: groups of up to kBatMax consecutive tokens, each group through every
// layer before the next group starts (the next group attends over this group's rows in
// every layer's cache).
extern "C" cfpp_status cfpp_stack_prefill(cfpp_ctx *ctx, const void *const *packed_layers, void *const *kv_layers,
                                          const void *x, int32_t pos0, int32_t n_tokens, int32_t b, void *out,
                                          cfpp_stream stream)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    cfpp_status st = prepare(ctx);
    if (st != CFPP_OK) return st;
    if (!aligned16(x) || !aligned16(out)) return fail(CFPP_EINVAL, "x or out is NULL or not 16-byte aligned");
    if (!packed_layers || !kv_layers) return fail(CFPP_EINVAL, "layer pointer arrays are NULL");
    const int L = ctx->cfg.n_layers;
    for (int l = 0; l < L; ++l)
        if (!aligned16(packed_layers[l]) || !aligned16(kv_layers[l]))
            return fail(CFPP_EINVAL, "layer %d: NULL or misaligned pointer", l);
    if (b < 0 || b >= ctx->cfg.max_batch) return fail(CFPP_EINVAL, "sequence %d outside [0, max_batch = %d)", b, ctx->cfg.max_batch);
    if (n_tokens <= 0 || pos0 < 0 || (long long)pos0 + n_tokens > ctx->cfg.max_seq)
        return fail(CFPP_EINVAL, "positions [%d, %d + %d) outside the cache of %d positions", pos0, pos0, n_tokens,
                    ctx->cfg.max_seq);
    {
        const char *xb = static_cast<const char *>(x), *ob = static_cast<const char *>(out);
        const size_t n = (size_t)n_tokens * ctx->dm.h * 2;
        if (xb < ob + n && ob < xb + n) return fail(CFPP_EINVAL, "out overlaps x");
    }
    Shape sh;
    if ((st = launch_shape(ctx, &sh)) != CFPP_OK) return st;
    if ((ctx->mode != 0 && ctx->mode != CFPP_MODE_AUTO) || (ctx->dm.flags & kFlagSequentialResidual))
        return fail(CFPP_EUNSUPPORTED, "prompt processing runs in launch mode 0 with the parallel residual form");
    if (!bat_supported(ctx->dm, sh.grid, sh.threads) || sh.grid < kBatMax)
        return fail(CFPP_EUNSUPPORTED, "prompt processing needs the batched projections: 512 threads, grid >= %d, hidden "
                    "and ffn multiples of 128, at most 64 matrix rows per workgroup", kBatMax);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t *pos_dev = reinterpret_cast<int32_t *>(ctx->ws + ctx->wl.pf_pos);
    HIP_OK(launch_fill_positions(pos_dev, pos0, n_tokens, s));
    // a group uses one workspace row per token: as many as the context has
    const int group = ctx->cfg.max_batch < kBatMax ? ctx->cfg.max_batch : kBatMax;
    const size_t h = (size_t)ctx->dm.h;
    for (int t0 = 0; t0 < n_tokens; t0 += group) {
        const int nb = n_tokens - t0 < group ? n_tokens - t0 : group;
        const __half *xg = static_cast<const __half *>(x) + (size_t)t0 * h;
        __half *og = static_cast<__half *>(out) + (size_t)t0 * h;
        for (int l = 0; l < L; ++l)
            if ((st = launch_batched_layer(ctx, sh, static_cast<const __half *>(packed_layers[l]),
                                           static_cast<__half *>(kv_layers[l]), l, L, xg, pos_dev + t0, nb, og, s,
                                           b)) != CFPP_OK)
                return st;
    }
    ctx->last_batch = 1;
    return CFPP_OK;
}

// Prompt processing with the weights read once per pass of up to `rows` tokens: every pass
// goes through all layers (LayerNorm inputs, four GEMMs and the causal attention per layer)
// before the next pass starts, which attends over this pass's rows in every layer's cache.
extern "C" cfpp_status cfpp_stack_prefill_gemm(cfpp_ctx *ctx, const void *const *packed_layers, void *const *kv_layers,
                                               const void *x, int32_t pos0, int32_t n_tokens, int32_t b, void *out,
                                               void *scratch, size_t scratch_bytes, int32_t rows, cfpp_stream stream)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    cfpp_status st = prepare(ctx);
    if (st != CFPP_OK) return st;
    if (!aligned16(x) || !aligned16(out)) return fail(CFPP_EINVAL, "x or out is NULL or not 16-byte aligned");
    if (!packed_layers || !kv_layers) return fail(CFPP_EINVAL, "layer pointer arrays are NULL");
    const int L = ctx->cfg.n_layers;
    for (int l = 0; l < L; ++l)
        if (!aligned16(packed_layers[l]) || !aligned16(kv_layers[l]))
            return fail(CFPP_EINVAL, "layer %d: NULL or misaligned pointer", l);
    if (b < 0 || b >= ctx->cfg.max_batch) return fail(CFPP_EINVAL, "sequence %d outside [0, max_batch = %d)", b, ctx->cfg.max_batch);
    if (n_tokens <= 0 || pos0 < 0 || (long long)pos0 + n_tokens > ctx->cfg.max_seq)
        return fail(CFPP_EINVAL, "positions [%d, %d + %d) outside the cache of %d positions", pos0, pos0, n_tokens,
                    ctx->cfg.max_seq);
    {
        const char *xb = static_cast<const char *>(x), *ob = static_cast<const char *>(out);
        const size_t n = (size_t)n_tokens * ctx->dm.h * 2;
        if (xb < ob + n && ob < xb + n) return fail(CFPP_EINVAL, "out overlaps x");
    }
    if (rows <= 0 || rows > kPfMaxRows || rows % kPfTile != 0)
        return fail(CFPP_EINVAL, "rows %d: a multiple of %d up to %d is needed", rows, kPfTile, kPfMaxRows);
    if (!pf_supported(ctx->dm))
        return fail(CFPP_EUNSUPPORTED, "the prompt-sized kernels need hidden and ffn multiples of %d, hidden <= 4096 and "
                    "the parallel residual form", kPfTile);
    const PfLayout pl = pf_layout(ctx->dm, rows);
    if (!scratch || (reinterpret_cast<uintptr_t>(scratch) & 255u))
        return fail(CFPP_EINVAL, "scratch is NULL or not 256-byte aligned");
    if (scratch_bytes < pl.total) return fail(CFPP_ENOMEM, "scratch of %zu bytes, %zu needed for %d rows", scratch_bytes, pl.total, rows);
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *sc = static_cast<char *>(scratch);
    const size_t h = (size_t)ctx->dm.h;
    for (int t0 = 0; t0 < n_tokens; t0 += rows) {
        PfParams P;
        std::memset(&P, 0, sizeof P);
        P.dm = ctx->dm; P.lay = ctx->lay;
        P.b = b; P.pos0 = pos0 + t0;
        P.n_rows = n_tokens - t0 < rows ? n_tokens - t0 : rows;
        P.rows = rows; P.n_layers = L;
        P.x_in = static_cast<const __half *>(x) + (size_t)t0 * h;
        P.out = static_cast<__half *>(out) + (size_t)t0 * h;
        P.y1h = reinterpret_cast<__half *>(sc + pl.y1h); P.y1l = reinterpret_cast<__half *>(sc + pl.y1l);
        P.y2h = reinterpret_cast<__half *>(sc + pl.y2h); P.y2l = reinterpret_cast<__half *>(sc + pl.y2l);
        P.stats = reinterpret_cast<float2 *>(sc + pl.stats);
        P.q = reinterpret_cast<float *>(sc + pl.q);
        P.oh = reinterpret_cast<__half *>(sc + pl.oh); P.ol = reinterpret_cast<__half *>(sc + pl.ol);
        P.mh = reinterpret_cast<__half *>(sc + pl.mh); P.ml = reinterpret_cast<__half *>(sc + pl.ml);
        P.part = reinterpret_cast<float *>(sc + pl.part);
        P.rope = reinterpret_cast<const float2 *>(ctx->ws + ctx->wl.rope);
        P.sync = reinterpret_cast<unsigned *>(ctx->ws + ctx->wl.sync);
        float *xa = reinterpret_cast<float *>(sc + pl.xres), *xb2 = reinterpret_cast<float *>(sc + pl.xnext);
        for (int l = 0; l < L; ++l) {
            P.layer = l;
            P.w = static_cast<const __half *>(packed_layers[l]);
            P.kv = static_cast<__half *>(kv_layers[l]);
            P.xres = (l & 1) ? xb2 : xa;                   // the block's output is the next block's input
            P.xnext = (l & 1) ? xa : xb2;
            HIP_OK(launch_pf_layer(P, s));
        }
    }
    ctx->last_batch = 1;
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_stack_capture(cfpp_ctx *ctx, const void *const *packed_layers,
                                          void *const *kv_layers, const void *x, const int32_t *pos_dev,
                                          int32_t batch, void *out, cfpp_stream stream)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!s) return fail(CFPP_EINVAL, "capture needs a non-default stream");
    cfpp_status st = prepare(ctx);
    if (st != CFPP_OK) return st;
    if (ctx->exec) { (void)hipGraphExecDestroy(ctx->exec); ctx->exec = nullptr; }
    if (ctx->graph) { (void)hipGraphDestroy(ctx->graph); ctx->graph = nullptr; }
    // validate and store the pointer table first (executes now, not captured)
    st = enqueue_stack(ctx, packed_layers, kv_layers, x, pos_dev, batch, out, s, true, false, &ctx->graph_epochs);
    if (st != CFPP_OK) return st;
    HIP_OK(hipStreamSynchronize(s));
    HIP_OK(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    st = enqueue_stack(ctx, packed_layers, kv_layers, x, pos_dev, batch, out, s, false, true);
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamEndCapture(s, &graph);
    if (st != CFPP_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return st;
    }
    if (e != hipSuccess) return fail(CFPP_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
    ctx->graph = graph;
    e = hipGraphInstantiate(&ctx->exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        ctx->exec = nullptr;
        return fail(CFPP_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
    }
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_stack_replay(cfpp_ctx *ctx, cfpp_stream stream)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    if (!ctx->exec) return fail(CFPP_ESTATE, "cfpp_stack_replay before cfpp_stack_capture");
    cfpp_status st = account_epochs(ctx, ctx->graph_epochs);
    if (st != CFPP_OK) return st;
    HIP_OK(hipGraphLaunch(ctx->exec, static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}

// ---- generation loop: embedding lookup, LM head, next token -----------------
static cfpp_status make_lm_params(cfpp_ctx *ctx, const cfpp_lm *lm, const int32_t *tokens_dev,
                                  const int32_t *pos_dev, Shape *sh, LmParams *L)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    if (!lm) return fail(CFPP_EINVAL, "lm is NULL");
    if (lm->vocab < 1) return fail(CFPP_EINVAL, "vocab %d < 1", lm->vocab);
    if (!aligned16(lm->embed) || !aligned16(lm->lnf_g) || !aligned16(lm->lnf_b) || !aligned16(lm->w_lm))
        return fail(CFPP_EINVAL, "an lm tensor is NULL or not 16-byte aligned");
    if (!tokens_dev || (reinterpret_cast<uintptr_t>(tokens_dev) & 3u) || !pos_dev ||
        (reinterpret_cast<uintptr_t>(pos_dev) & 3u))
        return fail(CFPP_EINVAL, "tokens_dev or pos_dev is NULL or misaligned");
    cfpp_status st = launch_shape(ctx, sh);
    if (st != CFPP_OK) return st;
    const Dims &dm = ctx->dm;
    std::memset(L, 0, sizeof *L);
    L->h = dm.h; L->vocab = lm->vocab; L->max_seq = dm.max_seq; L->eps = dm.ln_eps;
    L->embed = static_cast<const __half *>(lm->embed);
    L->lnf_g = static_cast<const __half *>(lm->lnf_g);
    L->lnf_b = static_cast<const __half *>(lm->lnf_b);
    L->w_lm = static_cast<const __half *>(lm->w_lm);
    L->tokens = tokens_dev; L->tokens_out = const_cast<int32_t *>(tokens_dev);
    L->pos = pos_dev; L->pos_out = const_cast<int32_t *>(pos_dev);
    L->best = reinterpret_cast<float *>(ctx->ws + ctx->wl.lm_best);
    L->sync = reinterpret_cast<unsigned *>(ctx->ws + ctx->wl.sync);
    L->rows = ceil_div(lm->vocab, sh->grid);
    if ((size_t)ceil_div(dm.h, kChunk) * kChunk > (size_t)kLmPerThread * sh->threads)
        return fail(CFPP_EUNSUPPORTED, "hidden %d needs more than %d values per thread at %d threads", dm.h,
                    kLmPerThread, sh->threads);
    const size_t lds = lm_head_lds_bytes(*L, sh->threads);
    if (lds > 160 * 1024)
        return fail(CFPP_EUNSUPPORTED, "the LM head needs %zu bytes of LDS with %d workgroups (> 160 KiB)", lds,
                    sh->grid);
    return CFPP_OK;
}

static cfpp_status prepare_lm(cfpp_ctx *ctx)
{
    if (ctx->lm_prepared) return CFPP_OK;
    HIP_OK(prepare_lm_kernels(160 * 1024));
    ctx->lm_prepared = true;
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_lm_embed(cfpp_ctx *ctx, const cfpp_lm *lm, const int32_t *tokens_dev,
                                     const int32_t *pos_dev, void *x, cfpp_stream stream)
{
    Shape sh;
    LmParams L;
    cfpp_status st = make_lm_params(ctx, lm, tokens_dev, pos_dev, &sh, &L);
    if (st != CFPP_OK) return st;
    if (!aligned16(x)) return fail(CFPP_EINVAL, "x is NULL or not 16-byte aligned");
    L.x = static_cast<__half *>(x);
    HIP_OK(launch_lm_embed(L, static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_lm_next(cfpp_ctx *ctx, const cfpp_lm *lm, const void *hidden, int32_t *tokens_dev,
                                    int32_t *pos_dev, float *logits_dev, cfpp_stream stream)
{
    Shape sh;
    LmParams L;
    cfpp_status st = make_lm_params(ctx, lm, tokens_dev, pos_dev, &sh, &L);
    if (st != CFPP_OK) return st;
    if (!aligned16(hidden)) return fail(CFPP_EINVAL, "hidden is NULL or not 16-byte aligned");
    if (logits_dev && (reinterpret_cast<uintptr_t>(logits_dev) & 3u)) return fail(CFPP_EINVAL, "logits_dev is misaligned");
    if ((st = prepare_lm(ctx)) != CFPP_OK) return st;
    L.hidden = static_cast<const __half *>(hidden);
    L.logits = logits_dev;
    HIP_OK(launch_lm_head(L, sh.grid, sh.threads, static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_generate_capture(cfpp_ctx *ctx, const void *const *packed_layers,
                                             void *const *kv_layers, const cfpp_lm *lm, int32_t *tokens_dev,
                                             int32_t *pos_dev, void *x_buf, void *hidden_buf, cfpp_stream stream)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!s) return fail(CFPP_EINVAL, "capture needs a non-default stream");
    Shape sh;
    LmParams L;
    cfpp_status st = make_lm_params(ctx, lm, tokens_dev, pos_dev, &sh, &L);
    if (st != CFPP_OK) return st;
    if (!aligned16(x_buf) || !aligned16(hidden_buf)) return fail(CFPP_EINVAL, "x_buf or hidden_buf is NULL or not 16-byte aligned");
    L.x = static_cast<__half *>(x_buf);
    L.hidden = static_cast<const __half *>(hidden_buf);
    if ((st = prepare(ctx)) != CFPP_OK) return st;
    if ((st = prepare_lm(ctx)) != CFPP_OK) return st;
    if (ctx->exec) { (void)hipGraphExecDestroy(ctx->exec); ctx->exec = nullptr; }
    if (ctx->graph) { (void)hipGraphDestroy(ctx->graph); ctx->graph = nullptr; }
    // validate and store the pointer table first (executes now, not captured)
    st = enqueue_stack(ctx, packed_layers, kv_layers, x_buf, pos_dev, 1, hidden_buf, s, true, false, &ctx->graph_epochs);
    if (st != CFPP_OK) return st;
    HIP_OK(hipStreamSynchronize(s));
    HIP_OK(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    hipError_t e = launch_lm_embed(L, s);
    if (e == hipSuccess) {
        st = enqueue_stack(ctx, packed_layers, kv_layers, x_buf, pos_dev, 1, hidden_buf, s, false, true);
        if (st == CFPP_OK) e = launch_lm_head(L, sh.grid, sh.threads, s);
    }
    hipGraph_t graph = nullptr;
    const hipError_t e2 = hipStreamEndCapture(s, &graph);
    if (st != CFPP_OK || e != hipSuccess || e2 != hipSuccess) {
        if (graph) (void)hipGraphDestroy(graph);
        if (st != CFPP_OK) return st;
        return fail(CFPP_EHIP, "capturing the generation step failed: %s", hipGetErrorString(e != hipSuccess ? e : e2));
    }
    ctx->graph = graph;
    e = hipGraphInstantiate(&ctx->exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        ctx->exec = nullptr;
        return fail(CFPP_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
    }
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_device_error(cfpp_ctx *ctx, cfpp_stream stream)
{
    if (!ctx) return fail(CFPP_EINVAL, "ctx is NULL");
    HIP_OK(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    unsigned words[64];
    HIP_OK(hipMemcpy(words, ctx->ws + ctx->wl.sync, sizeof words, hipMemcpyDeviceToHost));
    const unsigned err = words[kSyncErr];
    if (err == kErrNone) return CFPP_OK;
    // clear the flag and re-arm the barrier words and arrival counters
    {
        const cfpp_status st = reset_sync_words(ctx);
        if (st != CFPP_OK) return st;
    }
    if (err == kErrBadPos) return fail(CFPP_EDEVICE, "a position in pos_dev was outside [0, max_seq)");
    if (err == kErrBarrierTimeout) return fail(CFPP_EDEVICE, "grid barrier timed out (workgroups not co-resident?)");
    if (err == kErrBadToken) return fail(CFPP_EDEVICE, "a token in tokens_dev was outside [0, vocab)");
    return fail(CFPP_EDEVICE, "device error code %u", err);
}

// ---- block decode for callers that cannot allocate --------------------------------------
// The same step as cfpp_block_decode with the phase kernels, on a workspace that
// is a fixed array in device memory instead of a caller's buffer: nothing is
// allocated, no context is created.  Each GPU holds its own copy of the array at
// its own address; that address is looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kStaticMaxDevices = 16;
struct StaticSlot {
    char *ptr;              // device address of this GPU's copy of `scratch` (null: not looked up yet)
    bool configured;        // ctx below is set up for `cfg` and the array's sync words and rotary table match it
    cfpp_config cfg;
    cfpp_ctx ctx;
};
static StaticSlot g_static[kStaticMaxDevices];
static std::mutex g_static_mutex;

// words [0, n_zero) of `zero` cleared; the rotary table in double, as cfpp_create
// builds it on the host: angle = pos * base^(-2j/r)
__global__ void k_static_setup(unsigned *zero, int n_zero, float2 *rope, int max_seq, int half, int r, double base)
{
    const int stride = gridDim.x * blockDim.x;
    const int t0 = blockIdx.x * blockDim.x + threadIdx.x;
    for (int i = t0; i < n_zero; i += stride) zero[i] = 0u;
    for (long long i = t0; i < (long long)max_seq * half; i += stride) {
        const int t = (int)(i / half), j = (int)(i - (long long)t * half);
        const double a = (double)t * pow(base, -2.0 * j / (double)r);
        rope[i] = float2{(float)cos(a), (float)sin(a)};
    }
}

extern "C" cfpp_status cfpp_block_decode_static(const cfpp_config *c, const void *packed_layer, void *kv_layer,
                                                const void *x, const int32_t *pos_dev, int32_t batch, void *out,
                                                cfpp_stream stream)
{
    cfpp_status st = cfpp_validate_config(c);
    if (st != CFPP_OK) return st;
    const Dims dm = dims_of(*c);
    const WorkspaceLayout wl = workspace_layout(dm);
    if (wl.total > kStaticScratchBytes)
        return fail(CFPP_ENOMEM, "this configuration needs %zu bytes of workspace; the built-in array holds %zu "
                    "(lower max_seq or max_batch, or use cfpp_block_decode with a workspace of your own)",
                    wl.total, kStaticScratchBytes);
    int dev = 0;
    HIP_OK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return fail(CFPP_EUNSUPPORTED, "device %d: only devices 0..%d", dev, kStaticMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticSlot &S = g_static[dev];
    if (!S.ptr) {
        // (the array's name is a host-side stand-in; this is its address on the current device)
        char *ptr = nullptr;
        HIP_OK(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(CFPP_EHIP, "hipGetSymbolAddress returned a null address");
        S.ptr = ptr;
        S.configured = false;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!S.configured || std::memcmp(&S.cfg, c, sizeof *c) != 0) {
        int n_cu = 0;
        HIP_OK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
        int lds_limit = 0;
        HIP_OK(hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
        cfpp_ctx &ctx = S.ctx;
        const bool prepared = ctx.prepared, lm_prepared = ctx.lm_prepared;   // (kernel attributes: set once per process)
        ctx = cfpp_ctx();
        ctx.cfg = *c;
        ctx.dm = dm;
        ctx.lay = packed_layout(dm.h, dm.f);
        ctx.wl = wl;
        ctx.ws = S.ptr;
        ctx.n_cu = n_cu;
        ctx.mode = 0;
        ctx.grid = 0;
        ctx.threads = 512;
        ctx.epoch_limit = kEpochLimit;
        ctx.lds_limit = lds_limit > 0 ? (size_t)lds_limit : 65536;
        ctx.prepared = prepared;
        ctx.lm_prepared = lm_prepared;
        ctx.last_batch = 1;
        // the array keeps whatever the last configuration left: this one's sync words and
        // arrival counters start at zero, its rotary table is written (on `stream`, ahead of the step)
        const int half = dm.r / 2;
        hipLaunchKernelGGL(k_static_setup, dim3(256), dim3(256), 0, s, reinterpret_cast<unsigned *>(S.ptr + wl.sync),
                           (int)((wl.layer_ptrs - wl.sync) / 4), reinterpret_cast<float2 *>(S.ptr + wl.rope), dm.max_seq,
                           half, dm.r, (double)c->rope_base);
        HIP_OK(hipGetLastError());
        S.cfg = *c;
        S.configured = true;
    }
    return block_decode(&S.ctx, packed_layer, kv_layer, x, pos_dev, batch, out, stream, true);
}

#ifdef CFPP_PROFILE
// ---- profiling library only (declared in cfpp_profile.h) ------------------------------
extern "C" cfpp_status cfpp_debug_read(cfpp_ctx *ctx, int32_t which, float *dst_host, size_t count,
                                       cfpp_stream stream)
{
    if (!ctx || !dst_host) return fail(CFPP_EINVAL, "NULL argument");
    const Dims &dm = ctx->dm;
    size_t off, n;
    switch (which) {
    case 0: off = ctx->wl.q; n = (size_t)dm.max_batch * dm.h; break;
    case 1: off = ctx->wl.m; n = (size_t)dm.max_batch * dm.f; break;
    case 2: off = ctx->wl.g; n = (size_t)dm.max_batch * dm.h; break;
    case 3: off = ctx->wl.o; n = (size_t)dm.max_batch * dm.h; break;
    case 4: off = ctx->wl.trace; n = (size_t)kTraceWaves * kTraceLen * 4; break;   // raw timeline words
    default: return fail(CFPP_EINVAL, "unknown tap %d", which);
    }
    if (count > n) return fail(CFPP_EINVAL, "count %zu exceeds the buffer (%zu floats)", count, n);
    HIP_OK(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    HIP_OK(hipMemcpy(dst_host, ctx->ws + off, count * sizeof(float), hipMemcpyDeviceToHost));
    return CFPP_OK;
}

// ---- bandwidth calibration -------------------------------------------------------------
extern "C" cfpp_status cfpp_stream_read(const void *src, size_t bytes, void *sink, int32_t grid,
                                        int32_t threads, int32_t unroll, cfpp_stream stream)
{
    if (!aligned16(src) || !aligned16(sink) || (bytes & 15)) return fail(CFPP_EINVAL, "bad src/sink/bytes");
    if (grid <= 0 || grid > 65536 || (threads != 256 && threads != 512)) return fail(CFPP_EINVAL, "bad launch shape");
    HIP_OK(launch_stream_read(src, bytes, static_cast<unsigned *>(sink), grid, threads, unroll,
                              static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}

extern "C" cfpp_status cfpp_stream_copy(const void *src, void *dst, size_t bytes, int32_t grid,
                                        int32_t threads, cfpp_stream stream)
{
    if (!aligned16(src) || !aligned16(dst) || (bytes & 15)) return fail(CFPP_EINVAL, "bad src/dst/bytes");
    if (grid <= 0 || grid > 65536 || (threads != 256 && threads != 512)) return fail(CFPP_EINVAL, "bad launch shape");
    HIP_OK(launch_stream_copy(src, dst, bytes, grid, threads, static_cast<hipStream_t>(stream)));
    return CFPP_OK;
}
#endif  // CFPP_PROFILE
