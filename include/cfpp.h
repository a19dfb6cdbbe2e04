/*
 * cfpp — single-token decode of GPT-NeoX / Pythia decoder blocks on MI355X (gfx950).
 *
 * C ABI of the hot path of "ClusterFusion++" (arXiv 2604.23553): one call runs,
 * for one new token per sequence, the paper's fused region (Sec. 2.2)
 *
 *   pre-attention LayerNorm -> QKV projection + KV-cache update -> partial
 *   rotary embedding -> decode attention over the cache -> output projection
 *   -> post-attention LayerNorm -> MLP up / GELU / down -> residual
 *
 * in the residual form GPT-NeoX defines:
 *   out = x + Dense(Attn(LN1(x))) + Down(GELU(Up(LN2(x)))).
 * A second pair of calls runs an L-layer stack of such blocks as one launch
 * sequence or as one replayable HIP graph with static buffers (Sec. 2.3).
 *
 * Conventions
 *   - Every pointer named *device* is device memory owned by the caller
 *     (e.g. a torch tensor) that must stay alive while the library uses it;
 *     the library allocates no device memory.  Pointers must be 16-byte
 *     aligned.  Pointers named *host* are ordinary host memory.
 *   - fp16 means IEEE binary16.  All arithmetic accumulates in fp32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Compute calls only enqueue work; they never synchronise.
 *   - Every call returns a cfpp_status; nothing throws or exits.  The text of
 *     the last failure on the calling thread is in cfpp_last_error().
 *   - Results are bit-identical from run to run: every reduction has a fixed
 *     order and no floating-point atomics are used (the paper's fp16-atomic
 *     output accumulation, Sec. 3 "Output fidelity", is deliberately replaced).
 */
#ifndef CFPP_H
#define CFPP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t cfpp_status;
#define CFPP_OK            0
#define CFPP_EINVAL       (-1)  /* bad argument (null, misaligned, out of range)   */
#define CFPP_EUNSUPPORTED (-2)  /* valid request this build has no kernel for      */
#define CFPP_ENOMEM       (-3)  /* caller-provided buffer too small                */
#define CFPP_EHIP         (-4)  /* a HIP runtime call failed (see last_error)      */
#define CFPP_ESTATE       (-5)  /* call out of order (e.g. replay before capture)  */
#define CFPP_EDEVICE      (-6)  /* a kernel flagged an error (bad pos, barrier timeout) */

typedef void *cfpp_stream;      /* hipStream_t */

/* Model shape and limits.  Supported: head_dim in {64, 80, 128};
 * hidden == n_heads * head_dim; hidden and ffn multiples of 8; hidden <= 8192;
 * rotary_dims even, <= head_dim (Pythia: head_dim / 4, paper Sec. 2.2
 * "Architecture-Specific Adaptations"); 1 <= n_layers <= 64. */
typedef struct cfpp_config {
    int32_t hidden;       /* h                                               */
    int32_t n_heads;      /* H                                               */
    int32_t head_dim;     /* d                                               */
    int32_t rotary_dims;  /* r: leading dims of each head that are rotated   */
    int32_t ffn;          /* f: MLP width                                    */
    int32_t n_layers;     /* L: blocks in the stack                          */
    int32_t max_seq;      /* KV-cache capacity in positions (pos < max_seq)  */
    int32_t max_batch;    /* sequences the KV cache and workspace are sized for */
    float   rope_base;    /* 10000 for Pythia                                */
    float   ln_eps;       /* 1e-5 for Pythia                                 */
    int32_t flags;        /* CFPP_FLAG_* bits; 0 = the GPT-NeoX / Pythia block */
} cfpp_config;

/* The other readings of two points the paper leaves open (Sec. 2.2 says
 * "accelerated GELU" without naming the flavour, and lists the chain as output
 * projection with residual -> post-attention LayerNorm -> MLP with residual):
 *   CFPP_FLAG_TANH_GELU            gelu(z) = z/2 (1 + tanh(sqrt(2/pi)(z + 0.044715 z^3)))
 *                                  instead of the exact erf form (all launch modes)
 *   CFPP_FLAG_SEQUENTIAL_RESIDUAL  x1 = x + Dense(Attn(LN1(x))); out = x1 + Down(GELU(Up(LN2(x1))))
 *                                  instead of the parallel form (launch modes 0 and 1: two
 *                                  passes per block; mode 2 overlaps the two branches,
 *                                  which this form forbids, and returns
 *                                  CFPP_EUNSUPPORTED; CFPP_MODE_AUTO takes mode 0)      */
#define CFPP_FLAG_TANH_GELU 1
#define CFPP_FLAG_SEQUENTIAL_RESIDUAL 2

/* The 12 canonical fp16 tensors of one GPT-NeoX block, DEVICE pointers,
 * row-major.  w_qkv rows are interleaved per head (paper Sec. 2.2): row
 * (3*n + c)*d + i is dim i of q (c=0), k (c=1) or v (c=2) of head n. */
typedef struct cfpp_layer_src {
    const void *ln1_g, *ln1_b;      /* [h]  pre-attention LayerNorm  */
    const void *ln2_g, *ln2_b;      /* [h]  post-attention LayerNorm */
    const void *w_qkv, *b_qkv;      /* [3h, h], [3h]                 */
    const void *w_dense, *b_dense;  /* [h, h],  [h]                  */
    const void *w_up, *b_up;        /* [f, h],  [f]                  */
    const void *w_down, *b_down;    /* [h, f],  [h]                  */
} cfpp_layer_src;

typedef struct cfpp_ctx cfpp_ctx;

/* ---- errors -------------------------------------------------------------- */
const char *cfpp_status_string(cfpp_status s);
const char *cfpp_last_error(void);          /* thread-local, never NULL */

/* ---- host-only helpers (no GPU needed) ----------------------------------- */

/* CFPP_OK if `cfg` is a shape this build supports, else EINVAL / EUNSUPPORTED. */
cfpp_status cfpp_validate_config(const cfpp_config *cfg);

/* Bytes of one packed layer, of one layer's KV cache, and of the workspace.
 * 0 if cfg is invalid. */
size_t cfpp_packed_layer_bytes(const cfpp_config *cfg);
size_t cfpp_kv_layer_bytes(const cfpp_config *cfg);
size_t cfpp_workspace_bytes(const cfpp_config *cfg);

/* HBM bytes the method must move for one decode step of `n_layers` blocks:
 * per layer, the fp16 parameters (12h^2 + 13h values), the K and V rows of
 * positions 0..pos[b]-1 read, the new K and V rows written; plus x read and out
 * written once.  This is the numerator of the roofline fraction.  pos_host:
 * [batch] host array. */
cfpp_status cfpp_algorithmic_bytes(const cfpp_config *cfg, const int32_t *pos_host,
                                   int32_t batch, int32_t n_layers, uint64_t *bytes);

/* ---- one-time data preparation (device work, off the hot path) ----------- */

/* Packs one block's canonical tensors into the streaming layout the kernels
 * read: one blob with the LayerNorm parameters, the biases, and the four
 * matrices stored row-major so that a wavefront reads 1 KiB contiguous per
 * load; the QKV rows of each head are reordered so that the two rows of a
 * rotary pair (i, i + r/2) are adjacent.  Behind the tensors the blob carries
 * two fp32 values per row of the QKV and MLP-up matrices, computed here from
 * the packed tensors (s = W gamma, c = W beta + b of the LayerNorm in front of
 * the matrix, paper Sec. 2.2): the whole-stack kernel multiplies by gamma * x
 * and completes the LayerNorm in the epilogue with them.  packed_dst: DEVICE,
 * cfpp_packed_layer_bytes(cfg) bytes. */
cfpp_status cfpp_pack_layer(const cfpp_config *cfg, const cfpp_layer_src *src,
                            void *packed_dst, cfpp_stream stream);

/* KV cache of one layer, as the kernels keep it (DEVICE,
 * cfpp_kv_layer_bytes(cfg) bytes):
 *     fp16 [2 (K, V)][max_batch][n_heads][head_dim/16][max_seq][16]
 * i.e. for each head, 16-dim slabs with the position index next-to-innermost,
 * so that consecutive positions of a slab are contiguous 32-byte records.
 * Cached K rows are stored already rotated.
 *
 * cfpp_kv_import copies positions [0, n_pos) of sequence `b` from canonical
 * fp16 tensors k_src, v_src (DEVICE, [n_heads, src_capacity, head_dim]) into
 * kv_layer; cfpp_kv_export copies positions [pos_begin, pos_begin + n_pos) back
 * out into canonical tensors of the same shape convention (row t of the
 * destination receives position t). */
cfpp_status cfpp_kv_import(const cfpp_config *cfg, const void *k_src, const void *v_src,
                           int32_t src_capacity, int32_t n_pos, int32_t b,
                           void *kv_layer, cfpp_stream stream);
cfpp_status cfpp_kv_export(const cfpp_config *cfg, const void *kv_layer, int32_t b,
                           int32_t pos_begin, int32_t n_pos, int32_t dst_capacity,
                           void *k_dst, void *v_dst, cfpp_stream stream);

/* ---- context ------------------------------------------------------------- */

/* Creates a context over a caller-owned DEVICE workspace of at least
 * cfpp_workspace_bytes(cfg) bytes (static intermediate buffers, the rotary
 * cos/sin table, barrier words).  Initialises the workspace synchronously on
 * the current device.  The context holds only host bookkeeping and, after
 * cfpp_stack_capture, the instantiated graph. */
cfpp_status cfpp_create(const cfpp_config *cfg, void *workspace, size_t workspace_bytes,
                        cfpp_ctx **out_ctx);
void cfpp_destroy(cfpp_ctx *ctx);

/* Launch tuning.  Options may be changed between calls (not between capture
 * and replay).
 * Modes 1 and 2 launch persistent kernels whose workgroups wait for each other:
 * every workgroup of a launch must be resident at the same time.  The library
 * checks that one launch fits the device; the caller must not run them next to
 * other work on the same GPU (another stream or process): workgroups that do
 * not get a compute unit then stall the rest until a wait times out (after
 * about 2 s the step is abandoned and the device error flag raised, see
 * cfpp_device_error).  Calls of one context, and of contexts sharing a GPU,
 * belong on one stream. */
#define CFPP_OPT_MODE     1  /* CFPP_MODE_AUTO (the default): the fastest mode
                                that supports the call - the whole-stack kernel
                                (2) for a stack step and for a block of hidden
                                size >= 2048 when the shape and the device allow
                                it, the batched projections (0) for several
                                sequences, else the phase kernels (0); never
                                refuses a call for the mode's sake;
                                0: one kernel per phase (3 per block);
                                1: one persistent kernel per block;
                                2: one fused persistent kernel for the whole
                                   stack (cfpp_block_decode: for the one block),
                                   every grid-wide hand-over but the layer output
                                   hidden behind weight streaming (fastest; needs
                                   grid >= n_heads, hidden <= 4096, hidden and
                                   ffn multiples of 512, all workgroups resident,
                                   else CFPP_EUNSUPPORTED).                    */
#define CFPP_MODE_AUTO  (-1)
#define CFPP_OPT_GRID     2  /* workgroups; 0 = one per compute unit          */
#define CFPP_OPT_THREADS  3  /* threads per workgroup: 256 or 512             */
cfpp_status cfpp_set_option(cfpp_ctx *ctx, int32_t option, int64_t value);
cfpp_status cfpp_get_option(const cfpp_ctx *ctx, int32_t option, int64_t *value);

/* ---- the hot path --------------------------------------------------------- */

/* One decode step of ONE block (paper Sec. 2.2) for `batch` sequences.
 *   packed_layer : DEVICE, from cfpp_pack_layer
 *   kv_layer     : DEVICE, layout above; for sequence b the K and V rows of the
 *                  new token are written at position pos[b]; positions
 *                  0..pos[b]-1 are read; later positions are never touched
 *   x            : DEVICE fp16 [batch, hidden] block input
 *   pos_dev      : DEVICE int32 [batch]; 0 <= pos[b] < max_seq.  Read by the
 *                  kernels at run time (so a captured graph follows updates).
 *                  An out-of-range value makes the kernels skip the step and
 *                  raise the context's device error flag (cfpp_device_error).
 *   out          : DEVICE fp16 [batch, hidden] block output; must not alias x
 * Asynchronous on `stream`.
 * The sequences are independent and share the weights.  Launch mode 0 (and
 * CFPP_MODE_AUTO) with batch > 1 streams the weights once per group of up to 8 sequences (the
 * projections run on the matrix cores; needs 512 threads, hidden and ffn
 * multiples of 256, at most 64 matrix rows per workgroup, else - and in the
 * other launch modes - the sequences run one after the other).  With several
 * sequences a bad position in any of a group skips the whole group's step. */
cfpp_status cfpp_block_decode(cfpp_ctx *ctx, const void *packed_layer, void *kv_layer,
                              const void *x, const int32_t *pos_dev, int32_t batch,
                              void *out, cfpp_stream stream);

/* cfpp_block_decode for callers that cannot allocate device memory or keep a
 * context: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  It takes the configuration instead of a context and runs
 * the same step with the phase kernels (launch mode 0; several sequences: the
 * batched projections) on a workspace that is a fixed 16 MiB array in the
 * library's device image - no hipMalloc/hipFree, no workspace argument, nothing
 * to create or destroy.  Inputs and outputs are the caller's, as above.
 *   - CFPP_ENOMEM when cfpp_workspace_bytes(cfg) exceeds the 16 MiB (it grows
 *     with max_seq, max_batch, hidden and ffn: the Pythia-6.9B shape with 8
 *     sequences of 8192 positions needs about 8 MiB).
 *   - The first call on a GPU, and every call whose cfg differs from the
 *     previous call's on that GPU, first enqueues one small set-up kernel on
 *     `stream` (zeroes the array's counters, writes the rotary table for cfg).
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on
 *     one GPU (two streams, two threads) race; serialise them.  Each GPU has its
 *     own copy, held until the process ends.
 *   - An out-of-range position skips the step as in cfpp_block_decode; with no
 *     context there is no cfpp_device_error to report it: validate positions first.
 * Asynchronous on `stream`; host-side state is guarded by a mutex. */
cfpp_status cfpp_block_decode_static(const cfpp_config *cfg, const void *packed_layer, void *kv_layer,
                                     const void *x, const int32_t *pos_dev, int32_t batch,
                                     void *out, cfpp_stream stream);

/* One decode step through cfg.n_layers blocks.  packed_layers, kv_layers: HOST
 * arrays of n_layers DEVICE pointers.  The residual stream between blocks is
 * kept in fp32 in the workspace; fp16 only at x and out. */
cfpp_status cfpp_stack_decode(cfpp_ctx *ctx, const void *const *packed_layers,
                              void *const *kv_layers, const void *x,
                              const int32_t *pos_dev, int32_t batch, void *out,
                              cfpp_stream stream);

/* Prompt processing (the paper treats the prefill phase apart from its fused
 * decode kernel, Sec. 4.2 "Prefill Phase"; what it computes is the block applied
 * to every prompt token with causal attention, i.e. n_tokens decode steps one
 * after the other).  The tokens pass through all cfg.n_layers blocks in groups
 * of up to 8 consecutive positions (min(8, cfg.max_batch): a group uses one
 * workspace row per token): per group the weights are streamed once and the
 * projections run on the matrix cores, as for a batch of sequences, but every
 * row of the group is appended to the cache of sequence `b` before the group's
 * attention runs, so a token attends to the positions before it.
 *   x   : DEVICE [n_tokens][hidden] fp16, the tokens' input rows
 *   pos0: position of the first token (host value); positions below it must be
 *         cached already; rows pos0 .. pos0 + n_tokens - 1 of sequence b are
 *         written in every layer
 *   out : DEVICE [n_tokens][hidden] fp16, the last block's output per token;
 *         must not overlap x
 * Launch mode 0 or CFPP_MODE_AUTO only (CFPP_EUNSUPPORTED otherwise, or for shapes the batched
 * projections do not cover); CFPP_EINVAL for positions outside the cache.
 * Asynchronous on `stream`. */
cfpp_status cfpp_stack_prefill(cfpp_ctx *ctx, const void *const *packed_layers,
                               void *const *kv_layers, const void *x, int32_t pos0,
                               int32_t n_tokens, int32_t b, void *out, cfpp_stream stream);

/* The same computation for long prompts, with each layer's weights read once
 * per pass of up to `rows` tokens instead of once per 8: per layer a LayerNorm
 * launch, the four projections as LDS-tiled GEMMs on the matrix cores
 * (tokens x K activations times K x rows weights: here the paper's memory-bound
 * GEMVs, Sec. 2.2, are dense contractions), and one causal-attention launch over
 * the cache rows the pass has just appended.  Activations enter the fp16 matrix
 * instruction as head + remainder, so the products match the fp32 path to
 * rounding.  Arguments as for cfpp_stack_prefill, plus
 *   scratch      : DEVICE, 256-byte aligned, at least
 *                  cfpp_prefill_scratch_bytes(cfg, rows) bytes; the caller's,
 *                  contents undefined afterwards
 *   rows         : tokens per pass, a multiple of 128 up to 4096
 * Any launch mode (the kernels are its own).  CFPP_EUNSUPPORTED unless hidden and
 * ffn are multiples of 128, hidden <= 4096 and the residual form is the parallel
 * one; CFPP_ENOMEM for a scratch that is too small; CFPP_EINVAL as above.
 * cfpp_prefill_scratch_bytes returns 0 for an invalid configuration or rows.
 * Asynchronous on `stream`. */
size_t cfpp_prefill_scratch_bytes(const cfpp_config *cfg, int32_t rows);
cfpp_status cfpp_stack_prefill_gemm(cfpp_ctx *ctx, const void *const *packed_layers,
                                    void *const *kv_layers, const void *x, int32_t pos0,
                                    int32_t n_tokens, int32_t b, void *out, void *scratch,
                                    size_t scratch_bytes, int32_t rows, cfpp_stream stream);

/* Graph mode with static buffers (paper Sec. 2.3): capture records the whole
 * stack step for these exact pointers into one HIP graph (nothing executes);
 * each replay is one graph launch.  Between replays the caller updates the
 * CONTENTS of x and pos_dev.  `stream` must not be the default stream. */
cfpp_status cfpp_stack_capture(cfpp_ctx *ctx, const void *const *packed_layers,
                               void *const *kv_layers, const void *x,
                               const int32_t *pos_dev, int32_t batch, void *out,
                               cfpp_stream stream);
cfpp_status cfpp_stack_replay(cfpp_ctx *ctx, cfpp_stream stream);

/* ---- generation loop: the steps either side of the stack ---------------------
 * (paper Sec. 2.3 replays one graph per generated token with static buffers;
 * its Sec. 3 compares the generated tokens with the baseline's and does not name
 * the rule that picks them: the largest logit, lowest index among equals, is
 * taken here.)  One sequence.  The token sequence lives in DEVICE
 * memory indexed by position: tokens_dev[p] is the token whose K/V rows are
 * appended at cache row p; int32[max_seq + 1].
 *
 * cfpp_lm: DEVICE fp16 tensors, 16-byte aligned, owned by the caller:
 *   embed [vocab, hidden]   token embedding rows
 *   lnf_g, lnf_b [hidden]   final LayerNorm (eps = cfg.ln_eps, biased variance)
 *   w_lm  [vocab, hidden]   bias-free LM head, rows contiguous                  */
typedef struct cfpp_lm {
    const void *embed, *lnf_g, *lnf_b, *w_lm;
    int32_t vocab;
} cfpp_lm;

/* x[hidden] (DEVICE fp16) = embed[tokens_dev[*pos_dev]].  A token outside
 * [0, vocab) raises the device error flag (row 0 is used); a position outside
 * [0, max_seq) makes this and the next call do nothing (the stack step raises
 * the flag for it). */
cfpp_status cfpp_lm_embed(cfpp_ctx *ctx, const cfpp_lm *lm, const int32_t *tokens_dev,
                          const int32_t *pos_dev, void *x, cfpp_stream stream);

/* logits = w_lm LayerNorm(hidden) in fp32 (hidden: DEVICE fp16 [hidden], the
 * stack's output); tokens_dev[*pos_dev + 1] = index of the largest logit, the
 * lowest index among equal ones; then *pos_dev += 1.  logits_dev: DEVICE
 * float[vocab] that receives every logit, or NULL.  Uses the context's launch
 * shape (CFPP_OPT_GRID / CFPP_OPT_THREADS); CFPP_EUNSUPPORTED if vocab / grid rows
 * do not fit a workgroup's LDS. */
cfpp_status cfpp_lm_next(cfpp_ctx *ctx, const cfpp_lm *lm, const void *hidden, int32_t *tokens_dev,
                         int32_t *pos_dev, float *logits_dev, cfpp_stream stream);

/* Records embed -> stack step (batch 1, current launch mode) -> next token for
 * these exact pointers into the context's graph, replacing any captured one;
 * every cfpp_stack_replay then generates one token: it reads tokens_dev[pos],
 * appends the K/V rows at pos, writes tokens_dev[pos + 1] and advances *pos_dev.
 * x_buf, hidden_buf: DEVICE fp16 [hidden] scratch owned by the caller.  Replays
 * past the end of the cache (pos = max_seq) do nothing and raise the flag. */
cfpp_status cfpp_generate_capture(cfpp_ctx *ctx, const void *const *packed_layers,
                                  void *const *kv_layers, const cfpp_lm *lm, int32_t *tokens_dev,
                                  int32_t *pos_dev, void *x_buf, void *hidden_buf,
                                  cfpp_stream stream);

/* The whole-stack kernel marks the words its workgroups exchange with a 32-bit
 * epoch that every launch advances by n_layers + 1; the library counts the
 * epochs on the host and, before they could wrap (after about 2^32 / (n_layers + 1)
 * launches), waits for the device and zeroes the counter and the exchanged
 * words between two launches - once in days of continuous decoding; that one
 * call (cfpp_stack_decode, cfpp_block_decode or cfpp_stack_replay) synchronises. */

/* Synchronises `stream` and reports (and clears) the device error flag:
 * CFPP_OK, or CFPP_EDEVICE with the reason in cfpp_last_error(). */
cfpp_status cfpp_device_error(cfpp_ctx *ctx, cfpp_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CFPP_H */
