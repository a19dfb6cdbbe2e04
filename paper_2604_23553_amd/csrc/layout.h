// Shared host/device description of the model shape, the packed layer blob,
// the KV-cache layout and the workspace.  No arithmetic of the method lives here.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define CFPP_HD __host__ __device__ inline
#else
#define CFPP_HD inline
#endif

namespace cfpp {

constexpr int kChunk = 512;        // fp16 values one wavefront covers with one 16-byte load per lane
constexpr int kMaxLayers = 64;
constexpr int kMaxGrid = 1024;     // most workgroups any launch uses
constexpr int kTraceWaves = 8, kTraceLen = 512;   // timeline trace of one workgroup (profiling aid)

CFPP_HD size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Dims {
    int h, H, d, r, f;
    int max_seq, max_batch;
    float ln_eps;
    int flags;       // kFlagTanhGelu, kFlagSequentialResidual
};

enum { kFlagTanhGelu = 1, kFlagSequentialResidual = 2 };
// parts of a block a phase launch performs (the sequential residual form runs a block in two halves)
enum { kPartQkv = 1, kPartUp = 2, kPartAttention = 4, kPartDown = 8, kPartDense = 16, kPartAll = 31 };

// Offsets (in fp16 elements) of every section of a packed layer.  Each section
// starts on a 256-byte boundary.  Matrices are row-major [rows][cols]; w_qkv and
// b_qkv use the packed row order (see qkv_packed_to_canonical).  Behind the
// tensors themselves sit two fp32 constants per row of the QKV and MLP-up
// matrices, derived from them when the layer is packed: with them a kernel can
// run those products on gamma * x before the LayerNorm statistics are known,
//   W (gamma * (x - mu) * inv + beta) + b = inv * (W (gamma * x) - mu * s) + c,
//   s = W gamma,  c = W beta + b   (rc_* holds (s, c) per packed row).
struct PackedLayout {
    size_t ln1_g, ln1_b, ln2_g, ln2_b;
    size_t b_qkv, b_dense, b_up, b_down;
    size_t w_qkv, w_up, w_down, w_dense;
    size_t rc_qkv, rc_up;   // per-row constants, float2 each (4 fp16 elements per row): see launch_pack_layer
    size_t total;   // fp16 elements
};

CFPP_HD PackedLayout packed_layout(int h, int f)
{
    PackedLayout L;
    size_t o = 0;
    auto take = [&](size_t n) { size_t at = o; o = align_up(o + n, 128); return at; };
    L.ln1_g = take(h); L.ln1_b = take(h); L.ln2_g = take(h); L.ln2_b = take(h);
    L.b_qkv = take(3 * (size_t)h); L.b_dense = take(h); L.b_up = take(f); L.b_down = take(h);
    L.w_qkv = take(3 * (size_t)h * h);
    L.w_up = take((size_t)f * h);
    L.w_down = take((size_t)h * f);
    L.w_dense = take((size_t)h * h);
    L.rc_qkv = take(4 * 3 * (size_t)h);
    L.rc_up = take(4 * (size_t)f);
    L.total = o;
    return L;
}

// Packed QKV row p of head block -> canonical row.  Within the q and k parts of
// a head the rotary dims are stored pairwise: packed (2j, 2j+1) = canonical
// (j, j + r/2), so one thread finishing two adjacent rows holds a whole
// rotation pair.  The v part and the non-rotary dims keep their order.
CFPP_HD int qkv_packed_dim_to_canonical(int c, int i, int r)
{
    if (c < 2 && i < r) return (i & 1) ? (i >> 1) + (r >> 1) : (i >> 1);
    return i;
}
CFPP_HD int qkv_packed_to_canonical_row(int p, int d, int r)
{
    int n = p / (3 * d), rem = p - n * 3 * d;
    int c = rem / d, i = rem - c * d;
    return (3 * n + c) * d + qkv_packed_dim_to_canonical(c, i, r);
}

// KV cache of one layer: fp16 [2][max_batch][H][d/16][max_seq][16].
CFPP_HD size_t kv_head_stride(const Dims &m) { return (size_t)m.d * m.max_seq; }
CFPP_HD size_t kv_which_stride(const Dims &m) { return (size_t)m.max_batch * m.H * kv_head_stride(m); }
CFPP_HD size_t kv_offset(const Dims &m, int which, int b, int n, int dim, int t)
{
    return (size_t)which * kv_which_stride(m) + ((size_t)b * m.H + n) * kv_head_stride(m)
         + ((size_t)(dim >> 4) * m.max_seq + t) * 16 + (dim & 15);
}
CFPP_HD size_t kv_layer_elems(const Dims &m) { return 2 * kv_which_stride(m); }

// Sync words: the device error flag, the epoch counter of the tagged words,
// then kSyncBarriers independent grid barriers of kSyncBarrierWords words each
// (generation word, root counter and up to 16 leaf counters, 128 bytes apart).
enum { kSyncErr = 32, kSyncEpoch = 40, kSyncBarrier0 = 64, kSyncGen = 0, kSyncRoot = 32, kSyncLeaf0 = 64,
       kSyncLeafStride = 32, kSyncLeaves = 16, kSyncBarrierWords = kSyncLeaf0 + kSyncLeaves * kSyncLeafStride,
       kSyncBarriers = 4, kSyncWords = kSyncBarrier0 + kSyncBarriers * kSyncBarrierWords };

// Workspace: byte offsets of every static buffer.
struct WorkspaceLayout {
    size_t sync;      // uint32[kSyncWords]: grid-barrier words, device error flag
    size_t seg_cnt;   // uint32[max_batch*H]: arrivals per (sequence, head) in the split-KV combine
    size_t layer_ptrs; // device copy of the per-layer pointer table of the stack kernel
    size_t tagged;    // whole-stack kernel's tagged words (value, epoch): xt[2][h] (3 h unused) ot[h] part[H][slots][d+2]
    size_t rope;      // float2[max_seq][r/2]: (cos, sin) of pos * theta_j
    size_t xres;      // float[2][max_batch][h]: fp32 residual stream between blocks (ping-pong)
    size_t q;         // float[max_batch][h]: rotated queries
    size_t m;         // float[max_batch][f]: GELU(up)
    size_t g;         // float[max_batch][h]: down projection + bias
    size_t o;         // float[max_batch][h]: attention output
    size_t part;      // float[max_batch*H][part_slots][d+2]: split-KV partials (acc[d], max, sum)
    size_t lm_best;   // float[kMaxGrid][2]: (logit, row) of every workgroup of the LM-head kernel
    size_t pf_pos;    // int32[max_seq]: positions of a prompt's tokens (prompt processing)
    size_t trace;     // uint64[kTraceWaves][kTraceLen][2]: (tag, 100 MHz clock) pairs (profiling library only, else empty)
    size_t total;
    int part_slots;
};

CFPP_HD int part_slots_for(int H) { return kMaxGrid / (H < 1 ? 1 : H) + 2; }

CFPP_HD WorkspaceLayout workspace_layout(const Dims &m)
{
    WorkspaceLayout W;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    W.part_slots = part_slots_for(m.H);
    W.sync = take((size_t)kSyncWords * 4);
    W.seg_cnt = take((size_t)m.max_batch * m.H * 4);
    W.layer_ptrs = take(2 * kMaxLayers * sizeof(void *));
    W.tagged = take(8 * ((size_t)6 * m.h + (size_t)m.H * W.part_slots * (m.d + 2)));
    W.rope = take((size_t)m.max_seq * (m.r / 2 > 0 ? m.r / 2 : 1) * 8);
    W.xres = take(2 * (size_t)m.max_batch * m.h * 4);
    W.q = take((size_t)m.max_batch * m.h * 4);
    W.m = take((size_t)m.max_batch * m.f * 4);
    W.g = take((size_t)m.max_batch * m.h * 4);
    W.o = take((size_t)m.max_batch * m.h * 4);
    W.part = take((size_t)m.max_batch * m.H * W.part_slots * (m.d + 2) * 4);
    W.lm_best = take((size_t)kMaxGrid * 8);
    W.pf_pos = take((size_t)m.max_seq * 4);
#ifdef CFPP_PROFILE
    W.trace = take((size_t)kTraceWaves * kTraceLen * 16);
#else
    W.trace = take(0);
#endif
    W.total = o;
    return W;
}


// device error codes
enum { kErrNone = 0, kErrBadPos = 1, kErrBarrierTimeout = 2, kErrBadToken = 3 };

}  // namespace cfpp
