// Single-token decode of one GPT-NeoX block on gfx950, batch 1 per launch.
//
// The block (paper Sec. 2.2; residual form of GPT-NeoX, both branches read x)
// is cut into three phases separated by grid-wide dependencies:
//
//   A  LN1(x), LN2(x) (recomputed by every workgroup, x is a few KB)
//      -> QKV rows (+bias, partial rotary, K/V append, q to workspace)
//      -> MLP-up rows (+bias, exact GELU) -> m
//   B  split-KV attention partials over this workgroup's share of cache rows,
//      last-arriver fixed-order combine per head -> o;  MLP-down rows -> g
//   C  output-projection rows, out = x + (W_d o + b_d) + g
//
// Every matrix is row-split over workgroups (a workgroup owns whole output
// rows), so the only cross-workgroup reduction is the split-KV combine, which
// runs in a fixed order.  Nothing here uses floating-point atomics, so the
// output is bit-identical from run to run (unlike the fp16-atomic output
// accumulation the paper describes in Sec. 3).
//
// The same phase bodies are launched either as three kernels per block, as one
// persistent kernel per block, or as one persistent kernel for the whole stack
// (phases separated by a grid barrier; Sec. 2.3's graph mode wraps any of them).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "decode_params.h"
#include "device_utils.h"
#include "attention_common.h"

namespace cfpp {

constexpr int kMaxThreads = 512;
// After the attention the first wavefront still merges and publishes the partial
// while the others already stream the down projection: it takes a smaller share.
constexpr int kShare0AfterAttention = 0;
constexpr int kStageM = 16;       // the MLP intermediate is staged with up to 16 float2 per thread

// ---------------------------------------------------------------------------
// Row-split GEMV over this workgroup's rows.
//
// The rows a workgroup owns are contiguous in the packed layout, so its block of
// a matrix is one span of rows*K/512 "units" of 512 weights (1 KiB: one 16-byte
// load per lane).  Up to two such blocks (QKV rows then MLP-up rows) form one
// line of N units that is cut evenly over the wavefronts: wavefront w streams
// units [N*w/nw, N*(w+1)/nw) - a contiguous range of memory - and leaves one
// partial sum per row it touches in part[row*nw + w].  The epilogue adds the
// partials of a row in wavefront order.  The activation vector is in LDS (fp32,
// lds_perm order, zero padded to a unit multiple).
//
// Loads run two blocks of U units ahead of the arithmetic, and the first two
// blocks can be issued by the caller long before the activations exist (before a
// grid barrier, before the attention merges): weights depend on nothing.
#ifndef CFPP_GEMV_U
#define CFPP_GEMV_U 8
#endif
constexpr int kGemvU = CFPP_GEMV_U;
// the down projection's first blocks are in flight during the attention arithmetic, which
// needs most of the register file: smaller blocks there
constexpr int kGemvUDown = 4;

// The thread index as a value the optimiser cannot see through.  Inside the
// whole-stack kernel everything derived from the plain thread index is invariant
// across layers and would be hoisted out of the layer loop - dozens of
// precomputed addresses held in registers (or spilled) for the whole launch.
__device__ __forceinline__ int opaque_thread_index()
{
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

struct GemvSeg {
    const __half *W;     // first row of this workgroup's block
    const float *y;      // activations in LDS
    int K;               // row length
    int rows;            // rows in the block (may be 0)
};

template <int U_>
struct GemvSpan {
    static constexpr int U = U_;
    u32x4 a[U], b[U];
    const __half *w0, *w1;          // block bases (uniform)
    const __half *p0, *p1;          // the same, or `safe` when this wavefront streams nothing
    unsigned lane_off;              // this lane's byte offset inside a unit
    const float *y0, *y1;           // lane-adjusted activation bases
    int nch0, nch1, rows0, rows1, K0, K1;
    int n0, N, lo, hi, last, nw, wave, lane;
    const __half *safe;             // any readable 1 KiB: target of loads that are issued but not used
    int *bnd;
    bool regular;
    // walking state of consume()
    const float *yc;
    int c, nchc, rowg;
    float acc0, acc1;

    // bounds: nw + 1 ints of LDS (range starts of the wavefronts, then N).
    // share0: the first wavefront's share of the units in quarters of a full
    // share (4 = equal split); callers lower it when that wavefront has other
    // work to finish first.
    __device__ __forceinline__ void init(const GemvSeg &s0, const GemvSeg &s1, const __half *safe_, int tid,
                                         int *bounds, int share0 = 4)
    {
        safe = safe_;
        bnd = bounds;
        lane = tid & 63; wave = __builtin_amdgcn_readfirstlane(tid >> 6); nw = blockDim.x >> 6;
        w0 = s0.W; w1 = s1.W;
        lane_off = (unsigned)lane * 16u;
        y0 = s0.y + lane * 4; y1 = s1.y + lane * 4;
        K0 = s0.K; K1 = s1.K;
        rows0 = s0.rows; rows1 = s1.rows;
        regular = (s0.rows == 0 || s0.K % kChunk == 0) && (s1.rows == 0 || s1.K % kChunk == 0);
        nch0 = s0.K / kChunk; nch1 = s1.K / kChunk;
        n0 = rows0 * nch0;
        N = n0 + rows1 * nch1;
#ifdef CFPP_GEMV_INTERLEAVE
        // blocks of U units go round-robin over the wavefronts: the workgroup reads one moving window
        regular = regular && nch0 <= (nw - 1) * U && nch1 <= (nw - 1) * U;
        lo = regular ? wave * U : 0;
        hi = regular ? N : 0;
        last = regular && N > 0 ? N - 1 : -1;
#else
        {
            const int wtot = share0 + 4 * (nw - 1);
            const int c0 = wave == 0 ? 0 : share0 + 4 * (wave - 1), c1 = share0 + 4 * wave;
            lo = regular ? (int)((unsigned)N * (unsigned)c0 / (unsigned)wtot) : 0;
            hi = regular ? (int)((unsigned)N * (unsigned)c1 / (unsigned)wtot) : 0;
        }
        last = hi > lo ? hi - 1 : (regular && N > 0 ? (lo < N ? lo : N - 1) : -1);
#endif
        p0 = w0; p1 = w1;
        if (last < 0) { p0 = safe; p1 = safe; last = 0; }  // nothing to stream: loads go to the safe block
        const bool in1 = lo >= n0;
        nchc = in1 ? nch1 : nch0;
        const int local = in1 ? lo - n0 : lo;
        const int row = nchc ? local / nchc : 0;
        c = local - row * nchc;
        rowg = in1 ? rows0 + row : row;
        yc = in1 ? y1 : y0;
        acc0 = 0.f; acc1 = 0.f;
    }

    // Always exactly U load instructions on a single code path, so that the
    // hardware's in-order load counter (and the compiler's model of it) tells
    // precisely when an older block has landed while this one is still in
    // flight; a skipped or differently-routed load would force every wait to
    // drain the queue.  Units past the end of the range re-read its last unit.
    __device__ __forceinline__ const __half *unit_ptr(int u) const
    {
        const int uc = u < last ? u : last;
        const bool in0 = uc < n0;
        return (in0 ? p0 : p1) + (size_t)(in0 ? uc : uc - n0) * kChunk;
    }
    __device__ __forceinline__ void issue(u32x4 (&r)[U], int i) const
    {
#pragma unroll
        for (int j = 0; j < U; ++j) r[j] = load16_stream_at(unit_ptr(i + j), lane_off);
        // keep the instruction scheduler from sinking these loads towards their use
        __builtin_amdgcn_sched_barrier(0);
    }
    __device__ __forceinline__ void issue_first() { issue(a, lo); }
#ifdef CFPP_GEMV_INTERLEAVE
    __device__ __forceinline__ void issue_second() { issue(b, lo + nw * U); }
    __device__ __forceinline__ void seek(int i)
    {
        const bool in1 = i >= n0;
        nchc = in1 ? nch1 : nch0;
        const int local = in1 ? i - n0 : i;
        const int row = nchc ? local / nchc : 0;
        c = local - row * nchc;
        rowg = in1 ? rows0 + row : row;
        yc = in1 ? y1 : y0;
    }
#else
    __device__ __forceinline__ void issue_second() { issue(b, lo + U); }
#endif

    __device__ __forceinline__ void consume(const u32x4 (&r)[U], int i, float *part)
    {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int u = i + j;
            if (u < hi) {
                const float4 ya = *reinterpret_cast<const float4 *>(yc + c * kChunk);
                const float4 yb = *reinterpret_cast<const float4 *>(yc + c * kChunk + 256);
                if (j & 1) acc1 = dot8(r[j], ya, yb, acc1);
                else acc0 = dot8(r[j], ya, yb, acc0);
                ++c;
#ifdef CFPP_GEMV_INTERLEAVE
                if (c == nchc || u == hi - 1 || j == U - 1) {
#else
                if (c == nchc || u == hi - 1) {              // end of a row, or of this wavefront's range
#endif
                    const float tot = wave_sum(acc0 + acc1);
                    if (lane == 0) part[rowg * nw + wave] = tot;
                    acc0 = 0.f; acc1 = 0.f;
#ifdef CFPP_GEMV_INTERLEAVE
                    if (c == nchc) {
                        c = 0;
                        ++rowg;
                        if (rowg == rows0) { nchc = nch1; yc = y1; }
                    }
#else
                    c = 0;
                    ++rowg;
                    if (rowg == rows0) { nchc = nch1; yc = y1; }
#endif
                }
            }
        }
    }

    // rows with a ragged last unit (K not a multiple of 512): whole rows round-robin
    __device__ __forceinline__ void run_general(float *part) const
    {
        const int nrows = rows0 + rows1;
        for (int rg = wave; rg < nrows; rg += nw) {
            const bool in1 = rg >= rows0;
            const int K = in1 ? K1 : K0;
            const __half *wrow = (in1 ? w1 + (size_t)(rg - rows0) * K : w0 + (size_t)rg * K) + lane * 8;
            const float *yl = in1 ? y1 : y0;
            const int nchunk = (K + kChunk - 1) / kChunk;
            float acc = 0.f;
            for (int cc = 0; cc < nchunk; ++cc) {
                u32x4 wv = {0u, 0u, 0u, 0u};
                if (cc * kChunk + lane * 8 < K) wv = load16_stream(wrow + (size_t)cc * kChunk);
                const float4 ya = *reinterpret_cast<const float4 *>(yl + cc * kChunk);
                const float4 yb = *reinterpret_cast<const float4 *>(yl + cc * kChunk + 256);
                acc = dot8(wv, ya, yb, acc);
            }
            const float tot = wave_sum(acc);
            if (lane == 0) part[rg * nw] = tot;
        }
    }

    // consume everything; issue_first() and issue_second() have been called
    __device__ __forceinline__ void run(float *part)
    {
        if (!regular) { run_general(part); return; }
        int i = lo;
#ifdef CFPP_GEMV_INTERLEAVE
        const int st = nw * U;
        while (i < hi) {
            seek(i); consume(a, i, part); issue(a, i + 2 * st); i += st;
            if (i >= hi) break;
            seek(i); consume(b, i, part); issue(b, i + 2 * st); i += st;
        }
#else
        // Steady state: consume the older block, refill it two blocks ahead.  The
        // last two blocks are consumed without issuing anything, so that no load
        // is left in flight when the epilogue (or a grid barrier) waits on memory.
        bool a_older = true;
        while (i + 2 * U < hi) {
            consume(a, i, part); issue(a, i + 2 * U); i += U;
            a_older = false;
            if (i + 2 * U >= hi) break;
            consume(b, i, part); issue(b, i + 2 * U); i += U;
            a_older = true;
        }
        if (a_older) { consume(a, i, part); consume(b, i + U, part); }
        else { consume(b, i, part); consume(a, i + U, part); }
#endif
    }

    // after run() and a workgroup barrier: the dot product of global row rg
    // (0..rows0-1 first block, then the second block's rows).  Every wavefront
    // slot of the row is added, in wavefront order; slots of wavefronts that did
    // not touch the row hold the zero written by clear_partials().
    __device__ __forceinline__ float row_total(const float *part, int rg) const
    {
        const float *pr = part + rg * nw;
        float t = 0.f;
        for (int w = 0; w < nw; w += 4) {
            const float4 v = *reinterpret_cast<const float4 *>(pr + w);
            t = (((t + v.x) + v.y) + v.z) + v.w;
        }
        return t;
    }
};

// zero the (rows * nw) partial-sum slots; a workgroup barrier must follow before run()
__device__ __forceinline__ void clear_partials(float *part, int nslots, int tid)
{
    for (int i = tid; i < nslots; i += blockDim.x) part[i] = 0.f;
}

// Epilogue work items are dealt to lanes wavefront-major (item i -> wavefront
// i % nw), so that a few dozen rows are finished by all wavefronts together
// rather than by the first one alone.
__device__ __forceinline__ int spread_index(int tid)
{
    return (tid & 63) * (int)(blockDim.x >> 6) + (tid >> 6);
}

struct NoSync {
    static constexpr bool kInputsReady = true;    // everything this launch reads was written before it started

    __device__ __forceinline__ void wait() {}
    __device__ __forceinline__ void arrive() {}
};
struct GridSync {
    static constexpr bool kInputsReady = false;   // inputs appear behind a grid barrier
    GridBarrier &bar;
    __device__ __forceinline__ void wait() { bar.wait(); }
    __device__ __forceinline__ void arrive() { bar.arrive(); }
};

// sum of a value over the workgroup, fixed order; red: >= 16 floats of LDS
__device__ __forceinline__ float block_sum(float v, float *red, int tid)
{
    const int lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    v = wave_sum(v);
    __syncthreads();                 // red may still be read from a previous use
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < nw; ++w) t += red[w];
    return t;
}

struct LayerIO {
    const __half *x16;   // block input as fp16, or
    const float *x32;    // as fp32 (exactly one is non-null)
    __half *o16;         // block output as fp16, or
    float *o32;          // as fp32
};

__device__ __forceinline__ LayerIO layer_io(const StepParams &P, int layer)
{
    LayerIO io;
    io.x16 = layer == 0 ? P.x_in : nullptr;
    io.x32 = layer == 0 ? nullptr : P.xres + (size_t)((layer - 1) & 1) * P.dm.h;
    const bool last = layer == P.n_layers - 1;
    io.o16 = last ? P.out : nullptr;
    io.o32 = last ? nullptr : P.xres + (size_t)(layer & 1) * P.dm.h;
    return io;
}

__device__ __forceinline__ float load_x(const LayerIO &io, int i)
{
    return io.x16 ? __half2float(io.x16[i]) : xwg_load(io.x32 + i);
}

__device__ __forceinline__ int round_up_chunk(int k) { return (k + kChunk - 1) / kChunk * kChunk; }

// ---------------------------------------------------------------------------
// Phase A.  LDS: y1[Kp] y2[Kp] part[(rows_qkv + rows_up) * nw] bounds[16] red[16]
template <class Sync>
__device__ __forceinline__ void phase_a(const StepParams &P, const __half *__restrict__ w, __half *__restrict__ kv,
                                        int layer, int pos, float *lds, Sync &sync)
{
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, d = dm.d, r = dm.r;
    const int tid = opaque_thread_index(), nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(h);
    float *y1 = lds, *y2 = lds + Kp, *part = lds + 2 * Kp;
    int *bnd = reinterpret_cast<int *>(part + (P.rows_qkv + P.rows_up) * (nt >> 6));
    float *red = reinterpret_cast<float *>(bnd + 16);
    const LayerIO io = layer_io(P, layer);

    // weights first: they depend on nothing, so their loads overlap the wait for x
    const int q_begin = g * P.rows_qkv, q_n = max(0, min(P.rows_qkv, 3 * h - q_begin));
    const int u_begin = g * P.rows_up, u_n = max(0, min(P.rows_up, f - u_begin));
    GemvSpan<kGemvU> gs;
    gs.init(GemvSeg{w + P.lay.w_qkv + (size_t)q_begin * h, y1, h, q_n},
            GemvSeg{w + P.lay.w_up + (size_t)u_begin * h, y2, h, u_n}, w, tid, bnd);
    clear_partials(part, (P.rows_qkv + P.rows_up) * (nt >> 6), tid);
    // Epilogue items: the lower half of the wavefronts finishes pairs of QKV
    // rows, the upper half MLP-up rows, items dealt wavefront-major inside a
    // half.  What an item adds (biases, the rotary cos/sin) is requested now: a
    // load issued after the GEMV would cost a full memory round trip with
    // nothing left to hide it.
    const __half *bq = w + P.lay.b_qkv, *bu = w + P.lay.b_up;
    const int hw = nt >> 7, estride = 64 * hw;           // wavefronts per half, items per pass
    const bool up_half = (tid >> 6) >= hw;
    const int item0 = (tid & 63) * hw + ((tid >> 6) - (up_half ? hw : 0));
    float bq0 = 0.f, bq1 = 0.f, bu0 = 0.f;
    float2 cs0 = {1.f, 0.f};
    if (!up_half && item0 < q_n / 2) {
        const int p = q_begin + 2 * item0;
        const int i = p % d, c = (p / d) % 3;
        bq0 = __half2float(bq[p]); bq1 = __half2float(bq[p + 1]);
        if (c < 2 && i < r) cs0 = P.rope[(size_t)pos * (r >> 1) + (i >> 1)];
    }
    if (up_half && item0 < u_n) bu0 = __half2float(bu[u_begin + item0]);

    Tracer tr;
    tr.init(P, gs.wave, 0);
    tr.mark(1);
    if constexpr (!Sync::kInputsReady) gs.issue_first();   // weights stream while x is waited for
    sync.wait();
    tr.mark(2);

    // Both LayerNorms read the block input.  A thread owns up to GU groups of 8
    // consecutive elements; x and the four parameter vectors are fetched with
    // 16-byte loads that are all in flight together, statistics are two-pass on
    // registers.
    constexpr int GU = 4;
    const int ngrp = h >> 3, ngrp_p = Kp >> 3;
    float xv[GU][8];
    u32x4 pg1[GU], pb1[GU], pg2[GU], pb2[GU];
    const __half *g1 = w + P.lay.ln1_g, *b1 = w + P.lay.ln1_b;
    const __half *g2 = w + P.lay.ln2_g, *b2 = w + P.lay.ln2_b;
#pragma unroll
    for (int j = 0; j < GU; ++j) {
        const int gi = tid + j * nt;
        const u32x4 z = {0u, 0u, 0u, 0u};
        pg1[j] = z; pb1[j] = z; pg2[j] = z; pb2[j] = z;
#pragma unroll
        for (int e = 0; e < 8; ++e) xv[j][e] = 0.f;
        if (gi < ngrp) {
            if (io.x16) {
                const u32x4 xr = load16(io.x16 + gi * 8);
                const float2 a = unpack_h2(xr.x), b = unpack_h2(xr.y), c = unpack_h2(xr.z), e2 = unpack_h2(xr.w);
                xv[j][0] = a.x; xv[j][1] = a.y; xv[j][2] = b.x; xv[j][3] = b.y;
                xv[j][4] = c.x; xv[j][5] = c.y; xv[j][6] = e2.x; xv[j][7] = e2.y;
            } else {
                const float *xp = io.x32 + gi * 8;
                const float2 a = xwg_load2(xp), b = xwg_load2(xp + 2), c = xwg_load2(xp + 4), e2 = xwg_load2(xp + 6);
                xv[j][0] = a.x; xv[j][1] = a.y; xv[j][2] = b.x; xv[j][3] = b.y;
                xv[j][4] = c.x; xv[j][5] = c.y; xv[j][6] = e2.x; xv[j][7] = e2.y;
            }
            pg1[j] = load16(g1 + gi * 8); pb1[j] = load16(b1 + gi * 8);
            pg2[j] = load16(g2 + gi * 8); pb2[j] = load16(b2 + gi * 8);
        }
    }
    if constexpr (Sync::kInputsReady) gs.issue_first();    // x is already on its way: it returns first
    gs.issue_second();
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < GU; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) s += xv[j][e];
    const float mean = block_sum(s, red, tid) / (float)h;
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < GU; ++j) {
        if (tid + j * nt < ngrp) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dlt = xv[j][e] - mean;
                v += dlt * dlt;
            }
        }
    }
    const float var = block_sum(v, red, tid) / (float)h;
    const float inv = 1.0f / sqrtf(var + dm.ln_eps);
#pragma unroll
    for (int j = 0; j < GU; ++j) {
        const int gi = tid + j * nt;
        if (gi < ngrp_p) {
            float ya[8], yb[8];
            const bool real = gi < ngrp;
            const unsigned wg1[4] = {pg1[j].x, pg1[j].y, pg1[j].z, pg1[j].w};
            const unsigned wb1[4] = {pb1[j].x, pb1[j].y, pb1[j].z, pb1[j].w};
            const unsigned wg2[4] = {pg2[j].x, pg2[j].y, pg2[j].z, pg2[j].w};
            const unsigned wb2[4] = {pb2[j].x, pb2[j].y, pb2[j].z, pb2[j].w};
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const float2 ga = unpack_h2(wg1[e2]), ba = unpack_h2(wb1[e2]);
                const float2 gb = unpack_h2(wg2[e2]), bb = unpack_h2(wb2[e2]);
                const float t0 = (xv[j][2 * e2] - mean) * inv, t1 = (xv[j][2 * e2 + 1] - mean) * inv;
                ya[2 * e2] = real ? t0 * ga.x + ba.x : 0.f;
                ya[2 * e2 + 1] = real ? t1 * ga.y + ba.y : 0.f;
                yb[2 * e2] = real ? t0 * gb.x + bb.x : 0.f;
                yb[2 * e2 + 1] = real ? t1 * gb.y + bb.y : 0.f;
            }
            const int at = ((gi >> 6) << 9) + ((gi & 63) << 2);     // = lds_perm(8 * gi)
            *reinterpret_cast<float4 *>(y1 + at) = float4{ya[0], ya[1], ya[2], ya[3]};
            *reinterpret_cast<float4 *>(y1 + at + 256) = float4{ya[4], ya[5], ya[6], ya[7]};
            *reinterpret_cast<float4 *>(y2 + at) = float4{yb[0], yb[1], yb[2], yb[3]};
            *reinterpret_cast<float4 *>(y2 + at + 256) = float4{yb[4], yb[5], yb[6], yb[7]};
        }
    }
    __syncthreads();
    tr.mark(3);

    gs.run(part);
    tr.mark(4);
    __syncthreads();
    tr.mark(5);

    if (!up_half) {
        // QKV epilogue: one thread per pair of adjacent packed rows
        for (int pr = item0; pr < q_n / 2; pr += estride) {
            const int p = q_begin + 2 * pr;             // packed row, even
            const int pd = p / d, i = p - pd * d;       // i even
            const int n = pd / 3, c = pd - 3 * n;
            const bool rotary = c < 2 && i < r;         // rotary pair (j, j + r/2)
            float b0 = bq0, b1 = bq1;
            float2 cs = cs0;
            if (pr != item0) {                          // more pairs than threads: tiny grids only
                b0 = __half2float(bq[p]); b1 = __half2float(bq[p + 1]);
                if (rotary) cs = P.rope[(size_t)pos * (r >> 1) + (i >> 1)];
            }
            float v0 = gs.row_total(part, 2 * pr) + b0;
            float v1 = gs.row_total(part, 2 * pr + 1) + b1;
            int d0 = i, d1 = i + 1;
            if (rotary) {
                const int j = i >> 1;
                const float lo = v0 * cs.x - v1 * cs.y;
                const float hi = v1 * cs.x + v0 * cs.y;
                v0 = lo; v1 = hi;
                d0 = j; d1 = j + (r >> 1);
            }
            if (c == 0) {
                xwg_store(P.q + n * d + d0, v0);
                xwg_store(P.q + n * d + d1, v1);
            } else {
                xwg_store_half(kv + kv_offset(dm, c - 1, P.b, n, d0, pos), v0);
                xwg_store_half(kv + kv_offset(dm, c - 1, P.b, n, d1, pos), v1);
            }
        }
    } else {
        for (int t = item0; t < u_n; t += estride) {
            const float b = t == item0 ? bu0 : __half2float(bu[u_begin + t]);
            xwg_store(P.m + u_begin + t, gelu_erf(gs.row_total(part, q_n + t) + b));
        }
    }
    tr.mark(6);
    sync.arrive();
}

// ---------------------------------------------------------------------------
// Split-KV decode attention over this workgroup's share of the cache.
//
// LPP lanes share one cache position (2 for head_dim 64 and 80, 4 for 128), so a
// wavefront step ("row") covers PPW = 64/LPP positions.  Lane (position p,
// sub-lane u) handles the 8-dim pieces u, u+LPP, ... of the head; piece c lives
// in slab c/2, half c%2 of the cache layout, so one load instruction reads
// whole 32-byte records of consecutive positions (>= 512 B contiguous runs).
//
// All (head, row) pairs of the sequence form one line of T = H * ceil(n_tok/PPW)
// rows; workgroup g owns rows [T*g/G, T*(g+1)/G), which may cover the tail of
// one head and the start of the next.  Each lane group keeps its own
// online-softmax state (running max, sum, accumulators for its pieces); states
// are merged lane -> wavefront -> workgroup -> head, each in a fixed order.  The
// workgroup that delivers the last partial of a head combines all of that
// head's partials in slot order.  K/V loads of the next row are issued before
// the current row is processed.
// scr: nw*(D+2) + 4 + 2*D floats of LDS.
// pre(): called once, after the first row of already-cached K/V has been
// requested and before anything written during this launch (q, the new token's
// K/V) is read.  early(): called once, when every K/V load of the first two rows
// has been requested (the caller requests what it wants in flight during the
// arithmetic).  mid(): called once, ahead of the first workgroup barrier (the
// caller finishes staging its LDS vectors there).  tail(): called once, when the last K/V rows have been consumed,
// ahead of the last merges.
template <int D, class Pre, class Early, class Mid, class Tail>
__device__ __forceinline__ void attn_share(const StepParams &P, const __half *__restrict__ kv, int n_tok,
                                           float *scr, int tid, Pre &&pre, Early &&early, Mid &&mid, Tail &&tail,
                                           Tracer &tr)
{
    using A = AttnShape<D>;
    constexpr int LPP = A::LPP, PPW = A::PPW, NP = A::NP, NV = A::NV;
    const Dims &dm = P.dm;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = blockDim.x >> 6;
    const int sub = lane & (LPP - 1), tl = lane / LPP;
    const int H = dm.H;
    const int g = blockIdx.x;
    // (host-checked: rows * workgroups stays far below 2^31)
    const int R = (n_tok + PPW - 1) / PPW;
    const int T = R * H;
    // with fewer rows than workgroups only the first T workgroups take part, so
    // that every participant owns at least one row (no empty ranges in between)
    const int G = min((int)gridDim.x, T);
    const int r0 = g < G ? (int)((long long)T * g / G) : 0, r1 = g < G ? (int)((long long)T * (g + 1) / G) : 0;
    const float scale = 1.0f / sqrtf((float)D);
    const size_t hs = kv_head_stride(dm);
    const __half *Kb = kv + kv_offset(dm, 0, P.b, 0, 0, 0);
    const __half *Vb = kv + kv_offset(dm, 1, P.b, 0, 0, 0);
    float *wp = scr, *wm = scr + nw * D, *wl = wm + nw;
    float *qs = wl + nw + 4;                               // this head's query
    __half *kn = reinterpret_cast<__half *>(qs + D);       // the new token's K and V rows of this head
    __half *vn = kn + D;

    if (r0 >= r1) {                                        // no rows for this workgroup
        pre();
        early();
        mid();
        __syncthreads();
        tail();
        return;
    }

    // byte offset of this lane's piece k inside a head, for position 0 (a head's
    // K or V is d * max_seq * 2 bytes, far below 4 GiB)
    unsigned koff[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int pc = sub + LPP * k;
        koff[k] = ((unsigned)(pc >> 1) * (unsigned)dm.max_seq * 16u + (unsigned)(pc & 1) * 8u) * 2u;
    }

    // K/V of one row into registers: always exactly 2*NP load instructions with
    // every lane active, so that the in-order load counter tells when this row
    // has landed while the next one is still in flight.  Lanes past the last
    // cached position re-read it (their weight is zero); the new token's row
    // comes from LDS (kn, vn), not from here.
    const int t_last = n_tok >= 2 ? n_tok - 2 : 0;
    // (row < 0: nothing is needed, every lane reads the same record)
    auto issue = [&](u32x4 (&kk)[NP], u32x4 (&vv)[NP], const __half *Kh, const __half *Vh, int row) {
        const int t = row < 0 ? t_last : row * PPW + tl;
        const unsigned tb = (unsigned)(t < t_last ? t : t_last) * 32u;
#pragma unroll
        for (int k = 0; k < NP; ++k) kk[k] = load16_stream_at(Kh, koff[k] + tb);
#pragma unroll
        for (int k = 0; k < NP; ++k) vv[k] = load16_stream_at(Vh, koff[k] + tb);
        __builtin_amdgcn_sched_barrier(0);                 // the loads stay here, ahead of the arithmetic
    };

    // this head's query and the new token's K/V rows -> registers -> LDS
    float q_r = 0.f;
    __half kn_r = __float2half(0.f), vn_r = kn_r;
    auto head_issue = [&](int s) {
        if (tid < D) {
            q_r = xwg_load(P.q + s * D + tid);
            kn_r = xwg_load_half(kv + kv_offset(dm, 0, P.b, s, tid, n_tok - 1));
            vn_r = xwg_load_half(kv + kv_offset(dm, 1, P.b, s, tid, n_tok - 1));
        }
    };
    auto head_commit = [&] {
        if (tid < D) { qs[tid] = q_r; kn[tid] = kn_r; vn[tid] = vn_r; }
    };

    // Order of the requests: first row of cached K/V (needs nothing), then -
    // behind the caller's wait - the small vectors written during this launch,
    // then the second row and the caller's next weights.  The small loads return
    // while the bulk behind them is still streaming.
    u32x4 kA[NP], vA[NP], kB[NP], vB[NP];
    bool first = true;
    {
        const int s = r0 / R;
        const int se = min(r1, (s + 1) * R);
        const int row_lo = r0 - s * R, row_hi = se - s * R;
        const int row = row_lo + wave;
        issue(kA, vA, Kb + (size_t)s * hs, Vb + (size_t)s * hs, row < row_hi ? row : -1);
        pre();
        head_issue(s);
        issue(kB, vB, Kb + (size_t)s * hs, Vb + (size_t)s * hs, row + nw < row_hi ? row + nw : -1);
        early();
        head_commit();
        mid();
    }

    for (int sb = r0; sb < r1;) {
        const int s = sb / R;                              // head
        const int se = min(r1, (s + 1) * R);
        const int row_lo = sb - s * R, row_hi = se - s * R;
        const __half *Kh = Kb + (size_t)s * hs;
        const __half *Vh = Vb + (size_t)s * hs;

        int row = row_lo + wave;
        if (!first) {
            issue(kA, vA, Kh, Vh, row < row_hi ? row : -1);
            head_issue(s);
            issue(kB, vB, Kh, Vh, row + nw < row_hi ? row + nw : -1);
            head_commit();
        }
        first = false;
        __syncthreads();
        float acc[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = 0.f;
        float mrun = -INFINITY, lrun = 0.f;

        const bool last_seg = se == r1;
        // one row: scores, online softmax, weighted V.  kk/vv have landed when read.
        auto process = [&](u32x4 (&kk)[NP], u32x4 (&vv)[NP], int row_now) {
            const int t = row_now * PPW + tl;
            const bool valid = t < n_tok;
            if (t >= n_tok - 1) {                          // only in the last row of a head
#pragma unroll
                for (int k = 0; k < NP; ++k) {
                    const int pc = sub + LPP * k;
                    kk[k] = t == n_tok - 1 ? *reinterpret_cast<const u32x4 *>(kn + 8 * pc) : u32x4{0u, 0u, 0u, 0u};
                    vv[k] = t == n_tok - 1 ? *reinterpret_cast<const u32x4 *>(vn + 8 * pc) : u32x4{0u, 0u, 0u, 0u};
                }
            }
            // q is re-read from LDS for every row: the opaque offset keeps the reads
            // from being hoisted into 8*NP registers for the whole loop
            int qoff = 8 * sub;
            asm volatile("" : "+v"(qoff));
            float sp = 0.f;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                const float4 qa = *reinterpret_cast<const float4 *>(qs + qoff + 8 * LPP * k);
                const float4 qb = *reinterpret_cast<const float4 *>(qs + qoff + 8 * LPP * k + 4);
                sp = dot8(kk[k], qa, qb, sp);
            }
            sp += lane_xor<1>(sp);                         // the lanes sharing this position
            if constexpr (LPP == 4) sp += lane_xor<2>(sp);
            const float sc = valid ? sp * scale : -INFINITY;
            const float mn = fmaxf(mrun, sc);
            const float corr = mrun == -INFINITY ? 0.f : expf(mrun - mn);
            const float p = valid ? expf(sc - mn) : 0.f;
            lrun = lrun * corr + p;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                const float2 a = unpack_h2(vv[k].x), b = unpack_h2(vv[k].y);
                const float2 c = unpack_h2(vv[k].z), e = unpack_h2(vv[k].w);
                float *ac = acc + 8 * k;
                ac[0] = fmaf(p, a.x, ac[0] * corr); ac[1] = fmaf(p, a.y, ac[1] * corr);
                ac[2] = fmaf(p, b.x, ac[2] * corr); ac[3] = fmaf(p, b.y, ac[3] * corr);
                ac[4] = fmaf(p, c.x, ac[4] * corr); ac[5] = fmaf(p, c.y, ac[5] * corr);
                ac[6] = fmaf(p, e.x, ac[6] * corr); ac[7] = fmaf(p, e.y, ac[7] * corr);
            }
            mrun = mn;
        };
        // Two rows are in flight per wavefront; a register set is refilled as soon
        // as its row is consumed.  The sets swap roles instead of being copied: a
        // copy of a set whose loads are still in flight would have to wait for them.
        while (row < row_hi) {
            process(kA, vA, row);
            issue(kA, vA, Kh, Vh, row + 2 * nw < row_hi ? row + 2 * nw : -1);
            row += nw;
            if (row >= row_hi) break;
            process(kB, vB, row);
            issue(kB, vB, Kh, Vh, row + 2 * nw < row_hi ? row + 2 * nw : -1);
            row += nw;
        }

        // The first wavefront alone merges the wavefronts' states, publishes the
        // workgroup's partial and, if it was the last of the head, combines the head;
        // the others go on (to the caller's next weights) after one barrier.  Its own
        // next weights are requested only after its stores are acknowledged: that
        // wait covers every outstanding memory operation of the wavefront.
        if (last_seg && wave != 0) tail();

        // lanes -> wavefront
        const float mw = wave_max(mrun);
        const float fl = mrun == -INFINITY ? 0.f : expf(mrun - mw);
        const float lw = wave_sum(sub == 0 ? lrun * fl : 0.f);
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] *= fl;
        int off, cnt;
        reduce_scatter<NV, LPP>(acc, lane, off, cnt);
        constexpr int NLEFT = A::NLEFT;
#pragma unroll
        for (int i = 0; i < NLEFT; ++i) {
            if (i < cnt) {
                const int idx = off + i;                   // accumulator index: piece idx/8, element idx%8
                wp[wave * D + 8 * (sub + LPP * (idx >> 3)) + (idx & 7)] = acc[i];
            }
        }
        if (lane == 0) { wm[wave] = mw; wl[wave] = lw; }
        tr.mark(14);
        __syncthreads();

        if (wave == 0) {
            // wavefronts -> workgroup partial, slot = rank of this workgroup among
            // those covering head s.  A lane owns elements lane and lane + 64.
            constexpr int NE = (D + 63) / 64;
            const int g_lo = (int)((((long long)s * R + 1) * G - 1) / T);
            const int g_hi = (int)((((long long)(s + 1) * R) * G - 1) / T);
            const int ncover = g_hi - g_lo + 1;
            float *slot = P.part + ((size_t)s * P.part_slots + (size_t)(g - g_lo)) * (D + 2);
            {
                float M = -INFINITY;
                for (int wv = 0; wv < nw; ++wv) M = fmaxf(M, wm[wv]);
                float L = 0.f, O[NE];
#pragma unroll
                for (int e = 0; e < NE; ++e) O[e] = 0.f;
                for (int wv = 0; wv < nw; ++wv) {
                    const float ew = wm[wv] == -INFINITY ? 0.f : expf(wm[wv] - M);
                    L += wl[wv] * ew;
#pragma unroll
                    for (int e = 0; e < NE; ++e)
                        if (lane + 64 * e < D) O[e] += wp[wv * D + lane + 64 * e] * ew;
                }
#pragma unroll
                for (int e = 0; e < NE; ++e)
                    if (lane + 64 * e < D) xwg_store(slot + lane + 64 * e, O[e]);
                if (lane == 0) { xwg_store(slot + D, M); xwg_store(slot + D + 1, L); }
            }
            if (!(P.debug & 8)) {
                xwg_wait_stores();
                tr.mark(15);
                if (last_seg) tail();
                unsigned old = 0;
                if (lane == 0)
                    old = __hip_atomic_fetch_add(&P.seg_cnt[s], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const bool is_last = __builtin_amdgcn_readfirstlane(old) == (unsigned)(ncover - 1);
                if (is_last) {                             // this workgroup delivered the last partial
                    const float *base = P.part + (size_t)s * P.part_slots * (D + 2);
                    // loads of up to CB partials are in flight together (one round trip per batch)
                    constexpr int CB = 8;
                    float M = -INFINITY, L = 0.f, O[NE];
#pragma unroll
                    for (int e = 0; e < NE; ++e) O[e] = 0.f;
                    for (int j0 = 0; j0 < ncover; j0 += CB) {
                        float mj[CB], lj[CB], oj[CB][NE];
#pragma unroll
                        for (int j = 0; j < CB; ++j) {
                            const int jj = j0 + j < ncover ? j0 + j : ncover - 1;
                            const float *sj = base + (size_t)jj * (D + 2);
                            mj[j] = xwg_load(sj + D);
                            lj[j] = xwg_load(sj + D + 1);
#pragma unroll
                            for (int e = 0; e < NE; ++e) oj[j][e] = xwg_load(sj + (lane + 64 * e < D ? lane + 64 * e : 0));
                        }
#pragma unroll
                        for (int j = 0; j < CB; ++j) {
                            if (j0 + j < ncover) {         // running merge in slot order
                                const float mn = fmaxf(M, mj[j]);
                                const float c0 = M == -INFINITY ? 0.f : expf(M - mn);
                                const float c1 = mj[j] == -INFINITY ? 0.f : expf(mj[j] - mn);
                                L = L * c0 + lj[j] * c1;
#pragma unroll
                                for (int e = 0; e < NE; ++e) O[e] = O[e] * c0 + oj[j][e] * c1;
                                M = mn;
                            }
                        }
                    }
#pragma unroll
                    for (int e = 0; e < NE; ++e)
                        if (lane + 64 * e < D) xwg_store(P.o + s * D + lane + 64 * e, O[e] / L);
                    if (lane == 0)
                        __hip_atomic_store(&P.seg_cnt[s], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            } else if (last_seg) {
                tail();
            }
        }
        if (!last_seg) __syncthreads();                    // the scratch is reused by the next head
        tr.mark(16);
        sb = se;
    }
}

// Copy of an exchanged workspace vector (n a multiple of 8, at most
// 2 * UN * blockDim.x elements) into LDS in GEMV order, zero padded to a unit
// multiple: coherent 8-byte loads that are all in flight together, split into
// the request and the LDS write so that other loads can be queued in between.
template <int UN>
struct StagedVector {
    float2 v[UN];
    __device__ __forceinline__ void issue(const float *__restrict__ src, int n, int tid)
    {
        const int n2 = n >> 1, nt = blockDim.x;
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = tid + j * nt;
            v[j] = float2{0.f, 0.f};
            if (j * nt < n2) v[j] = xwg_load2(src + 2 * (i2 < n2 ? i2 : 0));
        }
    }
    __device__ __forceinline__ void commit(int n, float *dst, int tid) const
    {
        const int n2 = n >> 1, np2 = round_up_chunk(n) >> 1, nt = blockDim.x;
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = tid + j * nt;
            if (i2 < np2) *reinterpret_cast<float2 *>(dst + lds_perm(i2 * 2)) = i2 < n2 ? v[j] : float2{0.f, 0.f};
        }
    }
};

// Phase B.  LDS: m[Kp_f] part[rows_h*nw] bounds[16] scr[nw*(D+2)+4+2*D]
template <int D, class Sync>
__device__ __forceinline__ void phase_b(const StepParams &P, const __half *__restrict__ w,
                                        const __half *__restrict__ kv, int pos, float *lds, Sync &sync)
{
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, tid = opaque_thread_index(), nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(f);
    float *ml = lds, *part = lds + Kp;
    int *bnd = reinterpret_cast<int *>(part + P.rows_h * (nt >> 6));
    float *scr = reinterpret_cast<float *>(bnd + 16);
    const int r_begin = g * P.rows_h, r_n = max(0, min(P.rows_h, h - r_begin));
    GemvSpan<kGemvUDown> gs;
    gs.init(GemvSeg{w + P.lay.w_down + (size_t)r_begin * f, ml, f, r_n}, GemvSeg{w + P.lay.w_down, ml, f, 0}, w, tid, bnd, kShare0AfterAttention);
    // the first down-projection weights are requested behind the last K/V loads,
    // so that they stream while the attention partials are merged
    Tracer tr;
    tr.init(P, gs.wave, 16);
    tr.mark(10);
    clear_partials(part, P.rows_h * (nt >> 6), tid);
    const __half *bd = w + P.lay.b_down;
    const int item0 = spread_index(tid);
    const float bd0 = item0 < r_n ? __half2float(bd[r_begin + item0]) : 0.f;   // for the epilogue
    StagedVector<kStageM> sm;
    if constexpr (Sync::kInputsReady) sm.issue(P.m, f, tid);
    attn_share<D>(P, kv, pos + 1, scr, tid,
                  [&] {
                      sync.wait();
                      tr.mark(11);
                      if constexpr (!Sync::kInputsReady) sm.issue(P.m, f, tid);
                  },
                  [&] {
                      // The first down-projection weights are requested here, behind the
                      // K/V rows: they stream while the rows are processed and the partials
                      // merged.  (The first wavefront has no share of the GEMV: its loads
                      // re-read one cached block and cost nothing to wait for.)
                      gs.issue_first();
                      gs.issue_second();
                  },
                  [&] { sm.commit(f, ml, tid); tr.mark(12); },
                  [&] { tr.mark(13); }, tr);
    tr.mark(17);
    gs.run(part);            // (m became visible at the barrier inside attn_share)
    tr.mark(18);
    __syncthreads();
    for (int t = item0; t < r_n; t += nt)
        xwg_store(P.g + r_begin + t, gs.row_total(part, t) + (t == item0 ? bd0 : __half2float(bd[r_begin + t])));
    tr.mark(19);
    sync.arrive();
}

// Phase C.  LDS: o[Kp_h] part[rows_h*nw] bounds[16]
template <class Sync>
__device__ __forceinline__ void phase_c(const StepParams &P, const __half *__restrict__ w, int layer,
                                        float *lds, Sync &sync)
{
    const Dims &dm = P.dm;
    const int h = dm.h, tid = opaque_thread_index(), nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(h);
    float *ol = lds, *part = lds + Kp;
    int *bnd = reinterpret_cast<int *>(part + P.rows_h * (nt >> 6));
    const LayerIO io = layer_io(P, layer);
    const int r_begin = g * P.rows_h, r_n = max(0, min(P.rows_h, h - r_begin));
    GemvSpan<kGemvU> gs;
    gs.init(GemvSeg{w + P.lay.w_dense + (size_t)r_begin * h, ol, h, r_n}, GemvSeg{w + P.lay.w_dense, ol, h, 0}, w, tid, bnd);
    Tracer tr;
    tr.init(P, gs.wave, 48);
    tr.mark(20);
    clear_partials(part, P.rows_h * (nt >> 6), tid);
    StagedVector<kStageM> so;
    if constexpr (Sync::kInputsReady) so.issue(P.o, h, tid);
    gs.issue_first();
    gs.issue_second();
    sync.wait();
    tr.mark(21);
    if constexpr (!Sync::kInputsReady) so.issue(P.o, h, tid);
    // epilogue operands of this thread's first row
    const __half *bd = w + P.lay.b_dense;
    const int item0 = spread_index(tid);
    float bd0 = 0.f, x0 = 0.f, g0 = 0.f;
    if (item0 < r_n) {
        bd0 = __half2float(bd[r_begin + item0]);
        x0 = load_x(io, r_begin + item0);
        g0 = xwg_load(P.g + r_begin + item0);
    }
    so.commit(h, ol, tid);
    __syncthreads();
    tr.mark(22);
    gs.run(part);
    tr.mark(23);
    __syncthreads();
    for (int t = item0; t < r_n; t += nt) {
        const bool pre = t == item0;
        const float a = gs.row_total(part, t) + (pre ? bd0 : __half2float(bd[r_begin + t]));
        const float res = ((pre ? x0 : load_x(io, r_begin + t)) + a) + (pre ? g0 : xwg_load(P.g + r_begin + t));
        if (io.o16) io.o16[r_begin + t] = __float2half_rn(res);
        else xwg_store(io.o32 + r_begin + t, res);
    }
    tr.mark(24);
    sync.arrive();
}

// position of the new token; out of range raises the error flag (no work is done)
__device__ __forceinline__ bool read_pos(const StepParams &P, int *pos)
{
    const int p = *P.pos;
    *pos = p;
    if (p < 0 || p >= P.dm.max_seq) {
        if (threadIdx.x == 0 && blockIdx.x == 0)
            __hip_atomic_store(&P.sync[kSyncErr], (unsigned)kErrBadPos, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        return false;
    }
    return true;
}

// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kMaxThreads)
k_phase_a(StepParams P, const __half *w, __half *kv, int layer)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    NoSync sync;
    phase_a(P, w, kv, layer, pos, lds, sync);
}

template <int D>
__global__ void __launch_bounds__(kMaxThreads)
k_phase_b(StepParams P, const __half *w, const __half *kv)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    NoSync sync;
    phase_b<D>(P, w, kv, pos, lds, sync);
}

__global__ void __launch_bounds__(kMaxThreads)
k_phase_c(StepParams P, const __half *w, int layer)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    NoSync sync;
    phase_c(P, w, layer, lds, sync);
}

template <int D>
__global__ void __launch_bounds__(kMaxThreads)
k_block_persistent(StepParams P, const __half *w, __half *kv, int layer)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    GridBarrier bar;
    bar.init(P.sync, gridDim.x);
    GridSync sync{bar};
    phase_a(P, w, kv, layer, pos, lds, sync);
    phase_b<D>(P, w, kv, pos, lds, sync);
    phase_c(P, w, layer, lds, sync);
    bar.finish();
}

template <int D>
__global__ void __launch_bounds__(kMaxThreads)
k_stack_persistent(StepParams P, const LayerPtrs *__restrict__ ptrs)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    GridBarrier bar;
    bar.init(P.sync, gridDim.x);
    GridSync sync{bar};
#pragma clang loop unroll(disable)
    for (int layer = 0; layer < P.n_layers; ++layer) {
        const __half *w = ptrs->w[layer];
        __half *kv = ptrs->kv[layer];
        phase_a(P, w, kv, layer, pos, lds, sync);
        phase_b<D>(P, w, kv, pos, lds, sync);
        phase_c(P, w, layer, lds, sync);
    }
    bar.finish();
}

// ---------------------------------------------------------------------------
// host-side launchers

#define CFPP_TRY(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return e_; } while (0)

template <int D>
static hipError_t launch_phases_d(const StepParams &P, const __half *w, __half *kv, int layer,
                                  int grid, int threads, hipStream_t s)
{
    const size_t lds = (size_t)P.lds_floats * 4;
    hipLaunchKernelGGL(k_phase_a, dim3(grid), dim3(threads), lds, s, P, w, kv, layer);
    CFPP_TRY(hipGetLastError());
    hipLaunchKernelGGL(k_phase_b<D>, dim3(grid), dim3(threads), lds, s, P, w, (const __half *)kv);
    CFPP_TRY(hipGetLastError());
    hipLaunchKernelGGL(k_phase_c, dim3(grid), dim3(threads), lds, s, P, w, layer);
    return hipGetLastError();
}

hipError_t launch_phases(const StepParams &P, const __half *w, __half *kv, int layer,
                         int grid, int threads, hipStream_t s)
{
    switch (P.dm.d) {
    case 64: return launch_phases_d<64>(P, w, kv, layer, grid, threads, s);
    case 80: return launch_phases_d<80>(P, w, kv, layer, grid, threads, s);
    case 128: return launch_phases_d<128>(P, w, kv, layer, grid, threads, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_block_persistent(const StepParams &P, const __half *w, __half *kv, int layer,
                                   int grid, int threads, hipStream_t s)
{
    const size_t lds = (size_t)P.lds_floats * 4;
    switch (P.dm.d) {
    case 64: hipLaunchKernelGGL(k_block_persistent<64>, dim3(grid), dim3(threads), lds, s, P, w, kv, layer); break;
    case 80: hipLaunchKernelGGL(k_block_persistent<80>, dim3(grid), dim3(threads), lds, s, P, w, kv, layer); break;
    case 128: hipLaunchKernelGGL(k_block_persistent<128>, dim3(grid), dim3(threads), lds, s, P, w, kv, layer); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// one thread block copies the by-value table into device memory
__global__ void k_store_layer_ptrs(LayerPtrs src, LayerPtrs *dst, int n)
{
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        dst->w[i] = src.w[i];
        dst->kv[i] = src.kv[i];
    }
}

hipError_t launch_store_layer_ptrs(const LayerPtrs &ptrs, LayerPtrs *dst, int n, hipStream_t s)
{
    hipLaunchKernelGGL(k_store_layer_ptrs, dim3(1), dim3(64), 0, s, ptrs, dst, n);
    return hipGetLastError();
}

hipError_t launch_stack_persistent(const StepParams &P, const LayerPtrs *ptrs,
                                   int grid, int threads, hipStream_t s)
{
    const size_t lds = (size_t)P.lds_floats * 4;
    switch (P.dm.d) {
    case 64: hipLaunchKernelGGL(k_stack_persistent<64>, dim3(grid), dim3(threads), lds, s, P, ptrs); break;
    case 80: hipLaunchKernelGGL(k_stack_persistent<80>, dim3(grid), dim3(threads), lds, s, P, ptrs); break;
    case 128: hipLaunchKernelGGL(k_stack_persistent<128>, dim3(grid), dim3(threads), lds, s, P, ptrs); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t persistent_occupancy(int head_dim, int threads, size_t lds_bytes, int *blocks_per_cu)
{
    switch (head_dim) {
    case 64: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_persistent<64>, threads, lds_bytes);
    case 80: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_persistent<80>, threads, lds_bytes);
    case 128: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_persistent<128>, threads, lds_bytes);
    }
    return hipErrorInvalidValue;
}

// allow more than the default 64 KiB of dynamic LDS
hipError_t prepare_kernels(size_t lds_bytes)
{
    const int v = (int)lds_bytes;
    CFPP_TRY(hipFuncSetAttribute((const void *)k_phase_a, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_phase_c, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_phase_b<64>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_phase_b<80>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_phase_b<128>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_block_persistent<64>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_block_persistent<80>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_block_persistent<128>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_stack_persistent<64>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_stack_persistent<80>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_stack_persistent<128>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    return hipSuccess;
}

}  // namespace cfpp
