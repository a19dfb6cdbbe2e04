// Building blocks shared by the decode kernels: the balanced row-split GEMV,
// staged copies of exchanged vectors, workgroup sums, layer input/output views.
#pragma once
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
constexpr int kGemvU = 4;             // units per load block
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

// XB: extra register sets that only ever hold blocks 3 .. 2 + XB of the span - for a
// GEMV whose first blocks are requested long before its activations exist (ahead of a
// hand-over with nothing else to stream): the stretch then starts with 2 + XB blocks in
// registers and the queue is full again by the time they are consumed.
// STRIDED: the block is a column range of a wider row-major matrix (one segment only):
// a row's units are contiguous, consecutive rows lie `row_stride` elements apart.  Units
// are then addressed through a cursor that the load blocks advance in order.
template <int U_, int XB = 0, bool STRIDED = false>
struct GemvSpan {
    static constexpr int U = U_;
    u32x4 a[U], b[U];
    u32x4 ex[XB > 0 ? XB : 1][U];
    const __half *w0, *w1;          // block bases (uniform)
    const __half *p0, *p1;          // the same, or `safe` when this wavefront streams nothing
    unsigned lane_off;              // this lane's byte offset inside a unit
    const float *y0, *y1;           // lane-adjusted activation bases
    int nch0, nch1, rows0, rows1, K0, K1;
    int n0, N, lo, hi, last, nw, wave, lane;
    const __half *safe;             // any readable 1 KiB: target of loads that are issued but not used
    bool regular;
    // STRIDED: the next unit to request, its index inside its row, its offset from p0 in units, and the
    // units to skip at the end of a row
    int is_u, is_c, is_skip;
    unsigned is_off;
    // walking state of consume()
    const float *yc;
    int c, nchc, rowg;
    float acc0, acc1;

    // share0: the first wavefront's share of the units in quarters of a full
    // share (4 = equal split); callers lower it when that wavefront has other
    // work to finish first.
    __device__ __forceinline__ void init(const GemvSeg &s0, const GemvSeg &s1, const __half *safe_, int tid,
                                         int share0 = 4, int row_stride = 0)
    {
        safe = safe_;
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
        {
            const int wtot = share0 + 4 * (nw - 1);
            const int c0 = wave == 0 ? 0 : share0 + 4 * (wave - 1), c1 = share0 + 4 * wave;
            lo = regular ? (int)((unsigned)N * (unsigned)c0 / (unsigned)wtot) : 0;
            hi = regular ? (int)((unsigned)N * (unsigned)c1 / (unsigned)wtot) : 0;
        }
        last = hi > lo ? hi - 1 : (regular && N > 0 ? (lo < N ? lo : N - 1) : -1);
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
        if constexpr (STRIDED) {
            // (single segment, whole units: the caller guarantees rows1 == 0 and K0 % kChunk == 0)
            is_u = hi > lo ? lo : last;                     // (nothing to stream: the cursor stays on one readable unit)
            is_c = hi > lo ? c : 0;
            is_skip = row_stride / kChunk - nch0;
            is_off = hi > lo ? (unsigned)(row * (row_stride / kChunk) + c) : 0u;
        }
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
    __device__ __forceinline__ void issue(u32x4 (&r)[U], int i)
    {
        if constexpr (STRIDED) {
            // (i only documents the order: every call continues where the previous one ended)
#pragma unroll
            for (int j = 0; j < U; ++j) {
                r[j] = load16_stream_at(p0 + (size_t)is_off * kChunk, lane_off);
                advance_cursor();
            }
        } else {
#pragma unroll
            for (int j = 0; j < U; ++j) r[j] = load16_stream_at(unit_ptr(i + j), lane_off);
        }
        // keep the instruction scheduler from sinking these loads towards their use
        __builtin_amdgcn_sched_barrier(0);
    }
    // STRIDED: the cursor moves to the next unit of this wavefront's range; at its last unit it
    // stays.  Plain arithmetic on purpose: a branch here would make the loads conditional.
    __device__ __forceinline__ void advance_cursor()
    {
        const int adv = (int)(is_u < last);
        const int c1 = is_c + adv;
        const int wrap = (int)(c1 == nch0);               // (only ever with adv = 1: is_c < nch0)
        is_u += adv;
        is_c = c1 - wrap * nch0;
        is_off += (unsigned)(adv + wrap * is_skip);
    }
    __device__ __forceinline__ void issue_first() { issue(a, lo); }
    __device__ __forceinline__ void issue_second() { issue(b, lo + U); }
    // (XB > 0) blocks 3 .. 2 + XB
    __device__ __forceinline__ void issue_more()
    {
        static_assert(XB > 0, "issue_more() needs the extra register sets");
#pragma unroll
        for (int x = 0; x < XB; ++x)
#pragma unroll
            for (int j = 0; j < U; ++j) {
                if constexpr (STRIDED) {
                    ex[x][j] = load16_stream_at(p0 + (size_t)is_off * kChunk, lane_off);
                    advance_cursor();
                } else {
                    ex[x][j] = load16_stream_at(unit_ptr(lo + (2 + x) * U + j), lane_off);
                }
            }
        __builtin_amdgcn_sched_barrier(0);
    }

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
                if (c == nchc || u == hi - 1) {              // end of a row, or of this wavefront's range
                    const float tot = wave_sum(acc0 + acc1);
                    if (lane == 0) part[rowg * nw + wave] = tot;
                    acc0 = 0.f; acc1 = 0.f;
                    c = 0;
                    ++rowg;
                    if (rowg == rows0) { nchc = nch1; yc = y1; }
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

    // consume everything; issue_first() and issue_second() have been called.
    // before_drain(): called once when the last load of this GEMV has been
    // issued - the place to request whatever should stream next.
    __device__ __forceinline__ void run(float *part)
    {
        run(part, [] {});
    }
    template <class Hook>
    __device__ __forceinline__ void run(float *part, Hook &&before_drain)
    {
        run(part, [] {}, before_drain);
    }
    // after_start(): called once, a few blocks into the stretch (XB > 0: behind the first two
    // refills; else at once) - straight-line code, the place for loads that should join the stream late
    template <class Start, class Hook>
    __device__ __forceinline__ void run(float *part, Start &&after_start, Hook &&before_drain)
    {
        if (!regular) { after_start(); before_drain(); run_general(part); return; }
        int i = lo;
        if constexpr (XB == 0) after_start();
        if constexpr (XB > 0) {
            // 2 + XB blocks are in registers: the first two are replaced as they are consumed,
            // the others just drain
            consume(a, i, part); issue(a, i + (2 + XB) * U);
            consume(b, i + U, part); issue(b, i + (3 + XB) * U);
            after_start();
#pragma unroll
            for (int x = 0; x < XB; ++x) consume(ex[x], i + (2 + x) * U, part);
            i += (2 + XB) * U;
        }
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
        before_drain();
        if (a_older) { consume(a, i, part); consume(b, i + U, part); }
        else { consume(b, i, part); consume(a, i + U, part); }
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

// Both LayerNorms of a block (they read the same input): load() requests the
// input and the four parameter vectors, finish() computes the statistics and
// writes the two normalised vectors to LDS in GEMV order (zero padded); the
// caller places a workgroup barrier after finish().  A thread owns up to GU
// groups of 8 consecutive elements; everything is fetched with 16-byte loads
// that are all in flight together, statistics are two-pass on registers.
struct LnPair {
    static constexpr int GU = 4;
    float xv[GU][8];
    u32x4 pg1[GU], pb1[GU], pg2[GU], pb2[GU];

    __device__ __forceinline__ void load(const StepParams &P, const __half *__restrict__ w, const LayerIO &io, int tid)
    {
        const int h = P.dm.h, nt = blockDim.x;
        const int ngrp = h >> 3;
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
    }

    // The two halves of load() on their own: the parameters depend on nothing and
    // can be requested ahead of a wait; the input may already sit in LDS (fp32,
    // natural order).
    __device__ __forceinline__ void load_params(const StepParams &P, const __half *__restrict__ w, int tid)
    {
        const int h = P.dm.h, nt = blockDim.x;
        const int ngrp = h >> 3;
        const __half *g1 = w + P.lay.ln1_g, *b1 = w + P.lay.ln1_b;
        const __half *g2 = w + P.lay.ln2_g, *b2 = w + P.lay.ln2_b;
#pragma unroll
        for (int j = 0; j < GU; ++j) {
            const int gi = tid + j * nt;
            const u32x4 z = {0u, 0u, 0u, 0u};
            pg1[j] = z; pb1[j] = z; pg2[j] = z; pb2[j] = z;
            if (gi < ngrp) {
                pg1[j] = load16(g1 + gi * 8); pb1[j] = load16(b1 + gi * 8);
                pg2[j] = load16(g2 + gi * 8); pb2[j] = load16(b2 + gi * 8);
            }
        }
    }
    __device__ __forceinline__ void load_x_global(const StepParams &P, const LayerIO &io, int tid)
    {
        const int h = P.dm.h, nt = blockDim.x;
        const int ngrp = h >> 3;
#pragma unroll
        for (int j = 0; j < GU; ++j) {
            const int gi = tid + j * nt;
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
            }
        }
    }
    __device__ __forceinline__ void load_x_lds(const StepParams &P, const float *xs, int tid)
    {
        const int h = P.dm.h, nt = blockDim.x;
        const int ngrp = h >> 3;
#pragma unroll
        for (int j = 0; j < GU; ++j) {
            const int gi = tid + j * nt;
            const float4 a = gi < ngrp ? *reinterpret_cast<const float4 *>(xs + gi * 8) : float4{0.f, 0.f, 0.f, 0.f};
            const float4 b = gi < ngrp ? *reinterpret_cast<const float4 *>(xs + gi * 8 + 4) : float4{0.f, 0.f, 0.f, 0.f};
            xv[j][0] = a.x; xv[j][1] = a.y; xv[j][2] = a.z; xv[j][3] = a.w;
            xv[j][4] = b.x; xv[j][5] = b.y; xv[j][6] = b.z; xv[j][7] = b.w;
        }
    }

    __device__ __forceinline__ void finish(const StepParams &P, float *y1, float *y2, float *red, int tid)
    {
        const int h = P.dm.h;
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < GU; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) s += xv[j][e];
        const float mean = block_sum(s, red, tid) / (float)h;
        finish_with_mean(P, y1, y2, red, mean, tid);
    }

    // the same with the mean already known (second pass and the affine part)
    __device__ __forceinline__ void finish_with_mean(const StepParams &P, float *y1, float *y2, float *red, float mean,
                                                     int tid)
    {
        const Dims &dm = P.dm;
        const int h = dm.h, nt = blockDim.x;
        const int ngrp = h >> 3;
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
        apply(P, y1, y2, mean, inv, tid);
    }

    // the two normalised vectors into LDS (GEMV order, zero padded to whole units),
    // given the statistics of the loaded input
    __device__ __forceinline__ void apply(const StepParams &P, float *y1, float *y2, float mean, float inv, int tid)
    {
        const int h = P.dm.h, nt = blockDim.x;
        const int Kp = round_up_chunk(h);
        const int ngrp = h >> 3, ngrp_p = Kp >> 3;
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
    }
};

// Copy of an exchanged workspace vector (n a multiple of 8, at most
// 2 * UN * blockDim.x elements) into LDS in GEMV order, zero padded to a unit
// multiple: coherent 8-byte loads that are all in flight together, split into
// the request and the LDS write so that other loads can be queued in between.
template <int UN>
struct StagedVector {
    float2 v[UN];
    // tid in [0, nt): the threads that share the copy (default: the workgroup)
    __device__ __forceinline__ void issue(const float *__restrict__ src, int n, int tid, int nt = blockDim.x)
    {
        const int n2 = n >> 1;
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = tid + j * nt;
            v[j] = float2{0.f, 0.f};
            if (j * nt < n2) v[j] = xwg_load2(src + 2 * (i2 < n2 ? i2 : 0));
        }
    }
    __device__ __forceinline__ void commit(int n, float *dst, int tid, int nt = blockDim.x) const
    {
        const int n2 = n >> 1, np2 = round_up_chunk(n) >> 1;
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = tid + j * nt;
            if (i2 < np2) *reinterpret_cast<float2 *>(dst + lds_perm(i2 * 2)) = i2 < n2 ? v[j] : float2{0.f, 0.f};
        }
    }
};

}  // namespace cfpp
