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

// ---------------------------------------------------------------------------
// Row-split GEMV over this workgroup's rows.  Work unit = (row, K-slice), slice
// fastest, handed to wavefronts round-robin; a wavefront streams its slice with
// 16-byte loads per lane (1 KiB contiguous per instruction), multiplies with the
// activation vector held in LDS (fp32, lds_perm order, zero padded to a chunk
// multiple) and leaves the slice's partial sum in part[unit].
template <int U>
__device__ __forceinline__ void gemv_issue(u32x4 (&wv)[U], const __half *p)
{
#pragma unroll
    for (int i = 0; i < U; ++i) wv[i] = load16_stream(p + (size_t)i * kChunk);
}

template <int U>
__device__ __forceinline__ float gemv_consume(const u32x4 (&wv)[U], const float *yl, float acc)
{
    float a0 = acc, a1 = 0.f;
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const float4 ya = *reinterpret_cast<const float4 *>(yl + i * kChunk);
        const float4 yb = *reinterpret_cast<const float4 *>(yl + i * kChunk + 256);
        if (i & 1) a1 = dot8(wv[i], ya, yb, a1);
        else a0 = dot8(wv[i], ya, yb, a0);
    }
    return a0 + a1;
}

// Fast path: K a multiple of 512 and every slice a whole number of U-chunk
// steps.  The wavefront walks its (unit, step) sequence with the loads of the
// next step already in flight while it multiplies the current one, so the
// reduction at the end of a unit never drains the memory pipeline.
template <int U>
__device__ __forceinline__ void wg_gemv_pipelined(const __half *__restrict__ Wm, int K, int row_begin,
                                                  int nrows, int nsl, int cps, const float *y, float *part)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int spu = cps / U;                         // steps per unit
    const int nunits = nrows * nsl;
    const __half *wl = Wm + (size_t)row_begin * K + lane * 8;
    const float *yl = y + lane * 4;
    int u = wave, step = 0;
    if (u >= nunits) return;
    u32x4 cur[U], nxt[U];
    {
        const int rl = u / nsl, sl = u - rl * nsl;
        gemv_issue<U>(cur, wl + (size_t)rl * K + (size_t)(sl * cps) * kChunk);
    }
    float acc = 0.f;
    while (u < nunits) {
        int un = u, stn = step + 1;
        if (stn == spu) { stn = 0; un = u + nw; }
        if (un < nunits) {
            const int rl = un / nsl, sl = un - rl * nsl;
            gemv_issue<U>(nxt, wl + (size_t)rl * K + (size_t)(sl * cps + stn * U) * kChunk);
        }
        {
            const int sl = u % nsl;
            acc = gemv_consume<U>(cur, yl + (sl * cps + step * U) * kChunk, acc);
        }
        if (stn == 0) {
            const float tot = wave_sum(acc);
            if (lane == 0) part[u] = tot;
            acc = 0.f;
        }
#pragma unroll
        for (int i = 0; i < U; ++i) cur[i] = nxt[i];
        u = un;
        step = stn;
    }
}

// General path: any K that is a multiple of 8 (ragged last chunk), any slicing.
__device__ __forceinline__ void wg_gemv_general(const __half *__restrict__ Wm, int K, int row_begin,
                                                int nrows, int nsl, const float *y, float *part)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int nchunk = (K + kChunk - 1) / kChunk;
    const int cps = (nchunk + nsl - 1) / nsl;
    const int nunits = nrows * nsl;
    for (int u = wave; u < nunits; u += nw) {
        const int rl = u / nsl, sl = u - rl * nsl;
        const int c0 = sl * cps;
        const int c1 = min(nchunk, c0 + cps);
        const __half *wrow = Wm + (size_t)(row_begin + rl) * K + lane * 8;
        const float *yl = y + lane * 4;
        float acc = 0.f;
        for (int c = c0; c < c1; ++c) {
            u32x4 wv = {0u, 0u, 0u, 0u};
            if (c * kChunk + lane * 8 < K) wv = load16_stream(wrow + (size_t)c * kChunk);
            const float4 ya = *reinterpret_cast<const float4 *>(yl + c * kChunk);
            const float4 yb = *reinterpret_cast<const float4 *>(yl + c * kChunk + 256);
            acc = dot8(wv, ya, yb, acc);
        }
        const float tot = wave_sum(acc);
        if (lane == 0) part[u] = tot;
    }
}

__device__ __forceinline__ void wg_gemv(const __half *__restrict__ Wm, int K, int row_begin,
                                        int nrows, int nsl, const float *y, float *part)
{
    if (nrows <= 0) return;
    const int nchunk = (K + kChunk - 1) / kChunk;
    const int cps = (nchunk + nsl - 1) / nsl;
    const bool regular = (K % kChunk) == 0 && cps * nsl == nchunk;
    if (regular && cps % 8 == 0) wg_gemv_pipelined<8>(Wm, K, row_begin, nrows, nsl, cps, y, part);
    else if (regular && cps % 5 == 0) wg_gemv_pipelined<5>(Wm, K, row_begin, nrows, nsl, cps, y, part);
    else if (regular && cps % 4 == 0) wg_gemv_pipelined<4>(Wm, K, row_begin, nrows, nsl, cps, y, part);
    else wg_gemv_general(Wm, K, row_begin, nrows, nsl, y, part);
}

// sum of a value over the workgroup, fixed order; red: >= 16 floats of LDS
__device__ __forceinline__ float block_sum(float v, float *red)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
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
// Phase A.  LDS: y1[Kp] y2[Kp] part[rows_qkv + rows_up] red[16]
__device__ void phase_a(const StepParams &P, const __half *__restrict__ w, __half *__restrict__ kv,
                        int layer, int pos, float *lds)
{
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, d = dm.d, r = dm.r;
    const int tid = threadIdx.x, nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(h);
    float *y1 = lds, *y2 = lds + Kp, *part = lds + 2 * Kp;
    float *red = part + P.rows_qkv + P.rows_up;
    const LayerIO io = layer_io(P, layer);

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
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < GU; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) s += xv[j][e];
    const float mean = block_sum(s, red) / (float)h;
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
    const float var = block_sum(v, red) / (float)h;
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

    const int q_begin = g * P.rows_qkv, q_n = max(0, min(P.rows_qkv, 3 * h - q_begin));
    const int u_begin = g * P.rows_up, u_n = max(0, min(P.rows_up, f - u_begin));
    wg_gemv(w + P.lay.w_qkv, h, q_begin, q_n, 1, y1, part);
    wg_gemv(w + P.lay.w_up, h, u_begin, u_n, 1, y2, part + P.rows_qkv);
    __syncthreads();

    // QKV epilogue: one thread per pair of adjacent packed rows
    const __half *bq = w + P.lay.b_qkv;
    for (int pr = tid; pr < q_n / 2; pr += nt) {
        const int p = q_begin + 2 * pr;                 // packed row, even
        const int n = p / (3 * d), rem = p - n * 3 * d;
        const int c = rem / d, i = rem - c * d;          // i even
        float v0 = part[2 * pr] + __half2float(bq[p]);
        float v1 = part[2 * pr + 1] + __half2float(bq[p + 1]);
        int d0 = i, d1 = i + 1;
        if (c < 2 && i < r) {                            // rotary pair (j, j + r/2)
            const int j = i >> 1;
            const float2 cs = P.rope[(size_t)pos * (r >> 1) + j];
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
    const __half *bu = w + P.lay.b_up;
    for (int t = tid; t < u_n; t += nt)
        xwg_store(P.m + u_begin + t, gelu_erf(part[P.rows_qkv + t] + __half2float(bu[u_begin + t])));
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
// scr: nw*(D+2) + 4 floats of LDS.
template <int D>
__device__ void attn_share(const StepParams &P, const __half *__restrict__ kv, int n_tok, float *scr)
{
    using A = AttnShape<D>;
    constexpr int LPP = A::LPP, PPW = A::PPW, NP = A::NP, NV = A::NV;
    const Dims &dm = P.dm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int sub = lane & (LPP - 1), tl = lane / LPP;
    const int H = dm.H;
    const long long g = blockIdx.x;
    const int R = (n_tok + PPW - 1) / PPW;
    const long long T = (long long)R * H;
    // with fewer rows than workgroups only the first T workgroups take part, so
    // that every participant owns at least one row (no empty ranges in between)
    const long long G = min((long long)gridDim.x, T);
    const long long r0 = g < G ? T * g / G : 0, r1 = g < G ? T * (g + 1) / G : 0;
    const float scale = 1.0f / sqrtf((float)D);
    const size_t hs = kv_head_stride(dm);
    const __half *Kb = kv + kv_offset(dm, 0, P.b, 0, 0, 0);
    const __half *Vb = kv + kv_offset(dm, 1, P.b, 0, 0, 0);
    float *wp = scr, *wm = scr + nw * D, *wl = wm + nw;
    int *flag = reinterpret_cast<int *>(wl + nw);

    // element offset of this lane's piece k inside a head, for position 0
    size_t koff[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int pc = sub + LPP * k;
        koff[k] = (size_t)(pc >> 1) * dm.max_seq * 16 + (pc & 1) * 8;
    }

    for (long long sb = r0; sb < r1;) {
        const int s = (int)(sb / R);                       // head
        const long long se = min(r1, (long long)(s + 1) * R);
        const int row_lo = (int)(sb - (long long)s * R), row_hi = (int)(se - (long long)s * R);
        const __half *Kh = Kb + (size_t)s * hs;
        const __half *Vh = Vb + (size_t)s * hs;

        float q[NP][8];
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const float *qp = P.q + s * D + 8 * (sub + LPP * k);
            const float2 a = xwg_load2(qp), b = xwg_load2(qp + 2), c = xwg_load2(qp + 4), e = xwg_load2(qp + 6);
            q[k][0] = a.x; q[k][1] = a.y; q[k][2] = b.x; q[k][3] = b.y;
            q[k][4] = c.x; q[k][5] = c.y; q[k][6] = e.x; q[k][7] = e.y;
        }
        float acc[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = 0.f;
        float mrun = -INFINITY, lrun = 0.f;

        auto issue = [&](u32x4 (&kk)[NP], u32x4 (&vv)[NP], int row) {
            const int t = row * PPW + tl;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                kk[k] = u32x4{0u, 0u, 0u, 0u};
                vv[k] = u32x4{0u, 0u, 0u, 0u};
            }
            if (t < n_tok - 1) {
#pragma unroll
                for (int k = 0; k < NP; ++k) kk[k] = load16_stream(Kh + koff[k] + (size_t)t * 16);
#pragma unroll
                for (int k = 0; k < NP; ++k) vv[k] = load16_stream(Vh + koff[k] + (size_t)t * 16);
            } else if (t == n_tok - 1) {               // appended during this launch by other workgroups
#pragma unroll
                for (int k = 0; k < NP; ++k) kk[k] = xwg_load16(Kh + koff[k] + (size_t)t * 16);
#pragma unroll
                for (int k = 0; k < NP; ++k) vv[k] = xwg_load16(Vh + koff[k] + (size_t)t * 16);
            }
        };

        u32x4 kA[NP], vA[NP], kB[NP], vB[NP];
        int row = row_lo + wave;
        if (row < row_hi) issue(kA, vA, row);
        for (; row < row_hi; row += nw) {
            if (row + nw < row_hi) issue(kB, vB, row + nw);
            const bool valid = row * PPW + tl < n_tok;
            float sp = 0.f;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                const float4 qa = {q[k][0], q[k][1], q[k][2], q[k][3]};
                const float4 qb = {q[k][4], q[k][5], q[k][6], q[k][7]};
                sp = dot8(kA[k], qa, qb, sp);
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
                const float2 a = unpack_h2(vA[k].x), b = unpack_h2(vA[k].y);
                const float2 c = unpack_h2(vA[k].z), e = unpack_h2(vA[k].w);
                float *ac = acc + 8 * k;
                ac[0] = fmaf(p, a.x, ac[0] * corr); ac[1] = fmaf(p, a.y, ac[1] * corr);
                ac[2] = fmaf(p, b.x, ac[2] * corr); ac[3] = fmaf(p, b.y, ac[3] * corr);
                ac[4] = fmaf(p, c.x, ac[4] * corr); ac[5] = fmaf(p, c.y, ac[5] * corr);
                ac[6] = fmaf(p, e.x, ac[6] * corr); ac[7] = fmaf(p, e.y, ac[7] * corr);
            }
            mrun = mn;
#pragma unroll
            for (int k = 0; k < NP; ++k) { kA[k] = kB[k]; vA[k] = vB[k]; }
        }

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
        __syncthreads();

        // wavefronts -> workgroup partial, slot = rank of this workgroup among
        // those covering head s
        const long long g_lo = (((long long)s * R + 1) * G - 1) / T;
        const long long g_hi = (((long long)(s + 1) * R) * G - 1) / T;
        const int ncover = (int)(g_hi - g_lo + 1);
        float *slot = P.part + ((size_t)s * P.part_slots + (size_t)(g - g_lo)) * (D + 2);
        if (tid < D) {
            float M = -INFINITY;
            for (int wv = 0; wv < nw; ++wv) M = fmaxf(M, wm[wv]);
            float L = 0.f, O = 0.f;
            for (int wv = 0; wv < nw; ++wv) {
                const float e = wm[wv] == -INFINITY ? 0.f : expf(wm[wv] - M);
                L += wl[wv] * e;
                O += wp[wv * D + tid] * e;
            }
            xwg_store(slot + tid, O);
            if (tid == 0) { xwg_store(slot + D, M); xwg_store(slot + D + 1, L); }
        }
        if (P.debug & 8) { __syncthreads(); sb = se; continue; }
        xwg_wait_stores();
        __syncthreads();
        if (tid == 0) {
            const unsigned old = __hip_atomic_fetch_add(&P.seg_cnt[s], 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
            *flag = old == (unsigned)(ncover - 1);
        }
        __syncthreads();
        if (*flag) {                                       // this workgroup delivered the last partial
            if (tid < D) {
                const float *base = P.part + (size_t)s * P.part_slots * (D + 2);
                float M = -INFINITY;
                for (int j = 0; j < ncover; ++j) M = fmaxf(M, xwg_load(base + (size_t)j * (D + 2) + D));
                float L = 0.f, O = 0.f;
                for (int j = 0; j < ncover; ++j) {
                    const float *sj = base + (size_t)j * (D + 2);
                    const float e = expf(xwg_load(sj + D) - M);
                    L += xwg_load(sj + D + 1) * e;
                    O += xwg_load(sj + tid) * e;
                }
                xwg_store(P.o + s * D + tid, O / L);
            }
            if (tid == 0)
                __hip_atomic_store(&P.seg_cnt[s], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        sb = se;
    }
}

// copy an exchanged workspace vector (n a multiple of 8) into LDS in GEMV order,
// zero padded to a chunk multiple; coherent 8-byte loads, a batch in flight
// together
__device__ __forceinline__ void stage_vector(const float *__restrict__ src, int n, float *dst)
{
    constexpr int UN = 10;
    const int n2 = n >> 1, np2 = round_up_chunk(n) >> 1;
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int base = 0; base < np2; base += UN * nt) {
        float2 v[UN];
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = base + tid + j * nt;
            v[j] = i2 < n2 ? xwg_load2(src + 2 * i2) : float2{0.f, 0.f};
        }
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = base + tid + j * nt;
            if (i2 < np2) *reinterpret_cast<float2 *>(dst + lds_perm(i2 * 2)) = v[j];
        }
    }
}

// Phase B.  LDS: m[Kp_f] part[rows_h*nsl_down] scr[nw*(D+2)+4]
template <int D>
__device__ void phase_b(const StepParams &P, const __half *__restrict__ w, const __half *__restrict__ kv,
                        int pos, float *lds)
{
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, tid = threadIdx.x, nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(f);
    float *ml = lds, *part = lds + Kp, *scr = part + P.rows_h * P.nsl_down;
    if (!(P.debug & 1)) stage_vector(P.m, f, ml);
    if (!(P.debug & 2)) attn_share<D>(P, kv, pos + 1, scr);
    __syncthreads();
    const int r_begin = g * P.rows_h, r_n = max(0, min(P.rows_h, h - r_begin));
    if (!(P.debug & 4)) wg_gemv(w + P.lay.w_down, f, r_begin, r_n, P.nsl_down, ml, part);
    __syncthreads();
    const __half *bd = w + P.lay.b_down;
    for (int t = tid; t < r_n; t += nt) {
        float a = 0.f;
        for (int sl = 0; sl < P.nsl_down; ++sl) a += part[t * P.nsl_down + sl];
        xwg_store(P.g + r_begin + t, a + __half2float(bd[r_begin + t]));
    }
}

// Phase C.  LDS: o[Kp_h] part[rows_h*nsl_dense]
__device__ void phase_c(const StepParams &P, const __half *__restrict__ w, int layer, float *lds)
{
    const Dims &dm = P.dm;
    const int h = dm.h, tid = threadIdx.x, nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(h);
    float *ol = lds, *part = lds + Kp;
    const LayerIO io = layer_io(P, layer);
    stage_vector(P.o, h, ol);
    __syncthreads();
    const int r_begin = g * P.rows_h, r_n = max(0, min(P.rows_h, h - r_begin));
    wg_gemv(w + P.lay.w_dense, h, r_begin, r_n, P.nsl_dense, ol, part);
    __syncthreads();
    const __half *bd = w + P.lay.b_dense;
    for (int t = tid; t < r_n; t += nt) {
        float a = 0.f;
        for (int sl = 0; sl < P.nsl_dense; ++sl) a += part[t * P.nsl_dense + sl];
        a += __half2float(bd[r_begin + t]);
        const float res = (load_x(io, r_begin + t) + a) + xwg_load(P.g + r_begin + t);
        if (io.o16) io.o16[r_begin + t] = __float2half_rn(res);
        else xwg_store(io.o32 + r_begin + t, res);
    }
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
    phase_a(P, w, kv, layer, pos, lds);
}

template <int D>
__global__ void __launch_bounds__(kMaxThreads)
k_phase_b(StepParams P, const __half *w, const __half *kv)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    phase_b<D>(P, w, kv, pos, lds);
}

__global__ void __launch_bounds__(kMaxThreads)
k_phase_c(StepParams P, const __half *w, int layer)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    phase_c(P, w, layer, lds);
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
    phase_a(P, w, kv, layer, pos, lds);
    bar.wait();
    phase_b<D>(P, w, kv, pos, lds);
    bar.wait();
    phase_c(P, w, layer, lds);
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
#pragma clang loop unroll(disable)
    for (int layer = 0; layer < P.n_layers; ++layer) {
        const __half *w = ptrs->w[layer];
        __half *kv = ptrs->kv[layer];
        if (layer) bar.wait();
        phase_a(P, w, kv, layer, pos, lds);
        bar.wait();
        phase_b<D>(P, w, kv, pos, lds);
        bar.wait();
        phase_c(P, w, layer, lds);
    }
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
