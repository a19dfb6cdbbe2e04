// Several sequences per step (launch mode 0, batch > 1): the four projections
// of the block (paper Sec. 2.2) with the weights streamed ONCE for up to 8
// sequences.  Here the path is a dense contraction - rows x K weights times K x
// batch activations - so it runs on the matrix cores: v_mfma_f32_16x16x16_f16
// with a 16-row tile of the weight matrix as the A operand, straight from its
// row-major layout (one 16-byte load per lane: 16 rows x 32 columns per
// wavefront instruction), and the activations of the batch as the B operand
// from LDS.  Activations are fp32 values: each is split into an fp16 head and an
// fp16 remainder (y = hi + lo exactly to ~2^-22), two MFMAs per tile, fp32
// accumulation - the result matches the fp32 FMA path to rounding.
//
//   k_bat_qkv_up<TQ, TU>: both LayerNorms of every sequence (input and statistics
//                         once), QKV rows + bias, rotary, K/V append, q, then the
//                         MLP-up rows + bias + GELU
//   k_bat_out<T>        : output projection of the attention output, then the
//                         MLP-down rows (K in slices of `hidden` through the same
//                         LDS), + biases + residual -> the block output
//
// Attention stays per sequence (every sequence has its own cache) and runs the
// attention part of the per-sequence phase kernel in between.
//
// A workgroup owns `rows` consecutive rows (T = ceil(rows/16) tiles, T <= 4);
// its 8 wavefronts split K; their accumulators are added in wavefront order
// through LDS: one bit pattern per build.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "decode_blocks.h"
#include "batched_params.h"

namespace cfpp {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int kBatPad = 16;          // halves between the activation rows in LDS (spreads the banks)

__device__ __forceinline__ f16x4 lo_halves(u32x4 v)
{
    union { unsigned u[2]; f16x4 h; } c;
    c.u[0] = v.x; c.u[1] = v.y;
    return c.h;
}
__device__ __forceinline__ f16x4 hi_halves(u32x4 v)
{
    union { unsigned u[2]; f16x4 h; } c;
    c.u[0] = v.z; c.u[1] = v.w;
    return c.h;
}

// input of this layer for sequence b, element i
__device__ __forceinline__ float bat_x(const BatParams &P, int b, int i)
{
    if (P.layer == 0) return __half2float(P.x_in[(size_t)b * P.dm.h + i]);
    return P.xres[((size_t)b * 2 + ((P.layer - 1) & 1)) * P.dm.h + i];
}

// all positions of the group inside the cache?  (uniform over the grid)
__device__ __forceinline__ bool bat_positions_ok(const BatParams &P)
{
    bool ok = true;
    for (int b = 0; b < P.nb; ++b) {
        const int p = P.pos[b];
        ok = ok && p >= 0 && p < P.dm.max_seq;
    }
    if (!ok && threadIdx.x == 0 && blockIdx.x == 0)
        __hip_atomic_store(&P.sync[kSyncErr], (unsigned)kErrBadPos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return ok;
}

// One 16-row tile: its `steps` blocks of 32 columns (per wavefront) against the
// activations in LDS, into one accumulator.  A and B already hold the tile's
// first two sets of kBatSet loads; when the last load of the tile has been
// issued, the first two sets of the next tile (row `row_next`, if has_next) are
// requested into C and D, so the queue stays full across tiles.  Every set is
// exactly kBatSet load instructions on one code path; no exit from the middle
// of the loop (see GemvSpan for why).
constexpr int kBatSet = 4;

struct BatStreamCtx {
    const __half *W;          // matrix, offset to the first column of the range
    size_t K;                 // row length
    int col;                  // this lane's first column: 32 * wave + 8 * (lane / 16)
    int steps;                // blocks per tile and wavefront (256 columns apart)
    const __half *yh, *yl;    // this lane's activation row in LDS, at column `col`
};

__device__ __forceinline__ void bat_issue(const BatStreamCtx &C, u32x4 (&r)[kBatSet], int row, int m0)
{
#pragma unroll
    for (int j = 0; j < kBatSet; ++j) {
        const int step = m0 + j < C.steps ? m0 + j : C.steps - 1;     // past the end: re-read the last block
        const __half *p = C.W + (size_t)row * C.K + C.col + 256 * step;
        r[j] = __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4 *>(p)));
    }
    __builtin_amdgcn_sched_barrier(0);
}

// guard: a set at the end of the tile may be partly past it (its loads were clamped)
__device__ __forceinline__ void bat_consume(const BatStreamCtx &C, const u32x4 (&r)[kBatSet], f32x4 &acc, int m0,
                                            bool guard)
{
#pragma unroll
    for (int j = 0; j < kBatSet; ++j) {
        if (!guard || m0 + j < C.steps) {                 // (uniform)
            const u32x4 bh = *reinterpret_cast<const u32x4 *>(C.yh + 256 * (m0 + j));
            const u32x4 bl = *reinterpret_cast<const u32x4 *>(C.yl + 256 * (m0 + j));
            f32x4 c = acc;
            c = __builtin_amdgcn_mfma_f32_16x16x16f16(lo_halves(r[j]), lo_halves(bh), c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_16x16x16f16(hi_halves(r[j]), hi_halves(bh), c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_16x16x16f16(lo_halves(r[j]), lo_halves(bl), c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_16x16x16f16(hi_halves(r[j]), hi_halves(bl), c, 0, 0, 0);
            acc = c;
        }
    }
}

__device__ __forceinline__ void bat_tile(const BatStreamCtx &C, u32x4 (&A)[kBatSet], u32x4 (&B)[kBatSet],
                                         u32x4 (&Cn)[kBatSet], u32x4 (&Dn)[kBatSet], f32x4 &acc, int row,
                                         int row_next, bool has_next)
{
    constexpr int NS = kBatSet;
    int m0 = 0;
    while (m0 + 3 * NS < C.steps) {
        bat_consume(C, A, acc, m0, false); bat_issue(C, A, row, m0 + 2 * NS);
        bat_consume(C, B, acc, m0 + NS, false); bat_issue(C, B, row, m0 + 3 * NS);
        m0 += 2 * NS;
    }
    const bool one_more = m0 + 2 * NS < C.steps;
    if (one_more) { bat_consume(C, A, acc, m0, false); bat_issue(C, A, row, m0 + 2 * NS); }
    if (has_next) { bat_issue(C, Cn, row_next, 0); bat_issue(C, Dn, row_next, NS); }
    if (one_more) { bat_consume(C, B, acc, m0 + NS, true); bat_consume(C, A, acc, m0 + 2 * NS, true); }
    else { bat_consume(C, A, acc, m0, true); bat_consume(C, B, acc, m0 + NS, true); }
}

// Streams rows [r_begin, r_begin + 16 T) x columns [k_off, k_off + klen) of the
// row-major matrix W (row length K) against the activations in LDS (columns
// 0..klen of yh/yl, row stride Ks) and adds into acc[T].  Rows past r_last
// re-read row r_last (their results are not used).  The 8 wavefronts interleave
// blocks of 32 columns and work on one tile at a time: together they read every
// row of the tile in 512-byte steps with up to 4 KiB per row in flight - long
// runs for the DRAM pages.  Lanes of columns without a sequence read some
// sequence's activations: their products land in columns of the result that are
// never looked at.
template <int T>
struct BatStream {
    BatStreamCtx C;
    int arow[T + 1];
    u32x4 r0[kBatSet], r1[kBatSet], r2[kBatSet], r3[kBatSet];

    // requests the first two sets of the first tile: weights depend on nothing, so this
    // comes before the activations are even in LDS (yh, yl are only read by run())
    __device__ __forceinline__ void begin(const __half *__restrict__ W, int K, int r_begin, int r_last, int k_off,
                                          int klen, const __half *yh, const __half *yl, int Ks, int tid)
    {
        const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int n = lane & 15, q = lane >> 4;
        C.K = (size_t)K;
        C.col = 32 * wave + 8 * q;
        C.W = W + k_off;
        C.steps = klen >> 8;
        C.yh = yh + (n & (kBatMax - 1)) * Ks + C.col;
        C.yl = yl + (n & (kBatMax - 1)) * Ks + C.col;
#pragma unroll
        for (int t = 0; t <= T; ++t) arow[t] = min(r_begin + 16 * (t < T ? t : T - 1) + n, r_last);
        if (C.steps <= 0) return;
        bat_issue(C, r0, arow[0], 0);
        bat_issue(C, r1, arow[0], kBatSet);
    }
    __device__ __forceinline__ void run(f32x4 (&acc)[T])
    {
        if (C.steps <= 0) return;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            if (t & 1) bat_tile(C, r2, r3, r0, r1, acc[t], arow[t], arow[t + 1], t + 1 < T);
            else bat_tile(C, r0, r1, r2, r3, acc[t], arow[t], arow[t + 1], t + 1 < T);
        }
    }
};

// accumulators of the 8 wavefronts -> LDS red[wave][tile][row in tile][sequence]
template <int T>
__device__ __forceinline__ void bat_spill(float *red, const f32x4 (&acc)[T], int tid)
{
    const int lane = tid & 63, wave = tid >> 6, n = lane & 15, q = lane >> 4;
    if (n < kBatMax) {
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[((wave * T + t) * 16 + 4 * q + i) * kBatMax + n] = acc[t][i];
    }
}
// row (0..16T-1) of sequence b, wavefronts added in order
template <int T>
__device__ __forceinline__ float bat_total(const float *red, int row, int b)
{
    float s = 0.f;
    for (int w = 0; w < 8; ++w) s += red[((w * T + (row >> 4)) * 16 + (row & 15)) * kBatMax + b];
    return s;
}

// 8 consecutive fp32 values -> fp16 heads and remainders, one 16-byte LDS write each
__device__ __forceinline__ void bat_put8(__half *yh, __half *yl, int at, const float (&v)[8])
{
    union { __half h[8]; u32x4 u; } hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi.h[e] = __float2half_rn(v[e]);
        lo.h[e] = __float2half_rn(v[e] - __half2float(hi.h[e]));
    }
    *reinterpret_cast<u32x4 *>(yh + at) = hi.u;
    *reinterpret_cast<u32x4 *>(yl + at) = lo.u;
}

// src[b * stride + 0..klen) (fp32, klen <= 4096 a multiple of 8) of every sequence -> hi/lo rows in
// LDS: a thread owns one group of 8 values of every sequence; load() requests them all,
// commit() converts and writes (other loads can be queued in between)
struct BatStage {
    f32x4 v[kBatMax][2];
    __device__ __forceinline__ void load(const float *src, size_t stride, int klen, int nb, int tid)
    {
        const int c = tid < (klen >> 3) ? tid : 0;
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            const float *p = src + (size_t)(b < nb ? b : 0) * stride + 8 * c;
            v[b][0] = *as_global(reinterpret_cast<const f32x4 *>(p));
            v[b][1] = *as_global(reinterpret_cast<const f32x4 *>(p + 4));
        }
    }
    __device__ __forceinline__ void commit(int klen, __half *yh, __half *yl, int Ks, int nb, int tid) const
    {
        if (tid < (klen >> 3)) {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b) {
                if (b < nb) {
                    const float e[8] = {v[b][0][0], v[b][0][1], v[b][0][2], v[b][0][3], v[b][1][0], v[b][1][1], v[b][1][2], v[b][1][3]};
                    bat_put8(yh, yl, b * Ks + 8 * tid, e);
                }
            }
        }
    }
};

// Both LayerNorms of every sequence (they share input and statistics; two passes,
// biased variance) -> hi/lo rows in LDS.  A thread owns one group of 8 elements of
// every sequence (hidden <= 4096); the sums go through `red` (2 * 8 * kBatMax floats)
// in wavefront order.  load() requests the input and both parameter pairs, stats()
// works out mean and 1/sigma per sequence, write() puts one of the two normalised
// inputs into LDS: the first weights are requested between load() and stats() and
// stream while the statistics are worked out.
struct BatLn {
    u32x4 raw16[kBatMax];          // layer 0: fp16 input
    f32x4 raw32[kBatMax][2];       // later layers: fp32 residual stream
    u32x4 graw[2], braw[2];
    float xv[kBatMax][8], mean[kBatMax], inv[kBatMax];

    __device__ __forceinline__ void load(const BatParams &P, int tid)
    {
        const int h = P.dm.h, nchunk = h >> 3;
        const int c = tid < nchunk ? tid : 0;
        if (P.layer == 0) {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b)
                raw16[b] = *as_global(reinterpret_cast<const u32x4 *>(P.x_in + (size_t)(b < P.nb ? b : 0) * h + 8 * c));
        } else {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b) {
                const float *p = P.xres + ((size_t)(b < P.nb ? b : 0) * 2 + ((P.layer - 1) & 1)) * h + 8 * c;
                raw32[b][0] = *as_global(reinterpret_cast<const f32x4 *>(p));
                raw32[b][1] = *as_global(reinterpret_cast<const f32x4 *>(p + 4));
            }
        }
        const __half *w = P.w;
        graw[0] = *as_global(reinterpret_cast<const u32x4 *>(w + P.lay.ln1_g + 8 * c));
        braw[0] = *as_global(reinterpret_cast<const u32x4 *>(w + P.lay.ln1_b + 8 * c));
        graw[1] = *as_global(reinterpret_cast<const u32x4 *>(w + P.lay.ln2_g + 8 * c));
        braw[1] = *as_global(reinterpret_cast<const u32x4 *>(w + P.lay.ln2_b + 8 * c));
    }

    __device__ __forceinline__ void stats(const BatParams &P, float *red, int tid)
    {
        const int h = P.dm.h, nchunk = h >> 3, lane = tid & 63, wave = tid >> 6;
        const bool active = tid < nchunk;
        if (P.layer == 0) {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b) {
                const float2 a0 = unpack_h2(raw16[b].x), a1 = unpack_h2(raw16[b].y), a2 = unpack_h2(raw16[b].z), a3 = unpack_h2(raw16[b].w);
                xv[b][0] = a0.x; xv[b][1] = a0.y; xv[b][2] = a1.x; xv[b][3] = a1.y;
                xv[b][4] = a2.x; xv[b][5] = a2.y; xv[b][6] = a3.x; xv[b][7] = a3.y;
            }
        } else {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b)
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[b][e] = raw32[b][e >> 2][e & 3];
        }
        // pass 1: means
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s += xv[b][e];
            s = wave_sum(active ? s : 0.f);
            if (lane == 0) red[wave * kBatMax + b] = s;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            float s = 0.f;
            for (int w = 0; w < 8; ++w) s += red[w * kBatMax + b];
            mean[b] = s / (float)h;
        }
        // pass 2: variances
        float *red2 = red + 8 * kBatMax;
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dlt = xv[b][e] - mean[b];
                s += dlt * dlt;
            }
            s = wave_sum(active ? s : 0.f);
            if (lane == 0) red2[wave * kBatMax + b] = s;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            float s = 0.f;
            for (int w = 0; w < 8; ++w) s += red2[w * kBatMax + b];
            inv[b] = 1.0f / sqrtf(s / (float)h + P.dm.ln_eps);
        }
    }

    // which: 0 = the LayerNorm in front of QKV, 1 = the one in front of the MLP
    __device__ __forceinline__ void write(const BatParams &P, int which, __half *yh, __half *yl, int Ks, int tid) const
    {
        if (tid >= (P.dm.h >> 3)) return;
        const u32x4 g = graw[which], bt = braw[which];
        const unsigned gw[4] = {g.x, g.y, g.z, g.w}, bw[4] = {bt.x, bt.y, bt.z, bt.w};
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            if (b < P.nb) {
                float yv[8];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float2 g2 = unpack_h2(gw[e2]), b2 = unpack_h2(bw[e2]);
                    yv[2 * e2] = (xv[b][2 * e2] - mean[b]) * inv[b] * g2.x + b2.x;
                    yv[2 * e2 + 1] = (xv[b][2 * e2 + 1] - mean[b]) * inv[b] * g2.y + b2.y;
                }
                bat_put8(yh, yl, b * Ks + 8 * tid, yv);
            }
        }
    }
};

// QKV rows of this workgroup from the summed accumulators: + bias, rotary, K/V append, q.
// Pairs of adjacent packed rows (a rotary pair sits in one), as in the per-sequence epilogue.
template <int T>
__device__ __forceinline__ void bat_finish_qkv(const BatParams &P, const float *red, int r_begin, int r_n, int b,
                                               int tid)
{
    const Dims &dm = P.dm;
    const __half *bq = P.w + P.lay.b_qkv;
    const int h = dm.h, d = dm.d, r = dm.r, pos = P.pos[b];
    for (int pr = tid >> 3; 2 * pr < r_n; pr += 64) {
        const int p = r_begin + 2 * pr;                    // packed row, even (rows is even)
        const int pd = p / d, i = p - pd * d;
        const int nh = pd / 3, c = pd - 3 * nh;
        float v0 = bat_total<T>(red, 2 * pr, b) + __half2float(bq[p]);
        float v1 = bat_total<T>(red, 2 * pr + 1, b) + __half2float(bq[p + 1]);
        int d0 = i, d1 = i + 1;
        if (c < 2 && i < r) {
            const float2 cs = P.rope[(size_t)pos * (r >> 1) + (i >> 1)];
            const float lo = v0 * cs.x - v1 * cs.y, hi = v1 * cs.x + v0 * cs.y;
            v0 = lo; v1 = hi;
            d0 = i >> 1; d1 = (i >> 1) + (r >> 1);
        }
        if (c == 0) {
            P.q[(size_t)b * h + nh * d + d0] = v0;
            P.q[(size_t)b * h + nh * d + d1] = v1;
        } else {
            P.kv[kv_offset(dm, c - 1, P.kv_b0 + b * P.kv_bstep, nh, d0, pos)] = __float2half_rn(v0);
            P.kv[kv_offset(dm, c - 1, P.kv_b0 + b * P.kv_bstep, nh, d1, pos)] = __float2half_rn(v1);
        }
    }
}

// LayerNorms, QKV rows and MLP-up rows of a layer in one launch: the input is read and
// its statistics are worked out once; the MLP-up weights are requested before the QKV
// rows are finished, so the stream runs on across the two parts.  A workgroup owns
// P.rows QKV rows (TQ tiles) and P.rows2 MLP-up rows (TU tiles); either share may be
// empty at the end of the grid.
template <int TQ, int TU>
__global__ void __launch_bounds__(512) k_bat_qkv_up(BatParams P)
{
    extern __shared__ __align__(16) float lds[];
    if (!bat_positions_ok(P)) return;
    const Dims &dm = P.dm;
    const int h = dm.h, tid = threadIdx.x, Ks = h + kBatPad;
    __half *yh = reinterpret_cast<__half *>(lds), *yl = yh + kBatMax * Ks;
    const int q_begin = blockIdx.x * P.rows, q_n = max(0, min(P.rows, 3 * h - q_begin));
    const int u_begin = blockIdx.x * P.rows2, u_n = max(0, min(P.rows2, dm.f - u_begin));
    if (q_n == 0 && u_n == 0) return;                      // (whole workgroup)
    const __half *w = P.w;
    float *stat = reinterpret_cast<float *>(yl + kBatMax * Ks);     // behind the activations
    // order of the requests: LayerNorm inputs, then the first weights; the statistics are
    // worked out while those weights arrive.  Rows past a share's end re-read its last row
    // (an empty share streams the matrix's first row; its results are not used).
    BatLn ln;
    ln.load(P, tid);
    BatStream<TQ> bq;
    bq.begin(w + P.lay.w_qkv, h, q_n ? q_begin : 0, q_n ? q_begin + q_n - 1 : 0, 0, h, yh, yl, Ks, tid);
    ln.stats(P, stat, tid);
    ln.write(P, 0, yh, yl, Ks, tid);
    __syncthreads();
    f32x4 accq[TQ], accu[TU];
#pragma unroll
    for (int t = 0; t < TQ; ++t) accq[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < TU; ++t) accu[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    bq.run(accq);
    BatStream<TU> bu;
    bu.begin(w + P.lay.w_up, h, u_n ? u_begin : 0, u_n ? u_begin + u_n - 1 : 0, 0, h, yh, yl, Ks, tid);
    __syncthreads();                                       // the first normalised input is no longer read
    ln.write(P, 1, yh, yl, Ks, tid);
    __syncthreads();
    bu.run(accu);
    __syncthreads();                                       // the activations are no longer read: the space is reused
    float *redq = lds, *redu = lds + 8 * TQ * 16 * kBatMax;
    bat_spill<TQ>(redq, accq, tid);
    bat_spill<TU>(redu, accu, tid);
    __syncthreads();
    const int b = tid & (kBatMax - 1);
    if (b >= P.nb) return;
    bat_finish_qkv<TQ>(P, redq, q_begin, q_n, b, tid);
    const __half *bup = w + P.lay.b_up;
    for (int row = tid >> 3; row < u_n; row += 64)
        P.m[(size_t)b * dm.f + u_begin + row] =
            gelu_act(bat_total<TU>(redu, row, b) + __half2float(bup[u_begin + row]), dm.flags);
}

template <int T>
__global__ void __launch_bounds__(512) k_bat_out(BatParams P)
{
    extern __shared__ __align__(16) float lds[];
    if (!bat_positions_ok(P)) return;
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, tid = threadIdx.x, Ks = h + kBatPad;
    __half *yh = reinterpret_cast<__half *>(lds), *yl = yh + kBatMax * Ks;
    const int r_begin = blockIdx.x * P.rows, r_n = max(0, min(P.rows, h - r_begin));
    if (r_n == 0) return;
    const __half *w = P.w;
    f32x4 acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    // attention output of every sequence -> output projection.  In every stretch the
    // activations are requested first and the first weights right behind them, so the
    // weights stream while the activations are converted and written to LDS.
    BatStage st;
    BatStream<T> bs;
    st.load(P.o, (size_t)h, h, P.nb, tid);
    bs.begin(w + P.lay.w_dense, h, r_begin, r_begin + r_n - 1, 0, h, yh, yl, Ks, tid);
    st.commit(h, yh, yl, Ks, P.nb, tid);
    __syncthreads();
    bs.run(acc);
    // GELU(up) in slices of at most h columns -> down projection, same accumulators
    for (int k_off = 0; k_off < f; k_off += h) {
        const int klen = min(h, f - k_off);
        st.load(P.m + k_off, (size_t)f, klen, P.nb, tid);
        bs.begin(w + P.lay.w_down, f, r_begin, r_begin + r_n - 1, k_off, klen, yh, yl, Ks, tid);
        __syncthreads();                                   // the previous stretch no longer reads the activations
        st.commit(klen, yh, yl, Ks, P.nb, tid);
        __syncthreads();
        bs.run(acc);
    }
    __syncthreads();
    float *red = lds;
    bat_spill<T>(red, acc, tid);
    __syncthreads();
    const int b = tid & (kBatMax - 1);
    if (b >= P.nb) return;
    const __half *bde = w + P.lay.b_dense, *bdn = w + P.lay.b_down;
    const bool last = P.layer == P.n_layers - 1;
    for (int row = tid >> 3; row < r_n; row += 64) {
        const int i = r_begin + row;
        const float branches = (bat_total<T>(red, row, b) + __half2float(bde[i])) + __half2float(bdn[i]);
        const float res = bat_x(P, b, i) + branches;
        if (last) P.out[(size_t)b * h + i] = __float2half_rn(res);
        else P.xres[((size_t)b * 2 + (P.layer & 1)) * h + i] = res;
    }
}

size_t bat_lds_bytes(const Dims &dm)
{
    return (size_t)2 * kBatMax * (dm.h + kBatPad) * sizeof(__half) + 2 * 8 * kBatMax * sizeof(float);
}

bool bat_supported(const Dims &dm, int grid, int threads)
{
    // 8 wavefronts split K in steps of 32 columns; rows per workgroup fit 4 tiles; the
    // LayerNorm keeps hidden / 64 values per lane; the reduction space fits under the activations
    const int rows_up = (dm.f + grid - 1) / grid, rows_qkv = (((3 * dm.h + grid - 1) / grid) + 1) & ~1;
    const int rows_max = rows_up > rows_qkv ? rows_up : rows_qkv;
    // (the accumulators of the QKV and MLP-up tiles are spilled side by side: 8 wavefronts x 16 rows x
    // kBatMax floats per tile)
    const size_t tiles = (size_t)(rows_qkv + 15) / 16 + (size_t)(rows_up + 15) / 16;
    return threads == 512 && dm.h % 256 == 0 && dm.f % 256 == 0 && dm.h <= 64 * kBatLnPerLane && rows_max <= 64 &&
           bat_lds_bytes(dm) <= 160 * 1024 && tiles * 8 * 16 * kBatMax * 4 <= bat_lds_bytes(dm);
}

template <int TQ>
static hipError_t launch_qkv_up_tq(const BatParams &P, int grid, size_t lds, hipStream_t s)
{
    switch ((P.rows2 + 15) / 16) {
    case 1: hipLaunchKernelGGL((k_bat_qkv_up<TQ, 1>), dim3(grid), dim3(512), lds, s, P); break;
    case 2: hipLaunchKernelGGL((k_bat_qkv_up<TQ, 2>), dim3(grid), dim3(512), lds, s, P); break;
    case 3: hipLaunchKernelGGL((k_bat_qkv_up<TQ, 3>), dim3(grid), dim3(512), lds, s, P); break;
    case 4: hipLaunchKernelGGL((k_bat_qkv_up<TQ, 4>), dim3(grid), dim3(512), lds, s, P); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_bat_qkv_up(BatParams P, int grid, hipStream_t s)
{
    P.rows = (((3 * P.dm.h + grid - 1) / grid) + 1) & ~1;   // even: a rotary pair stays in one workgroup
    P.rows2 = (P.dm.f + grid - 1) / grid;
    const size_t lds = bat_lds_bytes(P.dm);
    switch ((P.rows + 15) / 16) {
    case 1: return launch_qkv_up_tq<1>(P, grid, lds, s);
    case 2: return launch_qkv_up_tq<2>(P, grid, lds, s);
    case 3: return launch_qkv_up_tq<3>(P, grid, lds, s);
    case 4: return launch_qkv_up_tq<4>(P, grid, lds, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_bat_out(BatParams P, int grid, hipStream_t s)
{
    P.rows = (P.dm.h + grid - 1) / grid;
    const size_t lds = bat_lds_bytes(P.dm);
    const int T = (P.rows + 15) / 16;
    switch (T) {
    case 1: hipLaunchKernelGGL(k_bat_out<1>, dim3(grid), dim3(512), lds, s, P); break;
    case 2: hipLaunchKernelGGL(k_bat_out<2>, dim3(grid), dim3(512), lds, s, P); break;
    case 3: hipLaunchKernelGGL(k_bat_out<3>, dim3(grid), dim3(512), lds, s, P); break;
    case 4: hipLaunchKernelGGL(k_bat_out<4>, dim3(grid), dim3(512), lds, s, P); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t prepare_bat_kernels(size_t lds_bytes)
{
#define CFPP_BAT_ATTR(k) \
    do { \
        hipError_t e_ = hipFuncSetAttribute(reinterpret_cast<const void *>(k), \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes); \
        if (e_ != hipSuccess) return e_; \
    } while (0)
    CFPP_BAT_ATTR((k_bat_qkv_up<1, 1>)); CFPP_BAT_ATTR((k_bat_qkv_up<1, 2>)); CFPP_BAT_ATTR((k_bat_qkv_up<1, 3>));
    CFPP_BAT_ATTR((k_bat_qkv_up<1, 4>)); CFPP_BAT_ATTR((k_bat_qkv_up<2, 1>)); CFPP_BAT_ATTR((k_bat_qkv_up<2, 2>));
    CFPP_BAT_ATTR((k_bat_qkv_up<2, 3>)); CFPP_BAT_ATTR((k_bat_qkv_up<2, 4>)); CFPP_BAT_ATTR((k_bat_qkv_up<3, 1>));
    CFPP_BAT_ATTR((k_bat_qkv_up<3, 2>)); CFPP_BAT_ATTR((k_bat_qkv_up<3, 3>)); CFPP_BAT_ATTR((k_bat_qkv_up<3, 4>));
    CFPP_BAT_ATTR((k_bat_qkv_up<4, 1>)); CFPP_BAT_ATTR((k_bat_qkv_up<4, 2>)); CFPP_BAT_ATTR((k_bat_qkv_up<4, 3>));
    CFPP_BAT_ATTR((k_bat_qkv_up<4, 4>));
    CFPP_BAT_ATTR(k_bat_out<1>); CFPP_BAT_ATTR(k_bat_out<2>); CFPP_BAT_ATTR(k_bat_out<3>); CFPP_BAT_ATTR(k_bat_out<4>);
#undef CFPP_BAT_ATTR
    return hipSuccess;
}

}  // namespace cfpp
