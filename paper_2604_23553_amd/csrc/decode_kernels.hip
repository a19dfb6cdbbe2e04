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

namespace cfpp {

constexpr int kMaxThreads = 512;

// ---------------------------------------------------------------------------
// Row-split GEMV over this workgroup's rows.  Work unit = (row, K-slice), slice
// fastest, handed to wavefronts round-robin; a wavefront streams its slice with
// 16-byte loads per lane (1 KiB contiguous per instruction), multiplies with the
// activation vector held in LDS (fp32, lds_perm order, zero padded to a chunk
// multiple) and leaves the slice's partial sum in part[unit].
template <int U>
__device__ __forceinline__ void wg_gemv_u(const __half *__restrict__ Wm, int K, int row_begin,
                                          int nrows, int nsl, const float *y, float *part)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int nchunk = (K + kChunk - 1) / kChunk;
    const int cps = (nchunk + nsl - 1) / nsl;
    const int nfull = K / kChunk;                  // chunks with all 512 columns present
    const int nunits = nrows * nsl;
    for (int u = wave; u < nunits; u += nw) {
        const int rl = u / nsl, sl = u - rl * nsl;
        const int c0 = sl * cps;
        const int c1 = min(nchunk, c0 + cps);
        const __half *wrow = Wm + (size_t)(row_begin + rl) * K + lane * 8;
        const float *yl = y + lane * 4;
        float acc0 = 0.f, acc1 = 0.f;
        int c = c0;
        for (; c + U <= c1 && c + U <= nfull; c += U) {
            u32x4 wv[U];
#pragma unroll
            for (int i = 0; i < U; ++i) wv[i] = load16_stream(wrow + (size_t)(c + i) * kChunk);
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const float4 ya = *reinterpret_cast<const float4 *>(yl + (c + i) * kChunk);
                const float4 yb = *reinterpret_cast<const float4 *>(yl + (c + i) * kChunk + 256);
                if (i & 1) acc1 = dot8(wv[i], ya, yb, acc1);
                else acc0 = dot8(wv[i], ya, yb, acc0);
            }
        }
        for (; c < c1; ++c) {                      // leftover chunks, the last may be ragged
            u32x4 wv = {0u, 0u, 0u, 0u};
            if (c * kChunk + lane * 8 < K) wv = load16_stream(wrow + (size_t)c * kChunk);
            const float4 ya = *reinterpret_cast<const float4 *>(yl + c * kChunk);
            const float4 yb = *reinterpret_cast<const float4 *>(yl + c * kChunk + 256);
            acc0 = dot8(wv, ya, yb, acc0);
        }
        const float tot = wave_sum(acc0 + acc1);
        if (lane == 0) part[u] = tot;
    }
}

__device__ __forceinline__ void wg_gemv(const __half *__restrict__ Wm, int K, int row_begin,
                                        int nrows, int nsl, const float *y, float *part)
{
    if (nrows <= 0) return;
    const int nchunk = (K + kChunk - 1) / kChunk;
    const int cps = (nchunk + nsl - 1) / nsl;
    if (cps % 8 == 0) wg_gemv_u<8>(Wm, K, row_begin, nrows, nsl, y, part);
    else if (cps % 5 == 0) wg_gemv_u<5>(Wm, K, row_begin, nrows, nsl, y, part);
    else wg_gemv_u<4>(Wm, K, row_begin, nrows, nsl, y, part);
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
    return io.x16 ? __half2float(io.x16[i]) : io.x32[i];
}

__device__ __forceinline__ int round_up_chunk(int k) { return (k + kChunk - 1) / kChunk * kChunk; }

// ---------------------------------------------------------------------------
// Phase A.  LDS: y1[Kp] y2[Kp] xs[Kp] part[rows_qkv + rows_up] red[16]
__device__ void phase_a(const StepParams &P, const __half *__restrict__ w, __half *__restrict__ kv,
                        int layer, int pos, float *lds)
{
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, d = dm.d, r = dm.r;
    const int tid = threadIdx.x, nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(h);
    float *y1 = lds, *y2 = lds + Kp, *xs = lds + 2 * Kp, *part = lds + 3 * Kp;
    float *red = part + P.rows_qkv + P.rows_up;
    const LayerIO io = layer_io(P, layer);

    // both LayerNorms read the block input: stage x in LDS (fp32), then two-pass
    // statistics and the two affine outputs from LDS
    constexpr int XU = 8;                       // loads in flight per thread
    float s = 0.f;
    for (int base = 0; base < h; base += XU * nt) {
        float xv[XU];
#pragma unroll
        for (int j = 0; j < XU; ++j) {
            const int i = base + tid + j * nt;
            xv[j] = i < h ? load_x(io, i) : 0.f;
        }
#pragma unroll
        for (int j = 0; j < XU; ++j) {
            const int i = base + tid + j * nt;
            if (i < h) xs[i] = xv[j];
            s += xv[j];
        }
    }
    const float mean = block_sum(s, red) / (float)h;    // (its barriers also publish xs)
    float v = 0.f;
    for (int i = tid; i < h; i += nt) {
        const float dlt = xs[i] - mean;
        v += dlt * dlt;
    }
    const float var = block_sum(v, red) / (float)h;
    const float inv = 1.0f / sqrtf(var + dm.ln_eps);
    const __half *g1 = w + P.lay.ln1_g, *b1 = w + P.lay.ln1_b;
    const __half *g2 = w + P.lay.ln2_g, *b2 = w + P.lay.ln2_b;
    for (int i = tid; i < Kp; i += nt) {
        float a = 0.f, b = 0.f;
        if (i < h) {
            const float t = (xs[i] - mean) * inv;
            a = t * __half2float(g1[i]) + __half2float(b1[i]);
            b = t * __half2float(g2[i]) + __half2float(b2[i]);
        }
        const int at = lds_perm(i);
        y1[at] = a;
        y2[at] = b;
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
            P.q[n * d + d0] = v0;
            P.q[n * d + d1] = v1;
        } else {
            kv[kv_offset(dm, c - 1, P.b, n, d0, pos)] = __float2half_rn(v0);
            kv[kv_offset(dm, c - 1, P.b, n, d1, pos)] = __float2half_rn(v1);
        }
    }
    const __half *bu = w + P.lay.b_up;
    for (int t = tid; t < u_n; t += nt)
        P.m[u_begin + t] = gelu_erf(part[P.rows_qkv + t] + __half2float(bu[u_begin + t]));
}

// ---------------------------------------------------------------------------
// Split-KV decode attention over this workgroup's share of the cache.
//
// All (head, 32-position row) pairs of the sequence form one line of
// T = H * ceil(n_tok/32) rows; workgroup g owns rows [T*g/G, T*(g+1)/G), which
// may cover the tail of one head and the start of the next.  Inside a head, a
// wavefront step covers 32 positions: lane l handles position l/2 and the 8-dim
// half (l & 1) of every 16-dim slab, so one load instruction reads 1 KiB
// contiguous.  Each lane pair keeps its own online-softmax state (running max,
// sum, d/2 accumulators); states are merged lane -> wavefront -> workgroup ->
// head in fixed orders.  The workgroup that delivers the last partial of a
// head combines all of that head's partials in slot order.
// scr: nw*(D+2) + 4 floats of LDS.
template <int D>
__device__ void attn_share(const StepParams &P, const __half *__restrict__ kv, int n_tok, float *scr)
{
    constexpr int NG = D / 16;
    const Dims &dm = P.dm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int hp = lane & 1, tl = lane >> 1;
    const int H = dm.H;
    const long long g = blockIdx.x;
    const int R = (n_tok + kRowPos - 1) / kRowPos;
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

    for (long long sb = r0; sb < r1;) {
        const int s = (int)(sb / R);                       // head
        const long long se = min(r1, (long long)(s + 1) * R);
        const int row_lo = (int)(sb - (long long)s * R), row_hi = (int)(se - (long long)s * R);
        const __half *Kh = Kb + (size_t)s * hs + hp * 8;
        const __half *Vh = Vb + (size_t)s * hs + hp * 8;

        float q[NG][8];
        {
            const float *qp = P.q + s * D + hp * 8;
#pragma unroll
            for (int jj = 0; jj < NG; ++jj) {
                const float4 a = *reinterpret_cast<const float4 *>(qp + 16 * jj);
                const float4 b = *reinterpret_cast<const float4 *>(qp + 16 * jj + 4);
                q[jj][0] = a.x; q[jj][1] = a.y; q[jj][2] = a.z; q[jj][3] = a.w;
                q[jj][4] = b.x; q[jj][5] = b.y; q[jj][6] = b.z; q[jj][7] = b.w;
            }
        }
        float acc[NG][8];
#pragma unroll
        for (int jj = 0; jj < NG; ++jj)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[jj][e] = 0.f;
        float mrun = -INFINITY, lrun = 0.f;

        for (int row = row_lo + wave; row < row_hi; row += nw) {
            const int t = row * kRowPos + tl;
            const bool valid = t < n_tok;
            u32x4 kk[NG], vv[NG];
#pragma unroll
            for (int jj = 0; jj < NG; ++jj) {
                kk[jj] = u32x4{0u, 0u, 0u, 0u};
                vv[jj] = u32x4{0u, 0u, 0u, 0u};
            }
            if (valid) {
#pragma unroll
                for (int jj = 0; jj < NG; ++jj)
                    kk[jj] = load16_stream(Kh + ((size_t)jj * dm.max_seq + t) * 16);
#pragma unroll
                for (int jj = 0; jj < NG; ++jj)
                    vv[jj] = load16_stream(Vh + ((size_t)jj * dm.max_seq + t) * 16);
            }
            float sp = 0.f;
#pragma unroll
            for (int jj = 0; jj < NG; ++jj) {
                const float4 qa = {q[jj][0], q[jj][1], q[jj][2], q[jj][3]};
                const float4 qb = {q[jj][4], q[jj][5], q[jj][6], q[jj][7]};
                sp = dot8(kk[jj], qa, qb, sp);
            }
            sp += dpp_mov<kDppXor1>(sp);                   // both halves of the head dim
            const float sc = valid ? sp * scale : -INFINITY;
            const float mn = fmaxf(mrun, sc);
            const float corr = mrun == -INFINITY ? 0.f : expf(mrun - mn);
            const float p = valid ? expf(sc - mn) : 0.f;
            lrun = lrun * corr + p;
#pragma unroll
            for (int jj = 0; jj < NG; ++jj) {
                const float2 a = unpack_h2(vv[jj].x), b = unpack_h2(vv[jj].y);
                const float2 c = unpack_h2(vv[jj].z), e = unpack_h2(vv[jj].w);
                acc[jj][0] = fmaf(p, a.x, acc[jj][0] * corr); acc[jj][1] = fmaf(p, a.y, acc[jj][1] * corr);
                acc[jj][2] = fmaf(p, b.x, acc[jj][2] * corr); acc[jj][3] = fmaf(p, b.y, acc[jj][3] * corr);
                acc[jj][4] = fmaf(p, c.x, acc[jj][4] * corr); acc[jj][5] = fmaf(p, c.y, acc[jj][5] * corr);
                acc[jj][6] = fmaf(p, e.x, acc[jj][6] * corr); acc[jj][7] = fmaf(p, e.y, acc[jj][7] * corr);
            }
            mrun = mn;
        }

        // lanes -> wavefront
        const float mw = wave_max(mrun);
        const float fl = mrun == -INFINITY ? 0.f : expf(mrun - mw);
        const float lw = wave_sum(hp == 0 ? lrun * fl : 0.f);
#pragma unroll
        for (int jj = 0; jj < NG; ++jj)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float tot = parity_sum(acc[jj][e] * fl);
                if (lane < 2) wp[wave * D + 16 * jj + 8 * hp + e] = tot;
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
            slot[tid] = O;
            if (tid == 0) { slot[D] = M; slot[D + 1] = L; }
        }
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            const unsigned old = __hip_atomic_fetch_add(&P.seg_cnt[s], 1u, __ATOMIC_ACQ_REL,
                                                        __HIP_MEMORY_SCOPE_AGENT);
            *flag = old == (unsigned)(ncover - 1);
        }
        __syncthreads();
        if (*flag) {                                       // this workgroup delivered the last partial
            __threadfence();
            if (tid < D) {
                const float *base = P.part + (size_t)s * P.part_slots * (D + 2);
                float M = -INFINITY;
                for (int j = 0; j < ncover; ++j) M = fmaxf(M, base[(size_t)j * (D + 2) + D]);
                float L = 0.f, O = 0.f;
                for (int j = 0; j < ncover; ++j) {
                    const float *sj = base + (size_t)j * (D + 2);
                    const float e = expf(sj[D] - M);
                    L += sj[D + 1] * e;
                    O += sj[tid] * e;
                }
                P.o[s * D + tid] = O / L;
            }
            if (tid == 0)
                __hip_atomic_store(&P.seg_cnt[s], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        sb = se;
    }
}

// copy a workspace vector into LDS in GEMV order, zero padded
__device__ __forceinline__ void stage_vector(const float *__restrict__ src, int n, float *dst)
{
    const int np = round_up_chunk(n);
    for (int i = threadIdx.x; i < np; i += blockDim.x) dst[lds_perm(i)] = i < n ? src[i] : 0.f;
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
    stage_vector(P.m, f, ml);
    attn_share<D>(P, kv, pos + 1, scr);
    __syncthreads();
    const int r_begin = g * P.rows_h, r_n = max(0, min(P.rows_h, h - r_begin));
    wg_gemv(w + P.lay.w_down, f, r_begin, r_n, P.nsl_down, ml, part);
    __syncthreads();
    const __half *bd = w + P.lay.b_down;
    for (int t = tid; t < r_n; t += nt) {
        float a = 0.f;
        for (int sl = 0; sl < P.nsl_down; ++sl) a += part[t * P.nsl_down + sl];
        P.g[r_begin + t] = a + __half2float(bd[r_begin + t]);
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
        const float res = (load_x(io, r_begin + t) + a) + P.g[r_begin + t];
        if (io.o16) io.o16[r_begin + t] = __float2half_rn(res);
        else io.o32[r_begin + t] = res;
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
