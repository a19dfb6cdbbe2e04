// Whole-stack decode as ONE persistent, wave-specialised kernel ("stream mode").
//
// Motivation (measured on MI355X): a kernel boundary costs ~4 us and a grid
// barrier with all waves draining ~2-3 us, against ~29 us of pure weight/KV
// streaming per Pythia-2.8B-shaped layer.  Here the memory pipe never drains:
//
//   * One workgroup per compute unit, 8 wavefronts: 7 "streamers" + 1 "service".
//   * A streamer does nothing but walk a static list of tiles (<= 10 sixteen-byte
//     loads per lane each: rows of W_qkv, W_up, this workgroup's share of the
//     KV cache, rows of W_down, rows of W_dense, then the next layer ...) with
//     the next tile's loads already in flight, multiply against activation
//     vectors held in LDS, and leave per-tile sums in LDS.  It never stores to
//     global memory and never waits on another workgroup directly.
//   * The service wavefront does everything else: LayerNorm of the layer input,
//     epilogues (bias, partial rotary, KV append, GELU, residual), the split-KV
//     merge and last-arriver combine, staging of exchanged vectors into LDS,
//     and all cross-workgroup signalling.
//   * Cross-workgroup dependencies are split-phase (produce early, consume
//     late).  The block (paper Sec. 2.2, GPT-NeoX residual form) has two
//     independent chains, attention (QKV -> attention -> dense) and MLP
//     (up -> down); their tiles are interleaved
//         QKV | up | attention | down | dense
//     so that "q/k/v of my heads written" is covered by the up-projection
//     stream, "all of m written" by the attention stream and "all heads
//     combined" by the down-projection stream.  Only "layer output complete"
//     (needed by the next LayerNorm) is exposed, and prefetched tiles cover most
//     of it.
//   * Small exchanged vectors (layer output, q/k/v of the new token, split-KV
//     partials, attention output) travel as 8-byte words (fp32 value, epoch
//     tag) written with one device-scope store each; a consumer polls the words
//     it needs until they all carry the current epoch, which costs one memory
//     hop and needs no counters.  The large GELU(up) vector keeps plain fp32 and
//     is announced by a two-level counter event.
//
// Exchange data uses device-scope (sc1) loads/stores (see device_utils.h); all
// reductions run in a fixed order, so results are bit-identical run to run.
// Every spin is bounded: on timeout an error flag is raised and every
// wavefront leaves its loops, so the grid always drains.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <type_traits>
#include "decode_params.h"
#include "device_utils.h"
#include "attention_common.h"

namespace cfpp {

constexpr int kStreamThreads = 512;

// ---- LDS control words ---------------------------------------------------------
enum { cFlagY = 0, cFlagQ, cFlagM, cFlagO, cAbort, cCnt2, cCnt3, cCnt5, cCnt6, cCntA0, cCntA1, cCntA2,
       cStage, cFlagXr, cGatherX, cFlagOr, cGatherO, cCtrlWords = 24 };

__device__ __forceinline__ int lds_ld(const int *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_st(int *p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// wait until *p >= target (or abort); all lanes of the wave call it together
__device__ __forceinline__ bool lds_wait_ge(int *ctrl, int word, int target, unsigned *err)
{
    unsigned spins = 0;
    while (lds_ld(ctrl + word) < target) {
        __builtin_amdgcn_s_sleep(1);
        if (lds_ld(ctrl + cAbort)) return false;
        if (++spins > (1u << 25)) {                     // seconds: something is stuck
            lds_st(ctrl + cAbort, 1);
            __hip_atomic_store(err, (unsigned)kErrBarrierTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return true;
}

// ---- cross-workgroup signalling ----------------------------------------------------
// (a) Tagged words: see the file header.  The epoch of layer l of this launch is
//     E0 + l + 1 with E0 = number of M events completed before the launch, so
//     epochs never repeat while the counters are not zeroed (the host zeroes the
//     tagged buffers together with the counters).
struct Abort {
    int *ctrl;
    unsigned *err;
    unsigned long long t0;
    unsigned spins;
    __device__ __forceinline__ void start() { t0 = wall_clock64(); spins = 0; }
    // call once per unsuccessful poll; true = give up
    __device__ __forceinline__ bool tick()
    {
        if ((++spins & 63u) == 0) {
            if (lds_ld(ctrl + cAbort)) return true;
            if (wall_clock64() - t0 > 200000000ull) {       // 2 s at 100 MHz
                lds_st(ctrl + cAbort, 1);
                __hip_atomic_store(err, (unsigned)kErrBarrierTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return true;
            }
        }
        return false;
    }
};

// One wavefront fetches n tagged words starting at buf (lane handles words
// lane, lane + 64, ...) until every one carries `epoch`; values go to dst
// through `put(i, value)`.  MAXJ*64 >= n.
template <int MAXJ, class Put>
__device__ __forceinline__ bool poll_tagged(const float *buf, int n, unsigned epoch, Abort &ab, Put put)
{
    const int lane = threadIdx.x & 63;
    ab.start();
    // cheap first: one word per lane, spread over the range, until those are there
    while (true) {
        const int i = (int)(((long long)lane * n) >> 6);
        const float2 w = xwg_load2(buf + 2 * i);
        if (__all(i >= n || __float_as_uint(w.y) == epoch)) break;
        if (ab.tick()) return false;
        __builtin_amdgcn_s_sleep(2);
    }
    while (true) {
        float2 w[MAXJ];
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            const int i = lane + 64 * j;
            w[j] = i < n ? xwg_load2(buf + 2 * i) : float2{0.f, __uint_as_float(epoch)};
        }
        bool ok = true;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) ok &= __float_as_uint(w[j].y) == epoch;
        if (__all(ok)) {
#pragma unroll
            for (int j = 0; j < MAXJ; ++j) {
                const int i = lane + 64 * j;
                if (i < n) put(i, w[j].x);
            }
            return true;
        }
        if (ab.tick()) return false;
    }
}

// One wavefront of `nparts` fetches its share of n tagged words (words
// (j*nparts + part)*64 + lane) until all carry `epoch`, passing values to put.
template <class Put>
__device__ __forceinline__ bool gather_tagged_share(const float *buf, int n, unsigned epoch, int part, int nparts,
                                                    Abort &ab, Put put)
{
    const int lane = threadIdx.x & 63;
    constexpr int UB = 4;
    ab.start();
    for (int base = 0; base < n; base += UB * nparts * 64) {
        while (true) {
            float2 w[UB];
#pragma unroll
            for (int j = 0; j < UB; ++j) {
                const int i = base + (j * nparts + part) * 64 + lane;
                w[j] = i < n ? xwg_load2(buf + 2 * i) : float2{0.f, __uint_as_float(epoch)};
            }
            bool ok = true;
#pragma unroll
            for (int j = 0; j < UB; ++j) ok &= __float_as_uint(w[j].y) == epoch;
            if (__all(ok)) {
#pragma unroll
                for (int j = 0; j < UB; ++j) {
                    const int i = base + (j * nparts + part) * 64 + lane;
                    if (i < n) put(i, w[j].x);
                }
                break;
            }
            if (ab.tick()) return false;
        }
    }
    return true;
}

// wait until one word per lane, spread over the n words, carries `epoch`
__device__ __forceinline__ bool sentinel_tagged(const float *buf, int n, unsigned epoch, Abort &ab)
{
    const int lane = threadIdx.x & 63;
    ab.start();
    while (true) {
        const int i = (int)(((long long)lane * n) >> 6);
        const float2 w = xwg_load2(buf + 2 * i);
        if (__all(__float_as_uint(w.y) == epoch)) return true;
        if (ab.tick()) return false;
        __builtin_amdgcn_s_sleep(2);
    }
}

// (b) The M event ("every workgroup has written its rows of GELU(up)"): a
//     two-level counter tree that only grows.  Workgroups add to their group's
//     counter (groups of 16), the last of a group adds to the top counter,
//     waiters poll the top counter; the k-th instance since the counters were
//     zeroed is complete when top >= ngroups * k.
struct MEvent {
    unsigned long long *base;     // [1 top + 64 groups] counters, one per 64-byte slot
    unsigned long long top0;      // top counter this launch started from (multiple of ngroups)
    int ngroups, gsize, g;

    __device__ __forceinline__ unsigned long long *top() const { return base; }
    __device__ __forceinline__ unsigned long long *group() const { return base + (size_t)(1 + (g >> 4)) * 8; }
    __device__ __forceinline__ void init(unsigned long long *b, int G, int wg)
    {
        base = b;
        g = wg;
        ngroups = (G + 15) >> 4;
        gsize = min(16, G - ((wg >> 4) << 4));
        const unsigned long long v = __hip_atomic_load(as_global(top()), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        top0 = v - v % (unsigned long long)ngroups;
    }
    __device__ __forceinline__ unsigned epoch0() const { return (unsigned)(top0 / (unsigned long long)ngroups); }
    // all of this wavefront's earlier exchange stores must be acknowledged first
    __device__ __forceinline__ void arrive()
    {
        xwg_wait_stores();
        if ((threadIdx.x & 63) == 0) {
            const unsigned long long old =
                __hip_atomic_fetch_add(as_global(group()), 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((old + 1) % (unsigned long long)gsize == 0)
                __hip_atomic_fetch_add(as_global(top()), 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __device__ __forceinline__ bool wait(int instance, Abort &ab)
    {
        const unsigned long long target = top0 + (unsigned long long)ngroups * instance;
        ab.start();
        while (__hip_atomic_load(as_global(top()), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (ab.tick()) return false;
            __builtin_amdgcn_s_sleep(2);
        }
        return true;
    }
};

// ---- timeline trace (profiling aid) ---------------------------------------------------
// ---- work split of one workgroup ---------------------------------------------------
template <int D, int CTH, int RTH, int CTF, int RTF>
struct Work {
    using A = AttnShape<D>;
    static constexpr int TLG = RTH * CTH > RTF * CTF ? RTH * CTH : RTF * CTF;
    static constexpr int TL = TLG > 2 * A::NP ? TLG : 2 * A::NP;     // loads per tile

    int q_begin, q_n, u_begin, u_n, r_begin, r_n;       // rows of W_qkv (packed), W_up, W_down/W_dense
    int n2, n3, n4, n5, n6, ntl;                         // tiles per step, per layer
    int nsl_f;                                           // K-slices of a W_down row
    // attention share
    int R;                                               // rows (PPW positions each) per head
    long long T, Geff, r0, r1;
    int s_first, nseg;

    __device__ __forceinline__ void init(const StepParams &P, int pos)
    {
        const Dims &dm = P.dm;
        const int g = blockIdx.x;
        q_begin = g * P.rows_qkv; q_n = max(0, min(P.rows_qkv, 3 * dm.h - q_begin));
        u_begin = g * P.rows_up;  u_n = max(0, min(P.rows_up, dm.f - u_begin));
        r_begin = g * P.rows_h;   r_n = max(0, min(P.rows_h, dm.h - r_begin));
        nsl_f = (dm.f / kChunk) / CTF;
        n2 = (q_n + RTH - 1) / RTH;
        n3 = (u_n + RTH - 1) / RTH;
        n5 = ((r_n + RTF - 1) / RTF) * nsl_f;
        n6 = (r_n + RTH - 1) / RTH;
        const int n_tok = pos + 1;
        R = (n_tok + A::PPW - 1) / A::PPW;
        T = (long long)R * dm.H;
        Geff = min((long long)gridDim.x, T);
        r0 = g < Geff ? T * g / Geff : 0;
        r1 = g < Geff ? T * (g + 1) / Geff : 0;
        n4 = (int)(r1 - r0);
        s_first = n4 ? (int)(r0 / R) : 0;
        nseg = n4 ? (int)((r1 - 1) / R) - s_first + 1 : 0;
        ntl = n2 + n3 + n4 + n5 + n6;
    }
};

// LDS offsets (in floats), filled in by the host
struct StreamLds {
    int ctrl, y1, y2, xs, qs, kn, vn, m, o, res2, res3, res5, res6, gloc, wpart, comb, total;
};

// tagged exchange buffers in the workspace (8 bytes per value)
struct StreamTagged {
    float *xt;      // [2][h]  layer output (ping-pong by layer parity)
    float *qt;      // [3][h]  q, k, v of the new token, (head, dim) order
    float *ot;      // [h]     attention output
    float *part;    // [H][part_slots][d+2] split-KV partials
};

struct StreamParams {
    StreamLds L;
    StreamTagged T;
    unsigned long long *events;
};

// ---- streamer ------------------------------------------------------------------------
template <int CT, int RT, int TL>
__device__ __forceinline__ void issue_gemv(u32x4 (&buf)[TL], const __half *__restrict__ Wm, int K, int row0,
                                           int nvalid, int chunk0, int lane)
{
#pragma unroll
    for (int i = 0; i < TL; ++i) buf[i] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        if (r < nvalid) {
            const __half *p = Wm + (size_t)(row0 + r) * K + (size_t)chunk0 * kChunk + lane * 8;
#pragma unroll
            for (int c = 0; c < CT; ++c) buf[r * CT + c] = load16_stream(p + (size_t)c * kChunk);
        }
    }
}

// RT row sums of one tile -> res[(row_local + r) * nsl + sl]
template <int CT, int RT, int TL>
__device__ __forceinline__ void consume_gemv(const u32x4 (&buf)[TL], const float *y, int chunk0, float *res,
                                             int row_local, int nvalid, int nsl, int sl, int lane)
{
    float acc[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) acc[r] = 0.f;
    const float *yl = y + (size_t)chunk0 * kChunk + lane * 4;
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const float4 ya = *reinterpret_cast<const float4 *>(yl + c * kChunk);
        const float4 yb = *reinterpret_cast<const float4 *>(yl + c * kChunk + 256);
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[r] = dot8(buf[r * CT + c], ya, yb, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const float tot = wave_sum(acc[r]);
        if (lane == 0 && r < nvalid) res[(row_local + r) * nsl + sl] = tot;
    }
}

template <int D, int CTH, int RTH, int CTF, int RTF>
__device__ __forceinline__ void streamer_main(const StepParams &P, const LayerPtrs *__restrict__ ptrs, const StreamParams &SP,
                              const Work<D, CTH, RTH, CTF, RTF> &W, int pos, float *lds, int wave, int NS)
{
    using WK = Work<D, CTH, RTH, CTF, RTF>;
    using A = AttnShape<D>;
    constexpr int TL = WK::TL, LPP = A::LPP, PPW = A::PPW, NP = A::NP, NV = A::NV;
    const Dims &dm = P.dm;
    const int lane = threadIdx.x & 63;
    const int sub = lane & (LPP - 1), tl = lane / LPP;
    const int h = dm.h, f = dm.f, L = P.n_layers;
    int *ctrl = reinterpret_cast<int *>(lds + SP.L.ctrl);
    unsigned *err = P.sync + kSyncErr;
    const float *y1 = lds + SP.L.y1, *y2 = lds + SP.L.y2, *ml = lds + SP.L.m, *ol = lds + SP.L.o;
    float *res2 = lds + SP.L.res2, *res3 = lds + SP.L.res3, *res5 = lds + SP.L.res5, *res6 = lds + SP.L.res6;
    const float *qs = lds + SP.L.qs;
    const unsigned *kn = reinterpret_cast<const unsigned *>(lds + SP.L.kn);
    const unsigned *vn = reinterpret_cast<const unsigned *>(lds + SP.L.vn);
    float *wpart = lds + SP.L.wpart;
    const float scale = 1.0f / sqrtf((float)D);
    const size_t hs = kv_head_stride(dm);
    const int ntot = W.ntl * L;                      // fits: checked on the host
    if (W.ntl == 0) return;
    Tracer tr;
    tr.init(P, wave);

    size_t koff[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int pc = sub + LPP * k;
        koff[k] = (size_t)(pc >> 1) * dm.max_seq * 16 + (pc & 1) * 8;
    }

    auto decode = [&](int Tt, int &layer, int &step, int &idx) {
        layer = Tt / W.ntl;
        int t = Tt - layer * W.ntl;
        if (t < W.n2) { step = 2; idx = t; return; }
        t -= W.n2;
        if (t < W.n3) { step = 3; idx = t; return; }
        t -= W.n3;
        if (t < W.n4) { step = 4; idx = t; return; }
        t -= W.n4;
        if (t < W.n5) { step = 5; idx = t; return; }
        step = 6;
        idx = t - W.n5;
    };

    auto issue = [&](u32x4 (&buf)[TL], int Tt) {
        int layer, step, idx;
        decode(Tt, layer, step, idx);
        const __half *w = ptrs->w[layer];
        if (step == 2) {
            issue_gemv<CTH, RTH, TL>(buf, w + P.lay.w_qkv, h, W.q_begin + idx * RTH, W.q_n - idx * RTH, 0, lane);
        } else if (step == 3) {
            issue_gemv<CTH, RTH, TL>(buf, w + P.lay.w_up, h, W.u_begin + idx * RTH, W.u_n - idx * RTH, 0, lane);
        } else if (step == 5) {
            const int rg = idx / W.nsl_f, sl = idx - rg * W.nsl_f;
            issue_gemv<CTF, RTF, TL>(buf, w + P.lay.w_down, f, W.r_begin + rg * RTF, W.r_n - rg * RTF, sl * CTF, lane);
        } else if (step == 6) {
            issue_gemv<CTH, RTH, TL>(buf, w + P.lay.w_dense, h, W.r_begin + idx * RTH, W.r_n - idx * RTH, 0, lane);
        } else {
            // attention row: NP pieces of K then NP pieces of V for this lane's position;
            // only cached positions (t < pos); the new token's row comes from LDS
            const int rho = (int)W.r0 + idx;
            const int s = rho / W.R, row = rho - s * W.R;
            const int t = row * PPW + tl;
            const __half *kvl = ptrs->kv[layer];
            const __half *Kh = kvl + kv_offset(dm, 0, P.b, s, 0, 0);
            const __half *Vh = kvl + kv_offset(dm, 1, P.b, s, 0, 0);
#pragma unroll
            for (int i = 0; i < TL; ++i) buf[i] = u32x4{0u, 0u, 0u, 0u};
            if (t < pos) {
#pragma unroll
                for (int k = 0; k < NP; ++k) buf[k] = load16_stream(Kh + koff[k] + (size_t)t * 16);
#pragma unroll
                for (int k = 0; k < NP; ++k) buf[NP + k] = load16_stream(Vh + koff[k] + (size_t)t * 16);
            }
            (void)hs;
        }
    };

    // attention state of this wavefront
    float acc[NV];
    float mrun = -INFINITY, lrun = 0.f;
    bool active = false;
    int act_sl = 0;
    int next_flush = 0;          // next segment of the current layer to flush
    int knownY = 0, knownQ = 0, knownM = 0;
    bool ok = true;

    auto need_flag = [&](int &known, int word, int target) {
        if (known < target) {
            tr.mark(100 + word);                       // starts waiting for an LDS flag
            ok = lds_wait_ge(ctrl, word, target, err);
            known = target;
            tr.mark(200 + word);                       // flag seen
        }
    };

    // publish this wavefront's partial of segment sl (a null partial if it had no row there)
    auto flush_seg = [&](int sl) {
        float *wp = wpart + ((size_t)sl * NS + wave) * (D + 2);
        if (active && act_sl == sl) {
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
                    const int ix = off + i;
                    wp[8 * (sub + LPP * (ix >> 3)) + (ix & 7)] = acc[i];
                }
            }
            if (lane == 0) { wp[D] = mw; wp[D + 1] = lw; }
            active = false;
        } else if (lane == 0) {
            wp[D] = -INFINITY;
            wp[D + 1] = 0.f;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0)
            __hip_atomic_fetch_add(ctrl + cCntA0 + sl, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    // flush of layer `layer`: segments next_flush .. upto_sl-1 (a null partial where this
    // wavefront had no row); never ahead of that layer's q/k/v
    auto flush_layer = [&](int layer, int upto_sl) {
        while (ok && next_flush < upto_sl) {
            need_flag(knownQ, cFlagQ, layer + 1);
            if (!ok) break;
            flush_seg(next_flush);
            ++next_flush;
        }
    };

    // Layer inputs x (layers 1..upto_layer) and attention outputs o (layers below
    // upto) arrive as tagged words; once the service wavefront has seen them
    // (nearly) complete, every streamer fetches its share into LDS.
    Abort ab;
    ab.ctrl = ctrl;
    ab.err = err;
    unsigned E0 = 0;
    {
        const unsigned long long v = __hip_atomic_load(as_global(SP.events), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long ng = (unsigned long long)((gridDim.x + 15) >> 4);
        E0 = (unsigned)((v - v % ng) / ng);
    }
    float *xs = lds + SP.L.xs, *olw = lds + SP.L.o;
    // x input of `layer` (> 0): this wavefront's share into LDS
    auto gather_x = [&](int layer) {
        int kf = 0;
        need_flag(kf, cFlagXr, layer);
        if (!ok) return;
        const float *xin_t = SP.T.xt + (size_t)((layer - 1) & 1) * 2 * h;
        ok = gather_tagged_share(xin_t, h, E0 + (unsigned)layer, wave, NS, ab, [&](int i, float v) { xs[i] = v; });
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_fetch_add(ctrl + cGatherX, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    // attention output of `layer`: share into LDS, then wait for the other streamers' shares
    auto gather_o = [&](int layer) {
        int kf = 0;
        need_flag(kf, cFlagOr, layer + 1);
        if (!ok) return;
        const int hp = (h + kChunk - 1) / kChunk * kChunk;
        ok = gather_tagged_share(SP.T.ot, h, E0 + (unsigned)layer + 1u, wave, NS, ab,
                                 [&](int i, float v) { olw[lds_perm(i)] = v; });
        for (int i = h + wave * 64 + lane; i < hp; i += NS * 64) olw[lds_perm(i)] = 0.f;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_fetch_add(ctrl + cGatherO, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (ok) ok = lds_wait_ge(ctrl, cGatherO, NS * (layer + 1), err);
    };
    // GELU(up) of `layer`: share into LDS once the service wavefront has seen the M event,
    // then wait for the other streamers' shares
    auto stage_m = [&](int layer) {
        need_flag(knownM, cFlagM, layer + 1);
        if (!ok) return;
        constexpr int UNM = 8;
        const int n2 = f >> 1, np2 = ((f + kChunk - 1) / kChunk * kChunk) >> 1;
        float *mw = lds + SP.L.m;
        for (int base = 0; base < np2; base += UNM * NS * 64) {
            float2 v[UNM];
#pragma unroll
            for (int j = 0; j < UNM; ++j) {
                const int i2 = base + (j * NS + wave) * 64 + lane;
                v[j] = i2 < n2 ? xwg_load2(P.m + 2 * i2) : float2{0.f, 0.f};
            }
#pragma unroll
            for (int j = 0; j < UNM; ++j) {
                const int i2 = base + (j * NS + wave) * 64 + lane;
                if (i2 < np2) *reinterpret_cast<float2 *>(mw + lds_perm(i2 * 2)) = v[j];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_fetch_add(ctrl + cStage, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        tr.mark(300);
        ok = lds_wait_ge(ctrl, cStage, NS * (layer + 1), err);
        tr.mark(301);
    };

    // Every streamer performs the same chain of obligations, in the order the
    // data become available: for each layer  0: fetch x (layers > 0)  1: flush
    // attention partials  2: stage m  3: fetch o.  `ob` = number completed
    // (index = 4 * layer + kind).  A tile may only need obligations that precede
    // it in this chain, so no streamer can wait on something that waits on it.
    int ob = 0;
    auto advance = [&](int target) {
        while (ok && ob < target) {
            const int layer = ob >> 2, kind = ob & 3;
            if (kind == 0) { if (layer > 0) gather_x(layer); }
            else if (kind == 1) { flush_layer(layer, W.nseg); next_flush = 0; }
            else if (kind == 2) stage_m(layer);
            else gather_o(layer);
            ++ob;
        }
    };

    auto done_tile = [&](int word) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_fetch_add(ctrl + word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };

    auto consume = [&](u32x4 (&buf)[TL], int Tt) {
        int layer, step, idx;
        decode(Tt, layer, step, idx);
        if (step == 4) {
            const int rho = (int)W.r0 + idx;
            const int s = rho / W.R, row = rho - s * W.R;
            const int sl = s - W.s_first;
            advance(4 * layer + 1);
            flush_layer(layer, sl);
            need_flag(knownQ, cFlagQ, layer + 1);
            if (!ok) return;
            if (!active) {                                   // first row of this wavefront in this head
#pragma unroll
                for (int i = 0; i < NV; ++i) acc[i] = 0.f;
                mrun = -INFINITY;
                lrun = 0.f;
                active = true;
                act_sl = sl;
            }
            const int t = row * PPW + tl;
            const bool valid = t <= pos;
            if (t == pos) {                                  // the token appended in this step
#pragma unroll
                for (int k = 0; k < NP; ++k) {
                    const int pc = sub + LPP * k;
                    buf[k] = *reinterpret_cast<const u32x4 *>(kn + sl * (D / 2) + pc * 4);
                    buf[NP + k] = *reinterpret_cast<const u32x4 *>(vn + sl * (D / 2) + pc * 4);
                }
            }
            float sp = 0.f;
#pragma unroll
            for (int k = 0; k < NP; ++k) {                   // q of this head sits in LDS
                const float *qp = qs + sl * D + 8 * (sub + LPP * k);
                const float4 qa = *reinterpret_cast<const float4 *>(qp);
                const float4 qb = *reinterpret_cast<const float4 *>(qp + 4);
                sp = dot8(buf[k], qa, qb, sp);
            }
            sp += lane_xor<1>(sp);
            if constexpr (LPP == 4) sp += lane_xor<2>(sp);
            const float sc = valid ? sp * scale : -INFINITY;
            const float mn = fmaxf(mrun, sc);
            const float corr = mrun == -INFINITY ? 0.f : expf(mrun - mn);
            const float p = valid ? expf(sc - mn) : 0.f;
            lrun = lrun * corr + p;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                const float2 a = unpack_h2(buf[NP + k].x), b = unpack_h2(buf[NP + k].y);
                const float2 c = unpack_h2(buf[NP + k].z), e = unpack_h2(buf[NP + k].w);
                float *ac = acc + 8 * k;
                ac[0] = fmaf(p, a.x, ac[0] * corr); ac[1] = fmaf(p, a.y, ac[1] * corr);
                ac[2] = fmaf(p, b.x, ac[2] * corr); ac[3] = fmaf(p, b.y, ac[3] * corr);
                ac[4] = fmaf(p, c.x, ac[4] * corr); ac[5] = fmaf(p, c.y, ac[5] * corr);
                ac[6] = fmaf(p, e.x, ac[6] * corr); ac[7] = fmaf(p, e.y, ac[7] * corr);
            }
            mrun = mn;
            return;
        }
        // a GEMV tile; steps 5 and 6 come after this layer's attention rows
        advance(4 * layer + (step <= 3 ? 1 : step == 5 ? 3 : 4));
        if (!ok) return;
        if (step == 2) {
            need_flag(knownY, cFlagY, layer + 1);
            if (!ok) return;
            consume_gemv<CTH, RTH, TL>(buf, y1, 0, res2, idx * RTH, W.q_n - idx * RTH, 1, 0, lane);
            done_tile(cCnt2);
        } else if (step == 3) {
            need_flag(knownY, cFlagY, layer + 1);
            if (!ok) return;
            consume_gemv<CTH, RTH, TL>(buf, y2, 0, res3, idx * RTH, W.u_n - idx * RTH, 1, 0, lane);
            done_tile(cCnt3);
        } else if (step == 5) {
            const int rg = idx / W.nsl_f, sl = idx - rg * W.nsl_f;
            consume_gemv<CTF, RTF, TL>(buf, ml, sl * CTF, res5, rg * RTF, W.r_n - rg * RTF, W.nsl_f, sl, lane);
            done_tile(cCnt5);
        } else {
            consume_gemv<CTH, RTH, TL>(buf, ol, 0, res6, idx * RTH, W.r_n - idx * RTH, 1, 0, lane);
            done_tile(cCnt6);
        }
    };

    // double-buffered walk over this wavefront's tiles: wave, wave + NS, ...
    u32x4 bufA[TL], bufB[TL];
    int Tt = wave;
    if (Tt < ntot) issue(bufA, Tt);
    while (Tt < ntot && ok) {
        if (Tt + NS < ntot) issue(bufB, Tt + NS);
        consume(bufA, Tt);
        Tt += NS;
        if (Tt >= ntot || !ok) break;
        if (Tt + NS < ntot) issue(bufA, Tt + NS);
        consume(bufB, Tt);
        Tt += NS;
    }
    advance(4 * L);
    tr.mark(999);
}

// ---- service wavefront ---------------------------------------------------------------
template <int D, int CTH, int RTH, int CTF, int RTF>
__device__ __forceinline__ void service_main(const StepParams &P, const LayerPtrs *__restrict__ ptrs, const StreamParams &SP,
                             const Work<D, CTH, RTH, CTF, RTF> &W, int pos, float *lds, int NS)
{
    const Dims &dm = P.dm;
    const int lane = threadIdx.x & 63, g = blockIdx.x;
    const int h = dm.h, d = dm.d, r = dm.r, L = P.n_layers;
    int *ctrl = reinterpret_cast<int *>(lds + SP.L.ctrl);
    unsigned *err = P.sync + kSyncErr;
    float *y1 = lds + SP.L.y1, *y2 = lds + SP.L.y2;
    const float *res2 = lds + SP.L.res2, *res3 = lds + SP.L.res3, *res5 = lds + SP.L.res5, *res6 = lds + SP.L.res6;
    float *qs = lds + SP.L.qs, *gloc = lds + SP.L.gloc, *comb = lds + SP.L.comb, *xs = lds + SP.L.xs;
    __half *kn = reinterpret_cast<__half *>(lds + SP.L.kn), *vn = reinterpret_cast<__half *>(lds + SP.L.vn);
    const float *wpart = lds + SP.L.wpart;
    float *qt = SP.T.qt, *kt = SP.T.qt + 2 * (size_t)h, *vt = SP.T.qt + 4 * (size_t)h;

    MEvent ev;
    ev.init(SP.events, gridDim.x, g);
    const unsigned E0 = ev.epoch0();
    Abort ab;
    ab.ctrl = ctrl;
    ab.err = err;
    Tracer tr;
    tr.init(P, NS);

    for (int layer = 0; layer < L; ++layer) {
        const __half *w = ptrs->w[layer];
        __half *kv = ptrs->kv[layer];
        const bool first = layer == 0, last = layer == L - 1;
        const unsigned epoch = E0 + (unsigned)layer + 1u;
        const float *xin_t = SP.T.xt + (size_t)((layer - 1) & 1) * 2 * h;    // tagged input of layers > 0
        float *xout_t = SP.T.xt + (size_t)(layer & 1) * 2 * h;

        // ---- C1: layer input complete -> LayerNorm 1 and 2 into LDS ----
        {
            u32x4 pg1[CTH], pb1[CTH], pg2[CTH], pb2[CTH];
            const int ngrp = h >> 3;
#pragma unroll
            for (int j = 0; j < CTH; ++j) {                  // parameters do not depend on x: fetch first
                const int gi = lane + 64 * j;
                const u32x4 z = {0u, 0u, 0u, 0u};
                pg1[j] = z; pb1[j] = z; pg2[j] = z; pb2[j] = z;
                if (gi < ngrp) {
                    pg1[j] = load16(w + P.lay.ln1_g + gi * 8); pb1[j] = load16(w + P.lay.ln1_b + gi * 8);
                    pg2[j] = load16(w + P.lay.ln2_g + gi * 8); pb2[j] = load16(w + P.lay.ln2_b + gi * 8);
                }
            }
            tr.mark(10);
            // x into LDS scratch (natural order), then registers by 8-element group
            if (first) {
                for (int gi = lane; gi < ngrp; gi += 64) {
                    const u32x4 xr = load16(P.x_in + gi * 8);
                    const float2 a = unpack_h2(xr.x), b = unpack_h2(xr.y), c = unpack_h2(xr.z), e2 = unpack_h2(xr.w);
                    *reinterpret_cast<float4 *>(xs + gi * 8) = float4{a.x, a.y, b.x, b.y};
                    *reinterpret_cast<float4 *>(xs + gi * 8 + 4) = float4{c.x, c.y, e2.x, e2.y};
                }
            } else {
                // tell the streamers when the previous layer's output looks complete; they
                // fetch it into LDS together
                if (!sentinel_tagged(xin_t, h, epoch - 1u, ab)) return;
                if (lane == 0) lds_st(ctrl + cFlagXr, layer);
                if (!lds_wait_ge(ctrl, cGatherX, NS * layer, err)) return;
            }
            tr.mark(11);
            float xv[CTH][8];
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < CTH; ++j) {
                const int gi = lane + 64 * j;
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[j][e] = 0.f;
                if (gi < ngrp) {
                    const float4 a = *reinterpret_cast<const float4 *>(xs + gi * 8);
                    const float4 b = *reinterpret_cast<const float4 *>(xs + gi * 8 + 4);
                    xv[j][0] = a.x; xv[j][1] = a.y; xv[j][2] = a.z; xv[j][3] = a.w;
                    xv[j][4] = b.x; xv[j][5] = b.y; xv[j][6] = b.z; xv[j][7] = b.w;
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) s += xv[j][e];
            }
            const float mean = wave_sum(s) / (float)h;
            float v = 0.f;
#pragma unroll
            for (int j = 0; j < CTH; ++j) {
                if (lane + 64 * j < ngrp) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) { const float dl = xv[j][e] - mean; v += dl * dl; }
                }
            }
            const float var = wave_sum(v) / (float)h;
            const float inv = 1.0f / sqrtf(var + dm.ln_eps);
#pragma unroll
            for (int j = 0; j < CTH; ++j) {
                const int gi = lane + 64 * j;
                const bool real = gi < ngrp;
                float ya[8], yb[8];
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
                const int at = (j << 9) + (lane << 2);          // = lds_perm(8 * gi)
                *reinterpret_cast<float4 *>(y1 + at) = float4{ya[0], ya[1], ya[2], ya[3]};
                *reinterpret_cast<float4 *>(y1 + at + 256) = float4{ya[4], ya[5], ya[6], ya[7]};
                *reinterpret_cast<float4 *>(y2 + at) = float4{yb[0], yb[1], yb[2], yb[3]};
                *reinterpret_cast<float4 *>(y2 + at + 256) = float4{yb[4], yb[5], yb[6], yb[7]};
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) lds_st(ctrl + cFlagY, layer + 1);
            tr.mark(12);
        }

        // ---- F2: QKV rows done -> bias, rotary; q, k, v as tagged words; k, v appended ----
        {
            const __half *bq = w + P.lay.b_qkv;
            const int npair = W.q_n >> 1;
            for (int base = 0; base < npair || base == 0; base += 64) {
                const int pr = base + lane;
                const bool act = pr < npair;
                const int p = W.q_begin + 2 * (act ? pr : 0);
                const int n = p / (3 * d), rem = p - n * 3 * d;
                const int c = rem / d, i = rem - c * d;
                const bool rot = c < 2 && i < r;
                float b0 = 0.f, b1 = 0.f;
                float2 cs = {1.f, 0.f};
                if (act) {
                    b0 = __half2float(bq[p]);
                    b1 = __half2float(bq[p + 1]);
                    if (rot) cs = P.rope[(size_t)pos * (r >> 1) + (i >> 1)];
                }
                if (base == 0 && !lds_wait_ge(ctrl, cCnt2, (layer + 1) * W.n2, err)) return;
                if (act) {
                    float v0 = res2[2 * pr] + b0, v1 = res2[2 * pr + 1] + b1;
                    int d0 = i, d1 = i + 1;
                    if (rot) {
                        const float lo = v0 * cs.x - v1 * cs.y, hi = v1 * cs.x + v0 * cs.y;
                        v0 = lo; v1 = hi;
                        d0 = i >> 1; d1 = (i >> 1) + (r >> 1);
                    }
                    if (c == 0) {
                        xwg_store_tagged(qt + 2 * (n * d + d0), v0, epoch);
                        xwg_store_tagged(qt + 2 * (n * d + d1), v1, epoch);
                        xwg_store(P.q + n * d + d0, v0);             // test tap
                        xwg_store(P.q + n * d + d1, v1);
                    } else {
                        // the cache gets the fp16 value; the tagged copy carries exactly that value
                        const __half h0 = __float2half_rn(v0), h1 = __float2half_rn(v1);
                        float *tb = c == 1 ? kt : vt;
                        xwg_store_tagged(tb + 2 * (n * d + d0), __half2float(h0), epoch);
                        xwg_store_tagged(tb + 2 * (n * d + d1), __half2float(h1), epoch);
                        xwg_store_half(kv + kv_offset(dm, c - 1, P.b, n, d0, pos), __half2float(h0));
                        xwg_store_half(kv + kv_offset(dm, c - 1, P.b, n, d1, pos), __half2float(h1));
                    }
                }
            }
            tr.mark(20);
        }

        // ---- C4: q, k, v of this workgroup's heads -> LDS ----
        {
            for (int sl = 0; sl < W.nseg; ++sl) {
                const int s = W.s_first + sl;
                if (!poll_tagged<(D + 63) / 64>(qt + 2 * (size_t)s * D, D, epoch, ab,
                                                [&](int i, float v) { qs[sl * D + i] = v; })) return;
                if (!poll_tagged<(D + 63) / 64>(kt + 2 * (size_t)s * D, D, epoch, ab,
                                                [&](int i, float v) { kn[sl * D + i] = __float2half_rn(v); })) return;
                if (!poll_tagged<(D + 63) / 64>(vt + 2 * (size_t)s * D, D, epoch, ab,
                                                [&](int i, float v) { vn[sl * D + i] = __float2half_rn(v); })) return;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) lds_st(ctrl + cFlagQ, layer + 1);
            tr.mark(31);
        }

        // ---- F3: up rows done -> bias, GELU, m to workspace; M event ----
        {
            const __half *bu = w + P.lay.b_up;
            for (int base = 0; base < W.u_n || base == 0; base += 64) {
                const int t = base + lane;
                const bool act = t < W.u_n;
                const float bias = act ? __half2float(bu[W.u_begin + t]) : 0.f;
                if (base == 0 && !lds_wait_ge(ctrl, cCnt3, (layer + 1) * W.n3, err)) return;
                if (act) xwg_store(P.m + W.u_begin + t, gelu_act(res3[t] + bias, P.dm.flags));
            }
            tr.mark(40);
            ev.arrive();
            tr.mark(41);
        }

        // ---- C5: all of m written -> tell the streamers (they copy it into LDS together) ----
        {
            if (!ev.wait(layer + 1, ab)) return;
            if (lane == 0) lds_st(ctrl + cFlagM, layer + 1);
            tr.mark(50);
        }

        // ---- F4: split-KV merge of this workgroup's heads -> tagged partial slots;
        //      the first workgroup covering a head combines that head's slots ----
        {
            for (int sl = 0; sl < W.nseg; ++sl) {
                const int s = W.s_first + sl;
                if (!lds_wait_ge(ctrl, cCntA0 + sl, (layer + 1) * NS, err)) return;
                tr.mark(60 + sl);
                const float *wp = wpart + (size_t)sl * NS * (D + 2);
                float M = -INFINITY;
                for (int wv = 0; wv < NS; ++wv) M = fmaxf(M, wp[wv * (D + 2) + D]);
                const long long g_lo = (((long long)s * W.R + 1) * W.Geff - 1) / W.T;
                float *slot = SP.T.part + 2 * ((size_t)s * P.part_slots + (size_t)(g - g_lo)) * (D + 2);
                for (int i = lane; i < D; i += 64) {
                    float O = 0.f;
                    for (int wv = 0; wv < NS; ++wv) {
                        const float mv = wp[wv * (D + 2) + D];
                        if (mv != -INFINITY) O += wp[wv * (D + 2) + i] * expf(mv - M);
                    }
                    xwg_store_tagged(slot + 2 * i, O, epoch);
                }
                if (lane == 0) {
                    float Ls = 0.f;
                    for (int wv = 0; wv < NS; ++wv) {
                        const float mv = wp[wv * (D + 2) + D];
                        if (mv != -INFINITY) Ls += wp[wv * (D + 2) + D + 1] * expf(mv - M);
                    }
                    xwg_store_tagged(slot + 2 * D, M, epoch);
                    xwg_store_tagged(slot + 2 * (D + 1), Ls, epoch);
                }
            }
            tr.mark(65);
            for (int sl = 0; sl < W.nseg; ++sl) {
                const int s = W.s_first + sl;
                const long long g_lo = (((long long)s * W.R + 1) * W.Geff - 1) / W.T;
                if (g_lo != g) continue;
                const long long g_hi = (((long long)(s + 1) * W.R) * W.Geff - 1) / W.T;
                const int ncover = (int)(g_hi - g_lo + 1);
                const float *base = SP.T.part + 2 * (size_t)s * P.part_slots * (D + 2);
                const int nwords = ncover * (D + 2);
                // slots of a head are contiguous; 16 words per lane per pass
                for (int w0 = 0; w0 < nwords; w0 += 1024) {
                    if (!poll_tagged<16>(base + 2 * w0, min(1024, nwords - w0), epoch, ab,
                                         [&](int i, float v) { comb[w0 + i] = v; })) return;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                float Mx = -INFINITY;
                for (int j = 0; j < ncover; ++j) Mx = fmaxf(Mx, comb[j * (D + 2) + D]);
                float Lx = 0.f;
                for (int j = 0; j < ncover; ++j) Lx += comb[j * (D + 2) + D + 1] * expf(comb[j * (D + 2) + D] - Mx);
                for (int i = lane; i < D; i += 64) {
                    float O = 0.f;
                    for (int j = 0; j < ncover; ++j) O += comb[j * (D + 2) + i] * expf(comb[j * (D + 2) + D] - Mx);
                    xwg_store_tagged(SP.T.ot + 2 * (s * D + i), O / Lx, epoch);
                    xwg_store(P.o + s * D + i, O / Lx);          // test tap
                }
            }
            tr.mark(66);
        }

        // ---- C6: attention output of all heads present -> the streamers fetch it into LDS ----
        {
            if (!sentinel_tagged(SP.T.ot, h, epoch, ab)) return;
            if (lane == 0) lds_st(ctrl + cFlagOr, layer + 1);
            tr.mark(71);
        }

        // ---- F5: down rows done -> g (kept in LDS, only this workgroup needs its rows) ----
        {
            const __half *bd = w + P.lay.b_down;
            for (int base = 0; base < W.r_n || base == 0; base += 64) {
                const int t = base + lane;
                const bool act = t < W.r_n;
                const float bias = act ? __half2float(bd[W.r_begin + t]) : 0.f;
                if (base == 0 && !lds_wait_ge(ctrl, cCnt5, (layer + 1) * W.n5, err)) return;
                if (act) {
                    float a = 0.f;
                    for (int sl = 0; sl < W.nsl_f; ++sl) a += res5[t * W.nsl_f + sl];
                    gloc[t] = a + bias;
                }
            }
            tr.mark(80);
        }

        // ---- F6: dense rows done -> out = x + (W_d o + b_d) + g ----
        {
            const __half *bd = w + P.lay.b_dense;
            for (int base = 0; base < W.r_n || base == 0; base += 64) {
                const int t = base + lane;
                const bool act = t < W.r_n;
                float bias = 0.f, xval = 0.f;
                if (act) {
                    bias = __half2float(bd[W.r_begin + t]);
                    xval = first ? __half2float(P.x_in[W.r_begin + t]) : xwg_load2(xin_t + 2 * (W.r_begin + t)).x;
                }
                if (base == 0 && !lds_wait_ge(ctrl, cCnt6, (layer + 1) * W.n6, err)) return;
                if (act) {
                    const float a = res6[t] + bias;
                    const float resv = (xval + a) + gloc[t];
                    if (last) P.out[W.r_begin + t] = __float2half_rn(resv);
                    else xwg_store_tagged(xout_t + 2 * (W.r_begin + t), resv, epoch);
                }
            }
            tr.mark(90);
        }
    }
}

// ---- kernel ----------------------------------------------------------------------------
template <int D, int CTH, int RTH, int CTF, int RTF>
__global__ void __launch_bounds__(kStreamThreads)
k_stack_stream(StepParams P, const LayerPtrs *__restrict__ ptrs, StreamParams SP)
{
    extern __shared__ __align__(16) float lds[];
    const int p = *P.pos;
    if (p < 0 || p >= P.dm.max_seq) {
        if (threadIdx.x == 0 && blockIdx.x == 0)
            __hip_atomic_store(&P.sync[kSyncErr], (unsigned)kErrBadPos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    int *ctrl = reinterpret_cast<int *>(lds + SP.L.ctrl);
    if (threadIdx.x < cCtrlWords) ctrl[threadIdx.x] = 0;
    __syncthreads();                                     // the only workgroup barrier

    Work<D, CTH, RTH, CTF, RTF> W;
    W.init(P, p);
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6, NS = nw - 1;
    if (wave < NS) streamer_main<D, CTH, RTH, CTF, RTF>(P, ptrs, SP, W, p, lds, wave, NS);
    else service_main<D, CTH, RTH, CTF, RTF>(P, ptrs, SP, W, p, lds, NS);
}

// ---- host side ---------------------------------------------------------------------------
static int stream_shape_class(const Dims &dm)
{
    const int nh = dm.h / kChunk, nf = dm.f / kChunk;
    if ((dm.h % kChunk) || (dm.f % kChunk)) return -1;
    if (dm.d == 80 && nh == 5 && nf % 10 == 0) return 0;
    if (dm.d == 128 && nh == 8 && nf % 8 == 0) return 1;
    if (dm.d == 64 && nh == 1 && nf % 4 == 0) return 2;
    return -1;
}

bool stream_supported(const Dims &dm, int grid)
{
    return stream_shape_class(dm) >= 0 && grid >= dm.H && grid <= kMaxGrid;
}

size_t stream_lds_bytes(const Dims &dm, const StepParams &P, int threads, StreamLds *out)
{
    const int NS = threads / 64 - 1;
    const int Kph = (dm.h + kChunk - 1) / kChunk * kChunk, Kpf = (dm.f + kChunk - 1) / kChunk * kChunk;
    const int cls = stream_shape_class(dm);
    const int ctf = cls == 0 ? 10 : cls == 1 ? 8 : 4;
    const int nsl_f = (dm.f / kChunk) / (ctf > 0 ? ctf : 1);
    StreamLds L;
    int o = 0;
    auto take = [&](int n) { int at = o; o = (o + n + 3) & ~3; return at; };
    L.ctrl = take(cCtrlWords);
    L.y1 = take(Kph); L.y2 = take(Kph); L.xs = take(Kph);
    L.qs = take(3 * dm.d); L.kn = take(3 * dm.d / 2); L.vn = take(3 * dm.d / 2);
    L.m = take(Kpf); L.o = take(Kph);
    L.res2 = take(P.rows_qkv + 8); L.res3 = take(P.rows_up + 8);
    L.res5 = take((P.rows_h + 8) * (nsl_f > 0 ? nsl_f : 1)); L.res6 = take(P.rows_h + 8);
    L.gloc = take(P.rows_h + 8);
    L.wpart = take(3 * NS * (dm.d + 2));
    L.comb = take(part_slots_for(dm.H) * (dm.d + 2));
    L.total = o;
    if (out) *out = L;
    return (size_t)o * 4;
}

template <int D, int CTH, int RTH, int CTF, int RTF>
static hipError_t launch_stream_t(const StepParams &P, const LayerPtrs *ptrs, const StreamParams &SP,
                                  int grid, int threads, hipStream_t s)
{
    hipLaunchKernelGGL((k_stack_stream<D, CTH, RTH, CTF, RTF>), dim3(grid), dim3(threads),
                       (size_t)SP.L.total * 4, s, P, ptrs, SP);
    return hipGetLastError();
}

hipError_t launch_stack_stream(const StepParams &P, const LayerPtrs *ptrs, unsigned long long *events,
                               float *tagged, int grid, int threads, hipStream_t s)
{
    StreamParams SP;
    SP.events = events;
    const size_t h = P.dm.h;
    SP.T.xt = tagged;
    SP.T.qt = SP.T.xt + 2 * 2 * h;
    SP.T.ot = SP.T.qt + 3 * 2 * h;
    SP.T.part = SP.T.ot + 2 * h;
    stream_lds_bytes(P.dm, P, threads, &SP.L);
    switch (stream_shape_class(P.dm)) {
    case 0: return launch_stream_t<80, 5, 2, 10, 1>(P, ptrs, SP, grid, threads, s);
    case 1: return launch_stream_t<128, 8, 1, 8, 1>(P, ptrs, SP, grid, threads, s);
    case 2: return launch_stream_t<64, 1, 8, 4, 2>(P, ptrs, SP, grid, threads, s);
    }
    return hipErrorInvalidValue;
}

hipError_t stream_occupancy(const Dims &dm, int threads, size_t lds_bytes, int *blocks_per_cu)
{
    switch (stream_shape_class(dm)) {
    case 0: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_stream<80, 5, 2, 10, 1>, threads, lds_bytes);
    case 1: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_stream<128, 8, 1, 8, 1>, threads, lds_bytes);
    case 2: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_stream<64, 1, 8, 4, 2>, threads, lds_bytes);
    }
    return hipErrorInvalidValue;
}

hipError_t prepare_stream_kernels(size_t lds_bytes)
{
    const int v = (int)lds_bytes;
    hipError_t e;
    e = hipFuncSetAttribute((const void *)k_stack_stream<80, 5, 2, 10, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, v);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_stack_stream<128, 8, 1, 8, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, v);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)k_stack_stream<64, 1, 8, 4, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, v);
}

}  // namespace cfpp
