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
//   * Cross-workgroup dependencies are split-phase events (arrive early, wait
//     late).  The block (paper Sec. 2.2, GPT-NeoX residual form) has two
//     independent chains, attention (QKV -> attention -> dense) and MLP
//     (up -> down); their tiles are interleaved
//         QKV | up | attention | down | dense
//     so that the wait for "all q/k/v written" is covered by the up-projection
//     stream, "all m written" by the attention stream and "all heads combined"
//     by the down-projection stream.  Only "layer output complete" (needed by
//     the next LayerNorm) is exposed, and prefetched tiles cover most of it.
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
       cCtrlWords = 16 };

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

// ---- cross-workgroup events ------------------------------------------------------
// Four event types (Q, M, O, X).  Each has a two-level counter tree that only
// grows: workgroups add to their group's counter (groups of 16), the last of a
// group adds to the top counter, waiters poll the top counter.  The k-th
// instance of a type since the counters were zeroed is complete when
// top >= ngroups * k.  (A full X event separates successive instances of every
// type, so instances cannot mix.)
struct Events {
    unsigned long long *base;     // [4][1 + 64] counters, one per 64-byte slot
    unsigned long long top0[4];   // top counter value this launch started from (multiple of ngroups)
    int ngroups, gsize, g;

    __device__ __forceinline__ unsigned long long *top(int type) const { return base + (size_t)type * 65 * 8; }
    __device__ __forceinline__ unsigned long long *group(int type) const
    {
        return base + ((size_t)type * 65 + 1 + (g >> 4)) * 8;
    }
    __device__ __forceinline__ void init(unsigned long long *b, int G, int wg)
    {
        base = b;
        g = wg;
        ngroups = (G + 15) >> 4;
        const int first = (wg >> 4) << 4;
        gsize = min(16, G - first);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const unsigned long long v = __hip_atomic_load(top(t), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            top0[t] = v - v % (unsigned long long)ngroups;
        }
    }
    // all of this wavefront's earlier exchange stores must be acknowledged first
    __device__ __forceinline__ void arrive(int type)
    {
        xwg_wait_stores();
        if ((threadIdx.x & 63) == 0) {
            const unsigned long long old =
                __hip_atomic_fetch_add(group(type), 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((old + 1) % (unsigned long long)gsize == 0)
                __hip_atomic_fetch_add(top(type), 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // instance: 1-based count of this type within the launch
    __device__ __forceinline__ bool wait(int type, int instance, int *ctrl, unsigned *err)
    {
        const unsigned long long target = top0[type] + (unsigned long long)ngroups * instance;
        const unsigned long long t0 = wall_clock64();
        unsigned spins = 0;
        while (__hip_atomic_load(top(type), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if ((++spins & 255u) == 0) {
                if (lds_ld(ctrl + cAbort)) return false;
                if (wall_clock64() - t0 > 200000000ull) {       // 2 s at 100 MHz
                    lds_st(ctrl + cAbort, 1);
                    __hip_atomic_store(err, (unsigned)kErrBarrierTimeout, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                    return false;
                }
            }
        }
        return true;
    }
};

// ---- timeline trace (profiling aid) ---------------------------------------------------
struct Tracer {
    unsigned long long *p;
    int n;
    __device__ __forceinline__ void init(const StepParams &P, int wave)
    {
        const bool on = (P.debug & 16) && (int)blockIdx.x == (P.debug >> 8) && wave < kTraceWaves;
        p = on ? P.trace + (size_t)wave * kTraceLen * 2 : nullptr;
        n = 0;
    }
    __device__ __forceinline__ void mark(int tag)
    {
        if (p && n < kTraceLen && (threadIdx.x & 63) == 0) {
            p[2 * n] = (unsigned long long)tag;
            p[2 * n + 1] = wall_clock64();
        }
        if (p) ++n;
    }
};

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
    int ctrl, y1, y2, qs, kn, vn, m, o, res2, res3, res5, res6, gloc, wpart, total;
};

struct StreamParams {
    StreamLds L;
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
__device__ void streamer_main(const StepParams &P, const LayerPtrs *__restrict__ ptrs, const StreamParams &SP,
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
    int flushed_layers = 0;      // layers whose segments this wavefront has all flushed
    int next_flush = 0;          // next segment to flush in layer `flushed_layers`
    int knownY = 0, knownQ = 0, knownM = 0, knownO = 0;
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
    // every layer below `upto_layer` fully flushed, then segments below upto_sl of that layer
    auto flush_until = [&](int upto_layer, int upto_sl) {
        while (ok && (flushed_layers < upto_layer || (flushed_layers == upto_layer && next_flush < upto_sl))) {
            if (next_flush >= W.nseg) { ++flushed_layers; next_flush = 0; continue; }
            need_flag(knownQ, cFlagQ, flushed_layers + 1);     // never ahead of that layer's q/k/v
            if (!ok) break;
            flush_seg(next_flush);
            ++next_flush;
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
            flush_until(layer, sl);
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
        flush_until(step > 4 ? layer + 1 : layer, 0);
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
            need_flag(knownM, cFlagM, layer + 1);
            if (!ok) return;
            const int rg = idx / W.nsl_f, sl = idx - rg * W.nsl_f;
            consume_gemv<CTF, RTF, TL>(buf, ml, sl * CTF, res5, rg * RTF, W.r_n - rg * RTF, W.nsl_f, sl, lane);
            done_tile(cCnt5);
        } else {
            need_flag(knownO, cFlagO, layer + 1);
            if (!ok) return;
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
    if (ok) flush_until(L, 0);
    tr.mark(999);
}

// ---- service wavefront ---------------------------------------------------------------
template <int D, int CTH, int RTH, int CTF, int RTF>
__device__ void service_main(const StepParams &P, const LayerPtrs *__restrict__ ptrs, const StreamParams &SP,
                             const Work<D, CTH, RTH, CTF, RTF> &W, int pos, float *lds, int NS)
{
    using A = AttnShape<D>;
    const Dims &dm = P.dm;
    const int lane = threadIdx.x & 63, g = blockIdx.x;
    const int h = dm.h, f = dm.f, d = dm.d, r = dm.r, L = P.n_layers;
    int *ctrl = reinterpret_cast<int *>(lds + SP.L.ctrl);
    unsigned *err = P.sync + kSyncErr;
    float *y1 = lds + SP.L.y1, *y2 = lds + SP.L.y2, *ml = lds + SP.L.m, *ol = lds + SP.L.o;
    const float *res2 = lds + SP.L.res2, *res3 = lds + SP.L.res3, *res5 = lds + SP.L.res5, *res6 = lds + SP.L.res6;
    float *qs = lds + SP.L.qs, *gloc = lds + SP.L.gloc;
    unsigned *kn = reinterpret_cast<unsigned *>(lds + SP.L.kn), *vn = reinterpret_cast<unsigned *>(lds + SP.L.vn);
    const float *wpart = lds + SP.L.wpart;

    Events ev;
    ev.init(SP.events, gridDim.x, g);
    Tracer tr;
    tr.init(P, NS);

    for (int layer = 0; layer < L; ++layer) {
        const __half *w = ptrs->w[layer];
        __half *kv = ptrs->kv[layer];
        const bool first = layer == 0, last = layer == L - 1;
        const float *xin32 = first ? nullptr : P.xres + (size_t)((layer - 1) & 1) * h;
        float *xout32 = last ? nullptr : P.xres + (size_t)(layer & 1) * h;

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
            if (!first && !ev.wait(3, layer, ctrl, err)) return;
            tr.mark(11);
            float xv[CTH][8];
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < CTH; ++j) {
                const int gi = lane + 64 * j;
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[j][e] = 0.f;
                if (gi < ngrp) {
                    if (first) {
                        const u32x4 xr = load16(P.x_in + gi * 8);
                        const float2 a = unpack_h2(xr.x), b = unpack_h2(xr.y), c = unpack_h2(xr.z), e2 = unpack_h2(xr.w);
                        xv[j][0] = a.x; xv[j][1] = a.y; xv[j][2] = b.x; xv[j][3] = b.y;
                        xv[j][4] = c.x; xv[j][5] = c.y; xv[j][6] = e2.x; xv[j][7] = e2.y;
                    } else {
                        const float *xp = xin32 + gi * 8;
                        const float2 a = xwg_load2(xp), b = xwg_load2(xp + 2), c = xwg_load2(xp + 4), e2 = xwg_load2(xp + 6);
                        xv[j][0] = a.x; xv[j][1] = a.y; xv[j][2] = b.x; xv[j][3] = b.y;
                        xv[j][4] = c.x; xv[j][5] = c.y; xv[j][6] = e2.x; xv[j][7] = e2.y;
                    }
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

        // ---- F2: QKV rows done -> bias, rotary, q to workspace, k/v appended ----
        {
            const __half *bq = w + P.lay.b_qkv;
            const int npair = W.q_n >> 1;
            for (int base = 0; base < npair; base += 64) {
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
                        xwg_store(P.q + n * d + d0, v0);
                        xwg_store(P.q + n * d + d1, v1);
                    } else {
                        xwg_store_half(kv + kv_offset(dm, c - 1, P.b, n, d0, pos), v0);
                        xwg_store_half(kv + kv_offset(dm, c - 1, P.b, n, d1, pos), v1);
                    }
                }
            }
            if (npair == 0 && !lds_wait_ge(ctrl, cCnt2, (layer + 1) * W.n2, err)) return;
            tr.mark(20);
            ev.arrive(0);
            tr.mark(21);
        }

        // ---- C4: all q/k/v written -> this workgroup's heads into LDS ----
        {
            if (!ev.wait(0, layer + 1, ctrl, err)) return;
            tr.mark(30);
            for (int sl = 0; sl < W.nseg; ++sl) {
                const int s = W.s_first + sl;
                for (int i2 = lane; i2 < D / 2; i2 += 64) {
                    const float2 v = xwg_load2(P.q + s * D + 2 * i2);
                    *reinterpret_cast<float2 *>(qs + sl * D + 2 * i2) = v;
                }
                // new K and V rows of head s: D halves each, fetched as 8-byte words (4 dims)
                for (int i4 = lane; i4 < D / 4; i4 += 64) {
                    const int dim = 4 * i4;
                    const float2 kw = xwg_load2(reinterpret_cast<const float *>(kv + kv_offset(dm, 0, P.b, s, dim, pos)));
                    const float2 vw = xwg_load2(reinterpret_cast<const float *>(kv + kv_offset(dm, 1, P.b, s, dim, pos)));
                    kn[sl * (D / 2) + 2 * i4] = __float_as_uint(kw.x);
                    kn[sl * (D / 2) + 2 * i4 + 1] = __float_as_uint(kw.y);
                    vn[sl * (D / 2) + 2 * i4] = __float_as_uint(vw.x);
                    vn[sl * (D / 2) + 2 * i4 + 1] = __float_as_uint(vw.y);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) lds_st(ctrl + cFlagQ, layer + 1);
            tr.mark(31);
        }

        // ---- F3: up rows done -> bias, GELU, m to workspace ----
        {
            const __half *bu = w + P.lay.b_up;
            for (int base = 0; base < W.u_n; base += 64) {
                const int t = base + lane;
                const bool act = t < W.u_n;
                const float bias = act ? __half2float(bu[W.u_begin + t]) : 0.f;
                if (base == 0 && !lds_wait_ge(ctrl, cCnt3, (layer + 1) * W.n3, err)) return;
                if (act) xwg_store(P.m + W.u_begin + t, gelu_erf(res3[t] + bias));
            }
            if (W.u_n == 0 && !lds_wait_ge(ctrl, cCnt3, (layer + 1) * W.n3, err)) return;
            tr.mark(40);
            ev.arrive(1);
            tr.mark(41);
        }

        // ---- C5: all of m written -> LDS ----
        {
            if (!ev.wait(1, layer + 1, ctrl, err)) return;
            tr.mark(50);
            constexpr int UN = 16;
            const int n2 = f >> 1, np2 = ((f + kChunk - 1) / kChunk * kChunk) >> 1;
            for (int base = 0; base < np2; base += UN * 64) {
                float2 v[UN];
#pragma unroll
                for (int j = 0; j < UN; ++j) {
                    const int i2 = base + lane + j * 64;
                    v[j] = i2 < n2 ? xwg_load2(P.m + 2 * i2) : float2{0.f, 0.f};
                }
#pragma unroll
                for (int j = 0; j < UN; ++j) {
                    const int i2 = base + lane + j * 64;
                    if (i2 < np2) *reinterpret_cast<float2 *>(ml + lds_perm(i2 * 2)) = v[j];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) lds_st(ctrl + cFlagM, layer + 1);
            tr.mark(51);
        }

        // ---- F4: split-KV merge of this workgroup's heads, last arriver combines ----
        {
            for (int sl = 0; sl < W.nseg; ++sl) {
                const int s = W.s_first + sl;
                if (!lds_wait_ge(ctrl, cCntA0 + sl, (layer + 1) * NS, err)) return;
                tr.mark(60 + sl);
                const float *wp = wpart + (size_t)sl * NS * (D + 2);
                float M = -INFINITY;
                for (int wv = 0; wv < NS; ++wv) M = fmaxf(M, wp[wv * (D + 2) + D]);
                const long long g_lo = (((long long)s * W.R + 1) * W.Geff - 1) / W.T;
                const long long g_hi = (((long long)(s + 1) * W.R) * W.Geff - 1) / W.T;
                const int ncover = (int)(g_hi - g_lo + 1);
                float *slot = P.part + ((size_t)s * P.part_slots + (size_t)(g - g_lo)) * (D + 2);
                for (int i = lane; i < D; i += 64) {
                    float O = 0.f;
                    for (int wv = 0; wv < NS; ++wv) {
                        const float mv = wp[wv * (D + 2) + D];
                        if (mv != -INFINITY) O += wp[wv * (D + 2) + i] * expf(mv - M);
                    }
                    xwg_store(slot + i, O);
                }
                if (lane == 0) {
                    float Ls = 0.f;
                    for (int wv = 0; wv < NS; ++wv) {
                        const float mv = wp[wv * (D + 2) + D];
                        if (mv != -INFINITY) Ls += wp[wv * (D + 2) + D + 1] * expf(mv - M);
                    }
                    xwg_store(slot + D, M);
                    xwg_store(slot + D + 1, Ls);
                }
                xwg_wait_stores();
                unsigned old = 0;
                if (lane == 0)
                    old = __hip_atomic_fetch_add(&P.seg_cnt[s], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                old = (unsigned)__builtin_amdgcn_readfirstlane((int)old);
                if (old == (unsigned)(ncover - 1)) {          // this workgroup delivered the last partial
                    const float *base = P.part + (size_t)s * P.part_slots * (D + 2);
                    float Mx = -INFINITY;
                    for (int j = 0; j < ncover; ++j) Mx = fmaxf(Mx, xwg_load(base + (size_t)j * (D + 2) + D));
                    float Lx = 0.f;
                    for (int j = 0; j < ncover; ++j) {
                        const float *sj = base + (size_t)j * (D + 2);
                        Lx += xwg_load(sj + D + 1) * expf(xwg_load(sj + D) - Mx);
                    }
                    for (int i = lane; i < D; i += 64) {
                        float O = 0.f;
                        for (int j = 0; j < ncover; ++j) {
                            const float *sj = base + (size_t)j * (D + 2);
                            O += xwg_load(sj + i) * expf(xwg_load(sj + D) - Mx);
                        }
                        xwg_store(P.o + s * D + i, O / Lx);
                    }
                    if (lane == 0)
                        __hip_atomic_store(&P.seg_cnt[s], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            tr.mark(65);
            ev.arrive(2);
            tr.mark(66);
        }

        // ---- C6: all heads combined -> attention output into LDS ----
        {
            if (!ev.wait(2, layer + 1, ctrl, err)) return;
            tr.mark(70);
            constexpr int UN = 16;
            const int n2 = h >> 1, np2 = ((h + kChunk - 1) / kChunk * kChunk) >> 1;
            for (int base = 0; base < np2; base += UN * 64) {
                float2 v[UN];
#pragma unroll
                for (int j = 0; j < UN; ++j) {
                    const int i2 = base + lane + j * 64;
                    v[j] = i2 < n2 ? xwg_load2(P.o + 2 * i2) : float2{0.f, 0.f};
                }
#pragma unroll
                for (int j = 0; j < UN; ++j) {
                    const int i2 = base + lane + j * 64;
                    if (i2 < np2) *reinterpret_cast<float2 *>(ol + lds_perm(i2 * 2)) = v[j];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) lds_st(ctrl + cFlagO, layer + 1);
            tr.mark(71);
        }

        // ---- F5: down rows done -> g (kept in LDS, only this workgroup needs its rows) ----
        {
            const __half *bd = w + P.lay.b_down;
            for (int base = 0; base < W.r_n; base += 64) {
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
            if (W.r_n == 0 && !lds_wait_ge(ctrl, cCnt5, (layer + 1) * W.n5, err)) return;
            tr.mark(80);
        }

        // ---- F6: dense rows done -> out = x + (W_d o + b_d) + g ----
        {
            const __half *bd = w + P.lay.b_dense;
            for (int base = 0; base < W.r_n; base += 64) {
                const int t = base + lane;
                const bool act = t < W.r_n;
                float bias = 0.f, xval = 0.f;
                if (act) {
                    bias = __half2float(bd[W.r_begin + t]);
                    xval = first ? __half2float(P.x_in[W.r_begin + t]) : xwg_load(xin32 + W.r_begin + t);
                }
                if (base == 0 && !lds_wait_ge(ctrl, cCnt6, (layer + 1) * W.n6, err)) return;
                if (act) {
                    const float a = res6[t] + bias;
                    const float resv = (xval + a) + gloc[t];
                    if (last) P.out[W.r_begin + t] = __float2half_rn(resv);
                    else xwg_store(xout32 + W.r_begin + t, resv);
                }
            }
            if (W.r_n == 0 && !lds_wait_ge(ctrl, cCnt6, (layer + 1) * W.n6, err)) return;
            tr.mark(90);
            ev.arrive(3);
            tr.mark(91);
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
    L.y1 = take(Kph); L.y2 = take(Kph);
    L.qs = take(3 * dm.d); L.kn = take(3 * dm.d / 2); L.vn = take(3 * dm.d / 2);
    L.m = take(Kpf); L.o = take(Kph);
    L.res2 = take(P.rows_qkv + 8); L.res3 = take(P.rows_up + 8);
    L.res5 = take((P.rows_h + 8) * (nsl_f > 0 ? nsl_f : 1)); L.res6 = take(P.rows_h + 8);
    L.gloc = take(P.rows_h + 8);
    L.wpart = take(3 * NS * (dm.d + 2));
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
                               int grid, int threads, hipStream_t s)
{
    StreamParams SP;
    SP.events = events;
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
