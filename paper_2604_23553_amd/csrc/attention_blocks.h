// Split-KV decode attention, the pieces the decode kernels assemble.
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
// head's partials in slot order.
#pragma once
#include "decode_blocks.h"

namespace cfpp {

template <int D>
struct AttnCore {
    using A = AttnShape<D>;
    static constexpr int LPP = A::LPP, PPW = A::PPW, NP = A::NP, NV = A::NV, NE = (D + 63) / 64;

    // geometry of this launch / workgroup / lane
    const Dims *dm;
    const __half *kv, *Kb, *Vb;
    int b, n_tok, t_last, lane, sub, tl;
    int R, T, G, g, r0, r1;
    size_t hs;
    float scale;
    unsigned koff[NP];       // byte offset of this lane's piece k inside a head, for position 0
    // online-softmax state of this lane group
    float acc[NV], mrun, lrun;

    __device__ __forceinline__ void init(const StepParams &P, const __half *kv_, int n_tok_, int lane_)
    {
        dm = &P.dm;
        kv = kv_;
        b = P.b;
        n_tok = n_tok_;
        t_last = n_tok >= 2 ? n_tok - 2 : 0;
        lane = lane_;
        sub = lane & (LPP - 1);
        tl = lane / LPP;
        g = (int)blockIdx.x - P.attn_g0;
        // (host-checked: rows * workgroups stays far below 2^31)
        R = (n_tok + PPW - 1) / PPW;
        T = R * dm->H;
        // with fewer rows than workgroups only the first T workgroups take part, so
        // that every participant owns at least one row (no empty ranges in between)
        G = min(P.attn_G > 0 ? P.attn_G : (int)gridDim.x, T);
        r0 = g < G ? (int)((long long)T * g / G) : 0;
        r1 = g < G ? (int)((long long)T * (g + 1) / G) : 0;
        scale = 1.0f / sqrtf((float)D);
        hs = kv_head_stride(*dm);
        Kb = kv + kv_offset(*dm, 0, b, 0, 0, 0);
        Vb = kv + kv_offset(*dm, 1, b, 0, 0, 0);
        // (a head's K or V is d * max_seq * 2 bytes, far below 4 GiB)
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const int pc = sub + LPP * k;
            koff[k] = ((unsigned)(pc >> 1) * (unsigned)dm->max_seq * 16u + (unsigned)(pc & 1) * 8u) * 2u;
        }
    }

    // rows [lo, hi) of head s that belong to this workgroup, for the segment starting at line row sb
    __device__ __forceinline__ void segment(int sb, int &s, int &se, int &row_lo, int &row_hi) const
    {
        s = sb / R;
        se = min(r1, (s + 1) * R);
        row_lo = sb - s * R;
        row_hi = se - s * R;
    }

    // K/V of one row of head s into registers: always exactly 2*NP load
    // instructions with every lane active, so that the in-order load counter
    // tells when this row has landed while the next one is still in flight.
    // Lanes past the last cached position re-read it (their weight is zero); the
    // new token's row comes from LDS, not from here.  row < 0: nothing is
    // needed, every lane reads the same record.
    __device__ __forceinline__ void issue(u32x4 (&kk)[NP], u32x4 (&vv)[NP], int s, int row) const
    {
        const __half *Kh = Kb + (size_t)s * hs, *Vh = Vb + (size_t)s * hs;
        const int t = row < 0 ? t_last : row * PPW + tl;
        const unsigned tb = (unsigned)(t < t_last ? t : t_last) * 32u;
#pragma unroll
        for (int k = 0; k < NP; ++k) kk[k] = load16_stream_at(Kh, koff[k] + tb);
#pragma unroll
        for (int k = 0; k < NP; ++k) vv[k] = load16_stream_at(Vh, koff[k] + tb);
        __builtin_amdgcn_sched_barrier(0);                 // the loads stay here, ahead of the arithmetic
    }

    __device__ __forceinline__ void reset()
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = 0.f;
        mrun = -INFINITY;
        lrun = 0.f;
    }

    // one row: scores, online softmax, weighted V.  kk/vv have landed when read.
    // qs: this head's query (fp32, D), kn/vn: the new token's K and V rows (fp16, D), all in LDS
    __device__ __forceinline__ void process(u32x4 (&kk)[NP], u32x4 (&vv)[NP], int row, const float *qs,
                                            const __half *kn, const __half *vn)
    {
        const int t = row * PPW + tl;
        const bool valid = t < n_tok;
        if (t >= n_tok - 1) {                              // only in the last row of a head
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
        sp += lane_xor<1>(sp);                             // the lanes sharing this position
        if constexpr (LPP == 4) sp += lane_xor<2>(sp);
        const float sc = valid ? sp * scale : -INFINITY;
        const float mn = fmaxf(mrun, sc);
        const float corr = mrun == -INFINITY ? 0.f : expf(mrun - mn);
        const float p = valid ? expf(sc - mn) : 0.f;
        lrun = lrun * corr + p;
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const float2 a = unpack_h2(vv[k].x), b2 = unpack_h2(vv[k].y);
            const float2 c = unpack_h2(vv[k].z), e = unpack_h2(vv[k].w);
            float *ac = acc + 8 * k;
            ac[0] = fmaf(p, a.x, ac[0] * corr); ac[1] = fmaf(p, a.y, ac[1] * corr);
            ac[2] = fmaf(p, b2.x, ac[2] * corr); ac[3] = fmaf(p, b2.y, ac[3] * corr);
            ac[4] = fmaf(p, c.x, ac[4] * corr); ac[5] = fmaf(p, c.y, ac[5] * corr);
            ac[6] = fmaf(p, e.x, ac[6] * corr); ac[7] = fmaf(p, e.y, ac[7] * corr);
        }
        mrun = mn;
    }

    // lanes -> wavefront: this wavefront's state into LDS slot `slot`
    // (wp[slot*D ..], wm[slot], wl[slot]); a wavefront without rows leaves (0, -inf, 0)
    __device__ __forceinline__ void wave_merge(float *wp, float *wm, float *wl, int slot)
    {
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
                wp[slot * D + 8 * (sub + LPP * (idx >> 3)) + (idx & 7)] = acc[i];
            }
        }
        if (lane == 0) { wm[slot] = mw; wl[slot] = lw; }
    }

    // workgroups covering head s: first one and how many
    __device__ __forceinline__ void cover(int s, int &g_lo, int &ncover) const
    {
        g_lo = (int)((((long long)s * R + 1) * G - 1) / T);
        const int g_hi = (int)((((long long)(s + 1) * R) * G - 1) / T);
        ncover = g_hi - g_lo + 1;
    }

    // One wavefront: the nslots wavefront states in LDS -> this workgroup's
    // partial of head s in the workspace (slot = rank of this workgroup among
    // those covering the head).  A lane owns elements lane and lane + 64.
    __device__ __forceinline__ void publish(const StepParams &P, int s, const float *wp, const float *wm,
                                            const float *wl, int nslots) const
    {
        int g_lo, ncover;
        cover(s, g_lo, ncover);
        float *slot = P.part + ((size_t)s * P.part_slots + (size_t)(g - g_lo)) * (D + 2);
        float M = -INFINITY;
        for (int wv = 0; wv < nslots; ++wv) M = fmaxf(M, wm[wv]);
        float L = 0.f, O[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) O[e] = 0.f;
        for (int wv = 0; wv < nslots; ++wv) {
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

    // One wavefront, after its publish() stores are acknowledged: count this
    // workgroup's partial of head s; the workgroup that delivers the last one
    // merges all partials of the head in slot order into P.o.  Returns whether
    // this workgroup did.
    __device__ __forceinline__ bool count_and_combine(const StepParams &P, int s) const
    {
        int g_lo, ncover;
        cover(s, g_lo, ncover);
        unsigned old = 0;
        if (lane == 0)
            old = __hip_atomic_fetch_add(&P.seg_cnt[s], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool is_last = (unsigned)__builtin_amdgcn_readfirstlane((int)old) == (unsigned)(ncover - 1);
        if (!is_last) return false;
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
                if (j0 + j < ncover) {                     // running merge in slot order
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
        return true;
    }

    // The same two steps with tagged words (value, tag pairs in `pt`, laid out like
    // P.part): the partial is published with single stores and nobody counts;
    // the first workgroup covering a head re-reads the head's slots until all
    // carry `tag`, merges them in slot order and stores the head's output, tagged
    // again, into ot[h].  Neither side waits for an acknowledgement.
    __device__ __forceinline__ void publish_tagged(const StepParams &P, float *pt, unsigned tag, int s,
                                                   const float *wp, const float *wm, const float *wl,
                                                   int nslots) const
    {
        int g_lo, ncover;
        cover(s, g_lo, ncover);
        float *slot = pt + 2 * ((size_t)s * P.part_slots + (size_t)(g - g_lo)) * (D + 2);
        float M = -INFINITY;
        for (int wv = 0; wv < nslots; ++wv) M = fmaxf(M, wm[wv]);
        float L = 0.f, O[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) O[e] = 0.f;
        for (int wv = 0; wv < nslots; ++wv) {
            const float ew = wm[wv] == -INFINITY ? 0.f : expf(wm[wv] - M);
            L += wl[wv] * ew;
#pragma unroll
            for (int e = 0; e < NE; ++e)
                if (lane + 64 * e < D) O[e] += wp[wv * D + lane + 64 * e] * ew;
        }
#pragma unroll
        for (int e = 0; e < NE; ++e)
            if (lane + 64 * e < D) xwg_store_tagged(slot + 2 * (lane + 64 * e), O[e], tag);
        if (lane == 0) { xwg_store_tagged(slot + 2 * D, M, tag); xwg_store_tagged(slot + 2 * (D + 1), L, tag); }
    }

    // true if this workgroup is the one that combines head s
    __device__ __forceinline__ bool combines(int s) const
    {
        int g_lo, ncover;
        cover(s, g_lo, ncover);
        return g == g_lo;
    }

    __device__ __forceinline__ void combine_tagged(const StepParams &P, const float *pt, float *ot, unsigned tag,
                                                   int s) const
    {
        int g_lo, ncover;
        cover(s, g_lo, ncover);
        const float *base = pt + 2 * (size_t)s * P.part_slots * (D + 2);
        constexpr int CB = 8;
        float M = -INFINITY, L = 0.f, O[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) O[e] = 0.f;
        PollGuard pg;
        pg.start(P.sync);
        for (int j0 = 0; j0 < ncover; j0 += CB) {
            float2 mj[CB], lj[CB], oj[CB][NE];
            bool ok;
            do {
#pragma unroll
                for (int j = 0; j < CB; ++j) {
                    const int jj = j0 + j < ncover ? j0 + j : ncover - 1;
                    const float *sj = base + 2 * (size_t)jj * (D + 2);
                    mj[j] = xwg_load2(sj + 2 * D);
                    lj[j] = xwg_load2(sj + 2 * (D + 1));
#pragma unroll
                    for (int e = 0; e < NE; ++e) oj[j][e] = xwg_load2(sj + 2 * (lane + 64 * e < D ? lane + 64 * e : 0));
                }
                ok = true;
#pragma unroll
                for (int j = 0; j < CB; ++j) {
                    ok = ok && __float_as_uint(mj[j].y) == tag && __float_as_uint(lj[j].y) == tag;
#pragma unroll
                    for (int e = 0; e < NE; ++e) ok = ok && __float_as_uint(oj[j][e].y) == tag;
                }
                ok = __all(ok);
            } while (!ok && !pg.give_up());
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                if (j0 + j < ncover) {                     // running merge in slot order
                    const float mn = fmaxf(M, mj[j].x);
                    const float c0 = M == -INFINITY ? 0.f : expf(M - mn);
                    const float c1 = mj[j].x == -INFINITY ? 0.f : expf(mj[j].x - mn);
                    L = L * c0 + lj[j].x * c1;
#pragma unroll
                    for (int e = 0; e < NE; ++e) O[e] = O[e] * c0 + oj[j][e].x * c1;
                    M = mn;
                }
            }
        }
#pragma unroll
        for (int e = 0; e < NE; ++e)
            if (lane + 64 * e < D) xwg_store_tagged(ot + 2 * (s * D + lane + 64 * e), O[e] / L, tag);
    }
};

// this head's query and the new token's K/V rows: workspace -> registers -> LDS,
// one element per thread (tid < D)
template <int D>
struct HeadStage {
    float q_r;
    __half kn_r, vn_r;
    __device__ __forceinline__ void issue(const StepParams &P, const __half *kv, int s, int n_tok, int tid)
    {
        q_r = 0.f;
        kn_r = __float2half(0.f);
        vn_r = kn_r;
        if (tid < D) {
            q_r = xwg_load(P.q + s * D + tid);
            kn_r = xwg_load_half(kv + kv_offset(P.dm, 0, P.b, s, tid, n_tok - 1));
            vn_r = xwg_load_half(kv + kv_offset(P.dm, 1, P.b, s, tid, n_tok - 1));
        }
    }
    __device__ __forceinline__ void commit(float *qs, __half *kn, __half *vn, int tid) const
    {
        if (tid < D) { qs[tid] = q_r; kn[tid] = kn_r; vn[tid] = vn_r; }
    }
};

}  // namespace cfpp
