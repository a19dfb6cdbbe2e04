// Whole-stack decode in one persistent kernel with every grid-wide dependency
// hidden behind streaming (launch mode 2).
//
// The block (paper Sec. 2.2; Sec. 2.3 wraps the stack in one graph) has two
// independent chains after the LayerNorms - attention and MLP - and each
// grid-wide hand-over of one chain can be waited for while the other chain's
// weights stream:
//
//   QKV rows      -> q,k,v published          ... waited for behind the MLP-up rows
//   up rows, A    -> first half of GELU(up)   ... waited for behind the B rows and the attention
//   up rows, B    -> second half of GELU(up)  ... waited for behind the attention and the down columns A
//   attention     -> o published              ... waited for behind the MLP-down columns
//   down, columns A then B (stay inside the workgroup)
//   dense rows    -> next layer's input       ... the one exposed hand-over per layer
//
// The MLP is cut in two so that its intermediate never has to be waited for: the
// up-projection rows [0, f_a) of all workgroups finish first, and the down
// projection starts with the matching columns [0, f_a) of its rows while the
// second half is still on its way (a workgroup's down rows are streamed as two
// column ranges of the row-major matrix).  Each half is copied to LDS
// optimistically: the loads are issued at a point where the half is normally
// complete (a flag in LDS, set by the chain wavefront once the half's grid
// barrier has been passed, says whether it was) and only written to LDS behind
// the stretch that streams meanwhile; when the flag was not yet set the copy is
// repeated there.
//
// Nothing but that hand-over stands between two layers: the QKV and MLP-up rows
// run on gamma * x, which needs no statistics, and the LayerNorm itself (paper
// Sec. 2.2) is completed in their epilogues from two constants per row that the
// packing derived (PackedLayout::rc_qkv, rc_up):
//   W (gamma (x - mu) inv + beta) + b = inv (W (gamma x) - mu s) + c.
// Mean and variance (two passes, biased) are worked out by the chain wavefront
// while the QKV rows stream.
//
// Wavefront 0 of every workgroup is the "chain" wavefront: it finishes rows
// (biases, rotary, GELU, residual), publishes them, drives the four grid
// barriers (one per hand-over, each independent) and stages the small vectors
// the next stretch needs.  The split-KV partials travel as tagged words (value
// and an epoch in one 8-byte store) that the combining workgroup re-reads until
// they are current - no acknowledgement or counter on that path.  The epoch of
// layer l is E0 + l + 1 with E0 a counter that every launch advances by more
// than its layer count when it ends: epochs never repeat until the host zeroes
// that counter together with the tagged region.
// Wavefronts 1.. stream weights and K/V; the loads of
// the next stretch are requested before the current one is drained, so the
// memory queue never empties at a hand-over.  Both roles meet at a fixed sequence
// of workgroup barriers.  All reductions are in a fixed order (row-split GEMVs,
// slot-ordered split-KV merges): the result is bit-identical from run to run
// (the paper's fp16-atomic output accumulation, Sec. 3, is not).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "decode_blocks.h"
#include "attention_blocks.h"

namespace cfpp {

constexpr int kFusedSegs = 2;       // a workgroup's share of the attention covers at most two heads
constexpr int kFusedSlots = 8;      // LDS slots for the streaming wavefronts' attention states
// units per load block of the down rows: the attention output's hand-overs (partials,
// combine, the poll for o) queue behind this stretch, and with 3 instead of 4 units per block
// they gain more than the stream loses (measured at the 2.8B shape; 2 loses more).  The
// head_dim-128 instance keeps 4: at the 6.9B shape the stretch is 2.5 times longer and the
// hand-overs end well inside it.
constexpr int kFusedUDown = 3;
constexpr int kStageHalf = 12;      // float2 per streaming thread when staging one half of GELU(up): f_a <= 24 * 64 * (nw - 1)
// words of FusedLds::ctr: rendezvous of the streaming wavefronts; A rows of the up projection done;
// first / second half of GELU(up) complete everywhere (layer + 1)
enum { kCtrRendezvous = 0, kCtrRowsA = 1, kCtrHalfA = 2, kCtrHalfB = 3 };

// LDS of the fused kernel, in floats
struct FusedLds {
    unsigned y1, y2, ml, ol, xs, pq, pua, pub, pda, pdb, pc, pset, qs, kn, vn, wp, wm, wl, ctr, total;
};

static __host__ __device__ inline FusedLds fused_lds(const Dims &dm, int rows_qkv, int rows_up_a, int rows_up_b, int rows_h,
                                                     int nw)
{
    FusedLds L;
    const unsigned Kph = (unsigned)((dm.h + kChunk - 1) / kChunk * kChunk);
    const unsigned Kpf = (unsigned)((dm.f + kChunk - 1) / kChunk * kChunk);
    unsigned o = 0;
    auto take = [&](unsigned n) { unsigned at = o; o += (n + 3u) & ~3u; return at; };
    L.y1 = take(Kph); L.y2 = take(Kph); L.ml = take(Kpf); L.ol = take(Kph); L.xs = take(Kph);
    L.pq = take((unsigned)(rows_qkv * nw));
    L.pua = take((unsigned)(rows_up_a * nw)); L.pub = take((unsigned)(rows_up_b * nw));
    L.pda = take((unsigned)(rows_h * nw)); L.pdb = take((unsigned)(rows_h * nw)); L.pc = take((unsigned)(rows_h * nw));
    // one set of partial-sum slots; a second set follows (layers alternate, so that the
    // next layer's slots can be cleared while this layer's are still being read)
    L.pset = o - L.pq;
    o += L.pset;
    L.qs = take((unsigned)(kFusedSegs * dm.d));
    L.kn = take((unsigned)(kFusedSegs * dm.d / 2)); L.vn = take((unsigned)(kFusedSegs * dm.d / 2));
    L.wp = take((unsigned)(kFusedSegs * kFusedSlots * dm.d));
    L.wm = take(kFusedSegs * kFusedSlots); L.wl = take(kFusedSegs * kFusedSlots);
    L.ctr = take(4);
    L.total = o;
    return L;
}

struct FusedCtx {
    const StepParams *P;
    const LayerPtrs *ptrs;          // per-layer pointer table in device memory, or null: one block, P->w_single / kv_single
    float *lds;
    FusedLds L;
    int pos, nw;
    int q_begin, q_n, r_begin, r_n;
    int ua_begin, ua_n, ub_begin, ub_n;   // this workgroup's up-projection rows of the first half [0, f_a) and of the second
    int f_a;                              // columns of the first half of GELU(up)
    unsigned E0;                    // epoch base of this launch
    float *xt, *ot, *pt;            // tagged words: layer outputs [2][h], attention output [h], split-KV partials
};

__device__ __forceinline__ const __half *layer_weights(const FusedCtx &C, int layer)
{
    return C.ptrs ? C.ptrs->w[layer] : C.P->w_single;
}
__device__ __forceinline__ __half *layer_cache(const FusedCtx &C, int layer)
{
    return C.ptrs ? C.ptrs->kv[layer] : C.P->kv_single;
}

// First part of every layer, all wavefronts: the layer input into LDS - as it is
// (for the statistics) and multiplied by the weights of the two LayerNorms, in
// GEMV order (the inputs of the QKV and MLP-up rows).  The wavefronts take
// 64-element pieces of the vector in turn.  Layer 0 reads the step's input;
// later layers read the previous layer's output, which travels as tagged words:
// every wavefront re-reads its pieces until each word carries this layer's
// epoch - one round trip after the last workgroup stored its rows.  The caller
// places a workgroup barrier behind it.
__device__ __forceinline__ void fused_input(const FusedCtx &C, const __half *w, int layer, int tid)
{
    constexpr int JB = 8;                                  // pieces per wavefront and pass
    const StepParams &P = *C.P;
    const int h = P.dm.h, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int step = C.nw * 64;
    const __half *g1 = w + P.lay.ln1_g, *g2 = w + P.lay.ln2_g;
    float *xs = C.lds + C.L.xs, *y1 = C.lds + C.L.y1, *y2 = C.lds + C.L.y2;
    const float *xt = C.xt + 2 * (size_t)((layer + 1) & 1) * h;      // written by layer - 1
    const unsigned want = C.E0 + (unsigned)layer;
    PollGuard pg;
    pg.start(P.sync);
    for (int e0 = wave * 64; e0 < h; e0 += JB * step) {
        float ga[JB], gb[JB], xv[JB];
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int i = e0 + j * step + lane;
            ga[j] = 0.f; gb[j] = 0.f; xv[j] = 0.f;
            if (e0 + j * step < h) {
                ga[j] = __half2float(g1[i]);
                gb[j] = __half2float(g2[i]);
                if (layer == 0) xv[j] = __half2float(P.x_in[i]);
            }
        }
        if (layer > 0) {
            bool ok;
            do {
                ok = true;
#pragma unroll
                for (int j = 0; j < JB; ++j) {
                    if (e0 + j * step < h) {
                        const float2 wd = xwg_load2(xt + 2 * (e0 + j * step + lane));
                        xv[j] = wd.x;
                        ok = ok && __float_as_uint(wd.y) == want;
                    }
                }
                ok = __all(ok);
            } while (!ok && !pg.give_up());
        }
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int i = e0 + j * step + lane;
            if (e0 + j * step < h) {
                xs[i] = xv[j];
                y1[lds_perm(i)] = ga[j] * xv[j];
                y2[lds_perm(i)] = gb[j] * xv[j];
            }
        }
    }
}

// segments (head, rows) of this workgroup's attention share
template <int D>
struct FusedSegs {
    int n, s[kFusedSegs], row_lo[kFusedSegs], row_hi[kFusedSegs];
    __device__ __forceinline__ void init(const AttnCore<D> &ac)
    {
        n = 0;
#pragma unroll
        for (int k = 0; k < kFusedSegs; ++k) { s[k] = 0; row_lo[k] = 0; row_hi[k] = 0; }
        int sb = ac.r0;
#pragma unroll
        for (int k = 0; k < kFusedSegs; ++k) {
            if (sb < ac.r1) {
                int se;
                ac.segment(sb, s[k], se, row_lo[k], row_hi[k]);
                sb = se;
                n = k + 1;
            }
        }
    }
};

// One half of GELU(up), workspace -> registers -> LDS (GEMV order), shared by the streaming
// threads.  Always exactly UN load instructions per thread on one code path (threads past the
// end re-read the first words), so that the loads can sit in the middle of a stream of weight
// loads without upsetting the in-order load counter.  n: a multiple of 512.
template <int UN>
struct StagedPart {
    float2 v[UN];
    __device__ __forceinline__ void issue(const float *__restrict__ src, int n, int tid, int nt)
    {
        const int n2 = n >> 1;
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = tid + j * nt;
            v[j] = xwg_load2(src + 2 * (i2 < n2 ? i2 : 0));
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    __device__ __forceinline__ void commit(int n, float *dst, int tid, int nt) const
    {
        const int n2 = n >> 1;
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int i2 = tid + j * nt;
            if (i2 < n2) *reinterpret_cast<float2 *>(dst + lds_perm(i2 * 2)) = v[j];
        }
    }
};

// ---- wavefronts 1.. : stream --------------------------------------------------
template <int D>
__device__ __forceinline__ void fused_stream(const FusedCtx &C)
{
    using AC = AttnCore<D>;
    constexpr int NP = AC::NP;
    constexpr int UD = D == 128 ? kGemvU : kFusedUDown;
    const StepParams &P = *C.P;
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, fa = C.f_a, fb = f - C.f_a, L = P.n_layers, nw = C.nw, NS = nw - 1;
    float *lds = C.lds;
    float *y1 = lds + C.L.y1, *y2 = lds + C.L.y2, *ml = lds + C.L.ml, *ol = lds + C.L.ol;
    int *ctr = reinterpret_cast<int *>(lds) + C.L.ctr;
    const int n_tok = C.pos + 1;

    // The two stretches that follow a gap with nothing to stream start with more blocks in
    // registers than the usual two: the QKV rows behind the layer-input hand-over (two more,
    // requested when that hand-over begins), the first down columns behind the attention merges
    // (one more).  Measured: more, or earlier, only lengthens the queue the hand-over's own
    // loads wait in.
    GemvSpan<kGemvU, 2> gsQ;
    GemvSpan<UD, 1, true> gsDA;                           // down rows, columns [0, f_a)
    GemvSpan<UD, 0, true> gsDB;                           // down rows, columns [f_a, f)
    GemvSpan<kGemvU> gsUA, gsUB, gsC;
    {
        const int tid0 = opaque_thread_index();
        const __half *w0 = layer_weights(C, 0);
        gsQ.init(GemvSeg{w0 + P.lay.w_qkv + (size_t)C.q_begin * h, y1, h, C.q_n}, GemvSeg{w0 + P.lay.w_qkv, y1, h, 0},
                 w0, tid0, 0);
        gsQ.issue_first();
        gsQ.issue_second();
        gsQ.issue_more();
    }
    Tracer tr;
    tr.init(P, gsQ.wave, 0);

#pragma clang loop unroll(disable)
    for (int layer = 0; layer < L; ++layer) {
        const int tid = opaque_thread_index();
        const int lane = tid & 63, si = gsQ.wave - 1;
        const __half *w = layer_weights(C, layer);
        const __half *kv = layer_cache(C, layer);
        tr.select_layer(P, layer, L);
        // this layer's set of partial-sum slots
        const unsigned set = (unsigned)(layer & 1) * C.L.pset;
        float *pq = lds + C.L.pq + set, *pua = lds + C.L.pua + set, *pub = lds + C.L.pub + set;
        float *pda = lds + C.L.pda + set, *pdb = lds + C.L.pdb + set, *pc = lds + C.L.pc + set;
        tr.mark(1);
        fused_input(C, w, layer, tid);
        __syncthreads();                                   // S0: the layer input is in LDS
        tr.mark(3);

        gsUA.init(GemvSeg{w + P.lay.w_up + (size_t)C.ua_begin * h, y2, h, C.ua_n}, GemvSeg{w + P.lay.w_up, y2, h, 0},
                  w, tid, 0);
        gsQ.run(pq, [&] { gsUA.issue_first(); gsUA.issue_second(); });
        tr.mark(4);
        __syncthreads();                                   // S1: QKV rows done
        tr.mark(5);

        gsUB.init(GemvSeg{w + P.lay.w_up + (size_t)C.ub_begin * h, y2, h, C.ub_n}, GemvSeg{w + P.lay.w_up, y2, h, 0},
                  w, tid, 0);
        gsUA.run(pua, [&] { gsUB.issue_first(); gsUB.issue_second(); });
        // the A rows' partial sums are in LDS: the chain wavefront finishes them (nobody waits here)
        lds_signal(ctr + kCtrRowsA, lane);
        tr.mark(6);

        // attention share: the first K/V row is requested behind the last up-projection weights, the
        // second behind the barrier (both ahead of it and the chain wavefront's GELU(up) stores
        // and barrier arrival queue behind 36 MB instead of 18: measured)
        AC ac;
        ac.init(P, kv, n_tok, lane);
        FusedSegs<D> sg;
        sg.init(ac);
        u32x4 kA[NP], vA[NP], kB[NP], vB[NP];
        const int row0 = sg.row_lo[0] + si;
        gsUB.run(pub, [&] { ac.issue(kA, vA, sg.s[0], sg.n > 0 && row0 < sg.row_hi[0] ? row0 : -1); });
        tr.mark(7);
        __syncthreads();                                   // S2: up rows done; q and the new K/V rows staged
        tr.mark(10);
        ac.issue(kB, vB, sg.s[0], sg.n > 0 && row0 + NS < sg.row_hi[0] ? row0 + NS : -1);

        gsDA.init(GemvSeg{w + P.lay.w_down + (size_t)C.r_begin * f, ml, fa, C.r_n}, GemvSeg{w + P.lay.w_down, ml, fa, 0},
                  w, tid, 0, f);
#pragma unroll
        for (int k = 0; k < kFusedSegs; ++k) {
            if (k < sg.n) {
                const float *qs = lds + C.L.qs + k * D;
                const __half *kn = reinterpret_cast<const __half *>(lds + C.L.kn) + k * D;
                const __half *vn = reinterpret_cast<const __half *>(lds + C.L.vn) + k * D;
                const int s = sg.s[k], row_hi = sg.row_hi[k];
                int row = sg.row_lo[k] + si;
                if (k > 0) {
                    ac.issue(kA, vA, s, row < row_hi ? row : -1);
                    ac.issue(kB, vB, s, row + NS < row_hi ? row + NS : -1);
                }
                ac.reset();
                while (row < row_hi) {
                    ac.process(kA, vA, row, qs, kn, vn);
                    ac.issue(kA, vA, s, row + 2 * NS < row_hi ? row + 2 * NS : -1);
                    row += NS;
                    if (row >= row_hi) break;
                    ac.process(kB, vB, row, qs, kn, vn);
                    ac.issue(kB, vB, s, row + 2 * NS < row_hi ? row + 2 * NS : -1);
                    row += NS;
                }
                ac.wave_merge(lds + C.L.wp + k * kFusedSlots * D, lds + C.L.wm + k * kFusedSlots,
                              lds + C.L.wl + k * kFusedSlots, si);
            }
        }
        // The first half of GELU(up) is normally complete by now (its grid barrier was passed
        // behind the B rows and the attention): its copy is requested here, ahead of the first
        // down-projection weights, and written to LDS behind the workgroup barrier.
        StagedPart<kStageHalf> sm;
        const bool a_ready = lds_peek(ctr + kCtrHalfA, layer + 1);
        sm.issue(P.m, fa, tid - 64, NS * 64);
        gsDA.issue_first();
        gsDA.issue_second();
        tr.mark(13);
        __syncthreads();                                   // S3: attention states in LDS
        tr.mark(14);
        if (!a_ready) {                                    // (uniform) not yet complete when it was read: again
            lds_await(ctr + kCtrHalfA, layer + 1, P.sync);
            sm.issue(P.m, fa, tid - 64, NS * 64);
        }
        gsDA.issue_more();
        sm.commit(fa, ml, tid - 64, NS * 64);
        // staged: a rendezvous of the streaming wavefronts only (the chain wavefront is
        // already publishing the attention partials)
        lds_rendezvous(ctr + kCtrRendezvous, NS * (2 * layer + 1), P.sync, lane);
        tr.mark(17);

        // down projection, columns A; the second half of GELU(up) is copied meanwhile, the same way
        // (requested a few blocks into the stretch: its flag is posted just behind the attention)
        gsDB.init(GemvSeg{w + P.lay.w_down + (size_t)C.r_begin * f + fa, ml + fa, fb, C.r_n},
                  GemvSeg{w + P.lay.w_down, ml, fb, 0}, w, tid, 0, f);
        bool b_ready = false;
        gsDA.run(pda,
                 [&] {
                     b_ready = lds_peek(ctr + kCtrHalfB, layer + 1);
                     sm.issue(P.m + fa, fb, tid - 64, NS * 64);
                 },
                 [&] { gsDB.issue_first(); gsDB.issue_second(); });
        tr.mark(18);
        if (!b_ready) {
            lds_await(ctr + kCtrHalfB, layer + 1, P.sync);
            sm.issue(P.m + fa, fb, tid - 64, NS * 64);
        }
        sm.commit(fb, ml + fa, tid - 64, NS * 64);
        lds_rendezvous(ctr + kCtrRendezvous, NS * (2 * layer + 2), P.sync, lane);
        tr.mark(19);

        gsC.init(GemvSeg{w + P.lay.w_dense + (size_t)C.r_begin * h, ol, h, C.r_n}, GemvSeg{w + P.lay.w_dense, ol, h, 0},
                 w, tid, 0);
        gsDB.run(pdb, [&] { gsC.issue_first(); gsC.issue_second(); });
        tr.mark(20);
        {
            // the next layer's first QKV weights stream while the attention output is waited for
            // (nothing for the last layer: the loads re-read one block)
            const bool more = layer + 1 < L;
            const __half *wn = layer_weights(C, more ? layer + 1 : layer);
            gsQ.init(GemvSeg{wn + P.lay.w_qkv + (size_t)C.q_begin * h, y1, h, more ? C.q_n : 0},
                     GemvSeg{wn + P.lay.w_qkv, y1, h, 0}, wn, tid, 0);
            gsQ.issue_first();
            gsQ.issue_second();
        }
        __syncthreads();                                   // S4: down rows done; attention output staged
        tr.mark(21);
        gsC.run(pc);
        tr.mark(23);
        __syncthreads();                                   // S6: dense rows done
        tr.mark(24);
        gsQ.issue_more();                                  // (the last layer's re-read one block)
        {
            // the next layer's partial-sum slots (the chain wavefront still reads this layer's)
            float *nx = lds + C.L.pq + (C.L.pset - set);
            for (int i = tid - 64; i < (int)C.L.pset; i += NS * 64) nx[i] = 0.f;
        }
    }
}

// ---- wavefront 0 : chain ------------------------------------------------------
template <int D>
__device__ __forceinline__ void fused_chain(const FusedCtx &C)
{
    using AC = AttnCore<D>;
    const StepParams &P = *C.P;
    const Dims &dm = P.dm;
    const int h = dm.h, d = dm.d, r = dm.r, L = P.n_layers, nw = C.nw, NS = nw - 1;
    float *lds = C.lds;
    float *ol = lds + C.L.ol;
    const int pos = C.pos, n_tok = pos + 1;
    const int q_begin = C.q_begin, q_n = C.q_n, r_begin = C.r_begin, r_n = C.r_n;
    const int ua_begin = C.ua_begin, ua_n = C.ua_n, ub_begin = C.ub_begin, ub_n = C.ub_n;
    int *ctr = reinterpret_cast<int *>(lds) + C.L.ctr;

    // one grid barrier per hand-over that is not self-describing: q/k/v, and the two halves of GELU(up)
    GridBarrier b1, b2, b3;
    b1.init(P.sync, gridDim.x, 0);
    b2.init(P.sync, gridDim.x, 1);
    b3.init(P.sync, gridDim.x, 2);
    // the partial sums of a row sit in wavefront slots; only the streaming wavefronts fill them
    GemvSpan<kGemvU> rt;                                  // (row_total() only)
    rt.nw = nw;
    Tracer tr;
    tr.init(P, 0, 0);
    float x_r = 0.f;                                       // this lane's row of the residual stream

#pragma clang loop unroll(disable)
    for (int layer = 0; layer < L; ++layer) {
        const int tid = opaque_thread_index();
        const int lane = tid & 63;
        const __half *w = layer_weights(C, layer);
        __half *kv = layer_cache(C, layer);
        const LayerIO io = layer_io(P, layer);
        const bool last_layer = layer == L - 1;
        tr.select_layer(P, layer, L);
        const unsigned set = (unsigned)(layer & 1) * C.L.pset;   // this layer's partial-sum slots
        const float *pq = lds + C.L.pq + set, *pua = lds + C.L.pua + set, *pub = lds + C.L.pub + set;
        const float *pda = lds + C.L.pda + set, *pdb = lds + C.L.pdb + set, *pc = lds + C.L.pc + set;
        tr.mark(1);
        fused_input(C, w, layer, tid);
        tr.mark(2);
        CFPP_STAMP(P, lane == 0 && layer == L - 1, 7);
        __syncthreads();                                   // S0: the layer input is in LDS
        tr.mark(3);

        // what the epilogues need for this lane's first rows: requested now, used behind the GEMVs
        // (rcq: the constants (s, c) of two adjacent packed QKV rows; rcu: of one MLP-up row)
        const float4 *rcq = reinterpret_cast<const float4 *>(w + P.lay.rc_qkv) + (q_begin >> 1);
        const float2 *rcua = reinterpret_cast<const float2 *>(w + P.lay.rc_up) + ua_begin;
        const float2 *rcub = reinterpret_cast<const float2 *>(w + P.lay.rc_up) + ub_begin;
        const __half *bdn = w + P.lay.b_down, *bde = w + P.lay.b_dense;
        float4 rq0 = {0.f, 0.f, 0.f, 0.f};
        float2 rua0 = {0.f, 0.f}, rub0 = {0.f, 0.f};
        float bdn0 = 0.f, bde0 = 0.f;
        float2 cs0 = {1.f, 0.f};
        if (lane < q_n / 2) {
            const int p = q_begin + 2 * lane;
            const int i = p % d, c = (p / d) % 3;
            rq0 = rcq[lane];
            if (c < 2 && i < r) cs0 = P.rope[(size_t)pos * (r >> 1) + (i >> 1)];
        }
        if (lane < ua_n) rua0 = rcua[lane];
        if (lane < ub_n) rub0 = rcub[lane];
        if (lane < r_n) {
            bdn0 = __half2float(bdn[r_begin + lane]);
            bde0 = __half2float(bde[r_begin + lane]);
            if (layer == 0) x_r = __half2float(io.x16[r_begin + lane]);
        }
        AC ac;
        ac.init(P, kv, n_tok, lane);
        FusedSegs<D> sg;
        sg.init(ac);
        // mean and 1 / sqrt(variance + eps) of the layer input: both LayerNorms share them
        float mean, inv;
        {
            const float *xs = lds + C.L.xs;
            float sum = 0.f;
            for (int i = lane * 4; i < h; i += 256) {
                const float4 v = *reinterpret_cast<const float4 *>(xs + i);
                sum += (v.x + v.y) + (v.z + v.w);
            }
            mean = wave_sum(sum) / (float)h;
            float sq = 0.f;
            for (int i = lane * 4; i < h; i += 256) {
                const float4 v = *reinterpret_cast<const float4 *>(xs + i);
                const float d0 = v.x - mean, d1 = v.y - mean, d2 = v.z - mean, d3 = v.w - mean;
                sq += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
            }
            inv = 1.0f / sqrtf(wave_sum(sq) / (float)h + dm.ln_eps);
        }

        __syncthreads();                                   // S1: QKV rows done
        tr.mark(5);
        // QKV epilogue: one lane per pair of adjacent packed rows
        for (int pr = lane; pr < q_n / 2; pr += 64) {
            const int p = q_begin + 2 * pr;                 // packed row, even
            const int pdv = p / d, i = p - pdv * d;         // i even
            const int n = pdv / 3, c = pdv - 3 * n;
            const bool rotary = c < 2 && i < r;             // rotary pair (j, j + r/2)
            float4 rq = rq0;
            float2 cs = cs0;
            if (pr != lane) {
                rq = rcq[pr];
                if (rotary) cs = P.rope[(size_t)pos * (r >> 1) + (i >> 1)];
            }
            float v0 = inv * (rt.row_total(pq, 2 * pr) - mean * rq.x) + rq.y;
            float v1 = inv * (rt.row_total(pq, 2 * pr + 1) - mean * rq.z) + rq.w;
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
        b1.arrive_wave();
        b1.propagate();                                    // (waits for the arrival to return: this wavefront is idle until the A rows are done anyway)
        // first half of GELU(up): its rows' partial sums are in LDS once every streaming wavefront
        // has passed them (this wavefront alone waits); its grid barrier runs behind the B rows
        lds_await(ctr + kCtrRowsA, NS * (layer + 1), P.sync);
        tr.mark(6);
        for (int t = lane; t < ua_n; t += 64) {
            const float2 ru = t == lane ? rua0 : rcua[t];
            xwg_store(P.m + ua_begin + t, gelu_act(inv * (rt.row_total(pua, t) - mean * ru.x) + ru.y, dm.flags));
        }
        b2.arrive_wave();
        b1.wait_wave();                                    // q and the new K/V rows are complete everywhere
        tr.mark(7);
        {
            // stage them for the heads of this workgroup's attention share (lanes own elements lane, lane + 64)
            float qv[kFusedSegs][AC::NE];
            __half knv[kFusedSegs][AC::NE], vnv[kFusedSegs][AC::NE];
#pragma unroll
            for (int k = 0; k < kFusedSegs; ++k)
#pragma unroll
                for (int e = 0; e < AC::NE; ++e) {
                    const int i = lane + 64 * e;
                    const int ii = i < D ? i : 0, s = sg.s[k];
                    qv[k][e] = xwg_load(P.q + s * D + ii);
                    knv[k][e] = xwg_load_half(kv + kv_offset(dm, 0, P.b, s, ii, n_tok - 1));
                    vnv[k][e] = xwg_load_half(kv + kv_offset(dm, 1, P.b, s, ii, n_tok - 1));
                }
            b2.propagate();                                // (behind the loads just requested: its arrival is older)
#pragma unroll
            for (int k = 0; k < kFusedSegs; ++k)
#pragma unroll
                for (int e = 0; e < AC::NE; ++e) {
                    const int i = lane + 64 * e;
                    if (i < D) {
                        lds[C.L.qs + k * D + i] = qv[k][e];
                        reinterpret_cast<__half *>(lds + C.L.kn)[k * D + i] = knv[k][e];
                        reinterpret_cast<__half *>(lds + C.L.vn)[k * D + i] = vnv[k][e];
                    }
                }
        }
        tr.mark(8);
        __syncthreads();                                   // S2: up rows done
        tr.mark(10);
        for (int t = lane; t < ub_n; t += 64) {
            const float2 ru = t == lane ? rub0 : rcub[t];
            xwg_store(P.m + ub_begin + t, gelu_act(inv * (rt.row_total(pub, t) - mean * ru.x) + ru.y, dm.flags));
        }
        b3.arrive_wave();
        b2.wait_wave();                                    // the first half of GELU(up) is complete everywhere
        lds_post(ctr + kCtrHalfA, layer + 1, lane);
        b3.propagate();
        tr.mark(12);
        __syncthreads();                                   // S3: attention states in LDS
        tr.mark(14);
        CFPP_STAMP(P, lane == 0, 0);
        tr.mark(15);
        // attention: this workgroup's partials; the heads it combines; the whole
        // attention output into LDS once every head is combined
        const unsigned epoch = C.E0 + (unsigned)layer + 1u;
#pragma unroll
        for (int k = 0; k < kFusedSegs; ++k)
            if (k < sg.n)
                ac.publish_tagged(P, C.pt, epoch, sg.s[k], lds + C.L.wp + k * kFusedSlots * D,
                                  lds + C.L.wm + k * kFusedSlots, lds + C.L.wl + k * kFusedSlots, NS);
        b3.wait_wave();                                    // the second half of GELU(up) is complete everywhere
        lds_post(ctr + kCtrHalfB, layer + 1, lane);
#pragma unroll
        for (int k = 0; k < kFusedSegs; ++k)
            if (k < sg.n && ac.combines(sg.s[k])) ac.combine_tagged(P, C.pt, C.ot, epoch, sg.s[k]);
        CFPP_STAMP(P, lane == 0, 1);
        tr.mark(16);
        {
            // the attention output, tagged: the whole vector is re-read until every word
            // is current (one round trip after the last head was stored), then staged
            constexpr int SB = 20;
            const int hp = round_up_chunk(h);
            PollGuard pg;
            pg.start(P.sync);
            for (int base = 0; base < hp; base += SB * 64) {
                float2 wd[SB];
                bool ok;
                do {
#pragma unroll
                    for (int j2 = 0; j2 < SB; ++j2) {
                        const int i2 = base + j2 * 64 + lane;
                        wd[j2] = xwg_load2(C.ot + 2 * (i2 < h ? i2 : 0));
                    }
                    ok = true;
#pragma unroll
                    for (int j2 = 0; j2 < SB; ++j2)
                        ok = ok && (base + j2 * 64 + lane >= h || __float_as_uint(wd[j2].y) == epoch);
                    ok = __all(ok);
                } while (!ok && !pg.give_up());
#pragma unroll
                for (int j2 = 0; j2 < SB; ++j2) {
                    const int i2 = base + j2 * 64 + lane;
                    if (i2 < hp) ol[lds_perm(i2)] = i2 < h ? wd[j2].x : 0.f;
                }
            }
        }
        CFPP_STAMP(P, lane == 0, 3);
        tr.mark(17);
        CFPP_STAMP(P, lane == 0, 4);
        __syncthreads();                                   // S4: down rows done
        CFPP_STAMP(P, lane == 0, 5);
        tr.mark(20);
        float g_r = 0.f;
        if (lane < r_n) g_r = (rt.row_total(pda, lane) + rt.row_total(pdb, lane)) + bdn0;
        __syncthreads();                                   // S6: dense rows done
        tr.mark(24);
        CFPP_STAMP(P, lane == 0 && layer == L - 2, 6);
        if (lane < r_n) {
            const float a = rt.row_total(pc, lane) + bde0;
            const float res = (x_r + a) + g_r;
            x_r = res;
            if (last_layer) io.o16[r_begin + lane] = __float2half_rn(res);
            else xwg_store_tagged(C.xt + 2 * ((size_t)(layer & 1) * h + r_begin + lane), res, epoch);
        }
        tr.mark(25);
    }
    b1.finish_wave();
    b2.finish_wave();
    b3.finish_wave();
    // every workgroup has read E0 and finished its layers: the next launch gets fresh epochs
    if (blockIdx.x == 0 && threadIdx.x == 0)
        __hip_atomic_store(as_global(P.sync + kSyncEpoch), C.E0 + (unsigned)L + 1u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
}

template <int D>
__global__ void __launch_bounds__(kMaxThreads)
k_stack_fused(StepParams P, const LayerPtrs *__restrict__ ptrs)
{
    extern __shared__ __align__(16) float lds[];
    int pos;
    if (!read_pos(P, &pos)) return;
    const Dims &dm = P.dm;
    FusedCtx C;
    C.P = &P;
    C.ptrs = ptrs;
    C.lds = lds;
    C.nw = blockDim.x >> 6;
    C.L = fused_lds(dm, P.rows_qkv, P.rows_up_a, P.rows_up_b, P.rows_h, C.nw);
    C.pos = pos;
    const int g = blockIdx.x;
    C.q_begin = g * P.rows_qkv; C.q_n = max(0, min(P.rows_qkv, 3 * dm.h - C.q_begin));
    C.f_a = P.f_a;
    C.ua_begin = g * P.rows_up_a;          C.ua_n = max(0, min(P.rows_up_a, P.f_a - C.ua_begin));
    C.ub_begin = P.f_a + g * P.rows_up_b;  C.ub_n = max(0, min(P.rows_up_b, dm.f - C.ub_begin));
    C.r_begin = g * P.rows_h;   C.r_n = max(0, min(P.rows_h, dm.h - C.r_begin));
    // (only changed at the very end of a launch, behind the last barriers)
    C.E0 = __hip_atomic_load(as_global(P.sync + kSyncEpoch), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    C.xt = P.tagged;
    C.ot = P.tagged + 2 * (size_t)5 * dm.h;
    C.pt = P.tagged + 2 * (size_t)6 * dm.h;
    if (threadIdx.x < 4) reinterpret_cast<int *>(lds)[C.L.ctr + threadIdx.x] = 0;    // (a workgroup barrier follows in both roles)
    clear_partials(lds + C.L.pq, (int)C.L.pset, threadIdx.x);          // layer 0's partial-sum slots
    if (__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) == 0) fused_chain<D>(C);
    else fused_stream<D>(C);
}

// ---- host side -----------------------------------------------------------------
size_t fused_lds_bytes(const Dims &dm, const StepParams &P, int threads)
{
    return (size_t)fused_lds(dm, P.rows_qkv, P.rows_up_a, P.rows_up_b, P.rows_h, threads / 64).total * 4;
}

// grid >= heads (a workgroup's attention share then covers at most two heads),
// at most 64 rows of the h-row matrices per workgroup (one lane each in the
// chain wavefront), at most 8 streaming wavefronts, and rows of whole 512-weight
// units (the streaming wavefronts' balanced split)
bool fused_supported(const Dims &dm, const StepParams &P, int grid, int threads)
{
    return !(dm.flags & kFlagSequentialResidual) && grid >= dm.H && P.rows_h <= 64 && dm.h <= 4096 && dm.h % kChunk == 0 && dm.f % kChunk == 0 &&
           dm.f >= 2 * kChunk && P.f_a % kChunk == 0 && P.f_a > 0 && P.f_a < dm.f &&
           (size_t)P.f_a <= (size_t)2 * kStageHalf * 64 * (threads / 64 - 1) && threads / 64 - 1 <= kFusedSlots && threads >= 128 &&
           (dm.d == 64 || dm.d == 80 || dm.d == 128);
}

hipError_t launch_stack_fused(const StepParams &P, const LayerPtrs *ptrs, int grid, int threads, hipStream_t s)
{
    const size_t lds = fused_lds_bytes(P.dm, P, threads);
    switch (P.dm.d) {
    case 64: hipLaunchKernelGGL(k_stack_fused<64>, dim3(grid), dim3(threads), lds, s, P, ptrs); break;
    case 80: hipLaunchKernelGGL(k_stack_fused<80>, dim3(grid), dim3(threads), lds, s, P, ptrs); break;
    case 128: hipLaunchKernelGGL(k_stack_fused<128>, dim3(grid), dim3(threads), lds, s, P, ptrs); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t fused_occupancy(int head_dim, int threads, size_t lds_bytes, int *blocks_per_cu)
{
    switch (head_dim) {
    case 64: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_fused<64>, threads, lds_bytes);
    case 80: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_fused<80>, threads, lds_bytes);
    case 128: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_stack_fused<128>, threads, lds_bytes);
    }
    return hipErrorInvalidValue;
}

hipError_t prepare_fused_kernels(size_t lds_bytes)
{
    const int v = (int)lds_bytes;
    hipError_t e = hipFuncSetAttribute((const void *)k_stack_fused<64>, hipFuncAttributeMaxDynamicSharedMemorySize, v);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_stack_fused<80>, hipFuncAttributeMaxDynamicSharedMemorySize, v);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_stack_fused<128>, hipFuncAttributeMaxDynamicSharedMemorySize, v);
    return e;
}

}  // namespace cfpp
