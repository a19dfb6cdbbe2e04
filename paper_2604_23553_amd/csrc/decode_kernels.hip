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
// The same phase bodies are launched either as three kernels per block or as
// one persistent kernel per block (phases separated by a grid barrier); the
// whole-stack kernel is in fused_kernel.hip.  Sec. 2.3's graph mode wraps any
// of them.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "decode_blocks.h"
#include "attention_blocks.h"

namespace cfpp {

// ---------------------------------------------------------------------------
// Phase A.  LDS: y1[Kp] y2[Kp] part[(rows_qkv + rows_up) * nw] red[16]
template <class Sync>
__device__ __forceinline__ void phase_a(const StepParams &P, const __half *__restrict__ w, __half *__restrict__ kv,
                                        int layer, int pos, float *lds, Sync &sync)
{
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, d = dm.d, r = dm.r;
    const int tid = opaque_thread_index(), nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(h);
    float *y1 = lds, *y2 = lds + Kp, *part = lds + 2 * Kp;
    float *red = part + (P.rows_qkv + P.rows_up) * (nt >> 6);
    const LayerIO io = layer_io(P, layer);

    // weights first: they depend on nothing, so their loads overlap the wait for x
    const int q_begin = g * P.rows_qkv, q_n = (P.parts & kPartQkv) ? max(0, min(P.rows_qkv, 3 * h - q_begin)) : 0;
    const int u_begin = g * P.rows_up, u_n = (P.parts & kPartUp) ? max(0, min(P.rows_up, f - u_begin)) : 0;
    GemvSpan<kGemvU> gs;
    gs.init(GemvSeg{w + P.lay.w_qkv + (size_t)q_begin * h, y1, h, q_n},
            GemvSeg{w + P.lay.w_up + (size_t)u_begin * h, y2, h, u_n}, w, tid);
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

    LnPair ln;
    ln.load(P, w, io, tid);
    if constexpr (Sync::kInputsReady) gs.issue_first();    // x is already on its way: it returns first
    gs.issue_second();
    ln.finish(P, y1, y2, red, tid);
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
            xwg_store(P.m + u_begin + t, gelu_act(gs.row_total(part, q_n + t) + b, dm.flags));
        }
    }
    tr.mark(6);
    sync.arrive();
}

// ---------------------------------------------------------------------------
// Split-KV decode attention over this workgroup's share of the cache, all
// wavefronts taking rows round-robin.
// scr: nw*(D+2) + 4 + 2*D floats of LDS.
// pre(): called once, after the first row of already-cached K/V has been
// requested and before anything written during this launch (q, the new token's
// K/V) is read.  early(): called once, when every K/V load of the first two rows
// has been requested (the caller requests what it wants in flight during the
// arithmetic).  mid(): called once, ahead of the first workgroup barrier (the
// caller finishes staging its LDS vectors there).  tail(): called once, when the
// last K/V rows have been consumed, ahead of the last merges.
template <int D, class Pre, class Early, class Mid, class Tail>
__device__ __forceinline__ void attn_share(const StepParams &P, const __half *__restrict__ kv, int n_tok,
                                           float *scr, int tid, Pre &&pre, Early &&early, Mid &&mid, Tail &&tail,
                                           Tracer &tr)
{
    using AC = AttnCore<D>;
    constexpr int NP = AC::NP;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = blockDim.x >> 6;
    float *wp = scr, *wm = scr + nw * D, *wl = wm + nw;
    float *qs = wl + nw + 4;                               // this head's query
    __half *kn = reinterpret_cast<__half *>(qs + D);       // the new token's K and V rows of this head
    __half *vn = kn + D;
    AC ac;
    ac.init(P, kv, n_tok, lane);

    if (ac.r0 >= ac.r1 || !(P.parts & kPartAttention)) {   // no rows for this workgroup, or no attention in this launch
        pre();
        early();
        mid();
        __syncthreads();
        tail();
        return;
    }

    // Order of the requests: first row of cached K/V (needs nothing), then -
    // behind the caller's wait - the small vectors written during this launch,
    // then the second row and the caller's next weights.  The small loads return
    // while the bulk behind them is still streaming.
    u32x4 kA[NP], vA[NP], kB[NP], vB[NP];
    HeadStage<D> hst;
    bool first = true;
    {
        int s, se, row_lo, row_hi;
        ac.segment(ac.r0, s, se, row_lo, row_hi);
        const int row = row_lo + wave;
        ac.issue(kA, vA, s, row < row_hi ? row : -1);
        pre();
        hst.issue(P, kv, s, n_tok, tid);
        ac.issue(kB, vB, s, row + nw < row_hi ? row + nw : -1);
        early();
        hst.commit(qs, kn, vn, tid);
        mid();
    }

    for (int sb = ac.r0; sb < ac.r1;) {
        int s, se, row_lo, row_hi;
        ac.segment(sb, s, se, row_lo, row_hi);
        int row = row_lo + wave;
        if (!first) {
            ac.issue(kA, vA, s, row < row_hi ? row : -1);
            hst.issue(P, kv, s, n_tok, tid);
            ac.issue(kB, vB, s, row + nw < row_hi ? row + nw : -1);
            hst.commit(qs, kn, vn, tid);
        }
        first = false;
        __syncthreads();
        ac.reset();
        const bool last_seg = se == ac.r1;
        // Two rows are in flight per wavefront; a register set is refilled as soon
        // as its row is consumed.  The sets swap roles instead of being copied: a
        // copy of a set whose loads are still in flight would have to wait for them.
        // (no exit between the two halves: with one, the load counter's model loses track of
        // which set is older and every wait drains the queue)
        while (row < row_hi) {
            ac.process(kA, vA, row, qs, kn, vn);
            ac.issue(kA, vA, s, row + 2 * nw < row_hi ? row + 2 * nw : -1);
            if (row + nw < row_hi) ac.process(kB, vB, row + nw, qs, kn, vn);
            ac.issue(kB, vB, s, row + 3 * nw < row_hi ? row + 3 * nw : -1);
            row += 2 * nw;
        }

        // The first wavefront alone merges the wavefronts' states, publishes the
        // workgroup's partial and, if it was the last of the head, combines the head;
        // the others go on after one barrier.
        if (last_seg && wave != 0) tail();
        ac.wave_merge(wp, wm, wl, wave);
        tr.mark(14);
        __syncthreads();
        if (wave == 0) {
            ac.publish(P, s, wp, wm, wl, nw);
            if (!CFPP_SKIPPED(P, 8)) {
                xwg_wait_stores();
                tr.mark(15);
                if (last_seg) tail();
                ac.count_and_combine(P, s);
            } else if (last_seg) {
                tail();
            }
        }
        if (!last_seg) __syncthreads();                    // the scratch is reused by the next head
        tr.mark(16);
        sb = se;
    }
}

// Phase B.  LDS: m[Kp_f] part[rows_h*nw] scr[nw*(D+2)+4+2*D]
template <int D, class Sync>
__device__ __forceinline__ void phase_b(const StepParams &P, const __half *__restrict__ w,
                                        const __half *__restrict__ kv, int pos, float *lds, Sync &sync)
{
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, tid = opaque_thread_index(), nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(f);
    float *ml = lds, *part = lds + Kp;
    float *scr = part + P.rows_h * (nt >> 6);
    const int r_begin = g * P.rows_h, r_n = (P.parts & kPartDown) ? max(0, min(P.rows_h, h - r_begin)) : 0;
    GemvSpan<kGemvUDown> gs;
    gs.init(GemvSeg{w + P.lay.w_down + (size_t)r_begin * f, ml, f, r_n}, GemvSeg{w + P.lay.w_down, ml, f, 0}, w, tid, kShare0AfterAttention);
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

// Phase C.  LDS: o[Kp_h] part[rows_h*nw]
template <class Sync>
__device__ __forceinline__ void phase_c(const StepParams &P, const __half *__restrict__ w, int layer,
                                        float *lds, Sync &sync)
{
    const Dims &dm = P.dm;
    const int h = dm.h, tid = opaque_thread_index(), nt = blockDim.x, g = blockIdx.x;
    const int Kp = round_up_chunk(h);
    float *ol = lds, *part = lds + Kp;
    const LayerIO io = layer_io(P, layer);
    const int r_begin = g * P.rows_h, r_n = max(0, min(P.rows_h, h - r_begin));
    const bool dense = P.parts & kPartDense, down = P.parts & kPartDown;   // branches this launch adds to the residual
    GemvSpan<kGemvU> gs;
    gs.init(GemvSeg{w + P.lay.w_dense + (size_t)r_begin * h, ol, h, dense ? r_n : 0}, GemvSeg{w + P.lay.w_dense, ol, h, 0}, w, tid);
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
        g0 = down ? xwg_load(P.g + r_begin + item0) : 0.f;
    }
    so.commit(h, ol, tid);
    __syncthreads();
    tr.mark(22);
    gs.run(part);
    tr.mark(23);
    __syncthreads();
    for (int t = item0; t < r_n; t += nt) {
        const bool pre = t == item0;
        const float a = dense ? gs.row_total(part, t) + (pre ? bd0 : __half2float(bd[r_begin + t])) : 0.f;
        const float res = ((pre ? x0 : load_x(io, r_begin + t)) + a) + (pre ? g0 : (down ? xwg_load(P.g + r_begin + t) : 0.f));
        if (io.o16) io.o16[r_begin + t] = __float2half_rn(res);
        else xwg_store(io.o32 + r_begin + t, res);
    }
    tr.mark(24);
    sync.arrive();
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

// The attention of several sequences in one launch.  P holds the parameters of
// the first sequence; sequence i follows at the workspace's usual strides.
// Every workgroup works out the split from the positions in device memory:
// workgroups are dealt in proportion to the cache rows of each sequence, at
// least one each (grid >= nb).
constexpr int kAttnBatchMax = 8;
template <int D>
__global__ void __launch_bounds__(kMaxThreads)
k_attention_batched(StepParams P, int nb, const __half *w, const __half *kv)
{
    extern __shared__ __align__(16) float lds[];
    constexpr int PPW = AttnShape<D>::PPW;
    const Dims &dm = P.dm;
    // (cache rows per head: every head of a sequence has the same number, so the shares are
    // the same as by rows of all heads, and spare * sum stays below 2^32: max_seq <= 2^20)
    unsigned rows[kAttnBatchMax];
    unsigned total = 0;
    bool ok = true;
#pragma unroll
    for (int i = 0; i < kAttnBatchMax; ++i) {
        rows[i] = 0;
        if (i < nb) {
            const int p = P.pos[i];
            ok = ok && p >= 0 && p < dm.max_seq;
            rows[i] = (unsigned)((p + 1 + PPW - 1) / PPW);
            total += rows[i];
        }
    }
    if (!ok) {
        if (threadIdx.x == 0 && blockIdx.x == 0)
            __hip_atomic_store(&P.sync[kSyncErr], (unsigned)kErrBadPos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    const unsigned spare = gridDim.x - (unsigned)nb;
    const int g = blockIdx.x;
    unsigned before = 0;
    int mine = -1, g0 = 0, g1 = 0;
    int lo = 0;
#pragma unroll
    for (int i = 0; i < kAttnBatchMax; ++i) {
        if (i < nb) {
            before += rows[i];
            const int hi = (int)(spare * before / total) + i + 1;
            if (g >= lo && g < hi) { mine = i; g0 = lo; g1 = hi; }
            lo = hi;
        }
    }
    if (mine < 0) return;
    StepParams Q = P;
    Q.b = P.b + mine * P.attn_bstep;
    Q.pos = P.pos + mine;
    Q.q = P.q + (size_t)mine * dm.h;
    Q.o = P.o + (size_t)mine * dm.h;
    Q.m = P.m + (size_t)mine * dm.f;
    Q.part = P.part + (size_t)mine * dm.H * P.part_slots * (dm.d + 2);
    Q.seg_cnt = P.seg_cnt + (size_t)mine * dm.H;
    Q.attn_g0 = g0;
    Q.attn_G = g1 - g0;
    Q.parts = kPartAttention;
    // the attention alone: nothing of the MLP-down stretch that shares phase B with it
    // (no GELU(up) staged into LDS, no weights requested)
    Tracer tr;
    tr.init(Q, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), 16);
    attn_share<D>(Q, kv, *Q.pos + 1, lds, opaque_thread_index(), [] {}, [] {}, [] {}, [] {}, tr);
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

// the attention of one sequence alone (the batched path runs the projections for all sequences at once)
hipError_t launch_attention_only(StepParams P, const __half *w, const __half *kv, int grid, int threads, hipStream_t s)
{
    P.parts = kPartAttention;
    const size_t lds = (size_t)P.lds_floats * 4;
    switch (P.dm.d) {
    case 64: hipLaunchKernelGGL(k_phase_b<64>, dim3(grid), dim3(threads), lds, s, P, w, kv); break;
    case 80: hipLaunchKernelGGL(k_phase_b<80>, dim3(grid), dim3(threads), lds, s, P, w, kv); break;
    case 128: hipLaunchKernelGGL(k_phase_b<128>, dim3(grid), dim3(threads), lds, s, P, w, kv); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_attention_batched(StepParams P, int nb, const __half *w, const __half *kv, int grid, int threads,
                                    hipStream_t s)
{
    if (nb < 1 || nb > kAttnBatchMax || grid < nb) return hipErrorInvalidValue;
    const size_t lds = (size_t)P.lds_floats * 4;
    switch (P.dm.d) {
    case 64: hipLaunchKernelGGL(k_attention_batched<64>, dim3(grid), dim3(threads), lds, s, P, nb, w, kv); break;
    case 80: hipLaunchKernelGGL(k_attention_batched<80>, dim3(grid), dim3(threads), lds, s, P, nb, w, kv); break;
    case 128: hipLaunchKernelGGL(k_attention_batched<128>, dim3(grid), dim3(threads), lds, s, P, nb, w, kv); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
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

hipError_t persistent_occupancy(int head_dim, int threads, size_t lds_bytes, int *blocks_per_cu)
{
    switch (head_dim) {
    case 64: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_block_persistent<64>, threads, lds_bytes);
    case 80: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_block_persistent<80>, threads, lds_bytes);
    case 128: return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, k_block_persistent<128>, threads, lds_bytes);
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
    CFPP_TRY(hipFuncSetAttribute((const void *)k_attention_batched<64>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_attention_batched<80>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_attention_batched<128>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_block_persistent<64>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_block_persistent<80>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    CFPP_TRY(hipFuncSetAttribute((const void *)k_block_persistent<128>, hipFuncAttributeMaxDynamicSharedMemorySize, v));
    return hipSuccess;
}

}  // namespace cfpp
