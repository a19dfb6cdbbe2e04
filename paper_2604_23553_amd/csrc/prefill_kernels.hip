// Prompt processing with the weights read once per pass over up to kPfMaxRows
// tokens (the paper names a prefill phase beside its fused decode kernel, Sec. 4.2;
// what is computed is the block of Sec. 2.2 applied to every prompt token with
// causal attention).  With hundreds of tokens the four projections are dense
// contractions - tokens x K activations times K x rows weights - and run as
// LDS-tiled GEMMs on the matrix cores (v_mfma_f32_32x32x16_f16); the attention of
// a pass reads the cache rows its own QKV launch appended.
//
//   k_pf_ln     : per token: mean, 1/sigma, and gamma_1 * x, gamma_2 * x as two fp16
//                 planes each (head + remainder: y = hi + lo to ~2^-22, so that the
//                 fp16 matrix instruction reproduces the fp32 product to rounding)
//   k_pf_gemm<> : C[tokens][n] = A[tokens][K] . W[n][K]^T, both operands K-major,
//                 fp32 accumulation, two instructions per tile (head, remainder);
//                 the epilogue completes the LayerNorm from the packing's row
//                 constants (QKV, MLP-up) and does what follows the product:
//                 rotary + cache append + q | GELU -> planes | residual sums
//   k_pf_attn<> : causal attention of a block of 16 queries of one head over the cache,
//                 keys in LDS tiles of 64 positions, both products on the matrix
//                 cores (v_mfma_f32_16x16x16_f16), online softmax in fp32
//
// Every sum has a fixed order: one bit pattern per build and pass size.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "device_utils.h"
#include "prefill_params.h"

namespace cfpp {

typedef _Float16 pf_f16x8 __attribute__((ext_vector_type(8)));
typedef float pf_f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void pf_split(float v, __half &hi, __half &lo)
{
    hi = __float2half_rn(v);
    lo = __float2half_rn(v - __half2float(hi));
}

__device__ __forceinline__ unsigned pf_pack2(float a, float b)
{
    return (unsigned)__half_as_ushort(__float2half_rn(a)) | (unsigned)__half_as_ushort(__float2half_rn(b)) << 16;
}

// ---------------------------------------------------------------------------
// One wavefront per scratch row, four rows per workgroup, no barrier: a lane holds the
// row's elements 4 (lane + 64 j) .. + 3, j < h / 256 (hidden: a multiple of 128, at most
// 4096; with an odd number of 128s the upper half of the lanes sits out the last j).
// Rows past the pass's tokens get zero planes (their products are never stored).
constexpr int kPfLnVec = 16;           // float4 per lane: hidden <= 4096
__global__ void __launch_bounds__(256) k_pf_ln(PfParams P)
{
    const Dims &dm = P.dm;
    const int h = dm.h, lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
    __half *y1h = P.y1h + (size_t)row * h, *y1l = P.y1l + (size_t)row * h;
    __half *y2h = P.y2h + (size_t)row * h, *y2l = P.y2l + (size_t)row * h;
    const int nv = h >> 2;                                 // groups of 4 elements in a row
    if (row >= P.n_rows) {
        const uint2 z = {0u, 0u};
        for (int g = lane; g < nv; g += 64) {
            *reinterpret_cast<uint2 *>(y1h + 4 * g) = z; *reinterpret_cast<uint2 *>(y1l + 4 * g) = z;
            *reinterpret_cast<uint2 *>(y2h + 4 * g) = z; *reinterpret_cast<uint2 *>(y2l + 4 * g) = z;
        }
        return;
    }
    f32x4 x[kPfLnVec];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kPfLnVec; ++j) {
        const int g = lane + 64 * j;
        x[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (g < nv) {
            if (P.layer == 0) {
                const uint2 w = *reinterpret_cast<const uint2 *>(P.x_in + (size_t)row * h + 4 * g);
                const float2 a = unpack_h2(w.x), b = unpack_h2(w.y);
                x[j] = f32x4{a.x, a.y, b.x, b.y};
                *reinterpret_cast<f32x4 *>(P.xres + (size_t)row * h + 4 * g) = x[j];
            } else {
                x[j] = *reinterpret_cast<const f32x4 *>(P.xres + (size_t)row * h + 4 * g);
            }
        }
        s += (x[j][0] + x[j][1]) + (x[j][2] + x[j][3]);
    }
    const float mean = wave_sum(s) / (float)h;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < kPfLnVec; ++j) {
        if (lane + 64 * j < nv) {
            const f32x4 dl = x[j] - mean;
            q += (dl[0] * dl[0] + dl[1] * dl[1]) + (dl[2] * dl[2] + dl[3] * dl[3]);
        }
    }
    const float inv = 1.0f / sqrtf(wave_sum(q) / (float)h + dm.ln_eps);
    if (lane == 0) P.stats[row] = float2{mean, inv};
    const __half *g1 = P.w + P.lay.ln1_g, *g2 = P.w + P.lay.ln2_g;
#pragma unroll
    for (int j = 0; j < kPfLnVec; ++j) {
        const int g = lane + 64 * j;
        if (g < nv) {
            const uint2 w1 = *reinterpret_cast<const uint2 *>(g1 + 4 * g), w2 = *reinterpret_cast<const uint2 *>(g2 + 4 * g);
            const float2 a1 = unpack_h2(w1.x), b1 = unpack_h2(w1.y), a2 = unpack_h2(w2.x), b2 = unpack_h2(w2.y);
            const float ga[4] = {a1.x, a1.y, b1.x, b1.y}, gb[4] = {a2.x, a2.y, b2.x, b2.y};
            __half h1[4], l1[4], h2[4], l2[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pf_split(x[j][e] * ga[e], h1[e], l1[e]);
                pf_split(x[j][e] * gb[e], h2[e], l2[e]);
            }
            *reinterpret_cast<uint2 *>(y1h + 4 * g) = *reinterpret_cast<const uint2 *>(h1);
            *reinterpret_cast<uint2 *>(y1l + 4 * g) = *reinterpret_cast<const uint2 *>(l1);
            *reinterpret_cast<uint2 *>(y2h + 4 * g) = *reinterpret_cast<const uint2 *>(h2);
            *reinterpret_cast<uint2 *>(y2l + 4 * g) = *reinterpret_cast<const uint2 *>(l2);
        }
    }
}

// ---------------------------------------------------------------------------
// What follows a product, for the element (row = token, col = output feature) with the
// K-sum `val`, in two steps because a rotation pair of the packed QKV order sits in two
// adjacent columns (the first one even) and each needs the other's completed value.
enum { kPfQkv = 0, kPfUp = 1, kPfDense = 2, kPfDown = 3 };

// the LayerNorm, completed: inv (W (gamma x) - mu s) + c, with c = W beta + b from the packing
template <int EPI>
__device__ __forceinline__ float pf_complete(const PfParams &P, int row, int col, float val)
{
    if (EPI == kPfQkv || EPI == kPfUp) {
        const float2 rc = reinterpret_cast<const float2 *>(P.w + (EPI == kPfQkv ? P.lay.rc_qkv : P.lay.rc_up))[col];
        const float2 st = P.stats[row];
        val = (val - st.x * rc.x) * st.y + rc.y;
    }
    return val;
}

// other: the completed value of the neighbouring column (col ^ 1) of the same row (QKV only)
template <int EPI>
__device__ __forceinline__ void pf_store(const PfParams &P, int row, int col, float val, float other)
{
    const Dims &dm = P.dm;
    const int h = dm.h;
    if (EPI == kPfQkv) {
        const int pd = col / dm.d, i = col - pd * dm.d, nh = pd / 3, c = pd - 3 * nh;
        int dim = i;
        if (c < 2 && i < dm.r) {
            const float2 cs = P.rope[(size_t)(P.pos0 + row) * (dm.r >> 1) + (i >> 1)];
            if (i & 1) { val = val * cs.x + other * cs.y; dim = (i >> 1) + (dm.r >> 1); }
            else { val = val * cs.x - other * cs.y; dim = i >> 1; }
        }
        if (c == 0) P.q[(size_t)row * h + nh * dm.d + dim] = val;
        else P.kv[kv_offset(dm, c - 1, P.b, nh, dim, P.pos0 + row)] = __float2half_rn(val);
    } else if (EPI == kPfUp) {
        __half hi, lo;
        pf_split(gelu_act(val, dm.flags), hi, lo);
        P.mh[(size_t)row * dm.f + col] = hi;
        P.ml[(size_t)row * dm.f + col] = lo;
    } else if (EPI == kPfDense) {
        P.xnext[(size_t)row * h + col] = P.xres[(size_t)row * h + col] + (val + __half2float(P.w[P.lay.b_dense + col]));
    } else {
        const float res = P.xnext[(size_t)row * h + col] + (val + __half2float(P.w[P.lay.b_down + col]));
        if (P.layer == P.n_layers - 1) P.out[(size_t)row * h + col] = __float2half_rn(res);
        else P.xnext[(size_t)row * h + col] = res;
    }
}

// ---------------------------------------------------------------------------
// GEMM.  Workgroup: 256 threads = 2 x 2 wavefronts, tile BM tokens x 128 output
// features, K in steps of BK through double-buffered LDS.  BM 128 with BK 32, or - when
// that is what brings several workgroups onto every CU: while one waits for LDS another
// multiplies - BM 64 with BK 64 (whole 128-byte lines per row and step).  Rows sit
// BK + 8 halves apart: the 16-byte fragment reads of 16 consecutive rows hit 16
// different groups of four banks.  A wavefront owns BM/2 x 64 of the tile: BM/64 x 2
// instruction tiles of 32 x 32 (v_mfma_f32_32x32x16_f16: a lane supplies 8
// consecutive K values of its row), each fed the head and the remainder plane of the
// activations; consecutive instructions go to different accumulators.
// Tiles are dealt so that consecutive numbers run on the same XCD (workgroup i runs on
// XCD i % 8).  An unsplit product numbers the token tiles fastest: the workgroups of an
// XCD that run together share a few weight tiles, and each XCD reads its part of the
// weights once; a split one numbers the weight tiles fastest (measured, a few percent each).
// splits > 1: workgroup z of a tile takes the z-th part of K and leaves its sums in
// part[z][row][col] (rows of whole token tiles); k_pf_reduce adds the parts in order and finishes.
// Otherwise the tile goes through LDS once more (fp32, completed LayerNorm, rotated
// pairs), and what follows the product is stored from there in whole 16-byte pieces
// along the destination's own order: the instruction's output layout would scatter
// 2- and 4-byte pieces, which cost a quarter of the kernel.
constexpr int kPfEpiStride = kPfTile + 8;                  // floats between rows of the staged tile: rows 4 apart sit 32 banks apart

template <int BM, int BK>
constexpr int pf_gemm_lds_bytes()
{
    constexpr int steps = (4 * BM + 2 * kPfTile) * (BK + 8) * 2, staged = BM * kPfEpiStride * 4;
    return steps > staged ? steps : staged;
}

template <int EPI, int BM, int BK>
__global__ void __launch_bounds__(256) k_pf_gemm(PfParams P, const __half *__restrict__ Ah, const __half *__restrict__ Al,
                                                  const __half *__restrict__ W, int K, int N, int splits, float *part)
{
    constexpr int kPfStride = BK + 8;                      // halves between rows in LDS
    constexpr int PR = BK / 8, RP = 256 / PR;              // 16-byte pieces of a row; rows the 256 threads cover at once
    constexpr int MT = BM / 64;                            // instruction tiles of a wavefront along the tokens
    constexpr int NA = BM / RP, NW = kPfTile / RP;         // 16-byte pieces per thread and step: of an activation plane, of the weights
    extern __shared__ __align__(16) __half pf_lds[];       // [buffer][head, remainder][BM][stride], then [buffer][128][stride]
    __half (*sA)[2][BM * kPfStride] = reinterpret_cast<__half (*)[2][BM * kPfStride]>(pf_lds);
    __half (*sW)[kPfTile * kPfStride] = reinterpret_cast<__half (*)[kPfTile * kPfStride]>(pf_lds + 4 * BM * kPfStride);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int mt = (P.n_rows + BM - 1) / BM, total = (N / kPfTile) * mt * splits;
    const int per_xcd = (total + 7) >> 3;
    const int v = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (v >= total) return;                               // (whole workgroup)
    const int tiles = total / splits, z = v / tiles, tile = v - z * tiles;
    const int ntn = N / kPfTile;
    const int m0 = (splits > 1 ? tile / ntn : tile % mt) * BM, n0 = (splits > 1 ? tile % ntn : tile / mt) * kPfTile;
    const int kb = (K / splits) * z, nk = K / splits / BK;
    // global -> LDS: RP rows x BK halves are 256 pieces of 16 bytes, one per thread
    const int lrow = tid / PR, lk = (tid % PR) * 8;
    const __half *pa_h = Ah + (size_t)(m0 + lrow) * K + kb + lk, *pa_l = Al + (size_t)(m0 + lrow) * K + kb + lk;
    const __half *pw = W + (size_t)(n0 + lrow) * K + kb + lk;
    const size_t rstep = (size_t)RP * K;
    const int st = lrow * kPfStride + lk;
    // Three register sets hold the tiles of the next three steps while the current one is
    // multiplied out of LDS: a global load has three steps to arrive.  A thread moves NP pieces of
    // 16 bytes per step (its rows of the head plane, of the remainder plane, of the weights).
    // A step is cut into its BK / 16 instruction groups, and each group requests its share of the
    // tile three steps ahead, reads its fragments, issues its matrix instructions and writes its
    // share of the next tile to the other LDS buffer: the vector-memory pipe, the LDS and the matrix
    // pipe then work side by side instead of one after the other (timestamps of a step that did
    // these four things in turn: 290 + 590 + 350 + 240 ns, each phase alone on its unit while both
    // workgroups of a CU were in the same phase).  No conditions around the loads (steps past the
    // end re-read the last tile and are not multiplied).
    constexpr int NP = 2 * NA + NW, KS = BK / 16, PK = NP / KS;
    static_assert(NP % KS == 0, "the pieces of a step divide evenly over its instruction groups");
    struct Regs { u32x4 p[NP]; } g0, g1, g2;
    const int nk1 = nk - 1;
    auto gsrc = [&](int i) { return i < NA ? pa_h + i * rstep : i < 2 * NA ? pa_l + (i - NA) * rstep : pw + (i - 2 * NA) * rstep; };
    auto ldst = [&](int buf, int i) {
        __half *base = i < NA ? &sA[buf][0][i * RP * kPfStride] : i < 2 * NA ? &sA[buf][1][(i - NA) * RP * kPfStride] : &sW[buf][(i - 2 * NA) * RP * kPfStride];
        return reinterpret_cast<u32x4 *>(base + st);
    };
    auto fetch = [&](Regs &g, int kt) {
        const int k0 = (kt < nk1 ? kt : nk1) * BK;
#pragma unroll
        for (int i = 0; i < NP; ++i) g.p[i] = load16(gsrc(i) + k0);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto stash = [&](const Regs &g, int buf) {
#pragma unroll
        for (int i = 0; i < NP; ++i) *ldst(buf, i) = g.p[i];
    };
    pf_f32x16 acc[MT][2];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
    // fragment of this lane: row lane % 32 of an instruction tile, halves 8 * (lane / 32) .. + 7 of a step of 16
    const int fr = lane & 31, fk = (lane >> 5) * 8;
    const int a_off = (wm * 32 * MT + fr) * kPfStride + fk, w_off = (wn * 64 + fr) * kPfStride + fk;
    // one step: tile `kt_next` into gn, the tile in LDS buffer `buf` multiplied (if `live`), gs into the other buffer
    auto step = [&](Regs &gn, int kt_next, int buf, bool live, const Regs &gs) {
        const int k0 = (kt_next < nk1 ? kt_next : nk1) * BK;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int i = ks * PK; i < (ks + 1) * PK; ++i) gn.p[i] = load16(gsrc(i) + k0);
            if (live) {
                pf_f16x8 ah[MT], al[MT], wf[2];
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    ah[t] = *reinterpret_cast<const pf_f16x8 *>(&sA[buf][0][a_off + t * 32 * kPfStride + ks * 16]);
                    al[t] = *reinterpret_cast<const pf_f16x8 *>(&sA[buf][1][a_off + t * 32 * kPfStride + ks * 16]);
                }
#pragma unroll
                for (int t = 0; t < 2; ++t) wf[t] = *reinterpret_cast<const pf_f16x8 *>(&sW[buf][w_off + t * 32 * kPfStride + ks * 16]);
#pragma unroll
                for (int a = 0; a < MT; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[a], wf[b], acc[a][b], 0, 0, 0);
#pragma unroll
                for (int a = 0; a < MT; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al[a], wf[b], acc[a][b], 0, 0, 0);
            }
#pragma unroll
            for (int i = ks * PK; i < (ks + 1) * PK; ++i) *ldst(buf ^ 1, i) = gs.p[i];
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };
    fetch(g0, 0);
    fetch(g1, 1);
    fetch(g2, 2);
    stash(g0, 0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 3) {                  // tile t sits in LDS buffer t % 2
        const int b0 = kt & 1;
        step(g0, kt + 3, b0, true, g1);
        step(g1, kt + 4, b0 ^ 1, kt + 1 < nk, g2);
        step(g2, kt + 5, b0, kt + 2 < nk, g0);
    }
    // this lane holds, per instruction tile, column lane % 32 and rows 8 (e / 4) + 4 (lane / 32) + e % 4
    const Dims &dm = P.dm;
    if (splits > 1) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int col = n0 + wn * 64 + b * 32 + (lane & 31);
#pragma unroll
            for (int a = 0; a < MT; ++a)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm * 32 * MT + a * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                    part[((size_t)z * mt * BM + row) * N + col] = acc[a][b][e];
                }
        }
        return;
    }
    __syncthreads();                                       // the last step's fragments have been read: the memory is free
    float *T = reinterpret_cast<float *>(pf_lds);          // [BM][kPfEpiStride]: the finished sums, columns in the packed order
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int cl = wn * 64 + b * 32 + (lane & 31), col = n0 + cl;
        int ri = -1;                                       // QKV: index of this column inside the rotated part of its head's q or k, else -1
        if (EPI == kPfQkv) {
            const int pd = col / dm.d, i = col - pd * dm.d;
            if (pd % 3 < 2 && i < dm.r) ri = i;
        }
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int rl = wm * 32 * MT + a * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const int row = m0 + rl < P.n_rows ? m0 + rl : 0;           // (rows past the pass's tokens are never stored)
                float val = pf_complete<EPI>(P, row, col, acc[a][b][e]);
                if (EPI == kPfQkv) {
                    const float other = dpp_mov<kDppXor1>(val);             // (all lanes: the neighbouring lane holds col ^ 1)
                    if (ri >= 0) {
                        const float2 cs = P.rope[(size_t)(P.pos0 + row) * (dm.r >> 1) + (ri >> 1)];
                        val = ri & 1 ? val * cs.x + other * cs.y : val * cs.x - other * cs.y;
                    }
                }
                T[rl * kPfEpiStride + cl] = val;
            }
    }
    __syncthreads();
    const int h = dm.h;
    if (EPI == kPfQkv) {
        // Work item: 8 consecutive dimensions of one token's q, k or v of one head.  Rotated dimension j
        // of a head comes from packed column 2 j (first half) or 2 (j - r/2) + 1.  q: dimensions fastest
        // (a row of q is contiguous); k, v: the two halves of a slab row, then tokens (the cache keeps
        // 32 bytes per token and slab, tokens one after the other).  A head cut by the tile's edge is
        // finished element by element, by this workgroup and its neighbour.
        const int d = dm.d, r = dm.r, G = d >> 3;
        const int pd_lo = n0 / d, pd_hi = (n0 + kPfTile - 1) / d, per_chunk = G * BM;
        const int n_items = (pd_hi - pd_lo + 1) * per_chunk;
        for (int it = tid; it < n_items; it += 256) {
            const int ch = it / per_chunk, wi = it - ch * per_chunk, pd = pd_lo + ch, nh = pd / 3, c = pd - 3 * nh;
            int rl, g;
            if (c == 0) { rl = wi / G; g = wi - rl * G; }
            else { const int slab = wi / (2 * BM), rem = wi - slab * 2 * BM; rl = rem >> 1; g = 2 * slab + (rem & 1); }
            const int row = m0 + rl;
            if (row >= P.n_rows || nh >= dm.H) continue;
            float v[8];
            unsigned in = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int dd = 8 * g + j;
                const int i = c < 2 && dd < r ? (dd < (r >> 1) ? 2 * dd : 2 * (dd - (r >> 1)) + 1) : dd;
                const int cl = pd * d + i - n0;
                const bool here = (unsigned)cl < (unsigned)kPfTile;
                v[j] = here ? T[rl * kPfEpiStride + cl] : 0.f;
                in |= (here ? 1u : 0u) << j;
            }
            if (c == 0) {
                float *dst = P.q + (size_t)row * h + nh * d + 8 * g;
                if (in == 0xffu) {
                    *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                    *reinterpret_cast<f32x4 *>(dst + 4) = f32x4{v[4], v[5], v[6], v[7]};
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (in >> j & 1) dst[j] = v[j];
                }
            } else {
                __half *dst = P.kv + kv_offset(dm, c - 1, P.b, nh, 8 * g, P.pos0 + row);
                if (in == 0xffu) {
                    u32x4 o;
                    o.x = pf_pack2(v[0], v[1]); o.y = pf_pack2(v[2], v[3]); o.z = pf_pack2(v[4], v[5]); o.w = pf_pack2(v[6], v[7]);
                    *reinterpret_cast<u32x4 *>(dst) = o;
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (in >> j & 1) dst[j] = __float2half_rn(v[j]);
                }
            }
        }
    } else if (EPI == kPfUp) {
        for (int it = tid; it < BM * 16; it += 256) {      // 8 columns of a token: one 16-byte piece of each plane
            const int rl = it >> 4, cg = (it & 15) * 8, row = m0 + rl;
            if (row >= P.n_rows) continue;
            const float *t = T + rl * kPfEpiStride + cg;
            const f32x4 v0 = *reinterpret_cast<const f32x4 *>(t), v1 = *reinterpret_cast<const f32x4 *>(t + 4);
            __half hi[8], lo[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pf_split(gelu_act(v0[j], dm.flags), hi[j], lo[j]);
                pf_split(gelu_act(v1[j], dm.flags), hi[4 + j], lo[4 + j]);
            }
            const size_t at = (size_t)row * dm.f + n0 + cg;
            *reinterpret_cast<u32x4 *>(P.mh + at) = *reinterpret_cast<const u32x4 *>(hi);
            *reinterpret_cast<u32x4 *>(P.ml + at) = *reinterpret_cast<const u32x4 *>(lo);
        }
    } else {
        const __half *bias = P.w + (EPI == kPfDense ? P.lay.b_dense : P.lay.b_down);
        const bool last = EPI == kPfDown && P.layer == P.n_layers - 1;
        const float *res_in = EPI == kPfDense ? P.xres : P.xnext;
        for (int it = tid; it < BM * 32; it += 256) {      // 4 columns of a token
            const int rl = it >> 5, c4 = (it & 31) * 4, row = m0 + rl;
            if (row >= P.n_rows) continue;
            const f32x4 v = *reinterpret_cast<const f32x4 *>(T + rl * kPfEpiStride + c4);
            const size_t at = (size_t)row * h + n0 + c4;
            const f32x4 x = *reinterpret_cast<const f32x4 *>(res_in + at);
            f32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = x[j] + (v[j] + __half2float(bias[n0 + c4 + j]));
            if (last) {
#pragma unroll
                for (int j = 0; j < 4; ++j) P.out[at + j] = __float2half_rn(o[j]);
            } else {
                *reinterpret_cast<f32x4 *>(P.xnext + at) = o;
            }
        }
    }
}

// the parts of a split-K product (part rows: prows per part), added in order, then what
// follows the product; a thread takes four consecutive columns of a row (two rotation pairs)
template <int EPI>
__global__ void __launch_bounds__(256) k_pf_reduce(PfParams P, const float *__restrict__ part, int N, int splits, int prows)
{
    const int n4 = N >> 2;
    const unsigned n_el = (unsigned)P.n_rows * (unsigned)n4;
    const size_t zstride = (size_t)prows * N;
    for (unsigned e = blockIdx.x * 256u + threadIdx.x; e < n_el; e += gridDim.x * 256u) {
        const int row = (int)(e / (unsigned)n4), col = (int)(e - (unsigned)row * (unsigned)n4) * 4;
        const float *p = part + (size_t)row * N + col;
        f32x4 s = *as_global(reinterpret_cast<const f32x4 *>(p));
        for (int z = 1; z < splits; ++z) s += *as_global(reinterpret_cast<const f32x4 *>(p + z * zstride));
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = pf_complete<EPI>(P, row, col + j, s[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) pf_store<EPI>(P, row, col + j, v[j], v[j ^ 1]);
    }
}

// ---------------------------------------------------------------------------
// Causal attention of kPfQB = 16 consecutive queries of one head: grid (H, blocks of
// queries), 4 wavefronts, on the matrix cores (v_mfma_f32_16x16x16_f16).  Keys and
// values of 64 positions at a time in LDS; wavefront w takes the tile's keys
// 16 w .. 16 w + 15:
//   S^T = K Q^T  (keys x queries): the instruction's result layout - a lane holds 4
//         consecutive keys of query lane % 16 - is at once the layout of the first
//         operand of the next product, so the weights never leave the registers;
//   O_w += P V   (queries x dimensions), P = exp(S - m) with the running maximum m of
//         the online softmax exchanged between the wavefronts through LDS once per
//         tile; V sits in LDS transposed ([dimension][key]) for that.
// q and P are fp32 values and enter as fp16 head + remainder (two instructions each),
// K and V are the cache's fp16; sums in fp32.  The wavefronts' partial outputs and
// partial softmax sums are added in wavefront order at the end.
constexpr int kPfQB = 16;
typedef _Float16 pf_f16x4 __attribute__((ext_vector_type(4)));

// maximum / sum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (the 16-lane rows of the wavefront)
__device__ __forceinline__ float pf_rows_max(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto p = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    v = fmaxf(__uint_as_float(p[0]), __uint_as_float(p[1]));
    const unsigned u2 = __float_as_uint(v);
    const auto q = __builtin_amdgcn_permlane32_swap(u2, u2, false, false);
    return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float pf_rows_sum(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto p = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    v = __uint_as_float(p[0]) + __uint_as_float(p[1]);
    const unsigned u2 = __float_as_uint(v);
    const auto q = __builtin_amdgcn_permlane32_swap(u2, u2, false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// A tile of 64 cache positions x D dimensions of K and V on its way into LDS: pieces of 8 halves
// (one 16-byte load, slab by slab) held in registers from the request, one tile ahead of the
// arithmetic, to the store - K as rows [position][dimension], V transposed [dimension][position].
// Positions past `last_pos` repeat that row (the callers mask them).
template <int D>
struct PfKvTile {
    static constexpr int kPieces = 64 * (D / 8), kPer = (kPieces + 255) / 256;
    u32x4 k[kPer], v[kPer];
    __device__ __forceinline__ void request(const __half *Kc, const __half *Vc, int t0, int last_pos, int max_seq, int tid)
    {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = min(tid + 256 * i, kPieces - 1);
            const int pc = e / 64, t = e - pc * 64;        // piece pc = dims 8 pc .. 8 pc + 7 of position t0 + t
            const int tp = min(t0 + t, last_pos);
            const size_t off = ((size_t)(pc >> 1) * max_seq + tp) * 16 + (pc & 1) * 8;
            k[i] = load16(Kc + off);
            v[i] = load16(Vc + off);
        }
    }
    __device__ __forceinline__ void store(__half *sK, __half *sVt, int QS, int VS, int tid) const
    {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = tid + 256 * i;
            if (e < kPieces) {
                const int pc = e / 64, t = e - pc * 64;
                unsigned *dk = reinterpret_cast<unsigned *>(&sK[t * QS + 8 * pc]);
                dk[0] = k[i].x; dk[1] = k[i].y; dk[2] = k[i].z; dk[3] = k[i].w;
                const __half *vh = reinterpret_cast<const __half *>(&v[i]);
#pragma unroll
                for (int j = 0; j < 8; ++j) sVt[(8 * pc + j) * VS + t] = vh[j];
            }
        }
    }
};

template <int D>
__global__ void __launch_bounds__(256) k_pf_attn(PfParams P)
{
    constexpr int QS = D + 4;                              // halves per row of q and K in LDS (8-byte fragment reads, spread over the banks)
    constexpr int VS = 64 + 4;                             // halves per row of V transposed
    constexpr int NB = D / 16;                             // 16-dimension blocks
    __shared__ __align__(16) __half sQh[kPfQB * QS], sQl[kPfQB * QS];
    constexpr int KVH = 64 * QS + D * VS;                  // halves of a tile of K and V
    static_assert(KVH * 2 >= 4 * kPfQB * D * 4 && (64 * QS) % 8 == 0, "the wavefronts' outputs reuse the tile's memory");
    __shared__ __align__(16) __half sKV[KVH];
    __shared__ float sMax[4][kPfQB], sCorr[4][kPfQB], sL[4][kPfQB];
    __half *sK = sKV, *sVt = sKV + 64 * QS;
    float (*sO)[kPfQB][D] = reinterpret_cast<float (*)[kPfQB][D]>(sKV);      // after the last tile
    const Dims &dm = P.dm;
    const int head = blockIdx.x, q0 = blockIdx.y * kPfQB, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (q0 >= P.n_rows) return;
    const int nq = min(kPfQB, P.n_rows - q0);
    const float scale = 1.0f / sqrtf((float)D);
    for (int e = tid; e < kPfQB * D; e += 256) {
        const int qi = e / D, dmi = e - qi * D;
        const float v = qi < nq ? P.q[(size_t)(q0 + qi) * dm.h + head * D + dmi] * scale : 0.f;
        __half hi, lo;
        pf_split(v, hi, lo);
        sQh[qi * QS + dmi] = hi; sQl[qi * QS + dmi] = lo;
    }
    const int col = lane & 15, grp = lane >> 4;            // column of a result tile, group of 4 rows / 4 K values
    const int qpos = P.pos0 + q0 + col;                    // position of the query this lane's S^T column belongs to
    const bool qlive = col < nq;
    float m_run = -INFINITY, l_part = 0.f;                 // running maximum (all wavefronts alike), this wavefront's sum
    f32x4 O[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) O[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int last_pos = P.pos0 + q0 + nq - 1;             // the block's last query attends up to here
    const __half *Kc = P.kv + kv_offset(dm, 0, P.b, head, 0, 0), *Vc = P.kv + kv_offset(dm, 1, P.b, head, 0, 0);
    PfKvTile<D> tile;
    tile.request(Kc, Vc, 0, last_pos, dm.max_seq, tid);
    for (int t0 = 0; t0 <= last_pos; t0 += 64) {
        __syncthreads();                                   // the previous tile is no longer read (first: q is written)
        tile.store(sK, sVt, QS, VS, tid);
        tile.request(Kc, Vc, t0 + 64, last_pos, dm.max_seq, tid);   // the next tile travels while this one is worked on
        __syncthreads();
        // S^T of this wavefront's 16 keys: rows = keys 16 wave + 4 grp + v, column = query col
        f32x4 st = {0.f, 0.f, 0.f, 0.f};
        const __half *ka = &sK[(16 * wave + col) * QS + 4 * grp];
        const __half *qh = &sQh[col * QS + 4 * grp], *ql = &sQl[col * QS + 4 * grp];
#pragma unroll
        for (int ks = 0; ks < NB; ++ks) {
            const pf_f16x4 kf = *reinterpret_cast<const pf_f16x4 *>(ka + 16 * ks);
            st = __builtin_amdgcn_mfma_f32_16x16x16f16(kf, *reinterpret_cast<const pf_f16x4 *>(qh + 16 * ks), st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_16x16x16f16(kf, *reinterpret_cast<const pf_f16x4 *>(ql + 16 * ks), st, 0, 0, 0);
        }
        const int key0 = t0 + 16 * wave + 4 * grp;
        float mloc = -INFINITY;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            st[v] = qlive && key0 + v <= qpos ? st[v] : -INFINITY;
            mloc = fmaxf(mloc, st[v]);
        }
        mloc = pf_rows_max(mloc);                          // over this wavefront's 16 keys, for query col
        if (lane < 16) sMax[wave][lane] = mloc;
        __syncthreads();
        const float mt = fmaxf(fmaxf(sMax[0][col], sMax[1][col]), fmaxf(sMax[2][col], sMax[3][col]));
        const float mn = fmaxf(m_run, mt);
        const float corr = m_run == -INFINITY ? 0.f : expf(m_run - mn);     // (mn finite whenever m_run is)
        float p[4], psum = 0.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            p[v] = st[v] == -INFINITY ? 0.f : expf(st[v] - mn);
            psum += p[v];
        }
        l_part = l_part * corr + pf_rows_sum(psum);
        m_run = mn;
        if (lane < 16) sCorr[wave][lane] = corr;           // (read below by this wavefront only: no barrier)
        pf_f16x4 ph, pl;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const _Float16 h = (_Float16)p[v];
            ph[v] = h;
            pl[v] = (_Float16)(p[v] - (float)h);
        }
        // O rows = queries 4 grp + v, column = dimension 16 nb + col: rescale, then add P V of this wavefront's keys
        float cr[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) cr[v] = sCorr[wave][4 * grp + v];
        const __half *vb = &sVt[col * VS + 16 * wave + 4 * grp];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            f32x4 o = O[nb];
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] *= cr[v];
            const pf_f16x4 vf = *reinterpret_cast<const pf_f16x4 *>(vb + 16 * nb * VS);
            o = __builtin_amdgcn_mfma_f32_16x16x16f16(ph, vf, o, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_16x16x16f16(pl, vf, o, 0, 0, 0);
            O[nb] = o;
        }
    }
    // the wavefronts' parts, added in wavefront order
    __syncthreads();                                       // (the last tile is no longer read)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) sO[wave][4 * grp + v][16 * nb + col] = O[nb][v];
    if (lane < 16) sL[wave][lane] = l_part;
    __syncthreads();
    for (int e = tid; e < nq * D; e += 256) {
        const int qi = e / D, dmi = e - qi * D;
        const float l = ((sL[0][qi] + sL[1][qi]) + sL[2][qi]) + sL[3][qi];
        const float o = ((sO[0][qi][dmi] + sO[1][qi][dmi]) + sO[2][qi][dmi]) + sO[3][qi][dmi];
        __half hi, lo;
        pf_split(o / l, hi, lo);
        const size_t at = (size_t)(q0 + qi) * dm.h + head * D + dmi;
        P.oh[at] = hi; P.ol[at] = lo;
    }
}

// The same attention for long passes: 64 consecutive queries per workgroup, 16 per wavefront,
// every wavefront over all 64 keys of a tile.  A tile of K and V is then fetched once per 64
// queries instead of once per 16 (at 4096 tokens the narrow kernel pulls 10 GB per layer out of
// the L2), a wavefront's softmax is its own (no exchange between wavefronts), its q stays in
// registers as instruction operands, and a wavefront skips the tiles behind its last query.
// Blocks of later queries (more tiles) are started first.
constexpr int kPfQW = 64;
#ifndef PF_WIDE_FROM
#define PF_WIDE_FROM 1024
#endif
constexpr int kPfWideFrom = PF_WIDE_FROM;             // tokens in a pass from which the wide kernel runs

template <int D>
__global__ void __launch_bounds__(256) k_pf_attn_wide(PfParams P)
{
    constexpr int QS = D + 4, VS = 64 + 4, NB = D / 16;
    __shared__ __align__(16) __half sK[64 * QS];
    __shared__ __align__(16) __half sVt[D * VS];
    __shared__ float sX[4][16];                            // a per-query value from the lanes of the score layout to those of the output layout
    const Dims &dm = P.dm;
    const int head = blockIdx.x, q0 = ((int)gridDim.y - 1 - (int)blockIdx.y) * kPfQW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (q0 >= P.n_rows) return;
    const int nq = min(kPfQW, P.n_rows - q0);
    const float scale = 1.0f / sqrtf((float)D);
    const int col = lane & 15, grp = lane >> 4;
    const int qw0 = q0 + 16 * wave, qi = qw0 + col;        // this wavefront's first query, this lane's query in the score layout
    const bool qlive = qi < P.n_rows;
    const int qpos = P.pos0 + qi;
    const int wave_last = qw0 < P.n_rows ? P.pos0 + min(qw0 + 15, P.n_rows - 1) : -1;
    pf_f16x4 qh[NB], ql[NB];                               // Q^T fragments: dimensions 16 ks + 4 grp .. + 3 of query col
#pragma unroll
    for (int ks = 0; ks < NB; ++ks)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float v = qlive ? P.q[(size_t)qi * dm.h + head * D + 16 * ks + 4 * grp + j] * scale : 0.f;
            const _Float16 hi = (_Float16)v;
            qh[ks][j] = hi;
            ql[ks][j] = (_Float16)(v - (float)hi);
        }
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 O[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) O[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int last_pos = P.pos0 + q0 + nq - 1;
    const __half *Kc = P.kv + kv_offset(dm, 0, P.b, head, 0, 0), *Vc = P.kv + kv_offset(dm, 1, P.b, head, 0, 0);
    PfKvTile<D> tile;
    tile.request(Kc, Vc, 0, last_pos, dm.max_seq, tid);
    for (int t0 = 0; t0 <= last_pos; t0 += 64) {
        __syncthreads();                                   // the previous tile is no longer read
        tile.store(sK, sVt, QS, VS, tid);
        tile.request(Kc, Vc, t0 + 64, last_pos, dm.max_seq, tid);   // the next tile travels while this one is worked on
        __syncthreads();
        if (t0 > wave_last) continue;                      // (whole wavefront; the barriers are above)
        // S^T of the tile's four key blocks: rows = keys 16 kb + 4 grp + v, column = query col
        f32x4 st[4];
        float mloc = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
            const __half *ka = &sK[(16 * kb + col) * QS + 4 * grp];
#pragma unroll
            for (int ks = 0; ks < NB; ++ks) {
                const pf_f16x4 kf = *reinterpret_cast<const pf_f16x4 *>(ka + 16 * ks);
                a = __builtin_amdgcn_mfma_f32_16x16x16f16(kf, qh[ks], a, 0, 0, 0);
                a = __builtin_amdgcn_mfma_f32_16x16x16f16(kf, ql[ks], a, 0, 0, 0);
            }
            const int key0 = t0 + 16 * kb + 4 * grp;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                a[v] = qlive && key0 + v <= qpos ? a[v] : -INFINITY;
                mloc = fmaxf(mloc, a[v]);
            }
            st[kb] = a;
        }
        mloc = pf_rows_max(mloc);                          // over the tile's 64 keys, for query col
        const float mn = fmaxf(m_run, mloc);
        const float corr = m_run == -INFINITY ? 0.f : expf(m_run - mn);
        float psum = 0.f;
        pf_f16x4 ph[4], pl[4];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float pv = st[kb][v] == -INFINITY ? 0.f : expf(st[kb][v] - mn);
                psum += pv;
                const _Float16 hi = (_Float16)pv;
                ph[kb][v] = hi;
                pl[kb][v] = (_Float16)(pv - (float)hi);
            }
        l_run = l_run * corr + pf_rows_sum(psum);
        m_run = mn;
        if (lane < 16) sX[wave][lane] = corr;              // (written and read by this wavefront only: no barrier)
        float cr[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) cr[v] = sX[wave][4 * grp + v];
        // O rows = queries 4 grp + v, column = dimension 16 nb + col
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            f32x4 o = O[nb];
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] *= cr[v];
            const __half *vb = &sVt[(16 * nb + col) * VS + 4 * grp];
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const pf_f16x4 vf = *reinterpret_cast<const pf_f16x4 *>(vb + 16 * kb);
                o = __builtin_amdgcn_mfma_f32_16x16x16f16(ph[kb], vf, o, 0, 0, 0);
                o = __builtin_amdgcn_mfma_f32_16x16x16f16(pl[kb], vf, o, 0, 0, 0);
            }
            O[nb] = o;
        }
    }
    if (lane < 16) sX[wave][lane] = l_run;
    float lr[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) lr[v] = sX[wave][4 * grp + v];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int qo = qw0 + 4 * grp + v;
        if (qo < P.n_rows) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                __half hi, lo;
                pf_split(O[nb][v] / lr[v], hi, lo);
                const size_t at = (size_t)qo * dm.h + head * D + 16 * nb + col;
                P.oh[at] = hi; P.ol[at] = lo;
            }
        }
    }
}

// ---------------------------------------------------------------------------
bool pf_supported(const Dims &dm)
{
    return dm.h % kPfTile == 0 && dm.f % kPfTile == 0 && dm.h <= 256 * kPfLnVec && (dm.d == 64 || dm.d == 80 || dm.d == 128) &&
           !(dm.flags & kFlagSequentialResidual) && dm.r % 2 == 0;
}

// Tile height and splits of K for a product: 64-token tiles while 128-token ones would leave
// fewer than two workgroups per CU; K halved while the tile parts stay within half of what the
// scratch holds (kPfSplitTiles, in 128 x 128 parts) and every part is whole K steps of the kernel.
struct PfPlan { int bm, splits; };
static PfPlan pf_plan(int n_rows, int N, int K)
{
    PfPlan p;
    const int ntn = N / kPfTile;
    p.bm = ntn * ((n_rows + 127) / 128) < 512 ? 64 : 128;
    const int tiles = ntn * ((n_rows + p.bm - 1) / p.bm);
    const int parts128 = p.bm == 64 ? (tiles + 1) / 2 : tiles;         // what a part costs in the scratch
    const int bk = p.bm == 64 ? 64 : 32;                              // (the kernel's K step for that height)
    p.splits = 1;
    while (p.splits < 8 && tiles * p.splits <= 256 && parts128 * p.splits <= kPfSplitTiles / 2 && K % (2 * p.splits * bk) == 0)
        p.splits *= 2;
    return p;
}

template <int EPI>
static hipError_t pf_gemm(const PfParams &P, const __half *Ah, const __half *Al, const __half *W, int K, int N, float *part,
                    hipStream_t s)
{
    const PfPlan pl = pf_plan(P.n_rows, N, K);
    const int mt = (P.n_rows + pl.bm - 1) / pl.bm, tiles = (N / kPfTile) * mt;
    const int grid = (tiles * pl.splits + 7) / 8 * 8;
    // the parts of a split product, [splits][mt * bm][N] floats, must fit what the scratch holds for them
    if (pl.splits > 1 && (size_t)pl.splits * mt * pl.bm * N > (size_t)kPfSplitTiles * kPfTile * kPfTile) return hipErrorInvalidValue;
    if (pl.bm == 64) {
        constexpr int lds = pf_gemm_lds_bytes<64, 64>();
        const hipError_t e = hipFuncSetAttribute((const void *)k_pf_gemm<EPI, 64, 64>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k_pf_gemm<EPI, 64, 64>), dim3(grid), dim3(256), lds, s, P, Ah, Al, W, K, N, pl.splits, part);
    } else {
        constexpr int lds = pf_gemm_lds_bytes<128, 32>();
        const hipError_t e = hipFuncSetAttribute((const void *)k_pf_gemm<EPI, 128, 32>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k_pf_gemm<EPI, 128, 32>), dim3(grid), dim3(256), lds, s, P, Ah, Al, W, K, N, pl.splits, part);
    }
    if (pl.splits > 1) {
        const size_t n_el = (size_t)P.n_rows * (N / 4);
        hipLaunchKernelGGL(k_pf_reduce<EPI>, dim3((unsigned)((n_el + 255) / 256)), dim3(256), 0, s, P, (const float *)part, N,
                           pl.splits, mt * pl.bm);
    }
    return hipSuccess;
}

hipError_t launch_pf_layer(const PfParams &P, hipStream_t s)
{
    const Dims &dm = P.dm;
    const int mt = (P.n_rows + kPfTile - 1) / kPfTile;
    const __half *w = P.w;
    hipLaunchKernelGGL(k_pf_ln, dim3(mt * kPfTile / 4), dim3(256), 0, s, P);
    hipError_t e = pf_gemm<kPfQkv>(P, P.y1h, P.y1l, w + P.lay.w_qkv, dm.h, 3 * dm.h, P.part, s);
    if (e != hipSuccess) return e;
    e = pf_gemm<kPfUp>(P, P.y2h, P.y2l, w + P.lay.w_up, dm.h, dm.f, P.part, s);
    if (e != hipSuccess) return e;
    if (P.n_rows >= kPfWideFrom) {
        const dim3 ag(dm.H, (P.n_rows + kPfQW - 1) / kPfQW);
        switch (dm.d) {
        case 64: hipLaunchKernelGGL(k_pf_attn_wide<64>, ag, dim3(256), 0, s, P); break;
        case 80: hipLaunchKernelGGL(k_pf_attn_wide<80>, ag, dim3(256), 0, s, P); break;
        case 128: hipLaunchKernelGGL(k_pf_attn_wide<128>, ag, dim3(256), 0, s, P); break;
        default: return hipErrorInvalidValue;
        }
    } else {
        const dim3 ag(dm.H, (P.n_rows + kPfQB - 1) / kPfQB);
        switch (dm.d) {
        case 64: hipLaunchKernelGGL(k_pf_attn<64>, ag, dim3(256), 0, s, P); break;
        case 80: hipLaunchKernelGGL(k_pf_attn<80>, ag, dim3(256), 0, s, P); break;
        case 128: hipLaunchKernelGGL(k_pf_attn<128>, ag, dim3(256), 0, s, P); break;
        default: return hipErrorInvalidValue;
        }
    }
    e = pf_gemm<kPfDense>(P, P.oh, P.ol, w + P.lay.w_dense, dm.h, dm.h, P.part, s);
    if (e != hipSuccess) return e;
    e = pf_gemm<kPfDown>(P, P.mh, P.ml, w + P.lay.w_down, dm.f, dm.h, P.part, s);
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace cfpp
