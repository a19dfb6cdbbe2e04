// The steps either side of the decode stack in a generation loop (paper Sec.
// 2.3: one graph replay per generated token with static buffers; Sec. 3 compares
// the generated tokens with the baseline's without naming the rule that picks
// them - the largest logit is taken here): the embedding row of the current token before it, and behind it
// the final LayerNorm, the bias-free LM head, and the index of the largest
// logit (lowest index among equal maxima), which becomes the next token while
// the position advances by one.
//
//   k_lm_embed : x[h] = embed[tokens[pos]]
//   k_lm_head  : every workgroup normalises the hidden vector (it is a few KB),
//                streams its share of the LM-head rows like any other GEMV of
//                this library and leaves the best (logit, row) of its share
//   k_lm_pick  : one workgroup picks the best of those in workgroup order,
//                writes tokens[pos + 1] and advances pos
//
// All three read pos from device memory and do nothing when it is outside
// [0, max_seq) (the stack kernels raise the error flag for that).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <climits>
#include "decode_blocks.h"
#include "lm_params.h"

namespace cfpp {

__global__ void __launch_bounds__(256) k_lm_embed(LmParams L)
{
    const int p = *L.pos;
    if (p < 0 || p >= L.max_seq) return;
    int tok = L.tokens[p];
    if (tok < 0 || tok >= L.vocab) {
        if (threadIdx.x == 0)
            __hip_atomic_store(&L.sync[kSyncErr], (unsigned)kErrBadToken, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        tok = 0;
    }
    const u32x4 *src = reinterpret_cast<const u32x4 *>(L.embed + (size_t)tok * L.h);
    u32x4 *dst = reinterpret_cast<u32x4 *>(L.x);
    for (int i = threadIdx.x; i < L.h / 8; i += blockDim.x) dst[i] = src[i];
}

// (logit, row) pairs: a beats b if its logit is larger, or equal with a lower row
__device__ __forceinline__ bool lm_better(float va, int ia, float vb, int ib)
{
    return va > vb || (va == vb && ia < ib);
}

__device__ __forceinline__ void lm_wave_best(float &v, int &i)
{
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) {
        const float ov = __shfl_xor(v, m, 64);
        const int oi = __shfl_xor(i, m, 64);
        if (lm_better(ov, oi, v, i)) { v = ov; i = oi; }
    }
}

__global__ void __launch_bounds__(kMaxThreads) k_lm_head(LmParams L)
{
    extern __shared__ __align__(16) float lds[];
    const int p = *L.pos;
    if (p < 0 || p >= L.max_seq) return;
    const int tid = threadIdx.x, nt = blockDim.x, nw = nt >> 6, h = L.h;
    const int Kp = round_up_chunk(h);
    float *y = lds, *part = lds + Kp, *red = part + L.rows * nw;
    const int r_begin = blockIdx.x * L.rows;
    const int r_n = max(0, min(L.rows, L.vocab - r_begin));

    // the first weights are requested before the LayerNorm needs anything
    GemvSpan<kGemvU> gs;
    gs.init(GemvSeg{L.w_lm + (size_t)r_begin * h, y, h, r_n}, GemvSeg{L.w_lm, y, h, 0}, L.w_lm, tid);
    gs.issue_first();
    gs.issue_second();

    // final LayerNorm (two passes, biased variance), output in GEMV order, zero padded
    float xv[kLmPerThread];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kLmPerThread; ++j) {
        const int i = tid + j * nt;
        xv[j] = i < h ? __half2float(L.hidden[i]) : 0.f;
        s += xv[j];
    }
    const float mean = block_sum(s, red, tid) / (float)h;
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < kLmPerThread; ++j) {
        const float dlt = tid + j * nt < h ? xv[j] - mean : 0.f;
        v += dlt * dlt;
    }
    const float var = block_sum(v, red, tid) / (float)h;
    const float inv = 1.0f / sqrtf(var + L.eps);
#pragma unroll
    for (int j = 0; j < kLmPerThread; ++j) {
        const int i = tid + j * nt;
        if (i < Kp)
            y[lds_perm(i)] = i < h ? (xv[j] - mean) * inv * __half2float(L.lnf_g[i]) + __half2float(L.lnf_b[i]) : 0.f;
    }
    clear_partials(part, L.rows * nw, tid);
    __syncthreads();
    gs.run(part);
    __syncthreads();

    // logits of this workgroup's rows; its best row
    float best = -INFINITY;
    int bi = INT_MAX;
    for (int t = tid; t < r_n; t += nt) {
        const float lg = gs.row_total(part, t);
        if (L.logits) L.logits[r_begin + t] = lg;
        if (lm_better(lg, r_begin + t, best, bi)) { best = lg; bi = r_begin + t; }
    }
    lm_wave_best(best, bi);
    __syncthreads();                                       // red was read by the block sums
    if ((tid & 63) == 0) { red[2 * (tid >> 6)] = best; red[2 * (tid >> 6) + 1] = __int_as_float(bi); }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < nw; ++w) {
            const float ov = red[2 * w];
            const int oi = __float_as_int(red[2 * w + 1]);
            if (lm_better(ov, oi, best, bi)) { best = ov; bi = oi; }
        }
        L.best[2 * blockIdx.x] = best;
        L.best[2 * blockIdx.x + 1] = __int_as_float(bi);
    }
}

__global__ void __launch_bounds__(64) k_lm_pick(LmParams L, int n_wg)
{
    const int p = *L.pos;
    if (p < 0 || p >= L.max_seq) return;
    const int lane = threadIdx.x;
    float best = -INFINITY;
    int bi = INT_MAX;
    for (int g = lane; g < n_wg; g += 64) {
        const float ov = L.best[2 * g];
        const int oi = __float_as_int(L.best[2 * g + 1]);
        if (lm_better(ov, oi, best, bi)) { best = ov; bi = oi; }
    }
    lm_wave_best(best, bi);
    if (lane == 0) {
        L.tokens_out[p + 1] = bi >= 0 && bi < L.vocab ? bi : 0;   // (no finite logit at all: token 0)
        *L.pos_out = p + 1;
    }
}

hipError_t launch_lm_embed(const LmParams &L, hipStream_t s)
{
    hipLaunchKernelGGL(k_lm_embed, dim3(1), dim3(256), 0, s, L);
    return hipGetLastError();
}

size_t lm_head_lds_bytes(const LmParams &L, int threads)
{
    const size_t Kp = (size_t)(L.h + kChunk - 1) / kChunk * kChunk;
    return (Kp + (size_t)L.rows * (threads / 64) + 32) * 4;
}

hipError_t launch_lm_head(const LmParams &L, int grid, int threads, hipStream_t s)
{
    hipLaunchKernelGGL(k_lm_head, dim3(grid), dim3(threads), lm_head_lds_bytes(L, threads), s, L);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_lm_pick, dim3(1), dim3(64), 0, s, L, grid);
    return hipGetLastError();
}

hipError_t prepare_lm_kernels(size_t lds_bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_lm_head), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)lds_bytes);
}

}  // namespace cfpp
