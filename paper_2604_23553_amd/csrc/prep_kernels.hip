// One-time data preparation kernels: packing a block's canonical tensors into
// the streaming layout, and moving KV rows between the canonical layout
// [n_heads, capacity, head_dim] and the slabbed cache layout.  Data movement
// and the per-row constants derived from the packed tensors, off the hot path.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "decode_params.h"

namespace cfpp {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// dst[p][:] = src[map(p)][:], 16 bytes per thread; cols % 8 == 0
__global__ void k_copy_rows(const __half *__restrict__ src, __half *__restrict__ dst, long long rows,
                            int cols, int qkv_d, int qkv_r)
{
    const long long per_row = cols / 8;
    const long long n = rows * per_row;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x) {
        const long long p = i / per_row, c8 = i - p * per_row;
        const long long sr = qkv_d ? qkv_packed_to_canonical_row((int)p, qkv_d, qkv_r) : p;
        *reinterpret_cast<u32x4 *>(dst + p * cols + c8 * 8) =
            *reinterpret_cast<const u32x4 *>(src + sr * cols + c8 * 8);
    }
}

__global__ void k_copy_vec(const __half *__restrict__ src, __half *__restrict__ dst, int n, int qkv_d,
                           int qkv_r)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x)
        dst[i] = src[qkv_d ? qkv_packed_to_canonical_row(i, qkv_d, qkv_r) : i];
}

// rc[p] = (sum_j W[p][j] gamma[j],  sum_j W[p][j] beta[j] + bias[p]) for every row of a
// packed matrix: one wavefront per row, fp64 sums in a fixed order, rounded once to fp32
__global__ void __launch_bounds__(256) k_row_constants(const __half *__restrict__ W, const __half *__restrict__ gamma,
                                                        const __half *__restrict__ beta, const __half *__restrict__ bias,
                                                        float2 *__restrict__ rc, int rows, int K)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const __half *wr = W + (size_t)row * K;
    double s = 0.0, c = 0.0;
    for (int j = lane; j < K; j += 64) {
        const double wv = (double)__half2float(wr[j]);
        s += wv * (double)__half2float(gamma[j]);
        c += wv * (double)__half2float(beta[j]);
    }
    for (int m = 32; m > 0; m >>= 1) {
        s += __shfl_xor(s, m, 64);
        c += __shfl_xor(c, m, 64);
    }
    if (lane == 0) rc[row] = float2{(float)s, (float)(c + (double)__half2float(bias[row]))};
}

hipError_t launch_pack_layer(const Dims &dm, const PackedLayout &lay, const void *const src[12],
                             __half *dst, hipStream_t s)
{
    const int h = dm.h, f = dm.f;
    auto vec = [&](int idx, size_t off, int n, bool qkv) {
        hipLaunchKernelGGL(k_copy_vec, dim3((n + 255) / 256), dim3(256), 0, s,
                           (const __half *)src[idx], dst + off, n, qkv ? dm.d : 0, dm.r);
    };
    auto mat = [&](int idx, size_t off, long long rows, int cols, bool qkv) {
        hipLaunchKernelGGL(k_copy_rows, dim3(2048), dim3(256), 0, s, (const __half *)src[idx],
                           dst + off, rows, cols, qkv ? dm.d : 0, dm.r);
    };
    // order of src: ln1_g ln1_b ln2_g ln2_b w_qkv b_qkv w_dense b_dense w_up b_up w_down b_down
    vec(0, lay.ln1_g, h, false); vec(1, lay.ln1_b, h, false);
    vec(2, lay.ln2_g, h, false); vec(3, lay.ln2_b, h, false);
    mat(4, lay.w_qkv, 3LL * h, h, true); vec(5, lay.b_qkv, 3 * h, true);
    mat(6, lay.w_dense, h, h, false); vec(7, lay.b_dense, h, false);
    mat(8, lay.w_up, f, h, false); vec(9, lay.b_up, f, false);
    mat(10, lay.w_down, h, f, false); vec(11, lay.b_down, h, false);
    // the row constants of the two products that follow a LayerNorm, from the packed copies
    // (same stream: behind the copies above)
    auto consts = [&](size_t w_off, size_t g_off, size_t b_off, size_t bias_off, size_t rc_off, int rows) {
        hipLaunchKernelGGL(k_row_constants, dim3((rows + 3) / 4), dim3(256), 0, s, dst + w_off, dst + g_off,
                           dst + b_off, dst + bias_off, reinterpret_cast<float2 *>(dst + rc_off), rows, h);
    };
    consts(lay.w_qkv, lay.ln1_g, lay.ln1_b, lay.b_qkv, lay.rc_qkv, 3 * h);
    consts(lay.w_up, lay.ln2_g, lay.ln2_b, lay.b_up, lay.rc_up, f);
    return hipGetLastError();
}

// one thread per (which, head, position, 8-dim group)
__global__ void k_kv_move(Dims dm, const __half *k_can, const __half *v_can, int cap, int pos_begin,
                          int n_pos, int b, __half *kv, int to_cache)
{
    const int d8 = dm.d / 8;
    const long long n = 2LL * dm.H * n_pos * d8;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x) {
        long long r = i;
        const int j = (int)(r % d8); r /= d8;
        const int t = (int)(r % n_pos); r /= n_pos;
        const int hd = (int)(r % dm.H);
        const int which = (int)(r / dm.H);
        const __half *can = which ? v_can : k_can;
        // canonical row index: import reads row pos, export writes row (pos - pos_begin)
        const int pos = pos_begin + t;
        const int crow = to_cache ? pos : t;
        __half *cp = const_cast<__half *>(can) + ((size_t)hd * cap + crow) * dm.d + j * 8;
        __half *kp = kv + kv_offset(dm, which, b, hd, j * 8, pos);
        if (to_cache) *reinterpret_cast<u32x4 *>(kp) = *reinterpret_cast<const u32x4 *>(cp);
        else *reinterpret_cast<u32x4 *>(cp) = *reinterpret_cast<const u32x4 *>(kp);
    }
}

hipError_t launch_kv_import(const Dims &dm, const __half *k_src, const __half *v_src, int src_cap,
                            int n_pos, int b, __half *kv, hipStream_t s)
{
    if (n_pos == 0) return hipSuccess;
    hipLaunchKernelGGL(k_kv_move, dim3(1024), dim3(256), 0, s, dm, k_src, v_src, src_cap, 0, n_pos, b,
                       kv, 1);
    return hipGetLastError();
}

hipError_t launch_kv_export(const Dims &dm, const __half *kv, int b, int pos_begin, int n_pos,
                            int dst_cap, __half *k_dst, __half *v_dst, hipStream_t s)
{
    if (n_pos == 0) return hipSuccess;
    hipLaunchKernelGGL(k_kv_move, dim3(1024), dim3(256), 0, s, dm, (const __half *)k_dst,
                       (const __half *)v_dst, dst_cap, pos_begin, n_pos, b, const_cast<__half *>(kv), 0);
    return hipGetLastError();
}


__global__ void k_fill_positions(int *dst, int first, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = first + i;
}

hipError_t launch_fill_positions(int *dst, int first, int n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_positions, dim3((n + 255) / 256), dim3(256), 0, s, dst, first, n);
    return hipGetLastError();
}

#ifdef CFPP_PROFILE
// ---- plain streaming kernels of known traffic (bandwidth calibration; profiling library only) ---------
// read: every 16-byte word of src is loaded once and folded into a checksum, one
// word per workgroup written to sink; copy: dst = src.
template <int U>
__global__ void __launch_bounds__(512) k_stream_read(const u32x4 *__restrict__ src, long long n16,
                                                      unsigned *__restrict__ sink)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    unsigned acc = 0;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int j = 0; j < U; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
        for (int j = 0; j < U; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    for (; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    for (int m = 32; m > 0; m >>= 1) acc ^= __shfl_xor(acc, m, 64);
    if ((threadIdx.x & 63) == 0) atomicXor(sink + blockIdx.x, acc);
}

__global__ void __launch_bounds__(512) k_stream_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                      long long n16)
{
    constexpr int U = 4;
    const long long stride = (long long)gridDim.x * blockDim.x;
    long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int j = 0; j < U; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
        for (int j = 0; j < U; ++j) __builtin_nontemporal_store(v[j], dst + i + j * stride);
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_stream_read(const void *src, size_t bytes, unsigned *sink, int grid, int threads,
                              int unroll, hipStream_t s)
{
    const long long n16 = (long long)(bytes / 16);
    const u32x4 *p = static_cast<const u32x4 *>(src);
    if (unroll >= 8) hipLaunchKernelGGL(k_stream_read<8>, dim3(grid), dim3(threads), 0, s, p, n16, sink);
    else if (unroll >= 4) hipLaunchKernelGGL(k_stream_read<4>, dim3(grid), dim3(threads), 0, s, p, n16, sink);
    else hipLaunchKernelGGL(k_stream_read<2>, dim3(grid), dim3(threads), 0, s, p, n16, sink);
    return hipGetLastError();
}

hipError_t launch_stream_copy(const void *src, void *dst, size_t bytes, int grid, int threads, hipStream_t s)
{
    hipLaunchKernelGGL(k_stream_copy, dim3(grid), dim3(threads), 0, s, static_cast<const u32x4 *>(src),
                       static_cast<u32x4 *>(dst), (long long)(bytes / 16));
    return hipGetLastError();
}
#endif  // CFPP_PROFILE

}  // namespace cfpp
