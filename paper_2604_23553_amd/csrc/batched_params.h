// Arguments of the batched projection kernels (batched_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "layout.h"

namespace cfpp {

constexpr int kBatMax = 8;             // sequences per launch (two 4-column blocks of the MFMA B operand)
constexpr int kBatLnPerLane = 64;      // hidden values a lane normalises at most (hidden <= 4096)

// All per-sequence pointers are already offset to the first sequence of the
// group (b0); sequence b of the group follows at the workspace's usual strides.
struct BatParams {
    Dims dm;
    PackedLayout lay;
    const __half *w;        // packed layer
    __half *kv;             // the layer's cache (whole, indexed with b0 + b)
    const int *pos;         // [nb]
    int nb, b0;
    // row i of the group appends to the cache of sequence kv_b0 + i * kv_bstep: its own
    // sequence (b0, 1), or - consecutive positions of one prompt - all the same one (b, 0)
    int kv_b0, kv_bstep;
    int layer, n_layers;    // position in the fp32 residual ping-pong
    const __half *x_in;     // [nb][h] fp16: input of layer 0
    __half *out;            // [nb][h] fp16: output of the last layer
    float *xres;            // [nb][2][h]
    float *q;               // [nb][h]
    float *m;               // [nb][f]
    float *o;               // [nb][h]
    const float2 *rope;
    unsigned *sync;
    int rows, rows2;        // matrix rows per workgroup (set by the launcher; rows2: the MLP-up rows of the
                            // launch that also runs the QKV rows)
};

bool bat_supported(const Dims &dm, int grid, int threads);
size_t bat_lds_bytes(const Dims &dm, int grid);
hipError_t launch_bat_qkv_up(BatParams P, int grid, hipStream_t s);
hipError_t launch_bat_out(BatParams P, int grid, hipStream_t s);
hipError_t prepare_bat_kernels(size_t lds_bytes);

}  // namespace cfpp
