// Arguments of the prompt-sized kernels (prefill_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "layout.h"

namespace cfpp {

constexpr int kPfTile = 128;           // rows (tokens) and columns (output features) of a GEMM workgroup tile
constexpr int kPfMaxRows = 4096;       // most tokens a pass takes
constexpr int kPfSplitTiles = 384;      // most 128 x 128 parts a split product leaves: K is halved only while the parts number
                                       // at most half of this, and the scratch holds this many

// Scratch of one pass over `rows` tokens (rows a multiple of kPfTile), byte
// offsets; the caller owns the memory.  Activations that feed a GEMM are kept
// as two fp16 planes, head and remainder (y = hi + lo to ~2^-22), row-major.
struct PfLayout {
    size_t xres, xnext;            // float [rows][h]: residual stream entering / leaving the block
    size_t y1h, y1l, y2h, y2l;     // half [rows][h]: gamma_1 * x and gamma_2 * x
    size_t stats;                  // float2 [rows]: mean, 1 / sqrt(variance + eps)
    size_t q;                      // float [rows][h]: rotated queries
    size_t oh, ol;                 // half [rows][h]: attention output
    size_t mh, ml;                 // half [rows][f]: GELU(up)
    size_t part;                   // float [kPfSplitTiles][128][128]: the parts of a product whose K is split over workgroups
    size_t total;
};

CFPP_HD PfLayout pf_layout(const Dims &m, int rows)
{
    PfLayout L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    const size_t rh = (size_t)rows * m.h, rf = (size_t)rows * m.f;
    L.xres = take(rh * 4); L.xnext = take(rh * 4);
    L.y1h = take(rh * 2); L.y1l = take(rh * 2); L.y2h = take(rh * 2); L.y2l = take(rh * 2);
    L.stats = take((size_t)rows * 8);
    L.q = take(rh * 4);
    L.oh = take(rh * 2); L.ol = take(rh * 2);
    L.mh = take(rf * 2); L.ml = take(rf * 2);
    L.part = take((size_t)kPfSplitTiles * kPfTile * kPfTile * 4);
    L.total = o;
    return L;
}

struct PfParams {
    Dims dm;
    PackedLayout lay;
    const __half *w;        // packed layer
    __half *kv;             // the layer's cache
    int b;                  // sequence inside the cache
    int pos0;               // position of the pass's first token
    int n_rows, rows;       // tokens in this pass, rows of the scratch (n_rows <= rows)
    int layer, n_layers;
    const __half *x_in;     // [n_rows][h] fp16: input of layer 0
    __half *out;            // [n_rows][h] fp16: output of the last layer
    float *xres, *xnext;
    __half *y1h, *y1l, *y2h, *y2l;
    float2 *stats;
    float *q;
    __half *oh, *ol, *mh, *ml;
    float *part;
    const float2 *rope;
    unsigned *sync;
};

bool pf_supported(const Dims &dm);
// one block for the tokens of a pass: LayerNorm inputs, QKV, attention, dense, up, down
hipError_t launch_pf_layer(const PfParams &P, hipStream_t s);

}  // namespace cfpp
