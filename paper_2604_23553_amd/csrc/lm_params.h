// Arguments of the generation-loop kernels (lm_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "layout.h"

namespace cfpp {

constexpr int kLmPerThread = 16;     // hidden values a thread of the LM-head kernel normalises at most

struct LmParams {
    int h, vocab, max_seq;
    float eps;
    const __half *embed;             // [vocab][h]
    const __half *lnf_g, *lnf_b;     // [h]
    const __half *w_lm;              // [vocab][h], rows contiguous
    const int *tokens;               // [max_seq + 1], indexed by position
    int *tokens_out;                 // the same array, written at pos + 1
    const int *pos;
    int *pos_out;                    // the same word, advanced by one
    __half *x;                       // [h]: embedding row of tokens[pos]
    const __half *hidden;            // [h]: output of the stack
    float *logits;                   // [vocab] or null
    float *best;                     // [grid][2]: (logit, row) of every workgroup
    unsigned *sync;
    int rows;                        // LM-head rows per workgroup
};

hipError_t launch_lm_embed(const LmParams &L, hipStream_t s);
hipError_t launch_lm_head(const LmParams &L, int grid, int threads, hipStream_t s);   // head + pick
size_t lm_head_lds_bytes(const LmParams &L, int threads);
hipError_t prepare_lm_kernels(size_t lds_bytes);

}  // namespace cfpp
