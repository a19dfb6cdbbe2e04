// Arguments the host passes (by value) to the decode kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "layout.h"

namespace cfpp {

struct StepParams {
    Dims dm;
    PackedLayout lay;
    // workspace views (already offset to this sequence where per-sequence)
    unsigned *sync;
    unsigned *seg_cnt;   // [H] for this sequence
    const float2 *rope;
    float *xres;         // [2][h] for this sequence
    float *q, *m, *g, *o;
    float *part;         // [H][part_slots][d+2] for this sequence
    float *tagged;       // tagged-word region (value, tag pairs): x[2][h], (3 h unused), o[h], part[H][part_slots][d+2]
    int part_slots;
    const int *pos;      // device, this sequence's position
    int b;               // sequence index inside the KV cache
    const __half *x_in;  // fp16 [h] input of layer 0
    __half *out;         // fp16 [h] output of the last layer
    int n_layers;
    int attn_g0, attn_G; // attention: the workgroups [attn_g0, attn_g0 + attn_G) share this sequence (attn_G 0: the whole grid)
    int attn_bstep;      // batched attention launch: row i reads the cache of sequence b + i * attn_bstep (1, or 0
                         // when the rows are consecutive positions of one sequence)
    int parts;           // kPart* bits: what a phase launch performs (kPartAll unless the block runs in two halves)
    // work split (chosen on the host from the grid and the workgroup size)
    int rows_qkv, rows_up, rows_h;   // matrix rows per workgroup (rows_qkv even)
    // whole-stack kernel: the MLP in two halves - up rows [0, f_a) and [f_a, f), rows of each per workgroup
    int f_a, rows_up_a, rows_up_b;
    int nsl_down, nsl_dense;         // K-slices per row for the two GEMVs with few rows
    unsigned lds_floats;             // dynamic LDS the launch provides, in floats
    int debug;                       // profiling library only (0 otherwise): bit mask of parts to skip (results
                                     // are then wrong); bit 16: workgroup (debug >> 8) records a timeline into `trace`
    unsigned long long *trace;
    // whole-stack kernel launched for one block on its own (no pointer table): that block's weights and cache
    const __half *w_single;
    __half *kv_single;
};

struct LayerPtrs {
    const __half *w[kMaxLayers];
    __half *kv[kMaxLayers];
};

// implemented in decode_kernels.hip
hipError_t launch_phases(const StepParams &P, const __half *w, __half *kv, int layer,
                         int grid, int threads, hipStream_t s);
hipError_t launch_block_persistent(const StepParams &P, const __half *w, __half *kv, int layer,
                                   int grid, int threads, hipStream_t s);
hipError_t launch_attention_only(StepParams P, const __half *w, const __half *kv, int grid, int threads, hipStream_t s);
// the attention of nb sequences (P: the first one's parameters) in one launch, workgroups dealt by cache length
hipError_t launch_attention_batched(StepParams P, int nb, const __half *w, const __half *kv, int grid, int threads,
                                    hipStream_t s);
// stores the per-layer pointer table in device memory (the whole-stack kernels read it there)
hipError_t launch_store_layer_ptrs(const LayerPtrs &ptrs, LayerPtrs *dst, int n, hipStream_t s);
// most co-resident workgroups per compute unit for the persistent kernels
hipError_t persistent_occupancy(int head_dim, int threads, size_t lds_bytes, int *blocks_per_cu);
hipError_t prepare_kernels(size_t lds_bytes);

// implemented in fused_kernel.hip: the whole-stack kernel with hidden hand-overs (mode 2)
bool fused_supported(const Dims &dm, const StepParams &P, int grid, int threads);
size_t fused_lds_bytes(const Dims &dm, const StepParams &P, int threads);
hipError_t launch_stack_fused(const StepParams &P, const LayerPtrs *ptrs, int grid, int threads, hipStream_t s);
hipError_t fused_occupancy(int head_dim, int threads, size_t lds_bytes, int *blocks_per_cu);
hipError_t prepare_fused_kernels(size_t lds_bytes);

// implemented in prep_kernels.hip
hipError_t launch_pack_layer(const Dims &dm, const PackedLayout &lay, const void *const src[12],
                             __half *dst, hipStream_t s);
hipError_t launch_kv_import(const Dims &dm, const __half *k_src, const __half *v_src, int src_cap,
                            int n_pos, int b, __half *kv, hipStream_t s);
hipError_t launch_kv_export(const Dims &dm, const __half *kv, int b, int pos_begin, int n_pos,
                            int dst_cap, __half *k_dst, __half *v_dst, hipStream_t s);

// dst[i] = first + i for i < n (the positions of a prompt's tokens)
hipError_t launch_fill_positions(int *dst, int first, int n, hipStream_t s);

hipError_t launch_stream_read(const void *src, size_t bytes, unsigned *sink, int grid, int threads,
                              int unroll, hipStream_t s);
hipError_t launch_stream_copy(const void *src, void *dst, size_t bytes, int grid, int threads, hipStream_t s);

}  // namespace cfpp
