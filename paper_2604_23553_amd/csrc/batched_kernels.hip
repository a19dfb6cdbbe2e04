// Several sequences per step (batch > 1, and groups of prompt tokens): the four
// projections of the block (paper Sec. 2.2) with the weights streamed ONCE for up
// to 8 sequences.  Here the path is a dense contraction - rows x K weights times
// K x batch activations - so it runs on the matrix cores.
//
// Which matrix instruction is decided by the memory side.  A wavefront load
// instruction (64 lanes x 16 bytes) that feeds v_mfma_f32_16x16x16_f16 covers
// 16 matrix rows x 64 bytes; with v_mfma_f32_4x4x4_16b_f16 (16 independent
// 4 x 4 x 4 blocks) the 16 blocks are 16 consecutive pieces of K, and the same
// instruction covers 4 rows x 256 contiguous bytes.  Measured on this GPU with
// pure loads over the 134 MB MLP-up matrix, two sets of four in flight per
// wavefront: 4.6 TB/s for the 16-row footprint, 6.0 TB/s for the 4-row one.
// The small blocks also waste nothing of the operand: 4 columns per block are
// 4 sequences, two instructions cover 8, where the 16-wide operand was half
// empty.
//
// Lane l of a wavefront: ri = l % 4, blk = l / 4.
//   A operand (weights):     row ri of the 4-row tile, 8 consecutive columns
//                            128 unit + 8 blk .. (two instructions of 4)
//   B operand (activations): sequence ri (and 4 + ri), the same 8 columns, from
//                            LDS; fp32 activations are split into an fp16 head
//                            and an fp16 remainder (y = hi + lo to ~2^-22), fp32
//                            accumulation: the result matches the fp32 FMA path
//                            to rounding
//   result:                  lane (j = l % 4, blk) holds rows 0..3 of sequence j
//                            (4 + j) for its piece of K; the 16 pieces are added
//                            by a fixed lane tree when the tile is done
// The 8 wavefronts interleave 128-column units (together 2 KiB contiguous per
// row and step); their per-tile sums go to LDS and are added in wavefront order:
// one bit pattern per build.
//
//   k_bat_qkv_up: both LayerNorms of every sequence (input and statistics once),
//                 QKV rows + bias, rotary, K/V append, q, then the MLP-up rows +
//                 bias + GELU
//   k_bat_out   : output projection of the attention output, then the MLP-down
//                 rows (K in slices of `hidden` through the same LDS), + biases +
//                 residual -> the block output
//
// Attention stays per sequence (every sequence has its own cache) and runs the
// attention kernel in between.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "decode_blocks.h"
#include "batched_params.h"

namespace cfpp {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

// halves between the activation rows in LDS: with hidden a multiple of 128 the rows of
// consecutive sequences start 16 banks apart, so the 16 lanes served together by a
// 16-byte LDS read (4 sequences x 4 pieces of 4 banks) hit 64 different banks
constexpr int kBatPad = 32;

__device__ __forceinline__ f16x4 lo_halves(u32x4 v)
{
    union { unsigned u[2]; f16x4 h; } c;
    c.u[0] = v.x; c.u[1] = v.y;
    return c.h;
}
__device__ __forceinline__ f16x4 hi_halves(u32x4 v)
{
    union { unsigned u[2]; f16x4 h; } c;
    c.u[0] = v.z; c.u[1] = v.w;
    return c.h;
}

// input of this layer for sequence b, element i
__device__ __forceinline__ float bat_x(const BatParams &P, int b, int i)
{
    if (P.layer == 0) return __half2float(P.x_in[(size_t)b * P.dm.h + i]);
    return P.xres[((size_t)b * 2 + ((P.layer - 1) & 1)) * P.dm.h + i];
}

// all positions of the group inside the cache?  (uniform over the grid)
__device__ __forceinline__ bool bat_positions_ok(const BatParams &P)
{
    bool ok = true;
    for (int b = 0; b < P.nb; ++b) {
        const int p = P.pos[b];
        ok = ok && p >= 0 && p < P.dm.max_seq;
    }
    if (!ok && threadIdx.x == 0 && blockIdx.x == 0)
        __hip_atomic_store(&P.sync[kSyncErr], (unsigned)kErrBadPos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return ok;
}

// One continuous stream over the matrices of a kernel.  A segment is rows
// [r_begin, r_begin + 4 nt) x `klen` columns of a row-major matrix inside the
// packed layer; every segment has the same klen (a multiple of 128), whose
// activations sit in LDS (columns 0..klen of yh/yl, row stride Ks) while the
// segment is worked on.  Segment 0 has its own description (A); segments 1..nB
// share one (B) and differ by a column offset that grows by `kstep` per segment
// (the MLP-down matrix in slices of `hidden` columns).  Per wavefront the sums
// of every row and sequence end up in red[(wave * kBatMax + seq) * rc + row] of
// the segment's description (segments from `acc_from` on add to what is there).
//
// A set is kBatSet = 4 load instructions: the same 128-column unit of four
// consecutive 4-row tiles (a group), so the activations of the unit are read
// from LDS once per set.  A wavefront's sets are ONE sequence - segment 0 group 0
// step 0, step 1, .., group 1 step 0, .., segment 1 .. - walked by two cursors,
// one for the requests and one three sets behind it for the arithmetic.  Every
// set is exactly four load instructions on one code path and the cursors advance
// without branches, so that the memory counter lets a wavefront work on one set
// while the next two are in flight (see GemvSpan); a load that has nothing to
// fetch (tiles past the share's last, sets that pad a segment to a multiple of
// three, everything past the end) reads one and the same 16 bytes in every lane:
// a single request.  The requests run on across the segments: when the
// arithmetic reaches a new segment, the caller's `boundary` (workgroup barriers
// around putting that segment's activations into LDS) runs with three sets of
// the new segment already on their way.  Lanes of sequences that do not exist
// read some row of the LDS region: their products land in columns of the result
// that are never looked at.
constexpr int kBatSet = 4;
constexpr int kBatCtrWords = 4;      // LDS words kept for the counter of k_bat_qkv_up (16 bytes: what follows stays aligned)
constexpr int kBatDepth = 3;         // sets in flight per wavefront (4 and more spill registers and are slower)

struct BatSeg {
    unsigned base;            // byte offset of the matrix (first column of the segment's range) in the packed layer
    unsigned row_bytes;       // row length of the matrix * 2
    int r_begin, r_n;         // first row, valid rows
    float *red;               // sums: [8 wavefronts][kBatMax][rc]
    int rc;
};

struct BatStream {
    struct Seg {              // a description as the cursors use it
        unsigned base, row_bytes;
        int nt, ng, sets, sets_padded;       // tiles, groups of 4 tiles, sets = ng * S, rounded up to a multiple of 3
        unsigned lane_full, lane_last;       // bytes: this lane's row inside a tile + its column piece (last tile: rows past the end re-read the last valid row)
        float *red;           // this wavefront's sums at sequence ri
        int rc;
    };
    const __half *W;          // packed layer (uniform)
    Seg A, B;
    int nseg;                 // 1 + number of B segments
    unsigned kstep;           // bytes between the column ranges of consecutive B segments
    int acc_from;             // segments >= acc_from add to the sums already there
    bool carry;               // all segments cover the same single group of rows and add up: the sums stay in
                              // registers until the last segment
    int ri, wave;
    int S, units;             // steps per group, 128-column units per row
    const __half *yh0, *yh1, *yl0, *yl1;   // sequences ri and 4 + ri at this lane's first column
    int iseg, ig, is, iset;   // request cursor: segment, group, step, set within the segment
    int cseg, cg, cs, cset;   // arithmetic cursor
    u32x4 r[kBatDepth][kBatSet];
    f32x4 acc[kBatSet][2];

    __device__ __forceinline__ void make(Seg &d, const BatSeg &g, int blk) const
    {
        d.base = g.base; d.row_bytes = g.row_bytes;
        d.nt = (g.r_n + 3) >> 2;
        d.ng = (d.nt + 3) >> 2;
        d.sets = d.ng * S;
        d.sets_padded = (d.sets + kBatDepth - 1) / kBatDepth * kBatDepth;
        const int in_last = g.r_n - 4 * (d.nt - 1);                        // valid rows of the last tile (1..4)
        d.lane_full = ((unsigned)g.r_begin + (unsigned)ri) * g.row_bytes + (unsigned)(16 * blk);
        d.lane_last = ((unsigned)g.r_begin + (unsigned)min(ri, in_last - 1)) * g.row_bytes + (unsigned)(16 * blk);
        d.rc = g.rc;
        d.red = g.red + ((size_t)wave * kBatMax + ri) * g.rc;
    }

    // the description in use, member by member (a reference to one of the two would put both in memory)
    __device__ __forceinline__ Seg pick(bool first) const
    {
        Seg d;
        d.base = first ? A.base : B.base; d.row_bytes = first ? A.row_bytes : B.row_bytes;
        d.nt = first ? A.nt : B.nt; d.ng = first ? A.ng : B.ng;
        d.sets = first ? A.sets : B.sets; d.sets_padded = first ? A.sets_padded : B.sets_padded;
        d.lane_full = first ? A.lane_full : B.lane_full; d.lane_last = first ? A.lane_last : B.lane_last;
        d.red = first ? A.red : B.red; d.rc = first ? A.rc : B.rc;
        return d;
    }

    __device__ __forceinline__ void issue(u32x4 (&r)[kBatSet])
    {
        const bool first = iseg == 0, live = iseg < nseg;
        const Seg d = pick(first);
        const int nt = d.nt;
        const bool real_set = live && iset < d.sets && 8 * is + wave < units;     // (a wavefront past the row's end in the last step: nothing to fetch)
        const int unit = 8 * is + wave;
        const unsigned set_off = d.base + (first ? 0u : (unsigned)(iseg - 1) * kstep) + 256u * (unsigned)unit;
        const unsigned tile_bytes = 4u * d.row_bytes;
#pragma unroll
        for (int j = 0; j < kBatSet; ++j) {
            const int tile = 4 * ig + j;
            const unsigned off = set_off + (unsigned)tile * tile_bytes + (tile == nt - 1 ? d.lane_last : d.lane_full);
            r[j] = load16_stream_at(W, real_set && tile < nt ? off : 16u * (unsigned)j);   // (distinct, or the four become one load and three copies)
        }
        __builtin_amdgcn_sched_barrier(0);
        const int padded = live ? d.sets_padded : 0x7fffffff;
        const int s1 = is + 1, swrap = (int)(s1 == S);
        const int n1 = iset + 1, nwrap = (int)(n1 >= padded);
        is = nwrap ? 0 : s1 - swrap * S;
        ig = nwrap ? 0 : ig + swrap;
        iset = nwrap ? 0 : n1;
        iseg += nwrap;
    }

    // the 16 pieces of K (lanes of equal l % 4) added by a fixed tree; every lane gets the total
    // (rows of 16 lanes: rotations inside a row, then the rows pairwise and the halves of the wavefront
    // through the lane-swap instructions, which exchange odd rows of one operand with even rows of the
    // other, resp. upper and lower 32 lanes)
    static __device__ __forceinline__ float pieces_sum(float v)
    {
        v += dpp_mov<kDppRor4>(v);
        v += dpp_mov<kDppRor8>(v);
        const unsigned u = __float_as_uint(v);
        const auto p = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        v = __uint_as_float(p[0]) + __uint_as_float(p[1]);
        const unsigned u2 = __float_as_uint(v);
        const auto q = __builtin_amdgcn_permlane32_swap(u2, u2, false, false);
        return __uint_as_float(q[0]) + __uint_as_float(q[1]);
    }

    __device__ __forceinline__ void finish_tile(const Seg &d, int j, int tile)
    {
        f32x4 t0, t1;
#pragma unroll
        for (int i = 0; i < 4; ++i) { t0[i] = pieces_sum(acc[j][0][i]); t1[i] = pieces_sum(acc[j][1][i]); }
        if ((threadIdx.x & 63) < 4) {
            f32x4 *d0 = reinterpret_cast<f32x4 *>(d.red + 4 * tile), *d1 = reinterpret_cast<f32x4 *>(d.red + 4 * d.rc + 4 * tile);
            if (cseg >= acc_from && !carry) { t0 += *d0; t1 += *d1; }
            *d0 = t0; *d1 = t1;
        }
        acc[j][0] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc[j][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // one set of the current segment (cseg, fixed by the caller's loop)
    __device__ __forceinline__ void consume(const u32x4 (&r)[kBatSet])
    {
        const Seg d = pick(cseg == 0);
        if (cset < d.sets) {                                              // (uniform)
            const int nt = d.nt;
            if (8 * cs + wave < units) {                                  // (uniform)
                const int at = 1024 * cs;
                const u32x4 h0 = *reinterpret_cast<const u32x4 *>(yh0 + at), h1 = *reinterpret_cast<const u32x4 *>(yh1 + at);
                const u32x4 l0 = *reinterpret_cast<const u32x4 *>(yl0 + at), l1 = *reinterpret_cast<const u32x4 *>(yl1 + at);
#pragma unroll
                for (int j = 0; j < kBatSet; ++j) {
                    if (4 * cg + j < nt) {                                // (uniform)
                        const f16x4 wa = lo_halves(r[j]), wb = hi_halves(r[j]);
                        f32x4 c0 = acc[j][0], c1 = acc[j][1];
                        c0 = __builtin_amdgcn_mfma_f32_4x4x4f16(wa, lo_halves(h0), c0, 0, 0, 0);
                        c1 = __builtin_amdgcn_mfma_f32_4x4x4f16(wa, lo_halves(h1), c1, 0, 0, 0);
                        c0 = __builtin_amdgcn_mfma_f32_4x4x4f16(wb, hi_halves(h0), c0, 0, 0, 0);
                        c1 = __builtin_amdgcn_mfma_f32_4x4x4f16(wb, hi_halves(h1), c1, 0, 0, 0);
                        c0 = __builtin_amdgcn_mfma_f32_4x4x4f16(wa, lo_halves(l0), c0, 0, 0, 0);
                        c1 = __builtin_amdgcn_mfma_f32_4x4x4f16(wa, lo_halves(l1), c1, 0, 0, 0);
                        c0 = __builtin_amdgcn_mfma_f32_4x4x4f16(wb, hi_halves(l0), c0, 0, 0, 0);
                        c1 = __builtin_amdgcn_mfma_f32_4x4x4f16(wb, hi_halves(l1), c1, 0, 0, 0);
                        acc[j][0] = c0; acc[j][1] = c1;
                    }
                }
            }
            if (cs == S - 1 && (!carry || cseg == nseg - 1)) {            // (uniform) the group is complete
#pragma unroll
                for (int j = 0; j < kBatSet; ++j)
                    if (4 * cg + j < nt) finish_tile(d, j, 4 * cg + j);
            }
        }
        const int s1 = cs + 1, swrap = (int)(s1 == S);
        ++cset; cs = s1 - swrap * S; cg += swrap;
    }

    // Requests the first three sets: weights depend on nothing, so this comes before the
    // activations are even in LDS (yh, yl are only read by run()).  nB B segments follow
    // segment A; a description without rows has no sets.
    __device__ __forceinline__ void begin(const __half *W_, const BatSeg &A_, const BatSeg &B_, int nB, unsigned kstep_,
                                          int acc_from_, int klen, const __half *yh, const __half *yl, int Ks, int tid)
    {
        const int lane = tid & 63;
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        ri = lane & 3;
        const int blk = lane >> 2;
        W = W_;
        units = klen >> 7;
        S = (units + 7) >> 3;
        make(A, A_, blk);
        make(B, B_, blk);
        if (B.nt <= 0) nB = 0;
        nseg = 1 + nB; kstep = kstep_; acc_from = acc_from_;
        carry = acc_from_ == 1 && A.ng == 1 && B.ng == 1 && A_.red == B_.red && A_.r_begin == B_.r_begin && A_.r_n == B_.r_n;
        const int col = 128 * wave + 8 * blk;
        yh0 = yh + ri * Ks + col; yh1 = yh + (4 + ri) * Ks + col;
        yl0 = yl + ri * Ks + col; yl1 = yl + (4 + ri) * Ks + col;
        iseg = A.nt > 0 ? 0 : 1;
        ig = is = iset = 0;
#pragma unroll
        for (int j = 0; j < kBatSet; ++j) {
            acc[j][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc[j][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int k = 0; k < kBatDepth; ++k) issue(r[k]);
    }
    // boundary(seg) runs in front of every segment >= 1 (also when segment 0 has no rows);
    // prefetch(seg) runs three sets before the end of segment seg - 1: what it requests is
    // followed by exactly three sets of weight requests on a straight path to boundary(seg),
    // so the wait for it there does not drain the weights behind it.
    template <class Prefetch, class Boundary>
    __device__ __forceinline__ void run(Prefetch prefetch, Boundary boundary)
    {
        for (cseg = 0; cseg < nseg; ++cseg) {
            if (cseg > 0) boundary(cseg);
            const int padded = cseg == 0 ? A.sets_padded : B.sets_padded;
            cg = cs = cset = 0;
            for (int n = 0; n + kBatDepth < padded; n += kBatDepth) {
#pragma unroll
                for (int k = 0; k < kBatDepth; ++k) { consume(r[k]); issue(r[k]); }
            }
            if (cseg + 1 < nseg) prefetch(cseg + 1);
            if (padded > 0) {
#pragma unroll
                for (int k = 0; k < kBatDepth; ++k) { consume(r[k]); issue(r[k]); }
            }
        }
    }
};

// row of sequence b: the wavefronts' sums added in order
__device__ __forceinline__ float bat_total(const float *red, int rc, int row, int b)
{
    float s = 0.f;
    for (int w = 0; w < 8; ++w) s += red[((size_t)w * kBatMax + b) * rc + row];
    return s;
}

// 8 consecutive fp32 values -> fp16 heads and remainders, one 16-byte LDS write each
__device__ __forceinline__ void bat_put8(__half *yh, __half *yl, int at, const float (&v)[8])
{
    union { __half h[8]; u32x4 u; } hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi.h[e] = __float2half_rn(v[e]);
        lo.h[e] = __float2half_rn(v[e] - __half2float(hi.h[e]));
    }
    *reinterpret_cast<u32x4 *>(yh + at) = hi.u;
    *reinterpret_cast<u32x4 *>(yl + at) = lo.u;
}

// The 8-column chunk of the activation rows that a thread owns (index in chunks, -1: none): one
// inside the 128-column units of its own wavefront (unit = wave + 8 k, the columns the wavefront's
// sets read; 16 chunks per unit).  What a wavefront reads from the activations in LDS it has then
// written itself, in program order: the stream needs no workgroup barrier around an exchange of
// activations, and the wavefronts do not wait for one another there.
__device__ __forceinline__ int bat_chunk(int tid, int klen)
{
    const int lane = tid & 63, unit = (tid >> 6) + 8 * (lane >> 4);
    return unit < (klen >> 7) ? 16 * unit + (lane & 15) : -1;
}

// src[b * stride + 0..klen) (fp32, klen <= 4096 a multiple of 128) of every sequence -> hi/lo rows in
// LDS: a thread owns one group of 8 values of every sequence; load() requests them all,
// commit() converts and writes (other loads can be queued in between)
struct BatStage {
    f32x4 v[kBatMax][2];
    __device__ __forceinline__ void load(const float *src, size_t stride, int klen, int nb, int tid)
    {
        const int ch = bat_chunk(tid, klen), c = ch < 0 ? 0 : ch;
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            const float *p = src + (size_t)(b < nb ? b : 0) * stride + 8 * c;
            v[b][0] = *as_global(reinterpret_cast<const f32x4 *>(p));
            v[b][1] = *as_global(reinterpret_cast<const f32x4 *>(p + 4));
        }
    }
    __device__ __forceinline__ void commit(int klen, __half *yh, __half *yl, int Ks, int nb, int tid) const
    {
        const int ch = bat_chunk(tid, klen);
        if (ch >= 0) {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b) {
                if (b < nb) {
                    const float e[8] = {v[b][0][0], v[b][0][1], v[b][0][2], v[b][0][3], v[b][1][0], v[b][1][1], v[b][1][2], v[b][1][3]};
                    bat_put8(yh, yl, b * Ks + 8 * ch, e);
                }
            }
        }
    }
};

// The two LayerNorms of every sequence share input and statistics, and neither is waited
// for: the matrices run on gamma * x, which needs no statistics, and the epilogues complete
//   W (gamma (x - mu) inv + beta) + b = inv (W (gamma x) - mu s) + c
// with the two constants per row, s = W gamma and c = W beta + b, that the packing left
// behind the tensors (PackedLayout::rc_qkv, rc_up; paper Sec. 2.2 for the operation).
// A thread owns one group of 8 elements of every sequence (bat_chunk; hidden <= 4096).  Mean
// and variance (two passes, biased) are summed per wavefront into `stat` (2 * 8 * kBatMax
// floats) and added in wavefront order by whoever needs them; a counter in LDS says when
// all wavefronts' sums of the first pass are there.
struct BatLn {
    u32x4 raw16[kBatMax];          // layer 0: fp16 input
    f32x4 raw32[kBatMax][2];       // later layers: fp32 residual stream
    u32x4 graw[2];
    float xv[kBatMax][8];

    __device__ __forceinline__ void load(const BatParams &P, int tid)
    {
        const int h = P.dm.h;
        const int ch = bat_chunk(tid, h), c = ch < 0 ? 0 : ch;
        if (P.layer == 0) {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b)
                raw16[b] = *as_global(reinterpret_cast<const u32x4 *>(P.x_in + (size_t)(b < P.nb ? b : 0) * h + 8 * c));
        } else {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b) {
                const float *p = P.xres + ((size_t)(b < P.nb ? b : 0) * 2 + ((P.layer - 1) & 1)) * h + 8 * c;
                raw32[b][0] = *as_global(reinterpret_cast<const f32x4 *>(p));
                raw32[b][1] = *as_global(reinterpret_cast<const f32x4 *>(p + 4));
            }
        }
        const __half *w = P.w;
        graw[0] = *as_global(reinterpret_cast<const u32x4 *>(w + P.lay.ln1_g + 8 * c));
        graw[1] = *as_global(reinterpret_cast<const u32x4 *>(w + P.lay.ln2_g + 8 * c));
    }

    __device__ __forceinline__ void unpack(const BatParams &P)
    {
        if (P.layer == 0) {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b) {
                const float2 a0 = unpack_h2(raw16[b].x), a1 = unpack_h2(raw16[b].y), a2 = unpack_h2(raw16[b].z), a3 = unpack_h2(raw16[b].w);
                xv[b][0] = a0.x; xv[b][1] = a0.y; xv[b][2] = a1.x; xv[b][3] = a1.y;
                xv[b][4] = a2.x; xv[b][5] = a2.y; xv[b][6] = a3.x; xv[b][7] = a3.y;
            }
        } else {
#pragma unroll
            for (int b = 0; b < kBatMax; ++b)
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[b][e] = raw32[b][e >> 2][e & 3];
        }
    }

    // which: 0 = gamma of the LayerNorm in front of QKV, 1 = of the one in front of the MLP
    __device__ __forceinline__ void write_scaled(const BatParams &P, int which, __half *yh, __half *yl, int Ks, int tid) const
    {
        const int ch = bat_chunk(tid, P.dm.h);
        if (ch < 0) return;
        const u32x4 g = graw[which];
        const float2 g0 = unpack_h2(g.x), g1 = unpack_h2(g.y), g2 = unpack_h2(g.z), g3 = unpack_h2(g.w);
        const float gv[8] = {g0.x, g0.y, g1.x, g1.y, g2.x, g2.y, g3.x, g3.y};
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            if (b < P.nb) {
                float yv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) yv[e] = xv[b][e] * gv[e];
                bat_put8(yh, yl, b * Ks + 8 * ch, yv);
            }
        }
    }

    // pass 1: this wavefront's sums of every sequence -> stat[wave][b]
    __device__ __forceinline__ void sums(const BatParams &P, float *stat, int tid) const
    {
        const int lane = tid & 63, wave = tid >> 6;
        const bool active = bat_chunk(tid, P.dm.h) >= 0;
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s += xv[b][e];
            s = wave_sum(active ? s : 0.f);
            if (lane == 0) stat[wave * kBatMax + b] = s;
        }
    }
    static __device__ __forceinline__ float mean_of(const BatParams &P, const float *stat, int b)
    {
        float s = 0.f;
        for (int w = 0; w < 8; ++w) s += stat[w * kBatMax + b];
        return s / (float)P.dm.h;
    }
    // pass 2 (the sums of pass 1 are visible): squared deviations -> stat[8 * kBatMax + wave * kBatMax + b]
    __device__ __forceinline__ void squares(const BatParams &P, float *stat, int tid) const
    {
        const int lane = tid & 63, wave = tid >> 6;
        const bool active = bat_chunk(tid, P.dm.h) >= 0;
        float *stat2 = stat + 8 * kBatMax;
#pragma unroll
        for (int b = 0; b < kBatMax; ++b) {
            const float mean = mean_of(P, stat, b);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dlt = xv[b][e] - mean;
                s += dlt * dlt;
            }
            s = wave_sum(active ? s : 0.f);
            if (lane == 0) stat2[wave * kBatMax + b] = s;
        }
    }
    static __device__ __forceinline__ float inv_of(const BatParams &P, const float *stat, int b)
    {
        const float *stat2 = stat + 8 * kBatMax;
        float s = 0.f;
        for (int w = 0; w < 8; ++w) s += stat2[w * kBatMax + b];
        return 1.0f / sqrtf(s / (float)P.dm.h + P.dm.ln_eps);
    }
};

// QKV rows of this workgroup from the wavefronts' sums: LayerNorm completion (which brings the
// bias), rotary, K/V append, q.  Pairs of adjacent packed rows (a rotary pair sits in one), as in
// the per-sequence epilogue.
__device__ __forceinline__ void bat_finish_qkv(const BatParams &P, const float *red, int rc, int r_begin, int r_n, int b,
                                               float mean, float inv, int tid)
{
    const Dims &dm = P.dm;
    const float2 *rcq = reinterpret_cast<const float2 *>(P.w + P.lay.rc_qkv);
    const int h = dm.h, d = dm.d, r = dm.r, pos = P.pos[b];
    for (int pr = tid >> 3; 2 * pr < r_n; pr += 64) {
        const int p = r_begin + 2 * pr;                    // packed row, even (rows is even)
        const int pd = p / d, i = p - pd * d;
        const int nh = pd / 3, c = pd - 3 * nh;
        const float2 k0 = rcq[p], k1 = rcq[p + 1];
        float v0 = (bat_total(red, rc, 2 * pr, b) - mean * k0.x) * inv + k0.y;
        float v1 = (bat_total(red, rc, 2 * pr + 1, b) - mean * k1.x) * inv + k1.y;
        int d0 = i, d1 = i + 1;
        if (c < 2 && i < r) {
            const float2 cs = P.rope[(size_t)pos * (r >> 1) + (i >> 1)];
            const float lo = v0 * cs.x - v1 * cs.y, hi = v1 * cs.x + v0 * cs.y;
            v0 = lo; v1 = hi;
            d0 = i >> 1; d1 = (i >> 1) + (r >> 1);
        }
        if (c == 0) {
            P.q[(size_t)b * h + nh * d + d0] = v0;
            P.q[(size_t)b * h + nh * d + d1] = v1;
        } else {
            P.kv[kv_offset(dm, c - 1, P.kv_b0 + b * P.kv_bstep, nh, d0, pos)] = __float2half_rn(v0);
            P.kv[kv_offset(dm, c - 1, P.kv_b0 + b * P.kv_bstep, nh, d1, pos)] = __float2half_rn(v1);
        }
    }
}

// rows of a workgroup's share, rounded up to whole 4-row tiles
__host__ __device__ __forceinline__ int bat_rc(int rows) { return (rows + 3) & ~3; }

// LayerNorms, QKV rows and MLP-up rows of a layer in one launch: the input is read and
// its statistics are worked out once, and the two matrices are one stream: the MLP-up
// weights are on their way while the second normalised input replaces the first in LDS.
// A workgroup owns P.rows QKV rows and P.rows2 MLP-up rows; either share may be empty at
// the end of the grid.  LDS: activations (heads, remainders) | LayerNorm sums | counter | QKV sums |
// MLP-up sums.
__global__ void __launch_bounds__(512) k_bat_qkv_up(BatParams P)
{
    extern __shared__ __align__(16) float lds[];
    if (!bat_positions_ok(P)) return;
    const Dims &dm = P.dm;
    const int h = dm.h, tid = threadIdx.x, Ks = h + kBatPad;
    __half *yh = reinterpret_cast<__half *>(lds), *yl = yh + kBatMax * Ks;
    const int q_begin = blockIdx.x * P.rows, q_n = max(0, min(P.rows, 3 * h - q_begin));
    const int u_begin = blockIdx.x * P.rows2, u_n = max(0, min(P.rows2, dm.f - u_begin));
    if (q_n == 0 && u_n == 0) return;                      // (whole workgroup)
    const __half *w = P.w;
    float *stat = reinterpret_cast<float *>(yl + kBatMax * Ks);     // behind the activations
    int *ctr = reinterpret_cast<int *>(stat + 2 * 8 * kBatMax);    // wavefronts whose first-pass sums are in `stat`
    const int rcq = bat_rc(P.rows), rcu = bat_rc(P.rows2);
    float *redq = stat + 2 * 8 * kBatMax + kBatCtrWords, *redu = redq + 8 * kBatMax * rcq;
    if (tid == 0) *ctr = 0;
    __syncthreads();                                       // the only meeting before the sums are added: nothing is in flight yet
    // order of the requests: the layer input, then the first weights; a wavefront puts gamma * x of
    // its own columns into LDS as soon as its part of the input is here and starts on its sets
    BatLn ln;
    ln.load(P, tid);
    const BatSeg sq{(unsigned)P.lay.w_qkv * 2u, (unsigned)h * 2u, q_begin, q_n, redq, rcq};
    const BatSeg su{(unsigned)P.lay.w_up * 2u, (unsigned)h * 2u, u_begin, u_n, redu, rcu};
    BatStream bs;
    bs.begin(w, sq, su, 1, 0u, 2, h, yh, yl, Ks, tid);
    ln.unpack(P);
    ln.write_scaled(P, 0, yh, yl, Ks, tid);
    ln.sums(P, stat, tid);
    lds_signal(ctr, tid & 63);
    bool squared = false;
    bs.run([](int) {}, [&](int) {
        lds_await(ctr, 8, P.sync);                         // (long since reached) the means can be formed
        ln.squares(P, stat, tid);
        squared = true;
        ln.write_scaled(P, 1, yh, yl, Ks, tid);            // this wavefront's columns: it alone reads them
    });
    if (!squared) {                                        // (uniform: no MLP-up rows in this workgroup)
        lds_await(ctr, 8, P.sync);
        ln.squares(P, stat, tid);
    }
    __syncthreads();
    const int b = tid & (kBatMax - 1);
    if (b >= P.nb) return;
    const float mean = BatLn::mean_of(P, stat, b), inv = BatLn::inv_of(P, stat, b);
    bat_finish_qkv(P, redq, rcq, q_begin, q_n, b, mean, inv, tid);
    const float2 *rcup = reinterpret_cast<const float2 *>(w + P.lay.rc_up);
    for (int row = tid >> 3; row < u_n; row += 64) {
        const float2 k = rcup[u_begin + row];
        P.m[(size_t)b * dm.f + u_begin + row] = gelu_act((bat_total(redu, rcu, row, b) - mean * k.x) * inv + k.y, dm.flags);
    }
}

// Output projection of the attention output, then the MLP-down rows with GELU(up) in
// slices of `hidden` columns through the same LDS, all added into the same sums; one
// stream over the five pieces: the next slice's activations are requested three sets
// before a segment ends and the next segment's weights are on their way while they are
// put into LDS.
__global__ void __launch_bounds__(512) k_bat_out(BatParams P)
{
    extern __shared__ __align__(16) float lds[];
    if (!bat_positions_ok(P)) return;
    const Dims &dm = P.dm;
    const int h = dm.h, f = dm.f, tid = threadIdx.x, Ks = h + kBatPad;
    __half *yh = reinterpret_cast<__half *>(lds), *yl = yh + kBatMax * Ks;
    const int r_begin = blockIdx.x * P.rows, r_n = max(0, min(P.rows, h - r_begin));
    if (r_n == 0) return;
    const __half *w = P.w;
    const int rc = bat_rc(P.rows), nslices = f / h;
    float *red = reinterpret_cast<float *>(yl + kBatMax * Ks);
    const BatSeg sd{(unsigned)P.lay.w_dense * 2u, (unsigned)h * 2u, r_begin, r_n, red, rc};
    const BatSeg sm{(unsigned)P.lay.w_down * 2u, (unsigned)f * 2u, r_begin, r_n, red, rc};
    BatStage st;
    BatStream bs;
    st.load(P.o, (size_t)h, h, P.nb, tid);
    bs.begin(w, sd, sm, nslices, (unsigned)h * 2u, 1, h, yh, yl, Ks, tid);
    st.commit(h, yh, yl, Ks, P.nb, tid);                   // this wavefront's columns: no meeting, here or between the segments
    bs.run([&](int seg) {                                  // seg = 1..nslices: slice seg - 1 of GELU(up), into registers
        st.load(P.m + (size_t)(seg - 1) * h, (size_t)f, h, P.nb, tid);
    }, [&](int) {
        st.commit(h, yh, yl, Ks, P.nb, tid);
    });
    __syncthreads();
    const int b = tid & (kBatMax - 1);
    if (b >= P.nb) return;
    const __half *bde = w + P.lay.b_dense, *bdn = w + P.lay.b_down;
    const bool last = P.layer == P.n_layers - 1;
    for (int row = tid >> 3; row < r_n; row += 64) {
        const int i = r_begin + row;
        const float branches = (bat_total(red, rc, row, b) + __half2float(bde[i])) + __half2float(bdn[i]);
        const float res = bat_x(P, b, i) + branches;
        if (last) P.out[(size_t)b * h + i] = __float2half_rn(res);
        else P.xres[((size_t)b * 2 + (P.layer & 1)) * h + i] = res;
    }
}

static void bat_rows(const Dims &dm, int grid, int *rows_qkv, int *rows_up, int *rows_h)
{
    *rows_qkv = (((3 * dm.h + grid - 1) / grid) + 1) & ~1;   // even: a rotary pair stays in one workgroup
    *rows_up = (dm.f + grid - 1) / grid;
    *rows_h = (dm.h + grid - 1) / grid;
}

// the larger of the two kernels' needs
size_t bat_lds_bytes(const Dims &dm, int grid)
{
    int rq, ru, rh;
    bat_rows(dm, grid, &rq, &ru, &rh);
    const size_t act = (size_t)2 * kBatMax * (dm.h + kBatPad) * sizeof(__half);
    const size_t qkv_up = act + (2 * 8 * kBatMax + kBatCtrWords + (size_t)8 * kBatMax * (bat_rc(rq) + bat_rc(ru))) * sizeof(float);
    const size_t out = act + (size_t)8 * kBatMax * bat_rc(rh) * sizeof(float);
    return qkv_up > out ? qkv_up : out;
}

bool bat_supported(const Dims &dm, int grid, int threads)
{
    // 8 wavefronts interleave units of 128 columns; the MLP-down matrix goes in slices of `hidden`
    // columns; the LayerNorm keeps hidden / 64 values per lane; the 32-bit byte offsets of the loads span a whole matrix; everything fits the LDS
    int rq, ru, rh;
    bat_rows(dm, grid, &rq, &ru, &rh);
    const int rows_max = ru > rq ? ru : rq;
    return threads == 512 && grid >= 1 && dm.h % 128 == 0 && dm.f % dm.h == 0 && dm.h <= 64 * kBatLnPerLane && rows_max <= 64 &&
           (unsigned long long)packed_layout(dm.h, dm.f).total * 2 < (1ull << 32) && bat_lds_bytes(dm, grid) <= 160 * 1024;
}

hipError_t launch_bat_qkv_up(BatParams P, int grid, hipStream_t s)
{
    int rh;
    bat_rows(P.dm, grid, &P.rows, &P.rows2, &rh);
    hipLaunchKernelGGL(k_bat_qkv_up, dim3(grid), dim3(512), bat_lds_bytes(P.dm, grid), s, P);
    return hipGetLastError();
}

hipError_t launch_bat_out(BatParams P, int grid, hipStream_t s)
{
    int rq, ru;
    bat_rows(P.dm, grid, &rq, &ru, &P.rows);
    hipLaunchKernelGGL(k_bat_out, dim3(grid), dim3(512), bat_lds_bytes(P.dm, grid), s, P);
    return hipGetLastError();
}

hipError_t prepare_bat_kernels(size_t lds_bytes)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_bat_qkv_up),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_bat_out), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)lds_bytes);
}

}  // namespace cfpp
