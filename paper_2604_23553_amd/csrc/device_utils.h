// Wavefront-level building blocks for gfx950 (wave64): DPP reductions, fp16
// unpacking, 128-bit streaming loads, and the grid barrier used by the
// persistent kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "layout.h"

namespace cfpp {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Pointers that come out of a table in memory (per-layer weights, KV caches) lose
// their address space; the explicit global address space keeps the compiler from
// emitting FLAT instructions (which also tie up the LDS counter) for them.
#define CFPP_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ CFPP_GLOBAL T *as_global(T *p)
{
    return (CFPP_GLOBAL T *)p;
}

// ---- data-parallel-primitive lane exchanges (row = 16 lanes) ---------------
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <- lane 7-i within each 8
constexpr int kDppMirror = 0x140;     // lane i <- lane 15-i within each 16
constexpr int kDppRor4 = 0x124;       // rotate right by 4 within each 16
constexpr int kDppRor8 = 0x128;       // rotate right by 8 within each 16

__device__ __forceinline__ float readlane_f(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Sum over the 64 lanes, same value returned in every lane.  Fixed tree.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_mov<kDppXor1>(v);
    v += dpp_mov<kDppXor2>(v);
    v += dpp_mov<kDppHalfMirror>(v);
    v += dpp_mov<kDppMirror>(v);      // every lane: sum of its row of 16
    return (readlane_f(v, 0) + readlane_f(v, 16)) + (readlane_f(v, 32) + readlane_f(v, 48));
}

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_mov<kDppXor1>(v));
    v = fmaxf(v, dpp_mov<kDppXor2>(v));
    v = fmaxf(v, dpp_mov<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_mov<kDppMirror>(v));
    return fmaxf(fmaxf(readlane_f(v, 0), readlane_f(v, 16)), fmaxf(readlane_f(v, 32), readlane_f(v, 48)));
}

// Sum over the 32 lanes that share this lane's parity (lane & 1); every lane
// gets its parity's total.  Fixed tree.
__device__ __forceinline__ float parity_sum(float v)
{
    v += dpp_mov<kDppXor2>(v);
    v += dpp_mov<kDppRor4>(v);
    v += dpp_mov<kDppRor8>(v);        // every lane: sum over its parity within its row
    const int odd = threadIdx.x & 1;
    float r0 = readlane_f(v, 0), r1 = readlane_f(v, 16), r2 = readlane_f(v, 32), r3 = readlane_f(v, 48);
    float s0 = readlane_f(v, 1), s1 = readlane_f(v, 17), s2 = readlane_f(v, 33), s3 = readlane_f(v, 49);
    float even_t = (r0 + r1) + (r2 + r3);
    float odd_t = (s0 + s1) + (s2 + s3);
    return odd ? odd_t : even_t;
}

// ---- fp16 ------------------------------------------------------------------
__device__ __forceinline__ float2 unpack_h2(unsigned w)
{
    __half2 h = *reinterpret_cast<const __half2 *>(&w);
    return __half22float2(h);
}

// 8 fp16 weights (one 16-byte load) times 8 fp32 activations, fp32 accumulate
__device__ __forceinline__ float dot8(u32x4 w, float4 ya, float4 yb, float acc)
{
    float2 a = unpack_h2(w.x), b = unpack_h2(w.y), c = unpack_h2(w.z), d = unpack_h2(w.w);
    acc = fmaf(a.x, ya.x, acc); acc = fmaf(a.y, ya.y, acc);
    acc = fmaf(b.x, ya.z, acc); acc = fmaf(b.y, ya.w, acc);
    acc = fmaf(c.x, yb.x, acc); acc = fmaf(c.y, yb.y, acc);
    acc = fmaf(d.x, yb.z, acc); acc = fmaf(d.y, yb.w, acc);
    return acc;
}

__device__ __forceinline__ u32x4 load16(const __half *p)
{
    return *as_global(reinterpret_cast<const u32x4 *>(p));
}
// streamed once, never reused: keep it from displacing the activations in cache
__device__ __forceinline__ u32x4 load16_stream(const __half *p)
{
    return __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4 *>(p)));
}

// uniform (scalar-register) base + 32-bit per-lane byte offset: one address
// register per load instead of two, and the base arithmetic stays on the scalar unit
__device__ __forceinline__ u32x4 load16_stream_at(const __half *ubase, unsigned byte_off)
{
    return __builtin_nontemporal_load(
        as_global(reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(ubase) + byte_off)));
}
// wavefront index inside the workgroup, as a scalar
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Position of activation element k inside an LDS vector laid out for the GEMV
// inner loop: per 512-element chunk, lane l reads elements 8l..8l+7 as two
// float4 at [l*4] and [256 + l*4], so that consecutive lanes touch consecutive
// 16-byte words (no bank conflicts).
__device__ __forceinline__ int lds_perm(int k)
{
    int c = k >> 9, w = k & 511, l = w >> 3, e = w & 7;
    return (c << 9) + ((e >> 2) << 8) + (l << 2) + (e & 3);
}

// tanh form of GELU
__device__ __forceinline__ float gelu_tanh(float z)
{
    return 0.5f * z * (1.0f + tanhf(0.79788456080286535588f * (z + 0.044715f * z * z * z)));
}

// exact (erf) GELU
__device__ __forceinline__ float gelu_erf(float z)
{
    return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f));
}
// the activation the configuration asks for (flags: Dims::flags)
__device__ __forceinline__ float gelu_act(float z, int flags)
{
    return (flags & 1) ? gelu_tanh(z) : gelu_erf(z);
}

// ---- data exchanged between workgroups --------------------------------------
// Values one workgroup writes and another reads within the same launch go
// through device-scope (sc1) stores and loads: those are coherent across the
// per-XCD L2 caches by themselves, so neither side needs an L2 write-back or
// invalidate (which cost tens of microseconds when every wavefront issues
// them).  Ordering is by program order plus xwg_wait_stores(): once it returns,
// this wavefront's earlier exchange stores have been acknowledged by memory.
__device__ __forceinline__ void xwg_store(float *p, float v)
{
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float xwg_load(const float *p)
{
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 xwg_load2(const float *p)      // p 8-byte aligned
{
    const unsigned long long v = __hip_atomic_load(as_global(reinterpret_cast<const unsigned long long *>(p)),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float2 f;
    f.x = __uint_as_float((unsigned)(v & 0xffffffffull));
    f.y = __uint_as_float((unsigned)(v >> 32));
    return f;
}
__device__ __forceinline__ void xwg_store_half(__half *p, float v)
{
    const __half hv = __float2half_rn(v);
    __hip_atomic_store(as_global(reinterpret_cast<unsigned short *>(p)), __half_as_ushort(hv), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ __half xwg_load_half(const __half *p)
{
    return __ushort_as_half(__hip_atomic_load(as_global(reinterpret_cast<const unsigned short *>(p)),
                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
// 16 bytes of fp16 as two coherent 8-byte loads
__device__ __forceinline__ u32x4 xwg_load16(const __half *p)
{
    CFPP_GLOBAL const unsigned long long *q = as_global(reinterpret_cast<const unsigned long long *>(p));
    const unsigned long long a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return u32x4{(unsigned)(a & 0xffffffffull), (unsigned)(a >> 32), (unsigned)(b & 0xffffffffull),
                 (unsigned)(b >> 32)};
}
// Tagged words: an exchanged fp32 value travels with a 32-bit tag in one 8-byte
// store, so a reader needs no separate flag or ordering: it re-reads a word
// until the tag is the one it expects.  p: 8-byte aligned pair (value, tag).
__device__ __forceinline__ void xwg_store_tagged(float *p, float v, unsigned tag)
{
    const unsigned long long w = ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v);
    __hip_atomic_store(as_global(reinterpret_cast<unsigned long long *>(p)), w, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void xwg_wait_stores()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// ---- grid barrier ------------------------------------------------------------
// All workgroups of a launch must be resident (the host checks the grid against
// the occupancy limit).  The barrier orders only exchange data (xwg_store /
// xwg_load): it issues no cache write-back or invalidate.
//
// Two levels: a workgroup arrives at one of up to 16 leaf counters (128 bytes
// apart, so arrivals at different leaves do not serialise), the last arrival of
// a leaf arrives at the root, the last arrival of the root publishes the next
// generation.  Counters count up on even barriers and down on odd ones, so they
// need no reset (and no ordering between a reset and the release); a launch that
// has run an odd number of barriers runs one more before it ends, which leaves
// every counter at zero whatever grid the next launch uses.
//
// The barrier is split: arrive() (after this workgroup's exchange stores) and
// wait().  Loads issued between the two - weights that do not depend on other
// workgroups - stay in flight across the wait.  Only thread 0 talks to memory;
// the value its arrival returns is not needed before wait().
// The wait is bounded: after ~2 s of wall clock the waiter sets the error flag
// and every later barrier falls through, so the grid always drains.
struct GridBarrier {
    unsigned *sync, *err;
    unsigned gen;        // generation this workgroup waits to leave (thread 0 only)
    unsigned nbar;       // barriers completed by this launch
    unsigned nleaf, members;
    unsigned *leaf;
    bool pending, last, propagated, released;

    // s: the workspace's sync words; which: one of the kSyncBarriers independent barriers
    __device__ __forceinline__ void init(unsigned *s, unsigned nwg, int which = 0)
    {
        err = s + kSyncErr;
        s += kSyncBarrier0 + which * kSyncBarrierWords;
        sync = s;
        nbar = 0;
        pending = false;
        last = false;
        propagated = false;
        released = false;
        nleaf = nwg < (unsigned)kSyncLeaves ? nwg : (unsigned)kSyncLeaves;
        const unsigned l = blockIdx.x % nleaf;
        members = (nwg - l + nleaf - 1) / nleaf;
        leaf = s + kSyncLeaf0 + l * kSyncLeafStride;
        gen = 0;
        if (threadIdx.x == 0)
            gen = __hip_atomic_load(as_global(&sync[kSyncGen]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // true when this arrival was the last of `n` at counter c
    __device__ __forceinline__ bool count(unsigned *c, unsigned n) const
    {
        if (nbar & 1u) {
            return __hip_atomic_fetch_add(as_global(c), 0xffffffffu, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 1u;
        }
        return __hip_atomic_fetch_add(as_global(c), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n - 1u;
    }

    __device__ __forceinline__ void arrive()
    {
        xwg_wait_stores();          // every wavefront: its exchange stores are in memory
        __syncthreads();
        if (threadIdx.x == 0) last = count(leaf, members);
        pending = true;
    }

    __device__ __forceinline__ void wait()
    {
        if (!pending) return;
        wait_leader();
        __syncthreads();
    }

    // The same barrier driven by the first wavefront alone (it has issued all of
    // the workgroup's exchange stores itself); the other wavefronts learn the
    // outcome at their next workgroup barrier with it.
    __device__ __forceinline__ void arrive_wave()
    {
        xwg_wait_stores();
        if (threadIdx.x == 0) last = count(leaf, members);
        pending = true;
    }
    __device__ __forceinline__ void wait_wave()
    {
        if (!pending) return;
        wait_leader();
    }

    // Second half of an arrival: the workgroup that was last at its leaf arrives at the root,
    // and the last one there publishes the next generation.  It needs the value the leaf
    // arrival returned, so it runs a little after arrive(); a caller that puts other work
    // between arrive and wait calls it in between (once the arrival has had time to return),
    // or the whole grid's release would wait for that work.  wait() runs it if nobody has.
    __device__ __forceinline__ void propagate()
    {
        if (!pending || propagated) return;
        propagated = true;
        released = false;
        if (threadIdx.x == 0 && last && count(sync + kSyncRoot, nleaf)) {
            __hip_atomic_store(as_global(&sync[kSyncGen]), gen + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            released = true;
        }
    }

    __device__ __forceinline__ void wait_leader()
    {
        propagate();
        pending = false;
        propagated = false;
        if (threadIdx.x == 0) {
            if (!released) {
                const unsigned long long t0 = wall_clock64();
                unsigned spins = 0;
                while (__hip_atomic_load(as_global(&sync[kSyncGen]), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT) == gen) {
                    __builtin_amdgcn_s_sleep(1);
                    if ((++spins & 1023u) == 0) {
                        if (__hip_atomic_load(as_global(err), __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT) == kErrBarrierTimeout)
                            break;
                        if (wall_clock64() - t0 > 200000000ull) {   // 100 MHz counter: 2 s
                            __hip_atomic_store(as_global(err), (unsigned)kErrBarrierTimeout,
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                    }
                }
            }
            gen += 1;
        }
        nbar += 1;
    }

    // before the launch ends: leave every counter at zero
    __device__ __forceinline__ void finish()
    {
        wait();
        if (nbar & 1u) { arrive(); wait(); }
    }
    __device__ __forceinline__ void finish_wave()
    {
        wait_wave();
        if (nbar & 1u) { arrive_wave(); wait_wave(); }
    }
};

// ---- bounded polling -----------------------------------------------------------
// A reader that re-reads exchanged words until they are current calls give_up()
// after every unsuccessful pass: after ~2 s of wall clock (or once any other
// wait of the launch has timed out) it raises the device error flag and returns
// true, so that every wavefront still runs to the end of the kernel.
struct PollGuard {
    unsigned *err;
    unsigned long long t0;
    unsigned spins;
    __device__ __forceinline__ void start(unsigned *sync_words)
    {
        err = sync_words + kSyncErr;
        t0 = wall_clock64();
        spins = 0;
    }
    __device__ __forceinline__ bool give_up()
    {
        if ((++spins & 15u) != 0) return false;
        // (the flag costs a memory round trip: looked at rarely; the clock is cheap)
        if ((spins & 4095u) == 0 &&
            __hip_atomic_load(as_global(err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == kErrBarrierTimeout)
            return true;
        if (wall_clock64() - t0 > 200000000ull) {           // 100 MHz counter: 2 s
            __hip_atomic_store(as_global(err), (unsigned)kErrBarrierTimeout, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            return true;
        }
        return false;
    }
};

// One wavefront waits until `count` tagged words carry `tag`: word i sits at
// base[2 * (first + i * stride)] (a sample of a larger vector - one word per
// producer - serves as a cheap "probably complete" test before the vector is
// read and verified in full).  Up to 16 words per lane.
__device__ __forceinline__ void wait_tagged_sample(const float *base, int first, int stride, int count, int last_index,
                                                   unsigned tag, unsigned *sync_words, int lane)
{
    PollGuard pg;
    pg.start(sync_words);
    for (int b0 = 0; b0 < count; b0 += 16 * 64) {
        bool ok;
        do {
            ok = true;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int i = b0 + j * 64 + lane;
                if (b0 + j * 64 < count) {
                    int idx = first + (i < count ? i : 0) * stride;
                    idx = idx < last_index ? idx : last_index;
                    const float2 w = xwg_load2(base + 2 * (size_t)idx);
                    ok = ok && (i >= count || __float_as_uint(w.y) == tag);
                }
            }
            ok = __all(ok);
        } while (!ok && !pg.give_up());
    }
}

// Rendezvous of `n` wavefronts of a workgroup through an LDS counter that only
// grows: each adds one and waits until it reaches `target` (the caller's running
// total).  Orders LDS traffic like a workgroup barrier for those wavefronts, and
// leaves the others alone.  Bounded like every other wait.
__device__ __forceinline__ void lds_rendezvous(int *counter, int target, unsigned *sync_words, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    PollGuard pg;
    pg.start(sync_words);
    while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target) {
        __builtin_amdgcn_s_sleep(1);
        if (pg.give_up()) break;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// One-sided signals through LDS words that only grow.  lds_signal: a wavefront adds one to a
// counter after its LDS writes; lds_post: a wavefront stores a value; lds_await: spins until the
// word has reached `target` (bounded like every other wait) and orders later LDS reads behind
// it; lds_peek: one look, no waiting.
__device__ __forceinline__ void lds_signal(int *counter, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_post(int *word, int value, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) __hip_atomic_store(word, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ bool lds_peek(const int *word, int target)
{
    return __hip_atomic_load(word, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= target;
}
__device__ __forceinline__ void lds_await(const int *word, int target, unsigned *sync_words)
{
    PollGuard pg;
    pg.start(sync_words);
    while (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target) {
        __builtin_amdgcn_s_sleep(1);
        if (pg.give_up()) break;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// ---- timeline trace (profiling build only) ---------------------------------------
// With CFPP_PROFILE defined (the separate profiling library), workgroup
// (debug >> 8) records (tag, 100 MHz wall clock) pairs per wavefront when bit 16
// of StepParams::debug is set; `first` lets each kernel of a multi-kernel step use
// its own part of a wavefront's kTraceLen entries.  In the product build the
// tracer is an empty object and every mark() compiles to nothing.
#ifdef CFPP_PROFILE
struct Tracer {
    unsigned long long *p;
    int n;
    template <class Params>
    __device__ __forceinline__ void init(const Params &P, int wave, int first = 0)
    {
        const bool on = (P.debug & 16) && (int)blockIdx.x == ((P.debug >> 8) & 0xfff) && wave < kTraceWaves;
        p = on ? P.trace + (size_t)wave * kTraceLen * 2 : nullptr;
        n = first;
    }
    // the whole-stack kernel records one layer: (debug >> 20) & 255 names it (1-based), 0 = the last
    template <class Params>
    __device__ __forceinline__ void select_layer(const Params &P, int layer, int n_layers)
    {
        const int want = ((P.debug >> 20) & 255) ? ((P.debug >> 20) & 255) - 1 : n_layers - 1;
        n = layer == want ? 0 : kTraceLen;
    }
    __device__ __forceinline__ void mark(int tag)
    {
        if (p && n < kTraceLen && (threadIdx.x & 63) == 0) {
            p[2 * n] = (unsigned long long)tag;
            p[2 * n + 1] = wall_clock64();
        }
        if (p) ++n;
    }
};
// a time stamp of workgroup-level events (bit 32 of debug), slot `slot` of this workgroup
#define CFPP_STAMP(P, cond, slot)                                                                      \
    do {                                                                                               \
        if (((P).debug & 32) && (cond)) (P).trace[blockIdx.x * 8 + (slot)] = wall_clock64();           \
    } while (0)
// parts of a phase that the profiling build can leave out (results are then wrong)
#define CFPP_SKIPPED(P, bit) (((P).debug & (bit)) != 0)
#else
struct Tracer {
    template <class Params>
    __device__ __forceinline__ void init(const Params &, int, int = 0) {}
    template <class Params>
    __device__ __forceinline__ void select_layer(const Params &, int, int) {}
    __device__ __forceinline__ void mark(int) {}
};
#define CFPP_STAMP(P, cond, slot) do { } while (0)
#define CFPP_SKIPPED(P, bit) false
#endif

}  // namespace cfpp
