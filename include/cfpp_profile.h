/*
 * cfpp profiling and test aids - NOT part of the library's ABI.
 *
 * These declarations exist only in the profiling build of the library
 * (libcfpp_profile.so, the same sources compiled with -DCFPP_PROFILE); the
 * product library (libcfpp.so) exports none of them, its kernels carry no
 * tracer and honour no skip bits.  They may change at any time.  Callers:
 * the kernel-timeline and counter-calibration runs behind the figures in the
 * design notes, and the tests that compare a block's intermediates with the CPU
 * oracle's.
 */
#ifndef CFPP_PROFILE_H
#define CFPP_PROFILE_H

#include "cfpp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* cfpp_set_option(): profiling switches.
 * CFPP_OPT_PROFILE_SKIP  Bits 0-3: sub-steps to skip so that the others can be
 *                        timed alone (results are then wrong).  Bit 4 (16):
 *                        workgroup ((value >> 8) & 0xfff) records a per-wavefront
 *                        timeline (mode 2: of layer ((value >> 20) & 255) - 1, of
 *                        the last layer when those bits are 0); bit 5 (32): every
 *                        workgroup records a few time stamps of the last layer
 *                        (mode 2); both are read back with cfpp_debug_read(which
 *                        = 4) and leave the results intact.
 * CFPP_OPT_EPOCH_LIMIT   number of tagged-word epochs after which the library
 *                        re-zeroes the epoch counter (default 0xF0000000); a test
 *                        sets it to a few launches' worth to exercise that path. */
#define CFPP_OPT_PROFILE_SKIP 100
#define CFPP_OPT_EPOCH_LIMIT  101

/* Test tap: synchronises `stream`, then copies a workspace intermediate of the
 * most recent block to HOST memory as fp32.  which: 0 = rotated q [batch, h],
 * 1 = GELU(up) [batch, f], 2 = down projection incl. bias [batch, h] (launch
 * modes 0 and 1; mode 2 keeps it in registers), 3 = attention output before the
 * output projection [batch, h] (modes 0 and 1), 4 = raw timeline words.
 * count = number of floats to copy (from the start). */
cfpp_status cfpp_debug_read(cfpp_ctx *ctx, int32_t which, float *dst_host, size_t count,
                            cfpp_stream stream);

/* Plain streaming kernels whose HBM traffic is known exactly, used to find the
 * streaming bandwidth this GPU sustains and to scale hardware traffic counters.
 * cfpp_stream_read loads every 16-byte word of src (DEVICE, `bytes` a multiple of
 * 16) once and XORs a checksum into sink (DEVICE, uint32[grid], caller-zeroed);
 * cfpp_stream_copy copies src to dst.  grid <= 65536, threads 256 or 512,
 * unroll = 16-byte loads in flight per thread (2, 4 or 8). */
cfpp_status cfpp_stream_read(const void *src, size_t bytes, void *sink, int32_t grid,
                             int32_t threads, int32_t unroll, cfpp_stream stream);
cfpp_status cfpp_stream_copy(const void *src, void *dst, size_t bytes, int32_t grid,
                             int32_t threads, cfpp_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CFPP_PROFILE_H */
