/*
 * bitstack_bench.h -- measurement hooks of libbitstack.so.  Not part of the
 * method's interface (that is bitstack.h): benchmarks and tests use these to
 * force a work split of the decode kernel and to probe the device's read rate.
 */
#ifndef BITSTACK_BENCH_H
#define BITSTACK_BENCH_H

#include "bitstack.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning of the decode kernel, process-wide (atomic integers: safe to set while
 * other threads call the library; a call uses the values it reads at launch).
 * value 0 restores the built-in choice.  Unknown options give BITSTACK_E_ARG; a
 * value the launcher cannot honour makes it fall back to its own choice or refuse
 * the launch with BITSTACK_E_HIP before anything is enqueued. */
enum {
    BITSTACK_OPT_DECODE_BGROUPS = 3,      /* workgroups sharing one (row slab, column range) pair; each
                                             walks every BGROUPS-th block of the loaded prefix (single calls) */
    BITSTACK_OPT_DECODE_TILES = 4,        /* 32-row tiles per wavefront: 2 or 4 (512 / 1024 rows per workgroup) */
    BITSTACK_OPT_DECODE_KS_CHUNKS = 5,    /* 256-column chunks per workgroup: 1..32 */
    BITSTACK_OPT_DECODE_EARLY = 6,        /* value - 1 = chunks of the first sign window requested at entry: 0, 2, 4 */
    BITSTACK_OPT_DENSE_TILE = 7           /* output tile of the dense product: 1 = 256 rows x 256 tokens, 2 = 128 x 256,
                                             3 = 128 x 128 */
};
int bitstack_set_option(int option, int value);

/* Reads device_buf[0, bytes) once with 128-bit loads (nothing is written unless
 * the xor of the data hits one magic value).  Gives the achievable HBM read rate
 * that the sign stream of the decode path is compared with.
 * device_buf 16-byte aligned, bytes % 16 == 0, device_sink >= 4 bytes. */
int bitstack_probe_read(const void* device_buf, size_t bytes, void* device_sink, int workgroups,
                        bitstack_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif
