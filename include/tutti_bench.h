/*
 * tutti_bench.h -- measurement aids of libtutti_bench.so.
 *
 * libtutti_bench.so is libtutti built with TUTTI_BENCH_BUILD: it exports every entry point of tutti.h, built
 * from the same sources, plus what is declared here: baseline kernels (ceilings and floors the product's rates
 * are compared with), and launch-tuning knobs together with every launch shape they can select.  None of it is
 * part of the product library, which holds the two launch shapes it uses and no knob.
 *
 * The knobs are per HOST THREAD: a tutti_set_* call changes the launches that the same thread makes afterwards
 * through this library and nobody else's.
 */
#ifndef TUTTI_BENCH_H
#define TUTTI_BENCH_H

#include <stdint.h>

#include "tutti.h"

#ifdef __cplusplus
extern "C" {
#endif

/* A plain contiguous device-to-device copy of `bytes` (multiple of 16, both pointers 16-byte aligned) with the
 * load/store width and launch shape of the unpack: the achievable ceiling of the pack / unpack rates. */
int tutti_copy_baseline(void *d_dst, const void *d_src, uint64_t bytes, uint32_t cu_budget, void *stream);

/* One direction only, with the copy's access and launch shape.  write = 0: read `bytes` from d_buf and xor every
 * 16-byte unit, as four 32-bit words, into d_xor: TUTTI_STREAM_SLOTS slots of four words, which the caller zeroes
 * first; each wavefront adds its part to one slot with atomics, so the xor over all slots is the xor of the
 * buffer's units, and calls on one d_xor accumulate.  write != 0: fill d_buf, 16-byte unit i becoming the words
 * { low 32 bits of i, high 32 bits of i, ~low, 0x54555454 }; d_xor is not used.  bytes a multiple of 16, d_buf
 * 16-byte aligned.  What one compute unit (under a CU budget) or the chip reads or writes when it does nothing
 * else. */
#define TUTTI_STREAM_SLOTS 4096u
int tutti_stream_baseline(void *d_buf, uint64_t bytes, uint32_t write, uint32_t *d_xor, uint32_t cu_budget,
                          void *stream);

/* The copy with one side scattered at `gran`-byte granularity and nothing else (no extents, no requests, no
 * K/V planes): piece i of the contiguous side, i < bytes/gran, pairs with the piece at d_scattered +
 * d_perm[i]*gran.  scatter_writes != 0: contiguous -> scattered (the shape of an unpack); 0: scattered ->
 * contiguous (a pack).  What the memory system itself gives for that access pattern when the scattered side is ONE
 * buffer (on the MI355X: one of the three 96 GB regions of the HBM, unless the buffer happens to straddle two).  gran a multiple of 4096;
 * bytes a multiple of gran; every d_perm[i]*gran + gran must lie inside the scattered buffer (span_bytes is
 * checked on the device, offending pieces are skipped).
 * shape: how the bytes are dealt to wavefronts.  Only TUTTI_SCATTER_WAVE_SLICE takes a cu_budget. */
#define TUTTI_SCATTER_WAVE_SLICE 0u        /* the product's: a wavefront per 4 KiB, 256-thread workgroups, nt */
#define TUTTI_SCATTER_WAVE_SLICE_1024 1u   /* the same in 1024-thread workgroups, two per compute unit */
#define TUTTI_SCATTER_WAVE_PIECE 2u        /* a wavefront walks a whole piece */
#define TUTTI_SCATTER_WG_PIECE 3u          /* a 256-thread workgroup walks a whole piece, nt loads and stores */
#define TUTTI_SCATTER_WG_PIECE_PLAIN 4u    /* ... plain loads and stores */
#define TUTTI_SCATTER_WG_PIECE_NT_LOADS 5u /* ... nt loads only */
#define TUTTI_SCATTER_WG_PIECE_NT_STORES 6u /* ... nt stores only */
#define TUTTI_SCATTER_SHAPE_MAX 6u
int tutti_scatter_baseline(void *d_scattered, uint64_t span_bytes, void *d_contig, uint64_t bytes,
                           const uint32_t *d_perm, uint32_t gran, uint32_t scatter_writes, uint32_t shape,
                           uint32_t cu_budget, void *stream);

/* What the host pays for one tutti_layer_restore call, without a language binding in between: the call is made
 * n_calls times in a row from C with these arguments (the launches are only enqueued; the caller synchronises
 * afterwards) and *host_ns_per_call <- wall time of that loop / n_calls.  Arguments as tutti_layer_restore's. */
int tutti_host_cost_of_restore(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks,
                               uint32_t n_req, const uint32_t *d_block_table, uint32_t table_len,
                               const uint32_t *d_file_id, uint32_t layer, const void *d_stage, uint64_t stage_cap,
                               uint64_t stage_addr, uint32_t sgl_id, tutti_extent *d_extents, uint64_t *d_totals,
                               tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t cu_budget, uint32_t *d_status,
                               void *stream, uint32_t n_calls, double *host_ns_per_call);

/* Launch tuning: wgs_per_cu persistent workgroups per compute unit for whole-GPU launches (0 = default),
 * unroll = 16-byte accesses in flight per lane (0 = default; 1, 2, 4 or 8). */
int tutti_set_tuning(uint32_t wgs_per_cu, uint32_t unroll);
/* Head-major pools: 0 = the library chooses (token tiles transposed in LDS when a (token, head) row is
 * shorter than 128 bytes and T, h and the row size are powers of two; else 16 bytes per lane straight
 * between the two orders), 1 = always the direct copy, 2 = through LDS whenever the shape allows. */
int tutti_set_hnd_mode(uint32_t mode);
/* How pack / unpack work items are dealt to workgroups.  0 (default): workgroup b starts at item 4b, so the
 * workgroups the dispatcher deals round-robin to the 8 XCDs take neighbouring 16 KiB; 1: each XCD takes one
 * contiguous eighth of the items. */
int tutti_set_xcd_mapping(uint32_t contiguous);
/* Cache policy of the copy loops: bit 0 = non-temporal 16-byte loads, bit 1 = non-temporal 16-byte stores
 * (default 3 = both). */
int tutti_set_nontemporal(uint32_t mask);

#ifdef __cplusplus
}
#endif
#endif /* TUTTI_BENCH_H */
