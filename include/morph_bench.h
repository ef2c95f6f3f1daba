/*
 * libmorph -- bench and test tooling.  NOT part of the serving interface (that is morph.h): the
 * library exports these so that bench.py, the profiling commands and the tests can sweep kernel
 * choices, calibrate hardware byte counters and measure what the device reaches with nothing in
 * the way.  A serving process has no reason to call any of them.
 *
 * morph_set_tuning changes PROCESS-WIDE state that the kernel selection of every later call reads
 * (all other entry points are stateless).  In particular it changes what morph_workspace_bytes()
 * answers: a workspace sized before the change may be too small afterwards; such a call is refused
 * with MORPH_ERR_WORKSPACE before anything is launched, never overrun.  Set the override, size the
 * workspace, run, and restore the default (value 0) -- as the tests do.
 */
#ifndef MORPH_BENCH_H
#define MORPH_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Override a kernel-selection heuristic (0 restores the default).  For benchmarking sweeps only;
 * defaults are chosen from the shape.  Keys: 0 = K-split factor of the decode kernels,
 * 1 = target workgroup count of the decode kernels, 2 = prefill tile (1 = 256x256 with 8 waves,
 * 2 = 128x128, 3 = 256x256 with 4 waves, 4 = 256x128 with 4 waves, 5 = 256x192, 6 = 256x128 with 8 waves),
 * 3 = waves per decode workgroup (4 or 8),
 * 4 = prefill: sharing the last partial round of tiles out along K (1 = never, 2 = always),
 * 5 = prefill: order in which tiles are dealt to workgroups (1 = row tiles of a column tile first,
 * 2 = blocks of 8 column tiles spread over the 8 XCDs), 6 = largest M the streaming kernels take
 * (32 .. 1024; replaces the choice by shape), 7 = rows one streaming workgroup takes (16 or 32),
 * 8 = non-temporal weight loads in the streaming kernels (1 = always, 2 = never),
 * 9 = streaming kernels: sum over the K splits shared out among the workgroups of a tile (1 = whenever
 * possible, 2 = never, 3 = whenever possible and no workgroup waits for the others, which leaves every
 * part to the last one out: exercises the path taken after a wait that ran out).
 * 10 = prefill: number of workgroups (at most one per compute unit; with key 4 = 2 and fewer tiles than
 * that, K is shared out over them).
 * 11 = prefill: who stages the tiles into LDS (1 = half the waves the weight tile and half the x tile,
 * 2 = every wave an equal share of both; quantized kinds only).
 * 12 = the register-tiled kernel for at most 64 rows of 4-bit weights (2 = never: the general streaming kernels
 *      take them; 3 = only up to 16 rows; 4 = the native code order always through the four-wave kernels,
 *      never the eight-wave one; 5 = always through the eight-wave one).
 * 13 = that kernel's hand-over: 1 = written through to memory instead of kept in one XCD's L2.
 * A change alters morph_workspace_bytes(); size the workspace after setting. */
int morph_set_tuning(int key, int value);

/* Plain device-to-device copy kernel (16-byte vectors; src, dst 16-byte aligned, bytes % 16 == 0).
 * The stack driver uses it for its taps; it is exported so that hardware byte counters can be
 * calibrated against a transfer of known size. */
int morph_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Peak probes, so that a benchmark can quote its fractions against what this very device reaches
 * as well as against the data sheet.  Both write one word per thread into `out` (device, 16-byte
 * aligned, at least morph_probe_out_bytes()), launch asynchronously on `stream` and touch nothing else.
 *   morph_probe_read: loads every 16-byte vector of src[0..bytes) once (bytes % 16 == 0): bytes over
 *     the launch time is the read bandwidth of a plain contiguous stream.
 *   morph_probe_mfma: every wave issues iters x 4 independent 32x32x16 fp16 MFMAs on registers;
 *     *flop (host, may be NULL) receives the flop of the launch: flop over the launch time is the rate
 *     the matrix cores sustain with nothing else in the way (1 <= iters <= 2^24). */
/* How a launch of at most 64 rows would be laid out on the device (host only, launches nothing):
 * plan[0] = 1 when the register-tiled kernels of decode_small.hip take it (else the rest is 0), plan[1] =
 * column tiles of 256, plan[2] = workgroups sharing the K range of a tile, plan[3] = slices of rows,
 * plan[4] = 1 for the eight-wave kernel.  kind as in morph.h (MORPH_KIND_W4A16_NATIVE for the native code
 * order).  The workgroups of a tile wait for each other, so the layout must fit the device at once:
 * tiles * splits * slices workgroups on its compute units, and ceil(tiles / 8) * splits * slices on the
 * compute units of one XCD (the tests check this over a sweep of shapes). */
int morph_plan_decode(int kind, int M, int K, int N, int* plan);

size_t morph_probe_out_bytes(void);
int morph_probe_read(const void* src, size_t bytes, void* out, size_t out_bytes, void* stream);
int morph_probe_mfma(int iters, void* out, size_t out_bytes, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MORPH_BENCH_H */
