/*
 * bsgd_debug.h — testing and measurement aids of libbsgd.
 *
 * None of these is part of a step (see bsgd.h for the product boundary).
 * They exist so that the tests can force every compiled code path and the
 * benchmark can count launches and calibrate hardware counters.  The two
 * setters change process-wide state that only affects HOW a step is launched,
 * never its result; a program that does not call them gets the automatic
 * choices.  Conventions (DEVICE / HOST pointers, stream, return codes) are
 * those of bsgd.h.
 */
#ifndef BSGD_DEBUG_H
#define BSGD_DEBUG_H

#include <stddef.h>
#include <stdint.h>

#include "bsgd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Launch shape of the reduce/update kernel, process-wide; for benchmarking.
 * A shape is (block, vec, unroll, nontemporal):
 *   block        threads per workgroup
 *   vec          float4 columns per thread
 *   unroll       kept rows per batch of the row loop
 *   nontemporal  0/1: gradient rows are loaded with the streaming hint
 * Every shape adds the kept rows in the same order, so results do not depend
 * on it.  By default the library picks a shape from the problem size (the
 * chunk width whose launches fill the chip best).
 * bsgd_set_tuning pins a compiled-in shape (-1 keeps a field of the current
 * one; all four -1 returns to the automatic choice) and returns BSGD_ERR_ARG
 * when that combination is not compiled in; bsgd_num_shapes / bsgd_get_shape
 * enumerate them (out4 is HOST int32[4] in the order above). */
int bsgd_set_tuning(int32_t block, int32_t vec, int32_t unroll, int32_t nontemporal);
int bsgd_num_shapes(void);
int bsgd_get_shape(int32_t i, int32_t* out4);

/* How a multi-tensor call hands its tensor table to the kernels, process-wide;
 * for testing and benchmarking.  mode 0 (default): every launch carries the
 * part of the table its columns fall into as a kernel argument, and only a
 * call in which some launch touches more tensors than fit there writes the
 * whole table into the workspace first; mode 1: always through the workspace.
 * Results do not depend on it.  Returns BSGD_ERR_ARG for another mode. */
int bsgd_set_table_mode(int32_t mode);

/* How many launches of the reduce/update kernel the calling thread's last
 * bsgd_step / bsgd_reduce_update enqueued (a step is cut into launches that
 * each fill the chip once; a clipped step counts both of its passes). */
int bsgd_last_launch_count(void);

/* Host logic made visible for testing, nothing is enqueued: the runs of chunks
 * a call with these tensors launches when a chunk is chunk_cols columns wide
 * (a multiple of 4).  Chunk c covers columns [base + c*chunk_cols, base +
 * (c+1)*chunk_cols) with base = the first tensor column rounded down to a
 * multiple of 4.  Chunks outside every run hold no tensor column and are
 * neither launched nor read; inside a run, gaps of up to 64 chunks are
 * tolerated.  tensors: HOST array as for bsgd_step (pointers only checked for
 * being non-NULL and 4-byte aligned, never dereferenced).  first / count: HOST
 * out int64[capacity]; n_runs: HOST out.  BSGD_ERR_ARG for bad tensors or
 * when there are more runs than `capacity`. */
int bsgd_debug_chunk_runs(const bsgd_tensor* tensors, int32_t T, int64_t chunk_cols, int64_t* first, int64_t* count,
                          int32_t capacity, int32_t* n_runs);

/* A step with at most 64 workers and no per-worker clipping does its selection
 * inside its first launch instead of in a kernel of its own; results and
 * everything the bsgd_last_* getters report are the same either way.
 * bsgd_set_fused_selection(0) makes every step use the separate selection
 * kernel (process-wide; 1 = default); bsgd_last_step_fused_selection tells
 * whether the calling thread's last bsgd_step / bsgd_step_ex /
 * bsgd_step_noalloc did it inside (1) or not (0). */
int bsgd_set_fused_selection(int32_t on);
int bsgd_last_step_fused_selection(void);

/* Measurement aid, not part of the step: a plain device-to-device copy of
 * `bytes` bytes (a multiple of 16; both pointers DEVICE, 16-byte aligned,
 * not overlapping).  It reads and writes exactly `bytes` bytes of HBM, which
 * makes it the yardstick hardware traffic counters are scaled against. */
int bsgd_calibration_copy(void* dst, const void* src, int64_t bytes, void* stream);

/* Measurement aid, not part of the step: one plain streaming kernel that reads
 * n_read buffers and writes n_write buffers of `bytes` bytes each (1 <= n_read
 * <= 4, 0 <= n_write <= 4; all DEVICE, 16-byte aligned; `bytes` a multiple of
 * 16; a written buffer may be one of those read).  read_ptrs / write_ptrs are
 * HOST arrays of DEVICE pointers.  `vec` (1, 2, 4 or 8) is the number of
 * 16-byte groups per thread, laid out like a chunk of the step's kernel.
 * Compiled mixes (n_read, n_write): (1,0) (3,3) (3,2) (2,2) (2,1) (1,1);
 * any other returns BSGD_ERR_ARG.
 * Its bandwidth is what the memory system gives a kernel with that mix of
 * read and written streams: the yardstick the step's passes are held
 * against (a read-only pass, the update's three read and three written
 * streams, pass 2 of a clipped step with three read and two written). */
int bsgd_yardstick_streams(const void* const* read_ptrs, int32_t n_read, void* const* write_ptrs, int32_t n_write,
                           int64_t bytes, int32_t vec, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BSGD_DEBUG_H */
