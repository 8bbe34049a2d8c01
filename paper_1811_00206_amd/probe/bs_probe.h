/*
 * bs_probe.h -- measurement helpers for the benchmark, NOT part of the method and not
 * part of libbs.so: they are built into a library of their own (libbs_probe.so) that
 * only bench.py and one GPU test load.
 *
 * The products of arXiv 1811.00206, Sec. 4 last a few microseconds on an MI355X, so a
 * reader needs the machine's floor next to every kernel time: what an empty launch
 * costs, what a kernel that only reads the same bytes reaches, what an LDS gather
 * costs, and what a grid-wide barrier costs (the price of a persistent multi-step
 * kernel for the recurrent models of Sec. 4.3).
 *
 * Conventions: pointers marked DEVICE are caller-owned device memory; `stream` is a
 * hipStream_t passed as void*; calls only enqueue; a non-zero return (1 null pointer,
 * 2 invalid size, 4 misaligned pointer, 5 HIP error) means nothing was enqueued.
 */
#ifndef BS_PROBE_H
#define BS_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* An empty kernel of `grid` workgroups (1..65536) of `threads` lanes (64..1024, a
 * multiple of 64). */
int bs_probe_empty(int grid, int threads, void* stream);

/* A one-lane kernel that stores the GPU's constant-rate wall clock into DEVICE `slot`
 * (8-byte aligned).  Two of them around a run of launches inside one captured graph time
 * that run on the GPU itself, free of what launching the graph costs.
 * bs_probe_wall_clock_khz: the clock's rate on the current device (0 if unknown). */
int bs_probe_timestamp(uint64_t* slot, void* stream);
int bs_probe_wall_clock_khz(void);

/* A kernel that only reads `bytes` bytes (a multiple of 16, at least 16) from DEVICE
 * `src`, 16 bytes per lane and load.
 * pieces_per_lane: 0 = the fastest known shape for the size (one piece per lane and as
 * many short-lived workgroups as needed up to 64 MB, 8 pieces in flight per lane on a
 * fixed grid above); 1, 2, 4 or 8 = that many pieces per lane.
 * store_mode: 0 = nothing is stored (`sink`, DEVICE memory of at least 256 bytes or NULL, is
 * never written for real data); 1, 2, 3 = one lane in `store_every` (>= 1) stores 4 bytes
 * to consecutive words of `sink` (what a matrix-vector product does with its row sums)
 * with a plain store, a non-temporal store, or an agent-scope atomic store; `sink_bytes`
 * must then cover one word per `store_every` lanes launched (bytes / (16 * pieces_per_lane)
 * lanes, rounded up to whole workgroups of 256) plus one.  store_mode 4: the first
 * `store_every` (1..32) lanes of every workgroup store adjacent words of a 128-byte line of
 * the workgroup's own (32: a whole line in one instruction); `sink` must be 128-byte
 * aligned for that and hold 128 bytes per workgroup. */
int bs_probe_stream_read(const void* src, size_t bytes, int pieces_per_lane, int store_mode,
                         int store_every, void* sink, size_t sink_bytes, void* stream);

/* 256 workgroups of `threads` lanes (64..1024, a multiple of 64) fill 120 KB of LDS and
 * then issue `reads` (a multiple of 8) 16-byte LDS reads per lane and nothing else.
 * pattern 0: a wavefront reads 1 KB of adjacent bytes; pattern 1: groups of
 * `group_lanes` (2, 4, 8 or 16) neighbouring lanes read adjacent 16-byte pieces of one
 * row of group_lanes*16 bytes, every group a random row; pattern 2: every lane reads 4
 * bytes (ds_read_b32) at a random word of its own, the gather of a matrix-vector
 * product (`group_lanes` ignored).
 * Time per wavefront read and compute unit = kernel time / (reads * threads / 64). */
int bs_probe_lds_gather(int threads, int pattern, int group_lanes, int reads, void* sink,
                        void* stream);

/* What one step of a persistent multi-step kernel would pay for its communication:
 * `wgs` workgroups (1..256: one per compute unit, all resident at once on an idle GPU) of
 * `threads` lanes run `steps` rounds; in each round every workgroup reads a vector of
 * `vec_floats` floats with agent-scope loads, writes its own slice of the next round's
 * vector with agent-scope stores, arrives on one atomic counter and waits, BOUNDED, until
 * all have arrived (spin_limit polls; when a wait runs out the workgroup raises the
 * abort flag and every workgroup leaves at its next round, so the kernel always ends).
 *   sync   DEVICE in/out  two uint32: [0] arrivals, [1] abort flag; the caller zeroes both
 *                         before every launch
 *   hbuf   DEVICE in/out  2 * vec_floats floats
 *   mode   0: every poll is an acquire load; 1: relaxed polls, one acquire fence at the end
 * Time per round = kernel time / steps. */
int bs_probe_grid_barrier(int wgs, int threads, int steps, int vec_floats, int mode,
                          uint32_t spin_limit, uint32_t* sync, float* hbuf, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BS_PROBE_H */
