/*
 * libtrjacobi, development interface: measurement aids and experiment knobs that are not
 * part of the method's boundary (that is trjacobi.h).  Tests and the benchmark use them.
 *
 * State: the knobs and the event timer are PROCESS-WIDE.  trj_set_tunable may be called
 * from any thread (it takes a lock), and every entry point of trjacobi.h copies the knobs
 * once on entry, so one call always sizes its workspace and shapes its launches from the
 * same values; but a workspace size asked for with trj_workspace_bytes is only valid for
 * the knob values current at that time: set knobs first, then query, then call.  The event
 * timer (trj_profile_*) is not thread-safe: one profiling session at a time, and no entry
 * point may run on another thread during it.
 */
#ifndef TRJACOBI_DEV_H
#define TRJACOBI_DEV_H

#include "trjacobi.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One projection alone (tests, roofline measurements): y[T][n_out] (fp32) = x W^T with
 * x[T][n_in] plain row-major in `dtype` and W a TRJ_PACK_PLAIN matrix.  split_k <= 0
 * lets the library choose.  workspace: at least
 * 2*ceil(T/128)*128*n_in + 4*8*T*n_out + 1024 bytes. */
int32_t trj_linear(const void* x, const void* w_packed, int32_t T, int32_t n_in, int32_t n_out,
                   int32_t dtype, int32_t split_k, void* workspace, size_t ws_bytes, float* y,
                   void* stream);

/* The launch plan a bf16 projection of the verify step gets at T token rows (section
 * "TR-Jacobi Decoding": the projections of the decoder forward over the tree's rows).
 * fused != 0: the QKV and gate/up projections (no k-split across workgroups); else the
 * plan of a projection that writes split-k partial sums.  h_plan[6] (HOST): token-row
 * tiles per pass, row tiles per workgroup, k-parts per workgroup, row tiles per wavefront,
 * grid k-splits, 1 if the many-rows kernel (packed batches) is used. */
int32_t trj_dev_gemm_plan(int32_t T, int32_t n_in, int32_t n_out, int32_t fused, int32_t* h_plan);

/* Launch-shape knobs for experiments: "gemm_target_wgs" (workgroups a split-k projection
 * is split up to), "max_split_k", "gemm_cfg" (0: choose the workgroup shape per
 * projection, 1..6 force one), "gemm_big_t" (padded token rows from which the packed-batch
 * projection kernel is used, 0: never), "gemm_big_wt" (row tiles per wavefront of that
 * kernel: 2, 4, or 0 to choose per projection), "attn_target_wgs" (attention workgroups aimed at
 * per launch), "attn_min_bpw" (32-slot blocks per wavefront, at least; 0 = chosen from the tree size), "attn_xchg_min_blocks" (blocks
 * per workgroup from which the two wavefronts of a key stream split their K/V loads and
 * exchange halves through LDS).  Results do not
 * depend on them beyond fp32 summation order.  Unknown name: TRJ_ERR_BAD_SHAPE. */
int32_t trj_set_tunable(const char* name, int32_t value);

/* Per-kernel timing for benchmarks.  Between trj_profile_begin(kernel_class, capacity)
 * and trj_profile_end, every launch of that kernel class inside the entry points is
 * bracketed by HIP events on its stream (the only HIP objects this library ever
 * creates).  trj_profile_end waits for them, writes up to `capacity` durations in
 * milliseconds to h_ms, their number to h_count, and destroys the events.  Classes:
 * 1 QKV projection, 2 tree attention, 3 attention merge, 4 output projection, 5 split-k
 * sum + residual + RMSNorm, 6 gate/up projection, 7 down projection, 8 LM head, 9 argmax,
 * 10 accept, 11 KV compaction. */
int32_t trj_profile_begin(int32_t kernel_class, int32_t capacity);
/* The same with a span: the start event goes before a launch of `first_class`, the stop
 * event after the next launch of `last_class` (which the entry point issues later in the
 * same step).  The difference between a span [A..B] and the single class B is the
 * duration of A up to the start of B without the cost of the event pair itself. */
int32_t trj_profile_begin_span(int32_t first_class, int32_t last_class, int32_t capacity);
int32_t trj_profile_end(float* h_ms, int32_t capacity, int32_t* h_count);
/* Average elapsed time between two events recorded back to back on `stream` (nothing
 * between them): the part of a trj_profile_* duration that is the event pair itself, not
 * the kernel it brackets.  `pairs` in 1..4096; synchronises the stream. */
int32_t trj_profile_event_overhead(int32_t pairs, float* h_avg_ms, void* stream);

/* Measurement aid: a plain copy of `bytes` (a multiple of 16) from src to dst, used to
 * calibrate the HBM traffic counters against a kernel whose traffic is known. */
int32_t trj_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/* Measurement aid: a streaming read of `bytes` (a multiple of 16) from src and nothing else
 * (sink: 4 bytes of device memory, written only if the data has one particular value). */
int32_t trj_read_probe(const void* src, size_t bytes, void* sink, void* stream);

/* What the current device reports (hipDeviceGetAttribute): h_info[6] (HOST) = compute
 * units, engine clock kHz, memory clock kHz, memory bus width in bits, L2 bytes, LDS bytes
 * per workgroup. */
int32_t trj_dev_device_info(int32_t* h_info);

#ifdef __cplusplus
}
#endif
#endif /* TRJACOBI_DEV_H */
