/*
 * libmedusa_hip: entry points for benchmarks and tests only.  Nothing here is part of the hot path's boundary
 * (include/medusa.h); a caller that only decodes never needs this header.  Same conventions: extern "C", mdz_status
 * return values, device pointers unless a parameter says HOST.
 */
#ifndef MEDUSA_BENCH_H
#define MEDUSA_BENCH_H

#include "medusa.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- per-kernel timing ------------------------------------------------------------------------------ */

/* Starts recording one HIP-event pair per launch the library makes, for at most max_launches launches (further
 * ones are counted as dropped).  The GEMM, norm and attention kernels are launched so that the dispatch itself
 * writes the kernel's start and end timestamps into the pair (no packets between kernels: the duration a kernel
 * trace shows); for the other calls the pair is recorded on the caller's stream around the call, which adds 1-2 us.
 * Creates its events here, so hot-path calls still allocate nothing.  Process-global; not thread-safe. */
int medusa_profile_begin(int max_launches);

/* Stops recording, waits for the recorded events, and writes one text line per kernel family into the HOST
 * buffer `report`: "name,launches,total_us,min_us,max_us\n" (families: gemm_w64 / gemm_n64 / gemm_w32 /
 * gemm_n32 = the weight-streaming GEMM instantiated for 128- or 64-column bands and 64 or <= 32 rows,
 * gemm_portable, gemm_large, attention, rmsnorm, rope, swiglu, embed, select, accept, kv_compact, misc). */
int medusa_profile_end(char* report, int64_t report_bytes);

/* ---- calibration streams ----------------------------------------------------------------------------- */

/* Enqueues a pure read of `bytes` bytes at src (16 bytes per lane, every wave a contiguous range, n_workgroups
 * workgroups of 256 threads): the practical HBM read ceiling the weight-streaming kernels are compared with.
 * Only medusa_stream_read_bytes(bytes, n_workgroups) bytes are read (whole 8 KiB rounds per wave).  sink4: 4
 * device bytes that keep the loads alive. */
int medusa_stream_read(const void* src, int64_t bytes, int n_workgroups, void* sink4, void* stream);
int64_t medusa_stream_read_bytes(int64_t bytes, int n_workgroups);

/* Enqueues a plain copy of `bytes` (multiple of 16) from src to dst: a transfer of known size for scaling
 * hardware byte counters. */
int medusa_stream_copy(const void* src, void* dst, int64_t bytes, void* stream);

/* ---- introspection of the weight-streaming GEMM's work decomposition (HOST only, nothing is enqueued) --- */

/* For X[M,K] x W[N,K]^T (16-bit, M <= 64, N % 32 == 0, K % 128 == 0): the (column band, K-stage) units, numbered
 * band-major, are cut into `grid` equal contiguous ranges, range w = [floor(w*U/grid), floor((w+1)*U/grid)),
 * U = (N / band_cols rounded up) * n_stages; every range that touches a band writes one partial-sum slot of it.
 * max_split bounds the slots per band (1: whole bands only).  medusa_gemm_slot_count returns the number of slots the
 * consumers add for output column `col` (negative: error). */
int medusa_gemm_plan(int dtype, int M, int N, int K, int max_split, int32_t* grid, int32_t* band_cols, int32_t* n_stages,
                     int32_t* max_slots);
int medusa_gemm_slot_count(int dtype, int M, int N, int K, int max_split, int col);

/* ---- test hook --------------------------------------------------------------------------------------- */

/* The layer runs RoPE + cache write either fused into the attention kernel's prologue (default) or as a kernel of
 * its own followed by the attention over the rotated queries; both orders are product paths (the second serves the
 * shapes the fused kernel does not cover).  on != 0 forces the second everywhere so that a test can compare them on
 * one shape.  Process-global; returns the previous setting. */
int medusa_test_force_unfused_rope(int on);

#ifdef __cplusplus
}
#endif
#endif /* MEDUSA_BENCH_H */
