/*
 * regione_bench.h - measurement aids of the RegionE library (NOT part of the method's ABI in regione.h): forced
 * kernel plans for same-process comparisons, per-kernel-class timing with HIP events, and a register-only probe of
 * what the chip's matrix cores sustain.  Used by the benchmark and by tests that sweep kernel plans.
 */
#ifndef REGIONE_BENCH_H
#define REGIONE_BENCH_H

#include "regione.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning knob for experiments: forces the GEMM wave tile (1 or 2 blocks of 32 columns; 3 or 4 =
 * the same two widths with the kernel that stages both operands through LDS, 5 or 6 = that
 * kernel with 256-row workgroup tiles) and the number of K splits of every later GEMM of this
 * context; 0 restores the automatic choice. */
int regione_tune_gemm(regione_ctx* ctx, int32_t wave_tile_blocks, int32_t k_splits);

/* Tuning knob for experiments: forces the number of key-range splits (1..8) of every later
 * attention call of this context; 0 restores the automatic choice. */
int regione_tune_attention(regione_ctx* ctx, int32_t key_splits);

/* Per-kernel-class timing for benchmarks (not part of the method).  While enabled, every
 * kernel launch group of the context is bracketed by a HIP event pair on its stream (at most
 * 8192 pairs between two reads).  regione_profile_read waits for the stream, adds the elapsed
 * milliseconds and the number of launch groups of each class into the two host arrays of
 * n_classes entries (index = REGIONE_PROF_*), and clears the recorded pairs. */
enum { REGIONE_PROF_PARTITION = 0, REGIONE_PROF_ROWS = 1, REGIONE_PROF_LAYERNORM = 2, REGIONE_PROF_GEMM = 3,
       REGIONE_PROF_ATTENTION = 4, REGIONE_PROF_VELOCITY = 5, REGIONE_PROF_CLASSES = 6 };
int regione_profile_enable(regione_ctx* ctx, int32_t on);
int regione_profile_read(regione_ctx* ctx, double* total_ms_host, int64_t* launches_host, int32_t n_classes);

/* Matrix-core peak probe for benchmarks (not part of the method): what the MFMA units of THIS
 * chip sustain at the clock it holds under load, to read the achieved TFLOP/s against.  Every
 * wave runs `iters` rounds of four independent register-only MFMAs (format 0: bf16
 * v_mfma_f32_32x32x16_bf16; 1: E4M3 v_mfma_f32_32x32x64_f8f6f4) on pseudo-random finite
 * operands and stores one float per lane so the work cannot be dropped.  n_workgroups
 * workgroups of 256 threads; out: float32 [n_workgroups * 256].  The launch is timed under
 * REGIONE_PROF_GEMM; *flops_host receives the work of the launch (n_workgroups * 4 waves *
 * iters * 4 * 2 * 32 * 32 * K, K = 16 or 64). */
int regione_mfma_peak_probe(regione_ctx* ctx, int32_t format, int32_t iters, int32_t n_workgroups, float* out, double* flops_host);

#ifdef __cplusplus
}
#endif
#endif /* REGIONE_BENCH_H */
