/*
 * peagle_bench.h - measurement aids of the parallel-drafting attention library (bench.py and the
 * profiling runs use them; they are not part of the method's call path declared in peagle.h):
 * per-kernel launch timing of a step, the measured matrix-core ceiling, and device facts.
 * Conventions (device / host pointers, stream, status codes) are those of peagle.h.
 */
#ifndef PEAGLE_BENCH_H
#define PEAGLE_BENCH_H

#include "peagle.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel kinds reported by peagle_attn_step_profiled. */
#define PEAGLE_KERNEL_FWD 0      /* forward (O, LSE) */
#define PEAGLE_KERNEL_DQ 1       /* Delta and dQ */
#define PEAGLE_KERNEL_DKDV 2     /* dK, dV */
#define PEAGLE_KERNEL_REDUCE 3   /* sum of the per-head depth-0 dK/dV partials into the accumulators */
#define PEAGLE_KERNEL_ROPE 4     /* rotation of Q and K (peagle_attn_step_rope_profiled only) */
#define PEAGLE_NUM_KERNEL_KINDS 5

typedef struct peagle_profile {
  float ms[PEAGLE_NUM_KERNEL_KINDS];          /* summed launch durations per kernel kind, milliseconds */
  int32_t launches[PEAGLE_NUM_KERNEL_KINDS];  /* launches per kind */
} peagle_profile_t;

/*
 * Measurement aid: the same work as peagle_attn_step_partitioned (Sec. 3.2 pass per segment),
 * with a HIP event pair recorded on `stream` around every kernel launch.  Waits for the work
 * to finish, then fills `profile` (host).  Creates and destroys events; not for hot loops.
 */
int peagle_attn_step_profiled(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg_begin,
                              int32_t seg_end, const void* q, const void* k, const void* v, const void* d_o,
                              void* o, float* lse, void* dq, float* dk_acc, float* dv_acc, void* workspace,
                              size_t ws_bytes, void* stream, peagle_profile_t* profile);

/* Measurement aid: the same for peagle_attn_step_partitioned_rope. */
int peagle_attn_step_rope_profiled(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg_begin,
                                   int32_t seg_end, const void* q, const void* k, const void* v, const void* d_o,
                                   const float* rope_table, int32_t n_pos, void* o, float* lse, void* dq,
                                   float* dk_acc, float* dv_acc, void* workspace, size_t ws_bytes, void* stream,
                                   peagle_profile_t* profile);

/*
 * Measurement aid: runs a register-only v_mfma_f32_32x32x16_bf16 issue loop on every CU of the
 * current device and writes the sustained rate (TFLOP/s, host float) to *tflops - the measured
 * matrix-core ceiling that attention throughput is compared with.  Allocates a small scratch
 * buffer and synchronises.
 */
int peagle_measure_mfma_ceiling(void* stream, float* tflops);

/*
 * Measurement aid: the same loop on pseudo-random operands (roughly uniform in (-2, 2), every significand
 * bit in use) that change from instruction to instruction.  The matrix cores draw more power on such data
 * than on the constant small integers of peagle_measure_mfma_ceiling and the chip lowers its clock to stay
 * inside its power limit: this is the rate the matrix cores sustain on operands like real Q, K, V.
 * Same arguments, allocation and synchronisation as peagle_measure_mfma_ceiling.
 */
int peagle_measure_mfma_ceiling_random(void* stream, float* tflops);

/*
 * Measurement aid: compute-unit count and peak engine clock (kHz) of the current device, as the
 * HIP runtime reports them (both host ints, out).
 */
int peagle_device_info(int32_t* compute_units, int32_t* clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* PEAGLE_BENCH_H */
