/*
 * lp_measure.h -- measurement aids of the LayerPipe library; NOT part of the training path of lp.h.
 *
 * Two things the benchmark needs from inside the library: timing events around every task launch on the
 * stream it is launched on (so that a per-kernel duration can be read inside the timed region), and a
 * kernel that issues nothing but the GEMMs' matrix instruction (what the matrix cores sustain on this
 * machine with nothing to feed them).  Neither changes any result of the calls in lp.h.
 */
#ifndef LAYERPIPE_LP_MEASURE_H
#define LAYERPIPE_LP_MEASURE_H

#include "lp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Task kinds of Fig. 1(b) as this library launches them. */
typedef enum {
  LP_TASK_F = 0,         /* forward product + activation (Eq. 1, Eq. 2)  */
  LP_TASK_DX = 1,        /* activation-gradient product (Eq. 4)          */
  LP_TASK_DW = 2,        /* weight-gradient product (Eq. 5)              */
  LP_TASK_HADAMARD = 3,  /* the moved f' factor (Eq. 3)                  */
  LP_TASK_LOSS = 4,      /* error and delta of the output layer          */
  LP_TASK_UPDATE = 5,    /* delayed SGD update (Eq. 6)                   */
  LP_TASK_COUNT = 6
} lp_task;

/* enable != 0: from now on every task launch is bracketed by two timing events recorded on the
 * stream the task is launched on (host memory and HIP events only; no device memory).  Tasks that
 * overlap on different streams each report their own begin-to-end time. */
int lp_profile(lp_ctx* ctx, int enable);
/* Waits for the recorded launches of `task`, adds their durations and returns the totals gathered
 * since the last reset: *total_ms (milliseconds) and *launches; either may be NULL.  reset != 0
 * clears the totals of this task afterwards. */
int lp_profile_read(lp_ctx* ctx, int task, double* total_ms, long* launches, int reset);
/* The same for one layer l = 1..L (the loss task belongs to no layer and is only in the totals). */
int lp_profile_read_layer(lp_ctx* ctx, int task, int l, double* total_ms, long* launches, int reset);

/* Calibration of the matrix-core roofline (no context needed): launches `workgroups` workgroups of eight
 * waves that each issue iters * 8 v_mfma_f32_32x32x16_bf16 on operands held in registers, nothing else --
 * 2 * 32 * 32 * 16 flop per instruction, so workgroups * 8 * iters * 8 * 32768 flop per launch.  out_dev
 * (device, out_elems >= workgroups * 512 floats, LP_ERR_SHAPE otherwise) receives one checksum per lane.
 * uniform_values = 0: pseudo-random operands in [-1, 1), as a real product has; != 0: the same few small
 * values in every lane (few bits toggle, so the chip's power limit allows a higher clock: the two differ).
 * Asynchronous on `stream`; returns LP_ERR_NULL / LP_ERR_SHAPE / LP_ERR_HIP without a message. */
int lp_probe_mfma(float* out_dev, size_t out_elems, int workgroups, int iters, int uniform_values, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LAYERPIPE_LP_MEASURE_H */
