/*
 * tsenor_profile.h - measurement aid of libtsenor.so, kept apart from the product interface (tsenor.h).
 *
 * Not part of the method: a benchmark calls this to see how the time of a pass divides between the stages of
 * the path (Algorithm 1 and the steps of Algorithm 2).  Unlike the entry points of tsenor.h it SYNCHRONISES
 * the stream and creates HIP events.
 */
#ifndef TSENOR_PROFILE_H
#define TSENOR_PROFILE_H

#include "tsenor.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Runs tsenor_mask_ex `repeats` times (1..4096) back to back on `stream` with HIP events recorded at the
 * stage boundaries, synchronises the stream, and writes to the HOST array stage_ms[TSENOR_NUM_STAGES] the
 * mean duration in milliseconds of
 *   [0] workspace reset + matrix maximum (REL_MATRIX_MAX only)   [1] tile load + Algorithm 1 + sort
 *   [2] greedy selection (Algorithm 2 lines 1-6)                 [3] local search (lines 7-13) + mask write
 *       and the optional outputs.
 * loop_clock_mhz (HOST, optional): the shader clock, in MHz, that the first wave of the Dykstra kernel saw over
 * its iteration loop in the last repeat (cycle counter against the constant-rate timer; 0 if not measured, as
 * for iters == 0).
 * Arguments, validation and outputs as tsenor_mask_ex (outputs are those of the last repeat).  Creates and
 * destroys its events; allocates no device memory. */
#define TSENOR_NUM_STAGES 4
int tsenor_mask_ex_profile(const tsenor_problem* p, void* workspace, size_t workspace_bytes, tsenor_stream_t stream,
                           int repeats, float* stage_ms, double* loop_clock_mhz);

#ifdef __cplusplus
}
#endif
#endif /* TSENOR_PROFILE_H */
