/* Measurement helpers of the NAtS-L hybrid-attention library: per-kernel timing for benchmarks and a
 * matrix-core issue probe.  No part of the method (Sections 3-4 of the paper define none of this); a
 * program that only computes includes nats.h alone.  Same conventions as nats.h: plain C, status codes,
 * nats_last_error() for the message. */
#ifndef NATS_MEASURE_H
#define NATS_MEASURE_H

#include "nats.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------- *
 * Optional per-kernel timing (for benchmarks; off by default)
 * ------------------------------------------------------------------------- */
/* Creates max_records hipEvent pairs and turns recording on: until nats_profile_end, every kernel
 * the forward / decode calls launch is bracketed by an event pair on the call's stream (records
 * beyond max_records are dropped).  This is the one place the library creates HIP objects. */
nats_status nats_profile_begin(int max_records);

/* Turns recording off, waits for the recorded events, and aggregates per kernel name:
 * names[i*32 .. i*32+31] (NUL-terminated), total_ms[i], launches[i] for up to max_kernels kernels.
 * All three arrays are HOST memory owned by the caller.  Destroys the events.
 * Returns the number of distinct kernels written, or a negative nats_status. */
int nats_profile_end(char* names, float* total_ms, int32_t* launches, int max_kernels);

/* Measurement helper, no part of the method: launches a kernel in which every wavefront of a
 * chip-filling grid issues iters x 8 independent 16x16x32 fp16 MFMA (the instruction the bf16 path
 * is built on) and nothing else.  out: DEVICE buffer of at least 2048 floats (scratch, overwritten).
 * Returns the floating-point operations that launch performs (the caller times it on the stream),
 * or a negative value on error (see nats_last_error). */
double nats_probe_mfma(int iters, float* out, size_t out_floats, void* hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* NATS_MEASURE_H */
