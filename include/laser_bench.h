/*
 * laser_bench.h -- measurement helpers of the routing library, for benchmarks only.
 *
 * Nothing here is part of the routing path, and nothing here follows the conventions of
 * laser.h: these calls create and destroy HIP events, synchronise, and launch probe
 * kernels of their own.  A timer is an opaque pool of HIP events; laser_bench_route is
 * laser_route with the launches of one call bracketed by three events of that pool
 * (before the projection/analysis kernels, between them and the tail kernel, after it),
 * so that timing is a property of the call that asks for it and the plain entry points
 * carry no trace of it.
 */
#ifndef LASER_BENCH_H_
#define LASER_BENCH_H_

#include "laser.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct laser_bench_timer laser_bench_timer_t;

/* A pool for up to `max_calls` timed calls (host object; *timer receives it). */
int laser_bench_timer_create(int32_t max_calls, laser_bench_timer_t** timer);
void laser_bench_timer_destroy(laser_bench_timer_t* timer);

/* laser_route, timed.  Calls beyond the pool's capacity return LASER_E_RANGE. */
int laser_bench_route(laser_bench_timer_t* timer, const void* hidden, const void* w_gate, int32_t T,
                      int32_t H, int32_t E, const laser_params_t* params, int32_t* loads_inout,
                      int32_t* expert_ids, float* weights, int32_t* permutation,
                      int32_t* expert_offsets, float* logits_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/*
 * Waits for the recorded events and returns, per timed call in call order, the
 * milliseconds between the first and second event (projection + analysis) in
 * first_ms[i] and between the second and third (tail kernel) in tail_ms[i] (host arrays
 * of `capacity` entries, either may be NULL); *calls receives the number of calls
 * recorded.  The record is cleared.  Every figure includes the cost of the events
 * themselves, see laser_bench_event_overhead.
 */
int laser_bench_timer_read(laser_bench_timer_t* timer, double* first_ms, double* tail_ms,
                           int64_t capacity, int64_t* calls);

/*
 * What a pair of HIP events adds to the kernel it brackets, in milliseconds (host
 * pointer): the library launches a kernel that spins for a fixed 10 microseconds of
 * the GPU's constant-rate clock between event pairs on `hip_stream`, synchronises,
 * and returns the median of (elapsed - 10 us).  Creates and destroys its own events.
 */
int laser_bench_event_overhead(void* hip_stream, double* overhead_ms);

/*
 * The box's own ceiling for a streaming read: a plain kernel (16-byte loads, nothing
 * else) reads `bytes` of `device_buf` (device pointer, 16-byte aligned) in back-to-back
 * launches of `bytes_per_launch` (a multiple of 16; a last partial piece is skipped) on
 * `hip_stream`, bracketed by one HIP event pair; the call synchronises and returns the
 * elapsed milliseconds and the number of launches (host pointers).  `device_sink` is a
 * device word the kernel may write.  Pass a buffer well beyond the 256 MB last-level
 * cache to measure HBM.
 */
int laser_bench_plain_read(const void* device_buf, size_t bytes, size_t bytes_per_launch,
                           void* device_sink, void* hip_stream, double* ms_total,
                           int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* LASER_BENCH_H_ */
