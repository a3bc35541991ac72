// Measurement helpers for benchmarks (include/laser_bench.h): an event pool that times the
// stages of a routing call, the cost of an event pair, and the box's plain streaming read.
// Not part of the routing path.
#include <algorithm>
#include <new>
#include <vector>

#include "../../include/laser_bench.h"
#include "laser_internal.h"

struct laser_bench_timer {
  laser::BenchTimer t;
};

namespace laser {

// Spins for `ticks` of the constant 100 MHz clock; used to calibrate event overhead.
__global__ void spin_kernel(long long ticks) {
  const long long t0 = wall_clock64();
  while (wall_clock64() - t0 < ticks) {
  }
}

// Reads `n16` 16-byte words and keeps nothing: the plain streaming read that other
// kernels' bandwidth is compared with.  The xor keeps the loads alive; the store
// never happens for real data streams short of a 2^-32 coincidence per thread, and
// `sink` is a valid device word in any case.
typedef unsigned int stream_u4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void plain_read_kernel(const uint4* __restrict__ p16, size_t n16,
                                                         unsigned* __restrict__ sink) {
  // (non-temporal loads, as the gate kernel uses for the rows it streams)
  const stream_u4* p = reinterpret_cast<const stream_u4*>(p16);
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  unsigned x = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const stream_u4 a = __builtin_nontemporal_load(p + i), b = __builtin_nontemporal_load(p + i + stride),
                    c = __builtin_nontemporal_load(p + i + 2 * stride),
                    d = __builtin_nontemporal_load(p + i + 3 * stride);
    x ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const stream_u4 a = __builtin_nontemporal_load(p + i);
    x ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (x == 0x9E3779B9u) *sink = x;
}

}  // namespace laser

using namespace laser;

extern "C" {

int laser_bench_timer_create(int32_t max_calls, laser_bench_timer_t** timer) {
  if (!timer) return LASER_E_NULL;
  *timer = nullptr;
  if (max_calls < 1 || max_calls > (1 << 20)) return LASER_E_RANGE;
  laser_bench_timer* h = new (std::nothrow) laser_bench_timer;
  if (!h) return LASER_E_RANGE;
  h->t.capacity = max_calls;
  h->t.used = 0;
  h->t.ev = new (std::nothrow) hipEvent_t[3 * (size_t)max_calls];
  if (!h->t.ev) {
    delete h;
    return LASER_E_RANGE;
  }
  for (size_t i = 0; i < 3 * (size_t)max_calls; ++i) {
    if (hipEventCreate(&h->t.ev[i]) != hipSuccess) {
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(h->t.ev[j]);
      delete[] h->t.ev;
      delete h;
      return LASER_E_LAUNCH;
    }
  }
  *timer = h;
  return LASER_OK;
}

void laser_bench_timer_destroy(laser_bench_timer_t* timer) {
  if (!timer) return;
  for (size_t i = 0; i < 3 * (size_t)timer->t.capacity; ++i) (void)hipEventDestroy(timer->t.ev[i]);
  delete[] timer->t.ev;
  delete timer;
}

int laser_bench_route(laser_bench_timer_t* timer, const void* hidden, const void* w_gate, int32_t T,
                      int32_t H, int32_t E, const laser_params_t* params, int32_t* loads_inout,
                      int32_t* expert_ids, float* weights, int32_t* permutation,
                      int32_t* expert_offsets, float* logits_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  if (!timer) return LASER_E_NULL;
  return route_impl(hidden, w_gate, 1, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, nullptr, nullptr, nullptr, workspace, workspace_bytes,
                    hip_stream, &timer->t);
}

int laser_bench_timer_read(laser_bench_timer_t* timer, double* first_ms, double* tail_ms,
                           int64_t capacity, int64_t* calls) {
  if (!timer || !calls) return LASER_E_NULL;
  const int n = timer->t.used;
  for (int i = 0; i < n; ++i) {
    hipEvent_t* ev = timer->t.ev + 3 * (size_t)i;
    if (hipEventSynchronize(ev[2]) != hipSuccess) return LASER_E_LAUNCH;
    float a = 0.0f, b = 0.0f;
    if (hipEventElapsedTime(&a, ev[0], ev[1]) != hipSuccess || hipEventElapsedTime(&b, ev[1], ev[2]) != hipSuccess)
      return LASER_E_LAUNCH;
    if (i < capacity) {
      if (first_ms) first_ms[i] = a;
      if (tail_ms) tail_ms[i] = b;
    }
  }
  *calls = n;
  timer->t.used = 0;
  return LASER_OK;
}

int laser_bench_event_overhead(void* hip_stream, double* overhead_ms) {
  if (!overhead_ms) return LASER_E_NULL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int reps = 21;
  const long long ticks = 1000;  // 10 us at 100 MHz
  std::vector<hipEvent_t> ev(2 * reps);
  for (size_t i = 0; i < ev.size(); ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) return LASER_E_LAUNCH;
  for (int i = 0; i < reps; ++i) {
    if (hipEventRecord(ev[2 * i], s) != hipSuccess) return LASER_E_LAUNCH;
    hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(64), 0, s, ticks);
    if (hipEventRecord(ev[2 * i + 1], s) != hipSuccess) return LASER_E_LAUNCH;
  }
  std::vector<float> ms(reps);
  int rc = LASER_OK;
  for (int i = 0; i < reps; ++i) {
    if (hipEventSynchronize(ev[2 * i + 1]) != hipSuccess ||
        hipEventElapsedTime(&ms[i], ev[2 * i], ev[2 * i + 1]) != hipSuccess)
      rc = LASER_E_LAUNCH;
  }
  for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  if (rc != LASER_OK) return rc;
  std::sort(ms.begin(), ms.end());
  *overhead_ms = (double)ms[reps / 2] - 0.010;
  return LASER_OK;
}

int laser_bench_plain_read(const void* device_buf, size_t bytes, size_t bytes_per_launch,
                             void* device_sink, void* hip_stream, double* ms_total,
                             int64_t* launches) {
  if (!device_buf || !device_sink || !ms_total || !launches) return LASER_E_NULL;
  if (bytes == 0 || bytes_per_launch == 0 || (bytes_per_launch & 15) != 0 ||
      (reinterpret_cast<uintptr_t>(device_buf) & 15) != 0)
    return LASER_E_RANGE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return LASER_E_LAUNCH;
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return LASER_E_LAUNCH;
  }
  int rc = LASER_OK;
  int64_t n = 0;
  if (hipEventRecord(e0, s) != hipSuccess) rc = LASER_E_LAUNCH;
  for (size_t off = 0; rc == LASER_OK && off + bytes_per_launch <= bytes; off += bytes_per_launch) {
    const size_t n16 = bytes_per_launch >> 4;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 2048);
    clear_stale_error();
    hipLaunchKernelGGL(plain_read_kernel, dim3(blocks), dim3(256), 0, s,
                       reinterpret_cast<const uint4*>(static_cast<const char*>(device_buf) + off), n16,
                       static_cast<unsigned*>(device_sink));
    if (hipGetLastError() != hipSuccess) rc = LASER_E_LAUNCH;
    ++n;
  }
  float ms = 0.0f;
  if (rc == LASER_OK && (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                         hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = LASER_E_LAUNCH;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != LASER_OK) return rc;
  *ms_total = ms;
  *launches = n;
  return LASER_OK;
}


}  // extern "C"
