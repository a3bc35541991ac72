// C ABI of the routing library: argument validation, workspace layout and the
// launch sequence.  Declarations and their contracts are in include/laser.h.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "../../include/laser.h"
#include "laser_internal.h"

namespace laser {

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct Layout {
  size_t logits, rec_cstar, rec_ids, rec_p, rec_Z, rec_lane, flexmask, fixed_cnt, tile_mask, base, chain_bits,
      chain_cum, flex_list, flex_ord, flex_tok_base, flex_slot, rec_cids, rec_pref, lin_copy, pool, status, total;
};

static Layout layout(int T, int E, bool need_logits) {
  Layout L;
  const size_t ntiles = ((size_t)T + kTile - 1) / kTile;
  const size_t slots = ntiles * kTile;
  const size_t EP = (size_t)padded_experts(E);
  size_t off = 0;
  L.logits = off;     off += align_up(need_logits ? (size_t)T * E * 4 : 0);
  L.rec_cstar = off;  off += align_up((size_t)T);
  L.rec_ids = off;    off += align_up((size_t)T * 16);
  L.rec_p = off;      off += align_up((size_t)T * 16 * 4);
  L.rec_Z = off;      off += align_up((size_t)T * 4);
  L.rec_lane = off;   off += align_up(slots * EP * 2);
  L.flexmask = off;   off += align_up(ntiles * 8);
  L.fixed_cnt = off;  off += align_up(ntiles * 64);
  L.tile_mask = off;  off += align_up(ntiles * 64 * 8);
  L.base = off;       off += align_up(ntiles * 64 * 4);
  const size_t words = (size_t)T / 32 + 2;
  L.chain_bits = off; off += align_up(words * 64 * 4);
  L.chain_cum = off;  off += align_up(words * 64 * 4);
  L.rec_cids = off;   off += align_up(slots * 16);
  L.rec_pref = off;   off += align_up(slots * 16);
  L.flex_list = off;  off += align_up(ntiles * 4);
  L.flex_ord = off;   off += align_up(ntiles * 4);
  L.flex_tok_base = off; off += align_up((ntiles + 1) * 4);
  L.flex_slot = off;  off += align_up((size_t)T * 4);
  L.lin_copy = off;   off += align_up(64 * 4);
  L.pool = off;       off += align_up((size_t)T * 4);
  L.status = off;     off += align_up(16);
  L.total = off + 256;
  return L;
}

size_t workspace_bytes(int T, int E, bool need_logits) { return layout(T, E, need_logits).total; }

Workspace carve_workspace(void* base, int T, int E, bool need_logits) {
  const Layout L = layout(T, E, need_logits);
  char* b = static_cast<char*>(base);
  Workspace w;
  w.logits = reinterpret_cast<float*>(b + L.logits);
  w.rec_cstar = reinterpret_cast<uint8_t*>(b + L.rec_cstar);
  w.rec_ids = reinterpret_cast<uint8_t*>(b + L.rec_ids);
  w.rec_p = reinterpret_cast<float*>(b + L.rec_p);
  w.rec_Z = reinterpret_cast<float*>(b + L.rec_Z);
  w.rec_lane = reinterpret_cast<uint16_t*>(b + L.rec_lane);
  w.flexmask = reinterpret_cast<unsigned long long*>(b + L.flexmask);
  w.tile_fixed_cnt = reinterpret_cast<uint8_t*>(b + L.fixed_cnt);
  w.tile_mask = reinterpret_cast<unsigned long long*>(b + L.tile_mask);
  w.tile_base = reinterpret_cast<int32_t*>(b + L.base);
  w.chain_bits = reinterpret_cast<uint32_t*>(b + L.chain_bits);
  w.chain_cum = reinterpret_cast<int32_t*>(b + L.chain_cum);
  w.rec_cids = reinterpret_cast<uint8_t*>(b + L.rec_cids);
  w.rec_pref = reinterpret_cast<uint8_t*>(b + L.rec_pref);
  w.flex_list = reinterpret_cast<int32_t*>(b + L.flex_list);
  w.flex_ord = reinterpret_cast<int32_t*>(b + L.flex_ord);
  w.flex_tok_base = reinterpret_cast<int32_t*>(b + L.flex_tok_base);
  w.flex_slot = reinterpret_cast<int32_t*>(b + L.flex_slot);
  w.lin_copy = reinterpret_cast<int32_t*>(b + L.lin_copy);
  w.pool = reinterpret_cast<int32_t*>(b + L.pool);
  w.status = reinterpret_cast<int32_t*>(b + L.status);
  return w;
}

// ------------------------------------------------------- stage timing pool ----
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

struct Profile {
  std::vector<hipEvent_t> ev;  // pairs: [2i] before, [2i+1] after the gate kernel
  int used = 0;                // pairs recorded
};
static Profile g_profile;

static int check_params(int32_t T, int32_t E, const laser_params_t* p) {
  if (!p) return LASER_E_NULL;
  if (p->struct_bytes != sizeof(laser_params_t)) return LASER_E_STRUCT;
  if (T < 0 || E < 1) return LASER_E_RANGE;
  if (p->k < 1 || p->c < p->k || p->c > E) return LASER_E_RANGE;
  if (!(p->eps_high > 0.0f) || !(p->t_fix > 0.0f) || !(p->t_fix <= 1.0f)) return LASER_E_RANGE;
  if ((int64_t)T * p->k > 0x7fffffffLL) return LASER_E_RANGE;
  if (p->trim_mode != LASER_TRIM_TOP && p->trim_mode != LASER_TRIM_RANDOM) return LASER_E_RANGE;
  if (E > LASER_MAX_E || p->c > LASER_MAX_C) return LASER_E_UNSUPPORTED;
  return LASER_OK;
}

static RouteArgs make_args(int32_t T, int32_t E, const laser_params_t* p) {
  RouteArgs a;
  a.T = T;
  a.E = E;
  a.EP = padded_experts(E);
  a.k = p->k;
  a.c = p->c;
  a.ntiles = (T + kTile - 1) / kTile;
  a.renormalize = p->renormalize ? 1 : 0;
  a.eps_high = p->eps_high;
  a.tau_ln = (float)log((double)p->t_fix);
  a.loads_in = nullptr;
  a.st_mass = nullptr;
  a.st_entropy = nullptr;
  a.st_pool = nullptr;
  a.pool_in_ws = 0;
  a.nbatch = 1;
  a.ws_stride = 0;
  return a;
}

static RandomArgs make_random(const laser_params_t* p) {
  RandomArgs r;
  r.seed = p->seed;
  r.token_offset = p->token_offset;
  r.stream = p->stream;
  return r;
}

static int route_tail(const RouteArgs& a, const Workspace& ws, int32_t* loads_inout,
                      int32_t* expert_ids, float* weights, int32_t* permutation,
                      int32_t* expert_offsets, hipStream_t s) {
  if (launch_tail(a, ws, loads_inout, expert_offsets, expert_ids, weights, permutation, s) != hipSuccess)
    return LASER_E_LAUNCH;
  return LASER_OK;
}

}  // namespace laser

using namespace laser;

extern "C" {

size_t laser_workspace_bytes(int32_t T, int32_t H, int32_t E, const laser_params_t* params) {
  if (check_params(T, E, params) != LASER_OK || H < 0) return 0;
  return workspace_bytes(T, E, true);
}

// B problems of one size, every array of problem b right behind that of problem b - 1.
static int route_impl(const void* hidden, const void* w_gate, int32_t B, int32_t T, int32_t H, int32_t E,
                      const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                      float* weights, int32_t* permutation, int32_t* expert_offsets,
                      float* logits_out, float* topk_mass, float* entropy, int32_t* pool_size,
                      void* workspace, size_t workspace_bytes_given, void* hip_stream) {
  int rc = check_params(T, E, params);
  if (rc != LASER_OK) return rc;
  if (B < 0 || B > 65535) return LASER_E_RANGE;  // (the problem index is a grid dimension)
  if (B == 0) return LASER_OK;
  if (!w_gate || !loads_inout || !expert_offsets || !workspace) return LASER_E_NULL;
  if (T > 0 && (!hidden || !expert_ids || !weights || !permutation)) return LASER_E_NULL;
  if (H < 1) return LASER_E_RANGE;
  if (params->dtype != LASER_DTYPE_F32 && params->dtype != LASER_DTYPE_BF16) return LASER_E_RANGE;
  if (params->dtype == LASER_DTYPE_BF16) {
    if (H % 8 != 0 || ((uintptr_t)hidden & 15) || ((uintptr_t)w_gate & 15)) return LASER_E_ALIGN;
  } else {
    if (H % 4 != 0 || ((uintptr_t)hidden & 15) || ((uintptr_t)w_gate & 15)) return LASER_E_ALIGN;
  }
  if ((uintptr_t)workspace & 255) return LASER_E_ALIGN;
  const bool need_logits = true;  // the layout always reserves the logits block
  const size_t ws_one = workspace_bytes(T, E, need_logits);  // a multiple of 256
  if (workspace_bytes_given / (size_t)B < ws_one) return LASER_E_WORKSPACE;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  RouteArgs a = make_args(T, E, params);
  a.nbatch = B;
  a.ws_stride = ws_one;
  a.loads_in = loads_inout;
  a.st_mass = topk_mass;
  a.st_entropy = entropy;
  a.st_pool = pool_size;
  const Workspace ws = carve_workspace(workspace, T, E, need_logits);
  const bool timed = !g_profile.ev.empty() && (size_t)(2 * g_profile.used + 1) < g_profile.ev.size() && T > 0;
  if (timed && hipEventRecord(g_profile.ev[2 * g_profile.used], s) != hipSuccess) return LASER_E_LAUNCH;
  const bool random = params->trim_mode == LASER_TRIM_RANDOM;
  // RANDOM trimming with c > k: the deterministic analysis, told to leave the pool sizes,
  // then a second look at the tokens whose pool exceeds c.  With c == k a sampled token
  // is not load-dependent but its experts are the sample: the stand-alone analysis.
  const bool resample = random && params->c > params->k;
  if (resample && !a.st_pool) a.pool_in_ws = 1;
  if (params->dtype == LASER_DTYPE_BF16) {
    float* logits = random ? (logits_out ? logits_out : ws.logits) : logits_out;
    const size_t lstride = logits_out ? (size_t)T * E : ws_one / sizeof(float);
    if (launch_gate_analyse_bf16(hidden, w_gate, H, a, ws, expert_ids, weights, logits, lstride, s) !=
        hipSuccess)
      return LASER_E_LAUNCH;
    if (random && (resample ? launch_random_resample(logits, lstride, a, ws, make_random(params), s)
                            : launch_analyse_random(logits, lstride, a, ws, make_random(params), expert_ids,
                                                    weights, s)) != hipSuccess)
      return LASER_E_LAUNCH;
  } else {
    float* logits = logits_out ? logits_out : ws.logits;
    const size_t lstride = logits_out ? (size_t)T * E : ws_one / sizeof(float);
    if (launch_gate_f32(static_cast<const float*>(hidden), static_cast<const float*>(w_gate), T, H, E, B,
                        logits, lstride, s) != hipSuccess)
      return LASER_E_LAUNCH;
    if (random && !resample) {
      if (launch_analyse_random(logits, lstride, a, ws, make_random(params), expert_ids, weights, s) !=
          hipSuccess)
        return LASER_E_LAUNCH;
    } else {
      if (launch_analyse(logits, lstride, a, ws, expert_ids, weights, s) != hipSuccess) return LASER_E_LAUNCH;
      if (resample && launch_random_resample(logits, lstride, a, ws, make_random(params), s) != hipSuccess)
        return LASER_E_LAUNCH;
    }
  }
  if (timed) {
    if (hipEventRecord(g_profile.ev[2 * g_profile.used + 1], s) != hipSuccess) return LASER_E_LAUNCH;
    ++g_profile.used;
  }
  return route_tail(a, ws, loads_inout, expert_ids, weights, permutation, expert_offsets, s);
}

int laser_route(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                float* weights, int32_t* permutation, int32_t* expert_offsets,
                float* logits_out, void* workspace, size_t workspace_bytes_given,
                void* hip_stream) {
  return route_impl(hidden, w_gate, 1, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, nullptr, nullptr, nullptr, workspace,
                    workspace_bytes_given, hip_stream);
}

int laser_route_batched(const void* hidden, const void* w_gate, int32_t B, int32_t T, int32_t H,
                        int32_t E, const laser_params_t* params, int32_t* loads_inout,
                        int32_t* expert_ids, float* weights, int32_t* permutation,
                        int32_t* expert_offsets, float* logits_out, void* workspace,
                        size_t workspace_bytes_given, void* hip_stream) {
  return route_impl(hidden, w_gate, B, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, nullptr, nullptr, nullptr, workspace,
                    workspace_bytes_given, hip_stream);
}

int laser_route_stats(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                      const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                      float* weights, int32_t* permutation, int32_t* expert_offsets,
                      float* logits_out, float* topk_mass, float* entropy, int32_t* pool_size,
                      void* workspace, size_t workspace_bytes_given, void* hip_stream) {
  return route_impl(hidden, w_gate, 1, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, topk_mass, entropy, pool_size, workspace,
                    workspace_bytes_given, hip_stream);
}

int laser_route_from_logits(const float* logits, int32_t T, int32_t E,
                            const laser_params_t* params, int32_t* loads_inout,
                            int32_t* expert_ids, float* weights, int32_t* permutation,
                            int32_t* expert_offsets, void* workspace,
                            size_t workspace_bytes_given, void* hip_stream) {
  int rc = check_params(T, E, params);
  if (rc != LASER_OK) return rc;
  if (!loads_inout || !expert_offsets || !workspace) return LASER_E_NULL;
  if (T > 0 && (!logits || !expert_ids || !weights || !permutation)) return LASER_E_NULL;
  if ((uintptr_t)workspace & 255) return LASER_E_ALIGN;
  if (workspace_bytes_given < workspace_bytes(T, E, true)) return LASER_E_WORKSPACE;
  RouteArgs a = make_args(T, E, params);
  a.loads_in = loads_inout;
  const Workspace ws = carve_workspace(workspace, T, E, true);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool random = params->trim_mode == LASER_TRIM_RANDOM;
  const bool resample = random && params->c > params->k;  // (see route_impl)
  if (resample) a.pool_in_ws = 1;
  if (random && !resample) {
    if (launch_analyse_random(logits, 0, a, ws, make_random(params), expert_ids, weights, s) != hipSuccess)
      return LASER_E_LAUNCH;
  } else {
    if (launch_analyse(logits, 0, a, ws, expert_ids, weights, s) != hipSuccess) return LASER_E_LAUNCH;
    if (resample && launch_random_resample(logits, 0, a, ws, make_random(params), s) != hipSuccess)
      return LASER_E_LAUNCH;
  }
  return route_tail(a, ws, loads_inout, expert_ids, weights, permutation, expert_offsets, s);
}

const char* laser_strerror(int code) {
  switch (code) {
    case LASER_OK: return "ok";
    case LASER_E_NULL: return "a required pointer is NULL";
    case LASER_E_RANGE: return "argument out of range (B, T, H, E, k, c, eps_high, t_fix or dtype)";
    case LASER_E_ALIGN: return "unsupported row length or pointer alignment";
    case LASER_E_WORKSPACE: return "workspace too small";
    case LASER_E_UNSUPPORTED: return "not built: E > 64 or c > 16";
    case LASER_E_STRUCT: return "laser_params_t.struct_bytes mismatch";
    case LASER_E_LAUNCH: return "HIP kernel launch failed";
    default: return "unknown error code";
  }
}

int laser_profile_enable(int32_t max_calls) {
  for (hipEvent_t e : g_profile.ev) (void)hipEventDestroy(e);
  g_profile.ev.clear();
  g_profile.used = 0;
  if (max_calls <= 0) return LASER_OK;
  g_profile.ev.resize((size_t)max_calls * 2);
  for (size_t i = 0; i < g_profile.ev.size(); ++i) {
    if (hipEventCreate(&g_profile.ev[i]) != hipSuccess) {
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(g_profile.ev[j]);
      g_profile.ev.clear();
      return LASER_E_LAUNCH;
    }
  }
  return LASER_OK;
}

int laser_profile_read(double* gate_ms_sum, int64_t* gate_launches) {
  if (!gate_ms_sum || !gate_launches) return LASER_E_NULL;
  double sum = 0.0;
  for (int i = 0; i < g_profile.used; ++i) {
    if (hipEventSynchronize(g_profile.ev[2 * i + 1]) != hipSuccess) return LASER_E_LAUNCH;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, g_profile.ev[2 * i], g_profile.ev[2 * i + 1]) != hipSuccess)
      return LASER_E_LAUNCH;
    sum += ms;
  }
  *gate_ms_sum = sum;
  *gate_launches = g_profile.used;
  g_profile.used = 0;
  return LASER_OK;
}

int laser_profile_event_overhead(void* hip_stream, double* overhead_ms) {
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

int laser_profile_plain_read(const void* device_buf, size_t bytes, size_t bytes_per_launch,
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
