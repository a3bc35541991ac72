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
  size_t status, logits, rec_cstar, rec_ids, rec_p, rec_Z, rec_lane, flexmask, fixed_cnt, tile_mask, base, chain_bits,
      chain_cum, flex_list, flex_ord, flex_tok_base, flex_slot, rec_cids, rec_pref, lin_copy, pool, seg, split, needed, total;
};

// cw: candidates per token record (record_width(c)).  The status words come first, so
// that laser_status() finds them without knowing the sizes of the call.
static Layout layout(int T, int E, int cw) {
  Layout L;
  const size_t ntiles = ((size_t)T + kTile - 1) / kTile;
  const size_t slots = ntiles * kTile;
  const size_t EP = (size_t)padded_experts(E);
  size_t off = 0;
  L.status = off;     off += align_up(16);
  L.logits = off;     off += align_up((size_t)T * E * 4);
  L.rec_cstar = off;  off += align_up((size_t)T);
  L.rec_ids = off;    off += align_up((size_t)T * cw);
  L.rec_p = off;      off += align_up((size_t)T * cw * 4);
  L.rec_Z = off;      off += align_up((size_t)T * 4);
  L.rec_lane = off;   off += align_up(slots * EP * 2);
  L.flexmask = off;   off += align_up(ntiles * 8);
  L.fixed_cnt = off;  off += align_up(ntiles * 64);
  L.tile_mask = off;  off += align_up(ntiles * 64 * 8);
  L.base = off;       off += align_up(ntiles * 64 * 4);
  // (a pipelined call numbers the flexible tokens of every segment from a multiple of 32:
  // up to 32 numbers, one word, are skipped per segment, of which there are fewer than ntiles)
  const size_t words = (size_t)T / 32 + 2 + ntiles;
  L.chain_bits = off; off += align_up(words * 64 * 4);
  L.chain_cum = off;  off += align_up(words * 64 * 4);
  L.rec_cids = off;   off += align_up(slots * 16);
  L.rec_pref = off;   off += align_up(slots * 16);
  L.flex_list = off;  off += align_up(ntiles * 4);
  L.flex_ord = off;   off += align_up(ntiles * 4);
  L.flex_tok_base = off; off += align_up((ntiles + 1) * 4);
  L.flex_slot = off;  off += align_up(((size_t)T + 32 * ntiles) * 4);
  L.lin_copy = off;   off += align_up(64 * 4);
  L.pool = off;       off += align_up((size_t)T * 4);
  L.seg = off;        off += align_up((kSegDone + ntiles) * 4);
  // (last, and optional: a call runs in `needed` bytes, without the split)
  L.needed = off + 256;
  L.split = off;      off += align_up(ntiles <= (size_t)kSplitMaxTiles ? ntiles * 8 * kTile * 64 * 4 : 0);
  L.total = off + 256;
  return L;
}

size_t workspace_bytes(int T, int E, int cw) { return layout(T, E, cw).total; }
size_t workspace_needed_bytes(int T, int E, int cw) { return layout(T, E, cw).needed; }

Workspace carve_workspace(void* base, int T, int E, int cw) {
  const Layout L = layout(T, E, cw);
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
  w.seg = reinterpret_cast<int32_t*>(b + L.seg);
  w.split_part = reinterpret_cast<float*>(b + L.split);
  return w;
}

static int check_params(int32_t T, int32_t E, const laser_params_t* p) {
  if (!p) return LASER_E_NULL;
  if (p->struct_bytes != sizeof(laser_params_t)) return LASER_E_STRUCT;
  if (T < 0 || E < 1) return LASER_E_RANGE;
  if (p->k < 1 || p->c < p->k || p->c > E) return LASER_E_RANGE;
  if (!(p->eps_high > 0.0f) || !(p->t_fix > 0.0f) || !(p->t_fix <= 1.0f)) return LASER_E_RANGE;
  if ((int64_t)T * p->k > 0x7fffffffLL) return LASER_E_RANGE;
  if (p->trim_mode != LASER_TRIM_TOP && p->trim_mode != LASER_TRIM_RANDOM) return LASER_E_RANGE;
  if (E > LASER_MAX_E || p->k > LASER_MAX_K) return LASER_E_UNSUPPORTED;
  return LASER_OK;
}

static RouteArgs make_args(int32_t T, int32_t E, const laser_params_t* p) {
  RouteArgs a;
  a.T = T;
  a.E = E;
  a.EP = padded_experts(E);
  a.k = p->k;
  a.c = p->c;
  a.cw = record_width(p->c);
  a.ntiles = (T + kTile - 1) / kTile;
  a.renormalize = p->renormalize ? 1 : 0;
  a.eps_high = p->eps_high;
  a.tau_ln = (float)log((double)p->t_fix);
  a.loads_in = nullptr;
  a.st_mass = nullptr;
  a.st_entropy = nullptr;
  a.st_pool = nullptr;
  a.pool_in_ws = 0;
  // the bounded waits of the tail kernel: sized from T unless the caller fixes them
  a.spin_limit = p->poll_budget != 0 ? (long long)p->poll_budget : kSpinFloor + kSpinPerToken * (long long)T;
  a.nbatch = 1;
  a.ws_stride = 0;
  a.seg_tiles = 0;
  a.seg_first = 0;
  a.nseg = 0;
  a.split = 0;
  a.split_cnt = nullptr;
  a.one_permutation = nullptr;
  a.one_expert_offsets = nullptr;
  a.one_loads = nullptr;
  return a;
}

static RandomArgs make_random(const laser_params_t* p) {
  RandomArgs r;
  r.seed = p->seed;
  r.token_offset = p->token_offset;
  r.stream = p->stream;
  return r;
}

// The segments of a pipelined call (a.seg_tiles == 0: the call is not pipelined), from
// laser_params_t.pipeline_tiles.  Left to itself the library pipelines batches of at least
// six rounds of the persistent grid (one workgroup per compute unit but one): a first
// segment of one round, so that the chain starts early, then segments of two rounds -- a
// segment is complete when its last round is, so whole rounds it is.  (Measured on the
// prefill shape: with many load-dependent tokens pipelining pays from three rounds on,
// -12 % at four, -24 % at eight; with none it costs 15 % at four rounds -- the compute
// unit given to the chain and the clearing launch -- and gains 5 % at eight, where the
// prefix over the tiles leaves the tail kernel.)
static void choose_segments(RouteArgs& a, uint32_t wanted) {
  a.seg_tiles = a.seg_first = a.nseg = 0;
  if (wanted == 1) return;
  if (wanted >= 2) {
    if ((uint32_t)a.ntiles <= wanted) return;
    a.seg_tiles = a.seg_first = (int)wanted;
  } else {
    const int round = pipeline_workgroups();
    if (a.ntiles < 6 * round) return;
    a.seg_first = round;
    a.seg_tiles = 2 * round;
  }
  a.nseg = 1 + (a.ntiles - a.seg_first + a.seg_tiles - 1) / a.seg_tiles;
}

// The fast analysis kernels carry at most kMaxC candidates per token.  A wide call runs
// them with the trimming size cut to that (for the logits and the statistics, which do
// not depend on c) and then the general analysis, which writes every record again.
static RouteArgs narrowed(const RouteArgs& a) {
  RouteArgs n = a;
  n.c = a.c < kMaxC ? a.c : kMaxC;
  n.k = a.k;
  return n;
}

// B problems of one size, every array of problem b right behind that of problem b - 1.
int route_impl(const void* hidden, const void* w_gate, int32_t B, int32_t T, int32_t H, int32_t E,
               const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids, float* weights,
               int32_t* permutation, int32_t* expert_offsets, float* logits_out, float* topk_mass,
               float* entropy, int32_t* pool_size, void* workspace, size_t workspace_bytes_given,
               void* hip_stream, BenchTimer* timer) {
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
  const int cw = record_width(params->c);
  // (a single problem runs in the bytes it needs; what laser_workspace_bytes reports beyond
  // them holds the partial tiles of a split call, so a workspace sized for a larger batch
  // always serves a smaller one)
  const size_t ws_one = workspace_bytes(T, E, cw);  // a multiple of 256
  const size_t ws_needed = B == 1 ? workspace_needed_bytes(T, E, cw) : ws_one;
  if (workspace_bytes_given / (size_t)B < ws_needed) return LASER_E_WORKSPACE;
  if (timer && timer->used >= timer->capacity) return LASER_E_RANGE;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  RouteArgs a = make_args(T, E, params);
  a.nbatch = B;
  a.ws_stride = ws_one;
  a.loads_in = loads_inout;
  a.st_mass = topk_mass;
  a.st_entropy = entropy;
  a.st_pool = pool_size;
  const Workspace ws = carve_workspace(workspace, T, E, cw);
  hipEvent_t* ev = timer ? timer->ev + 3 * (size_t)timer->used : nullptr;
  if (ev && hipEventRecord(ev[0], s) != hipSuccess) return LASER_E_LAUNCH;
  const bool random = params->trim_mode == LASER_TRIM_RANDOM;
  const bool wide = cw > kMaxC;
  // RANDOM trimming with c > k: the deterministic analysis, told to leave the pool sizes,
  // then a second look at the tokens whose pool exceeds c.  With c == k a sampled token
  // is not load-dependent but its experts are the sample: the general analysis.
  const bool resample = random && params->c > params->k && !wide;
  const bool general = wide || (random && !resample);
  if (resample && !a.st_pool) a.pool_in_ws = 1;
  // Pipelined: one problem through the fused bf16 kernel, nothing between it and the tail
  // kernel.
  if (params->dtype == LASER_DTYPE_BF16 && B == 1 && !general && !resample) {
    choose_segments(a, params->pipeline_tiles);
  }
  // Small calls, one problem through the fused bf16 kernel (whatever follows it): eight or
  // four workgroups per tile share the contraction axis (gate_split.hip).
  if (params->dtype == LASER_DTYPE_BF16 && B == 1 && a.nseg == 0 && a.ntiles >= 1 &&
      a.ntiles <= kSplitMaxTiles && params->split_k != 1 && workspace_bytes_given >= ws_one) {
    int32_t* counters = split_counters_for(workspace);
    if (counters != nullptr) {
      a.split = a.ntiles <= kSplitEightTiles ? 8 : 4;
      a.split_cnt = counters;
      if (a.ntiles == 1 && !general && !resample) {  // (nothing between the fused kernel and the tail kernel)
        a.one_permutation = permutation;
        a.one_expert_offsets = expert_offsets;
        a.one_loads = loads_inout;
      }
    }
  }
  const RouteArgs an = wide ? narrowed(a) : a;  // what the fast analysis kernels are given
  const size_t lstride = logits_out ? (size_t)T * E : ws_one / sizeof(float);
  float* logits;
  if (params->dtype == LASER_DTYPE_BF16) {
    logits = (random || wide) ? (logits_out ? logits_out : ws.logits) : logits_out;
    if (launch_gate_analyse_bf16(hidden, w_gate, H, an, ws, expert_ids, weights, logits, lstride, s) !=
        hipSuccess)
      return LASER_E_LAUNCH;
  } else {
    logits = logits_out ? logits_out : ws.logits;
    if (launch_gate_f32(static_cast<const float*>(hidden), static_cast<const float*>(w_gate), T, H, E, B,
                        logits, lstride, s) != hipSuccess)
      return LASER_E_LAUNCH;
    // (before the general analysis only where the statistics are wanted)
    if ((!general || wants_stats(a)) && launch_analyse(logits, lstride, an, ws, expert_ids, weights, s) != hipSuccess)
      return LASER_E_LAUNCH;
  }
  if (general) {
    if (launch_analyse_general(logits, lstride, a, ws, random, make_random(params), expert_ids, weights, s) !=
        hipSuccess)
      return LASER_E_LAUNCH;
  } else if (resample) {
    if (launch_random_resample(logits, lstride, a, ws, make_random(params), s) != hipSuccess)
      return LASER_E_LAUNCH;
  }
  if (ev && hipEventRecord(ev[1], s) != hipSuccess) return LASER_E_LAUNCH;
  if (launch_tail(a, ws, loads_inout, expert_offsets, expert_ids, weights, permutation, s) != hipSuccess)
    return LASER_E_LAUNCH;
  if (ev) {
    if (hipEventRecord(ev[2], s) != hipSuccess) return LASER_E_LAUNCH;
    ++timer->used;
  }
  return LASER_OK;
}

// ---- the workspace of laser_route_static ------------------------------------------
// One array per GPU, part of the library's code object: it exists from the moment the
// library is loaded on a device until the process ends.  In host code the array's name
// is only a handle for the runtime's symbol lookup, not a device address; the address
// on each device is looked up once (with that device current) and kept.
constexpr size_t kStaticBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

struct StaticWorkspace {
  void* ptr[kMaxDevices] = {};
};
static StaticWorkspace g_static;

// The current device's copy of the array, or NULL if the lookup failed.
static void* static_workspace() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  if (g_static.ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_static.ptr[dev] = p;
  }
  return g_static.ptr[dev];
}

}  // namespace laser

using namespace laser;

extern "C" {

size_t laser_static_workspace_bytes(void) { return kStaticBytes; }

int laser_route_static(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                       const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                       float* weights, int32_t* permutation, int32_t* expert_offsets,
                       float* logits_out, void* hip_stream) {
  const int rc = check_params(T, E, params);
  if (rc != LASER_OK) return rc;
  if (workspace_needed_bytes(T, E, record_width(params->c)) > kStaticBytes) return LASER_E_WORKSPACE;
  void* ws = static_workspace();
  if (!ws) return LASER_E_LAUNCH;
  return route_impl(hidden, w_gate, 1, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, nullptr, nullptr, nullptr, ws, kStaticBytes, hip_stream,
                    nullptr);
}

int laser_status_static(void* hip_stream, int32_t* status) {
  void* ws = static_workspace();
  if (!ws) return LASER_E_LAUNCH;
  return laser_status(ws, hip_stream, status);
}

size_t laser_workspace_bytes(int32_t T, int32_t H, int32_t E, const laser_params_t* params) {
  if (check_params(T, E, params) != LASER_OK || H < 0) return 0;
  return workspace_bytes(T, E, record_width(params->c));
}

int laser_route(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                float* weights, int32_t* permutation, int32_t* expert_offsets,
                float* logits_out, void* workspace, size_t workspace_bytes_given,
                void* hip_stream) {
  return route_impl(hidden, w_gate, 1, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, nullptr, nullptr, nullptr, workspace,
                    workspace_bytes_given, hip_stream, nullptr);
}

int laser_route_batched(const void* hidden, const void* w_gate, int32_t B, int32_t T, int32_t H,
                        int32_t E, const laser_params_t* params, int32_t* loads_inout,
                        int32_t* expert_ids, float* weights, int32_t* permutation,
                        int32_t* expert_offsets, float* logits_out, void* workspace,
                        size_t workspace_bytes_given, void* hip_stream) {
  return route_impl(hidden, w_gate, B, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, nullptr, nullptr, nullptr, workspace,
                    workspace_bytes_given, hip_stream, nullptr);
}

int laser_route_stats(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                      const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                      float* weights, int32_t* permutation, int32_t* expert_offsets,
                      float* logits_out, float* topk_mass, float* entropy, int32_t* pool_size,
                      void* workspace, size_t workspace_bytes_given, void* hip_stream) {
  return route_impl(hidden, w_gate, 1, T, H, E, params, loads_inout, expert_ids, weights, permutation,
                    expert_offsets, logits_out, topk_mass, entropy, pool_size, workspace,
                    workspace_bytes_given, hip_stream, nullptr);
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
  const int cw = record_width(params->c);
  if (workspace_bytes_given < workspace_bytes(T, E, cw)) return LASER_E_WORKSPACE;
  RouteArgs a = make_args(T, E, params);
  a.loads_in = loads_inout;
  const Workspace ws = carve_workspace(workspace, T, E, cw);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool random = params->trim_mode == LASER_TRIM_RANDOM;
  const bool wide = cw > kMaxC;
  const bool resample = random && params->c > params->k && !wide;  // (see route_impl)
  if (resample) a.pool_in_ws = 1;
  if (wide || (random && !resample)) {
    if (launch_analyse_general(logits, 0, a, ws, random, make_random(params), expert_ids, weights, s) !=
        hipSuccess)
      return LASER_E_LAUNCH;
  } else {
    if (launch_analyse(logits, 0, a, ws, expert_ids, weights, s) != hipSuccess) return LASER_E_LAUNCH;
    if (resample && launch_random_resample(logits, 0, a, ws, make_random(params), s) != hipSuccess)
      return LASER_E_LAUNCH;
  }
  if (launch_tail(a, ws, loads_inout, expert_offsets, expert_ids, weights, permutation, s) != hipSuccess)
    return LASER_E_LAUNCH;
  return LASER_OK;
}

int laser_status(const void* workspace, void* hip_stream, int32_t* status) {
  if (!workspace || !status) return LASER_E_NULL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int32_t words[4] = {0, 0, 0, 0};
  // (the status words are the first bytes of a workspace)
  if (hipMemcpyAsync(words, workspace, sizeof(words), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return LASER_E_LAUNCH;
  *status = words[kStatusError];
  return LASER_OK;
}

const char* laser_strerror(int code) {
  switch (code) {
    case LASER_OK: return "ok";
    case LASER_E_NULL: return "a required pointer is NULL";
    case LASER_E_RANGE: return "argument out of range (B, T, H, E, k, c, eps_high, t_fix or dtype)";
    case LASER_E_ALIGN: return "unsupported row length or pointer alignment";
    case LASER_E_WORKSPACE: return "workspace too small";
    case LASER_E_UNSUPPORTED: return "not built: E > 64 or k > 16";
    case LASER_E_STRUCT: return "laser_params_t.struct_bytes mismatch";
    case LASER_E_LAUNCH: return "a HIP call failed (kernel launch, event, copy)";
    default: return "unknown error code";
  }
}

}  // extern "C"
