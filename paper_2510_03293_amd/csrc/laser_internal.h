// Internal declarations shared by the HIP translation units of the routing
// library: workspace layout, per-call parameters, kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace laser {

constexpr int kTile = 64;        // tokens per tile (one wave-wide bit mask per tile)
constexpr int kMaxE = 64;        // experts: one lane of a wavefront per expert
constexpr int kMaxC = 16;        // trimming size the fast kernels carry (candidate ranks fit 4 bits)
constexpr int kWideC = 64;       // trimming sizes above kMaxC: records of kWideC candidates, general kernels
constexpr int kMaxK = 16;        // experts per token
constexpr int kSplitMaxTiles = 64;  // calls of up to this many tiles may cut the contraction axis over workgroups
constexpr int kSplitEightTiles = 32;  // ... over eight per tile up to here, over four beyond

// Per-call scalars handed to every kernel by value.
struct RouteArgs {
  int T;            // tokens
  int E;            // experts
  int EP;           // experts padded to 8/16/32/64 (8 lanes per token x EP/8 each)
  int k;            // experts per token
  int c;            // trimming size
  int cw;           // candidates per token record: kMaxC, or kWideC when c > kMaxC ("wide" calls)
  int ntiles;       // ceil(T / kTile)
  int renormalize;  // weights over the chosen k (1) or raw softmax scores (0)
  float eps_high;   // top-k mass threshold
  float tau_ln;     // fl32(ln t_fix): pool cut-off in the logit domain
  const int32_t* loads_in;  // [E] the caller's counters before token 0 (copied to the workspace
                            // by the analysis so that the tail can read them while it writes)
  // optional per-token statistics, [T] each, any may be NULL (all NULL: not computed)
  float* st_mass;      // top-k mass M_k
  float* st_entropy;   // Shannon entropy of the scores, nats
  int32_t* st_pool;    // pool size m (candidates above the cut, united with the top-k)
  int pool_in_ws;      // 1: nobody asked for st_pool but RANDOM trimming needs the pool sizes:
                       // the kernels write and read them in the workspace (Workspace::pool)
  // batched calls: the kernels run with the problem index in blockIdx.y
  long long spin_limit;  // polls a finishing wavefront spends on one flag of the chain before it gives up
  int nbatch;          // problems in the call (1: all of the above is the one problem's)
  size_t ws_stride;    // bytes from one problem's workspace to the next
  // pipelined calls (large single problems through the fused bf16 kernel): the tiles are cut
  // into segments of seg_tiles tiles, and the chain over a segment runs, inside the gate
  // kernel, as soon as the segment's tiles have been analysed (see Workspace::seg)
  int seg_tiles;       // tiles per segment; 0: the call is not pipelined
  int seg_first;       // tiles of segment 0 (a short one lets the chain start early)
  int nseg;            // segments: 1 + ceil((ntiles - seg_first) / seg_tiles); 0 when not pipelined
  // small single problems through the fused bf16 kernel: the contraction axis of a tile cut
  // over `split` workgroups (gate_split.hip)
  int split;           // workgroups per tile (4 or 8); 0: one workgroup per tile
  int32_t* split_cnt;  // [ntiles] arrival counters, zero between calls (the library's own memory)
  // a split call of one tile without load-dependent tokens is finished by the workgroup
  // that analyses it (the tail kernel then returns at once); NULL: never
  int32_t* one_permutation;     // the call's permutation ...
  int32_t* one_expert_offsets;  // ... expert_offsets ...
  int32_t* one_loads;           // ... and loads_inout
};
// First tile of segment j of a pipelined call (j <= nseg; segment nseg starts at ntiles or beyond).
__host__ __device__ inline int segment_start(const RouteArgs& a, int j) {
  return j == 0 ? 0 : a.seg_first + (j - 1) * a.seg_tiles;
}
// Trimming mode RANDOM: what makes the sample reproducible.
struct RandomArgs {
  unsigned long long seed;          // generator key
  unsigned long long token_offset;  // index of token 0 of this call in the caller's numbering
  uint32_t stream;                  // caller's stream id (e.g. the layer)
};
inline bool wants_stats(const RouteArgs& a) { return a.st_mass || a.st_entropy || a.st_pool || a.pool_in_ws; }

// Device workspace carved out of the caller's buffer.  Records are written by
// the per-token analysis, consumed by the load-ordered chain and the finishing
// pass.  "slot" = tile * kTile + (rank of the token among its tile's flexible
// tokens), so a tile's flexible records are contiguous.
struct Workspace {
  float* logits;               // [T,E]   gate logits (unless the caller gave a buffer)
  uint8_t* rec_cstar;          // [T]     working-set size of a flexible token, else 0
  uint8_t* rec_ids;            // [T,cw]  experts by descending score
  float* rec_p;                // [T,cw]  their softmax numerators exp(z - z_max)
  float* rec_Z;                // [T]     softmax normaliser
  uint16_t* rec_lane;          // [slot,EP] per expert: (fixed-prefix << 4 | rank) or 0xFFFF
                               //           (wide calls: fixed-prefix << 6 | rank)
  unsigned long long* flexmask;    // [ntiles] bit i: token i of the tile is flexible
  uint8_t* tile_fixed_cnt;     // [ntiles,64] assignments of the tile's non-flexible tokens (<= 64)
  unsigned long long* tile_mask;   // [ntiles,64] per expert: the tile's non-flexible tokens
                               //           assigned to it (bit = token within the tile)
  int32_t* tile_base;          // [ntiles,64] assignments of all earlier tiles, per expert
  uint8_t* rec_cids;           // [slot,16] lanes the chain reads: candidates by rank, padded
  uint8_t* rec_pref;           // [slot,16] per candidate (by rank): earlier fixed tokens of the
                               //           tile assigned to it (<= 63); 0xFF beyond the working set
  int32_t* flex_list;          // [ntiles]  tiles that hold flexible tokens, ascending
  int32_t* flex_ord;           // [ntiles]  number of such tiles before this tile
  int32_t* flex_tok_base;      // [ntiles+1] flexible tokens in earlier tiles; [ntiles] = all
  int32_t* flex_slot;          // [T]       slot of the f-th flexible token (token order)
  uint32_t* chain_bits;        // [T/32+1,64] per expert: bit f%32 of word f/32 = chosen for
                               //           the f-th flexible token
  int32_t* chain_cum;          // [T/32+2,64] per expert: choices by flexible tokens < 32*w
  int32_t* lin_copy;           // [64] loads before token 0 (0 beyond E)
  int32_t* pool;               // [T] pool sizes, when RANDOM trimming needs them (see pool_in_ws)
  int32_t* status;             // [4] see kStatus*: cleared by the analysis kernel of a call (the
                               //     first bytes of the workspace, so that a query needs no sizes)
  int32_t* seg;                // [kSegDone + ntiles] pipelined calls only, see kSeg*: how far the
                               //     chain has come, and per tile how much of its analysis is written
  float* split_part;           // [ntiles,8,64,64] split calls only (ntiles <= kSplitMaxTiles): the partial
                               //     logit tiles of the eight wavefront roles
};

// Problem b of a batched call.  All problems share the sizes; every array of problem
// b follows that of problem b - 1 without a gap, the workspaces ws_stride bytes apart.
__device__ __forceinline__ RouteArgs problem_args(const RouteArgs& a0, int b) {
  RouteArgs a = a0;
  a.loads_in = a0.loads_in + (size_t)b * a0.E;
  if (a0.st_mass) a.st_mass = a0.st_mass + (size_t)b * a0.T;
  if (a0.st_entropy) a.st_entropy = a0.st_entropy + (size_t)b * a0.T;
  if (a0.st_pool) a.st_pool = a0.st_pool + (size_t)b * a0.T;
  return a;
}
template <typename P>
__device__ __forceinline__ P* shifted(P* p, size_t bytes) {
  return reinterpret_cast<P*>(reinterpret_cast<char*>(p) + bytes);
}
__device__ __forceinline__ Workspace problem_workspace(const Workspace& w0, size_t bytes) {
  Workspace w;
  w.logits = shifted(w0.logits, bytes);
  w.rec_cstar = shifted(w0.rec_cstar, bytes);
  w.rec_ids = shifted(w0.rec_ids, bytes);
  w.rec_p = shifted(w0.rec_p, bytes);
  w.rec_Z = shifted(w0.rec_Z, bytes);
  w.rec_lane = shifted(w0.rec_lane, bytes);
  w.flexmask = shifted(w0.flexmask, bytes);
  w.tile_fixed_cnt = shifted(w0.tile_fixed_cnt, bytes);
  w.tile_mask = shifted(w0.tile_mask, bytes);
  w.tile_base = shifted(w0.tile_base, bytes);
  w.rec_cids = shifted(w0.rec_cids, bytes);
  w.rec_pref = shifted(w0.rec_pref, bytes);
  w.flex_list = shifted(w0.flex_list, bytes);
  w.flex_ord = shifted(w0.flex_ord, bytes);
  w.flex_tok_base = shifted(w0.flex_tok_base, bytes);
  w.flex_slot = shifted(w0.flex_slot, bytes);
  w.chain_bits = shifted(w0.chain_bits, bytes);
  w.chain_cum = shifted(w0.chain_cum, bytes);
  w.lin_copy = shifted(w0.lin_copy, bytes);
  w.pool = shifted(w0.pool, bytes);
  w.status = shifted(w0.status, bytes);
  w.seg = shifted(w0.seg, bytes);
  w.split_part = shifted(w0.split_part, bytes);
  return w;
}

constexpr int kStatusPhase = 0;      // 1: fixed prefix published, 2: chain finished, 3: nothing left for the tail kernel
constexpr int kPhaseAllDone = 3;
constexpr int kStatusFlexTiles = 1;  // number of tiles that hold flexible tokens
constexpr int kStatusError = 2;      // 0, or why the outputs of the call are incomplete (kError*)
constexpr int kErrorTimeout = 1;        // a bounded wait in the tail kernel ran out (LASER_STATUS_TIMEOUT)
constexpr int kErrorInconsistent = 2;   // a dispatch slot fell outside the table (LASER_STATUS_INCONSISTENT)
// Polls of one flag before a finishing wavefront gives up (a poll is a memory round trip
// plus a short sleep, about a microsecond): a floor for the chain workgroup's start-up
// plus an allowance per token of the call, far above the chain's cost per token.
constexpr long long kSpinFloor = 1ll << 22;
constexpr long long kSpinPerToken = 16;
constexpr int kStatusSweeps = 3;     // sweeps of the chain's window evaluation (diagnostic)

// Workspace::seg of a pipelined call.  Cleared by a small kernel before the gate kernel.
constexpr int kSegNext = 0;     // segments the chain has finished
constexpr int kSegFlexBase = 1; // number the next segment's first flexible token gets (a multiple of 32)
constexpr int kSegOrdBase = 2;  // tiles with flexible tokens in the finished segments
constexpr int kSegCarry = 4;    // [64] per expert: assignments in the finished segments
constexpr int kSegDone = 128;   // [ntiles] wavefronts of the tile's analysis workgroup that have written their records

inline int record_width(int c) { return c > kMaxC ? kWideC : kMaxC; }
size_t workspace_bytes(int T, int E, int cw);         // what laser_workspace_bytes reports
size_t workspace_needed_bytes(int T, int E, int cw);  // what a single problem cannot do without
Workspace carve_workspace(void* base, int T, int E, int cw);

inline int padded_experts(int E) { return E <= 8 ? 8 : E <= 16 ? 16 : E <= 32 ? 32 : 64; }

// A workgroup barrier at which only LDS traffic has to be settled: loads from memory that
// are in flight stay in flight across it (__syncthreads() waits for them as well).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Large dynamic LDS must be allowed per kernel and per device before the first launch.
// `done` is the kernel's own record of the devices it has been allowed on.
constexpr int kMaxDevices = 64;
struct LdsAttr {
  bool done[kMaxDevices] = {};
};
inline hipError_t allow_dynamic_lds(const void* fn, int bytes, LdsAttr& rec) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool known = dev >= 0 && dev < kMaxDevices;
  if (known && rec.done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && known) rec.done[dev] = true;
  return e;
}

// Analysis workgroups of the persistent gate kernel of pipelined calls: one per compute
// unit of the current device but the one the chain workgroup occupies (255 if the device
// cannot be asked).  Cached per device.
inline int pipeline_workgroups() {
  static int cached[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 255;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 2) n = 256;
    cached[dev] = n - 1;
  }
  return cached[dev];
}

// A launcher reports the status of its own launch: an error that an earlier HIP call of
// the caller left behind is cleared first, not mistaken for a failed launch.
inline void clear_stale_error() { (void)hipGetLastError(); }

// Launchers (enqueue only; return the HIP error of the launch).
// gate projection fused with the per-token analysis (logits_out may be NULL;
// logits_stride: floats from one problem's logits to the next)
hipError_t launch_gate_analyse_bf16(const void* hidden, const void* w, int H, const RouteArgs& a,
                                    const Workspace& ws, int32_t* expert_ids, float* weights,
                                    float* logits_out, size_t logits_stride, hipStream_t s);
// the same for a pipelined call (a.nseg > 0, one problem): clearing kernel + persistent kernel
hipError_t launch_gate_pipeline_bf16(const void* hidden, const void* w, int H, const RouteArgs& a,
                                     const Workspace& ws, int32_t* expert_ids, float* weights,
                                     float* logits_out, hipStream_t s);
// the same for a split call (a.split > 0, one problem)
hipError_t launch_gate_split_bf16(const void* hidden, const void* w, int H, const RouteArgs& a,
                                  const Workspace& ws, int32_t* expert_ids, float* weights,
                                  float* logits_out, hipStream_t s);
// the arrival counters of split calls on this workspace (device memory of the current device;
// NULL if none can be had: the call then runs without the split)
int32_t* split_counters_for(const void* workspace);
// (problem b of `nbatch`: hidden + b*T*H, w + b*E*H -> logits + b*logits_stride floats)
hipError_t launch_gate_f32(const float* hidden, const float* w, int T, int H, int E, int nbatch,
                           float* logits, size_t logits_stride, hipStream_t s);
// (logits_stride: floats from one problem's logits to the next)
hipError_t launch_analyse(const float* logits, size_t logits_stride, const RouteArgs& a, const Workspace& ws,
                          int32_t* expert_ids, float* weights, hipStream_t s);
// the whole per-token analysis from logits [T,E] by the general kernel: either trimming
// mode (sample: RANDOM; problem b draws with stream id rnd.stream + b), any record width ...
hipError_t launch_analyse_general(const float* logits, size_t logits_stride, const RouteArgs& a,
                                  const Workspace& ws, bool sample, const RandomArgs& rnd,
                                  int32_t* expert_ids, float* weights, hipStream_t s);
// ... or, behind the deterministic analysis run with pool sizes (c > k only), a second
// look at the tokens whose pool exceeds c: their records are rewritten for the sample
hipError_t launch_random_resample(const float* logits, size_t logits_stride, const RouteArgs& a,
                                  const Workspace& ws, const RandomArgs& rnd, hipStream_t s);
hipError_t launch_tail(const RouteArgs& a, const Workspace& ws, int32_t* loads_inout,
                       int32_t* expert_offsets, int32_t* expert_ids, float* weights,
                       int32_t* permutation, hipStream_t s);


// ---- host side shared by the C ABI files ------------------------------------------

// Events of the benchmark timer (laser_bench.h): three per timed call.
struct BenchTimer {
  hipEvent_t* ev;
  int capacity;  // calls
  int used;      // calls recorded
};

}  // namespace laser

struct laser_params;
namespace laser {
// The routing call behind laser_route, laser_route_batched and laser_route_stats
// (timer: NULL, or where laser_bench_route records its events).
int route_impl(const void* hidden, const void* w_gate, int32_t B, int32_t T, int32_t H, int32_t E,
               const laser_params* params, int32_t* loads_inout, int32_t* expert_ids, float* weights,
               int32_t* permutation, int32_t* expert_offsets, float* logits_out, float* topk_mass,
               float* entropy, int32_t* pool_size, void* workspace, size_t workspace_bytes_given,
               void* hip_stream, BenchTimer* timer);
}  // namespace laser
