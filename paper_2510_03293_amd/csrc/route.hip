// Algorithm 1 of the paper (appendix "Pseudo Code"; Method: Expansion rule,
// Final assignment) applied to the tokens of a layer in token order, plus the
// dispatch tables.  The analysis runs either fused behind the gate projection or as
// the stand-alone kernel below; the tail kernel holds the chain and the finishing
// pass:
//
//   analyse  (parallel over tokens)  everything about a token that does not
//            depend on the load counters: scores, descending order statistics,
//            top-k mass test, pool size, working set.  A token whose decision
//            cannot depend on loads ("fixed": top-k mass reached, or working set
//            no larger than k) gets its final experts here.  The others
//            ("flexible") leave a record.
//   chain    (one wavefront, lane = expert)  walks the flexible tokens in token
//            order against the live counters; fixed tokens enter as per-tile
//            per-expert counts plus, inside a tile, a per-record prefix count.
//   finish   (parallel over tiles)  expands the chain's choices into expert ids
//            and weights and scatters the stable counting-sort permutation.
//
// Decision arithmetic is binary32 with a fixed operation order (this file is
// compiled with -ffp-contract=off; fused operations are written explicitly):
//   order        logit descending, equal logits by lower expert index
//   p_i          exp_fixed(max(z_i - z_max, -80))
//   Z            tree sum: pad to a power of two, add element i+s onto i for
//                s = P/2, ..., 1
//   S_k          left-to-right sum of the k largest p in order
//   top-k branch S_k >= fl(eps_high * Z)
//   pool member  z_i - z_max >= fl32(ln t_fix)
#include "analyse.h"
#include "laser_internal.h"
#include "tail.h"

namespace laser {

template <int NE, bool STATS>  // NE = padded experts / 8
__global__ __launch_bounds__(512) void analyse_kernel(const float* __restrict__ logits,
                                                      size_t logits_stride, const RouteArgs a0,
                                                      const Workspace ws0,
                                                      int32_t* __restrict__ expert_ids,
                                                      float* __restrict__ weights) {
  constexpr int ZS = 8 * NE + 8;
  __shared__ __align__(16) float lz[kTile * ZS];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  // blockIdx.y: the problem of a batched call
  const int prob = blockIdx.y;
  RouteArgs a = problem_args(a0, prob);
  const Workspace ws = problem_workspace(ws0, (size_t)prob * a0.ws_stride);
  if (STATS && a.pool_in_ws) a.st_pool = ws.pool;
  logits += (size_t)prob * logits_stride;
  expert_ids += (size_t)prob * a.T * a.k;
  weights += (size_t)prob * a.T * a.k;
  const int tile = blockIdx.x;
  const int E = a.E;
  const int rows = min(kTile, a.T - tile * kTile);
  const float* src = logits + (size_t)tile * kTile * E;
  // at most 8 elements per thread (64 tokens x 64 experts / 512); every load is issued
  // before the first use, so the tile costs one memory latency, not one per element
  constexpr int kPer = kTile * kMaxE / 512;
  float x[kPer];
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int idx = threadIdx.x + u * 512;
    x[u] = idx < rows * E ? src[idx] : 0.0f;
  }
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int idx = threadIdx.x + u * 512;
    if (idx < rows * E) {
      const int tok = idx / E;
      lz[tok * ZS + (idx - tok * E)] = x[u];
    }
  }
  __syncthreads();
  analyse_tile<NE, 1, STATS>(lz, ZS, mask64, &flex_lds, tile, a, ws, expert_ids, weights, nullptr);
}

hipError_t launch_analyse(const float* logits, size_t logits_stride, const RouteArgs& a, const Workspace& ws,
                          int32_t* expert_ids, float* weights, hipStream_t s) {
  if (a.ntiles == 0) return hipSuccess;
  const dim3 grid(a.ntiles, a.nbatch), block(512);
  const bool st = wants_stats(a);
  clear_stale_error();
#define LASER_LAUNCH_ANALYSE(NE_)                                                                  \
  if (st)                                                                                          \
    hipLaunchKernelGGL((analyse_kernel<NE_, true>), grid, block, 0, s, logits, logits_stride, a,   \
                       ws, expert_ids, weights);                                                   \
  else                                                                                             \
    hipLaunchKernelGGL((analyse_kernel<NE_, false>), grid, block, 0, s, logits, logits_stride, a,  \
                       ws, expert_ids, weights);
  switch (a.EP) {
    case 8: LASER_LAUNCH_ANALYSE(1) break;
    case 16: LASER_LAUNCH_ANALYSE(2) break;
    case 32: LASER_LAUNCH_ANALYSE(4) break;
    default: LASER_LAUNCH_ANALYSE(8) break;
  }
#undef LASER_LAUNCH_ANALYSE
  return hipGetLastError();
}

template <bool BATCH>  // blockIdx.y is the problem of a batched call (a kernel of its own: the
                       // longer prologue would delay the first loads of the single-problem kernel)
__global__ __launch_bounds__(kTailThreads) void tail_kernel(const RouteArgs a0, const Workspace ws0,
                                                            int32_t* __restrict__ loads_inout,
                                                            int32_t* __restrict__ expert_offsets,
                                                            int32_t* __restrict__ expert_ids,
                                                            float* __restrict__ weights,
                                                            int32_t* __restrict__ permutation) {
  extern __shared__ __align__(16) uint8_t tail_lds[];
  // (each problem has its own chain workgroup)
  const int prob = BATCH ? blockIdx.y : 0;
  const RouteArgs a = BATCH ? problem_args(a0, prob) : a0;
  const Workspace ws = BATCH ? problem_workspace(ws0, (size_t)prob * a0.ws_stride) : ws0;
  if (BATCH) {
    loads_inout += (size_t)prob * a.E;
    expert_offsets += (size_t)prob * (a.E + 1);
    expert_ids += (size_t)prob * a.T * a.k;
    weights += (size_t)prob * a.T * a.k;
    permutation += (size_t)prob * a.T * a.k;
  }
  tail_role(blockIdx.x, tail_lds, a, ws, loads_inout, expert_offsets, expert_ids, weights, permutation);
}

template <bool BATCH>
static hipError_t launch_tail_b(const RouteArgs& a, const Workspace& ws, int32_t* loads_inout,
                                int32_t* expert_offsets, int32_t* expert_ids, float* weights,
                                int32_t* permutation, hipStream_t s) {
  static LdsAttr allowed;
  const hipError_t e =
      allow_dynamic_lds(reinterpret_cast<const void*>(&tail_kernel<BATCH>), kChainLdsBytes, allowed);
  if (e != hipSuccess) return e;
  const int grid = 1 + (a.ntiles + kChainWaves - 1) / kChainWaves;
  clear_stale_error();
  hipLaunchKernelGGL(tail_kernel<BATCH>, dim3(grid, a.nbatch), dim3(kTailThreads), kChainLdsBytes, s, a, ws,
                     loads_inout, expert_offsets, expert_ids, weights, permutation);
  return hipGetLastError();
}

hipError_t launch_tail(const RouteArgs& a, const Workspace& ws, int32_t* loads_inout,
                       int32_t* expert_offsets, int32_t* expert_ids, float* weights,
                       int32_t* permutation, hipStream_t s) {
  if (a.nbatch > 1)
    return launch_tail_b<true>(a, ws, loads_inout, expert_offsets, expert_ids, weights, permutation, s);
  return launch_tail_b<false>(a, ws, loads_inout, expert_offsets, expert_ids, weights, permutation, s);
}

}  // namespace laser
