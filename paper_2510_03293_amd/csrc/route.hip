// Algorithm 1 of the paper (appendix "Pseudo Code"; Method: Expansion rule,
// Final assignment) applied to the tokens of a layer in token order, plus the
// dispatch tables.  Three kernels:
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

namespace laser {

template <int NE>
__global__ __launch_bounds__(256) void analyse_kernel(const float* __restrict__ logits,
                                                      const RouteArgs a, const Workspace ws,
                                                      int32_t* __restrict__ expert_ids,
                                                      float* __restrict__ weights) {
  constexpr int ZS = 4 * NE + 4;
  __shared__ float lz[kTile * ZS];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  const int tile = blockIdx.x;
  const int E = a.E;
  const int rows = min(kTile, a.T - tile * kTile);
  const float* src = logits + (size_t)tile * kTile * E;
  for (int idx = threadIdx.x; idx < rows * E; idx += 256) {
    const int tok = idx / E;
    lz[tok * ZS + (idx - tok * E)] = src[idx];
  }
  __syncthreads();
  analyse_tile<NE, 1>(lz, ZS, mask64, &flex_lds, tile, a, ws, expert_ids, weights, nullptr);
}

hipError_t launch_analyse(const float* logits, const RouteArgs& a, const Workspace& ws,
                          int32_t* expert_ids, float* weights, hipStream_t s) {
  if (a.ntiles == 0) return hipSuccess;
  const dim3 grid(a.ntiles), block(256);
  switch (a.EP) {
    case 8:
      hipLaunchKernelGGL(analyse_kernel<2>, grid, block, 0, s, logits, a, ws, expert_ids, weights);
      break;
    case 16:
      hipLaunchKernelGGL(analyse_kernel<4>, grid, block, 0, s, logits, a, ws, expert_ids, weights);
      break;
    case 32:
      hipLaunchKernelGGL(analyse_kernel<8>, grid, block, 0, s, logits, a, ws, expert_ids, weights);
      break;
    default:
      hipLaunchKernelGGL(analyse_kernel<16>, grid, block, 0, s, logits, a, ws, expert_ids, weights);
      break;
  }
  return hipGetLastError();
}

// ----------------------------------------------------------------- chain -----
//
// One workgroup of 16 wavefronts.
//   prefix  (all waves)  exclusive prefix over tiles of the fixed tokens' per-expert
//           counts -> tile_base; ordered list of the tiles that hold flexible tokens.
//   chain   (wave 0, lane e = expert e)  walks the flexible tiles in order.  The
//           counters a flexible token sees are loads_in + fixed prefix of its tile
//           + fixed tokens before it inside the tile (carried by its record) +
//           flexible choices so far.  Candidate key = (load << 4) + rank: ascending
//           load, ties by score rank.  An expert is chosen iff fewer than k
//           candidate keys are smaller than its own; the candidates' keys are
//           fetched with one lane read each (CP reads per token, CP = c rounded up
//           to 4, 8 or 16).  Waves 1..12 copy the next batch of records into LDS
//           meanwhile, so the chain never waits on memory.
//   fix-up  (all waves)  tiles without flexible tokens add the flexible choices
//           made before them to their tile_base.
//
// Output of the chain: for every flexible tile and expert, one bit per flexible
// token of the tile (bit r of word r/32: chosen for the tile's r-th flexible token).

constexpr int kChainWaves = 16;
constexpr int kChainThreads = kChainWaves * 64;
constexpr int kChainBatch = 6;  // flexible tiles per LDS batch

struct ChainBatch {
  int tile[kChainBatch];
  int nflex[kChainBatch];
  int base[kChainBatch][64];
  uint4 cids[kChainBatch][kTile];              // 16 candidate lanes per record
  uint16_t rec[kChainBatch][kTile * kMaxE];    // per record and expert: prefix<<4 | rank
};
constexpr int kChainLdsBytes = 2 * (int)sizeof(ChainBatch);
constexpr int kChainStageTiles = kChainLdsBytes / 64;  // tiles of byte counts that fit the LDS

__device__ void chain_prefetch(ChainBatch* dst, int batch, int nflex_tiles, const RouteArgs& a,
                               const Workspace& ws, int hwave, int lane) {
  // two helper waves per tile of the batch
  const int tl = hwave >> 1;
  const int part = hwave & 1;
  if (tl >= kChainBatch) return;
  const int f = batch * kChainBatch + tl;
  if (f >= nflex_tiles) return;
  const int tile = ws.flex_list[f];
  const int n = __builtin_popcountll(ws.flexmask[tile]);
  if (part == 0) {
    if (lane == 0) {
      dst->tile[tl] = tile;
      dst->nflex[tl] = n;
    }
    dst->base[tl][lane] = ws.tile_base[(size_t)tile * 64 + lane];
    if (lane < n) dst->cids[tl][lane] = reinterpret_cast<const uint4*>(ws.rec_cids)[(size_t)tile * kTile + lane];
  }
  const int words = (n * a.EP) >> 1;  // EP is even
  const unsigned* src = reinterpret_cast<const unsigned*>(ws.rec_lane + (size_t)tile * kTile * a.EP);
  unsigned* d32 = reinterpret_cast<unsigned*>(dst->rec[tl]);
  for (int wd = part * 64 + lane; wd < words; wd += 128) d32[wd] = src[wd];
}

// One flexible token: returns whether this lane's expert is chosen.
template <int CP>
__device__ __forceinline__ bool chain_step(unsigned key, bool cand, const uint4 ids, int k) {
  unsigned w[4];
  w[0] = __builtin_amdgcn_readfirstlane(ids.x);
  if (CP > 4) w[1] = __builtin_amdgcn_readfirstlane(ids.y);
  if (CP > 8) {
    w[2] = __builtin_amdgcn_readfirstlane(ids.z);
    w[3] = __builtin_amdgcn_readfirstlane(ids.w);
  }
  int smaller = 0;
#pragma unroll
  for (int j = 0; j < CP; ++j) {
    const int e = (w[j >> 2] >> (8 * (j & 3))) & 0xFF;
    const unsigned other = __builtin_amdgcn_readlane(key, e);
    smaller += (other < key) ? 1 : 0;
  }
  return cand && smaller < k;
}

template <int CP>
__device__ __forceinline__ void chain_walk(ChainBatch* buf, int nflex_tiles, const RouteArgs& a,
                                           const Workspace& ws, int wave, int lane, int lin,
                                           int& gflex) {
  const int nbatch = (nflex_tiles + kChainBatch - 1) / kChainBatch;
  const int NE = a.EP >> 2;
  const int mypos = (lane & 3) * NE + (lane >> 2);  // where expert `lane` sits in a record row
  const bool lane_ok = lane < a.EP;
  const int EP = a.EP;
  const int k = a.k;
  if (wave != 0) chain_prefetch(&buf[0], 0, nflex_tiles, a, ws, wave - 1, lane);
  __syncthreads();
  for (int b = 0; b < nbatch; ++b) {
    if (wave != 0) {
      if (b + 1 < nbatch) chain_prefetch(&buf[(b + 1) & 1], b + 1, nflex_tiles, a, ws, wave - 1, lane);
    } else {
      const ChainBatch* cur = &buf[b & 1];
      for (int tl = 0; tl < kChainBatch; ++tl) {
        const int f = b * kChainBatch + tl;
        if (f >= nflex_tiles) break;
        const int tile = __builtin_amdgcn_readfirstlane(cur->tile[tl]);
        const int n = __builtin_amdgcn_readfirstlane(cur->nflex[tl]);
        const int fb = cur->base[tl][lane];
        ws.tile_base[(size_t)tile * 64 + lane] = fb + gflex;
        int lsum = lin + fb + gflex;
        const uint16_t* recp = cur->rec[tl] + (lane_ok ? mypos : 0);
        const uint4* cidp = cur->cids[tl];
        unsigned rec_next = recp[0];
        uint4 ids_next = cidp[0];
        for (int r0 = 0; r0 < n; r0 += 32) {
          const int r1 = min(n, r0 + 32);
          unsigned hist = 0;
          for (int r = r0; r < r1; ++r) {
            const unsigned rec = rec_next;
            const uint4 ids = ids_next;
            if (r + 1 < n) {  // next record's LDS reads fly during this step
              rec_next = recp[(r + 1) * EP];
              ids_next = cidp[r + 1];
            }
            const bool cand = lane_ok && rec != 0xFFFFu;
            const unsigned key = cand ? (((unsigned)lsum << 4) + rec) : 0xFFFFFFFFu;
            const bool chosen = chain_step<CP>(key, cand, ids, k);
            lsum += chosen ? 1 : 0;
            hist |= (chosen ? 1u : 0u) << (r - r0);
          }
          ws.chain_out[((size_t)tile * 2 + (r0 >> 5)) * 64 + lane] = hist;
        }
        gflex = lsum - lin - fb;
        ws.gsnap[(size_t)f * 64 + lane] = gflex;
      }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(kChainThreads) void chain_kernel(const RouteArgs a, const Workspace ws,
                                                              int32_t* __restrict__ loads_inout,
                                                              int32_t* __restrict__ expert_offsets) {
  extern __shared__ __align__(16) uint8_t chain_lds[];
  ChainBatch* buf = reinterpret_cast<ChainBatch*>(chain_lds);
  __shared__ int wave_tot[kChainWaves][64];
  __shared__ int wave_flex[kChainWaves];
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int ntiles = a.ntiles;

  // ---- which tiles hold flexible tokens (groups of 64 tiles per ballot) ------
  const int groups = (ntiles + 63) >> 6;
  const int gper = (groups + kChainWaves - 1) / kChainWaves;
  const int ga = min(wave * gper, groups), gb = min(ga + gper, groups);
  int nfl = 0;
  for (int g = ga; g < gb; ++g) {
    const int tile = g * 64 + lane;
    const bool f = tile < ntiles && ws.flexmask[tile] != 0ull;
    nfl += __builtin_popcountll(__builtin_amdgcn_ballot_w64(f));
  }
  if (lane == 0) wave_flex[wave] = nfl;

  // ---- prefix over tiles of the fixed tokens' counts -------------------------
  // The byte counts are staged through LDS in super-batches with one wide load per
  // thread; wave w then scans a contiguous run of tiles for its lane's expert.
  int carry = 0;  // fixed assignments in earlier super-batches (lane's expert)
  uint8_t* stage = chain_lds;
  for (int sb0 = 0; sb0 < ntiles; sb0 += kChainStageTiles) {
    const int nt = min(kChainStageTiles, ntiles - sb0);
    const uint4* src = reinterpret_cast<const uint4*>(ws.tile_fixed_cnt + (size_t)sb0 * 64);
    for (int i = threadIdx.x; i < nt * 4; i += kChainThreads) reinterpret_cast<uint4*>(stage)[i] = src[i];
    __syncthreads();
    const int per_wave = (nt + kChainWaves - 1) / kChainWaves;
    const int ta = min(wave * per_wave, nt), tb = min(ta + per_wave, nt);
    int tot = 0;
    for (int tile = ta; tile < tb; ++tile) tot += stage[tile * 64 + lane];
    wave_tot[wave][lane] = tot;
    __syncthreads();
    int run = carry;
    for (int w = 0; w < kChainWaves; ++w) {
      const int v = wave_tot[w][lane];
      run += w < wave ? v : 0;
      carry += v;
    }
    for (int tile = ta; tile < tb; ++tile) {
      ws.tile_base[(size_t)(sb0 + tile) * 64 + lane] = run;
      run += stage[tile * 64 + lane];
    }
    __syncthreads();  // stage and wave_tot are reused by the next super-batch
  }
  const int total_fixed = carry;
  if (ntiles == 0) __syncthreads();  // wave_flex visible even when the loop above did not run

  int fbefore = 0, nflex_tiles = 0;
  for (int w = 0; w < kChainWaves; ++w) {
    const int fl = wave_flex[w];
    fbefore += w < wave ? fl : 0;
    nflex_tiles += fl;
  }
  for (int g = ga; g < gb; ++g) {
    const int tile = g * 64 + lane;
    const bool f = tile < ntiles && ws.flexmask[tile] != 0ull;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(f);
    const int ord = fbefore + __builtin_popcountll(bal & lanes_below(lane));
    if (tile < ntiles) ws.flex_ord[tile] = ord;
    if (f) ws.flex_list[ord] = tile;
    fbefore += __builtin_popcountll(bal);
  }
  __syncthreads();  // tile_base, flex_list, flex_ord visible to the whole workgroup

  int lin = 0;
  if (lane < a.E) lin = loads_inout[lane];
  int gflex = 0;  // flexible assignments so far (meaningful in wave 0)

  if (nflex_tiles > 0) {
    if (a.c <= 4)
      chain_walk<4>(buf, nflex_tiles, a, ws, wave, lane, lin, gflex);
    else if (a.c <= 8)
      chain_walk<8>(buf, nflex_tiles, a, ws, wave, lane, lin, gflex);
    else
      chain_walk<16>(buf, nflex_tiles, a, ws, wave, lane, lin, gflex);
    // tiles without flexible tokens: add the flexible choices made before them
    const long long total = (long long)ntiles * 64;
    for (long long idx = threadIdx.x; idx < total; idx += kChainThreads) {
      const int tile = (int)(idx >> 6);
      if (ws.flexmask[tile] == 0ull) {
        const int ord = ws.flex_ord[tile];
        if (ord > 0) ws.tile_base[idx] += ws.gsnap[(size_t)(ord - 1) * 64 + (idx & 63)];
      }
    }
  }

  if (wave == 0) {
    const int cnt = lane < a.E ? total_fixed + gflex : 0;
    if (lane < a.E) loads_inout[lane] = lin + cnt;
    // exclusive prefix sums of the per-expert assignment counts
    int incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane < a.E) expert_offsets[lane] = incl - cnt;
    if (lane == a.E - 1) expert_offsets[a.E] = incl;
  }
}

hipError_t launch_chain(const RouteArgs& a, const Workspace& ws, int32_t* loads_inout,
                        int32_t* expert_offsets, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&chain_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kChainLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(chain_kernel, dim3(1), dim3(kChainThreads), kChainLdsBytes, s, a, ws,
                     loads_inout, expert_offsets);
  return hipGetLastError();
}

// ---------------------------------------------------------------- finish -----
//
// One wavefront per tile, lane = token.  Flexible tokens get their experts (in
// score order) and weights from the chain's chosen-expert mask; then every
// assignment slot t*k+j is placed at
//   expert_offsets[e] + (assignments to e in earlier tiles) + (earlier tokens of
//   this tile assigned to e),
// which is the stable counting sort of the flat expert_ids array.

__global__ __launch_bounds__(64) void finish_kernel(const RouteArgs a, const Workspace ws,
                                                    const int32_t* __restrict__ expert_offsets,
                                                    int32_t* __restrict__ expert_ids,
                                                    float* __restrict__ weights,
                                                    int32_t* __restrict__ permutation) {
  __shared__ unsigned long long mask64[64];
  __shared__ uint8_t ids_lds[kTile][kMaxC];
  const int tile = blockIdx.x;
  const int lane = threadIdx.x;
  const int t = tile * kTile + lane;
  const bool live = t < a.T;
  const int k = a.k;
  mask64[lane] = 0ull;

  const int cstar = live ? ws.rec_cstar[t] : 0;
  if (cstar > 0) {
    const unsigned long long fm = ws.flexmask[tile];
    const int slot = tile * kTile + __builtin_popcountll(fm & lanes_below(lane));
    const int r = slot - tile * kTile;
    const unsigned* cw = ws.chain_out + ((size_t)tile * 2 + (r >> 5)) * 64;
    unsigned long long chosen = 0ull;
    for (int j = 0; j < cstar; ++j)
      chosen |= (unsigned long long)((cw[ws.rec_ids[(size_t)t * 16 + j]] >> (r & 31)) & 1u)
                << ws.rec_ids[(size_t)t * 16 + j];
    const uint8_t* ids = ws.rec_ids + (size_t)t * 16;
    const float* pv = ws.rec_p + (size_t)t * 16;
    float denom = 0.0f;
    if (a.renormalize) {
      bool first = true;
      for (int j = 0; j < cstar; ++j) {
        if ((chosen >> ids[j]) & 1ull) {
          denom = first ? pv[j] : denom + pv[j];
          first = false;
        }
      }
    } else {
      denom = ws.rec_Z[t];
    }
    int n = 0;
    for (int j = 0; j < cstar; ++j) {
      const int e = ids[j];
      if ((chosen >> e) & 1ull) {
        expert_ids[(size_t)t * k + n] = e;
        weights[(size_t)t * k + n] = pv[j] / denom;
        ids_lds[lane][n] = (uint8_t)e;
        ++n;
      }
    }
  } else if (live) {
    for (int j = 0; j < k; ++j) ids_lds[lane][j] = (uint8_t)expert_ids[(size_t)t * k + j];
  }
  __syncthreads();
  if (live)
    for (int j = 0; j < k; ++j) atomicOr(&mask64[ids_lds[lane][j]], 1ull << lane);
  __syncthreads();
  if (live) {
    const unsigned long long below = lanes_below(lane);
    for (int j = 0; j < k; ++j) {
      const int e = ids_lds[lane][j];
      const int pos = expert_offsets[e] + ws.tile_base[(size_t)tile * 64 + e] +
                      __builtin_popcountll(mask64[e] & below);
      permutation[pos] = t * k + j;
    }
  }
}

hipError_t launch_finish(const RouteArgs& a, const Workspace& ws, const int32_t* expert_offsets,
                         int32_t* expert_ids, float* weights, int32_t* permutation,
                         hipStream_t s) {
  if (a.ntiles == 0) return hipSuccess;
  hipLaunchKernelGGL(finish_kernel, dim3(a.ntiles), dim3(64), 0, s, a, ws, expert_offsets,
                     expert_ids, weights, permutation);
  return hipGetLastError();
}

}  // namespace laser
