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
#include "laser_internal.h"

namespace laser {

// ---------------------------------------------------------------- helpers ----

template <int CTRL>
__device__ __forceinline__ int dpp_int(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_float(float v) {
  return __int_as_float(dpp_int<CTRL>(__float_as_int(v)));
}
// quad_perm controls: lane j of every 4-lane group reads lane sel[j]
constexpr int kQuadXor1 = 1 | (0 << 2) | (3 << 4) | (2 << 6);
constexpr int kQuadXor2 = 2 | (3 << 2) | (0 << 4) | (1 << 6);
constexpr int kQuadBcast0 = 0;

// exp(x) for x in [-80, 0]: n = rint(x * log2 e); r = x - n ln2 with a two-part
// ln2 and fused multiply-adds; degree-7 Taylor polynomial of exp(r), Horner with
// fused multiply-adds, coefficients fl32(1/j!); scaling by 2^n through the
// exponent field.  exp_fixed(0) == 1.
__device__ __forceinline__ float exp_fixed(float x) {
  const float n = __builtin_rintf(x * 0x1.715476p+0f);
  float r = __builtin_fmaf(n, -0x1.62e4p-1f, x);
  r = __builtin_fmaf(n, -0x1.7f7d1cp-20f, r);
  float q = 0x1.a01a02p-13f;
  q = __builtin_fmaf(q, r, 0x1.6c16c2p-10f);
  q = __builtin_fmaf(q, r, 0x1.111112p-7f);
  q = __builtin_fmaf(q, r, 0x1.555556p-5f);
  q = __builtin_fmaf(q, r, 0x1.555556p-3f);
  q = __builtin_fmaf(q, r, 0.5f);
  q = __builtin_fmaf(q, r, 1.0f);
  q = __builtin_fmaf(q, r, 1.0f);
  return __int_as_float(__float_as_int(q) + ((int)n << 23));
}

__device__ __forceinline__ unsigned long long lanes_below(int i) {
  return (1ull << i) - 1ull;  // i in [0, 63]
}

// --------------------------------------------------------------- analyse -----
//
// 256 threads per tile of 64 tokens: 4 lanes per token, lane q of a token owns
// the experts e = 4*i + q (i < NE).  Strides >= 4 of the Z tree then stay inside
// a lane and the last two levels are quad exchanges.

constexpr int kNegInfBits = 0xff800000;

template <int NE>
__device__ __forceinline__ void extract_round(float (&zw)[NE], int q, float& win_v, int& win_e) {
  // local best: first maximum in index order
  float bv = zw[0];
  int bi = 0;
#pragma unroll
  for (int i = 1; i < NE; ++i) {
    const bool better = zw[i] > bv;
    bv = better ? zw[i] : bv;
    bi = better ? i : bi;
  }
  int be = 4 * bi + q;
  // best of the quad under (value desc, expert asc)
  {
    const float ov = dpp_float<kQuadXor1>(bv);
    const int oe = dpp_int<kQuadXor1>(be);
    const bool take = (ov > bv) || (ov == bv && oe < be);
    bv = take ? ov : bv;
    be = take ? oe : be;
  }
  {
    const float ov = dpp_float<kQuadXor2>(bv);
    const int oe = dpp_int<kQuadXor2>(be);
    const bool take = (ov > bv) || (ov == bv && oe < be);
    bv = take ? ov : bv;
    be = take ? oe : be;
  }
  win_v = bv;
  win_e = be;
  // the owner strikes the winner out
  const bool owner = (be & 3) == q;
  const int wi = be >> 2;
#pragma unroll
  for (int i = 0; i < NE; ++i)
    zw[i] = (owner && wi == i) ? __int_as_float(kNegInfBits) : zw[i];
}

template <int NE>
__device__ void analyse_tile(const float* __restrict__ lz, int zs, unsigned long long* mask64,
                             unsigned long long* flex_lds, int tile, const RouteArgs a,
                             const Workspace ws, int32_t* __restrict__ expert_ids,
                             float* __restrict__ weights) {
  const int tid = threadIdx.x;
  const int itok = tid >> 2;
  const int q = tid & 3;
  const int t = tile * kTile + itok;
  const bool live = t < a.T;
  const int k = a.k, c = a.c;

  if (tid < 64) mask64[tid] = 0ull;
  if (tid == 0) *flex_lds = 0ull;

  float z[NE], zw[NE];
#pragma unroll
  for (int i = 0; i < NE; ++i) {
    const int e = 4 * i + q;
    z[i] = (live && e < a.E) ? lz[itok * zs + e] : __int_as_float(kNegInfBits);
    zw[i] = z[i];
  }
  __syncthreads();  // masks zeroed before anyone ORs into them

  float top_v[kMaxC];
  int top_e[kMaxC];
#pragma unroll
  for (int j = 0; j < kMaxC; ++j) {
    top_v[j] = 0.0f;
    top_e[j] = 0;
  }
#pragma unroll
  for (int j = 0; j < kMaxC; ++j) {
    if (j < k) extract_round<NE>(zw, q, top_v[j], top_e[j]);
  }

  const float zmax = top_v[0];
  float p[NE];
  int npool = 0;
#pragma unroll
  for (int i = 0; i < NE; ++i) {
    const int e = 4 * i + q;
    const float d = z[i] - zmax;
    npool += (d >= a.tau_ln) ? 1 : 0;  // -inf padding never qualifies
    p[i] = (e < a.E) ? exp_fixed(d < -80.0f ? -80.0f : d) : 0.0f;
  }
  // Z: in-lane levels (expert stride 4*s), then quad levels (stride 2, stride 1)
#pragma unroll
  for (int s = NE / 2; s >= 1; s >>= 1)
#pragma unroll
    for (int i = 0; i < s; ++i) p[i] = p[i] + p[i + s];
  float zsum = p[0];
  {
    const float other = dpp_float<kQuadXor2>(zsum);  // lanes 0,1 receive lanes 2,3
    zsum = zsum + other;                              // valid in lanes 0,1
    const float other1 = dpp_float<kQuadXor1>(zsum);  // lane 0 receives lane 1
    zsum = zsum + other1;                             // valid in lane 0
    zsum = dpp_float<kQuadBcast0>(zsum);
  }
  npool += dpp_int<kQuadXor1>(npool);
  npool += dpp_int<kQuadXor2>(npool);

  float ptop[kMaxC];
#pragma unroll
  for (int j = 0; j < kMaxC; ++j) {
    ptop[j] = 0.0f;
    if (j < k) {
      const float d = top_v[j] - zmax;
      ptop[j] = exp_fixed(d < -80.0f ? -80.0f : d);
    }
  }
  float sk = ptop[0];
#pragma unroll
  for (int j = 1; j < kMaxC; ++j)
    if (j < k) sk = sk + ptop[j];

  const bool mass_ok = sk >= a.eps_high * zsum;
  const int m = npool > k ? npool : k;
  const int cstar = c < m ? c : m;
  const bool flex = live && !mass_ok && cstar > k;

  // the rest of the order statistics, only where some token of the wave needs them
  if (__builtin_amdgcn_ballot_w64(flex) != 0ull) {
#pragma unroll
    for (int j = 1; j < kMaxC; ++j) {
      if (j >= k && j < c) {
        extract_round<NE>(zw, q, top_v[j], top_e[j]);
        const float d = top_v[j] - zmax;
        ptop[j] = exp_fixed(d < -80.0f ? -80.0f : d);
      }
    }
  }

  if (live && !flex) {
    const float denom = a.renormalize ? sk : zsum;
#pragma unroll
    for (int j = 0; j < kMaxC; ++j) {
      if (j < k && (j & 3) == q) {
        expert_ids[(size_t)t * k + j] = top_e[j];
        weights[(size_t)t * k + j] = ptop[j] / denom;
        atomicOr(&mask64[top_e[j]], 1ull << itok);
      }
    }
  }
  if (flex && q == 0) atomicOr(flex_lds, 1ull << itok);
  if (live && q == 0) {
    ws.rec_cstar[t] = flex ? (uint8_t)cstar : (uint8_t)0;
    ws.rec_Z[t] = zsum;
  }
  __syncthreads();

  if (tid < 64)
    ws.tile_fixed_cnt[(size_t)tile * 64 + tid] = __builtin_popcountll(mask64[tid]);
  const unsigned long long fm = *flex_lds;
  if (tid == 0) ws.flexmask[tile] = fm;

  if (flex) {
    const int slot = tile * kTile + __builtin_popcountll(fm & lanes_below(itok));
    // ranks 4q..4q+3 of the ordered list go out through lane q
    unsigned idw = 0;
    float pv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int j = 0; j < kMaxC; ++j) {
      if ((j >> 2) == q) {
        idw |= (unsigned)top_e[j] << (8 * (j & 3));
        pv[j & 3] = ptop[j];
      }
    }
    reinterpret_cast<unsigned*>(ws.rec_ids)[(size_t)t * 4 + q] = idw;
    reinterpret_cast<float4*>(ws.rec_p)[(size_t)t * 4 + q] = make_float4(pv[0], pv[1], pv[2], pv[3]);
    // per owned expert: rank in the working set and the number of earlier fixed
    // tokens of this tile assigned to it
    uint16_t* row = ws.rec_lane + (size_t)slot * a.EP + q * NE;
    const unsigned long long below = lanes_below(itok);
#pragma unroll
    for (int i = 0; i < NE; ++i) {
      const int e = 4 * i + q;
      int rank = -1;
#pragma unroll
      for (int j = 0; j < kMaxC; ++j)
        if (j < cstar && top_e[j] == e) rank = j;
      const int fw = __builtin_popcountll(mask64[e] & below);
      row[i] = rank >= 0 ? (uint16_t)((fw << 4) | rank) : (uint16_t)0xFFFF;
    }
  }
}

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
  analyse_tile<NE>(lz, ZS, mask64, &flex_lds, tile, a, ws, expert_ids, weights);
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
// One workgroup.  Wave 0 owns the counters (lane e = expert e) and walks the
// tiles in order; waves 1..3 copy the next batch of records into LDS while it
// works, so that no load of the chain waits on memory.  For a flexible token the
// candidates' keys are (load << 4) + record, record = (fixed-prefix << 4 | rank):
// ascending load, ties by score rank.  An expert is chosen iff fewer than k
// candidate keys are smaller than its own.

constexpr int kChainBatch = 3;  // tiles per LDS batch (two batches fit 64 KiB of LDS)

struct ChainBatch {
  unsigned long long flexmask[kChainBatch];
  int fixed_cnt[kChainBatch][64];
  uint16_t rec[kChainBatch][kTile * kMaxE];
};

__device__ void chain_prefetch(ChainBatch* dst, int batch, const RouteArgs& a,
                               const Workspace& ws, int ptid, int pthreads) {
  for (int tl = 0; tl < kChainBatch; ++tl) {
    const int tile = batch * kChainBatch + tl;
    if (tile >= a.ntiles) break;
    const unsigned long long fm = ws.flexmask[tile];
    if (ptid == 0) dst->flexmask[tl] = fm;
    for (int e = ptid; e < 64; e += pthreads)
      dst->fixed_cnt[tl][e] = ws.tile_fixed_cnt[(size_t)tile * 64 + e];
    const int words = (__builtin_popcountll(fm) * a.EP) >> 1;  // EP is even
    const unsigned* src = reinterpret_cast<const unsigned*>(ws.rec_lane + (size_t)tile * kTile * a.EP);
    unsigned* d32 = reinterpret_cast<unsigned*>(dst->rec[tl]);
    for (int wd = ptid; wd < words; wd += pthreads) d32[wd] = src[wd];
  }
}

__global__ __launch_bounds__(256) void chain_kernel(const RouteArgs a, const Workspace ws,
                                                    int32_t* __restrict__ loads_inout,
                                                    int32_t* __restrict__ expert_offsets) {
  __shared__ ChainBatch buf[2];
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int nbatch = (a.ntiles + kChainBatch - 1) / kChainBatch;
  const int NE = a.EP >> 2;
  const int mypos = (lane & 3) * NE + (lane >> 2);  // where expert `lane` sits in a record row

  int lin = 0, lsum = 0;
  if (wave == 0 && lane < a.E) lin = loads_inout[lane];
  lsum = lin;

  if (nbatch > 0) chain_prefetch(&buf[0], 0, a, ws, threadIdx.x, 256);
  __syncthreads();

  for (int b = 0; b < nbatch; ++b) {
    if (wave != 0) {
      if (b + 1 < nbatch) chain_prefetch(&buf[(b + 1) & 1], b + 1, a, ws, threadIdx.x - 64, 192);
    } else {
      const ChainBatch* cur = &buf[b & 1];
      for (int tl = 0; tl < kChainBatch; ++tl) {
        const int tile = b * kChainBatch + tl;
        if (tile >= a.ntiles) break;
        ws.tile_base[(size_t)tile * 64 + lane] = lsum - lin;
        unsigned long long fm = cur->flexmask[tl];
        const int nflex = __builtin_popcountll(fm);
        for (int r = 0; r < nflex; ++r) {
          const unsigned rec = cur->rec[tl][r * a.EP + mypos];
          const bool cand = (rec != 0xFFFFu) && (lane < a.EP);
          const unsigned key = cand ? (((unsigned)lsum << 4) + rec) : 0xFFFFFFFFu;
          unsigned long long cm = __builtin_amdgcn_ballot_w64(cand);
          int smaller = 0;
          while (cm) {
            const int e = __builtin_ctzll(cm);
            cm &= cm - 1ull;
            const unsigned other = __builtin_amdgcn_readlane(key, e);
            smaller += (other < key) ? 1 : 0;
          }
          const bool chosen = cand && smaller < a.k;
          const unsigned long long chosen_mask = __builtin_amdgcn_ballot_w64(chosen);
          lsum += chosen ? 1 : 0;
          if (lane == 0) ws.chain_out[(size_t)tile * kTile + r] = chosen_mask;
        }
        lsum += cur->fixed_cnt[tl][lane];
      }
    }
    __syncthreads();
  }

  if (wave == 0) {
    if (lane < a.E) loads_inout[lane] = lsum;
    // exclusive prefix sums of the per-expert assignment counts
    const int cnt = lane < a.E ? lsum - lin : 0;
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
  hipLaunchKernelGGL(chain_kernel, dim3(1), dim3(256), 0, s, a, ws, loads_inout, expert_offsets);
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
    const unsigned long long chosen = ws.chain_out[slot];
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
