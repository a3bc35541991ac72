// Per-token analysis of a tile of logits held in LDS: everything Algorithm 1 needs
// about a token that does not depend on the load counters.  Shared by the fused
// gate kernel and by the stand-alone kernel that starts from given logits.
//
// Decision arithmetic is binary32 with a fixed operation order (compile with
// -ffp-contract=off; fused operations are written explicitly):
//   order        logit descending, equal logits by lower expert index
//   p_i          exp_fixed(max(z_i - z_max, -80))
//   Z            tree sum: pad to a power of two, add element i+s onto i for
//                s = P/2, ..., 1
//   S_k          left-to-right sum of the k largest p in order
//   top-k branch S_k >= fl(eps_high * Z)
//   pool member  z_i - z_max >= fl32(ln t_fix)
#pragma once

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

// lz: NP partial logit tiles in LDS, [NP][kTile rows][zs floats]; a token's logit is
// the sum of its NP partials in the order ((p0 + p1) + p2) + p3.  mask64 (64 words)
// and flex_lds (1 word) are LDS scratch.  logits_out (global, may be NULL) receives
// the summed logits.  Must be called by all 256 threads of the workgroup.
template <int NE, int NP>
__device__ void analyse_tile(const float* __restrict__ lz, int zs, unsigned long long* mask64,
                             unsigned long long* flex_lds, int tile, const RouteArgs a,
                             const Workspace ws, int32_t* __restrict__ expert_ids,
                             float* __restrict__ weights, float* __restrict__ logits_out) {
  const int tid = threadIdx.x;
  const int itok = tid >> 2;
  const int q = tid & 3;
  const int t = tile * kTile + itok;
  const bool live = t < a.T;
  const int k = a.k, c = a.c;

  if (tid < 64) mask64[tid] = 0ull;
  if (tid == 0) *flex_lds = 0ull;
  // the tail kernel of this call polls these words; they are cleared here, one
  // kernel earlier on the same stream
  if (tile == 0 && tid < 4) ws.status[tid] = 0;

  float z[NE], zw[NE];
#pragma unroll
  for (int i = 0; i < NE; ++i) {
    const int e = 4 * i + q;
    float v = lz[itok * zs + e];
#pragma unroll
    for (int pt = 1; pt < NP; ++pt) v = v + lz[pt * kTile * zs + itok * zs + e];
    const bool real = live && e < a.E;
    if (logits_out != nullptr && real) logits_out[(size_t)t * a.E + e] = v;
    z[i] = real ? v : __int_as_float(kNegInfBits);
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
    ws.tile_fixed_cnt[(size_t)tile * 64 + tid] = (uint8_t)__builtin_popcountll(mask64[tid]);
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
    // the chain reads exactly CP candidate lanes per token: ranks beyond the working
    // set point at a lane that holds no candidate (its key compares as largest)
    int padlane = a.E;  // lanes E..63 never hold a candidate
    if (a.E == 64) {
      unsigned used = 0;
#pragma unroll
      for (int j = 0; j < kMaxC; ++j)
        if (j < cstar && top_e[j] < 32) used |= 1u << top_e[j];
      padlane = __builtin_ctz(~used);  // at most 16 of the 32 low experts are candidates
    }
    unsigned cidw = 0;
#pragma unroll
    for (int j = 0; j < kMaxC; ++j)
      if ((j >> 2) == q) cidw |= (unsigned)(j < cstar ? top_e[j] : padlane) << (8 * (j & 3));
    reinterpret_cast<unsigned*>(ws.rec_cids)[(size_t)slot * 4 + q] = cidw;
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

}  // namespace laser
