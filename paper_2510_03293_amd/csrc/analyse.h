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
// Logits must be finite and above -3.4028234e38 (the value that stands in for
// experts that do not exist).
#pragma once

#include "laser_internal.h"

namespace laser {

// ---------------------------------------------------------------- helpers ----

template <int CTRL>
__device__ __forceinline__ int dpp_int(int v) {
  // bound_ctrl: lanes whose source does not exist read 0 (no prior value to keep)
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
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

// A store of something the chain workgroup of a pipelined call reads while the kernel
// that writes it is still running (PUB): written through to where every compute unit of
// the device sees it, so that the writer's own "stores done" count covers it.  Otherwise
// a plain store.
template <bool PUB, typename P>
__device__ __forceinline__ void store_for_chain(P* p, P v) {
  if (PUB)
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    *p = v;
}

__device__ __forceinline__ unsigned long long lanes_below(int i) {
  return (1ull << i) - 1ull;  // i in [0, 63]
}

// --------------------------------------------------------------- analyse -----
//
// 512 threads per tile of 64 tokens: 8 lanes per token.  Lane q of a token owns NE =
// (padded E)/8 experts in runs of G = min(4, NE) consecutive ones (so that a run is
// one LDS read): run g, element r is expert g*(padded E)/NG + G*q + r, NG = NE/G runs
// (two only for 64 experts).  The Z tree then starts with one in-lane level (64
// experts), goes through three exchanges inside the 8-lane group and ends in-lane.
//
// Order statistics.  Each logit becomes a 64-bit key that sorts, as an IEEE double,
// exactly like (logit descending, expert ascending): the logit widened to double
// (exact; the low 29 mantissa bits are free) with 6 tie-break bits in the lowest
// mantissa bits -- 63 - e for non-negative logits, e for negative ones, because a
// larger mantissa makes a negative number smaller.  All keys of a token are
// distinct, so sorting needs nothing but double max/min: a sorting network inside
// the lane, then three bitonic merges across the group (partners 7-l, l^1, l^2)
// keep the CT best.  Every lane of the group ends with the same sorted list; expert
// and logit are read back from the key.

constexpr float kLowestLogit = -3.4028234663852886e38f;  // stands in for missing experts
constexpr double kPadKey = -1.0e300;                      // below every real key

__device__ __forceinline__ double make_key(float z, int e) {
  const float zc = z + 0.0f;  // -0 -> +0: equal logits must give equal high parts
  const int m = __float_as_int(zc) >> 31;  // 0 or -1
  const unsigned code = ((unsigned)(e ^ 63) ^ (unsigned)m) & 63u;
  return __longlong_as_double(__double_as_longlong((double)zc) | (long long)code);
}
__device__ __forceinline__ int key_expert(double key) {
  const long long b = __double_as_longlong(key);
  const int m = (int)(b >> 32) >> 31;
  return ~((int)b ^ m) & 63;
}
__device__ __forceinline__ float key_logit(double key) {
  return (float)__longlong_as_double(__double_as_longlong(key) & ~63LL);
}
// Keys are never NaN, so the bare instructions do; the library max/min would first
// pass every operand through a quieting operation of its own.
__device__ __forceinline__ double key_max(double a, double b) {
  double r;
  asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ double key_min(double a, double b) {
  double r;
  asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ void order_pair(double& hi, double& lo) {
  const double a = key_max(hi, lo), b = key_min(hi, lo);
  hi = a;
  lo = b;
}
template <int CTRL>
__device__ __forceinline__ double dpp_double(double v) {
  const long long b = __double_as_longlong(v);
  const unsigned lo = (unsigned)dpp_int<CTRL>((int)b);
  const unsigned hi = (unsigned)dpp_int<CTRL>((int)(b >> 32));
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Batcher's odd-even merge sort for N = 2^m inputs as a list of compare-exchanges.
template <int N>
struct SortNet {
  int a[N * N], b[N * N], n;
};
template <int N>
constexpr SortNet<N> make_sort_net() {
  SortNet<N> r{};
  r.n = 0;
  for (int p = 1; p < N; p *= 2)
    for (int k = p; k >= 1; k /= 2)
      for (int j = k % p; j + k < N; j += 2 * k)
        for (int i = 0; i < k && i + j + k < N; ++i)
          if ((i + j) / (2 * p) == (i + j + k) / (2 * p)) {
            r.a[r.n] = i + j;
            r.b[r.n] = i + j + k;
            ++r.n;
          }
  return r;
}
template <int N>
__device__ __forceinline__ void sort_descending(double (&K)[N]) {
  constexpr SortNet<N> net = make_sort_net<N>();
#pragma unroll
  for (int i = 0; i < net.n; ++i) order_pair(K[net.a[i]], K[net.b[i]]);
}
// L: sorted descending.  Afterwards: the CT largest of L and of the partner lane's L,
// sorted descending (the same list in both lanes).
template <int CT, int CTRL>
__device__ __forceinline__ void merge_with_partner(double (&L)[CT]) {
  double M[CT];
#pragma unroll
  for (int i = 0; i < CT; ++i) M[i] = key_max(L[i], dpp_double<CTRL>(L[CT - 1 - i]));
#pragma unroll
  for (int stride = CT / 2; stride >= 1; stride /= 2)
#pragma unroll
    for (int i = 0; i < CT; ++i)
      if ((i & stride) == 0) order_pair(M[i], M[i + stride]);
#pragma unroll
  for (int i = 0; i < CT; ++i) L[i] = M[i];
}

__device__ __forceinline__ float clamp_exp_arg(float d) { return d < -80.0f ? -80.0f : d; }

// DPP controls
constexpr int kRowShl4 = 0x104, kRowShr4 = 0x114, kRowShr1 = 0x111, kRowShl7 = 0x107;
constexpr int kRowHalfMirror = 0x141;

// value of lane `src` (0..7) of this lane's 8-lane group
__device__ __forceinline__ float group_read(float v, int src) {
  const int lane = threadIdx.x & 63;
  return __int_as_float(__builtin_amdgcn_ds_bpermute(((lane & ~7) | src) << 2, __float_as_int(v)));
}
// lane 0 of the group -> all 8 lanes
__device__ __forceinline__ float group_bcast0(float v, int q) {
  const float lo = dpp_float<kQuadBcast0>(v);
  const float hi = dpp_float<kRowShr4>(lo);
  return q < 4 ? lo : hi;
}
__device__ __forceinline__ float group_sum_f(float x, int q) {
  x += dpp_float<kQuadXor1>(x);
  x += dpp_float<kQuadXor2>(x);
  const float up = dpp_float<kRowShl4>(x), down = dpp_float<kRowShr4>(x);
  return x + (q < 4 ? up : down);
}
__device__ __forceinline__ int group_sum(int x, int q) {
  x += dpp_int<kQuadXor1>(x);
  x += dpp_int<kQuadXor2>(x);
  const int up = dpp_int<kRowShl4>(x), down = dpp_int<kRowShr4>(x);
  return x + (q < 4 ? up : down);
}

// lz: NP partial logit tiles in LDS, [NP][kTile rows][zs floats]; a token's logit is
// the sum of its NP partials in the order (((p0 + p1) + p2) + ...).  mask64 (64 words)
// and flex_lds (1 word) are LDS scratch.  logits_out (global, may be NULL) receives
// the summed logits.  CT (8 or 16) bounds the trimming size c.  STATS: also write the
// per-token statistics asked for in `a` (top-k mass, entropy, pool size; plain fp32,
// not part of any decision).  Must be called by all 512 threads of the workgroup.
template <int NE, int NP, int CT, bool STATS, bool PUB>
__device__ void analyse_tile_ct(const float* __restrict__ lz, int zs, unsigned long long* mask64,
                                unsigned long long* flex_lds, int tile, const RouteArgs a,
                                const Workspace ws, int32_t* __restrict__ expert_ids,
                                float* __restrict__ weights, float* __restrict__ logits_out) {
  constexpr int NS = CT / 8;  // ranks 8*s + q are handled by lane q ("slots")
  int tid = threadIdx.x;
  // (PUB: called from a loop over tiles.  Everything derived from the thread index is
  // then computed anew for every tile: held in registers across the loop it would crowd
  // out the loads that are in flight around this call)
  if (PUB) asm volatile("" : "+v"(tid));
  const int itok = tid >> 3;
  const int q = tid & 7;
  const int t = tile * kTile + itok;
  const bool live = t < a.T;
  const int k = a.k, c = a.c;

  if (tid < 64) mask64[tid] = 0ull;
  if (tid == 0) *flex_lds = 0ull;
  // the tail kernel of this call polls these words; they are cleared here, one
  // kernel earlier on the same stream
  // (PUB: a kernel before this one has done it, and copied the counters)
  if (!PUB && tile == 0 && tid < 4) ws.status[tid] = 0;
  // Tile 0 keeps a copy of the counters before token 0 for the tail kernel (which
  // overwrites them in place).  Loaded here, stored at the very end: the wait for the
  // load then costs nothing.
  const bool lin_copier = !PUB && tile == 0 && tid < 64;
  const int lin_before = (lin_copier && tid < a.E) ? a.loads_in[tid] : 0;

  constexpr int G = NE < 4 ? NE : 4;      // consecutive experts per run
  constexpr int NG = NE / G;              // runs per lane
  constexpr int kRunStride = 8 * NE / NG;  // experts between the starts of two runs
  typedef float run_t __attribute__((ext_vector_type(G)));
  auto owned = [&](int i) { return (i / G) * kRunStride + G * q + (i % G); };

  float z[NE];
  double K[NE];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const float* src = lz + itok * zs + g * kRunStride + G * q;
    float v[G];
    {
      const run_t first = *reinterpret_cast<const run_t*>(src);
#pragma unroll
      for (int r = 0; r < G; ++r) v[r] = G == 1 ? *src : first[r < G ? r : 0];
    }
#pragma unroll
    for (int pt = 1; pt < NP; ++pt) {
      const run_t more = *reinterpret_cast<const run_t*>(src + pt * kTile * zs);
#pragma unroll
      for (int r = 0; r < G; ++r) v[r] = v[r] + more[r < G ? r : 0];
    }
#pragma unroll
    for (int r = 0; r < G; ++r) {
      const int i = g * G + r;
      const int e = owned(i);
      const bool real = live && e < a.E;
      z[i] = real ? v[r] : kLowestLogit;
      K[i] = make_key(z[i], e);
    }
  }
  if (logits_out != nullptr) {  // (one uniform test instead of one per element)
#pragma unroll
    for (int i = 0; i < NE; ++i)
      if (live && owned(i) < a.E) logits_out[(size_t)t * a.E + owned(i)] = z[i];
  }
  // masks zeroed before anyone ORs into them  (PUB: the next tile's loads are in flight
  // around this call and must stay so; the barriers order LDS traffic only)
  if (PUB) lds_barrier(); else __syncthreads();

  // ---- the CT best of the token, sorted, in every lane of its group -----------
  sort_descending<NE>(K);
  double L[CT];
#pragma unroll
  for (int i = 0; i < CT; ++i) L[i] = i < NE ? K[i < NE ? i : 0] : kPadKey;
  merge_with_partner<CT, kRowHalfMirror>(L);  // {l, 7-l}
  merge_with_partner<CT, kQuadXor1>(L);       // + {l^1}: 4 lanes' experts
  merge_with_partner<CT, kQuadXor2>(L);       // + {l^2}: all 8

  const float zmax = key_logit(L[0]);
  // this lane's slots: rank 8*s + q
  int my_e[NS];
  float my_d[NS], my_p[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    // (the empty asm keeps the compiler from turning the selects into an indexed
    // access of L, which would move the whole list to scratch memory)
    double sel = L[8 * s];
#pragma unroll
    for (int r = 1; r < 8; ++r) {
      double alt = L[8 * s + r];
      asm volatile("" : "+v"(alt));
      sel = q == r ? alt : sel;
    }
    my_e[s] = key_expert(sel);
    my_d[s] = key_logit(sel) - zmax;
    my_p[s] = exp_fixed(clamp_exp_arg(my_d[s]));
  }

  // ---- softmax normaliser over all experts ------------------------------------
  float p[NE];
#pragma unroll
  for (int i = 0; i < NE; ++i) p[i] = (owned(i) < a.E) ? exp_fixed(clamp_exp_arg(z[i] - zmax)) : 0.0f;
  float plogp = 0.0f;  // this lane's part of sum_i p_i * d_i
  int above = 0;       // this lane's experts at or above the pool cut
  if (STATS) {
#pragma unroll
    for (int i = 0; i < NE; ++i) {
      const float di = z[i] - zmax;
      plogp = __builtin_fmaf(p[i], clamp_exp_arg(di), plogp);
      above += (owned(i) < a.E && di >= a.tau_ln) ? 1 : 0;
    }
  }
  // the tree, top level first: stride (padded E)/2 pairs the two runs of a lane; the
  // next three strides pair lane q with q+4, q+2, q+1; the rest is inside the run
  if (NG == 2) {
#pragma unroll
    for (int r = 0; r < G; ++r) p[r] = p[r] + p[G + r];
  }
#pragma unroll
  for (int r = 0; r < G; ++r) p[r] = p[r] + dpp_float<kRowShl4>(p[r]);   // valid in lanes 0..3
#pragma unroll
  for (int r = 0; r < G; ++r) p[r] = p[r] + dpp_float<kQuadXor2>(p[r]);  // valid in lanes 0,1
#pragma unroll
  for (int r = 0; r < G; ++r) p[r] = p[r] + dpp_float<kQuadXor1>(p[r]);  // valid in lane 0
#pragma unroll
  for (int s = G / 2; s >= 1; s >>= 1)
#pragma unroll
    for (int r = 0; r < s; ++r) p[r] = p[r] + p[r + s];
  const float zsum = group_bcast0(p[0], q);

  // ---- top-k mass: left-to-right sum in rank order ------------------------------
  // rank j lives in lane j%8, slot j/8; the running sum hops from lane to lane
  float run = my_p[0];
#pragma unroll
  for (int j = 1; j < CT; ++j) {
    if (j < k) {
      const float moved = (j & 7) != 0 ? dpp_float<kRowShr1>(run) : dpp_float<kRowShl7>(run);
      const float next = moved + my_p[j >> 3];
      run = q == (j & 7) ? next : run;
    }
  }
  const float sk = group_read(run, (k - 1) & 7);
  const bool mass_ok = sk >= a.eps_high * zsum;
  // the pool is a prefix of the order, so its size beyond k is the number of ranks in
  // [k, c) that pass the cut
  int extra = 0;
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int j = 8 * s + q;
    extra += (j >= k && j < c && my_d[s] >= a.tau_ln) ? 1 : 0;
  }
  extra = group_sum(extra, q);
  const int cstar = k + extra;
  const bool flex = live && !mass_ok && cstar > k;
  if (STATS) {
    // H = -sum s_i ln s_i with s_i = p_i / Z and ln s_i = d_i - ln Z
    const float s1 = group_sum_f(plogp, q);
    const int inpool = group_sum(above, q);
    if (live && q == 0) {
      if (a.st_mass) a.st_mass[t] = sk / zsum;
      if (a.st_entropy) a.st_entropy[t] = __builtin_logf(zsum) - s1 / zsum;
      if (a.st_pool) a.st_pool[t] = inpool > k ? inpool : k;
    }
  }

  // ---- tokens whose experts are final: outputs, per-expert masks ----------------
  if (live && !flex) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
      if (8 * s + q < k) atomicOr(&mask64[my_e[s]], 1ull << itok);
  }
  if (flex && q == 0) atomicOr(flex_lds, 1ull << itok);
  if (PUB) lds_barrier(); else __syncthreads();
  // (global stores only after the barrier: a barrier waits for the stores before it)
  if (live && !flex) {
    const float denom = a.renormalize ? sk : zsum;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int j = 8 * s + q;
      if (j < k) {
        expert_ids[(size_t)t * k + j] = my_e[s];
        weights[(size_t)t * k + j] = my_p[s] / denom;
      }
    }
  }
  if (live && q == 0) {
    ws.rec_cstar[t] = flex ? (uint8_t)cstar : (uint8_t)0;
    ws.rec_Z[t] = zsum;
  }

  if (tid < 64) {
    store_for_chain<PUB>(&ws.tile_fixed_cnt[(size_t)tile * 64 + tid], (uint8_t)__builtin_popcountll(mask64[tid]));
    ws.tile_mask[(size_t)tile * 64 + tid] = mask64[tid];
  }
  const unsigned long long fm = *flex_lds;
  if (tid == 0) store_for_chain<PUB>(&ws.flexmask[tile], fm);

  // ---- records of the flexible tokens (rare or chain-bound: not tuned) ----------
  if (__builtin_amdgcn_ballot_w64(flex) != 0ull) {
    int top_e[CT];
    float ptop[CT];
#pragma unroll
    for (int j = 0; j < CT; ++j) {
      top_e[j] = key_expert(L[j]);
      ptop[j] = group_read(my_p[j >> 3], j & 7);
    }
    if (flex) {
      const int slot = tile * kTile + __builtin_popcountll(fm & lanes_below(itok));
      if (q < 4) {
        // ranks 4q..4q+3 of the ordered list go out through lane q
        unsigned idw = 0, cidw = 0, prefw = 0;
        float pv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        const unsigned long long earlier = lanes_below(itok);
        // the chain reads exactly CP candidate lanes per token: ranks beyond the working
        // set point at a lane that holds no candidate (its key compares as largest)
        int padlane = a.E;  // lanes E..63 never hold a candidate
        if (a.E == 64) {
          unsigned used = 0;
#pragma unroll
          for (int j = 0; j < CT; ++j)
            if (j < cstar && top_e[j] < 32) used |= 1u << top_e[j];
          padlane = __builtin_ctz(~used);  // at most 16 of the 32 low experts are candidates
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          if ((j >> 2) == q) {
            const int ej = j < CT ? top_e[j < CT ? j : 0] : 0;
            idw |= (unsigned)ej << (8 * (j & 3));
            cidw |= (unsigned)(j < cstar ? ej : padlane) << (8 * (j & 3));
            pv[j & 3] = j < CT ? ptop[j < CT ? j : 0] : 0.0f;
            // fixed tokens of the tile before this one that were assigned to candidate j
            // (0xFF marks the ranks beyond the working set)
            const int fwj = j < cstar ? __builtin_popcountll(mask64[ej] & earlier) : 0xFF;
            prefw |= (unsigned)fwj << (8 * (j & 3));
          }
        }
        reinterpret_cast<unsigned*>(ws.rec_ids)[(size_t)t * 4 + q] = idw;
        reinterpret_cast<float4*>(ws.rec_p)[(size_t)t * 4 + q] = make_float4(pv[0], pv[1], pv[2], pv[3]);
        store_for_chain<PUB>(&reinterpret_cast<unsigned*>(ws.rec_cids)[(size_t)slot * 4 + q], cidw);
        store_for_chain<PUB>(&reinterpret_cast<unsigned*>(ws.rec_pref)[(size_t)slot * 4 + q], prefw);
      }
      // per owned expert: rank in the working set and the number of earlier fixed
      // tokens of this tile assigned to it; row in expert order
      uint16_t* row = ws.rec_lane + (size_t)slot * a.EP;
      const unsigned long long below = lanes_below(itok);
#pragma unroll
      for (int i = 0; i < NE; ++i) {
        const int e = owned(i);
        int rank = -1;
#pragma unroll
        for (int j = 0; j < CT; ++j)
          if (j < cstar && top_e[j] == e) rank = j;
        const int fw = __builtin_popcountll(mask64[e] & below);
        store_for_chain<PUB>(&row[e], rank >= 0 ? (uint16_t)((fw << 4) | rank) : (uint16_t)0xFFFF);
      }
    }
  }
  if (lin_copier) ws.lin_copy[tid] = lin_before;
}

// NE = padded experts / 8 (1, 2, 4 or 8).
template <int NE, int NP, bool STATS = false, bool PUB = false>
__device__ __forceinline__ void analyse_tile(const float* __restrict__ lz, int zs,
                                             unsigned long long* mask64, unsigned long long* flex_lds,
                                             int tile, const RouteArgs a, const Workspace ws,
                                             int32_t* __restrict__ expert_ids,
                                             float* __restrict__ weights,
                                             float* __restrict__ logits_out) {
  if (a.c <= 8)
    analyse_tile_ct<NE, NP, 8, STATS, PUB>(lz, zs, mask64, flex_lds, tile, a, ws, expert_ids, weights, logits_out);
  else
    analyse_tile_ct<NE, NP, 16, STATS, PUB>(lz, zs, mask64, flex_lds, tile, a, ws, expert_ids, weights, logits_out);
}

}  // namespace laser
