// The tail of a routing call: the load-ordered chain over the flexible tokens and the
// finishing pass that writes the dispatch tables (Algorithm 1 of the paper, appendix
// "Pseudo Code"; Method: Final assignment).  Device code only, shared by the tail kernel
// and by the fused kernel that runs a whole single-tile call in one launch.
#pragma once

#include "analyse.h"
#include "laser_internal.h"

namespace laser {

// ------------------------------------------------------------------ tail -----
//
// One kernel after the analysis: workgroup 0 is the chain, every other workgroup
// finishes 4 tiles (one wavefront each).
//
// Chain workgroup (4 wavefronts):
//   prefix  (all waves)  exclusive prefix over tiles of the fixed tokens' per-expert
//           counts -> tile_base; ordered list of the tiles that hold flexible tokens;
//           for every tile the number of flexible tokens before it.  Then flag 1 is
//           published: everything is final if no tile holds a flexible token.
//   chain   decides the flexible tokens in token order.  The counters a flexible token
//           sees are loads_in + fixed prefix of its tile + fixed tokens before it
//           inside the tile (carried by its record) + flexible choices so far.
//           Candidate key = (load << 4) + rank: ascending load, ties by score rank; the
//           k smallest keys win.  Two evaluations, same result:
//           - window (wave 0, lane = token): 64 consecutive flexible tokens per sweep,
//             see "window evaluation" below; used first when there are enough tokens;
//           - sequential (wave 0, lane = expert): an expert is chosen iff fewer than k
//             candidate keys are smaller than its own; the candidates' keys are fetched
//             with one lane read each (CP reads per token, CP = c rounded up to 4, 8 or
//             16).  Takes over where the window evaluation stops paying.
//           The other waves stage the records in LDS ahead of wave 0.
//   totals  loads and offsets, then flag 2.
//   Output of the chain, per expert: one bit per flexible token of the call in token
//   order (chain_bits, 32 per word) and the running count of chosen bits at every
//   32-token boundary (chain_cum).
//
// Finishing wavefront (lane = token of its tile): loads what does not depend on the
// chain, waits for flag 1 (and for flag 2 if any tile holds flexible tokens), then
// gives flexible tokens their experts (in score order) and weights from the chain's
// bits and places every assignment slot t*k+j at
//   expert_offsets[e] + (assignments to e in earlier tiles) + (earlier tokens of
//   this tile assigned to e),
// which is the stable counting sort of the flat expert_ids array.  The middle term is
// the fixed tokens' prefix (tile_base) plus the flexible choices of earlier tiles
// (chain_cum at the last boundary + the bits since).
//
// The waits are bounded polls of flags that the analysis kernel of the same call
// cleared; workgroup 0 has the lowest index, is dispatched first and never waits,
// so the polls end.  A poll that runs out sets ws.status[kStatusError] and the wave
// leaves without writing; the caller learns of it through laser_status().

constexpr int kChainWaves = 4;
constexpr int kTailThreads = kChainWaves * 64;
constexpr int kChainBatch = 3;  // flexible tiles per LDS batch
constexpr int kSelfPrefixTiles = 1024;  // up to here finishing workgroups sum the counts themselves
// (see "a handful of flexible tokens" below)
constexpr int kFastMaxTiles = 256;
constexpr int kFastTiles = 4;
constexpr int kFastTokens = 8;

// (not for wide calls: the shortcut reads the 16-candidate records)
__device__ __forceinline__ bool fast_path_applies(int ntiles, int nflex_tiles, int nflex_tok, int cw) {
  return cw == kMaxC && ntiles <= kFastMaxTiles && nflex_tiles > 0 && nflex_tiles <= kFastTiles &&
         nflex_tok <= kFastTokens;
}


struct ChainBatch {
  int tile[kChainBatch];
  int nflex[kChainBatch];
  int base[kChainBatch][64];
  uint4 cids[kChainBatch][kTile];              // 16 candidate lanes per record
  uint16_t rec[kChainBatch][kTile * kMaxE];    // per record and expert: prefix<<4 | rank
};
constexpr int kChainLdsBytes = 2 * (int)sizeof(ChainBatch);
constexpr int kChainStageTiles = kChainLdsBytes / 64;  // tiles of byte counts that fit the LDS

// Data published by the chain workgroup is read with agent-scope atomic loads: they
// see what the publisher wrote back before raising the flag, without the reader
// having to invalidate its whole L2 (the chain may run on another XCD).
__device__ __forceinline__ int load_published(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned load_published(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Flips this lane's bit of a 64-bit mask of lanes in LDS.  As a 32-bit operation on the
// word the bit is in: lanes 0..31 and 32..63 that flip bits of the same mask then work on
// different addresses, and an LDS atomic on one address is served lane after lane.
__device__ __forceinline__ void flip_lane_bit(unsigned long long* mask, int lane) {
  atomicXor(reinterpret_cast<unsigned*>(mask) + (lane >> 5), 1u << (lane & 31));
}

// Orders this wavefront's LDS traffic (another lane's write before this lane's read)
// without waiting for anything in flight to memory: a fence at workgroup scope would
// also wait for the chain's output stores.
__device__ __forceinline__ void lds_wave_fence() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// (every lane its own word)
__device__ __forceinline__ bool poll_word(const int* word, int want, long long limit) {
  for (long long it = 0; it < limit; ++it) {
    if (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= want) return true;
    __builtin_amdgcn_s_sleep(4);
  }
  return false;
}
__device__ __forceinline__ bool poll_flag(const int* flag, int want, long long limit) {
  for (long long it = 0; it < limit; ++it) {
    const int seen = __builtin_amdgcn_readfirstlane(
        __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (seen >= want) return true;
    __builtin_amdgcn_s_sleep(4);
  }
  return false;
}

__device__ __forceinline__ void chain_prefetch(ChainBatch* dst, int batch, int ft0, int nflex_tiles, const RouteArgs& a,
                               const Workspace& ws, int hwave, int lane) {
  for (int tl = hwave; tl < kChainBatch; tl += kChainWaves - 1) {
    const int f = ft0 + batch * kChainBatch + tl;
    if (f >= nflex_tiles) return;
    const int tile = ws.flex_list[f];
    const int n = __builtin_popcountll(ws.flexmask[tile]);
    if (lane == 0) {
      dst->tile[tl] = tile;
      dst->nflex[tl] = n;
    }
    dst->base[tl][lane] = ws.tile_base[(size_t)tile * 64 + lane];
    if (lane < n) dst->cids[tl][lane] = reinterpret_cast<const uint4*>(ws.rec_cids)[(size_t)tile * kTile + lane];
    const int words = (n * a.EP) >> 1;  // EP is even
    const unsigned* src = reinterpret_cast<const unsigned*>(ws.rec_lane + (size_t)tile * kTile * a.EP);
    unsigned* d32 = reinterpret_cast<unsigned*>(dst->rec[tl]);
    for (int wd = lane; wd < words; wd += 64) d32[wd] = src[wd];
  }
}

// cnt += number of the 4 lanes named by the bytes of `w` whose key is smaller than this
// lane's key.  Written in assembly because the order of the instructions is the
// point: on gfx950 a vector instruction that reads an SGPR written by the vector
// instruction just before it (lane read -> compare -> add-with-carry) needs two wait
// states each time; grouped as 4 lane reads, 4 compares, 4 adds every producer is at
// least three instructions ahead of its consumer and nothing waits.
__device__ __forceinline__ void count_smaller4(unsigned key, unsigned w, int& cnt) {
  unsigned e0, e1, e2, e3;
  unsigned long long c0, c1, c2, c3, cy;
  asm volatile(
      "s_nop 1\n\t"
      "s_bfe_u32 %[e0], %[w], 0x80000\n\t"
      "s_bfe_u32 %[e1], %[w], 0x80008\n\t"
      "s_bfe_u32 %[e2], %[w], 0x80010\n\t"
      "s_lshr_b32 %[e3], %[w], 24\n\t"
      "v_readlane_b32 %[e0], %[key], %[e0]\n\t"
      "v_readlane_b32 %[e1], %[key], %[e1]\n\t"
      "v_readlane_b32 %[e2], %[key], %[e2]\n\t"
      "v_readlane_b32 %[e3], %[key], %[e3]\n\t"
      "v_cmp_lt_u32_e64 %[c0], %[e0], %[key]\n\t"
      "v_cmp_lt_u32_e64 %[c1], %[e1], %[key]\n\t"
      "v_cmp_lt_u32_e64 %[c2], %[e2], %[key]\n\t"
      "v_cmp_lt_u32_e64 %[c3], %[e3], %[key]\n\t"
      "v_addc_co_u32_e64 %[cnt], %[cy], %[cnt], 0, %[c0]\n\t"
      "v_addc_co_u32_e64 %[cnt], %[cy], %[cnt], 0, %[c1]\n\t"
      "v_addc_co_u32_e64 %[cnt], %[cy], %[cnt], 0, %[c2]\n\t"
      "v_addc_co_u32_e64 %[cnt], %[cy], %[cnt], 0, %[c3]\n\t"
      "s_nop 1\n\t"
      : [cnt] "+v"(cnt), [e0] "=&s"(e0), [e1] "=&s"(e1), [e2] "=&s"(e2), [e3] "=&s"(e3),
        [c0] "=&s"(c0), [c1] "=&s"(c1), [c2] "=&s"(c2), [c3] "=&s"(c3), [cy] "=&s"(cy)
      : [key] "v"(key), [w] "s"(w)
      : "scc");  // (the scalar bit-field extracts and the shift set SCC)
}

// One flexible token: returns whether this lane's expert is chosen.
template <int CP>
__device__ __forceinline__ bool chain_step(unsigned key, bool cand, const uint4 ids, int k) {
  // (two counts: the second group's additions do not wait for the first group's)
  int smaller = 0, more = 0;
  count_smaller4(key, __builtin_amdgcn_readfirstlane(ids.x), smaller);
  if (CP > 4) count_smaller4(key, __builtin_amdgcn_readfirstlane(ids.y), more);
  if (CP > 8) {
    count_smaller4(key, __builtin_amdgcn_readfirstlane(ids.z), smaller);
    count_smaller4(key, __builtin_amdgcn_readfirstlane(ids.w), more);
  }
  return cand && smaller + more < k;
}

// Wave-wide minimum as a scalar: two exchanges inside the quads, the half-row and row
// mirrors (every lane of a 16-lane row then holds the row's minimum), one lane of each
// row read out.
__device__ __forceinline__ unsigned wave_min_u32(unsigned v) {
  constexpr int kRowMirror = 0x140;
  v = min(v, (unsigned)dpp_int<kQuadXor1>((int)v));
  v = min(v, (unsigned)dpp_int<kQuadXor2>((int)v));
  v = min(v, (unsigned)dpp_int<kRowHalfMirror>((int)v));
  v = min(v, (unsigned)dpp_int<kRowMirror>((int)v));
  const unsigned r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
  const unsigned r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
  return min(min(r0, r1), min(r2, r3));
}

// One flexible token of a wide call (up to 64 candidates), lane = expert: the k
// candidates with the smallest (load, rank), found in k rounds -- the least load among
// the remaining candidates, then the least rank among those that have it.  Any loads
// below 2^32 - 1; not tuned (the trimming sizes the paper evaluates are at most 10).
__device__ __forceinline__ bool chain_step_wide(unsigned load, unsigned rank, bool cand, int k) {
  bool remaining = cand, chosen = false;
  for (int r = 0; r < k; ++r) {
    const unsigned lmin = wave_min_u32(remaining ? load : 0xFFFFFFFFu);
    const bool tie = remaining && load == lmin;
    const unsigned rmin = wave_min_u32(tie ? rank : 0xFFFFFFFFu);
    const bool pick = tie && rank == rmin;
    chosen = chosen || pick;
    remaining = remaining && !pick;
  }
  return chosen;
}

// Sequential walk (wave 0, lane = expert) over the flexible tiles from flexible tile
// `ft0`, record `r_start` of that tile, which is flexible token `f0` of the call;
// `hist0` holds the bits of output word f0/32 that are decided already.  The output
// (chain_bits, chain_cum) is indexed by the flexible token's number within the call.
// CP = 0: a wide call (records of up to 64 candidates, per-expert rows only).
template <int CP>
__device__ __forceinline__ void chain_walk(ChainBatch* buf, int ft0, int r_start, int f0,
                                           unsigned hist0, int nflex_tiles, const RouteArgs& a, const Workspace& ws,
                                           int wave, int lane, int lin, int& gflex) {
  // wave-uniform values that arrive through LDS or memory: tell the compiler so, or the
  // loops below are compiled as divergent ones
  ft0 = __builtin_amdgcn_readfirstlane(ft0);
  r_start = __builtin_amdgcn_readfirstlane(r_start);
  nflex_tiles = __builtin_amdgcn_readfirstlane(nflex_tiles);
  const int nbatch = (nflex_tiles - ft0 + kChainBatch - 1) / kChainBatch;
  const int mypos = lane;  // a record row is in expert order
  const bool lane_ok = lane < a.EP;
  const int EP = a.EP;
  const int k = a.k;
  int f = __builtin_amdgcn_readfirstlane(f0);
  unsigned hist = hist0;  // bits of the current output word decided before this walk
  if (wave != 0) chain_prefetch(&buf[0], 0, ft0, nflex_tiles, a, ws, wave - 1, lane);
  __syncthreads();
  for (int b = 0; b < nbatch; ++b) {
    if (wave != 0) {
      if (b + 1 < nbatch) chain_prefetch(&buf[(b + 1) & 1], b + 1, ft0, nflex_tiles, a, ws, wave - 1, lane);
    } else {
      const ChainBatch* cur = &buf[b & 1];
      for (int tl = 0; tl < kChainBatch; ++tl) {
        const int ft = ft0 + b * kChainBatch + tl;
        if (ft >= nflex_tiles) break;
        const int n = __builtin_amdgcn_readfirstlane(cur->nflex[tl]);
        const int fb = cur->base[tl][lane];
        int lsum = lin + fb + gflex;
        int r = (ft == ft0) ? r_start : 0;
        if (r >= n) continue;
        const uint16_t* recp = cur->rec[tl] + (lane_ok ? mypos : 0);
        const uint4* cidp = cur->cids[tl];
        // the record of token r is in (rec_a, ids_a) at the top of every round; the next
        // record's LDS reads fly during a step.  Two tokens per round, so that the records
        // alternate between two sets of registers instead of being copied.
        unsigned rec_a = recp[r * EP], rec_b = 0;
        uint4 ids_a = cidp[r], ids_b = make_uint4(0, 0, 0, 0);
        auto step = [&](unsigned rec, const uint4 ids, int sh) {
          const bool cand = lane_ok && rec != 0xFFFFu;
          bool chosen;
          if constexpr (CP == 0) {
            chosen = chain_step_wide((unsigned)lsum + (rec >> 6), rec & 63u, cand, k);
          } else {
            const unsigned key = cand ? (((unsigned)lsum << 4) + rec) : 0xFFFFFFFFu;
            chosen = chain_step<CP>(key, cand, ids, k);
          }
          lsum += chosen ? 1 : 0;
          hist |= (chosen ? 1u : 0u) << sh;
        };
        while (r < n) {
          // up to the end of the tile or of the 32-token output word, whichever is first
          const int sh0 = f & 31;
          const int seg = min(n - r, 32 - sh0);
          const int end = sh0 + seg;
          int sh = sh0;
          for (; sh + 2 <= end; sh += 2, r += 2) {
            rec_b = recp[(r + 1) * EP];  // (r + 1 < n: two tokens are left)
            ids_b = cidp[r + 1];
            step(rec_a, ids_a, sh);
            if (r + 2 < n) {
              rec_a = recp[(r + 2) * EP];
              ids_a = cidp[r + 2];
            }
            step(rec_b, ids_b, sh + 1);
          }
          if (sh < end) {
            if (r + 1 < n) {
              rec_b = recp[(r + 1) * EP];
              ids_b = cidp[r + 1];
            }
            step(rec_a, ids_a, sh);
            rec_a = rec_b;
            ids_a = ids_b;
            ++r;
          }
          f += seg;
          if ((f & 31) == 0) {
            ws.chain_bits[(size_t)((f >> 5) - 1) * 64 + lane] = hist;
            ws.chain_cum[(size_t)(f >> 5) * 64 + lane] = lsum - lin - fb;
            hist = 0;
          }
        }
        gflex = lsum - lin - fb;
      }
    }
    __syncthreads();
  }
  if (wave == 0 && (f & 31) != 0) ws.chain_bits[(size_t)(f >> 5) * 64 + lane] = hist;
}

// ------------------------------------------------ window evaluation of the chain ----
//
// The sequential walk above costs one dependent step per flexible token.  Where
// consecutive flexible tokens rarely compete for the same experts at nearly equal
// loads, most of them can be decided side by side.  Wave 0 holds a window of 64
// consecutive flexible tokens, one per lane, each with a tentative choice.  A sweep
// re-decides every token of the window against
//     counters before the window  +  tentative choices of the window tokens before it,
// all lanes at once.  If q is the first token whose choice changed in a sweep, the new
// choices of tokens 0..q are final: each was computed from choices that did not change,
// hence from final ones (induction from the window head, whose inputs are all final).
// They leave the window, the next tokens enter with an empty tentative choice.  The
// result is the sequential one exactly, whatever the order of evaluation.  A sweep
// costs about as much as five sequential steps; if a run of sweeps retires fewer
// tokens than that, the workgroup goes back to the sequential walk for the rest.
//
// Lane = token side: candidates by rank (ids), their counters without any flexible
// choice (b: loads_in + fixed prefix of the tile + fixed tokens before it inside the
// tile), tentative choice as a bit mask over ranks.  Lane = expert side, in LDS: the
// window lanes that tentatively chose the expert (64-bit mask) and the final
// flexible choices so far (G).  Lane l holds the token f of the window with
// f % 64 == l, so nothing moves when the window advances.
//
// Waves 1 to 3 prepare the per-token data two segments ahead in an LDS ring; the
// workgroup meets at a barrier once per segment of 192 tokens.

constexpr int kSpecSeg = 192;                 // tokens per segment (64 per producer wave)
constexpr int kSpecRing = 3 * kSpecSeg;       // tokens in the LDS ring
constexpr unsigned kSpecInvalid = 1u << 27;   // counter of a rank beyond the working set
constexpr int kSpecMinTokens = 256;           // fewer flexible tokens: sequential walk
constexpr int kSpecCheckSweeps = 8;           // progress is judged over this many sweeps ...
// ... in which at least this many tokens must retire (measured: a sweep costs about
// 0.56 / 0.96 us for 4 / 8 candidates, a sequential step 0.12 / 0.17 us)
constexpr int kSpecGuessProgress = 26 * kSpecCheckSweeps;  // (without guesses at most 32 per sweep retire)
constexpr int spec_min_progress(int cp) { return cp <= 4 ? 40 : cp <= 8 ? 48 : 56; }

template <int CP>
struct SpecTok {
  uint4 ids;       // candidate experts by rank, one byte each
  unsigned b[CP];  // their counters without flexible choices
};
struct __align__(16) SpecExp {
  unsigned long long mask;  // window lanes that tentatively chose the expert
  int G;                    // final flexible choices of the expert so far
  int pad;
};
static_assert(kSpecRing * (int)sizeof(SpecTok<16>) <= kChainLdsBytes, "ring must fit the chain LDS");

template <int N>
__device__ __forceinline__ void sort_ascending_u32(unsigned (&K)[N]) {
  constexpr SortNet<N> net = make_sort_net<N>();
#pragma unroll
  for (int i = 0; i < net.n; ++i) {
    const unsigned lo = min(K[net.a[i]], K[net.b[i]]), hi = max(K[net.a[i]], K[net.b[i]]);
    K[net.a[i]] = lo;
    K[net.b[i]] = hi;
  }
}

// Bit mask over the CP key slots (slot = low 4 bits of a key) of the K smallest keys.
// With K known: a partial network that finds the min(K, CP - K) extreme keys by merging
// sorted pairs, quads, ... and keeping only that many per group; the keys are distinct.
template <int N, int M, bool LARGEST>
__device__ __forceinline__ void extreme_keys(const unsigned (&K)[N], unsigned (&out)[M]) {
  // groups of G keys, each reduced to its M' = min(G, M) extreme keys, sorted (most
  // extreme first); G doubles every round
  unsigned cur[N];
#pragma unroll
  for (int i = 0; i < N; ++i) cur[i] = K[i];
  auto better = [](unsigned x, unsigned y) { return LARGEST ? max(x, y) : min(x, y); };
  auto worse = [](unsigned x, unsigned y) { return LARGEST ? min(x, y) : max(x, y); };
  static_assert(M == 1 || M == 2, "at most two extreme keys");
  if (M == 1) {
#pragma unroll
    for (int g = 1; g < N; g *= 2)
#pragma unroll
      for (int i = 0; i + g < N; i += 2 * g) cur[i] = better(cur[i], cur[i + g]);
    out[0] = cur[0];
  } else {
    // pairs: (first, second)
#pragma unroll
    for (int i = 0; i < N; i += 2) {
      const unsigned a = better(cur[i], cur[i + 1]), b = worse(cur[i], cur[i + 1]);
      cur[i] = a;
      cur[i + 1] = b;
    }
#pragma unroll
    for (int g = 2; g < N; g *= 2)
#pragma unroll
      for (int i = 0; i + g < N; i += 2 * g) {
        const unsigned a0 = cur[i], b0 = cur[i + 1], a1 = cur[i + g], b1 = cur[i + g + 1];
        cur[i] = better(a0, a1);
        cur[i + 1] = better(worse(a0, a1), better(b0, b1));
      }
    out[0] = cur[0];
    out[1] = cur[1];
  }
}

template <int CP, int KK>
__device__ __forceinline__ unsigned smallest_k_slots(unsigned (&key)[CP], int k) {
  unsigned sel = 0;
  if (KK > 0 && KK <= 2 && KK < CP) {
    unsigned ext[KK > 0 && KK <= 2 ? KK : 1];
    extreme_keys<CP, (KK > 0 && KK <= 2 ? KK : 1), false>(key, ext);
#pragma unroll
    for (int i = 0; i < KK; ++i) sel |= 1u << (ext[i < 2 ? i : 0] & 15u);
  } else if (KK > 0 && CP - KK >= 1 && CP - KK <= 2) {
    constexpr int D = (KK > 0 && CP - KK >= 1 && CP - KK <= 2) ? CP - KK : 1;
    unsigned ext[D];
    extreme_keys<CP, D, true>(key, ext);
    sel = (1u << CP) - 1u;
#pragma unroll
    for (int i = 0; i < D; ++i) sel &= ~(1u << (ext[i] & 15u));
  } else {
    sort_ascending_u32<CP>(key);
#pragma unroll
    for (int i = 0; i < CP; ++i)
      if (i < k) sel |= 1u << (key[i] & 15u);
  }
  return sel;
}

__device__ __forceinline__ unsigned long long rotl64(unsigned long long x, int s) {  // s in [0, 63]
  return s ? (x << s) | (x >> (64 - s)) : x;
}
__device__ __forceinline__ unsigned long long rotr64(unsigned long long x, int s) {
  return s ? (x >> s) | (x << (64 - s)) : x;
}

// Producer: tokens seg*192 + half*64 + lane of the call -> ring (half = 0, 1, 2).
// Bit 31 of a counter marks the rank as part of the token's first tentative choice: the
// k least loaded candidates by the counters without any flexible choice.  Any first
// guess gives the same final result; a good one saves the sweep a token otherwise
// needs only to get a tentative choice, and lets the tokens behind it retire with it.
template <int CP, int KK, bool GUESS>
__device__ __forceinline__ void spec_fill(SpecTok<CP>* ring, int seg, int half, int nflex_tok, const Workspace& ws,
                          const int* lin_tab, int lane, int k) {
  const int f = seg * kSpecSeg + half * 64 + lane;
  if (f >= nflex_tok) return;
  const int slot = ws.flex_slot[f];
  const int tile = slot >> 6;
  const uint4 ids = reinterpret_cast<const uint4*>(ws.rec_cids)[slot];
  const uint4 pref = reinterpret_cast<const uint4*>(ws.rec_pref)[slot];
  const unsigned idw[4] = {ids.x, ids.y, ids.z, ids.w};
  const unsigned pfw[4] = {pref.x, pref.y, pref.z, pref.w};
  SpecTok<CP>* dst = &ring[f % kSpecRing];
  dst->ids = ids;
  int base[CP];
#pragma unroll
  for (int j = 0; j < CP; ++j) {
    const int e = (idw[j >> 2] >> (8 * (j & 3))) & 255;
    base[j] = ws.tile_base[(size_t)tile * 64 + e] + lin_tab[e];
  }
  unsigned bj[CP], key[CP];
#pragma unroll
  for (int j = 0; j < CP; ++j) {
    const unsigned pf = (pfw[j >> 2] >> (8 * (j & 3))) & 255u;
    bj[j] = pf == 0xFFu ? kSpecInvalid : (unsigned)base[j] + pf;
    key[j] = (bj[j] << 4) | (unsigned)j;
  }
  const unsigned guess = GUESS ? smallest_k_slots<CP, KK>(key, k) : 0u;
#pragma unroll
  for (int j = 0; j < CP; ++j) dst->b[j] = bj[j] | (((guess >> j) & 1u) << 31);
}

// Runs the window evaluation from flexible token 0.  All four waves call it.  Returns
// (to every wave) the number of flexible tokens decided; wave 0 leaves the flexible
// choices so far in `gflex` (lane = expert) and the bits of the unfinished output
// word in `hist`.  KK = k when known at compile time, else 0.
// LDS of the window evaluation beside the ring (one copy for all compiled variants).
struct SpecShared {
  SpecExp M[64];
  int lin_tab[64];
  int sh_done[2], sh_bail[2];  // by segment parity: written before, read after a barrier
};

template <int CP, int KK, bool GUESS>
__device__ __forceinline__ int spec_walk(uint8_t* lds, SpecShared& sp, int nflex_tok, const RouteArgs& a,
                         const Workspace& ws, int wave, int lane, int lin, int& gflex, unsigned& hist) {
  nflex_tok = __builtin_amdgcn_readfirstlane(nflex_tok);
  SpecTok<CP>* ring = reinterpret_cast<SpecTok<CP>*>(lds);
  SpecExp* M = sp.M;
  int* lin_tab = sp.lin_tab;
  int* sh_done = sp.sh_done;
  int* sh_bail = sp.sh_bail;
  const int k = KK > 0 ? KK : a.k;
  if (wave == 0) {
    M[lane].mask = 0ull;
    M[lane].G = 0;
    lin_tab[lane] = lin;
  }
  __syncthreads();
  const bool producer = wave != 0;
  if (producer) {
    spec_fill<CP, KK, GUESS>(ring, 0, wave - 1, nflex_tok, ws, lin_tab, lane, k);
    spec_fill<CP, KK, GUESS>(ring, 1, wave - 1, nflex_tok, ws, lin_tab, lane, k);
  }
  __syncthreads();

  // consumer state (wave 0)
  int ex[CP];       // candidate experts by rank
  unsigned b[CP];   // their counters without flexible choices
#pragma unroll
  for (int j = 0; j < CP; ++j) {
    ex[j] = 0;
    b[j] = kSpecInvalid;
  }
  unsigned sel = 0;
  int cur_f = -1;                  // token whose data this lane holds
  int ridx = lane - 64;            // its place in the ring (advances by 64 per token)
  int done = 0;                    // tokens decided (uniform)
  int G = 0;                       // lane = expert: final flexible choices
  unsigned long long pend = 0ull;  // lane = expert: decided bits not yet written, from token 32*w
  int pn = 0, w = 0, gflushed = 0;
  int sweeps = 0, done_mark = 0, total_sweeps = 0;
  bool bail = false;
  // First guesses pay where whole windows retire at once (tokens that rarely compete);
  // where a sweep ends at an early conflict anyway they only add their insertion.  They
  // are used while the last run of sweeps retired more than kSpecGuessProgress tokens.
  bool guess_on = GUESS;
  int decided = 0;
  const unsigned long long lb = lanes_below(lane);

  const int nep = (nflex_tok + kSpecSeg - 1) / kSpecSeg;
  for (int ep = 0; ep < nep; ++ep) {
    if (producer) {
      spec_fill<CP, KK, GUESS>(ring, ep + 2, wave - 1, nflex_tok, ws, lin_tab, lane, k);
    } else {
      const int avail = min(nflex_tok, (ep + 2) * kSpecSeg);
      const int target = min(nflex_tok, (ep + 1) * kSpecSeg);
      while (done < target && !bail) {
        const int head = done & 63;
        // this lane's token of the window [done, done + 64)
        const int f_lane = done + ((lane - head) & 63);
        const bool enters = f_lane < avail && cur_f != f_lane;
        if (enters) {
          ridx += 64;
          ridx = ridx >= kSpecRing ? ridx - kSpecRing : ridx;
          const SpecTok<CP>* src = &ring[ridx];
          const uint4 ids = src->ids;
          const unsigned idw[4] = {ids.x, ids.y, ids.z, ids.w};
          sel = 0;
#pragma unroll
          for (int j = 0; j < CP; ++j) {
            ex[j] = (idw[j >> 2] >> (8 * (j & 3))) & 255;
            b[j] = src->b[j];  // (bit 31, the guess, drops out of the key's shift below)
          }
          if (GUESS && guess_on) {
#pragma unroll
            for (int j = 0; j < CP; ++j) sel |= (b[j] >> 31) << j;  // the producer's first guess
          }
          cur_f = f_lane;
        }
        const bool valid = cur_f == f_lane;
        if (!valid) sel = 0;
        if (GUESS && guess_on && __builtin_amdgcn_ballot_w64(enters) != 0ull) {
          // the guesses join the masks before anybody counts (the lane's bit is clear:
          // the token that held the lane took its bits along when it retired)
          if (enters) {
#pragma unroll
            for (int j = 0; j < CP; ++j)
              if ((sel >> j) & 1u) flip_lane_bit(&M[ex[j]].mask, lane);
          }
          lds_wave_fence();
          __builtin_amdgcn_wave_barrier();
        }
        const unsigned long long hb = lanes_below(head);
        const unsigned long long earlier = lane >= head ? (lb & ~hb) : (~hb | lb);
        unsigned key[CP];
#pragma unroll
        for (int j = 0; j < CP; ++j) {
          const uint4 m = *reinterpret_cast<const uint4*>(&M[ex[j]]);  // mask lo, hi, G, -
          const unsigned cnt = (unsigned)(__builtin_popcount(m.x & (unsigned)earlier) +
                                          __builtin_popcount(m.y & (unsigned)(earlier >> 32)));
          key[j] = ((b[j] + m.z + cnt) << 4) | (unsigned)j;
        }
        unsigned newsel = smallest_k_slots<CP, KK>(key, k);
        newsel = valid ? newsel : 0u;
        const unsigned diff = sel ^ newsel;
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(diff != 0u);
        if (bal != 0ull) {
          // flip this lane's bit in the masks of the experts whose choice changed
#pragma unroll
          for (int j = 0; j < CP; ++j)
            if ((diff >> j) & 1u) flip_lane_bit(&M[ex[j]].mask, lane);
        }
        sel = newsel;
        // tokens up to the first changed one are final
        const unsigned long long rot = rotr64(bal, head);
        const int q = rot ? __builtin_ctzll(rot) : 64;
        // (without guesses more than 32 is rare: a token needs a sweep to get a choice)
        const int fin = min(min(q + 1, avail - done), GUESS ? 64 : 32);
        lds_wave_fence();
        __builtin_amdgcn_wave_barrier();
        {  // lane = expert
          unsigned long long mk = M[lane].mask;
          // tokens done + off .. + part - 1 (part <= 32: what the output takes at a time)
          auto retire = [&](int off, int part) {
            const int h2 = (head + off) & 63;
            const unsigned long long finmask = rotl64((1ull << part) - 1ull, h2);
            const unsigned long long fbits = mk & finmask;
            G += __builtin_popcountll(fbits);
            mk &= ~finmask;
            const unsigned ob = (unsigned)rotr64(fbits, h2);  // bit i: token done + off + i
            pend |= (unsigned long long)ob << pn;             // pn < 32 bits were held
            pn += part;
            if (pn >= 32) {
              const unsigned word = (unsigned)pend;
              gflushed += __builtin_popcount(word);
              ws.chain_bits[(size_t)w * 64 + lane] = word;
              ws.chain_cum[(size_t)(w + 1) * 64 + lane] = gflushed;
              pend >>= 32;
              pn -= 32;
              ++w;
            }
          };
          retire(0, min(fin, 32));
          if (GUESS && fin > 32) retire(32, fin - 32);
          M[lane].mask = mk;
          M[lane].G = G;
        }
        lds_wave_fence();
        __builtin_amdgcn_wave_barrier();
        done += fin;
        ++total_sweeps;
        if (++sweeps == kSpecCheckSweeps) {
          // give up only if both the last run of sweeps and the average so far are
          // below break-even: the switch is one-way
          if (done - done_mark < spec_min_progress(CP) &&
              done * kSpecCheckSweeps < spec_min_progress(CP) * total_sweeps &&
              nflex_tok - done > 2 * kSpecSeg)
            bail = true;
          if (GUESS) guess_on = done - done_mark >= kSpecGuessProgress;
          sweeps = 0;
          done_mark = done;
        }
      }
      if (lane == 0) {
        sh_done[ep & 1] = done;
        sh_bail[ep & 1] = bail ? 1 : 0;
      }
    }
    __syncthreads();
    decided = __builtin_amdgcn_readfirstlane(sh_done[ep & 1]);
    if (__builtin_amdgcn_readfirstlane(sh_bail[ep & 1])) break;
  }
  if (wave == 0) {
    gflex = G;
    hist = (unsigned)pend;  // the decided % 32 bits of the unfinished word
    if (decided == nflex_tok && pn > 0) ws.chain_bits[(size_t)w * 64 + lane] = (unsigned)pend;
    if (lane == 0) ws.status[kStatusSweeps] = total_sweeps;
  }
  __syncthreads();  // the ring is dead: the sequential walk may reuse the LDS
  return decided;
}

// ---- window of 128 tokens, two consumer wavefronts -----------------------------------
//
// Where tokens rarely compete (many experts behind each candidate: the variants with
// first guesses) a sweep usually retires most of its window, so a wider window decides
// more tokens for the same chain of dependent steps.  Waves 0 and 1 each hold 64 of the
// 128 window positions (position = flexible token number mod 128; wave = position / 64,
// lane = position mod 64) and evaluate them exactly as above; an expert's tentative
// choices are a 128-bit mask, of which each consumer wave writes only its own half.
// A sweep has two workgroup barriers that settle LDS traffic only: after the
// evaluation both waves publish which of their lanes changed, so that every wave finds
// the same first changed token; after the retirement (each consumer wave, lane =
// expert, retires its own half of the masks) the next evaluation may read.  Waves 2
// and 3 take part in the barriers and in between stage the per-token data into an LDS
// ring of 512 tokens: each stages 64 tokens per sweep, with the three dependent loads of
// a token (its slot, its record, the counters of its candidates) spread over three
// sweeps so that none of them is waited for.  Decided bits go to a small ring of output
// words in LDS; wave 3 writes out the words that are complete.
constexpr int kRing2 = 512;         // tokens in the LDS ring
constexpr int kSpecOutWords = 16;   // output staging ring, words of 32 tokens
constexpr int kSpecMeetPolls = 1 << 14;  // looks of one consumer wave for the other one, per sweep


struct __align__(16) SpecExp2 {
  unsigned long long mask[2];  // window positions 0..63 / 64..127 that tentatively chose the expert
  int G;                       // final flexible choices of the expert so far
  int pad[3];
};
struct SpecShared2 {
  SpecExp2 M[64];
  unsigned obits[kSpecOutWords][64];  // per expert: chosen bits of 32 flexible tokens, not yet written out
  int met[2];                         // consumer wave: sweeps in which its new tokens' guesses are in the masks
  unsigned long long bal[2][2];       // [sweep parity][consumer wave]: lanes whose choice changed
  int staged[2][2];                   // [sweep parity][producer wave]: tokens below this number are in the ring
  int pub_done[2], pub_flags[2];      // [sweep parity] written by wave 0 before the second barrier
  int lin_tab[64];
};
constexpr int kShared2Offset = kRing2 * (int)sizeof(SpecTok<16>);
static_assert(kShared2Offset + (int)sizeof(SpecShared2) <= kChainLdsBytes, "ring and state must fit the chain LDS");

// The positions before x of the 128-position ring, as two 64-bit halves.
__device__ __forceinline__ void below128(int x, unsigned long long& lo, unsigned long long& hi) {
  lo = x >= 64 ? ~0ull : (1ull << x) - 1ull;
  hi = x > 64 ? (x >= 128 ? ~0ull : (1ull << (x - 64)) - 1ull) : 0ull;
}

// Runs the window evaluation from flexible token 0 (see spec_walk for the contract).
template <int CP, int KK>
__device__ __forceinline__ int spec_walk2(uint8_t* lds, int nflex_tok, const RouteArgs& a, const Workspace& ws,
                                          int wave, int lane, int lin, int& gflex, unsigned& hist) {
  nflex_tok = __builtin_amdgcn_readfirstlane(nflex_tok);
  SpecTok<CP>* ring = reinterpret_cast<SpecTok<CP>*>(lds);
  SpecShared2& S = *reinterpret_cast<SpecShared2*>(lds + kShared2Offset);
  SpecExp2* M = S.M;
  const int k = KK > 0 ? KK : a.k;
  const int tid = threadIdx.x;
  if (tid < 64) {
    M[tid].mask[0] = M[tid].mask[1] = 0ull;
    M[tid].G = 0;
    S.lin_tab[tid] = lin;
  }
  for (int i = tid; i < kSpecOutWords * 64; i += kTailThreads) (&S.obits[0][0])[i] = 0u;
  if (tid < 4) (&S.bal[0][0])[tid] = 0ull;
  if (tid < 2) S.met[tid] = 0;
  if (tid < 4) (&S.staged[0][0])[tid] = 0;
  if (tid < 2) {
    S.pub_done[tid] = 0;
    S.pub_flags[tid] = 2;  // (bit 0: give up, bit 1: first guesses in use)
  }
  __syncthreads();

  const bool consumer = wave < 2;
  const int pw = wave & 1;  // consumer: which half of the window; producer: which half of a batch
  const unsigned long long lb = lanes_below(lane);

  // ---- consumer state ------------------------------------------------------------------
  int ex[CP];       // candidate experts by rank
  unsigned b[CP];   // their counters without flexible choices
#pragma unroll
  for (int j = 0; j < CP; ++j) {
    ex[j] = 0;
    b[j] = kSpecInvalid;
  }
  unsigned sel = 0;
  int cur_f = -1;      // token whose data this lane holds
  bool fresh = false;  // it came in after the last sweep: its first guess is not in the masks yet

  // ---- producer state: batch n of a producer is the tokens 128 n + 64 pw + lane ----------
  // in flight: the slot of batch nb + 2, slot and record of batch nb + 1, and for batch
  // nb the record (arrived) whose candidates' counters are fetched in the sweep it is staged
  int nb = 0;
  int slot0 = 0, slot1 = 0, slot2 = 0;
  uint4 ids1 = make_uint4(0, 0, 0, 0), pref1 = ids1, ids2 = ids1, pref2 = ids1;
  auto tok = [&](int n) { return 128 * n + 64 * pw + lane; };
  if (!consumer) {
    slot2 = tok(0) < nflex_tok ? ws.flex_slot[tok(0)] : 0;
    slot1 = tok(1) < nflex_tok ? ws.flex_slot[tok(1)] : 0;
    slot0 = tok(2) < nflex_tok ? ws.flex_slot[tok(2)] : 0;
    ids2 = reinterpret_cast<const uint4*>(ws.rec_cids)[slot2];
    pref2 = reinterpret_cast<const uint4*>(ws.rec_pref)[slot2];
    ids1 = reinterpret_cast<const uint4*>(ws.rec_cids)[slot1];
    pref1 = reinterpret_cast<const uint4*>(ws.rec_pref)[slot1];
  }

  int done = 0, avail = 0;  // tokens decided, tokens in the ring (both uniform, the same in every wave)
  int sweeps = 0, done_mark = 0, total_sweeps = 0;
  bool bail = false, guess_on = true;
  int wout = 0, gflushed = 0;  // wave 3, lane = expert: output words written, their bits so far

  for (;;) {
    const int par = total_sweeps & 1;
    const int head = done & 127;
    if (consumer) {
      // ---- this lane's token of the window [done, done + 128) -----------------------------
      // (its data was fetched between the barriers of the sweep before, see below)
      const int pos = 64 * pw + lane;
      const int f_lane = done + ((pos - head) & 127);
      const bool valid = cur_f == f_lane;
      if (!valid) sel = 0;
      const bool enters = fresh;  // a new token (sel: its first guess, if guesses are on)
      fresh = false;
      bool met = true;
      if (guess_on) {
        // The guesses join the masks before anybody counts (the lane's bit is clear: the
        // token that held the lane took its bits along when it retired).  "Anybody" is
        // both consumer waves: a new token in the other half of the window counts this
        // half's new guesses too.  The two waves meet here through a pair of sweep numbers
        // in LDS (the producers are busy staging and take no part).
        if (enters) {
#pragma unroll
          for (int j = 0; j < CP; ++j)
            if ((sel >> j) & 1u) flip_lane_bit(&M[ex[j]].mask[pw], lane);
        }
        lds_wave_fence();
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) S.met[pw] = total_sweeps + 1;
        met = false;
        for (int it = 0; it < kSpecMeetPolls && !met; ++it) {
          lds_wave_fence();
          // (read as LDS: through a plain volatile pointer the compiler emits a flat load,
          // which takes the long way through the vector memory pipeline)
          typedef __attribute__((address_space(3))) volatile int lds_volatile_int;
          met = __builtin_amdgcn_readfirstlane(*(lds_volatile_int*)&S.met[pw ^ 1]) > total_sweeps;
        }
      }
      // the window positions before this one: from the head up to pos, cyclically
      unsigned long long bh0, bh1;
      below128(head, bh0, bh1);
      const unsigned long long bp0 = pw ? ~0ull : lb, bp1 = pw ? lb : 0ull;
      const bool ge = pos >= head;
      const unsigned long long e0 = ge ? (bp0 & ~bh0) : (bp0 | ~bh0);
      const unsigned long long e1 = ge ? (bp1 & ~bh1) : (bp1 | ~bh1);
      unsigned key[CP];
#pragma unroll
      for (int j = 0; j < CP; ++j) {
        const uint4 m = *reinterpret_cast<const uint4*>(&M[ex[j]]);  // the two halves of the mask
        const unsigned g = (unsigned)M[ex[j]].G;
        const unsigned cnt = (unsigned)(__builtin_popcount(m.x & (unsigned)e0) + __builtin_popcount(m.y & (unsigned)(e0 >> 32)) +
                                        __builtin_popcount(m.z & (unsigned)e1) + __builtin_popcount(m.w & (unsigned)(e1 >> 32)));
        key[j] = ((b[j] + g + cnt) << 4) | (unsigned)j;
      }
      unsigned newsel = smallest_k_slots<CP, KK>(key, k);
      newsel = valid ? newsel : 0u;
      const unsigned diff = sel ^ newsel;
      unsigned long long bal = __builtin_amdgcn_ballot_w64(diff != 0u);
      if (bal != 0ull) {
        // flip this lane's bit in the masks of the experts whose choice changed
#pragma unroll
        for (int j = 0; j < CP; ++j)
          if ((diff >> j) & 1u) flip_lane_bit(&M[ex[j]].mask[pw], lane);
      }
      sel = newsel;
      // (should the other wave not have shown up in time, which does not happen while both
      // run: this sweep's new tokens may have missed guesses, so none of them is final yet
      // but the first -- it counts as changed)
      if (!met) bal |= __builtin_amdgcn_ballot_w64(enters);
      if (lane == 0) S.bal[par][pw] = bal;
    } else {
      // ---- producer: stage batch nb if the ring has room for it ----------------------------
      // (the ring holds the tokens [done, done + kRing2); `done` is at most one sweep old)
      if (128 * nb + 128 <= done + kRing2 && 128 * nb < nflex_tok) {
        const int f = tok(nb);
        const bool live = f < nflex_tok;
        const unsigned idw[4] = {ids2.x, ids2.y, ids2.z, ids2.w};
        const unsigned pfw[4] = {pref2.x, pref2.y, pref2.z, pref2.w};
        const int tile = slot2 >> 6;
        int base[CP];
#pragma unroll
        for (int j = 0; j < CP; ++j) {
          const int e = (idw[j >> 2] >> (8 * (j & 3))) & 255;
          base[j] = ws.tile_base[(size_t)tile * 64 + e] + S.lin_tab[e];
        }
        // the loads of the batches behind it: asked for now, used one and two sweeps on
        const uint4 ids_n = reinterpret_cast<const uint4*>(ws.rec_cids)[slot0];
        const uint4 pref_n = reinterpret_cast<const uint4*>(ws.rec_pref)[slot0];
        const int slot_n = tok(nb + 3) < nflex_tok ? ws.flex_slot[tok(nb + 3)] : 0;
        unsigned bj[CP], key[CP];
#pragma unroll
        for (int j = 0; j < CP; ++j) {
          const unsigned pf = (pfw[j >> 2] >> (8 * (j & 3))) & 255u;
          const int e = (idw[j >> 2] >> (8 * (j & 3))) & 255;
          bj[j] = pf == 0xFFu ? kSpecInvalid : (unsigned)base[j] + pf;
          // (the guess also counts the flexible choices that are final by now: a few
          // hundred tokens stale when this token enters the window, better than none)
          key[j] = ((bj[j] + (unsigned)M[e].G) << 4) | (unsigned)j;
        }
        const unsigned guess = smallest_k_slots<CP, KK>(key, k);
        if (live) {
          SpecTok<CP>* dst = &ring[f & (kRing2 - 1)];
          dst->ids = ids2;
#pragma unroll
          for (int j = 0; j < CP; ++j) dst->b[j] = bj[j] | (((guess >> j) & 1u) << 31);
        }
        slot2 = slot1;
        ids2 = ids1;
        pref2 = pref1;
        slot1 = slot0;
        ids1 = ids_n;
        pref1 = pref_n;
        slot0 = slot_n;
        ++nb;
      }
      // (by sweep parity: a producer that is already in the next sweep must not change what
      // a consumer still reads after the second barrier of this one)
      if (lane == 0) S.staged[par][pw] = 128 * nb;
    }
    lds_barrier();

    // ---- tokens up to the first changed one are final (every wave works it out) ------------
    int fin;
    {
      unsigned long long c0 = S.bal[par][0], c1 = S.bal[par][1];
      c0 = ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned)(c0 >> 32)) << 32) |
           (unsigned)__builtin_amdgcn_readfirstlane((unsigned)c0);
      c1 = ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned)(c1 >> 32)) << 32) |
           (unsigned)__builtin_amdgcn_readfirstlane((unsigned)c1);
      if (head >= 64) {
        const unsigned long long t = c0;
        c0 = c1;
        c1 = t;
      }
      const int sh = head & 63;
      const unsigned long long r0 = sh ? (c0 >> sh) | (c1 << (64 - sh)) : c0;
      const unsigned long long r1 = sh ? (c1 >> sh) | (c0 << (64 - sh)) : c1;
      const int q = r0 ? __builtin_ctzll(r0) : r1 ? 64 + __builtin_ctzll(r1) : 128;
      fin = min(min(q + 1, 128), avail - done);
    }
    if (!consumer) {
      // ---- the producers retire them: lane = expert, wave 2 + pw the half pw of the window
      // positions head .. head + fin - 1 (the consumers fetch their next tokens meanwhile)
      if (fin > 0) {
        unsigned long long lo0, hi0, lo1, hi1;
        below128(head, lo0, hi0);
        const int end = head + fin;  // (up to 255: the range may wrap)
        below128(end > 128 ? 128 : end, lo1, hi1);
        unsigned long long ret0 = lo1 & ~lo0, ret1 = hi1 & ~hi0;  // head .. min(end, 128) - 1
        if (end > 128) {
          unsigned long long wl, wh;
          below128(end - 128, wl, wh);
          ret0 |= wl;
          ret1 |= wh;
        }
        const unsigned long long mine = pw ? ret1 : ret0;
        const unsigned long long mk = M[lane].mask[pw];
        const unsigned long long fb = mk & mine;
        // (unconditional: lanes without retiring bits add nothing)
        atomicAdd(&M[lane].G, __builtin_popcountll(fb));
        M[lane].mask[pw] = mk & ~mine;
        // a quarter of the mask (32 positions) is bit-aligned with the output word of its
        // tokens; only the quarter of the head can hold tokens of two words (the positions
        // below the head belong to tokens four words on)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int qi = 2 * pw + h;              // quarter of the ring
          const unsigned qb = (unsigned)(fb >> (32 * h));
          const int cut = (head >> 5) == qi ? (head & 31) : 0;
          const int first = (done + ((32 * qi + cut - head) & 127)) >> 5;  // word of the positions >= cut
          const unsigned below_cut = (1u << cut) - 1u;
          atomicOr(&S.obits[first & (kSpecOutWords - 1)][lane], qb & ~below_cut);
          if (cut != 0) atomicOr(&S.obits[(first + 4) & (kSpecOutWords - 1)][lane], qb & below_cut);
        }
      }
    } else {
      // ---- the consumers fetch the tokens that take the freed positions --------------------
      // (only their data: the masks belong to the producers until the barrier below; the
      // first guesses join them at the start of the next sweep)
      {
        const int d2 = done + fin;
        // (the switch for the first guesses, as wave 0 works it out for everybody below)
        const bool g2 = sweeps + 1 == kSpecCheckSweeps ? d2 - done_mark >= kSpecGuessProgress : guess_on;
        const int avail2 = min(nflex_tok, min(__builtin_amdgcn_readfirstlane(S.staged[par][0]),
                                              __builtin_amdgcn_readfirstlane(S.staged[par][1])));
        const int pos = 64 * pw + lane;
        const int f2 = d2 + ((pos - (d2 & 127)) & 127);
        if (f2 < avail2 && cur_f != f2) {
          const SpecTok<CP>* src = &ring[f2 & (kRing2 - 1)];
          const uint4 ids = src->ids;
          const unsigned idw[4] = {ids.x, ids.y, ids.z, ids.w};
          sel = 0;
#pragma unroll
          for (int j = 0; j < CP; ++j) {
            ex[j] = (idw[j >> 2] >> (8 * (j & 3))) & 255;
            b[j] = src->b[j];  // (bit 31, the guess, drops out of the key's shift)
          }
          if (g2) {
#pragma unroll
            for (int j = 0; j < CP; ++j) sel |= (b[j] >> 31) << j;  // the producer's first guess
          }
          cur_f = f2;
          fresh = true;
        }
      }
      if (wave == 0) {
        int d = done + fin;
        bool gv = bail, gg = guess_on;
        int sw = sweeps + 1, dm = done_mark;
        if (sw == kSpecCheckSweeps) {
          // give up only if both the last run of sweeps and the average so far are
          // below break-even: the switch is one-way
          if (d - dm < spec_min_progress(CP) && d * kSpecCheckSweeps < spec_min_progress(CP) * (total_sweeps + 1) &&
              nflex_tok - d > 2 * kSpecSeg && avail - done >= 128)
            gv = true;
          gg = d - dm >= kSpecGuessProgress;
        }
        if (lane == 0) {
          S.pub_done[par] = d;
          S.pub_flags[par] = (gv ? 1 : 0) | (gg ? 2 : 0);
        }
      }
    }
    lds_barrier();

    // ---- every wave takes over the books ------------------------------------------------
    done = __builtin_amdgcn_readfirstlane(S.pub_done[par]);
    const int flags = __builtin_amdgcn_readfirstlane(S.pub_flags[par]);
    bail = (flags & 1) != 0;
    avail = min(nflex_tok, min(__builtin_amdgcn_readfirstlane(S.staged[par][0]),
                               __builtin_amdgcn_readfirstlane(S.staged[par][1])));
    ++total_sweeps;
    if (++sweeps == kSpecCheckSweeps) {
      guess_on = (flags & 2) != 0;
      sweeps = 0;
      done_mark = done;
    }
    // ---- output words that are complete (wave 3, lane = expert) ---------------------------
    if (wave == kChainWaves - 1) {
      while (32 * (wout + 1) <= done) {
        unsigned* slot = &S.obits[wout & (kSpecOutWords - 1)][lane];
        const unsigned word = *slot;
        *slot = 0u;
        gflushed += __builtin_popcount(word);
        ws.chain_bits[(size_t)wout * 64 + lane] = word;
        ws.chain_cum[(size_t)(wout + 1) * 64 + lane] = gflushed;
        ++wout;
      }
    }
    // (every sweep with tokens in the ring retires at least one, and the ring refills
    // within two sweeps; the cap only keeps a mistake from turning into an endless loop:
    // the sequential walk then takes over, and the result is still exact)
    if (total_sweeps > nflex_tok + (nflex_tok >> 5) + 64) bail = true;
    if (done >= nflex_tok || bail) break;
  }
  const int decided = done;
  if (wave == 0) {
    gflex = M[lane].G;
    hist = S.obits[(decided >> 5) & (kSpecOutWords - 1)][lane];  // the decided % 32 bits of the unfinished word
    if (decided == nflex_tok && (decided & 31) != 0) ws.chain_bits[(size_t)(decided >> 5) * 64 + lane] = hist;
    if (lane == 0) ws.status[kStatusSweeps] = total_sweeps;
  }
  __syncthreads();  // the ring is dead: the sequential walk may reuse the LDS
  return decided;
}

// One segment of a pipelined call, as chain_workgroup sees it: `a` and `ws` are then the
// segment's own view (tile 0 = the segment's first tile, flexible token 0 = its first
// flexible token), and what the earlier segments did comes in through here.
struct ChainSeg {
  bool on;        // false: the whole call in one go (everything below unused)
  int carry0;     // lane = expert: assignments in the earlier segments
  int fbase;      // number of the segment's first flexible token in the call's numbering
  int* out;       // LDS, 66 words: [lane] assignments up to the segment's end, [64] its tiles
                  // with flexible tokens, [65] its flexible tokens
};

__device__ __forceinline__ void chain_workgroup(uint8_t* lds, const RouteArgs& a, const Workspace& ws,
                                int32_t* __restrict__ loads_inout,
                                int32_t* __restrict__ expert_offsets, const ChainSeg seg) {
  ChainBatch* buf = reinterpret_cast<ChainBatch*>(lds);
  __shared__ int wave_tot[kChainWaves][64];
  __shared__ __align__(16) int tb_rows[kChainWaves][4 * 64];
  __shared__ int wave_flex[kChainWaves], wave_tok[kChainWaves];
  __shared__ SpecShared spec_sh;
  // (as a scalar: branches on the wave number are then uniform for the compiler, and
  // values carried around them stay in scalar registers)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int ntiles = a.ntiles;

  // (a call without tokens has no analysis kernel that would have cleared the status
  // words, and no finishing workgroup that polls them)
  if (!seg.on && ntiles == 0 && threadIdx.x < 4) ws.status[threadIdx.x] = 0;
  // Everything the workgroup reads first is requested before anything is consumed:
  // the counters, the first super-batch of byte counts, the flexible-tile masks.
  int lin = 0;
  if (lane < a.E) lin = loads_inout[lane];
  uint8_t* stage = lds;
  uint4 sv[8];  // 8 loads in flight per thread
  auto stage_load = [&](int sb0, int i0) {
    const int nt = min(kChainStageTiles, ntiles - sb0);
    const uint4* src = reinterpret_cast<const uint4*>(ws.tile_fixed_cnt + (size_t)sb0 * 64);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * kTailThreads;
      sv[u] = i < nt * 4 ? src[i] : make_uint4(0, 0, 0, 0);
    }
  };
  auto stage_store = [&](int sb0, int i0) {
    const int nt = min(kChainStageTiles, ntiles - sb0);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * kTailThreads;
      if (i < nt * 4) reinterpret_cast<uint4*>(stage)[i] = sv[u];
    }
  };
  if (ntiles > 0) stage_load(0, threadIdx.x);

  // ---- which tiles hold flexible tokens (groups of 64 tiles per ballot) ------
  const int groups = (ntiles + 63) >> 6;
  const int gper = (groups + kChainWaves - 1) / kChainWaves;
  const int ga = min(wave * gper, groups), gb = min(ga + gper, groups);
  int nfl = 0, ntok = 0;
  // masks of this lane's tiles in the wave's first two groups (kept for the second pass
  // over the groups below: a segment of a pipelined call has no more per wave)
  unsigned long long first_fm = 0ull, second_fm = 0ull;
  for (int g = ga; g < gb; ++g) {
    const int tile = g * 64 + lane;
    const unsigned long long fm = tile < ntiles ? ws.flexmask[tile] : 0ull;
    if (g == ga) first_fm = fm;
    if (g == ga + 1) second_fm = fm;
    nfl += __builtin_popcountll(__builtin_amdgcn_ballot_w64(fm != 0ull));
    ntok += __builtin_popcountll(fm);
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) ntok += __shfl_xor(ntok, d, 64);
  if (lane == 0) {
    wave_flex[wave] = nfl;
    wave_tok[wave] = ntok;
  }
  __syncthreads();
  int fbefore = 0, nflex_tiles = 0, tokbefore = 0, nflex_tok = 0;  // nflex_tok: flexible tokens of the call
  for (int w = 0; w < kChainWaves; ++w) {
    const int fl = wave_flex[w], tk = wave_tok[w];
    fbefore += w < wave ? fl : 0;
    tokbefore += w < wave ? tk : 0;
    nflex_tiles += fl;
    nflex_tok += tk;
  }
  // a handful of flexible tokens: the finishing workgroups resolve them themselves and
  // write the totals; nothing to do here
  // (never in a pipelined call: the finishing workgroups judge by the whole call's sizes)
  if (!seg.on && fast_path_applies(ntiles, nflex_tiles, nflex_tok, a.cw)) return;
  // Without flexible tokens, small problems are finished without tile_base (the
  // finishing workgroups sum the byte counts themselves): only the totals are needed.
  // (A segment cannot know what the later segments hold.)
  const bool need_tile_base = seg.on || nflex_tiles > 0 || ntiles > kSelfPrefixTiles;

  // ---- prefix over tiles of the fixed tokens' counts -------------------------
  // The byte counts are staged through LDS in super-batches with wide loads; wave
  // w then scans a contiguous run of tiles for its lane's expert.
  int carry = seg.on ? seg.carry0 : 0;  // assignments before this super-batch (lane's expert)
  for (int sb0 = 0; sb0 < ntiles; sb0 += kChainStageTiles) {
    const int nt = min(kChainStageTiles, ntiles - sb0);
    for (int i0 = threadIdx.x; i0 < nt * 4; i0 += kTailThreads * 8) {
      if (sb0 != 0 || i0 != (int)threadIdx.x) stage_load(sb0, i0);  // the very first batch is in flight
      stage_store(sb0, i0);
    }
    __syncthreads();
    const int per_wave = (nt + kChainWaves - 1) / kChainWaves;
    const int ta = min(wave * per_wave, nt), tb = min(ta + per_wave, nt);
    int tot = 0;
#pragma unroll 16
    for (int tile = ta; tile < tb; ++tile) tot += stage[tile * 64 + lane];
    wave_tot[wave][lane] = tot;
    __syncthreads();
    int run = carry;
    for (int w = 0; w < kChainWaves; ++w) {
      const int v = wave_tot[w][lane];
      run += w < wave ? v : 0;
      carry += v;
    }
    if (need_tile_base) {
      // Four tiles per store: a wavefront has at most 64 memory operations in flight, and
      // with one store per tile a long run of tiles (a segment of a pipelined call: 128
      // per wave) would wait for memory round trips.  The four rows meet in a wave-private
      // piece of LDS, laid out like the rows of tile_base, and leave as 16 bytes per lane.
      int* rows = tb_rows[wave];
      int tile = ta;
      for (; tile + 4 <= tb; tile += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          rows[u * 64 + lane] = run;
          run += stage[(tile + u) * 64 + lane];
        }
        const int4 v = reinterpret_cast<const int4*>(rows)[lane];
        reinterpret_cast<int4*>(ws.tile_base + (size_t)(sb0 + tile) * 64)[lane] = v;
      }
      for (; tile < tb; ++tile) {
        ws.tile_base[(size_t)(sb0 + tile) * 64 + lane] = run;
        run += stage[tile * 64 + lane];
      }
    }
    // stage and wave_tot are reused by the next super-batch (after the last one nothing
    // writes LDS before the next barrier, and that barrier then waits for the stores
    // above once, together with those below)
    if (sb0 + kChainStageTiles < ntiles) __syncthreads();
  }
  const int total_fixed = carry;

  nflex_tiles = __builtin_amdgcn_readfirstlane(nflex_tiles);
  nflex_tok = __builtin_amdgcn_readfirstlane(nflex_tok);
  const bool wide = a.cw > kMaxC;
  const bool use_spec = nflex_tok >= kSpecMinTokens && !wide;
  // order of the flexible tiles, and for every tile the number of flexible tokens before it
  const int fbase = seg.on ? seg.fbase : 0;
  for (int g = ga; g < gb && (nflex_tiles > 0 || seg.on); ++g) {
    const int tile = g * 64 + lane;
    const unsigned long long fm =
        g == ga ? first_fm : g == ga + 1 ? second_fm : (tile < ntiles ? ws.flexmask[tile] : 0ull);
    const bool f = fm != 0ull;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(f);
    const int ord = fbefore + __builtin_popcountll(bal & lanes_below(lane));
    const int np = __builtin_popcountll(fm);
    int incl = np;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (tile < ntiles) {
      ws.flex_ord[tile] = ord;
      ws.flex_tok_base[tile] = fbase + tokbefore + incl - np;  // (read by the finishing pass only)
      if (tile == ntiles - 1 && !seg.on) ws.flex_tok_base[ntiles] = tokbefore + incl;
    }
    if (f) ws.flex_list[ord] = tile;
    if (use_spec) {
      // slot (tile * 64 + rank among the tile's flexible tokens) of every flexible token:
      // every lane lists its own tile's
      const int mybase = tokbefore + incl - np;
      for (int i = 0; __builtin_amdgcn_ballot_w64(i < np) != 0ull; ++i)
        if (i < np) ws.flex_slot[mybase + i] = (tile << 6) + i;
    }
    fbefore += __builtin_popcountll(bal);
    tokbefore += __shfl(incl, 63, 64);
  }

  int gflex = 0;  // flexible assignments so far (meaningful in wave 0)

  auto write_totals = [&]() {  // wave 0: final loads and the exclusive prefix over experts
    const int cnt = lane < a.E ? total_fixed + gflex : 0;
    if (lane < a.E) loads_inout[lane] = lin + cnt;
    int incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane < a.E) expert_offsets[lane] = incl - cnt;
    if (lane == a.E - 1) expert_offsets[a.E] = incl;
  };

  // A segment hands its results to the caller instead of publishing anything.
  auto segment_result = [&]() {  // wave 0
    seg.out[lane] = total_fixed + gflex;
    if (lane == 0) {
      seg.out[64] = nflex_tiles;
      seg.out[65] = nflex_tok;
    }
  };
  if (wave == 0 && (nflex_tiles > 0 || seg.on)) ws.chain_cum[lane] = 0;  // nothing chosen before flexible token 0
  if (seg.on) {
    if (nflex_tiles == 0) {
      if (wave == 0) segment_result();
      return;
    }
    __syncthreads();  // tile_base, flex_list, flex_ord, flex_slot written by every wave
  } else {
    if (nflex_tiles == 0 && wave == 0) write_totals();  // already final
    __syncthreads();  // tile_base, flex_list, flex_ord (and the totals) written by every wave
    if (threadIdx.x == 0) {
      ws.status[kStatusFlexTiles] = nflex_tiles;
      __hip_atomic_store(&ws.status[kStatusPhase], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (nflex_tiles == 0) return;
  }

  int decided = 0;
  unsigned hist0 = 0;
  if (use_spec) {
    // First guesses and the window of 128 where tokens rarely compete: many experts per
    // candidate.  With few experts every sweep ends at an early conflict and the guesses
    // only cost: one consumer wave, a window of 64.
#define LASER_SPEC_WALK(CP_, KK_)                                                                   \
  (a.E >= 4 * CP_ ? spec_walk2<CP_, KK_>(lds, nflex_tok, a, ws, wave, lane, lin, gflex, hist0) \
                  : spec_walk<CP_, KK_, false>(lds, spec_sh, nflex_tok, a, ws, wave, lane, lin, gflex, hist0))
    if (a.c <= 4) {
      decided = a.k == 2 ? LASER_SPEC_WALK(4, 2) : LASER_SPEC_WALK(4, 0);
    } else if (a.c <= 8) {
      decided = a.k == 6 ? LASER_SPEC_WALK(8, 6) : LASER_SPEC_WALK(8, 0);
    } else {
      decided = LASER_SPEC_WALK(16, 0);
    }
#undef LASER_SPEC_WALK
  }
  if (decided < nflex_tok) {
    // the rest (or everything) one token after the other
    int ft0 = 0, r0 = 0;
    if (decided > 0) {
      const int slot = ws.flex_slot[decided];
      ft0 = ws.flex_ord[slot >> 6];
      r0 = slot & 63;
    }
    if (wide)
      chain_walk<0>(buf, ft0, r0, decided, hist0, nflex_tiles, a, ws, wave, lane, lin, gflex);
    else if (a.c <= 4)
      chain_walk<4>(buf, ft0, r0, decided, hist0, nflex_tiles, a, ws, wave, lane, lin, gflex);
    else if (a.c <= 8)
      chain_walk<8>(buf, ft0, r0, decided, hist0, nflex_tiles, a, ws, wave, lane, lin, gflex);
    else
      chain_walk<16>(buf, ft0, r0, decided, hist0, nflex_tiles, a, ws, wave, lane, lin, gflex);
  }
  if (seg.on) {
    if (wave == 0) segment_result();
    return;
  }
  if (wave == 0) write_totals();
  __syncthreads();
  if (threadIdx.x == 0)
    __hip_atomic_store(&ws.status[kStatusPhase], 2, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- pipelined calls: the chain segment by segment ---------------------------------
//
// Algorithm 1 orders the tokens of a batch, so the chain over tiles [0, n) needs nothing
// of the tiles behind them.  A large call is therefore cut into segments of a.seg_tiles
// tiles; the chain over a segment starts as soon as the gate kernel has analysed the
// segment's tiles, inside that kernel (workgroup 0 of its grid), while the other
// workgroups go on streaming the later tiles.  Every wavefront of an analysis workgroup
// counts itself into its tile's word of ws.seg when its records are written and
// acknowledged (what the chain reads is stored write-through); the chain workgroup waits
// for all tiles of a segment to be complete and then invalidates its caches (acquire).
// The wait is bounded: should it ever give up, the tail kernel's chain workgroup takes
// over where it stopped, behind the kernel boundary; otherwise the tail kernel's finds
// every segment done and only writes the totals and raises the flags.
// What is carried from segment to segment (ws.seg) is small: per expert the assignments
// so far, and where the numbering of flexible tokens and tiles goes on.  A segment's
// flexible tokens are numbered from a multiple of 32 (words of chain_bits / chain_cum
// are not shared between segments), chain_cum restarts at 0 in every segment, and
// tile_base carries the earlier segments' choices -- the finishing pass reads all of it
// exactly as in a call that is not pipelined.

// The chain numbers the tiles, the flexible tokens and the tiles with flexible tokens of a
// segment from 0.  `v` becomes the view of the arrays in which those are dtiles tiles,
// dflex flexible tokens (a multiple of 32) and dord flexible tiles further on than in `v`.
// (Advanced in place from segment to segment: one set of pointers in scalar registers.)
__device__ __forceinline__ void advance_view(Workspace& v, const RouteArgs& a, int dtiles, int dflex, int dord) {
  const size_t tok = (size_t)dtiles * kTile;  // tokens and record slots
  v.rec_cstar += tok;
  v.rec_ids += tok * a.cw;
  v.rec_p += tok * a.cw;
  v.rec_Z += tok;
  v.rec_lane += tok * a.EP;
  v.flexmask += dtiles;
  v.tile_fixed_cnt += (size_t)dtiles * 64;
  v.tile_mask += (size_t)dtiles * 64;
  v.tile_base += (size_t)dtiles * 64;
  v.rec_cids += tok * 16;
  v.rec_pref += tok * 16;
  v.flex_list += dord;
  v.flex_ord += dtiles;
  v.flex_tok_base += dtiles;
  v.flex_slot += dflex;
  v.chain_bits += (size_t)(dflex >> 5) * 64;
  v.chain_cum += (size_t)(dflex >> 5) * 64;
}

// Polls of a segment's counter before the chain workgroup inside the gate kernel leaves
// the rest to the tail kernel (a poll is a memory round trip plus a short sleep).
constexpr long long kSegPollLimit = 1ll << 20;
// Every wavefront of an analysis workgroup counts itself into its tile's word.
constexpr int kGateSignals = 8;

// The chain of a call, by the chain workgroup (kTailThreads threads) of the gate kernel
// (IN_GATE: as far as the analysed tiles allow, nothing is published) or of the tail
// kernel (the rest, then the totals and the flags the finishing workgroups wait for).
template <bool IN_GATE>
__device__ __forceinline__ void chain_segments(uint8_t* lds, const RouteArgs& a, const Workspace& ws,
                                               int32_t* __restrict__ loads_inout,
                                               int32_t* __restrict__ expert_offsets) {
  ChainSeg sg;
  sg.on = a.nseg > 0;  // (not pipelined: one round over the whole call, which publishes for itself)
  sg.carry0 = 0;
  sg.fbase = 0;
  __shared__ int seg_out[66];
  __shared__ int seg_ready;
  sg.out = seg_out;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int32_t* const status = ws.status;
  int32_t* const segw = ws.seg;
  int j = 0, fbase = 0, ordbase = 0, carry = 0;
  RouteArgs av = a;
  Workspace wv = ws;
  if (sg.on) {
    // (written by the kernel before this one: the clearing kernel, or the gate kernel)
    j = __builtin_amdgcn_readfirstlane(segw[kSegNext]);
    fbase = __builtin_amdgcn_readfirstlane(segw[kSegFlexBase]);
    ordbase = __builtin_amdgcn_readfirstlane(segw[kSegOrdBase]);
    carry = segw[kSegCarry + lane];
    advance_view(wv, a, min(segment_start(a, j), a.ntiles), fbase, ordbase);
  }
  const int rounds = sg.on ? a.nseg : 1;
  for (; j < rounds; ++j) {
    if (sg.on) {
      const int tile0 = segment_start(a, j);
      const int nt = min(segment_start(a, j + 1), a.ntiles) - tile0;
      if (IN_GATE) {
        // every thread waits for some of the segment's tiles (all of their wavefronts
        // counted in), then the workgroup agrees on whether all of them are there
        if (threadIdx.x == 0) seg_ready = 1;
        __syncthreads();
        bool mine = true;
        for (int i = threadIdx.x; i < nt && mine; i += kTailThreads)
          mine = poll_word(&segw[kSegDone + tile0 + i], kGateSignals, kSegPollLimit);
        if (!mine) seg_ready = 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        __syncthreads();
        const bool ready = seg_ready != 0;
        __syncthreads();  // (seg_ready is written again in the next round)
        if (!ready) break;
      }
      av.ntiles = nt;
      av.T = min(a.T - tile0 * kTile, nt * kTile);
      sg.carry0 = carry;
      sg.fbase = fbase;
    }
    chain_workgroup(lds, av, wv, loads_inout, expert_offsets, sg);
    if (!sg.on) return;
    __syncthreads();  // seg_out written (wave 0); the chain's LDS is free again
    carry = seg_out[lane];
    // (as scalars: the next segment's view is then computed in scalar registers)
    const int dord = __builtin_amdgcn_readfirstlane(seg_out[64]);
    const int dflex = (__builtin_amdgcn_readfirstlane(seg_out[65]) + 32) & ~31;
    advance_view(wv, a, av.ntiles, dflex, dord);
    ordbase += dord;
    fbase += dflex;
    __syncthreads();  // (seg_out is written again in the next round)
  }
  if (IN_GATE) {
    // for the tail kernel, behind the kernel boundary
    if (wave == 0) segw[kSegCarry + lane] = carry;
    if (threadIdx.x == 0) {
      segw[kSegNext] = j;
      segw[kSegFlexBase] = fbase;
      segw[kSegOrdBase] = ordbase;
    }
    return;
  }
  // the totals, and the flags of the finishing workgroups
  if (wave == 0) {
    const int lin = lane < a.E ? loads_inout[lane] : 0;
    const int cnt = lane < a.E ? carry : 0;
    if (lane < a.E) loads_inout[lane] = lin + cnt;
    int incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane < a.E) expert_offsets[lane] = incl - cnt;
    if (lane == a.E - 1) expert_offsets[a.E] = incl;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    status[kStatusFlexTiles] = ordbase;
    __hip_atomic_store(&status[kStatusPhase], 2, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// ---- a handful of flexible tokens: every finishing workgroup resolves them itself ----
//
// With thresholds like the paper's, a layer of a skewed gate has no or very few
// flexible tokens.  Waiting for the chain workgroup then costs several dependent
// memory round trips and two flag hand-overs for one or two chain steps.  Instead,
// when the call has at most kFastTokens flexible tokens in at most kFastTiles tiles
// (and at most kFastMaxTiles tiles in all, so that one batch of loads covers every
// tile's counts), every finishing workgroup sums, beside its own prefix, the fixed
// assignments before each flexible tile, fetches the few records and walks them with
// the same step as the sequential chain.  All workgroups compute the same choices;
// nobody waits for anybody, and the chain workgroup has nothing to do.
struct FastShared {
  unsigned long long bal[kChainWaves];          // wave w: which of tiles 64w .. 64w+63 are flexible
  unsigned long long fmtile[kFastMaxTiles];     // flexible-token mask of a flexible tile
  int fbefore[kFastTiles][kChainWaves][64];     // per wave: fixed assignments in the tiles before
                                                // the f-th flexible tile, per expert
  // the n-th flexible token of the call:
  unsigned rec[kFastTokens][64];                // its record row (lane = expert)
  uint4 cids[kFastTokens];                      // candidate experts by rank, padded
  uint8_t rids[kFastTokens][kMaxC];             // candidate experts by rank
  float p[kFastTokens][kMaxC];                  // their probabilities
  float Z[kFastTokens];                         // the softmax denominator
  int tok[kFastTokens];                         // token index
  int tokf[kFastTokens];                        // index of its flexible tile
  unsigned long long emask[kFastTokens];        // the experts chosen for it
};

struct FinishLds {
  unsigned long long mask64[64];
  int before[64];  // per expert: slots of all earlier experts + of this expert in earlier tiles
  uint8_t ids[kTile][kMaxC];
};

// What a finishing wave can read before anything else of the tail kernel has run.
struct FinishPrologue {
  int cstar;               // working-set size of a flexible token, else 0
  unsigned long long fm;   // the tile's flexible-token mask
  unsigned long long tmask;  // lane = expert: the tile's non-flexible tokens assigned to it
  int ids[kMaxC];          // experts of the token as the analysis left them (k entries)
};

// Requests the loads only; nothing here waits for them.
__device__ __forceinline__ FinishPrologue finish_prologue(int tile, const RouteArgs& a, const Workspace& ws,
                                                          const int32_t* __restrict__ expert_ids) {
  const int lane = threadIdx.x & 63;
  const int t = tile * kTile + lane;
  const bool live = t < a.T;
  FinishPrologue p;
  p.cstar = live ? ws.rec_cstar[t] : 0;
  p.fm = ws.flexmask[tile];
  p.tmask = ws.tile_mask[(size_t)tile * 64 + lane];
#pragma unroll
  for (int j = 0; j < kMaxC; ++j) p.ids[j] = (live && j < a.k) ? expert_ids[(size_t)t * a.k + j] : 0;
  return p;
}

// experts of the tokens that are final already go to LDS (rows of flexible tokens hold
// stale data; they are overwritten in finish_tile)
__device__ __forceinline__ void finish_commit(FinishLds* fl, const FinishPrologue& p, int k) {
  const int lane = threadIdx.x & 63;
  fl->mask64[lane] = p.tmask;  // the flexible tokens add themselves in finish_tile
#pragma unroll
  for (int j = 0; j < kMaxC; ++j)
    if (j < k) fl->ids[lane][j] = (uint8_t)p.ids[j];
}

// One wavefront, one tile; `fl` is this wave's private LDS.
// If `self` is set the caller has already computed, for every expert, the number of
// assignments in earlier tiles (own_base, LDS, 64 words) and the exclusive prefix over
// experts of the totals (own_offsets, LDS, 64 words); nothing is awaited then.
__device__ __forceinline__ void finish_tile(FinishLds* fl, int tile, const FinishPrologue pro, const RouteArgs& a,
                            const Workspace& ws, const int32_t* __restrict__ expert_offsets,
                            int32_t* __restrict__ expert_ids, float* __restrict__ weights,
                            int32_t* __restrict__ permutation, bool self, const int* own_base,
                            const int* own_offsets, int fast_n = 0, const FastShared* fast = nullptr) {
  const int lane = threadIdx.x & 63;
  const int t = tile * kTile + lane;
  const bool live = t < a.T;
  const int k = a.k;
  const int cstar = pro.cstar;
  const unsigned long long fm = pro.fm;

  bool any_flex = false;
  if (__builtin_expect(!self, 0)) {
    if (!poll_flag(&ws.status[kStatusPhase], 1, a.spin_limit)) {
      ws.status[kStatusError] = kErrorTimeout;
      return;
    }
    any_flex = load_published(&ws.status[kStatusFlexTiles]) > 0;
    if (any_flex && !poll_flag(&ws.status[kStatusPhase], 2, a.spin_limit)) {
      ws.status[kStatusError] = kErrorTimeout;
      return;
    }
  }

  // lane = expert: where this tile's first slot of the expert goes.  With flexible
  // tokens about, the choices made for the f0 flexible tokens of earlier tiles are
  // the running count at the last 32-token boundary plus the bits since.
  const int f0 = any_flex ? load_published(&ws.flex_tok_base[tile]) : 0;
  {
    int bef;
    if (__builtin_expect(self, 1)) {
      bef = own_offsets[lane] + own_base[lane];
    } else {
      bef = (lane < a.E ? load_published(&expert_offsets[lane]) : 0) +
            load_published(&ws.tile_base[(size_t)tile * 64 + lane]);
      if (any_flex) {
        const size_t w = (size_t)(f0 >> 5) * 64 + lane;
        const unsigned bits = load_published(&ws.chain_bits[w]) & ((1u << (f0 & 31)) - 1u);
        bef += load_published(&ws.chain_cum[w]) + __builtin_popcount(bits);
      }
    }
    fl->before[lane] = bef;
  }

  if (__builtin_expect(cstar > 0, 0)) {
    const int f = f0 + __builtin_popcountll(fm & lanes_below(lane));
    const unsigned* cw = ws.chain_bits + (size_t)(f >> 5) * 64;
    // (called twice so that each copy knows its address space: LDS or memory)
    auto write_row = [&](const uint8_t* ids, const float* pv, float Z, unsigned long long chosen) {
      float denom = Z;
      if (a.renormalize) {
        bool first = true;
        for (int j = 0; j < cstar; ++j) {
          if ((chosen >> ids[j]) & 1ull) {
            denom = first ? pv[j] : denom + pv[j];
            first = false;
          }
        }
      }
      int n = 0;
      for (int j = 0; j < cstar; ++j) {
        const int e = ids[j];
        if (((chosen >> e) & 1ull) && n < k) {  // (exactly k bits are set; n < k keeps the row)
          expert_ids[(size_t)t * k + n] = e;
          weights[(size_t)t * k + n] = pv[j] / denom;
          fl->ids[lane][n] = (uint8_t)e;
          ++n;
        }
      }
    };
    if (fast_n > 0) {
      // the workgroup resolved the call's few flexible tokens itself: all is in LDS
      int n = 0;
      for (int i = 0; i < fast_n; ++i) n = fast->tok[i] == t ? i : n;
      write_row(fast->rids[n], fast->p[n], fast->Z[n], fast->emask[n]);
    } else {
      const uint8_t* ids = ws.rec_ids + (size_t)t * a.cw;
      unsigned long long chosen = 0ull;
      for (int j = 0; j < cstar; ++j)
        chosen |= (unsigned long long)((load_published(&cw[ids[j]]) >> (f & 31)) & 1u) << ids[j];
      write_row(ids, ws.rec_p + (size_t)t * a.cw, a.renormalize ? 0.0f : ws.rec_Z[t], chosen);
    }
  }
  // LDS traffic of one wavefront is processed in order; the fences only stop the
  // compiler from moving reads above the other lanes' writes
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  // (the masks came from the analysis with the non-flexible tokens in them)
  if (__builtin_expect(cstar > 0, 0))
    for (int j = 0; j < k; ++j) atomicOr(&fl->mask64[fl->ids[lane][j]], 1ull << lane);
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  if (live) {
    const unsigned long long below = lanes_below(lane);
    for (int j = 0; j < k; ++j) {
      const int e = fl->ids[lane][j];
      const int pos = fl->before[e] + __builtin_popcountll(fl->mask64[e] & below);
      // (pos is a slot number by construction; the check turns any inconsistency of
      // the inputs into a missing entry instead of a stray store)
      if ((unsigned)pos < (unsigned)(a.T * k))
        permutation[pos] = t * k + j;
      else
        ws.status[kStatusError] = kErrorInconsistent;
    }
  }
}

// Per-expert assignment counts of the tiles before `t0` and of all tiles, summed by
// the whole workgroup straight from the analysis kernel's byte counts.  Only valid
// when no tile holds a flexible token (then the fixed counts are all there is).
// Lane l of a load takes experts 4*(l%16)..+3 of tile 4*j + l/16; bytes are
// accumulated pairwise in 16-bit fields (at most 64 per tile, ntiles <= 1024).
__device__ __forceinline__ void self_prefix(int t0, const RouteArgs& a, const Workspace& ws, int (*sh_before)[64],
                            int (*sh_all)[64], int* sh_anyflex, unsigned long long& fm_first) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ntiles = a.ntiles;
  const int sub = lane >> 4;  // which of the 4 tiles of a load
  const unsigned* cnt32 = reinterpret_cast<const unsigned*>(ws.tile_fixed_cnt);
  unsigned b02 = 0, b13 = 0, a02 = 0, a13 = 0;
  // flexible-tile masks first (ntiles <= kSelfPrefixTiles: at most 4 per thread), so that
  // their latency overlaps the count loads
  unsigned long long fmv[kSelfPrefixTiles / kTailThreads];
#pragma unroll
  for (int u = 0; u < kSelfPrefixTiles / kTailThreads; ++u) {
    const int i = threadIdx.x + u * kTailThreads;
    fmv[u] = i < ntiles ? ws.flexmask[i] : 0ull;
  }
  const int nload = (ntiles + 3) >> 2;
  constexpr int kBatch = 16;  // loads issued together: the loop is bound by latency, not by volume
  for (int j0 = wave; j0 < nload; j0 += kChainWaves * kBatch) {
    unsigned wd[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int tile = 4 * (j0 + u * kChainWaves) + sub;
      wd[u] = tile < ntiles ? cnt32[(size_t)tile * 16 + (lane & 15)] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int tile = 4 * (j0 + u * kChainWaves) + sub;
      const unsigned lo = wd[u] & 0x00FF00FFu, hi = (wd[u] >> 8) & 0x00FF00FFu;
      a02 += lo;
      a13 += hi;
      b02 += tile < t0 ? lo : 0u;
      b13 += tile < t0 ? hi : 0u;
    }
  }
  // fold the 4 tile sub-groups of the wave (lanes l, l+16, l+32, l+48)
#pragma unroll
  for (int d = 16; d < 64; d <<= 1) {
    a02 += __shfl_xor(a02, d, 64);
    a13 += __shfl_xor(a13, d, 64);
    b02 += __shfl_xor(b02, d, 64);
    b13 += __shfl_xor(b13, d, 64);
  }
  if (lane < 16) {
    const int e = 4 * lane;
    sh_all[wave][e] = a02 & 0xFFFF;
    sh_all[wave][e + 1] = a13 & 0xFFFF;
    sh_all[wave][e + 2] = a02 >> 16;
    sh_all[wave][e + 3] = a13 >> 16;
    sh_before[wave][e] = b02 & 0xFFFF;
    sh_before[wave][e + 1] = b13 & 0xFFFF;
    sh_before[wave][e + 2] = b02 >> 16;
    sh_before[wave][e + 3] = b13 >> 16;
  }
  fm_first = fmv[0];  // the mask of tile threadIdx.x
  bool flex = false;
#pragma unroll
  for (int u = 0; u < kSelfPrefixTiles / kTailThreads; ++u) flex |= fmv[u] != 0ull;
  const bool any = __builtin_amdgcn_ballot_w64(flex) != 0ull;  // (all lanes take part)
  if (lane == 0) sh_anyflex[wave] = any ? 1 : 0;
}

// Called by a whole finishing workgroup once it knows that some tile holds flexible
// tokens (ntiles <= kFastMaxTiles: thread i looked at tile i's flexible mask, fm_mine).
// Returns 0, having done nothing but look, if there are too many; otherwise the
// number of flexible tokens, with own_base / own_offsets and the choices (fs.emask,
// fs.tok) ready for finish_tile.  sh_before / sh_all hold the four waves' partial sums
// of the fixed counts before this workgroup's tiles / of all tiles.  A lone wavefront
// issues an instruction every few cycles only, so the point here is few instructions:
// per-token state lives in LDS and the loops over tokens are not unrolled.  (Inlined
// by force, like every helper of this kernel: a real call gives the kernel a stack,
// and every wave of it a slower start.)
__device__ __forceinline__ int finish_fast(int block, FastShared& fs, unsigned long long fm_mine,
                                           const int (&wg_cnt)[kChainWaves - 1], int (*sh_before)[64],
                                           int (*sh_all)[64], int (*own_base)[64], int* own_offsets,
                                           const RouteArgs& a, const Workspace& ws,
                                           int32_t* __restrict__ loads_inout,
                                           int32_t* __restrict__ expert_offsets) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int ntiles = a.ntiles;
  const int t0 = (block - 1) * kChainWaves;
  const int tile = t0 + wave;

  // ---- the flexible tiles (wave w looked at tiles 64w .. 64w+63) ---------------------
  {
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(fm_mine != 0ull);
    if (fm_mine != 0ull) fs.fmtile[threadIdx.x] = fm_mine;
    if (lane == 0) fs.bal[wave] = bal;
  }
  __syncthreads();
  unsigned long long bal[kChainWaves];
  int nft = 0;
#pragma unroll
  for (int w = 0; w < kChainWaves; ++w) {
    const unsigned long long b = fs.bal[w];
    bal[w] = ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned)(b >> 32)) << 32) |
             (unsigned)__builtin_amdgcn_readfirstlane((unsigned)b);
    nft += __builtin_popcountll(bal[w]);
  }
  if (nft > kFastTiles) return 0;
  // in ascending order, with their masks and the number of flexible tokens
  int ftile[kFastTiles];
  unsigned long long fmask[kFastTiles];
  int ntok = 0;
#pragma unroll
  for (int f = 0; f < kFastTiles; ++f) {
    ftile[f] = 0x7fffffff;
    fmask[f] = 0ull;
    if (f < nft) {
      int tl = 0;
      bool found = false;
#pragma unroll
      for (int w = 0; w < kChainWaves; ++w) {
        if (!found && bal[w] != 0ull) {
          tl = 64 * w + __builtin_ctzll(bal[w]);
          bal[w] &= bal[w] - 1ull;
          found = true;
        }
      }
      ftile[f] = tl;
      const unsigned long long m = fs.fmtile[tl];
      fmask[f] = ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned)(m >> 32)) << 32) |
                 (unsigned)__builtin_amdgcn_readfirstlane((unsigned)m);
      ntok += __builtin_popcountll(fmask[f]);
    }
  }
  if (!fast_path_applies(ntiles, nft, ntok, a.cw)) return 0;

  // ---- lane n < ntok: the n-th flexible token of the call ---------------------------
  int my_tok = 0, my_slot = 0, my_f = 0;
  {
    int r = lane;
#pragma unroll
    for (int f = 0; f < kFastTiles - 1; ++f) {
      const int pc = __builtin_popcountll(fmask[f]);
      if (my_f == f && r >= pc) {
        r -= pc;
        my_f = f + 1;
      }
    }
    unsigned long long m = fmask[0];
    int tl = ftile[0];
#pragma unroll
    for (int f = 1; f < kFastTiles; ++f) {
      m = my_f == f ? fmask[f] : m;
      tl = my_f == f ? ftile[f] : tl;
    }
    if (lane < ntok) {
      for (int i = 0; i < r; ++i) m &= m - 1ull;  // (r < kFastTokens)
      my_tok = tl * kTile + __builtin_ctzll(m);
      my_slot = tl * kTile + r;
    }
  }

  // ---- loads: wave w fetches what belongs to tokens w and w + 4; every wave the
  // tiles' counts once more (one batch; they are near, having just been read) ----------
  static_assert(kFastTokens <= 2 * kChainWaves, "two tokens per wave");
  static_assert(kFastMaxTiles == kTailThreads, "thread i looks at tile i");
  unsigned rv[2];
  float pv[2];
  int tk[2], tf[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int n = wave + h * kChainWaves;
    rv[h] = 0xFFFFu;
    pv[h] = 0.0f;
    tk[h] = tf[h] = 0;
    if (n < ntok) {
      const int slot = __builtin_amdgcn_readlane(my_slot, n);
      tk[h] = __builtin_amdgcn_readlane(my_tok, n);
      tf[h] = __builtin_amdgcn_readlane(my_f, n);
      // lanes 0..EP-1: the record row; then 4 lanes each for the two id rows, 16 for the
      // probabilities, one for the denominator -- as bits, sorted out after the wait
      if (lane < a.EP) rv[h] = ws.rec_lane[(size_t)slot * a.EP + lane];
      const unsigned* extra = lane < 4    ? reinterpret_cast<const unsigned*>(ws.rec_cids) + (size_t)slot * 4 + lane
                              : lane < 8  ? reinterpret_cast<const unsigned*>(ws.rec_ids) + (size_t)tk[h] * 4 + (lane - 4)
                              : lane < 24 ? reinterpret_cast<const unsigned*>(ws.rec_p) + (size_t)tk[h] * 16 + (lane - 8)
                                          : reinterpret_cast<const unsigned*>(ws.rec_Z) + tk[h];
      if (lane < 25) pv[h] = __uint_as_float(*extra);
    }
  }
  const int lin = ws.lin_copy[lane];
  const int sub = lane >> 4;  // which of the 4 tiles of a count load
  const unsigned* cnt32 = reinterpret_cast<const unsigned*>(ws.tile_fixed_cnt);
  constexpr int kBatch = kFastMaxTiles / (4 * kChainWaves);  // 16 loads cover 256 tiles
  unsigned wd[kBatch];
#pragma unroll
  for (int u = 0; u < kBatch; ++u) {
    const int tl = 4 * (wave + u * kChainWaves) + sub;
    wd[u] = tl < ntiles ? cnt32[(size_t)tl * 16 + (lane & 15)] : 0u;
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int n = wave + h * kChainWaves;
    if (n < ntok) {
      fs.rec[n][lane] = rv[h];
      const unsigned bits = __float_as_uint(pv[h]);
      if (lane < 4) reinterpret_cast<unsigned*>(&fs.cids[n])[lane] = bits;
      else if (lane < 8) reinterpret_cast<unsigned*>(fs.rids[n])[lane - 4] = bits;
      else if (lane < 24) fs.p[n][lane - 8] = pv[h];
      else if (lane == 24) fs.Z[n] = pv[h];
      if (lane == 0) {
        fs.tok[n] = tk[h];
        fs.tokf[n] = tf[h];
      }
    }
  }

  // ---- fixed assignments before each flexible tile -----------------------------------
#pragma unroll
  for (int f = 0; f < kFastTiles; ++f) {
    if (f < nft) {
      unsigned c02 = 0u, c13 = 0u;
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int tl = 4 * (wave + u * kChainWaves) + sub;
        c02 += tl < ftile[f] ? (wd[u] & 0x00FF00FFu) : 0u;
        c13 += tl < ftile[f] ? ((wd[u] >> 8) & 0x00FF00FFu) : 0u;
      }
#pragma unroll
      for (int d = 16; d < 64; d <<= 1) {
        c02 += __shfl_xor(c02, d, 64);
        c13 += __shfl_xor(c13, d, 64);
      }
      if (lane < 16) {
        const int e = 4 * lane;
        fs.fbefore[f][wave][e] = c02 & 0xFFFF;
        fs.fbefore[f][wave][e + 1] = c13 & 0xFFFF;
        fs.fbefore[f][wave][e + 2] = c02 >> 16;
        fs.fbefore[f][wave][e + 3] = c13 >> 16;
      }
    }
  }
  __syncthreads();

  // ---- wave 0 walks the flexible tokens (lane = expert), as the sequential chain does ----
  if (wave == 0) {
    int gflex = 0;
    for (int n = 0; n < ntok; ++n) {
      const int f = __builtin_amdgcn_readfirstlane(fs.tokf[n]);
      int base = lin + gflex;
#pragma unroll
      for (int w = 0; w < kChainWaves; ++w) base += fs.fbefore[f][w][lane];
      const unsigned rec = fs.rec[n][lane];
      const bool cand = lane < a.EP && rec != 0xFFFFu;
      const unsigned key = cand ? (((unsigned)base << 4) + rec) : 0xFFFFFFFFu;
      const bool chosen = chain_step<16>(key, cand, fs.cids[n], a.k);
      gflex += chosen ? 1 : 0;
      const unsigned long long em = __builtin_amdgcn_ballot_w64(chosen);
      if (lane == 0) fs.emask[n] = em;
    }
  }
  __syncthreads();

  // ---- as on the path without flexible tokens, plus the flexible choices ------------
  int before = 0, all = 0, flex_before = 0, flex_all = 0;  // lane = expert
#pragma unroll
  for (int w = 0; w < kChainWaves; ++w) {
    before += sh_before[w][lane];
    all += sh_all[w][lane];
  }
#pragma unroll
  for (int j = 0; j < kChainWaves - 1; ++j) before += wg_cnt[j];
  for (int n = 0; n < ntok; ++n) {
    const int bit = (int)((fs.emask[n] >> lane) & 1ull);
    flex_all += bit;
    flex_before += (fs.tok[n] < tile * kTile) ? bit : 0;
  }
  own_base[wave][lane] = before + flex_before;
  const int cnt = lane < a.E ? all + flex_all : 0;
  if (wave == 0) {
    int incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    own_offsets[lane] = incl - cnt;
    if (block == 1) {
      // the chain workgroup leaves such calls alone: the totals are written here
      if (lane < a.E) {
        loads_inout[lane] = lin + cnt;
        expert_offsets[lane] = incl - cnt;
      }
      if (lane == a.E - 1) expert_offsets[a.E] = incl;
    }
  }
  __syncthreads();
  return ntok;
}

// What workgroup `block` of the tail grid does (kTailThreads threads): 0 is the chain,
// b >= 1 finishes tiles kChainWaves * (b - 1) ... .  tail_lds: kChainLdsBytes of LDS.
__device__ __forceinline__ void tail_role(int block, uint8_t* tail_lds, const RouteArgs& a,
                                          const Workspace& ws, int32_t* __restrict__ loads_inout,
                                          int32_t* __restrict__ expert_offsets,
                                          int32_t* __restrict__ expert_ids, float* __restrict__ weights,
                                          int32_t* __restrict__ permutation) {
  // (a split call of one tile may have been finished by the workgroup that analysed it)
  if (a.one_permutation != nullptr && ws.status[kStatusPhase] == kPhaseAllDone) return;
  if (block == 0) {
    chain_segments<false>(tail_lds, a, ws, loads_inout, expert_offsets);
    return;
  }
  __shared__ int sh_before[kChainWaves][64], sh_all[kChainWaves][64];
  __shared__ int own_base[kChainWaves][64], own_offsets[64];
  __shared__ int sh_anyflex[kChainWaves];  // per wave: some tile it looked at holds flexible tokens
  __shared__ FastShared fs;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t0 = (block - 1) * kChainWaves;
  const int tile = t0 + wave;
  // Small problems without flexible tokens need nothing from the chain workgroup:
  // every finishing workgroup sums the byte counts itself.
  FinishLds* fl = reinterpret_cast<FinishLds*>(tail_lds) + wave;
  const bool small = a.ntiles <= kSelfPrefixTiles;
  // (no barrier from here to the end of self_prefix: a barrier waits for every load in
  // flight, and the point is to have all of this workgroup's loads in flight at once)
  FinishPrologue pro;
  pro.cstar = 0;
  pro.fm = 0ull;
  pro.tmask = 0ull;
  if (tile < a.ntiles) pro = finish_prologue(tile, a, ws, expert_ids);
  bool self = false;
  int fast_n = 0;  // flexible tokens resolved by this workgroup itself
  // fixed counts of the workgroup's earlier tiles (needed by the self path)
  int wg_cnt[kChainWaves - 1];
#pragma unroll
  for (int j = 0; j < kChainWaves - 1; ++j)
    wg_cnt[j] = (small && j < wave && t0 + j < a.ntiles) ? ws.tile_fixed_cnt[(size_t)(t0 + j) * 64 + lane] : 0;
  if (__builtin_expect(small, 1)) {
    unsigned long long fm_mine = 0ull;
    self_prefix(t0, a, ws, sh_before, sh_all, sh_anyflex, fm_mine);
    if (tile < a.ntiles) finish_commit(fl, pro, a.k);
    __syncthreads();
    self = (sh_anyflex[0] | sh_anyflex[1] | sh_anyflex[2] | sh_anyflex[3]) == 0;
    if (__builtin_expect(self, 1)) {
      int before = 0, all = 0;
      for (int w = 0; w < kChainWaves; ++w) {
        before += sh_before[w][lane];
        all += sh_all[w][lane];
      }
      int wg_before = 0;
#pragma unroll
      for (int j = 0; j < kChainWaves - 1; ++j) wg_before += wg_cnt[j];
      own_base[wave][lane] = before + wg_before;  // this wave's tile: plus the workgroup's earlier tiles
      if (wave == 0) {
        int incl = lane < a.E ? all : 0;
        const int cnt = incl;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const int up = __shfl_up(incl, d, 64);
          if (lane >= d) incl += up;
        }
        own_offsets[lane] = incl - cnt;
      }
    }
    __syncthreads();
    // a handful of flexible tokens: resolved here, by every workgroup for itself
    // (not in a pipelined call: there the chain workgroup walks every flexible token)
    if (__builtin_expect(!self && a.ntiles <= kFastMaxTiles && a.nseg == 0, 0)) {
      fast_n = finish_fast(block, fs, fm_mine, wg_cnt, sh_before, sh_all, own_base, own_offsets, a, ws, loads_inout,
                           expert_offsets);
      self = fast_n > 0;
    }
  } else if (tile < a.ntiles) {
    finish_commit(fl, pro, a.k);
  }
  if (tile >= a.ntiles) return;
  finish_tile(fl, tile, pro, a, ws, expert_offsets, expert_ids, weights, permutation, self,
              own_base[wave], own_offsets, fast_n, &fs);
}

}  // namespace laser
