// Per-token analysis for Algorithm 1 with trimming mode RANDOM (Method: Final
// assignment, "trimming can be ... randomized (sampling c uniformly)"; appendix Pseudo
// Code, the RANDOM branch): a pool larger than c is cut down to a uniform sample of c
// of its members instead of its c best.  Everything else (scores, order, top-k mass
// test, pool, records for the chain, dispatch) is as in the deterministic analysis, in
// the same binary32 arithmetic and the same workspace layout, so the chain and the
// finishing pass do not know the difference.
//
// The sample must be reproducible, so it is defined by a counter-based generator:
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC 2011) with key = seed and counter =
// (token index low, token index high, stream, block); draw i of a token is word i % 4
// of block i / 4.  A partial Fisher-Yates shuffle of the pool's positions [0, m) in
// the score order swaps position i with i + floor(r_i * (m - i) / 2^32) for
// i = 0..c-1; the first c positions, in ascending order, are the candidates.
//
// Two kernels.  analyse_general_kernel is the whole analysis in either trimming mode:
// one workgroup per tile of 64 tokens, lane = token, per-token arrays in LDS, order
// statistics by counting (E^2 compares per token, shared by four waves), everything
// after that one wavefront's work; written for clarity.  It is used for RANDOM trimming
// where c == k (a sampled token is then not load-dependent, but its experts are the
// sample), and in both modes for trimming sizes above the 16 candidates that the fast
// analysis carries ("wide" calls: up to 64 candidates per token, e.g. the load-only
// baseline of the paper's evaluation, c = n).  Where 16 >= c > k the deterministic
// analysis already gives everything but the candidates of the tokens it trimmed, and
// random_resample_kernel only redoes those.
#include "analyse.h"
#include "laser_internal.h"

namespace laser {

constexpr int kRowF = 65;  // floats per token row in LDS (64 + 1: no bank conflicts)
constexpr int kRowB = 68;  // bytes per token row of the byte arrays (17 words)

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0;
    c1 = lo1;
    c2 = n2;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

constexpr int kRandomWaves = 4;  // the counting pass is shared by 4 waves, the rest is wave 0's

// SAMPLE: trimming mode RANDOM (otherwise the c best of the pool are kept).
template <bool SAMPLE>
__global__ __launch_bounds__(64 * kRandomWaves) void analyse_general_kernel(const float* __restrict__ logits,
                                                            size_t logits_stride, const RouteArgs a0,
                                                            const Workspace ws0, const RandomArgs rnd0,
                                                            int32_t* __restrict__ expert_ids,
                                                            float* __restrict__ weights) {
  // blockIdx.y: the problem of a batched call; it draws with its own stream id
  const int prob = blockIdx.y;
  const RouteArgs a = problem_args(a0, prob);
  const Workspace ws = problem_workspace(ws0, (size_t)prob * a0.ws_stride);
  RandomArgs rnd = rnd0;
  rnd.stream += (uint32_t)prob;
  logits += (size_t)prob * logits_stride;
  expert_ids += (size_t)prob * a.T * a.k;
  weights += (size_t)prob * a.T * a.k;
  __shared__ float zl[kTile * kRowF], pl[kTile * kRowF], tl[kTile * kRowF];
  __shared__ uint8_t ordl[kTile * kRowB], arrl[kTile * kRowB];
  __shared__ unsigned long long maskl[64];
  const int tile = blockIdx.x, lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int t = tile * kTile + lane;
  const bool live = t < a.T;
  const int E = a.E, k = a.k, c = a.c;

  // the tail kernel of this call polls these words; they are cleared here, one
  // kernel earlier on the same stream
  if (tile == 0 && threadIdx.x < 4) ws.status[threadIdx.x] = 0;
  if (tile == 0 && threadIdx.x < 64) ws.lin_copy[threadIdx.x] = (int)threadIdx.x < a.E ? a.loads_in[threadIdx.x] : 0;

  const int rows = min(kTile, a.T - tile * kTile);
  const float* src = logits + (size_t)tile * kTile * E;
  for (int idx = threadIdx.x; idx < kTile * E; idx += 64 * kRandomWaves) {
    const int tok = idx / E;
    zl[tok * kRowF + (idx - tok * E)] = tok < rows ? src[idx] : 0.0f;
  }
  __syncthreads();

  float* z = zl + lane * kRowF;
  float* p = pl + lane * kRowF;
  float* tr = tl + lane * kRowF;
  uint8_t* ord = ordl + lane * kRowB;  // expert at each position of the score order
  uint8_t* arr = arrl + lane * kRowB;  // candidate positions

  // ---- order: logit descending, equal logits by lower index -------------------
  // (wave w places experts w, w + 4, ...; every wave sees all 64 tokens)
  for (int i = wave; i < E; i += kRandomWaves) {
    const float zi = z[i];
    int before = 0;
    for (int j = 0; j < E; ++j) {
      const float zj = z[j];
      before += (zj > zi || (zj == zi && j < i)) ? 1 : 0;
    }
    ord[before] = (uint8_t)i;
  }
  __syncthreads();
  if (wave != 0) return;  // (a barrier counts only the waves that are still running)
  const float zmax = z[ord[0]];

  // ---- scores, normaliser (fixed tree), top-k mass, pool ------------------------
  int inpool = 0;
  for (int i = 0; i < E; ++i) {
    const float d = z[i] - zmax;
    p[i] = exp_fixed(clamp_exp_arg(d));
    inpool += d >= a.tau_ln ? 1 : 0;
  }
  int P = 1;
  while (P < E) P <<= 1;
  for (int i = 0; i < P; ++i) tr[i] = i < E ? p[i] : 0.0f;
  for (int s = P >> 1; s >= 1; s >>= 1)
    for (int i = 0; i < s; ++i) tr[i] = tr[i] + tr[i + s];
  const float zsum = tr[0];
  float sk = p[ord[0]];
  for (int i = 1; i < k; ++i) sk = sk + p[ord[i]];
  const bool mass_ok = sk >= a.eps_high * zsum;
  const int m = inpool > k ? inpool : k;
  const int cstar = mass_ok ? k : (c < m ? c : m);

  // ---- candidates: positions in the score order, ascending ----------------------
  if (SAMPLE && !mass_ok && m > c) {
    for (int i = 0; i < m; ++i) arr[i] = (uint8_t)i;
    const unsigned long long g = rnd.token_offset + (unsigned long long)t;
    uint32_t wv[4] = {0u, 0u, 0u, 0u};
    for (int i = 0; i < c; ++i) {
      if ((i & 3) == 0)
        philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), rnd.stream, (uint32_t)(i >> 2),
                      (uint32_t)rnd.seed, (uint32_t)(rnd.seed >> 32), wv);
      const uint32_t r = (i & 3) == 0 ? wv[0] : (i & 3) == 1 ? wv[1] : (i & 3) == 2 ? wv[2] : wv[3];
      const int j = i + (int)__umulhi(r, (uint32_t)(m - i));
      const uint8_t tmp = arr[i];
      arr[i] = arr[j];
      arr[j] = tmp;
    }
    for (int i = 1; i < c; ++i) {  // insertion sort of the first c
      const uint8_t x = arr[i];
      int j = i - 1;
      while (j >= 0 && arr[j] > x) {
        arr[j + 1] = arr[j];
        --j;
      }
      arr[j + 1] = x;
    }
  } else {
    for (int i = 0; i < cstar; ++i) arr[i] = (uint8_t)i;
  }
  const bool flex = live && !mass_ok && cstar > k;
  const bool fixed = live && !flex;

  // ---- tokens whose experts are final ------------------------------------------
  if (fixed) {
    float denom = zsum;
    if (a.renormalize) {
      denom = p[ord[arr[0]]];
      for (int j = 1; j < k; ++j) denom = denom + p[ord[arr[j]]];
    }
    for (int j = 0; j < k; ++j) {
      const int e = ord[arr[j]];
      expert_ids[(size_t)t * k + j] = e;
      weights[(size_t)t * k + j] = p[e] / denom;
    }
  }
  // per expert: the fixed tokens of the tile assigned to it
  unsigned long long mymask = 0ull;
  for (int e = 0; e < 64; ++e) {
    bool has = false;
    if (fixed)
      for (int j = 0; j < k; ++j) has = has || (int)ord[arr[j]] == e;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(has);
    if (lane == e) mymask = bal;
  }
  maskl[lane] = mymask;
  ws.tile_fixed_cnt[(size_t)tile * 64 + lane] = (uint8_t)__builtin_popcountll(mymask);
  ws.tile_mask[(size_t)tile * 64 + lane] = mymask;
  const unsigned long long fm = __builtin_amdgcn_ballot_w64(flex);
  if (lane == 0) ws.flexmask[tile] = fm;
  if (live) {
    ws.rec_cstar[t] = flex ? (uint8_t)cstar : (uint8_t)0;
    ws.rec_Z[t] = zsum;
  }
  __syncthreads();

  // ---- records of the flexible tokens -------------------------------------------
  if (flex) {
    const int slot = tile * kTile + __builtin_popcountll(fm & lanes_below(lane));
    const unsigned long long below = lanes_below(lane);
    const int cw = a.cw;
    const bool wide = cw > kMaxC;  // (the wide chain reads the per-expert rows only)
    // ranks beyond the working set point the chain at a lane that holds no candidate
    int padlane = E;
    if (E == 64 && !wide) {
      unsigned used = 0;
      for (int j = 0; j < cstar; ++j) {
        const int e = ord[arr[j]];
        if (e < 32) used |= 1u << e;
      }
      padlane = __builtin_ctz(~used);  // at most 16 of the 32 low experts are candidates
    }
    uint16_t* row = ws.rec_lane + (size_t)slot * a.EP;
    for (int e = 0; e < a.EP; ++e) row[e] = (uint16_t)0xFFFF;
    for (int j = 0; j < cw; ++j) {
      const bool in = j < cstar;
      const int e = in ? (int)ord[arr[j]] : 0;
      const int pref = in ? __builtin_popcountll(maskl[e] & below) : 0xFF;
      ws.rec_ids[(size_t)t * cw + j] = (uint8_t)e;
      ws.rec_p[(size_t)t * cw + j] = in ? p[e] : 0.0f;
      if (!wide) {
        ws.rec_cids[(size_t)slot * 16 + j] = (uint8_t)(in ? e : padlane);
        ws.rec_pref[(size_t)slot * 16 + j] = (uint8_t)pref;
      }
      if (in) row[e] = (uint16_t)(wide ? ((pref << 6) | j) : ((pref << 4) | j));
    }
  }
}

// RANDOM trimming with c > k, behind the deterministic analysis.  That analysis has
// written, for every token, what the RANDOM mode would write too -- except the
// candidates of the tokens it trimmed: load-dependent tokens whose pool is larger than c
// (working-set size c in both modes).  Those are found here by (rec_cstar > 0, pool
// size > c); their c candidates are drawn instead of taken from the top, and their
// records are written again.  Fixed tokens, masks, counts and the flexible-token masks
// are not touched: none of them depends on which candidates a flexible token has.
// One workgroup per tile; tiles without such a token cost two loads per lane.
__global__ __launch_bounds__(64 * kRandomWaves) void random_resample_kernel(const float* __restrict__ logits,
                                                             size_t logits_stride, const RouteArgs a0,
                                                             const Workspace ws0, const RandomArgs rnd0) {
  const int prob = blockIdx.y;  // the problem of a batched call; it draws with its own stream id
  const RouteArgs a = problem_args(a0, prob);
  const Workspace ws = problem_workspace(ws0, (size_t)prob * a0.ws_stride);
  RandomArgs rnd = rnd0;
  rnd.stream += (uint32_t)prob;
  logits += (size_t)prob * logits_stride;
  __shared__ float zl[kTile * kRowF];
  __shared__ uint8_t ordl[kTile * kRowB], arrl[kTile * kRowB];
  __shared__ unsigned long long maskl[64];
  const int tile = blockIdx.x, lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int t = tile * kTile + lane;
  const bool live = t < a.T;
  const int E = a.E, c = a.c;
  const int32_t* pool = a.pool_in_ws ? ws.pool : a.st_pool;

  const int cst = live ? (int)ws.rec_cstar[t] : 0;
  const int m = live ? pool[t] : 0;
  const bool sampled = cst > 0 && m > c;  // (then cst == c)
  const unsigned long long smask = __builtin_amdgcn_ballot_w64(sampled);  // the same in all four waves
  if (smask == 0ull) return;

  const int rows = min(kTile, a.T - tile * kTile);
  const float* src = logits + (size_t)tile * kTile * E;
  for (int idx = threadIdx.x; idx < kTile * E; idx += 64 * kRandomWaves) {
    const int tok = idx / E;
    zl[tok * kRowF + (idx - tok * E)] = tok < rows ? src[idx] : 0.0f;
  }
  if (wave == 0) maskl[lane] = ws.tile_mask[(size_t)tile * 64 + lane];
  const unsigned long long fm = ws.flexmask[tile];
  __syncthreads();

  const float* z = zl + lane * kRowF;
  uint8_t* ord = ordl + lane * kRowB;  // expert at each position of the score order
  uint8_t* arr = arrl + lane * kRowB;  // candidate positions

  // ---- order: logit descending, equal logits by lower index (wave w places experts
  // w, w + 4, ...) -----------------------------------------------------------------
  if (sampled) {
    for (int i = wave; i < E; i += kRandomWaves) {
      const float zi = z[i];
      int before = 0;
      for (int j = 0; j < E; ++j) {
        const float zj = z[j];
        before += (zj > zi || (zj == zi && j < i)) ? 1 : 0;
      }
      ord[before] = (uint8_t)i;
    }
  }
  __syncthreads();
  if (wave != 0 || !sampled) return;
  const float zmax = z[ord[0]];

  // ---- the sample: positions in the score order, ascending -----------------------
  for (int i = 0; i < m; ++i) arr[i] = (uint8_t)i;
  const unsigned long long g = rnd.token_offset + (unsigned long long)t;
  uint32_t wv[4] = {0u, 0u, 0u, 0u};
  for (int i = 0; i < c; ++i) {
    if ((i & 3) == 0)
      philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), rnd.stream, (uint32_t)(i >> 2), (uint32_t)rnd.seed,
                    (uint32_t)(rnd.seed >> 32), wv);
    const uint32_t r = (i & 3) == 0 ? wv[0] : (i & 3) == 1 ? wv[1] : (i & 3) == 2 ? wv[2] : wv[3];
    const int j = i + (int)__umulhi(r, (uint32_t)(m - i));
    const uint8_t tmp = arr[i];
    arr[i] = arr[j];
    arr[j] = tmp;
  }
  for (int i = 1; i < c; ++i) {  // insertion sort of the first c
    const uint8_t x = arr[i];
    int j = i - 1;
    while (j >= 0 && arr[j] > x) {
      arr[j + 1] = arr[j];
      --j;
    }
    arr[j + 1] = x;
  }

  // ---- the token's records, as the analysis writes them --------------------------
  const int slot = tile * kTile + __builtin_popcountll(fm & lanes_below(lane));
  const unsigned long long below = lanes_below(lane);
  int padlane = E;  // ranks beyond the working set point the chain at a lane that holds no candidate
  if (E == 64) {
    unsigned used = 0;
    for (int j = 0; j < c; ++j) {
      const int e = ord[arr[j]];
      if (e < 32) used |= 1u << e;
    }
    padlane = __builtin_ctz(~used);  // at most 16 of the 32 low experts are candidates
  }
  uint16_t* row = ws.rec_lane + (size_t)slot * a.EP;
  for (int e = 0; e < a.EP; ++e) row[e] = (uint16_t)0xFFFF;
  for (int j = 0; j < kMaxC; ++j) {
    const bool in = j < c;
    const int e = in ? (int)ord[arr[j]] : 0;
    const int pref = in ? __builtin_popcountll(maskl[e] & below) : 0xFF;
    ws.rec_ids[(size_t)t * 16 + j] = (uint8_t)e;
    ws.rec_p[(size_t)t * 16 + j] = in ? exp_fixed(clamp_exp_arg(z[e] - zmax)) : 0.0f;
    ws.rec_cids[(size_t)slot * 16 + j] = (uint8_t)(in ? e : padlane);
    ws.rec_pref[(size_t)slot * 16 + j] = (uint8_t)pref;
    if (in) row[e] = (uint16_t)((pref << 4) | j);
  }
}

hipError_t launch_random_resample(const float* logits, size_t logits_stride, const RouteArgs& a,
                                  const Workspace& ws, const RandomArgs& rnd, hipStream_t s) {
  if (a.ntiles == 0) return hipSuccess;
  clear_stale_error();
  hipLaunchKernelGGL(random_resample_kernel, dim3(a.ntiles, a.nbatch), dim3(64 * kRandomWaves), 0, s, logits,
                     logits_stride, a, ws, rnd);
  return hipGetLastError();
}

hipError_t launch_analyse_general(const float* logits, size_t logits_stride, const RouteArgs& a,
                                  const Workspace& ws, bool sample, const RandomArgs& rnd,
                                  int32_t* expert_ids, float* weights, hipStream_t s) {
  if (a.ntiles == 0) return hipSuccess;
  clear_stale_error();
  if (sample)
    hipLaunchKernelGGL(analyse_general_kernel<true>, dim3(a.ntiles, a.nbatch), dim3(64 * kRandomWaves), 0, s,
                       logits, logits_stride, a, ws, rnd, expert_ids, weights);
  else
    hipLaunchKernelGGL(analyse_general_kernel<false>, dim3(a.ntiles, a.nbatch), dim3(64 * kRandomWaves), 0, s,
                       logits, logits_stride, a, ws, rnd, expert_ids, weights);
  return hipGetLastError();
}

}  // namespace laser
