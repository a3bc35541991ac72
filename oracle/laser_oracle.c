/*
 * CPU oracle for the per-layer LASER routing step.  TEST INFRASTRUCTURE ONLY:
 * slow, single-threaded, written to be checked against the paper by eye.  It
 * shares no code, header, table or constant with the GPU library and must never
 * be called from the product path.
 *
 * What it computes (paper: section "The Method", appendix "Pseudo Code",
 * Algorithm 1 "per token, per layer"):
 *   gate projection   z[t,e] = sum_h hidden[t,h] * W[e,h]            (fp64)
 *   scores            s = softmax(z)        (non-negative, summing to one)
 *   top-k mass        M_k = s_(1) + ... + s_(k)
 *   expansion rule    M_k >= eps_high  ->  A = top-k, stop
 *   candidate pool    T = { i : s_i >= t_fix * s_(1) }  union  top-k
 *   trimming (TOP)    Cand = the c* = min(c, |T|) highest-scoring members of T
 *   final assignment  sort Cand by (load ascending, score descending); A = first k
 * applied to tokens 0..T-1 in index order, each expert of A getting load += 1
 * before the next token is routed (the paper's current load L_e; Algorithm 1
 * itself has no update line -- this is the reading taken here), followed by the
 * token-to-expert dispatch tables (per-expert counts, their exclusive prefix
 * sums, and the stable counting-sort permutation of the T*k assignments).
 *
 * Two routers live here:
 *   laser_oracle_route          decisions in binary32 under the fixed operation
 *                               order documented at exp_canon()/route below (the
 *                               precision the GPU kernels decide in), weights in
 *                               fp64.
 *   laser_oracle_route_literal  everything in fp64 with libm, formulas exactly as
 *                               printed in the paper; used to check that the
 *                               binary32 reading has the paper's meaning.
 *
 * Pins (tests/test_oracle_*.py): hand-worked cases, reduction to a library top-k
 * (c = k, small eps_high, t_fix = 1), brute-force subset enumeration, the
 * load-only closed form (equal final loads), counting invariants, split-call
 * equivalence, numpy stable argsort for the dispatch, numpy fp64 matmul for the
 * gate, libm exp for exp_canon.  No function here is "parity unpinned"; what is
 * unpinned is agreement with the paper's own runs, which print no routing values.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_E_ARG (-1)
#define ORACLE_E_MEM (-2)

/* ------------------------------------------------------------------ gate -- */

static double bf16_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* Gate function: the learned linear map from a token's hidden state to one
 * logit per expert (Introduction: the small gating network whose output is the score
 * distribution over experts).  dtype 0 = fp32 inputs, 1 = bf16 bit patterns.
 * hidden [T,H] row-major, w [E,H] row-major, logits [T,E] fp64. */
int laser_oracle_gate(const void* hidden, const void* w, int32_t T, int32_t H,
                      int32_t E, int32_t dtype, double* logits) {
  if (T < 0 || H < 1 || E < 1 || (dtype != 0 && dtype != 1)) return ORACLE_E_ARG;
  for (int32_t t = 0; t < T; ++t) {
    for (int32_t e = 0; e < E; ++e) {
      double acc = 0.0;
      for (int32_t h = 0; h < H; ++h) {
        double x, y;
        if (dtype == 1) {
          x = bf16_to_double(((const uint16_t*)hidden)[(size_t)t * H + h]);
          y = bf16_to_double(((const uint16_t*)w)[(size_t)e * H + h]);
        } else {
          x = (double)((const float*)hidden)[(size_t)t * H + h];
          y = (double)((const float*)w)[(size_t)e * H + h];
        }
        acc += x * y;
      }
      logits[(size_t)t * E + e] = acc;
    }
  }
  return ORACLE_OK;
}

/* ------------------------------------------------- binary32 building blocks -- */

/* exp(x) for x in [-80, 0] as a fixed sequence of binary32 operations, so that
 * two independent implementations return the same bits:
 *   n = rint(x * fl(log2 e));  r = x - n*ln2 (two-constant Cody-Waite, fused);
 *   q = degree-7 Taylor polynomial of exp(r) in Horner form with fused
 *   multiply-adds, coefficients fl(1/j!);  result = q * 2^n (exact scaling).
 * exp_canon(0) is exactly 1. */
float laser_oracle_exp(float x) {
  const float log2e = 0x1.715476p+0f;
  const float ln2_hi = 0x1.62e4p-1f;
  const float ln2_lo = 0x1.7f7d1cp-20f;
  float n = rintf(x * log2e);
  float r = fmaf(n, -ln2_hi, x);
  r = fmaf(n, -ln2_lo, r);
  float q = 0x1.a01a02p-13f;          /* 1/7! */
  q = fmaf(q, r, 0x1.6c16c2p-10f);    /* 1/6! */
  q = fmaf(q, r, 0x1.111112p-7f);     /* 1/5! */
  q = fmaf(q, r, 0x1.555556p-5f);     /* 1/4! */
  q = fmaf(q, r, 0x1.555556p-3f);     /* 1/3! */
  q = fmaf(q, r, 0.5f);               /* 1/2! */
  q = fmaf(q, r, 1.0f);
  q = fmaf(q, r, 1.0f);
  return ldexpf(q, (int)n);
}

/* Sum of v[0..n) in binary32 by the fixed tree: pad with +0 to a power of two P,
 * then for s = P/2, P/4, ..., 1 add element i+s onto element i for all i < s. */
float laser_oracle_tree_sum(const float* v, int32_t n) {
  int32_t P = 1;
  while (P < n) P *= 2;
  float* b = (float*)calloc((size_t)P, sizeof(float));
  if (!b) return NAN;
  for (int32_t i = 0; i < n; ++i) b[i] = v[i];
  for (int32_t s = P / 2; s >= 1; s /= 2)
    for (int32_t i = 0; i < s; ++i) b[i] = b[i] + b[i + s];
  float r = b[0];
  free(b);
  return r;
}

/* Descending order of experts by logit, equal logits by lower index first: the one
 * total order used wherever the paper orders scores: the descending order statistics,
 * the highest-scoring pool members, the score tie-break of the load sort (Method;
 * Algorithm 1).  Softmax is monotone, so ordering logits
 * orders scores, without merging scores that round to the same value. */
static void order_desc_f32(const float* z, int32_t E, int32_t* ord) {
  for (int32_t i = 0; i < E; ++i) ord[i] = i;
  for (int32_t i = 1; i < E; ++i) {            /* insertion sort, stable */
    int32_t x = ord[i];
    int32_t j = i - 1;
    while (j >= 0 && z[ord[j]] < z[x]) { ord[j + 1] = ord[j]; --j; }
    ord[j + 1] = x;
  }
}

static void order_desc_f64(const double* z, int32_t E, int32_t* ord) {
  for (int32_t i = 0; i < E; ++i) ord[i] = i;
  for (int32_t i = 1; i < E; ++i) {
    int32_t x = ord[i];
    int32_t j = i - 1;
    while (j >= 0 && z[ord[j]] < z[x]) { ord[j + 1] = ord[j]; --j; }
    ord[j + 1] = x;
  }
}

/* The stable sort of the working set by load (Algorithm 1, final assignment; Method:
 * Final assignment): primary key ascending load, ties by position in the
 * score-descending candidate list; returns the first k in `chosen` as positions
 * into cand[], then re-listed in score order (the output lists A by descending
 * score). */
static void pick_least_loaded(const int32_t* cand, int32_t cstar, int32_t k,
                              const int64_t* L, int32_t* chosen_pos) {
  int32_t pos[256];
  for (int32_t i = 0; i < cstar; ++i) pos[i] = i;
  for (int32_t i = 1; i < cstar; ++i) {        /* stable insertion sort by load */
    int32_t x = pos[i];
    int32_t j = i - 1;
    while (j >= 0 && L[cand[pos[j]]] > L[cand[x]]) { pos[j + 1] = pos[j]; --j; }
    pos[j + 1] = x;
  }
  for (int32_t i = 0; i < k; ++i) chosen_pos[i] = pos[i];
  for (int32_t i = 1; i < k; ++i) {            /* back to score order */
    int32_t x = chosen_pos[i];
    int32_t j = i - 1;
    while (j >= 0 && chosen_pos[j] > x) { chosen_pos[j + 1] = chosen_pos[j]; --j; }
    chosen_pos[j + 1] = x;
  }
}

/* Dispatch tables from the final assignment (the paper only says tokens are then
 * routed to experts by an all-to-all; this is the index structure that move
 * needs): counts per expert, exclusive prefix sums, and the flat assignment slots
 * t*k+j listed expert by expert, ascending slot order inside an expert. */
static void build_dispatch(const int32_t* ids, int32_t T, int32_t k, int32_t E,
                           int32_t* permutation, int32_t* offsets) {
  int64_t n = (int64_t)T * k;
  int32_t pos = 0;
  for (int32_t e = 0; e < E; ++e) {
    offsets[e] = pos;
    for (int64_t s = 0; s < n; ++s)
      if (ids[s] == e) permutation[pos++] = (int32_t)s;
  }
  offsets[E] = pos;
}

static int check_args(int32_t T, int32_t E, int32_t k, int32_t c, double eps, double tfix) {
  if (T < 0 || E < 1 || E > 256 || k < 1 || c < k || c > E) return ORACLE_E_ARG;
  if (!(eps > 0.0) || !(tfix > 0.0) || tfix > 1.0) return ORACLE_E_ARG;
  if ((int64_t)T * k > 0x7fffffff) return ORACLE_E_ARG;
  return ORACLE_OK;
}

/* ------------------------------------------------- the router, binary32 ---- */

/* logits [T,E] fp32.  Outputs: expert_ids [T,k] (score-descending inside a
 * token), weights [T,k] fp64, loads_out [E], permutation [T*k], offsets [E+1];
 * optional diagnostics expanded [T] (1 = took the load-aware branch) and
 * cstar [T] (size of the working set; k on the top-k branch).
 *
 * Decision arithmetic, all binary32, round-to-nearest-even, no contraction:
 *   d_i = z_i - z_(1);  p_i = exp_canon(max(d_i, -80));  Z = tree_sum(p);
 *   S_k = ((p_(1) + p_(2)) + ...) + p_(k);
 *   top-k branch  <=>  S_k >= fl(eps_high * Z)          [M_k >= eps_high]
 *   pool member   <=>  d_i >= fl32(ln t_fix)            [s_i >= t_fix * s_(1)]
 * The pool test is monotone in the ordering, so the pool is a prefix of it and
 * "the c* highest-scoring members" are the first c* of the ordering. */
int laser_oracle_route(const float* logits, int32_t T, int32_t E, int32_t k, int32_t c,
                       float eps_high, float t_fix, int32_t renormalize,
                       const int32_t* loads_in, int32_t* loads_out,
                       int32_t* expert_ids, double* weights,
                       int32_t* permutation, int32_t* offsets,
                       uint8_t* expanded, int32_t* cstar_out) {
  int rc = check_args(T, E, k, c, eps_high, t_fix);
  if (rc) return rc;
  const float tau_ln = (float)log((double)t_fix);
  int64_t L[256];
  int32_t ord[256], chosen[256];
  float d[256], p[256];
  for (int32_t e = 0; e < E; ++e) L[e] = loads_in[e];

  for (int32_t t = 0; t < T; ++t) {
    const float* z = logits + (size_t)t * E;
    order_desc_f32(z, E, ord);
    const float zmax = z[ord[0]];
    for (int32_t i = 0; i < E; ++i) {
      d[i] = z[i] - zmax;
      p[i] = laser_oracle_exp(d[i] < -80.0f ? -80.0f : d[i]);
    }
    const float Z = laser_oracle_tree_sum(p, E);
    float Sk = p[ord[0]];
    for (int32_t i = 1; i < k; ++i) Sk = Sk + p[ord[i]];

    int32_t cstar = k;
    int took_branch = 0;
    if (Sk >= eps_high * Z) {
      for (int32_t i = 0; i < k; ++i) chosen[i] = i;          /* A = top-k */
    } else {
      took_branch = 1;
      int32_t in_pool = 0;
      for (int32_t i = 0; i < E; ++i) in_pool += (d[i] >= tau_ln);
      int32_t m = in_pool > k ? in_pool : k;                   /* pool union top-k */
      cstar = c < m ? c : m;
      pick_least_loaded(ord, cstar, k, L, chosen);             /* Cand = ord[0..c*) */
    }

    /* weights: in fp64 from the same logits (the GPU's are checked to tolerance) */
    double denom = 0.0;
    if (renormalize) {
      for (int32_t i = 0; i < k; ++i) denom += exp((double)z[ord[chosen[i]]] - (double)zmax);
    } else {
      for (int32_t i = 0; i < E; ++i) denom += exp((double)z[i] - (double)zmax);
    }
    for (int32_t i = 0; i < k; ++i) {
      int32_t e = ord[chosen[i]];
      expert_ids[(size_t)t * k + i] = e;
      weights[(size_t)t * k + i] = exp((double)z[e] - (double)zmax) / denom;
    }
    for (int32_t i = 0; i < k; ++i) L[ord[chosen[i]]] += 1;    /* load update */
    if (expanded) expanded[t] = (uint8_t)took_branch;
    if (cstar_out) cstar_out[t] = cstar;
  }
  for (int32_t e = 0; e < E; ++e) loads_out[e] = (int32_t)L[e];
  build_dispatch(expert_ids, T, k, E, permutation, offsets);
  return ORACLE_OK;
}

/* ------------------------------------------------- randomized trimming ------ */

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
 * 1, 2, 3", SC 2011): a counter-based generator, 128-bit counter, 64-bit key, ten
 * rounds of two 32x32->64 multiplications; the key is bumped by the Weyl constants
 * after every round. */
void laser_oracle_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform sample of c pool members, drawn without replacement (Algorithm 1,
 * mode RANDOM), made reproducible: the pool is the first m positions of the score
 * order; a partial Fisher-Yates shuffle of [0, m) takes, for draw i = 0..c-1, the
 * i-th 32-bit word r_i of the Philox stream with key = seed and counter =
 * (token index low, token index high, stream, i / 4), and swaps position i with
 * position i + floor(r_i * (m - i) / 2^32).  The first c positions, listed in
 * ascending order, are the sample.  Needs c < m <= 256. */
void laser_oracle_sample_ranks(int32_t m, int32_t c, uint64_t seed, uint32_t stream,
                               uint64_t token, int32_t* ranks_out) {
  int32_t arr[256];
  uint32_t words[4];
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  for (int32_t i = 0; i < m; ++i) arr[i] = i;
  for (int32_t i = 0; i < c; ++i) {
    if ((i & 3) == 0) {
      const uint32_t ctr[4] = {(uint32_t)token, (uint32_t)(token >> 32), stream, (uint32_t)(i >> 2)};
      laser_oracle_philox4x32(ctr, key, words);
    }
    const int32_t j = i + (int32_t)(((uint64_t)words[i & 3] * (uint64_t)(m - i)) >> 32);
    const int32_t tmp = arr[i]; arr[i] = arr[j]; arr[j] = tmp;
  }
  for (int32_t i = 1; i < c; ++i) {            /* ascending */
    int32_t x = arr[i];
    int32_t j = i - 1;
    while (j >= 0 && arr[j] > x) { arr[j + 1] = arr[j]; --j; }
    arr[j + 1] = x;
  }
  for (int32_t i = 0; i < c; ++i) ranks_out[i] = arr[i];
}

/* Algorithm 1 with mode RANDOM: as laser_oracle_route, except that a pool larger
 * than c is trimmed to a uniform sample of c of its members (positions in the score
 * order from laser_oracle_sample_ranks, token index = token_offset + t) instead of
 * its c best.  The sampled candidates are listed in score order, so the score
 * tie-break of the load sort and the output order are as before.  The top-k experts need not
 * be in the sample. */
int laser_oracle_route_random(const float* logits, int32_t T, int32_t E, int32_t k, int32_t c,
                              float eps_high, float t_fix, int32_t renormalize,
                              uint64_t seed, uint32_t stream, uint64_t token_offset,
                              const int32_t* loads_in, int32_t* loads_out,
                              int32_t* expert_ids, double* weights,
                              int32_t* permutation, int32_t* offsets,
                              uint8_t* expanded, int32_t* cstar_out) {
  int rc = check_args(T, E, k, c, eps_high, t_fix);
  if (rc) return rc;
  const float tau_ln = (float)log((double)t_fix);
  int64_t L[256];
  int32_t ord[256], chosen[256], ranks[256], cand[256];
  float d[256], p[256];
  for (int32_t e = 0; e < E; ++e) L[e] = loads_in[e];

  for (int32_t t = 0; t < T; ++t) {
    const float* z = logits + (size_t)t * E;
    order_desc_f32(z, E, ord);
    const float zmax = z[ord[0]];
    for (int32_t i = 0; i < E; ++i) {
      d[i] = z[i] - zmax;
      p[i] = laser_oracle_exp(d[i] < -80.0f ? -80.0f : d[i]);
    }
    const float Z = laser_oracle_tree_sum(p, E);
    float Sk = p[ord[0]];
    for (int32_t i = 1; i < k; ++i) Sk = Sk + p[ord[i]];

    int32_t cstar = k;
    int took_branch = 0;
    if (Sk >= eps_high * Z) {
      for (int32_t i = 0; i < k; ++i) cand[i] = ord[i];        /* A = top-k */
      for (int32_t i = 0; i < k; ++i) chosen[i] = i;
    } else {
      took_branch = 1;
      int32_t in_pool = 0;
      for (int32_t i = 0; i < E; ++i) in_pool += (d[i] >= tau_ln);
      int32_t m = in_pool > k ? in_pool : k;
      cstar = c < m ? c : m;
      if (m > c) laser_oracle_sample_ranks(m, c, seed, stream, token_offset + (uint64_t)t, ranks);
      else for (int32_t i = 0; i < cstar; ++i) ranks[i] = i;
      for (int32_t i = 0; i < cstar; ++i) cand[i] = ord[ranks[i]];
      pick_least_loaded(cand, cstar, k, L, chosen);
    }

    double denom = 0.0;
    if (renormalize) {
      for (int32_t i = 0; i < k; ++i) denom += exp((double)z[cand[chosen[i]]] - (double)zmax);
    } else {
      for (int32_t i = 0; i < E; ++i) denom += exp((double)z[i] - (double)zmax);
    }
    for (int32_t i = 0; i < k; ++i) {
      int32_t e = cand[chosen[i]];
      expert_ids[(size_t)t * k + i] = e;
      weights[(size_t)t * k + i] = exp((double)z[e] - (double)zmax) / denom;
    }
    for (int32_t i = 0; i < k; ++i) L[cand[chosen[i]]] += 1;
    if (expanded) expanded[t] = (uint8_t)took_branch;
    if (cstar_out) cstar_out[t] = cstar;
  }
  for (int32_t e = 0; e < E; ++e) loads_out[e] = (int32_t)L[e];
  build_dispatch(expert_ids, T, k, E, permutation, offsets);
  return ORACLE_OK;
}

/* ------------------------------------------------ per-token gate statistics -- */

/* The statistics the paper reads off the gate scores to choose the thresholds
 * (Layer Variability in Gate Score Distributions; Parameter setting and layer-wise
 * choices), per token, from fp32 logits:
 *   topk_mass  M_k = sum of the k largest softmax scores          (fp64)
 *   entropy    H = - sum_i s_i ln s_i, natural logarithm           (fp64)
 *   pool_size  m = | {i : s_i >= t_fix * s_(1)} union top-k |      (integer)
 * The integer is decided exactly as the router decides pool membership (binary32,
 * d_i >= fl32(ln t_fix)), so that min(c, m) is the router's working-set size. */
int laser_oracle_token_stats(const float* logits, int32_t T, int32_t E, int32_t k, float t_fix,
                             double* topk_mass, double* entropy, int32_t* pool_size) {
  if (!logits && T > 0) return ORACLE_E_ARG;
  if (T < 0 || E < 1 || E > 256 || k < 1 || k > E) return ORACLE_E_ARG;
  if (!(t_fix > 0.0f) || !(t_fix <= 1.0f)) return ORACLE_E_ARG;
  const float tau_ln = (float)log((double)t_fix);
  int32_t ord[256];
  for (int32_t t = 0; t < T; ++t) {
    const float* z = logits + (size_t)t * E;
    order_desc_f32(z, E, ord);
    const double zmax = (double)z[ord[0]];
    double Z = 0.0;
    for (int32_t i = 0; i < E; ++i) Z += exp((double)z[i] - zmax);
    double mk = 0.0, h = 0.0;
    for (int32_t i = 0; i < k; ++i) mk += exp((double)z[ord[i]] - zmax) / Z;
    for (int32_t i = 0; i < E; ++i) {
      const double s = exp((double)z[i] - zmax) / Z;
      if (s > 0.0) h -= s * log(s);
    }
    int32_t in_pool = 0;
    for (int32_t i = 0; i < E; ++i) in_pool += ((z[i] - z[ord[0]]) >= tau_ln);
    if (topk_mass) topk_mass[t] = mk;
    if (entropy) entropy[t] = h;
    if (pool_size) pool_size[t] = in_pool > k ? in_pool : k;
  }
  return ORACLE_OK;
}

/* ------------------------------------------------------- imbalance metrics -- */

/* Expert- and GPU-level imbalance of per-layer assignment counts (Problem statement:
 * the imbalance factor I, its aggregate over layers, and the GPU-level version under
 * a placement matrix; Evaluation / Metrics: max violation).
 *   counts     [L,E] tokens assigned to expert e in layer l
 *   placement  [G,E] share of expert e served by GPU g (columns sum to 1), or NULL
 *   weights    [L] layer weights w_l, or NULL for 1/L
 *   I[l]       max_e N / mean_e N          MV[l] = I[l] - 1 (excess of the most loaded
 *   Igpu[l]    max_g N_g / mean_g N_g      expert over the average, relative)
 *   agg[0] = sum_l w_l I[l],  agg[1] = sum_l w_l Igpu[l]
 * A layer without assignments has I = Igpu = 1 (nothing is unbalanced). */
int laser_oracle_imbalance(const int32_t* counts, int32_t L, int32_t E, const double* placement,
                           int32_t G, const double* weights, double* I, double* MV, double* Igpu,
                           double* agg) {
  if (L < 0 || E < 1 || (placement && G < 1)) return ORACLE_E_ARG;
  double a0 = 0.0, a1 = 0.0;
  for (int32_t l = 0; l < L; ++l) {
    const int32_t* n = counts + (size_t)l * E;
    double mx = 0.0, sum = 0.0;
    for (int32_t e = 0; e < E; ++e) {
      sum += (double)n[e];
      if ((double)n[e] > mx) mx = (double)n[e];
    }
    const double il = sum > 0.0 ? mx / (sum / E) : 1.0;
    double ig = 1.0;
    if (placement) {
      double gmx = 0.0, gsum = 0.0;
      for (int32_t g = 0; g < G; ++g) {
        double ng = 0.0;
        for (int32_t e = 0; e < E; ++e) ng += placement[(size_t)g * E + e] * (double)n[e];
        gsum += ng;
        if (ng > gmx) gmx = ng;
      }
      ig = gsum > 0.0 ? gmx / (gsum / G) : 1.0;
    }
    const double w = weights ? weights[l] : 1.0 / L;
    if (I) I[l] = il;
    if (MV) MV[l] = il - 1.0;
    if (Igpu) Igpu[l] = ig;
    a0 += w * il;
    a1 += w * ig;
  }
  if (agg) {
    agg[0] = a0;
    agg[1] = a1;
  }
  return ORACLE_OK;
}

/* Percentiles of n values (Evaluation, Metrics: I_agg is summarised by its 50th and
 * 95th percentile across batches).  The paper does not say how a percentile that falls
 * between two batches is read; the reading here is the common one: sort ascending, the
 * q-th percentile sits at position h = (n - 1) q / 100 of the sorted list and is
 * interpolated linearly between the two neighbours, x[lo] + (h - lo)(x[lo+1] - x[lo]).
 * P50 of an odd number of values is the middle one, P0 the smallest, P100 the largest. */
int laser_oracle_percentiles(const double* values, int32_t n, const double* q, int32_t nq,
                             double* out) {
  if (n < 1 || nq < 0) return ORACLE_E_ARG;
  double* x = (double*)malloc((size_t)n * sizeof(double));
  if (!x) return ORACLE_E_ARG;
  for (int32_t i = 0; i < n; ++i) x[i] = values[i];
  for (int32_t i = 1; i < n; ++i) { /* insertion sort */
    const double v = x[i];
    int32_t j = i - 1;
    while (j >= 0 && x[j] > v) {
      x[j + 1] = x[j];
      --j;
    }
    x[j + 1] = v;
  }
  for (int32_t i = 0; i < nq; ++i) {
    if (!(q[i] >= 0.0 && q[i] <= 100.0)) {
      free(x);
      return ORACLE_E_ARG;
    }
    const double h = (double)(n - 1) * q[i] / 100.0;
    int32_t lo = (int32_t)h; /* h >= 0: truncation is the floor */
    if (lo > n - 1) lo = n - 1;
    const int32_t hi = lo + 1 < n ? lo + 1 : lo;
    out[i] = x[lo] + (h - (double)lo) * (x[hi] - x[lo]);
  }
  free(x);
  return ORACLE_OK;
}

/* ------------------------------------------------- the router, literal fp64 -- */

/* Same interface on fp64 logits, formulas as printed: s = softmax(z) with libm
 * exp, M_k = sum of the k largest s, M_k >= eps_high, t = t_fix * s_(1),
 * pool = {s_i >= t} union top-k, Cand = c* largest, stable sort by load. */
int laser_oracle_route_literal(const double* logits, int32_t T, int32_t E, int32_t k,
                               int32_t c, double eps_high, double t_fix,
                               int32_t renormalize, const int32_t* loads_in,
                               int32_t* loads_out, int32_t* expert_ids, double* weights,
                               int32_t* permutation, int32_t* offsets,
                               uint8_t* expanded, int32_t* cstar_out) {
  int rc = check_args(T, E, k, c, eps_high, t_fix);
  if (rc) return rc;
  int64_t L[256];
  int32_t ord[256], chosen[256], cand[256];
  double s[256];
  for (int32_t e = 0; e < E; ++e) L[e] = loads_in[e];

  for (int32_t t = 0; t < T; ++t) {
    const double* z = logits + (size_t)t * E;
    order_desc_f64(z, E, ord);
    double sum = 0.0;
    for (int32_t i = 0; i < E; ++i) { s[i] = exp(z[i] - z[ord[0]]); sum += s[i]; }
    for (int32_t i = 0; i < E; ++i) s[i] /= sum;

    double Mk = 0.0;
    for (int32_t i = 0; i < k; ++i) Mk += s[ord[i]];

    int32_t cstar = k;
    int took_branch = 0;
    if (Mk >= eps_high) {
      for (int32_t i = 0; i < k; ++i) chosen[i] = i;
      for (int32_t i = 0; i < k; ++i) cand[i] = ord[i];
    } else {
      took_branch = 1;
      const double cut = t_fix * s[ord[0]];
      /* pool, kept in score order: members are those with s_i >= cut, plus the
       * top-k; walk the ordering and keep what qualifies */
      int32_t m = 0;
      for (int32_t r = 0; r < E; ++r) {
        int32_t i = ord[r];
        if (s[i] >= cut || r < k) cand[m++] = i;
      }
      cstar = c < m ? c : m;                                   /* keep c* largest */
      pick_least_loaded(cand, cstar, k, L, chosen);
    }
    double denom = 0.0;
    if (renormalize) for (int32_t i = 0; i < k; ++i) denom += s[cand[chosen[i]]];
    else denom = 1.0;
    for (int32_t i = 0; i < k; ++i) {
      int32_t e = cand[chosen[i]];
      expert_ids[(size_t)t * k + i] = e;
      weights[(size_t)t * k + i] = s[e] / denom;
    }
    for (int32_t i = 0; i < k; ++i) L[cand[chosen[i]]] += 1;
    if (expanded) expanded[t] = (uint8_t)took_branch;
    if (cstar_out) cstar_out[t] = cstar;
  }
  for (int32_t e = 0; e < E; ++e) loads_out[e] = (int32_t)L[e];
  build_dispatch(expert_ids, T, k, E, permutation, offsets);
  return ORACLE_OK;
}
