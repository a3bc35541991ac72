/*
 * Drives every entry point of the CPU oracle (oracle/laser_oracle.c) on small inputs,
 * for a build with -fsanitize=address,undefined: the point is that the run ends clean
 * (no out-of-bounds access, no undefined operation), not what it computes.  Inputs: the
 * hand-worked cases given on the command line as a text file (one case per line:
 * E k c eps t_fix T, then E loads, T*E scores, T*k expected experts), and seeded
 * pseudo-random shapes that include the extremes the arguments allow (one expert,
 * k = E, the largest E, no tokens).  Returns 0 when every call succeeded and the hand
 * cases came out as expected.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int laser_oracle_gate(const void*, const void*, int32_t, int32_t, int32_t, int32_t, double*);
float laser_oracle_exp(float);
float laser_oracle_tree_sum(const float*, int32_t);
int laser_oracle_route(const float*, int32_t, int32_t, int32_t, int32_t, float, float, int32_t,
                       const int32_t*, int32_t*, int32_t*, double*, int32_t*, int32_t*, uint8_t*, int32_t*);
int laser_oracle_route_literal(const double*, int32_t, int32_t, int32_t, int32_t, double, double, int32_t,
                               const int32_t*, int32_t*, int32_t*, double*, int32_t*, int32_t*, uint8_t*,
                               int32_t*);
void laser_oracle_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void laser_oracle_sample_ranks(int32_t, int32_t, uint64_t, uint32_t, uint64_t, int32_t*);
int laser_oracle_route_random(const float*, int32_t, int32_t, int32_t, int32_t, float, float, int32_t, uint64_t,
                              uint32_t, uint64_t, const int32_t*, int32_t*, int32_t*, double*, int32_t*,
                              int32_t*, uint8_t*, int32_t*);
int laser_oracle_token_stats(const float*, int32_t, int32_t, int32_t, float, double*, double*, int32_t*);
int laser_oracle_imbalance(const int32_t*, int32_t, int32_t, const double*, int32_t, const double*, double*,
                           double*, double*, double*);
int laser_oracle_percentiles(const double*, int32_t, const double*, int32_t, double*);

static uint64_t rng_state = 88172645463325252ull;
static double uniform(void) { /* xorshift64, in [0, 1) */
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / 9007199254740992.0;
}

/* exact-size allocations, so that an access one past the end is caught */
static void* take(size_t n) {
  void* p = malloc(n ? n : 1);
  if (!p) exit(3);
  return p;
}

static int run_shape(int32_t T, int32_t E, int32_t k, int32_t c, float eps, float tfix, int ties) {
  float* z = take((size_t)T * E * sizeof(float));
  double* zd = take((size_t)T * E * sizeof(double));
  for (size_t i = 0; i < (size_t)T * E; ++i) {
    double v = ties ? floor(uniform() * 3.0) * 0.25 : (uniform() - 0.5) * 4.0;
    z[i] = (float)v;
    zd[i] = (double)z[i];
  }
  int32_t* lin = take((size_t)E * sizeof(int32_t));
  for (int32_t e = 0; e < E; ++e) lin[e] = (int32_t)(uniform() * 5.0);
  int32_t* lout = take((size_t)E * sizeof(int32_t));
  int32_t* ids = take((size_t)T * k * sizeof(int32_t));
  double* wts = take((size_t)T * k * sizeof(double));
  int32_t* perm = take((size_t)T * k * sizeof(int32_t));
  int32_t* offs = take((size_t)(E + 1) * sizeof(int32_t));
  uint8_t* expd = take((size_t)T);
  int32_t* cst = take((size_t)T * sizeof(int32_t));
  int bad = 0;
  for (int renorm = 0; renorm < 2; ++renorm) {
    bad |= laser_oracle_route(z, T, E, k, c, eps, tfix, renorm, lin, lout, ids, wts, perm, offs, expd, cst);
    long sum = 0;
    for (int32_t e = 0; e < E; ++e) sum += lout[e] - lin[e];
    bad |= sum != (long)T * k || offs[E] != T * k;
    bad |= laser_oracle_route_literal(zd, T, E, k, c, eps, tfix, renorm, lin, lout, ids, wts, perm, offs, expd, cst);
    bad |= laser_oracle_route_random(z, T, E, k, c, eps, tfix, renorm, 0x123456789abcdefull, 7u,
                                     0xfffffffffffffff0ull, lin, lout, ids, wts, perm, offs, expd, cst);
  }
  double* mass = take((size_t)T * sizeof(double));
  double* ent = take((size_t)T * sizeof(double));
  int32_t* pool = take((size_t)T * sizeof(int32_t));
  bad |= laser_oracle_token_stats(z, T, E, k, tfix, mass, ent, pool);
  free(z); free(zd); free(lin); free(lout); free(ids); free(wts); free(perm); free(offs); free(expd);
  free(cst); free(mass); free(ent); free(pool);
  return bad;
}

static int run_hand_cases(const char* path) {
  FILE* f = fopen(path, "r");
  if (!f) return 1;
  int bad = 0, n = 0;
  int32_t E, k, c, T;
  double eps, tfix;
  while (fscanf(f, "%d %d %d %lf %lf %d", &E, &k, &c, &eps, &tfix, &T) == 6) {
    int32_t* lin = take((size_t)E * sizeof(int32_t));
    float* z = take((size_t)T * E * sizeof(float));
    int32_t* want = take((size_t)T * k * sizeof(int32_t));
    for (int32_t e = 0; e < E; ++e) bad |= fscanf(f, "%d", &lin[e]) != 1;
    for (int32_t i = 0; i < T * E; ++i) {
      double p;
      bad |= fscanf(f, "%lf", &p) != 1;
      z[i] = (float)log(p);
    }
    for (int32_t i = 0; i < T * k; ++i) bad |= fscanf(f, "%d", &want[i]) != 1;
    int32_t* lout = take((size_t)E * sizeof(int32_t));
    int32_t* ids = take((size_t)T * k * sizeof(int32_t));
    double* wts = take((size_t)T * k * sizeof(double));
    int32_t* perm = take((size_t)T * k * sizeof(int32_t));
    int32_t* offs = take((size_t)(E + 1) * sizeof(int32_t));
    bad |= laser_oracle_route(z, T, E, k, c, (float)eps, (float)tfix, 1, lin, lout, ids, wts, perm, offs, NULL, NULL);
    for (int32_t i = 0; i < T * k; ++i) bad |= ids[i] != want[i];
    free(lin); free(z); free(want); free(lout); free(ids); free(wts); free(perm); free(offs);
    ++n;
  }
  fclose(f);
  return bad || n == 0;
}

int main(int argc, char** argv) {
  int bad = 0;
  if (argc > 1) bad |= run_hand_cases(argv[1]);
  /* T, E, k, c */
  static const int32_t shapes[][4] = {{0, 4, 2, 3},    {1, 1, 1, 1},     {7, 2, 2, 2},     {33, 8, 2, 4},
                                      {50, 64, 6, 8},  {40, 64, 6, 64},  {9, 256, 8, 16},  {5, 256, 256, 256},
                                      {6, 256, 1, 256}, {65, 33, 4, 33}, {20, 5, 5, 5},    {300, 8, 2, 8}};
  for (size_t i = 0; i < sizeof shapes / sizeof shapes[0]; ++i) {
    const int32_t* s = shapes[i];
    bad |= run_shape(s[0], s[1], s[2], s[3], 2.0f, 1e-30f, 0);
    bad |= run_shape(s[0], s[1], s[2], s[3], 0.6f, 0.5f, 0);
    bad |= run_shape(s[0], s[1], s[2], s[3], 0.9f, 1.0f, 1);
  }
  /* gate: both storage types, ragged sizes */
  {
    const int32_t T = 5, H = 37, E = 3;
    float* h = take((size_t)T * H * sizeof(float));
    float* w = take((size_t)E * H * sizeof(float));
    uint16_t* hb = take((size_t)T * H * sizeof(uint16_t));
    uint16_t* wb = take((size_t)E * H * sizeof(uint16_t));
    double* out = take((size_t)T * E * sizeof(double));
    for (int i = 0; i < T * H; ++i) { h[i] = (float)(uniform() - 0.5); hb[i] = (uint16_t)(0x3f00 + (int)(uniform() * 255)); }
    for (int i = 0; i < E * H; ++i) { w[i] = (float)(uniform() - 0.5); wb[i] = (uint16_t)(0xbf00 + (int)(uniform() * 255)); }
    bad |= laser_oracle_gate(h, w, T, H, E, 0, out);
    bad |= laser_oracle_gate(hb, wb, T, H, E, 1, out);
    bad |= laser_oracle_gate(h, w, 0, H, E, 0, out);
    free(h); free(w); free(hb); free(wb); free(out);
  }
  /* the scalar helpers, the generator, the sampler at its extremes */
  {
    float v[256];
    for (int i = 0; i < 256; ++i) v[i] = laser_oracle_exp(-80.0f * (float)i / 255.0f);
    for (int n = 1; n <= 256; n += 17) bad |= !(laser_oracle_tree_sum(v, n) > 0.0f);
    bad |= laser_oracle_exp(0.0f) != 1.0f;
    const uint32_t ctr[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}, key[2] = {0xffffffffu, 0xffffffffu};
    uint32_t out[4];
    laser_oracle_philox4x32(ctr, key, out);
    int32_t ranks[255];
    laser_oracle_sample_ranks(256, 255, ~0ull, ~0u, ~0ull, ranks);
    laser_oracle_sample_ranks(2, 1, 0, 0, 0, ranks);
    for (int i = 0; i < 1; ++i) bad |= ranks[i] < 0 || ranks[i] > 1;
  }
  /* metrics */
  {
    const int32_t L = 3, E = 5, G = 2;
    int32_t counts[15];
    double placement[10], weights[3] = {0.5, 0.25, 0.25}, I[3], MV[3], Ig[3], agg[2];
    for (int i = 0; i < 15; ++i) counts[i] = i < 5 ? 0 : (int32_t)(uniform() * 100.0);
    for (int e = 0; e < E; ++e) { placement[e] = e % 2; placement[E + e] = 1 - e % 2; }
    bad |= laser_oracle_imbalance(counts, L, E, placement, G, weights, I, MV, Ig, agg);
    bad |= laser_oracle_imbalance(counts, L, E, NULL, 0, NULL, I, MV, Ig, agg);
    bad |= laser_oracle_imbalance(counts, 0, E, NULL, 0, NULL, I, MV, Ig, agg);
    double vals[7] = {3, 1, 4, 1, 5, 9, 2}, q[4] = {0, 50, 95, 100}, out[4];
    bad |= laser_oracle_percentiles(vals, 7, q, 4, out);
    bad |= laser_oracle_percentiles(vals, 1, q, 4, out);
    bad |= out[0] != 3.0;
  }
  printf("%s\n", bad ? "FAILED" : "clean");
  return bad ? 1 : 0;
}
