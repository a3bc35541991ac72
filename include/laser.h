/*
 * laser.h -- C ABI of the MI355X (gfx950) LASER routing library.
 *
 * One call routes the T tokens of one MoE layer: gate projection of the hidden
 * states to expert logits, softmax scores, the top-k-mass test that either keeps
 * the k strongest experts or widens to a thresholded candidate set, selection of
 * the k least-loaded candidates against running per-expert load counters that
 * advance after every token, and the token-to-expert dispatch tables.
 * (Paper: section "The Method" -- Problem Formulation, Expansion rule, Final
 * assignment; appendix "Pseudo Code", Algorithm 1 "per token, per layer".)
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless marked host.  The caller
 *     allocates and owns all buffers, including the workspace.  The library
 *     allocates nothing, frees nothing, never synchronises and never prints:
 *     all work is enqueued on `hip_stream` (a hipStream_t, NULL = default
 *     stream) and the call returns at once.  The one exception is laser_status(),
 *     a query that waits for the stream.  (The library's code object holds two
 *     arrays of device memory of its own, there on every GPU from the moment it is
 *     loaded: the workspace of laser_route_static and 256 KiB of counters that
 *     small calls use, see split_k.)
 *   - Return value: LASER_OK (0) or a negative LASER_E_* code.  Arguments are
 *     validated on the host before anything is enqueued; on error nothing was
 *     enqueued and no buffer was touched.  laser_strerror() names a code.
 *   - Tokens are routed in row order 0..T-1; the load counters a token sees are
 *     loads_inout as passed in plus one per expert for every earlier token that
 *     was assigned to it (both branches of the expansion rule count).
 *   - Scores are ordered by logit, equal logits by lower expert index first.
 *     That one order decides top-k membership, trimming to c, the score tie-break
 *     of the load sort, and the order in which a token's k experts are listed.
 *   - A workspace belongs to one call at a time: calls that share a workspace (or any
 *     output buffer) must be ordered, e.g. by being enqueued on one stream.  Calls with
 *     their own workspaces and outputs may run side by side on different streams.
 *   - Inputs must be finite; loads_inout[e] + T must stay below 2^27.
 *   - Limits: 1 <= k <= min(c, 16); c <= E <= 64; bf16 needs H % 8 == 0 and
 *     16-byte aligned hidden / w_gate; fp32 needs H % 4 == 0.  Trimming sizes
 *     c <= 16 (the paper evaluates c <= 10) run on the tuned kernels; 16 < c <= E
 *     (up to the load-only baseline of the paper's evaluation, c = n) is routed
 *     exactly by general kernels that are not tuned.
 *   - Completion.  The kernels of a call hand data to one another through the
 *     workspace; the workgroups that write the dispatch tables wait for the
 *     workgroup that walks the load-dependent tokens with a bounded number of
 *     polls (laser_params_t.poll_budget) and, should that bound ever run out, leave
 *     without writing: the call's outputs are then incomplete.  This is recorded
 *     in the workspace and reported by laser_status(); it does not happen while
 *     the GPU makes progress on the call's own kernels.
 */
#ifndef LASER_H_
#define LASER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LASER_OK 0
#define LASER_E_NULL (-1)        /* a required pointer is NULL                    */
#define LASER_E_RANGE (-2)       /* T, H, E, k, c, eps_high or t_fix out of range */
#define LASER_E_ALIGN (-3)       /* row length or pointer alignment not supported */
#define LASER_E_WORKSPACE (-4)   /* workspace smaller than laser_workspace_bytes  */
#define LASER_E_UNSUPPORTED (-5) /* E or c above the built limit                  */
#define LASER_E_STRUCT (-6)      /* params->struct_bytes does not match           */
#define LASER_E_LAUNCH (-7)      /* the HIP runtime refused a kernel launch       */

#define LASER_DTYPE_F32 0
#define LASER_DTYPE_BF16 1

#define LASER_TRIM_TOP 0    /* keep the c highest-scoring pool members (built)       */
#define LASER_TRIM_RANDOM 1 /* uniform sample of c pool members, see laser_params_t  */

#define LASER_MAX_E 64
#define LASER_MAX_K 16
#define LASER_MAX_C 64      /* (c <= E) */
#define LASER_FAST_C 16     /* trimming sizes up to here run on the tuned kernels */

/* What laser_status() reports about the last call that used a workspace. */
#define LASER_STATUS_COMPLETE 0
#define LASER_STATUS_TIMEOUT 1       /* a bounded wait ran out: outputs incomplete      */
#define LASER_STATUS_INCONSISTENT 2  /* a dispatch slot fell outside the table (inputs  */
                                     /* overwritten while the call ran): outputs incomplete */

/* Parameters of Algorithm 1 plus the storage type of the gate operands. */
typedef struct laser_params {
  uint32_t struct_bytes; /* = sizeof(laser_params_t)                                */
  int32_t k;             /* experts per token                                       */
  int32_t c;             /* trimming size, k <= c <= E                              */
  float eps_high;        /* top-k mass threshold; > 0.  The paper uses (0,1); a     */
                         /* value above 1 sends every token to the load-aware branch */
  float t_fix;           /* pool cut-off relative to the best score, in (0, 1]      */
  int32_t trim_mode;     /* LASER_TRIM_*                                            */
  int32_t renormalize;   /* 1: weights sum to 1 over the k chosen; 0: raw scores    */
  int32_t dtype;         /* LASER_DTYPE_* of hidden and w_gate (laser_route only)   */
  /* LASER_TRIM_RANDOM only (Algorithm 1, mode RANDOM: the working set is a uniform
   * sample of the pool, drawn without replacement).  The sample of a token is a function of
   * (seed, stream, token_offset + t) alone: Philox4x32-10 with key = seed and counter
   * = (token index low, high, stream, block); a partial Fisher-Yates shuffle of the
   * pool's positions [0, m) in the score order swaps position i with
   * i + floor(r_i * (m - i) / 2^32), i = 0..c-1, r_i the i-th 32-bit word of the
   * token's stream; the first c positions are the candidates.  Pools of at most c
   * members are not sampled.  Ignored for LASER_TRIM_TOP. */
  uint64_t seed;         /* generator key                                           */
  uint64_t token_offset; /* caller's index of token 0 of this call (split calls)    */
  uint32_t stream;       /* caller's stream id, e.g. the layer                      */
  uint32_t poll_budget;  /* 0: the library sizes its bounded waits from T (millions of */
                         /* polls); otherwise the number of polls after which a waiting */
                         /* workgroup gives up (see "Completion" above)                 */
  uint32_t pipeline_tiles; /* Large bf16 calls of laser_route are pipelined: the walk over */
                         /* the load-dependent tokens of a segment of the batch (Algorithm */
                         /* 1 orders the tokens, so it needs nothing of later tokens) runs */
                         /* while the projection of the later segments still streams.      */
                         /* 0: the library decides (segments of about 32 K tokens for      */
                         /* batches of 96 K tokens or more); 1: never; n >= 2: segments of */
                         /* n tiles of 64 tokens whenever the batch has more tiles.  The   */
                         /* results do not depend on it.                                   */
  uint32_t split_k;      /* Small bf16 calls of laser_route (up to 4096 tokens): the        */
                         /* contraction axis of the projection is cut over eight workgroups */
                         /* per tile of 64 tokens (four beyond 2048 tokens).  0: the        */
                         /* library decides; 1: never.  The results, logits included, do    */
                         /* not depend on it.                                               */
} laser_params_t;

/* Bytes of device workspace a call with these sizes needs (0 on bad arguments).
 * H may be 0 when only laser_route_from_logits will be called.  A workspace of this size
 * for T tokens also serves every call with fewer tokens (and the same E and params): for
 * up to 4096 tokens the size includes 128 KiB per tile of 64 tokens that only the small-
 * call split (split_k) uses, and a call that finds less room runs without the split. */
size_t laser_workspace_bytes(int32_t T, int32_t H, int32_t E, const laser_params_t* params);

/*
 * The whole routing step of one layer (gate function + Algorithm 1 per token in
 * token order + dispatch tables).
 *   hidden         [T,H] row-major, dtype per params           in
 *   w_gate         [E,H] row-major (one row per expert)        in
 *   loads_inout    [E] int32: loads before token 0 / after token T-1
 *   expert_ids     [T,k] int32: the chosen experts, best score first      out
 *   weights        [T,k] fp32: combine weights of those experts           out
 *   permutation    [T*k] int32: flat assignment slots t*k+j grouped by    out
 *                  expert, ascending slot order inside an expert (the stable
 *                  counting sort of expert_ids)
 *   expert_offsets [E+1] int32: exclusive prefix sums of the per-expert   out
 *                  assignment counts; [E] = T*k
 *   logits_out     [T,E] fp32 gate logits, or NULL if not wanted          out
 *   workspace      >= laser_workspace_bytes(T,H,E,params) bytes, 256-byte aligned
 * T = 0 is valid (offsets are zeroed, loads untouched).
 */
int laser_route(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                float* weights, int32_t* permutation, int32_t* expert_offsets,
                float* logits_out, void* workspace, size_t workspace_bytes,
                void* hip_stream);

/*
 * B independent routing problems of one size in one call: the layers (or layer x
 * micro-batch pairs) whose inputs are all at hand.  Algorithm 1 orders the tokens of
 * ONE layer's batch (its counters start at that layer's loads); different layers and
 * batches share nothing, so their chains run side by side, one workgroup each, and the
 * projections share one launch.  Every array is that of laser_route with a leading
 * dimension B, problems stored back to back:
 *   hidden [B,T,H], w_gate [B,E,H], loads_inout [B,E], expert_ids and weights [B,T,k],
 *   permutation [B,T*k] (slot numbers t*k+j local to the problem), expert_offsets
 *   [B,E+1], logits_out [B,T,E] or NULL,
 *   workspace >= B * laser_workspace_bytes(T,H,E,params) bytes, 256-byte aligned.
 * Each problem's result is exactly laser_route's on its slices.  With
 * LASER_TRIM_RANDOM problem b draws with stream id params->stream + b.
 * 0 <= B <= 65535; B = 0 does nothing.
 */
int laser_route_batched(const void* hidden, const void* w_gate, int32_t B, int32_t T, int32_t H,
                        int32_t E, const laser_params_t* params, int32_t* loads_inout,
                        int32_t* expert_ids, float* weights, int32_t* permutation,
                        int32_t* expert_offsets, float* logits_out, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/*
 * The same step starting after the gate function, from given fp32 logits [T,E]
 * (Algorithm 1's input is the score vector; scores are softmax(logits)).
 * params->dtype is ignored.
 */
int laser_route_from_logits(const float* logits, int32_t T, int32_t E,
                            const laser_params_t* params, int32_t* loads_inout,
                            int32_t* expert_ids, float* weights, int32_t* permutation,
                            int32_t* expert_offsets, void* workspace,
                            size_t workspace_bytes, void* hip_stream);

/*
 * laser_route, and in the same pass the per-token statistics of the gate scores that
 * the paper uses to choose eps_high and t_fix per layer (Observations: Layer
 * Variability in Gate Score Distributions; Method: Parameter setting and layer-wise
 * choices).  Device arrays of T entries, each may be NULL:
 *   topk_mass   fp32  M_k, the sum of the k largest softmax scores
 *   entropy     fp32  Shannon entropy of the scores, natural logarithm
 *   pool_size   int32 m = |{i : s_i >= t_fix * s_(1)} united with the top-k|
 *               (min(c, m) is the size of the working set of Algorithm 1)
 * Plain fp32 arithmetic from the quantities the router computes anyway; they take
 * part in no decision.  Everything else as laser_route.
 */
int laser_route_stats(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                      const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                      float* weights, int32_t* permutation, int32_t* expert_offsets,
                      float* logits_out, float* topk_mass, float* entropy, int32_t* pool_size,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Imbalance metrics of per-layer assignment counts (Problem statement: imbalance
 * factor, aggregate over layers, GPU-level imbalance under a placement; Evaluation,
 * Metrics: max violation).  All pointers are device pointers.
 *   counts         [L,E] int32  tokens assigned to expert e in layer l          in
 *   placement      [G,E] fp32   share of expert e served by GPU g (columns sum  in
 *                  to 1), or NULL: no GPU-level figure
 *   layer_weights  [L] fp32 w_l, or NULL for 1/L                                in
 *   I              [L] fp64     max_e N / mean_e N                              out
 *   MV             [L] fp64     I - 1, or NULL                                  out
 *   I_gpu          [L] fp64     max_g N_g / mean_g N_g with N_g = sum_e A[g,e] N[e]
 *                  (required when placement is given, else may be NULL)         out
 *   agg            [2] fp64     sum_l w_l I[l], sum_l w_l I_gpu[l] (1 without    out
 *                  placement)
 * A layer without assignments counts as balanced (1).  Limits: G <= 4096.
 */
int laser_imbalance(const int32_t* counts, int32_t L, int32_t E, const float* placement,
                    int32_t G, const float* layer_weights, double* I, double* MV, double* I_gpu,
                    double* agg, void* hip_stream);

/*
 * Percentiles of n values on the device, e.g. of the aggregate imbalance factor of n
 * batches (Evaluation, Metrics: the aggregate is summarised by its 50th and 95th
 * percentile across batches).  The q-th percentile sits at position (n-1)*q/100 of the
 * ascending list and is interpolated linearly between its two neighbours.
 *   values  [n] fp64, device pointer, no NaN                       in
 *   q       [nq] fp64, HOST pointer, each in [0, 100]              in
 *   out     [nq] fp64, device pointer                              out
 * Limits: 1 <= n <= 4096 (more: LASER_E_UNSUPPORTED), nq <= 16.
 */
int laser_percentiles(const double* values, int32_t n, const double* q, int32_t nq, double* out,
                      void* hip_stream);

/*
 * Mean and percentiles of n fp32 values on the device: a layer's per-token top-k mass
 * or entropy from laser_route_stats, summarised the way the paper looks at the gate
 * scores layer by layer (Observations: Layer Variability in Gate Score Distributions;
 * Method: Parameter setting and layer-wise choices).  Percentiles as laser_percentiles
 * (position (n-1)*q/100, linear interpolation; the order statistics are exact), the
 * mean in fp64.  Integer statistics (pool sizes) are converted to fp32 by the caller.
 *   values  [n] fp32, device pointer, no NaN                       in
 *   q       [nq] fp64, HOST pointer, each in [0, 100], nq <= 16    in
 *   mean    fp64, device pointer, or NULL                          out
 *   out     [nq] fp64, device pointer (may be NULL if nq = 0)      out
 * One workgroup, no scratch memory; time grows with n * nq.
 */
int laser_summary_f32(const float* values, int32_t n, const double* q, int32_t nq, double* mean,
                      double* out, void* hip_stream);

/* Static, NUL-terminated description of a return code (host pointer). */
const char* laser_strerror(int code);

/*
 * Whether the last call that used `workspace` (the start of one problem's workspace; for
 * problem b of a batched call, workspace + b * laser_workspace_bytes(...)) wrote all of
 * its outputs: waits for `hip_stream`, then stores LASER_STATUS_* in *status (host
 * pointer).  The record is cleared by the next call that uses the workspace.  This is
 * the library's only call that synchronises.
 */
int laser_status(const void* workspace, void* hip_stream, int32_t* status);

/*
 * laser_route for callers that cannot allocate device memory or carry a workspace
 * around: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The workspace is an array inside the library (one per GPU, held until the
 * process ends) of laser_static_workspace_bytes() bytes; a call that needs more
 * returns LASER_E_WORKSPACE.  The
 * call allocates nothing and otherwise behaves as laser_route.  All such calls on one
 * GPU share the array: they must be ordered (one stream, or events), calls that overlap
 * race.  laser_status_static() is laser_status() for the current device's array.
 */
size_t laser_static_workspace_bytes(void);
int laser_route_static(const void* hidden, const void* w_gate, int32_t T, int32_t H, int32_t E,
                       const laser_params_t* params, int32_t* loads_inout, int32_t* expert_ids,
                       float* weights, int32_t* permutation, int32_t* expert_offsets,
                       float* logits_out, void* hip_stream);
int laser_status_static(void* hip_stream, int32_t* status);

#ifdef __cplusplus
}
#endif
#endif /* LASER_H_ */
