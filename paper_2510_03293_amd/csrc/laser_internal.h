// Internal declarations shared by the HIP translation units of the routing
// library: workspace layout, per-call parameters, kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace laser {

constexpr int kTile = 64;        // tokens per tile (one wave-wide bit mask per tile)
constexpr int kMaxE = 64;        // experts: one lane of a wavefront per expert
constexpr int kMaxC = 16;        // trimming size limit (candidate ranks fit 4 bits)

// Per-call scalars handed to every kernel by value.
struct RouteArgs {
  int T;            // tokens
  int E;            // experts
  int EP;           // experts padded to 8/16/32/64 (8 lanes per token x EP/8 each)
  int k;            // experts per token
  int c;            // trimming size
  int ntiles;       // ceil(T / kTile)
  int renormalize;  // weights over the chosen k (1) or raw softmax scores (0)
  float eps_high;   // top-k mass threshold
  float tau_ln;     // fl32(ln t_fix): pool cut-off in the logit domain
  const int32_t* loads_in;  // [E] the caller's counters before token 0 (copied to the workspace
                            // by the analysis so that the tail can read them while it writes)
  // optional per-token statistics, [T] each, any may be NULL (all NULL: not computed)
  float* st_mass;      // top-k mass M_k
  float* st_entropy;   // Shannon entropy of the scores, nats
  int32_t* st_pool;    // pool size m (candidates above the cut, united with the top-k)
};
// Trimming mode RANDOM: what makes the sample reproducible.
struct RandomArgs {
  unsigned long long seed;          // generator key
  unsigned long long token_offset;  // index of token 0 of this call in the caller's numbering
  uint32_t stream;                  // caller's stream id (e.g. the layer)
};
inline bool wants_stats(const RouteArgs& a) { return a.st_mass || a.st_entropy || a.st_pool; }

// Device workspace carved out of the caller's buffer.  Records are written by
// the per-token analysis, consumed by the load-ordered chain and the finishing
// pass.  "slot" = tile * kTile + (rank of the token among its tile's flexible
// tokens), so a tile's flexible records are contiguous.
struct Workspace {
  float* logits;               // [T,E]   gate logits (unless the caller gave a buffer)
  uint8_t* rec_cstar;          // [T]     working-set size of a flexible token, else 0
  uint8_t* rec_ids;            // [T,16]  experts by descending score
  float* rec_p;                // [T,16]  their softmax numerators exp(z - z_max)
  float* rec_Z;                // [T]     softmax normaliser
  uint16_t* rec_lane;          // [slot,EP] per expert: (fixed-prefix << 4 | rank) or 0xFFFF
  unsigned long long* flexmask;    // [ntiles] bit i: token i of the tile is flexible
  uint8_t* tile_fixed_cnt;     // [ntiles,64] assignments of the tile's non-flexible tokens (<= 64)
  unsigned long long* tile_mask;   // [ntiles,64] per expert: the tile's non-flexible tokens
                               //           assigned to it (bit = token within the tile)
  int32_t* tile_base;          // [ntiles,64] assignments of all earlier tiles, per expert
  uint8_t* rec_cids;           // [slot,16] lanes the chain reads: candidates by rank, padded
  uint8_t* rec_pref;           // [slot,16] per candidate (by rank): earlier fixed tokens of the
                               //           tile assigned to it (<= 63); 0xFF beyond the working set
  int32_t* flex_list;          // [ntiles]  tiles that hold flexible tokens, ascending
  int32_t* flex_ord;           // [ntiles]  number of such tiles before this tile
  int32_t* flex_tok_base;      // [ntiles+1] flexible tokens in earlier tiles; [ntiles] = all
  int32_t* flex_slot;          // [T]       slot of the f-th flexible token (token order)
  uint32_t* chain_bits;        // [T/32+1,64] per expert: bit f%32 of word f/32 = chosen for
                               //           the f-th flexible token
  int32_t* chain_cum;          // [T/32+2,64] per expert: choices by flexible tokens < 32*w
  int32_t* lin_copy;           // [64] loads before token 0 (0 beyond E)
  int32_t* status;             // [4] see kStatus*: cleared by the analysis kernel of a call
};

constexpr int kStatusPhase = 0;      // 1: fixed prefix published, 2: chain finished
constexpr int kStatusFlexTiles = 1;  // number of tiles that hold flexible tokens
constexpr int kStatusError = 2;      // a bounded wait in the tail kernel ran out
constexpr int kStatusSweeps = 3;     // sweeps of the chain's window evaluation (diagnostic)

size_t workspace_bytes(int T, int E, bool need_logits);
Workspace carve_workspace(void* base, int T, int E, bool need_logits);

inline int padded_experts(int E) { return E <= 8 ? 8 : E <= 16 ? 16 : E <= 32 ? 32 : 64; }

// Launchers (enqueue only; return the HIP error of the launch).
// gate projection fused with the per-token analysis (logits_out may be NULL)
hipError_t launch_gate_analyse_bf16(const void* hidden, const void* w, int H, const RouteArgs& a,
                                    const Workspace& ws, int32_t* expert_ids, float* weights,
                                    float* logits_out, hipStream_t s);
hipError_t launch_gate_f32(const float* hidden, const float* w, int T, int H, int E,
                           float* logits, hipStream_t s);
hipError_t launch_analyse(const float* logits, const RouteArgs& a, const Workspace& ws,
                          int32_t* expert_ids, float* weights, hipStream_t s);
// per-token analysis with RANDOM trimming, from logits [T,E]
hipError_t launch_analyse_random(const float* logits, const RouteArgs& a, const Workspace& ws,
                                 const RandomArgs& rnd, int32_t* expert_ids, float* weights,
                                 hipStream_t s);
hipError_t launch_tail(const RouteArgs& a, const Workspace& ws, int32_t* loads_inout,
                       int32_t* expert_offsets, int32_t* expert_ids, float* weights,
                       int32_t* permutation, hipStream_t s);

}  // namespace laser
