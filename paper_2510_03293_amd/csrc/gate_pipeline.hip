// The bf16 gate projection and analysis of pipelined calls: persistent workgroups, with
// the chain workgroup of the call in front of them (see the comment above the kernel, and
// chain_segments in tail.h).
#include <algorithm>

#include "gate_tile.h"
#include "tail.h"

namespace laser {

// ---- pipelined calls (large single problems) ----------------------------------------
//
// The same projection and analysis by persistent workgroups: workgroup 0 of the grid is the
// chain workgroup (see chain_segments), workgroup b >= 1 takes tiles slot(b), slot(b) + G,
// slot(b) + 2G, ... of the G = gridDim.x - 1 tiles of every round, so that early tiles are
// finished early.  Two things follow from staying on the compute unit:
//   - the first loads of the next tile are issued before the analysis of the current one
//     and arrive while it runs, so the memory pipeline of the compute unit does not drain
//     between tiles;
//   - a tile is reported to the chain workgroup (every wavefront counts itself into the
//     tile's word) one step into the next tile, when the stores of its
//     records have long been acknowledged: nobody waits for a store.
// What the chain workgroup reads is stored write-through (store_for_chain); a wavefront
// counts itself in only after all its stores are acknowledged, and the chain workgroup
// invalidates its caches after seeing a segment complete.
template <int EB, int NE, int NM, bool STATS>
__global__ __launch_bounds__(kGateThreads) void gate_pipeline_bf16_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ w, int H, const RouteArgs a0,
    const Workspace ws, int32_t* __restrict__ expert_ids, float* __restrict__ weights,
    float* __restrict__ logits_out) {
  extern __shared__ __align__(16) unsigned char gate_lds[];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  RouteArgs a = a0;
  if (STATS && a.pool_in_ws) a.st_pool = ws.pool;
  if (blockIdx.x == 0) {
    if (threadIdx.x < kTailThreads)
      chain_segments<true>(gate_lds, a, ws, const_cast<int32_t*>(a.loads_in), nullptr);
    return;
  }
  const int T = a.T, E = a.E, ntiles = a.ntiles;
  const int G = (int)gridDim.x - 1;
  // Workgroups go to the eight XCDs in turn; the workgroups of one XCD take neighbouring
  // tiles of a round (slot = position in the order "XCD, then index within the XCD").
  int slot;
  {
    const int wg = (int)blockIdx.x - 1, x = wg & 7;
    int before = 0;
    for (int y = 0; y < 8; ++y) before += y < x ? (G - y + 7) >> 3 : 0;  // workgroups wg' % 8 == y
    slot = before + (wg >> 3);
  }
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);

  const int lrow = lane >> 3, lpiece = lane & 7;
  const size_t row_bytes = (size_t)H * 2;
  const unsigned char* wbase = reinterpret_cast<const unsigned char*>(w);
  unsigned hoff[8], woff[2 * EB];
#pragma unroll
  for (int q = 0; q < 2 * EB; ++q) woff[q] = (unsigned)(min(q * 8 + lrow, E - 1) * row_bytes) + lpiece * 16;
  unsigned char* strip = gate_lds + wave_u * kStripBytes;
  unsigned char* st_wr = strip + lrow * kRowBytes + lpiece * 16;
  unsigned char* st_rd = strip + (lane & 15) * kRowBytes + (lane >> 4) * 16;

  const int nfull = NM > 0 ? 8 * NM : H >> 6;
  const int nmine = (nfull - wave_u + kGateWaves - 1) / kGateWaves;
  const int lim = nfull * 128;
  const int cstride = kGateWaves * 128;
  auto step = [&](int k) { k += cstride; return k >= lim ? k - lim : k; };

  // per tile: where its rows start, the row offsets (rows past T are clamped), the chunk
  // the wave starts at
  const unsigned char* hbase;
  int koff, kw;
  auto set_tile = [&](int tile) {
    hbase = reinterpret_cast<const unsigned char*>(hidden) + (size_t)tile * kTile * row_bytes;
    const int last_row = T - 1 - tile * kTile;  // >= 0
    // (computed anew for every tile rather than kept, in parts, in registers across the loop)
    int l = lane;
    asm volatile("" : "+v"(l));
    const int lrow = l >> 3, lpiece = l & 7;
#pragma unroll
    for (int q = 0; q < 8; ++q) hoff[q] = (unsigned)(min(q * 8 + lrow, last_row) * row_bytes) + lpiece * 16;
    koff = nfull > 0 ? ((tile * 5 + wave_u) % nfull) * 128 : 0;
    kw = koff;
  };

  u32x4 rh[8], rw[2 * EB], rh2[8];
  // The loads a tile starts with: its hidden rows (from HBM; issued before the analysis of
  // the tile before) and then the W rows of its first chunk (from L2; issued after that
  // analysis -- holding them across it as well would not fit the register file, and
  // issuing them inside it, ahead of its stores, measured slower).
#define GATE_FIRST_H()              \
  if constexpr (NM > 0) {           \
    GATE_GH(rh, koff)               \
    koff = step(koff);              \
    GATE_GH(rh2, koff)              \
  } else if (nmine > 0) {           \
    GATE_GH(rh, koff)               \
  }
#define GATE_FIRST_W()              \
  if (NM > 0 || nmine > 0) {        \
    GATE_GW(rw, kw)                 \
  }

  int tile = slot;
  if (tile >= ntiles) return;  // (only when the call has fewer tiles than the grid has workgroups)
  int reported = -1;           // the tile whose records are written but not yet counted in
  // Counts this wavefront into the word of tile `reported`, all its stores acknowledged.
  // Called one step into the next tile, right after the wave has waited for that step's
  // loads: what is still in flight then was issued long before the tile's last store, so
  // the wait here costs nothing.
  auto report = [&]() {
    if (reported >= 0) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      // (written out: the compiler would count it among the loads it orders its waits
      // by, and then wait for everything in flight at the next step)
      int* word = &ws.seg[kSegDone + reported];
      const int one = 1;
      if (lane == 0) asm volatile("global_atomic_add %0, %1, off sc1" : : "v"(word), "v"(one) : "memory");
      reported = -1;
    }
  };
  set_tile(tile);
  GATE_FIRST_H()
  for (;;) {
    GATE_FIRST_W()
    f32x4 acc[EB][4];
#pragma unroll
    for (int eb = 0; eb < EB; ++eb)
#pragma unroll
      for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[eb][tb][r] = 0.0f;
    if constexpr (NM > 0) {
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        if (i % 2 == 0) {
          GATE_S(rh, rw)
        } else {
          GATE_S(rh2, rw)
        }
        if (i == 0) report();
        if (i + 1 < NM) {
          kw = step(kw);
          GATE_GW(rw, kw)
        }
        if (i + 2 < NM) {
          koff = step(koff);
          if (i % 2 == 0) {
            GATE_GH(rh, koff)
          } else {
            GATE_GH(rh2, koff)
          }
        }
        GATE_M()
      }
    } else {
      if (nmine > 0) {
        for (int i = 0; i + 1 < nmine; ++i) {
          GATE_S(rh, rw)
          if (i == 0) report();
          koff = step(koff);
          GATE_GH(rh, koff)
          GATE_GW(rw, koff)
          GATE_M()
        }
        GATE_S(rh, rw)
        GATE_M()
      }
      report();  // (nothing left to do if it was counted in above)
      if ((H & 63) != 0 && wave_u == (nfull & (kGateWaves - 1))) {
        const u32x4 zero4 = {0u, 0u, 0u, 0u};
        const bool kin = nfull * 64 + lpiece * 8 < H;
        const int off = kin ? nfull * 128 : -lpiece * 16;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const u32x4 v = load_global_16(hbase + hoff[q] + off);
          rh[q] = kin ? v : zero4;
        }
#pragma unroll
        for (int q = 0; q < 2 * EB; ++q) {
          const u32x4 v = load_global_16(wbase + woff[q] + off);
          rw[q] = kin ? v : zero4;
        }
        GATE_S(rh, rw)
        GATE_M()
      }
    }
    lds_barrier();  // all strips are dead: the partial tiles reuse the space
    float* part = reinterpret_cast<float*>(gate_lds);
    float* mine = part + (size_t)wave * kTile * kPartStride;
    const int n = lane & 15, kgrp = lane >> 4;
#pragma unroll
    for (int eb = 0; eb < EB; ++eb)
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
        float4 v = make_float4(acc[eb][tb][0], acc[eb][tb][1], acc[eb][tb][2], acc[eb][tb][3]);
        *reinterpret_cast<float4*>(mine + (tb * 16 + n) * kPartStride + eb * 16 + 4 * kgrp) = v;
      }
    lds_barrier();
    const int done = tile;
    const int next = tile + G;
    const bool more = next < ntiles;
    if (more) {
      // the next tile's first loads travel while this tile is analysed
      set_tile(next);
      GATE_FIRST_H()
    }
    analyse_tile<NE, kGateWaves, STATS, true>(part, kPartStride, mask64, &flex_lds, done, a, ws, expert_ids,
                                               weights, logits_out);
    reported = done;
    if (!more) break;
    tile = next;
    lds_barrier();  // the partial tiles have been read: the strips may be written again
  }
  report();
#undef GATE_FIRST_H
#undef GATE_FIRST_W
}

// What the first tile's analysis does for other calls -- clear the status words, keep a
// copy of the counters before token 0 -- and the words a pipelined call counts in.
__global__ __launch_bounds__(256) void seg_clear_kernel(int32_t* seg, int words, int32_t* status,
                                                        const int32_t* loads_in, int32_t* lin_copy, int E) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < words; i += gridDim.x * 256) seg[i] = 0;
  if (blockIdx.x != 0) return;
  if (threadIdx.x < 4) status[threadIdx.x] = 0;
  if (threadIdx.x < 64) lin_copy[threadIdx.x] = (int)threadIdx.x < E ? loads_in[threadIdx.x] : 0;
}

// A pipelined call: the clearing kernel, then the persistent gate kernel -- the chain
// workgroup plus one workgroup for every other compute unit.
template <int EB, int NE, int NM, bool STATS>
static hipError_t launch_pipeline(const void* hidden, const void* w, int H, const RouteArgs& a,
                                  const Workspace& ws, int32_t* expert_ids, float* weights,
                                  float* logits_out, hipStream_t s) {
  static LdsAttr allowed;
  const void* fn = reinterpret_cast<const void*>(&gate_pipeline_bf16_kernel<EB, NE, NM, STATS>);
  const hipError_t e = allow_dynamic_lds(fn, kGateLdsBytes, allowed);
  if (e != hipSuccess) return e;
  const int G = std::min(a.ntiles, pipeline_workgroups());
  clear_stale_error();
  const int words = kSegDone + a.ntiles;
  hipLaunchKernelGGL(seg_clear_kernel, dim3(std::min(64, (words + 255) / 256)), dim3(256), 0, s, ws.seg, words,
                     ws.status, a.loads_in, ws.lin_copy, a.E);
  hipLaunchKernelGGL((gate_pipeline_bf16_kernel<EB, NE, NM, STATS>), dim3(G + 1), dim3(kGateThreads), kGateLdsBytes, s,
                     static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(w), H, a, ws, expert_ids,
                     weights, logits_out);
  return hipGetLastError();
}


template <int EB, int NE>
static hipError_t launch_pipeline_one(const void* hidden, const void* w, int H, const RouteArgs& a,
                                      const Workspace& ws, int32_t* expert_ids, float* weights,
                                      float* logits_out, hipStream_t s) {
  if (wants_stats(a)) {
    if (H == 2048) return launch_pipeline<EB, NE, 4, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    if (H == 4096) return launch_pipeline<EB, NE, 8, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    return launch_pipeline<EB, NE, 0, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  }
  if (H == 2048) return launch_pipeline<EB, NE, 4, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  if (H == 4096) return launch_pipeline<EB, NE, 8, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  return launch_pipeline<EB, NE, 0, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
}

hipError_t launch_gate_pipeline_bf16(const void* hidden, const void* w, int H, const RouteArgs& a,
                                     const Workspace& ws, int32_t* expert_ids, float* weights,
                                     float* logits_out, hipStream_t s) {
  switch (a.EP) {
    case 8: return launch_pipeline_one<1, 1>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 16: return launch_pipeline_one<1, 2>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 32: return launch_pipeline_one<2, 4>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    default: return launch_pipeline_one<4, 8>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  }
}

}  // namespace laser
