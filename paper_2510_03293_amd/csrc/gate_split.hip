// The bf16 gate projection and analysis of small calls: the contraction axis of a tile
// cut over several workgroups (see the comment above the kernel).
#include <atomic>

#include "gate_tile.h"

namespace laser {

// ---- small calls (at most a quarter as many tiles as the chip has compute units) ------
//
// In gate_analyse_bf16_kernel one workgroup streams the 64 rows of its tile and all of W
// through one compute unit; with a handful of tiles the rest of the chip idles while that
// unit pulls its half megabyte at what one unit can pull.  Here the eight wavefront roles
// of that kernel -- role r owns the chunks r, r + 8, ... of the contraction axis, from
// load to MFMA, in the same order -- go to `split` workgroups of 8 / split roles each.
// Every workgroup leaves its roles' partial tiles in the workspace (stored write-through)
// and, all stores acknowledged, counts itself into the tile's counter; the workgroup that
// finds the count complete fetches the eight partial tiles (agent-scope loads), and goes on
// exactly as the other kernel does: the analysis adds the same eight partial tiles in the
// same order, so the logits, and with them everything else, are bit for bit those of a
// call that is not split.  Nobody waits for anybody.
//
// The counters must be zero before the first workgroup arrives and the caller's workspace
// holds whatever it held, so they live in the library's own memory: an array that is part
// of the code object (zero when it is loaded) of which every workspace address gets a slice
// on first sight.  The last workgroup of a tile sets the tile's counter back to zero.  Calls
// that share a workspace must not overlap anyway, so a slice has one user at a time.
template <int EB, int NE, int NR, bool STATS>  // NR: wavefront roles per workgroup, 1 or 2
__global__ __launch_bounds__(kGateThreads) void gate_split_bf16_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ w, int H, const RouteArgs a0,
    const Workspace ws, int32_t* __restrict__ expert_ids, float* __restrict__ weights,
    float* __restrict__ logits_out) {
  static_assert(NR == 1 || NR == 2, "one or two roles per workgroup");
  extern __shared__ __align__(16) unsigned char gate_lds[];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  __shared__ int sh_last;
  RouteArgs a = a0;
  if (STATS && a.pool_in_ws) a.st_pool = ws.pool;
  const int T = a.T, E = a.E;
  constexpr int split = kGateWaves / NR;  // workgroups per tile (the launcher sees to a.split == split)
  constexpr int nroles = NR;
  // (the workgroups of a tile are ntiles apart in the grid)
  const int tile = (int)blockIdx.x % a.ntiles;
  const int part_of_tile = (int)blockIdx.x / a.ntiles;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);

  // The chunks of role r are those of wave r of the unsplit kernel, in its order: chunk i
  // is (start + 8 i) mod nfull.  Here the chunks of the workgroup's roles form one list
  // (role by role); wave v of the workgroup loads and stages item v + 8 n in round n, so
  // that all items of a round are in flight at once (the projection shapes with 2048 or
  // 4096 columns are one or two rounds).  Then four waves per role multiply the round's
  // chunks of that role, in the role's order, each into its own 16x16 blocks of the role's
  // partial tile (a 2x2 patch of blocks for 64 experts: two operands of each kind per
  // product step instead of three for two blocks).  Block (eb, tb) accumulates exactly the
  // products it accumulates in the unsplit kernel, in the same order, whoever runs the
  // instructions.
  constexpr int EBW = EB >= 4 ? 2 : 1;  // expert blocks per multiplying wave
  constexpr int TBW = EB >= 2 ? 2 : 1;  // token blocks per multiplying wave
  const int mrole = NR == 2 ? wave_u >> 2 : 0;       // the role this wave multiplies for ...
  const bool multiplies = NR == 2 || wave_u < 4;     // ... if it does
  const int mq = wave_u & 3;
  const int eb0 = EB >= 4 ? 2 * (mq >> 1) : EB == 2 ? (mq >> 1) : 0;
  const int tb0 = EB >= 2 ? 2 * (mq & 1) : mq;
  f32x4 acc[EBW][TBW];
#pragma unroll
  for (int e = 0; e < EBW; ++e)
#pragma unroll
    for (int t = 0; t < TBW; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[e][t][r] = 0.0f;

  const int lrow = lane >> 3, lpiece = lane & 7;
  const size_t row_bytes = (size_t)H * 2;
  const unsigned char* hbase = reinterpret_cast<const unsigned char*>(hidden) + (size_t)tile * kTile * row_bytes;
  const unsigned char* wbase = reinterpret_cast<const unsigned char*>(w);
  const int last_row = T - 1 - tile * kTile;  // >= 0
  unsigned hoff[8], woff[2 * EB];
#pragma unroll
  for (int q = 0; q < 8; ++q) hoff[q] = (unsigned)(min(q * 8 + lrow, last_row) * row_bytes) + lpiece * 16;
#pragma unroll
  for (int q = 0; q < 2 * EB; ++q) woff[q] = (unsigned)(min(q * 8 + lrow, E - 1) * row_bytes) + lpiece * 16;
  unsigned char* st_wr = gate_lds + wave_u * kStripBytes + lrow * kRowBytes + lpiece * 16;
  const unsigned rd_lane = (lane & 15) * kRowBytes + (lane >> 4) * 16;

  const int nfull = H >> 6;
  // per role: its full chunks, where it starts, and whether the ragged end of the
  // contraction axis (H % 64 != 0) is its to take, after its full chunks, as in the unsplit
  // kernel (pieces past H are read from the start of the row instead and replaced by zeros)
  int nmine[NR], start[NR], nitem[NR];
#pragma unroll
  for (int rr = 0; rr < NR; ++rr) {
    const int role = part_of_tile * NR + rr;
    nmine[rr] = (nfull - role + kGateWaves - 1) / kGateWaves;
    start[rr] = nfull > 0 ? (tile * 5 + role) % nfull : 0;
    nitem[rr] = nmine[rr] + (((H & 63) != 0 && role == (nfull & (kGateWaves - 1))) ? 1 : 0);
  }
  const int nitems = nitem[0] + (NR == 2 ? nitem[NR - 1] : 0);
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  u32x4 rh[8], rw[2 * EB];
  auto load_item = [&](int it) {
    const int rr = (NR == 2 && it >= nitem[0]) ? 1 : 0;
    const int i = it - (rr ? nitem[0] : 0);
    if (i < nmine[rr]) {  // chunk i of the role
      const int koff = ((start[rr] + kGateWaves * i) % nfull) * 128;
      GATE_GH(rh, koff)
      GATE_GW(rw, koff)
    } else {  // the ragged end
      const bool kin = nfull * 64 + lpiece * 8 < H;  // H % 8 == 0: a piece is all in or all out
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
    }
  };
  // the item in strip j, if it is one of this wave's role
  auto multiply = [&](int j) {
    const unsigned char* st_rd = gate_lds + j * kStripBytes + rd_lane;
#pragma unroll
    for (int s_ = 0; s_ < 2; ++s_) {
      u32x4 a_[EBW], b_[TBW];
#pragma unroll
      for (int t = 0; t < TBW; ++t) b_[t] = *(lds_u4_ptr)(st_rd + (tb0 + t) * 16 * kRowBytes + s_ * 64);
#pragma unroll
      for (int e = 0; e < EBW; ++e)
        a_[e] = *(lds_u4_ptr)(st_rd + kTile * kRowBytes + (eb0 + e) * 16 * kRowBytes + s_ * 64);
#pragma unroll
      for (int e = 0; e < EBW; ++e)
#pragma unroll
        for (int t = 0; t < TBW; ++t)
          acc[e][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a_[e]),
                                                              __builtin_bit_cast(bf16x8, b_[t]), acc[e][t], 0, 0, 0);
    }
  };
  if (wave_u < nitems) load_item(wave_u);
  for (int r0 = 0; r0 < nitems; r0 += kGateWaves) {
    if (r0 + wave_u < nitems) {
      GATE_S(rh, rw)  // (waits for the loads)
    }
    __syncthreads();
    // the next round's loads travel while this round is multiplied
    if (r0 + kGateWaves + wave_u < nitems) load_item(r0 + kGateWaves + wave_u);
    if (multiplies) {
      // strips [j0, j1) hold this wave's role's items of the round
      const int lo = mrole == 0 ? 0 : nitem[0], hi = mrole == 0 ? nitem[0] : nitems;
      const int j0 = max(lo - r0, 0), j1 = min(min(hi - r0, kGateWaves), nitems - r0);
      // (written out for the usual sizes, so that the operand reads of a chunk do not wait
      // for the products of the chunk before)
      if (j1 - j0 == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) multiply(j0 + j);
      } else if (j1 - j0 == 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) multiply(j);
      } else {
        for (int j = j0; j < j1; ++j) multiply(j);
      }
    }
    __syncthreads();  // the strips are free again (after the last round: dead, the partial tiles reuse the space)
  }
  if (nitems == 0) __syncthreads();

  float* part = reinterpret_cast<float*>(gate_lds);  // [roles][64][kPartStride]
  if (multiplies) {
    const int n = lane & 15, kgrp = lane >> 4;
    float* mine = part + (size_t)mrole * kTile * kPartStride;
#pragma unroll
    for (int e = 0; e < EBW; ++e)
#pragma unroll
      for (int t = 0; t < TBW; ++t) {
        const float4 v = make_float4(acc[e][t][0], acc[e][t][1], acc[e][t][2], acc[e][t][3]);
        *reinterpret_cast<float4*>(mine + ((tb0 + t) * 16 + n) * kPartStride + (eb0 + e) * 16 + 4 * kgrp) = v;
      }
  }
  __syncthreads();

  // ---- this workgroup's partial tiles -> workspace, 64 x 64 floats per role ------------
  // (element j of a role's tile, 8 bytes: row j / 32, columns 2 (j % 32) and the next)
  constexpr int kPairs = kTile * 64 / 2;  // 8-byte elements per partial tile
  auto lds_pair = [&](int r, int jj) {
    return reinterpret_cast<unsigned long long*>(part + ((size_t)r * kTile + (jj >> 5)) * kPartStride + 2 * (jj & 31));
  };
  unsigned long long* const tile_parts =
      reinterpret_cast<unsigned long long*>(ws.split_part) + (size_t)tile * kGateWaves * kPairs;
  {
    unsigned long long* dst = tile_parts + (size_t)part_of_tile * nroles * kPairs;
    for (int j = threadIdx.x; j < nroles * kPairs; j += kGateThreads)
      __hip_atomic_store(dst + j, *lds_pair(j / kPairs, j % kPairs), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // every store acknowledged ...
  __syncthreads();                                   // ... by every wavefront
  if (threadIdx.x == 0) {
    int32_t* counter = a.split_cnt + tile;
    const int before = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = before == split - 1;
    if (last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next call
    sh_last = last;
  }
  __syncthreads();
  if (sh_last == 0) return;

  // ---- the last workgroup of the tile: all eight partial tiles -> LDS, then the analysis ----
  // Wave w fetches the tile of role w: 16 loads of 16 bytes per lane, 1 KiB per instruction
  // (with 8-byte loads the fetch took twice as long: the memory pipeline takes a wave's
  // instruction every 16 cycles whatever its width).  Agent-scope loads of 16 bytes exist
  // only as instructions, so they are written out, all of them and the wait for them in one
  // block: the compiler takes an output of a block as valid when the block ends.
  {
    const unsigned char* src = reinterpret_cast<const unsigned char*>(tile_parts) + (size_t)wave * (kPairs * 8) + lane * 16;
    const unsigned char *s0 = src, *s1 = src + 4096, *s2 = src + 8192, *s3 = src + 12288;
    u32x4 v[16];
    asm volatile(
        "global_load_dwordx4 %0, %16, off sc1\n\t"
        "global_load_dwordx4 %1, %16, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %16, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %16, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %4, %17, off sc1\n\t"
        "global_load_dwordx4 %5, %17, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %6, %17, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %7, %17, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %8, %18, off sc1\n\t"
        "global_load_dwordx4 %9, %18, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %10, %18, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %11, %18, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %12, %19, off sc1\n\t"
        "global_load_dwordx4 %13, %19, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %14, %19, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %15, %19, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7]),
          "=&v"(v[8]), "=&v"(v[9]), "=&v"(v[10]), "=&v"(v[11]), "=&v"(v[12]), "=&v"(v[13]), "=&v"(v[14]),
          "=&v"(v[15])
        : "v"(s0), "v"(s1), "v"(s2), "v"(s3)
        : "memory");
    // bytes 1024 u + 16 lane of the tile = row 4 u + lane / 16, columns 4 (lane % 16) ...
#pragma unroll
    for (int u = 0; u < 16; ++u)
      *reinterpret_cast<u32x4*>(part + ((size_t)wave * kTile + 4 * u + (lane >> 4)) * kPartStride + 4 * (lane & 15)) = v[u];
  }
  __syncthreads();
  analyse_tile<NE, kGateWaves, STATS>(part, kPartStride, mask64, &flex_lds, tile, a, ws, expert_ids, weights,
                                      logits_out);

  // ---- a call of one tile without load-dependent tokens ends here -----------------------
  // Everything the dispatch tables need is in this workgroup: per expert the tokens
  // assigned to it (mask64) and, just written, the tokens' experts in rank order.  The
  // tables are those the tail kernel would write (a stable counting sort of the T k
  // assignments); it finds the mark and returns at once.
  if (NR == 1 && a.one_permutation != nullptr) {  // (a.ntiles == 1)
    __shared__ int sh_off[64];
    __syncthreads();  // the expert ids are stored, mask64 and flex_lds are final
    if (flex_lds != 0ull) return;
    if (wave == 0) {  // lane = expert
      const int cnt = lane < E ? __builtin_popcountll(mask64[lane]) : 0;
      int incl = cnt;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
      }
      sh_off[lane] = incl - cnt;
      if (lane < E) {
        a.one_expert_offsets[lane] = incl - cnt;
        a.one_loads[lane] += cnt;
      }
      if (lane == E - 1) a.one_expert_offsets[E] = incl;
    }
    __syncthreads();
    const int k = a.k;
    for (int slot = threadIdx.x; slot < T * k; slot += kGateThreads) {
      const int t = slot / k;
      const int e = expert_ids[slot];
      a.one_permutation[sh_off[e] + __builtin_popcountll(mask64[e] & lanes_below(t))] = slot;
    }
    if (threadIdx.x == 0) ws.status[kStatusPhase] = kPhaseAllDone;
  }
}

// ---- the counters ---------------------------------------------------------------------
constexpr int kSplitSlices = 1024;
static __device__ int32_t split_counters[kSplitSlices * kSplitMaxTiles];

struct SplitTable {
  std::atomic<uintptr_t> key[kSplitSlices];  // workspace address that owns the slice, 0: free
  std::atomic<int32_t*> base;                // the array's address on this device
};
static SplitTable g_split[kMaxDevices];

int32_t* split_counters_for(const void* workspace) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  SplitTable& t = g_split[dev];
  int32_t* base = t.base.load(std::memory_order_acquire);
  if (base == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(split_counters)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    base = static_cast<int32_t*>(p);
    t.base.store(base, std::memory_order_release);
  }
  const uintptr_t k = reinterpret_cast<uintptr_t>(workspace);
  const unsigned h = (unsigned)((k >> 8) * 0x9E3779B1u);
  for (int probe = 0; probe < 64; ++probe) {
    const unsigned i = (h + (unsigned)probe) % kSplitSlices;
    uintptr_t cur = t.key[i].load(std::memory_order_acquire);
    if (cur == 0) {
      if (t.key[i].compare_exchange_strong(cur, k, std::memory_order_acq_rel)) cur = k;
      // (on failure `cur` holds what another thread put there)
    }
    if (cur == k) return base + (size_t)i * kSplitMaxTiles;
  }
  return nullptr;  // the table is crowded: the call runs without the split
}

template <int EB, int NE, int NR, bool STATS>
static hipError_t launch_split(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                               int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  static LdsAttr allowed;
  const void* fn = reinterpret_cast<const void*>(&gate_split_bf16_kernel<EB, NE, NR, STATS>);
  const hipError_t e = allow_dynamic_lds(fn, kGateLdsBytes, allowed);
  if (e != hipSuccess) return e;
  if (a.split * NR != kGateWaves) return hipErrorInvalidValue;
  clear_stale_error();
  hipLaunchKernelGGL((gate_split_bf16_kernel<EB, NE, NR, STATS>), dim3(a.ntiles * a.split), dim3(kGateThreads),
                     kGateLdsBytes, s, static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(w), H, a, ws,
                     expert_ids, weights, logits_out);
  return hipGetLastError();
}

template <int EB, int NE>
static hipError_t launch_split_one(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                                   int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  const bool st = wants_stats(a);
  if (a.split == kGateWaves) {
    if (st) return launch_split<EB, NE, 1, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    return launch_split<EB, NE, 1, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  }
  if (st) return launch_split<EB, NE, 2, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  return launch_split<EB, NE, 2, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
}

hipError_t launch_gate_split_bf16(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                                  int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  switch (a.EP) {
    case 8: return launch_split_one<1, 1>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 16: return launch_split_one<1, 2>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 32: return launch_split_one<2, 4>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    default: return launch_split_one<4, 8>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  }
}

}  // namespace laser
