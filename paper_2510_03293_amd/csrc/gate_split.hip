// The bf16 gate projection and analysis of small calls: the contraction axis of a tile
// cut over several workgroups (see the comment above the kernel).
#include <atomic>

#include "gate_tile.h"

namespace laser {

// ---- small calls (fewer tiles than an eighth of the compute units) -------------------
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
template <int EB, int NE, int NM, bool STATS>
__global__ __launch_bounds__(kGateThreads) void gate_split_bf16_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ w, int H, const RouteArgs a0,
    const Workspace ws, int32_t* __restrict__ expert_ids, float* __restrict__ weights,
    float* __restrict__ logits_out) {
  extern __shared__ __align__(16) unsigned char gate_lds[];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  __shared__ int sh_last;
  RouteArgs a = a0;
  if (STATS && a.pool_in_ws) a.st_pool = ws.pool;
  const int T = a.T, E = a.E;
  const int split = a.split;               // 2, 4 or 8 workgroups per tile
  const int nroles = kGateWaves / split;   // wavefront roles of this workgroup
  // (the workgroups of a tile are ntiles apart in the grid)
  const int tile = (int)blockIdx.x % a.ntiles;
  const int part_of_tile = (int)blockIdx.x / a.ntiles;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int role = part_of_tile * nroles + wave_u;  // meaningful where wave_u < nroles

  f32x4 acc[EB][4];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[eb][tb][r] = 0.0f;

  if (wave_u < nroles) {
    // (what follows is the main loop of gate_analyse_bf16_kernel with the role in the place
    // of the wave number; the LDS strip is this wave's)
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
    unsigned char* strip = gate_lds + wave_u * kStripBytes;
    unsigned char* st_wr = strip + lrow * kRowBytes + lpiece * 16;
    unsigned char* st_rd = strip + (lane & 15) * kRowBytes + (lane >> 4) * 16;

    const int nfull = NM > 0 ? 8 * NM : H >> 6;
    const int nmine = (nfull - role + kGateWaves - 1) / kGateWaves;  // chunks role, role+8, ...
    const int lim = nfull * 128;
    const int cstride = kGateWaves * 128;
    int koff = nfull > 0 ? ((tile * 5 + role) % nfull) * 128 : 0;
    auto step = [&](int k) { k += cstride; return k >= lim ? k - lim : k; };

    u32x4 rh[8], rw[2 * EB];
    if constexpr (NM > 0) {
      u32x4 rh2[8];
      int kw = koff;
      GATE_GH(rh, koff)
      GATE_GW(rw, kw)
      koff = step(koff);
      GATE_GH(rh2, koff)
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        if (i % 2 == 0) {
          GATE_S(rh, rw)
        } else {
          GATE_S(rh2, rw)
        }
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
    } else if (nmine > 0) {
      GATE_GH(rh, koff)
      GATE_GW(rw, koff)
      for (int i = 0; i + 1 < nmine; ++i) {
        GATE_S(rh, rw)
        koff = step(koff);
        GATE_GH(rh, koff)
        GATE_GW(rw, koff)
        GATE_M()
      }
      GATE_S(rh, rw)
      GATE_M()
    }
    // ragged tail of the contraction axis (H % 64 != 0), taken by one role
    if (NM == 0 && (H & 63) != 0 && role == (nfull & (kGateWaves - 1))) {
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
  __syncthreads();  // all strips are dead: the partial tiles reuse the space

  float* part = reinterpret_cast<float*>(gate_lds);  // [8][64][kPartStride]
  if (wave_u < nroles) {
    float* mine = part + (size_t)wave * kTile * kPartStride;
    const int n = lane & 15, kgrp = lane >> 4;
#pragma unroll
    for (int eb = 0; eb < EB; ++eb)
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
        float4 v = make_float4(acc[eb][tb][0], acc[eb][tb][1], acc[eb][tb][2], acc[eb][tb][3]);
        *reinterpret_cast<float4*>(mine + (tb * 16 + n) * kPartStride + eb * 16 + 4 * kgrp) = v;
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
  {
    constexpr int kPer = kGateWaves * kPairs / kGateThreads;  // 32 elements per thread
    unsigned long long v[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u)
      v[u] = __hip_atomic_load(tile_parts + threadIdx.x + u * kGateThreads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int j = threadIdx.x + u * kGateThreads;
      *lds_pair(j / kPairs, j % kPairs) = v[u];
    }
  }
  __syncthreads();
  analyse_tile<NE, kGateWaves, STATS>(part, kPartStride, mask64, &flex_lds, tile, a, ws, expert_ids, weights,
                                      logits_out);
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

template <int EB, int NE, int NM, bool STATS>
static hipError_t launch_split(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                               int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  static LdsAttr allowed;
  const void* fn = reinterpret_cast<const void*>(&gate_split_bf16_kernel<EB, NE, NM, STATS>);
  const hipError_t e = allow_dynamic_lds(fn, kGateLdsBytes, allowed);
  if (e != hipSuccess) return e;
  clear_stale_error();
  hipLaunchKernelGGL((gate_split_bf16_kernel<EB, NE, NM, STATS>), dim3(a.ntiles * a.split), dim3(kGateThreads),
                     kGateLdsBytes, s, static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(w), H, a, ws,
                     expert_ids, weights, logits_out);
  return hipGetLastError();
}

template <int EB, int NE>
static hipError_t launch_split_one(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                                   int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  if (wants_stats(a)) {
    if (H == 2048) return launch_split<EB, NE, 4, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    if (H == 4096) return launch_split<EB, NE, 8, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    return launch_split<EB, NE, 0, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  }
  if (H == 2048) return launch_split<EB, NE, 4, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  if (H == 4096) return launch_split<EB, NE, 8, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  return launch_split<EB, NE, 0, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
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
